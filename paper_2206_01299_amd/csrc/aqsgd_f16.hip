// Codec kernels instantiated for f16 activations, buffers and outputs.
#include "aqsgd_instantiate.h"

namespace aqsgd {
AQSGD_INSTANTIATE_DTYPE(AQSGD_F16)
}
