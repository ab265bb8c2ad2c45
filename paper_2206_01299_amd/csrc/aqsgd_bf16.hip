// Codec kernels instantiated for bf16 activations, buffers and outputs.
#include "aqsgd_instantiate.h"

namespace aqsgd {
AQSGD_INSTANTIATE_DTYPE(AQSGD_BF16)
}
