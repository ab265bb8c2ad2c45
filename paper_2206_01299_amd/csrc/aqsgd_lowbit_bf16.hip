// Low-precision-storage codec kernels instantiated for bf16 activations and outputs.
#include "aqsgd_lowbit.h"

namespace aqsgd {
AQSGD_INSTANTIATE_LOWBIT_DTYPE(AQSGD_BF16)
}
