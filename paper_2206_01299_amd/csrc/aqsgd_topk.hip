// Launch table of the sparsified-backward kernels (all three dtypes; the
// kernels are small next to the codec's, so one translation unit holds them).
#include "aqsgd_topk.h"

namespace aqsgd {

template <int DT, int MODE>
static hipError_t launch_topk_cpl(int cpl, unsigned blocks, const TopkArgs& a, hipStream_t s) {
    switch (cpl) {
    case 1: return launch_kernel(topk_kernel<DT, 1, MODE>, dim3(blocks), dim3(kTopkBlock), s, a);
    case 2: return launch_kernel(topk_kernel<DT, 2, MODE>, dim3(blocks), dim3(kTopkBlock), s, a);
    case 3: return launch_kernel(topk_kernel<DT, 3, MODE>, dim3(blocks), dim3(kTopkBlock), s, a);
    case 4: return launch_kernel(topk_kernel<DT, 4, MODE>, dim3(blocks), dim3(kTopkBlock), s, a);
    default: return hipErrorInvalidValue;
    }
}

template <int DT>
static hipError_t launch_topk_dt(int cpl, bool sender, unsigned blocks, const TopkArgs& a, hipStream_t s) {
    if (!sender) return launch_topk_cpl<DT, 0>(cpl, blocks, a, s);
    return a.stochastic ? launch_topk_cpl<DT, 2>(cpl, blocks, a, s) : launch_topk_cpl<DT, 1>(cpl, blocks, a, s);
}

hipError_t launch_topk(int dtype, int cpl, bool sender, unsigned blocks, const TopkArgs& a, hipStream_t s) {
    switch (dtype) {
    case AQSGD_F32:  return launch_topk_dt<AQSGD_F32>(cpl, sender, blocks, a, s);
    case AQSGD_F16:  return launch_topk_dt<AQSGD_F16>(cpl, sender, blocks, a, s);
    case AQSGD_BF16: return launch_topk_dt<AQSGD_BF16>(cpl, sender, blocks, a, s);
    default:         return hipErrorInvalidValue;
    }
}

}  // namespace aqsgd
