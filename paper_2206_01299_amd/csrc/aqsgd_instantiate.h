// Launch tables of one storage dtype: every (rounding, team shape, 3-bit or not) of the job
// kernel that hosts quantising jobs and every unroll of the one that holds
// dequantising jobs alone.  Each dtype gets its own translation unit so the three
// compile in parallel.
#pragma once

#include "aqsgd_kernels.h"

namespace aqsgd {

template <int DT, int ROUND, bool THREE, int TEAM, int CPL>
static hipError_t launch_cj(const JobTable& t, hipStream_t stream) {
    constexpr int threads = TEAM > kWave ? TEAM : kBlock;
    return launch_kernel(codec_jobs_kernel<DT, ROUND, TEAM, CPL, THREE>, dim3(t.total_blocks), dim3(threads),
                         stream, t);
}

template <int DT, int ROUND, bool THREE>
static hipError_t launch_cj_shape(int shape, const JobTable& t, hipStream_t stream) {
    switch (shape) {
    case kTeam8x1:    return launch_cj<DT, ROUND, THREE, 8, 1>(t, stream);
    case kTeam16x1:   return launch_cj<DT, ROUND, THREE, 16, 1>(t, stream);
    case kTeam32x1:   return launch_cj<DT, ROUND, THREE, 32, 1>(t, stream);
    case kTeam64x1:   return launch_cj<DT, ROUND, THREE, 64, 1>(t, stream);
    case kTeam64x2:   return launch_cj<DT, ROUND, THREE, 64, 2>(t, stream);
    case kTeam64x3:   return launch_cj<DT, ROUND, THREE, 64, 3>(t, stream);
    case kTeam64x4:   return launch_cj<DT, ROUND, THREE, 64, 4>(t, stream);
    case kTeam256x2:  return launch_cj<DT, ROUND, THREE, 256, 2>(t, stream);
    case kTeam256x4:  return launch_cj<DT, ROUND, THREE, 256, 4>(t, stream);
    case kTeam1024x2: return launch_cj<DT, ROUND, THREE, 1024, 2>(t, stream);
    case kTeam1024x4: return launch_cj<DT, ROUND, THREE, 1024, 4>(t, stream);
    default:          return hipErrorInvalidValue;
    }
}

template <int DT>
hipError_t launch_codec_jobs_dt(int rounding, int shape, bool three, const JobTable& t, hipStream_t stream) {
    if (rounding == AQSGD_ROUND_STOCHASTIC)
        return three ? launch_cj_shape<DT, AQSGD_ROUND_STOCHASTIC, true>(shape, t, stream)
                     : launch_cj_shape<DT, AQSGD_ROUND_STOCHASTIC, false>(shape, t, stream);
    return three ? launch_cj_shape<DT, AQSGD_ROUND_NEAREST, true>(shape, t, stream)
                 : launch_cj_shape<DT, AQSGD_ROUND_NEAREST, false>(shape, t, stream);
}

template <int DT>
hipError_t launch_dequant_jobs_dt(int unroll, const JobTable& t, hipStream_t stream) {
    const dim3 grid(t.total_blocks), block(kBlock);
    switch (unroll) {
    case 1: return launch_kernel(dequant_jobs_kernel<DT, 1>, grid, block, stream, t);
    case 2: return launch_kernel(dequant_jobs_kernel<DT, 2>, grid, block, stream, t);
    case 4: return launch_kernel(dequant_jobs_kernel<DT, 4>, grid, block, stream, t);
    default: return hipErrorInvalidValue;
    }
}

template <int DT>
hipError_t launch_quant_anyshape_dt(int bits, int rounding, const QuantJob& a, hipStream_t stream) {
    return launch_kernel(quant_anyshape_kernel<DT>, dim3(a.grid_x, a.grid_y), dim3(kBlock), stream, a, bits,
                         rounding);
}

template <int DT>
hipError_t launch_dequant_anyshape_dt(const DequantJob& a, hipStream_t stream) {
    return launch_kernel(dequant_anyshape_kernel<DT>, dim3(a.grid_x, a.grid_y), dim3(kBlock), stream, a);
}

#define AQSGD_INSTANTIATE_DTYPE(DT)                                                               \
    template hipError_t launch_codec_jobs_dt<DT>(int, int, bool, const JobTable&, hipStream_t);   \
    template hipError_t launch_dequant_jobs_dt<DT>(int, const JobTable&, hipStream_t);            \
    template hipError_t launch_quant_anyshape_dt<DT>(int, int, const QuantJob&, hipStream_t);     \
    template hipError_t launch_dequant_anyshape_dt<DT>(const DequantJob&, hipStream_t);

}  // namespace aqsgd
