// Launch tables of one storage dtype: every (bits, rounding, team shape) of the
// quantising kernel and every (bits, unroll) of the dequantising kernel.  Each
// dtype gets its own translation unit so the three compile in parallel.
#pragma once

#include "aqsgd_kernels.h"

namespace aqsgd {

template <int DT, int BITS, int ROUND, int TEAM, int CPL>
static hipError_t launch_qt(LaunchGeom g, const QuantArgs& a, hipStream_t stream) {
    constexpr int threads = TEAM > kWave ? TEAM : kBlock;
    return launch_kernel(quant_team_kernel<DT, BITS, ROUND, TEAM, CPL>, dim3(g.grid_x, g.grid_y),
                         dim3(threads), stream, a);
}

template <int DT, int BITS, int ROUND>
static hipError_t launch_qt_shape(int shape, LaunchGeom g, const QuantArgs& a, hipStream_t stream) {
    switch (shape) {
    case kTeam8x1:    return launch_qt<DT, BITS, ROUND, 8, 1>(g, a, stream);
    case kTeam16x1:   return launch_qt<DT, BITS, ROUND, 16, 1>(g, a, stream);
    case kTeam32x1:   return launch_qt<DT, BITS, ROUND, 32, 1>(g, a, stream);
    case kTeam64x1:   return launch_qt<DT, BITS, ROUND, 64, 1>(g, a, stream);
    case kTeam64x2:   return launch_qt<DT, BITS, ROUND, 64, 2>(g, a, stream);
    case kTeam64x3:   return launch_qt<DT, BITS, ROUND, 64, 3>(g, a, stream);
    case kTeam64x4:   return launch_qt<DT, BITS, ROUND, 64, 4>(g, a, stream);
    case kTeam256x2:  return launch_qt<DT, BITS, ROUND, 256, 2>(g, a, stream);
    case kTeam256x4:  return launch_qt<DT, BITS, ROUND, 256, 4>(g, a, stream);
    case kTeam1024x2: return launch_qt<DT, BITS, ROUND, 1024, 2>(g, a, stream);
    case kTeam1024x4: return launch_qt<DT, BITS, ROUND, 1024, 4>(g, a, stream);
    default:          return hipErrorInvalidValue;
    }
}

template <int DT, int BITS>
static hipError_t launch_qt_round(int rounding, int shape, LaunchGeom g, const QuantArgs& a,
                                  hipStream_t stream) {
    return rounding == AQSGD_ROUND_STOCHASTIC
               ? launch_qt_shape<DT, BITS, AQSGD_ROUND_STOCHASTIC>(shape, g, a, stream)
               : launch_qt_shape<DT, BITS, AQSGD_ROUND_NEAREST>(shape, g, a, stream);
}

template <int DT>
hipError_t launch_quant_team_dt(int bits, int rounding, int shape, LaunchGeom g, const QuantArgs& a,
                                hipStream_t stream) {
    switch (bits) {
    case 2: return launch_qt_round<DT, 2>(rounding, shape, g, a, stream);
    case 3: return launch_qt_round<DT, 3>(rounding, shape, g, a, stream);
    case 4: return launch_qt_round<DT, 4>(rounding, shape, g, a, stream);
    case 6: return launch_qt_round<DT, 6>(rounding, shape, g, a, stream);
    case 8: return launch_qt_round<DT, 8>(rounding, shape, g, a, stream);
    default: return hipErrorInvalidValue;
    }
}

template <int DT, int BITS>
static hipError_t launch_df_unroll(int unroll, LaunchGeom g, const DequantArgs& a, hipStream_t stream) {
    const dim3 grid(g.grid_x, g.grid_y), block(kBlock);
    switch (unroll) {
    case 1: return launch_kernel(dequant_flat_kernel<DT, BITS, 1>, grid, block, stream, a);
    case 2: return launch_kernel(dequant_flat_kernel<DT, BITS, 2>, grid, block, stream, a);
    case 4: return launch_kernel(dequant_flat_kernel<DT, BITS, 4>, grid, block, stream, a);
    default: return hipErrorInvalidValue;
    }
}

template <int DT>
hipError_t launch_dequant_flat_dt(int bits, int unroll, LaunchGeom g, const DequantArgs& a,
                                  hipStream_t stream) {
    switch (bits) {
    case 2: return launch_df_unroll<DT, 2>(unroll, g, a, stream);
    case 3: return launch_df_unroll<DT, 3>(unroll, g, a, stream);
    case 4: return launch_df_unroll<DT, 4>(unroll, g, a, stream);
    case 6: return launch_df_unroll<DT, 6>(unroll, g, a, stream);
    case 8: return launch_df_unroll<DT, 8>(unroll, g, a, stream);
    default: return hipErrorInvalidValue;
    }
}

template <int DT>
hipError_t launch_quant_anyshape_dt(int bits, int rounding, LaunchGeom g, const QuantArgs& a,
                                    hipStream_t stream) {
    return launch_kernel(quant_anyshape_kernel<DT>, dim3(g.grid_x, g.grid_y), dim3(kBlock), stream, a,
                         bits, rounding);
}

template <int DT>
hipError_t launch_dequant_anyshape_dt(int bits, LaunchGeom g, const DequantArgs& a, hipStream_t stream) {
    return launch_kernel(dequant_anyshape_kernel<DT>, dim3(g.grid_x, g.grid_y), dim3(kBlock), stream, a,
                         bits);
}

#define AQSGD_INSTANTIATE_DTYPE(DT)                                                               \
    template hipError_t launch_quant_team_dt<DT>(int, int, int, LaunchGeom, const QuantArgs&,     \
                                                 hipStream_t);                                    \
    template hipError_t launch_dequant_flat_dt<DT>(int, int, LaunchGeom, const DequantArgs&,      \
                                                   hipStream_t);                                  \
    template hipError_t launch_quant_anyshape_dt<DT>(int, int, LaunchGeom, const QuantArgs&,      \
                                                     hipStream_t);                                \
    template hipError_t launch_dequant_anyshape_dt<DT>(int, LaunchGeom, const DequantArgs&,       \
                                                       hipStream_t);

}  // namespace aqsgd
