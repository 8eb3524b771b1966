// Body of gemm_dispatch<MODE, BT>: maps the run-time launch shape onto the
// instantiations of gemm_kernel.  Included by the bb_gemm_inst_*.hip sources,
// each of which instantiates it for one MODE and one weight layout, so that
// the instantiations compile side by side.
#pragma once
#include <type_traits>

#include "bb_gemm.h"
#include "bb_launch.h"

namespace bb {

template <int MODE, bool BT>
void gemm_dispatch(int bm, bool full, bool odd, bool split, dim3 grid, hipStream_t st, const GemmArgs& a) {
    using T = std::true_type;
    using F_ = std::false_type;
    // Complete 256-row tiles run with eight wavefronts (two per SIMD): one wavefront's fragment reads, load-to-LDS
    // instructions and prologue arithmetic issue under the other's matrix instructions.  Without a prologue the
    // wavefronts lie 2 x 4 over the tile (128 x 64 accumulators each; 86 % instead of 78 % of the cycles of a step
    // are matrix cycles, and the chip's clock gives most of that back); with the norm prologue 8 x 1 (32 x 256
    // each), so that no A fragment is prepared twice (kernel traces: c3's gate/up with the statistics in the loop
    // 362 -> 336 us, c5's LN product 1035-1100 -> 991 us).  Transposed weights: c3's gate/up 295 -> 287 us, c5's
    // product 861 -> 827 us (relative to the row-major kernels of the same runs).
    auto go = [&](auto BMc, auto FULLc, auto ODDc, auto SPLITc) {
        constexpr int BM = decltype(BMc)::value;
        constexpr bool FULL = decltype(FULLc)::value;
        constexpr int NW = (BM == 256 && FULL) ? 8 : 4;
        hipLaunchKernelGGL((gemm_kernel<MODE, BM, FULL, decltype(ODDc)::value, decltype(SPLITc)::value, BT, NW>), grid,
                           dim3(64 * NW), 0, st, a);
    };
    auto by_odd = [&](auto BMc, auto FULLc, auto SPLITc) {
        if (odd) go(BMc, FULLc, T(), SPLITc); else go(BMc, FULLc, F_(), SPLITc);
    };
    using B128 = std::integral_constant<int, 128>;
    using B256 = std::integral_constant<int, 256>;
    if (split) {
        if constexpr (MODE == MODE_PLAIN || MODE == MODE_GATEUP) {
            if (bm == 256) {
                // (PLAIN only) 256-row tiles; complete tiles and equal shares of the contraction run without bounds checks
                if constexpr (MODE == MODE_PLAIN) {
                    if (full) by_odd(B256(), T(), T()); else by_odd(B256(), F_(), T());
                }
            } else {
                by_odd(B128(), F_(), T());
            }
        }
        return;
    }
    if (bm == 256) {
        if (full) by_odd(B256(), T(), F_()); else by_odd(B256(), F_(), F_());
    } else {
        if (full) by_odd(B128(), T(), F_()); else by_odd(B128(), F_(), F_());
    }
}

}  // namespace bb
