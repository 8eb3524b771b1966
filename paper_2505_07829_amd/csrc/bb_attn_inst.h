// Bodies of the attention launch functions: map the run-time launch shape onto
// the instantiations of the attention kernels.  Included by bb_attn_inst_*.hip,
// one source per pair of head dimensions.
#pragma once
#include <type_traits>

#include "bb_attn.h"
#include "bb_launch.h"

namespace bb {

// tail: iterations left after the two-per-trip main loop (1..4); nw: wavefronts per workgroup (4 or 8);
// ksplit > 1: keys split over ksplit workgroups per (problem, query block), then the combine kernel
template <int DK, int DV>
void attn_tiled_launch(int tail, int nw, int ksplit, dim3 grid, dim3 block, hipStream_t st, const AttnArgs& a) {
    auto go_nw = [&](auto NWC) {
        constexpr int NW = decltype(NWC)::value;
        if (tail == 1) hipLaunchKernelGGL((attention_kernel<DK, DV, 1, NW>), grid, block, 0, st, a);
        else if (tail == 2) hipLaunchKernelGGL((attention_kernel<DK, DV, 2, NW>), grid, block, 0, st, a);
        else if (tail == 3) hipLaunchKernelGGL((attention_kernel<DK, DV, 3, NW>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((attention_kernel<DK, DV, 4, NW>), grid, block, 0, st, a);
    };
    if (ksplit > 1) {
        if (tail == 1) hipLaunchKernelGGL((attention_kernel<DK, DV, 1, 4, true>), grid, block, 0, st, a);
        else if (tail == 2) hipLaunchKernelGGL((attention_kernel<DK, DV, 2, 4, true>), grid, block, 0, st, a);
        else if (tail == 3) hipLaunchKernelGGL((attention_kernel<DK, DV, 3, 4, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((attention_kernel<DK, DV, 4, 4, true>), grid, block, 0, st, a);
        hipLaunchKernelGGL((attention_combine_kernel<DV>), dim3((unsigned)((size_t)a.B * a.M)), dim3(64), 0, st,
                           (const float*)a.part, (const float*)a.ml, a.O, ksplit, a.c);
    } else if (nw == 8) {
        go_nw(std::integral_constant<int, 8>{});
    } else {
        go_nw(std::integral_constant<int, 4>{});
    }
}

template <int DK, int DV>
void attn_decode_launch(dim3 grid, hipStream_t st, const AttnArgs& a) {
    hipLaunchKernelGGL((attention_decode_kernel<DK, DV>), grid, dim3(256), 0, st, a);
}

}  // namespace bb
