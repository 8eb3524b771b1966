// The fully fused nest for small model dimensions and its launch function.
#include "bb_nest.h"
#include "bb_launch.h"

namespace bb {

void nest_launch(int nd, int grid, hipStream_t st, const NestArgs& a) {
    if (nd <= 2) hipLaunchKernelGGL(ffn_nest_kernel<2>, dim3(grid), dim3(64 * nest_waves(2)), 0, st, a);
    else hipLaunchKernelGGL(ffn_nest_kernel<4>, dim3(grid), dim3(64 * nest_waves(4)), 0, st, a);
}

}  // namespace bb
