// gemm_kernel instantiations: MODE_GATEUP, weights row-major ([K, N])
#include "bb_gemm_inst.h"
namespace bb {
template void gemm_dispatch<MODE_GATEUP, false>(int, bool, bool, bool, dim3, hipStream_t, const GemmArgs&);
}
