// gemm_kernel instantiations: MODE_LN, weights row-major ([K, N])
#include "bb_gemm_inst.h"
namespace bb {
template void gemm_dispatch<MODE_LN, false>(int, bool, bool, bool, dim3, hipStream_t, const GemmArgs&);
}
