// gemm_kernel instantiations: MODE_LN, weights transposed ([N, K])
#include "bb_gemm_inst.h"
namespace bb {
template void gemm_dispatch<MODE_LN, true>(int, bool, bool, bool, dim3, hipStream_t, const GemmArgs&);
}
