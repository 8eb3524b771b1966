// The weight-streaming kernels (row-major and transposed weights), the
// reduction kernel of the split contraction, and their launch functions.
#include "bb_gemm.h"
#include "bb_launch.h"
#include "bb_stream.h"
#include "bb_stream_t.h"

namespace bb {

template <int MT>
static int stream_resident_mt(hipError_t* err) {
    int n = 0;
    *err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, ffn_stream_kernel<MT>, STREAM_THREADS, 0);
    return n;
}
int stream_resident(int mt, hipError_t* err) { return mt == 1 ? stream_resident_mt<1>(err) : stream_resident_mt<2>(err); }
void stream_launch(int mt, int G, hipStream_t st, const StreamArgs& a) {
    if (mt == 1) hipLaunchKernelGGL(ffn_stream_kernel<1>, dim3(G), dim3(STREAM_THREADS), 0, st, a);
    else hipLaunchKernelGGL(ffn_stream_kernel<2>, dim3(G), dim3(STREAM_THREADS), 0, st, a);
}
int stream_t_resident(int lds_bytes, hipError_t* err) {
    *err = hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_stream_t_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, STREAMT_LDS);
    if (*err != hipSuccess) return 0;
    int n = 0;
    *err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, ffn_stream_t_kernel, STREAMT_THREADS, lds_bytes);
    return n;
}
void stream_t_launch(int G, int lds_bytes, hipStream_t st, const StreamTArgs& a) {
    hipLaunchKernelGGL(ffn_stream_t_kernel, dim3(G), dim3(STREAMT_THREADS), lds_bytes, st, a);
}

void splitk_reduce_dispatch(int mode, const float* part, const float* ssqpart, unsigned short* C, int M, int N, int K,
                            int ldp, int ldc, int nsplit, float eps, const unsigned short* res, int ldr,
                            hipStream_t st) {
    const size_t threads = (size_t)M * (N / 8);
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    if (mode == MODE_GATEUP)
        hipLaunchKernelGGL((splitk_reduce_kernel<MODE_GATEUP>), grid, block, 0, st, part, ssqpart, C, M, N, K, ldp, ldc,
                           nsplit, eps, res, ldr);
    else
        hipLaunchKernelGGL((splitk_reduce_kernel<MODE_PLAIN>), grid, block, 0, st, part, ssqpart, C, M, N, K, ldp, ldc,
                           nsplit, eps, res, ldr);
}

}  // namespace bb
