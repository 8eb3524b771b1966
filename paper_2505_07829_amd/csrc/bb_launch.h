// Kernel launches across translation units.  The library is built from several
// sources compiled side by side (one per family of kernel instantiations);
// bb_api.hip owns validation, workspace and variant selection and reaches the
// kernels through the functions declared here.  A launch function only enqueues:
// the caller checks hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>

namespace bb {

struct GemmArgs;
struct StreamArgs;
struct StreamTArgs;
struct AttnArgs;
struct NestArgs;

// gemm_kernel<MODE, bm, full, odd, split, bt> on `grid` workgroups (defined per MODE and per weight
// layout in bb_gemm_inst_*.hip); split launches exist for MODE_PLAIN and MODE_GATEUP only
template <int MODE, bool BT>
void gemm_dispatch(int bm, bool full, bool odd, bool split, dim3 grid, hipStream_t st, const GemmArgs& a);

// splitk_reduce_kernel<mode> (mode = MODE_PLAIN or MODE_GATEUP)
void splitk_reduce_dispatch(int mode, const float* part, const float* ssqpart, unsigned short* C, int M, int N, int K,
                            int ldp, int ldc, int nsplit, float eps, const unsigned short* res, int ldr,
                            hipStream_t st);

// streaming kernels: workgroups of the kernel one compute unit can hold (hipError_t in *err), launch
// (row-major weights: ffn_stream_kernel<mt>, mt = 1 or 2 groups of 16 rows)
int stream_resident(int mt, hipError_t* err);
void stream_launch(int mt, int G, hipStream_t st, const StreamArgs& a);
int stream_t_resident(int lds_bytes, hipError_t* err);
void stream_t_launch(int G, int lds_bytes, hipStream_t st, const StreamTArgs& a);

// fully fused nest for small model dimensions: ffn_nest_kernel<nd>, nd = blocks of 128 model channels (2 or 4)
void nest_launch(int nd, int grid, hipStream_t st, const NestArgs& a);

// attention: tiled kernel (ksplit > 1: split keys + combine kernel), one-query streaming kernel
// (defined per pair of head dimensions in bb_attn_inst_*.hip)
template <int DK, int DV>
void attn_tiled_launch(int tail, int nw, int ksplit, dim3 grid, dim3 block, hipStream_t st, const AttnArgs& a);
template <int DK, int DV>
void attn_decode_launch(dim3 grid, hipStream_t st, const AttnArgs& a);

}  // namespace bb
