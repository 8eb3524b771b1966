// C ABI of the bb library: argument validation, workspace management, variant
// selection and kernel launches.  See include/bb.h for the contract.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>

#include "../../include/bb.h"
#define BB_HOST_ONLY        // the streaming kernels themselves are compiled in bb_stream_inst.hip
#include "bb_attn.h"
#include "bb_gemm.h"
#include "bb_launch.h"
#include "bb_misc.h"
#include "bb_stream.h"
#include "bb_stream_t.h"
#include "bb_nest.h"

namespace {

using namespace bb;

constexpr int64_t kStreamMaxM = 16 * STREAM_MAXMT;   // rows the weight-streaming kernel handles (row-major weights)
constexpr int64_t kStreamTMaxM = 16;  // rows the weight-streaming kernel for transposed weights handles
constexpr int64_t kPrescaleFloorM = 16; // up to this many rows no room is planned for BB_VARIANT_PRESCALE's gain-scaled copy of X
constexpr int64_t kNestAutoMaxD = 256, kNestAutoMaxF = 768, kNestAutoMaxM = 16 * 256;   // shapes on which AUTO runs the fully fused nest
constexpr int64_t kPrescaleMinM = 256; // rows from which AUTO runs the statistics loop as a kernel of its own
constexpr size_t kAlign = 256;

std::mutex g_mu;
int g_variant = -1;                    // -1: not yet read from the environment
int g_last_hip = 0;
int g_log = -1;

struct Workspace {
    void* ptr = nullptr;
    size_t bytes = 0;
    bool user = false;
    size_t clean = 0;                  // leading bytes known to be zero
    size_t attn_zone = 0;              // leading bytes that hold arrival counters of bb_attention, all zero
    int device = -1;
} g_ws;

// optional per-kernel timing of the most recent calls (bb_profile_*): a ring of the last kProfRing
// operator calls, so that a caller can time kernels inside a run of back-to-back calls
constexpr int kMaxProf = 8;
constexpr int kProfRing = 64;
struct ProfCall {
    int n = 0;                         // kernels recorded by this call
    hipEvent_t ev[kMaxProf + 1] = {};
    const char* name[kMaxProf] = {};
};
struct Profile {
    bool on = false;
    bool created = false;
    long calls = 0;                    // operator calls recorded since profiling was switched on
    ProfCall ring[kProfRing];
    ProfCall& cur() { return ring[(calls + kProfRing - 1) % kProfRing]; }   // the most recent call (calls >= 1)
} g_prof;

struct DeviceInfo {
    bool known = false;
    bool gfx950 = false;
    int cus = 0;
    // one word of pinned host memory the streaming kernels write when a bounded wait on another workgroup
    // gives up (mapped into the device: the kernels store to fault_dev, the host reads *fault_host)
    volatile unsigned* fault_host = nullptr;
    unsigned* fault_dev = nullptr;
    // this device's copy of the static scratch array (bb_rmsnorm_swiglu_ffn_static) and what is known of its contents
    void* static_ptr = nullptr;
    size_t static_clean = 0;
} g_dev[64];

// Scratch of bb_rmsnorm_swiglu_ffn_static, the entry point for callers that must not allocate.  Every
// device the library is loaded on holds its own copy until the process ends.  In host code this name is a
// stand-in, not an address: the device address comes from hipGetSymbolAddress (current_device_info).
__device__ __align__(256) unsigned char scratch[BB_STATIC_SCRATCH_BYTES];
unsigned g_spin_limit = 8000000u;      // polls after which a wait on another workgroup gives up (about two seconds)

bool log_on() {
    if (g_log < 0) g_log = std::getenv("BB_LOG") ? 1 : 0;
    return g_log == 1;
}

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

int hip_fail(hipError_t e) {
    g_last_hip = (int)e;
    (void)hipGetLastError();
    return BB_ERR_HIP;
}

#define BB_HIP(expr)                                   \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return hip_fail(e_);     \
    } while (0)

int current_device_info(const DeviceInfo** out) {
    int dev = 0;
    BB_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return BB_ERR_ARCH;
    DeviceInfo& d = g_dev[dev];
    if (!d.known) {
        hipDeviceProp_t prop;
        BB_HIP(hipGetDeviceProperties(&prop, dev));
        d.gfx950 = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0;
        d.cus = prop.multiProcessorCount;
        if (d.gfx950 && d.fault_host == nullptr) {
            void* h = nullptr;
            void* dp = nullptr;
            BB_HIP(hipHostMalloc(&h, 64, hipHostMallocMapped));
            *reinterpret_cast<volatile unsigned*>(h) = 0u;
            BB_HIP(hipHostGetDevicePointer(&dp, h, 0));
            d.fault_host = reinterpret_cast<volatile unsigned*>(h);
            d.fault_dev = reinterpret_cast<unsigned*>(dp);
        }
        if (d.gfx950 && d.static_ptr == nullptr) {
            void* sp = nullptr;
            BB_HIP(hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)));
            if (sp == nullptr || ((uintptr_t)sp & (kAlign - 1))) return BB_ERR_WORKSPACE;
            d.static_ptr = sp;
            d.static_clean = 0;        // (zero when the code object was loaded; cleared anyway before the first use)
        }
        d.known = true;
    }
    *out = &d;
    return d.gfx950 ? BB_OK : BB_ERR_ARCH;
}

int read_variant() {
    if (g_variant < 0) {
        g_variant = BB_VARIANT_AUTO;
        if (const char* e = std::getenv("BB_VARIANT")) {
            if (!std::strcmp(e, "stream")) g_variant = BB_VARIANT_STREAM;
            else if (!std::strcmp(e, "snapshot1")) g_variant = BB_VARIANT_SNAPSHOT1;
            else if (!std::strcmp(e, "unfused")) g_variant = BB_VARIANT_UNFUSED;
            else if (!std::strcmp(e, "prescale")) g_variant = BB_VARIANT_PRESCALE;
            else if (!std::strcmp(e, "nest")) g_variant = BB_VARIANT_NEST;
        }
    }
    return g_variant;
}

// measured selections (bb_*_tune): (op, M, D, F or N) -> variant
struct TuneKey {
    int op;
    int64_t M, D, FN;
    bool operator<(const TuneKey& o) const {
        return std::tie(op, M, D, FN) < std::tie(o.op, o.M, o.D, o.FN);
    }
};
std::map<TuneKey, int> g_tuned;

// AUTO: a measured selection for exactly this shape if there is one, else the rule of thumb
// (the fully fused nest for small weight matrices, else the weight-streaming kernel up to kStreamMaxM rows and
// the tiled kernels beyond; LN always fused)
int auto_variant(int op, int64_t M, int64_t D, int64_t FN) {
    auto it = g_tuned.find(TuneKey{op, M, D, FN});
    if (it != g_tuned.end()) return it->second;
    // (measured on D = 4096, F = 11008: from 256 rows on the separate statistics pass beats the
    // statistics inside the product loop by 7-9 %; below, the split contraction needs the fused form)
    if (op == BB_OP_RMSNORM_SWIGLU_FFN) {
        // The fully fused nest (one launch, a block of 16 rows per compute unit, which reads all three weight
        // matrices alone) where its six wavefront pairs take all hidden blocks in one trip: measured 10-19 us against
        // 15-35 us for the best other program on 16...4096 rows of 64 x 256, 128 x 768, 192 x 768, 256 x 704 and
        // 256 x 768 (D x F).  With a second trip (F = 1024...1536) it wins only from some thousand rows on, with
        // D > 256 (four pairs, twice the steps per block) nowhere: left to the measured selection.  Beyond 4096 rows
        // (more blocks of 16 rows than compute units: a second round) the tiled kernels win again.
        if (D <= kNestAutoMaxD && FN <= kNestAutoMaxF && M <= kNestAutoMaxM) return BB_VARIANT_NEST;
        if (M <= kStreamMaxM) return BB_VARIANT_STREAM;
        return M >= kPrescaleMinM ? BB_VARIANT_PRESCALE : BB_VARIANT_SNAPSHOT1;
    }
    return M >= kPrescaleMinM ? BB_VARIANT_PRESCALE : BB_VARIANT_SNAPSHOT1;
}

int ffn_locked(int variant, const void* X, const void* g, const void* W1, const void* W3, const void* W2,
               void* Y, int64_t M, int64_t D, int64_t F, float eps, void* stream, const void* R = nullptr);
int ffn_unfused_locked(const void* X, const void* g, const void* W1, const void* W3, const void* W2, void* Y,
                       int64_t M, int64_t D, int64_t F, float eps, void* stream);
int ln_locked(int variant, const void* X, const void* gamma, const void* beta, const void* W, void* Y,
              int64_t M, int64_t D, int64_t N, float eps, void* stream);
int ffn_t_locked(const void* X, const void* g, const void* W1t, const void* W3t, const void* W2t, void* Y,
                 int64_t M, int64_t D, int64_t F, float eps, void* stream, const void* R);
int ln_unfused_locked(const void* X, const void* gamma, const void* beta, const void* W, void* Y, int64_t M,
                      int64_t D, int64_t N, float eps, void* stream);

void prof_begin(hipStream_t st) {
    if (!g_prof.on) return;
    ++g_prof.calls;
    ProfCall& c = g_prof.cur();
    c.n = 0;
    (void)hipEventRecord(c.ev[0], st);
}
void prof_mark(const char* name, hipStream_t st) {
    if (!g_prof.on || g_prof.calls == 0) return;
    ProfCall& c = g_prof.cur();
    if (c.n >= kMaxProf) return;
    c.name[c.n] = name;
    ++c.n;
    (void)hipEventRecord(c.ev[c.n], st);
}

// ---------------------------------------------------------------- validation
bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}
bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

int check_dims(int64_t M, int64_t D, int64_t F) {
    if (M < 0 || D <= 0 || F <= 0) return BB_ERR_SHAPE;
    if ((D & 7) || (F & 7)) return BB_ERR_SHAPE;
    // int32 indexing inside tiles: leading dimensions and tile counts must fit
    if (D > (1 << 24) || F > (1 << 24) || M > (1 << 24)) return BB_ERR_SHAPE;
    return BB_OK;
}
int check_eps(float eps) { return (std::isfinite(eps) && eps >= 0.f) ? BB_OK : BB_ERR_EPS; }

int validate_ffn(const void* X, const void* g, const void* W1, const void* W3, const void* W2, void* Y,
                 int64_t M, int64_t D, int64_t F, float eps) {
    if (int rc = check_dims(M, D, F)) return rc;
    if (int rc = check_eps(eps)) return rc;
    if (M == 0) return BB_OK;
    if (!X || !g || !W1 || !W3 || !W2 || !Y) return BB_ERR_NULL;
    if (misaligned(X) || misaligned(g) || misaligned(W1) || misaligned(W3) || misaligned(W2) || misaligned(Y))
        return BB_ERR_ALIGN;
    const size_t ny = (size_t)M * D * 2, nw = (size_t)D * F * 2;
    if (overlaps(Y, ny, X, ny) || overlaps(Y, ny, g, (size_t)D * 2) || overlaps(Y, ny, W1, nw) ||
        overlaps(Y, ny, W3, nw) || overlaps(Y, ny, W2, nw))
        return BB_ERR_ALIAS;
    return BB_OK;
}

// Y = R + FFN(X): R [M, D].  R may be X.  Y may be R itself (in place; then it may also be X, which
// every kernel has finished reading before the last one writes), otherwise Y overlaps nothing.
int validate_ffn_residual(const void* X, const void* g, const void* W1, const void* W3, const void* W2,
                          const void* R, void* Y, int64_t M, int64_t D, int64_t F, float eps) {
    if (int rc = check_dims(M, D, F)) return rc;
    if (int rc = check_eps(eps)) return rc;
    if (M == 0) return BB_OK;
    if (!X || !g || !W1 || !W3 || !W2 || !R || !Y) return BB_ERR_NULL;
    if (misaligned(X) || misaligned(g) || misaligned(W1) || misaligned(W3) || misaligned(W2) || misaligned(R) ||
        misaligned(Y))
        return BB_ERR_ALIGN;
    const size_t ny = (size_t)M * D * 2, nw = (size_t)D * F * 2;
    const bool in_place = (Y == R);
    if (!in_place && overlaps(Y, ny, R, ny)) return BB_ERR_ALIAS;
    if (!(in_place && R == X) && overlaps(Y, ny, X, ny)) return BB_ERR_ALIAS;
    if (overlaps(Y, ny, g, (size_t)D * 2) || overlaps(Y, ny, W1, nw) || overlaps(Y, ny, W3, nw) ||
        overlaps(Y, ny, W2, nw))
        return BB_ERR_ALIAS;
    return BB_OK;
}

int validate_ln(const void* X, const void* gamma, const void* beta, const void* W, void* Y, int64_t M,
                int64_t D, int64_t N, float eps) {
    if (int rc = check_dims(M, D, N)) return rc;
    if (int rc = check_eps(eps)) return rc;
    if (M == 0) return BB_OK;
    if (!X || !gamma || !beta || !W || !Y) return BB_ERR_NULL;
    if (misaligned(X) || misaligned(gamma) || misaligned(beta) || misaligned(W) || misaligned(Y))
        return BB_ERR_ALIGN;
    const size_t ny = (size_t)M * N * 2;
    if (overlaps(Y, ny, X, (size_t)M * D * 2) || overlaps(Y, ny, gamma, (size_t)D * 2) ||
        overlaps(Y, ny, beta, (size_t)D * 2) || overlaps(Y, ny, W, (size_t)D * N * 2))
        return BB_ERR_ALIAS;
    return BB_OK;
}

// ------------------------------------------------------------ workspace plan
struct StreamPlan {
    size_t bar_off, zero_off, epoch_off, cnt_off, zone_bytes, ppart_off, spart_off, h_off, ypart_off, total_bytes;
    int MT, Fp, nkb1, nfb, items1, per1, S1, nkb2, nnb, items2, per2, S2;
};

// groups of 16 rows the streaming kernel is instantiated for
int stream_mt(int64_t M) { return M <= 16 ? 1 : 2; }

// Layout of the streaming kernels' scratch for G workgroups and M rows.  Only the "zone"
// (barrier words, a block of zeros that nothing ever writes, the kernels' count of completed grid
// barriers, and the arrival counters of the output blocks) has to be zero before the first call: the
// barrier words and the count only ever increase, a counter is put back to zero by the workgroup that
// sees it complete, and only the kernels touch them.
StreamPlan stream_plan(int64_t M, int64_t D, int64_t F, int G) {
    StreamPlan s;
    s.MT = stream_mt(M);
    s.Fp = (int)((F + 127) / 128 * 128);
    s.nkb1 = (int)((D + 31) / 32);
    s.nfb = (int)((F + 127) / 128);
    s.items1 = s.nkb1 * s.nfb;
    s.per1 = std::max((s.items1 + G - 1) / G, 1);
    s.S1 = (s.nkb1 - 1) / s.per1 + 2;
    s.nkb2 = (int)((F + 31) / 32);
    s.nnb = (int)((D + 127) / 128);
    s.items2 = s.nkb2 * s.nnb;
    s.per2 = std::max((s.items2 + G - 1) / G, 1);
    s.S2 = (s.nkb2 - 1) / s.per2 + 2;
    s.bar_off = 0;
    s.zero_off = align_up((size_t)BAR_WORDS * 4);               // 256 bytes that stay zero
    s.epoch_off = s.zero_off + kAlign;                          // the kernels' count of completed grid barriers
    s.cnt_off = s.epoch_off + kAlign;
    s.zone_bytes = s.cnt_off + align_up((size_t)s.nnb * 4);
    s.ppart_off = s.zone_bytes;
    s.spart_off = s.ppart_off + align_up((size_t)s.nfb * s.S1 * s.MT * 4096 * 4);
    s.h_off = s.spart_off + align_up((size_t)s.S1 * 16 * s.MT * 4);
    s.ypart_off = s.h_off + align_up((size_t)16 * s.MT * s.Fp * 2);
    s.total_bytes = s.ypart_off + align_up((size_t)s.nnb * s.S2 * s.MT * 2048 * 4);
    return s;
}

constexpr int kPlanCUs = 256;   // workgroups assumed by bb_workspace_bytes (one per compute unit of an MI355X)

// Split contraction: with fewer 128-row tiles than half the compute units (few
// rows), nsplit workgroups share a tile's contraction range.  Returns nsplit
// (1 = no split) and the steps per workgroup.
// A second case (PLAIN only, *bm = 256): at most half as many 256-row tiles as
// compute units, a long contraction, and either too many 128-row tiles for
// the first case or at least 512 rows: 256-row tiles, which need fewer loads
// per flop, with the contraction split so that every compute unit gets one.
int plan_split(int mode, int M, int N, int K, int cus, int* nk_split, int* bm = nullptr) {
    const int ncol = (mode == MODE_GATEUP || mode == MODE_GATEUP_PRE) ? 128 : 256;
    int tiles = ((M + 127) / 128) * ((N + ncol - 1) / ncol);
    const int nk = (K + GEMM_BK - 1) / GEMM_BK;
    *nk_split = nk;
    if (bm) *bm = 128;
    if (mode == MODE_LN || mode == MODE_GATEUP_PRE || mode == MODE_LN_PRE) return 1;
    const int tiles256 = ((M + 255) / 256) * ((N + ncol - 1) / ncol);
    const bool can256 = mode == MODE_PLAIN && M >= 256 && tiles256 * 2 <= cus && nk >= 64;
    // (measured on D=4096, F=11008: from 512 rows on the 256-row tiles win also where 128-row tiles could split)
    if (tiles * 2 > cus || (can256 && M >= 512)) {
        if (!can256) return 1;
        tiles = tiles256;
        if (bm) *bm = 256;
    }
    int S = std::min(std::min(cus / tiles, 16), nk / 4);     // at least four steps per workgroup
    if (S < 2) return 1;
    const int per = (nk + S - 1) / S;
    S = (nk + per - 1) / per;                                // no workgroup without a step
    *nk_split = per;
    return S;
}
// bytes of partial results a split launch of this shape needs (0 = not split)
size_t split_bytes(int mode, int64_t M, int64_t N, int64_t K, int cus) {
    int per = 0;
    const int S = plan_split(mode, (int)M, (int)N, (int)K, cus, &per);
    if (S < 2) return 0;
    const size_t cols = (mode == MODE_GATEUP) ? 2 * (size_t)N : (size_t)N;
    return align_up((size_t)S * M * cols * 4) + align_up((size_t)S * M * 4);
}


// Key splits of the attention kernel for `wgs` (problem, query block) pairs and nt key blocks:
// the largest divisor of nt that keeps about two workgroups per compute unit and at least two
// key blocks per workgroup; 1 = no split (enough workgroups already, or a short sequence).
// arrival counters of attention_decode_kernel, one per problem, at the workspace's start
size_t attn_zone_bytes(int64_t B) { return align_up((size_t)B * 4); }

// One query per problem: blocks of 64 keys per wavefront of attention_decode_kernel (a workgroup has four), so
// that the launch has about three workgroups per compute unit; *nsplit = workgroups per problem.
int attn_decode_plan(int64_t B, int64_t N, int cus, int64_t* nsplit) {
    const int64_t nblocks = (N + ATTN_BK - 1) / ATTN_BK, units = B * ((nblocks + 3) / 4);
    const int64_t per = std::min<int64_t>(std::max<int64_t>((units + 3 * cus - 1) / (3 * (int64_t)cus), 1), 64);
    *nsplit = (nblocks + 4 * per - 1) / (4 * per);
    return (int)per;
}

int attn_key_splits(int64_t wgs, int64_t nt, int cus) {
    if (wgs * 2 > cus || nt < 8) return 1;
    const int64_t target = std::min<int64_t>((2 * (int64_t)cus) / wgs, nt / 2);
    for (int64_t s = target; s >= 2; --s)
        if (nt % s == 0) return (int)s;
    return 1;
}

size_t zone_bytes(int op, int64_t M, int64_t D, int64_t F) {
    if (op == BB_OP_RMSNORM_SWIGLU_FFN && M <= kStreamMaxM) return stream_plan(M, D, F, kPlanCUs).total_bytes;
    return 0;
}

size_t scratch_bytes(int op, int64_t M, int64_t D, int64_t F) {
    switch (op) {
        // (the FFN ops end with room for the partial results of a split contraction)
        case BB_OP_RMSNORM_SWIGLU_FFN:      // hidden | partial results of a split | gain-scaled X and inverse norms (PRESCALE)
            return align_up((size_t)M * F * 2) +
                   std::max(split_bytes(MODE_GATEUP, M, F, D, kPlanCUs), split_bytes(MODE_PLAIN, M, D, F, kPlanCUs)) +
                   (M > kPrescaleFloorM ? align_up((size_t)M * D * 2) + align_up((size_t)M * 4) : 0);
        case BB_OP_LAYERNORM_MATMUL:        // column vectors and their partial sums | gamma-scaled X and row statistics (PRESCALE)
            return (2 + 2 * COLVEC_SPLITS) * align_up((size_t)F * 4) + align_up((size_t)M * D * 2) +
                   align_up((size_t)M * 8);
        case BB_OP_RMSNORM_SWIGLU_FFN_UNFUSED:
            return align_up((size_t)M * D * 2) + 3 * align_up((size_t)M * F * 2) +
                   std::max(split_bytes(MODE_PLAIN, M, F, D, kPlanCUs), split_bytes(MODE_PLAIN, M, D, F, kPlanCUs));
        case BB_OP_LAYERNORM_MATMUL_UNFUSED: return align_up((size_t)M * D * 2);
        default: return 0;
    }
}

// Makes sure a workspace of `need` bytes exists on the current device.
int ensure_workspace(size_t need) {
    int dev = 0;
    BB_HIP(hipGetDevice(&dev));
    if (g_ws.user) return (g_ws.bytes >= need) ? BB_OK : BB_ERR_WORKSPACE;
    if (g_ws.ptr && g_ws.device == dev && g_ws.bytes >= need) return BB_OK;
    if (g_ws.ptr) {
        BB_HIP(hipDeviceSynchronize());
        BB_HIP(hipFree(g_ws.ptr));
        g_ws = Workspace();
    }
    void* p = nullptr;
    BB_HIP(hipMalloc(&p, need));
    g_ws.ptr = p;
    g_ws.bytes = need;
    g_ws.user = false;
    g_ws.clean = 0;
    g_ws.device = dev;
    if (log_on()) std::fprintf(stderr, "[bb] workspace %zu bytes allocated\n", need);
    return BB_OK;
}

int fill_zero(void* p, size_t bytes, hipStream_t st) {
    const size_t n16 = bytes / 16;
    const int grid = (int)std::min<size_t>((n16 + 255) / 256, 2048);
    if (grid == 0) return BB_OK;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, st, (u32x4*)p, n16);
    BB_HIP(hipGetLastError());
    return BB_OK;
}

// scratch region [off, off+len) is about to be written: it is no longer zero
void mark_dirty(size_t off) {
    if (off < g_ws.clean) g_ws.clean = off;
    if (off < g_ws.attn_zone) g_ws.attn_zone = 0;
}

// ------------------------------------------------------------------- launches
// Row tiles per group of the tile order (see gemm_kernel's tile coordinates).  The 32 workgroups that an XCD runs
// together should need few distinct operand tiles: its L2 fetches each of them over the fabric once per step.  With
// g row tiles and 32 / g column tiles that is g A tiles + 32 / g B tiles; measured (gate/up of 4096 x 8192 x 28672,
// ms): g = 16 (the order by columns) 3.07, 8 2.81, 4 2.76, 2 2.85, 1 3.08; the product of 8192 x 4096 x 16384: 32
// 0.946, 8 0.845, 4 0.830.  Four beats eight although both fetch 12 tiles: an A tile is 256 pieces of 128 bytes, a B
// tile 64 pieces of 512.  128-row tiles have A tiles of half the size: eight.  BB_GROUP_M overrides (measurements).
int gemm_group_m(int BM) {
    static const int forced = [] { const char* e = std::getenv("BB_GROUP_M"); return e ? std::atoi(e) : 0; }();
    return forced > 0 ? forced : (BM == 256 ? 4 : 8);
}
// `split`: device scratch of split_bytes(...) for this launch, or nullptr (never split).
// BT: B0/B1 are given transposed ([N, K] row-major, ldb = K).
template <int MODE, bool BT = false>
int launch_gemm(const u16* A, int lda, const u16* B0, const u16* B1, int ldb, u16* C, int ldc,
                const u16* gain, const float* colc, const float* colb, int M, int N, int K, float eps,
                int cus, hipStream_t st, void* split = nullptr, const u16* res = nullptr, int ldr = 0,
                const float* rowstat = nullptr) {
    GemmArgs a;
    a.res = res; a.ldr = ldr; a.rowstat = rowstat;
    a.nsplit = 1; a.nk_split = 0; a.ldp = 0; a.part = nullptr; a.ssqpart = nullptr;
    a.A = A; a.B0 = B0; a.B1 = B1; a.C = C; a.gain = gain; a.colc = colc; a.colb = colb;
    a.M = M; a.N = N; a.K = K; a.lda = lda; a.ldb = ldb; a.ldc = ldc; a.eps = eps;
    const int ncol = (MODE == MODE_GATEUP || MODE == MODE_GATEUP_PRE) ? 128 : 256;
    a.tiles_n = (N + ncol - 1) / ncol;
    const int tiles256 = ((M + 255) / 256) * a.tiles_n;
    int nk_split = 0, split_bm = 128;
    // (planned for kPlanCUs compute units whatever the device has: the scratch for the partial results was sized with
    // that plan, and a plan for fewer units can ask for more splits than it has room for)
    const int nsplit = split ? plan_split(MODE, M, N, K, kPlanCUs, &nk_split, &split_bm) : 1;
    const bool do_split = nsplit >= 2;
    // 256-row tiles or 128-row tiles: whichever needs less time for its rounds on `cus` compute units.  A 128-row
    // tile costs about 0.75 of a 256-row tile (the same weight loads for half the flops, one wavefront per SIMD).
    // E.g. 512 rows of c3's gate/up: 172 tiles of 256 rows in one round against 344 of 128 rows in two; 640 rows:
    // 258 tiles of 256 rows would need a second round for two tiles, 430 of 128 rows take two short rounds
    const int tiles128 = ((M + 127) / 128) * a.tiles_n;
    const int rounds256 = (tiles256 + cus - 1) / cus, rounds128 = (tiles128 + cus - 1) / cus;
    const bool big = do_split ? split_bm == 256 : (M >= 256 && 100 * rounds256 <= 75 * rounds128);
    const int BM = big ? 256 : 128;
    a.tiles_m = (M + BM - 1) / BM;
    a.group_m = std::min(a.tiles_m, gemm_group_m(BM));
    const int tiles = a.tiles_m * a.tiles_n;
    if (do_split) {
        a.nsplit = nsplit;
        a.nk_split = nk_split;
        a.ldp = (MODE == MODE_GATEUP) ? 2 * N : N;
        a.part = (float*)split;
        a.ssqpart = (float*)((char*)split + align_up((size_t)nsplit * M * a.ldp * 4));
    }
    a.tiles_per_xcd = (tiles * a.nsplit + 7) / 8;
    const dim3 grid(8 * a.tiles_per_xcd), block(GEMM_THREADS);
    if (log_on())
        std::fprintf(stderr, "[bb] gemm mode %d%s BM %d M %d N %d K %d tiles %dx%d split %d x %d steps\n", MODE,
                     BT ? " (B transposed)" : "", BM, M, N, K, a.tiles_m, a.tiles_n, a.nsplit,
                     do_split ? nk_split : (K + GEMM_BK - 1) / GEMM_BK);
    // tiles complete in the contraction (any number of rows and columns: a ragged last tile reads its last valid row
    // or chunk of columns in place of the missing ones and stores only the valid elements), and operands small
    // enough for the kernels' 32-bit byte offsets
    const size_t bbytes = BT ? (size_t)N * ldb * 2 : (size_t)K * ldb * 2;
    const bool small = (size_t)M * lda * 2 < (1ull << 32) && bbytes < (1ull << 32);
    const bool full = (K % GEMM_BK == 0) && small;
    const bool odd = ((do_split ? nk_split : (K + GEMM_BK - 1) / GEMM_BK) & 1) != 0;
    if (do_split) {
        constexpr int SM = (MODE == MODE_PLAIN || MODE == MODE_GATEUP) ? MODE : MODE_PLAIN;   // (the others are never split)
        // 256-row tiles (PLAIN only): complete tiles and equal shares of the contraction run without bounds checks
        const bool sfull = big && full && ((K + GEMM_BK - 1) / GEMM_BK) % nsplit == 0;
        gemm_dispatch<SM, BT>(BM, sfull, odd, true, grid, st, a);
        BB_HIP(hipGetLastError());
        splitk_reduce_dispatch(SM, (const float*)a.part, (const float*)a.ssqpart, C, M, N, K, a.ldp, ldc, nsplit, eps,
                               res, ldr, st);
    } else {
        gemm_dispatch<MODE, BT>(BM, full, odd, false, grid, st, a);
    }
    BB_HIP(hipGetLastError());
    prof_mark(MODE == MODE_GATEUP ? "gemm_gateup" : MODE == MODE_GATEUP_PRE ? "gemm_gateup_prescaled"
              : MODE == MODE_LN ? "gemm_ln" : MODE == MODE_LN_PRE ? "gemm_ln_prescaled" : "gemm_plain", st);
    return BB_OK;
}

// the barrier words of the streaming kernels must be zero before their first use in a workspace
int prepare_barrier_zone(const StreamPlan& sp, hipStream_t st) {
    g_ws.attn_zone = 0;                // (the streaming kernels leave their own words there)
    if (g_ws.clean < sp.zone_bytes) {
        if (int rc = fill_zero(g_ws.ptr, sp.zone_bytes, st)) return rc;
        g_ws.clean = sp.zone_bytes;
    }
    return BB_OK;
}

// A streaming kernel of an earlier launch on this device gave up a bounded wait on another workgroup (it
// did not have the whole device, or its synchronisation words had been overwritten): that launch's output is
// invalid.  Reported ONCE, by the first call that notices; the flag is cleared and the zone is zeroed again
// before the next launch (the barrier words and the kernels' count of completed barriers start over).
int check_fault(const DeviceInfo* dev) {
    if (dev->fault_host == nullptr || *dev->fault_host == 0u) return BB_OK;
    *dev->fault_host = 0u;
    g_ws.clean = 0;
    g_ws.attn_zone = 0;
    g_dev[dev - g_dev].static_clean = 0;
    if (log_on()) std::fprintf(stderr, "[bb] a streaming kernel gave up a wait on another workgroup\n");
    return BB_ERR_TIMEOUT;
}

int run_stream(const u16* X, const u16* g, const u16* W1, const u16* W3, const u16* W2, const u16* R, u16* Y, int M,
               int D, int F, float eps, const DeviceInfo* dev, hipStream_t st) {
    const int cus = dev->cus;
    const int G = std::min(cus, kPlanCUs);
    const StreamPlan sp = stream_plan(M, D, F, G);
    static int resident[STREAM_MAXMT + 1] = {-1, -1, -1};   // workgroups of the kernel one compute unit can hold
    if (resident[sp.MT] < 0) {
        hipError_t e = hipSuccess;
        const int n = stream_resident(sp.MT, &e);
        BB_HIP(e);
        resident[sp.MT] = n;
    }
    if (resident[sp.MT] < 1) return BB_ERR_VARIANT;   // the grid barrier needs every workgroup resident
    char* base = (char*)g_ws.ptr;
    if (int rc = prepare_barrier_zone(sp, st)) return rc;
    StreamArgs a;
    a.X = X; a.g = g; a.W1 = W1; a.W3 = W3; a.W2 = W2; a.Y = Y; a.R = R;
    a.ppart = (float*)(base + sp.ppart_off);
    a.spart = (float*)(base + sp.spart_off);
    a.H = (u16*)(base + sp.h_off);
    a.ypart = (float*)(base + sp.ypart_off);
    a.cnt = (unsigned*)(base + sp.cnt_off);
    a.bar = (unsigned*)(base + sp.bar_off);
    a.zeros = (const u16*)(base + sp.zero_off);
    a.epoch = (unsigned*)(base + sp.epoch_off);
    a.fault = dev->fault_dev;
    a.spin_limit = g_spin_limit;
    a.M = M; a.D = D; a.F = F; a.Fp = sp.Fp; a.eps = eps;
    a.nkb1 = sp.nkb1; a.nfb = sp.nfb; a.items1 = sp.items1; a.per1 = sp.per1; a.S1 = sp.S1;
    a.nkb2 = sp.nkb2; a.nnb = sp.nnb; a.items2 = sp.items2; a.per2 = sp.per2; a.S2 = sp.S2;
    if (log_on())
        std::fprintf(stderr, "[bb] stream M %d (%d x 16 rows) D %d F %d items %d/%d per wg %d/%d slots %d/%d\n", M, sp.MT, D,
                     F, a.items1, a.items2, a.per1, a.per2, a.S1, a.S2);
    prof_begin(st);   // (a refill of the zone above, if any, is not part of the kernel's time)
    stream_launch(sp.MT, G, st, a);
    BB_HIP(hipGetLastError());
    prof_mark("ffn_stream", st);
    return BB_OK;
}

// Plan of the streaming kernel for transposed weights: rows per workgroup, the k-block of bf16(x g)
// that fits LDS next to the partial sums.  ok = false: the shape needs more than STREAMT_MAXG groups of
// 16 rows per workgroup (the tiled kernels take it).
struct StreamTPlan {
    bool ok;
    int upw, cpw, kblk, cq2, red_off, stat_off, lds;
};
StreamTPlan stream_t_plan(int64_t D, int64_t F, int G) {
    StreamTPlan s{};
    s.upw = (int)((F + G - 1) / G);
    s.cpw = (int)((D + G - 1) / G);
    const int ng = (s.upw + 15) / 16, ng2 = (s.cpw + 15) / 16;
    if (ng > STREAMT_MAXG || ng2 > STREAMT_MAXG) return s;
    const int red = std::max(4 * ng * 2048, 4 * ng2 * 1024);
    const int room = STREAMT_LDS - red - 320;                     // bytes left for 16 rows of kblk + 8 elements
    int kblk = (room / 32 - 8) / 512 * 512;
    kblk = std::min(kblk, (int)((D + 511) / 512 * 512));
    if (kblk < 512) return s;
    s.kblk = kblk;
    s.cq2 = (int)(((F / 8 + 3) / 4 + 15) / 16 * 16);
    s.red_off = 16 * (kblk + 8) * 2;
    s.stat_off = s.red_off + red;
    s.lds = s.stat_off + 320;                                      // 16 inverse norms, 4 x 16 partial sums
    s.ok = true;
    return s;
}

// BB_ERR_VARIANT: not applicable to this shape or device (the caller falls back to the tiled kernels)
int run_stream_t(const u16* X, const u16* g, const u16* W1t, const u16* W3t, const u16* W2t, const u16* R, u16* Y,
                 int M, int D, int F, float eps, const DeviceInfo* dev, hipStream_t st) {
    const int cus = dev->cus;
    if (M < 1 || M > kStreamTMaxM) return BB_ERR_VARIANT;      // (the kernel clamps row numbers to M - 1)
    const int G = std::min(cus, kPlanCUs);
    const StreamTPlan tp = stream_t_plan(D, F, G);
    if (!tp.ok) return BB_ERR_VARIANT;
    static int resident = -1;
    if (resident < 0) {
        hipError_t e = hipSuccess;
        const int nres = stream_t_resident(tp.lds, &e);
        BB_HIP(e);
        resident = nres;
    }
    if (resident < 1) return BB_ERR_VARIANT;    // the grid barrier needs every workgroup resident
    const StreamPlan sp = stream_plan(M, D, F, G);     // (barrier words and hidden block: the same places)
    char* base = (char*)g_ws.ptr;
    if (int rc = prepare_barrier_zone(sp, st)) return rc;
    StreamTArgs a;
    a.X = X; a.g = g; a.W1t = W1t; a.W3t = W3t; a.W2t = W2t; a.R = R; a.Y = Y;
    a.H = (u16*)(base + sp.h_off);
    a.bar = (unsigned*)(base + sp.bar_off);
    a.zeros = (const u16*)(base + sp.zero_off);
    a.epoch = (unsigned*)(base + sp.epoch_off);
    a.fault = dev->fault_dev;
    a.spin_limit = g_spin_limit;
    a.M = M; a.D = D; a.F = F; a.Fp = sp.Fp; a.eps = eps;
    a.upw = tp.upw; a.cpw = tp.cpw; a.kblk = tp.kblk; a.cq2 = tp.cq2;
    a.red_off = tp.red_off; a.stat_off = tp.stat_off;
    if (log_on())
        std::fprintf(stderr, "[bb] stream_t M %d D %d F %d units/wg %d columns/wg %d kblk %d lds %d\n", M, D, F, a.upw,
                     a.cpw, a.kblk, tp.lds);
    prof_begin(st);
    stream_t_launch(G, tp.lds, st, a);
    BB_HIP(hipGetLastError());
    prof_mark("ffn_stream_t", st);
    return BB_OK;
}

hipStream_t as_stream(void* s) { return (hipStream_t)s; }

}  // namespace

// ============================================================== exported API
extern "C" {

int bb_version(void) { return BB_VERSION; }
int bb_last_hip_error(void) { return g_last_hip; }

const char* bb_status_string(int s) {
    switch (s) {
        case BB_OK: return "ok";
        case BB_ERR_NULL: return "null pointer";
        case BB_ERR_SHAPE: return "bad shape";
        case BB_ERR_ALIGN: return "pointer not 16-byte aligned";
        case BB_ERR_EPS: return "bad eps";
        case BB_ERR_ALIAS: return "output overlaps an input";
        case BB_ERR_ARCH: return "device is not gfx950";
        case BB_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
        case BB_ERR_HIP: return "HIP call failed";
        case BB_ERR_VARIANT: return "bad variant";
        case BB_ERR_INIT: return "bb_init has not been called on the current device";
        case BB_ERR_TIMEOUT: return "a streaming kernel of an earlier launch gave up waiting for another workgroup";
        default: return "unknown status";
    }
}

int bb_set_variant(int v) {
    if (v < BB_VARIANT_AUTO || v > BB_VARIANT_NEST) return BB_ERR_VARIANT;
    std::lock_guard<std::mutex> lk(g_mu);
    g_variant = v;
    return BB_OK;
}

int bb_get_variant(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    return read_variant();
}

int bb_init(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    const DeviceInfo* dev = nullptr;
    return current_device_info(&dev);
}

int bb_rmsnorm_swiglu_ffn_static(const void* X, const void* g, const void* W1, const void* W3, const void* W2,
                                 void* Y, int64_t M, int64_t D, int64_t F, float eps, void* stream) {
    if (int rc = validate_ffn(X, g, W1, W3, W2, Y, M, D, F, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    int devno = 0;
    BB_HIP(hipGetDevice(&devno));
    if (devno < 0 || devno >= 64) return BB_ERR_ARCH;
    DeviceInfo& d = g_dev[devno];
    if (!d.known) return BB_ERR_INIT;                      // (setting a device up allocates its fault word)
    if (!d.gfx950) return BB_ERR_ARCH;
    int variant = read_variant();
    if (variant == BB_VARIANT_UNFUSED) return BB_ERR_VARIANT;
    if (variant == BB_VARIANT_STREAM && M > kStreamMaxM) return BB_ERR_VARIANT;
    if (variant == BB_VARIANT_AUTO) variant = auto_variant(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F);
    if (variant == BB_VARIANT_UNFUSED) variant = BB_VARIANT_SNAPSHOT1;
    if (zone_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F) + scratch_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F) >
        (size_t)BB_STATIC_SCRATCH_BYTES) {
        if (log_on())
            std::fprintf(stderr, "[bb] bb_rmsnorm_swiglu_ffn_static: M %lld D %lld F %lld needs %zu bytes of scratch, the static array has %zu\n",
                         (long long)M, (long long)D, (long long)F,
                         zone_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F) + scratch_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F),
                         (size_t)BB_STATIC_SCRATCH_BYTES);
        return BB_ERR_WORKSPACE;
    }
    // The operator runs as in bb_rmsnorm_swiglu_ffn with the static array in the place of the workspace: a
    // caller-owned workspace is never grown or freed (ensure_workspace), the zone is cleared by a fill
    // kernel, and per-kernel profiling (which creates events) is off for the duration of the call.
    if (int rc = check_fault(&d)) return rc;               // (marks the zones of both workspaces for clearing)
    const Workspace saved = g_ws;
    const bool prof_was_on = g_prof.on;
    g_ws = Workspace();
    g_ws.ptr = d.static_ptr;
    g_ws.bytes = (size_t)BB_STATIC_SCRATCH_BYTES;
    g_ws.user = true;
    g_ws.clean = d.static_clean;
    g_ws.device = devno;
    g_prof.on = false;
    const int rc = ffn_locked(variant, X, g, W1, W3, W2, Y, M, D, F, eps, stream);
    d.static_clean = g_ws.clean;
    g_prof.on = prof_was_on;
    g_ws = saved;
    return rc;
}

int bb_check_fault(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    return check_fault(dev);
}

int bb_debug_inject_fault(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    *dev->fault_host = 1u;
    return BB_OK;
}

int bb_debug_set_spin_limit(unsigned polls) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_spin_limit = polls;
    return BB_OK;
}

size_t bb_workspace_bytes(int op, int64_t M, int64_t D, int64_t F) {
    if (op < BB_OP_RMSNORM_SWIGLU_FFN || op > BB_OP_LAYERNORM_MATMUL_UNFUSED) return 0;
    if (check_dims(M, D, F) != BB_OK) return 0;
    return zone_bytes(op, M, D, F) + scratch_bytes(op, M, D, F);
}

int bb_set_workspace(void* dptr, size_t bytes) {
    std::lock_guard<std::mutex> lk(g_mu);
    if ((dptr == nullptr) != (bytes == 0)) return BB_ERR_WORKSPACE;
    if ((uintptr_t)dptr & (kAlign - 1)) return BB_ERR_WORKSPACE;
    g_tuned.clear();                   // selections were measured with the previous workspace arrangement
    if (g_ws.ptr && !g_ws.user) {
        BB_HIP(hipDeviceSynchronize());
        BB_HIP(hipFree(g_ws.ptr));
    }
    g_ws = Workspace();
    if (dptr) {
        g_ws.ptr = dptr;
        g_ws.bytes = bytes;
        g_ws.user = true;
        g_ws.clean = bytes;    // handed over zero-filled (contract)
    }
    return BB_OK;
}

int bb_shutdown(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_ws.ptr && !g_ws.user) {
        BB_HIP(hipDeviceSynchronize());
        BB_HIP(hipFree(g_ws.ptr));
    }
    g_ws = Workspace();
    return BB_OK;
}

int bb_rmsnorm_swiglu_ffn(const void* X, const void* g, const void* W1, const void* W3, const void* W2,
                          void* Y, int64_t M, int64_t D, int64_t F, float eps, void* stream) {
    if (int rc = validate_ffn(X, g, W1, W3, W2, Y, M, D, F, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    int variant = read_variant();
    if (variant == BB_VARIANT_STREAM && M > kStreamMaxM) return BB_ERR_VARIANT;
    if (variant == BB_VARIANT_AUTO) variant = auto_variant(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F);
    return ffn_locked(variant, X, g, W1, W3, W2, Y, M, D, F, eps, stream);
}

} // extern "C"

namespace {

// the operators with the library lock held and arguments validated
// R: residual added in the last kernel's epilogue, or null (the unfused program has no such epilogue)
int ffn_locked(int variant, const void* X, const void* g, const void* W1, const void* W3, const void* W2,
               void* Y, int64_t M, int64_t D, int64_t F, float eps, void* stream, const void* R) {
    if (variant == BB_VARIANT_UNFUSED && R == nullptr)
        return ffn_unfused_locked(X, g, W1, W3, W2, Y, M, D, F, eps, stream);
    if (variant == BB_VARIANT_UNFUSED) variant = BB_VARIANT_SNAPSHOT1;
    if (variant == BB_VARIANT_PRESCALE && M <= kPrescaleFloorM) return BB_ERR_VARIANT;   // (no room is planned for so few rows)
    if (variant == BB_VARIANT_NEST && D > NEST_MAXD) return BB_ERR_VARIANT;          // (the block of outputs no longer fits the registers)
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    if (int rc = check_fault(dev)) return rc;
    if (variant == BB_VARIANT_NEST) {
        // last snapshot (one block of output columns): one launch, no workspace
        NestArgs a;
        a.X = (const u16*)X; a.g = (const u16*)g; a.W1 = (const u16*)W1; a.W3 = (const u16*)W3; a.W2 = (const u16*)W2;
        a.Y = (u16*)Y; a.R = (const u16*)R; a.M = (int)M; a.D = (int)D; a.F = (int)F; a.eps = eps;
        hipStream_t nst = as_stream(stream);
        prof_begin(nst);
        nest_launch((int)((D + 127) / 128), (int)((M + NEST_ROWS - 1) / NEST_ROWS), nst, a);
        BB_HIP(hipGetLastError());
        prof_mark("ffn_nest", nst);
        return BB_OK;
    }
    const size_t zone = zone_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F);
    if (int rc = ensure_workspace(zone + scratch_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F))) return rc;
    hipStream_t st = as_stream(stream);
    const u16 *x = (const u16*)X, *gg = (const u16*)g, *w1 = (const u16*)W1, *w3 = (const u16*)W3,
              *w2 = (const u16*)W2;
    if (variant == BB_VARIANT_STREAM)
        return run_stream(x, gg, w1, w3, w2, (const u16*)R, (u16*)Y, (int)M, (int)D, (int)F, eps, dev, st);
    // first snapshot: hidden written once (bf16), then contracted with W2
    u16* H = (u16*)((char*)g_ws.ptr + zone);
    void* split = (char*)H + align_up((size_t)M * F * 2);
    const int pcus = std::min(dev->cus, kPlanCUs);          // (the workspace was sized for this many)
    mark_dirty(zone);
    prof_begin(st);
    if (variant == BB_VARIANT_PRESCALE) {
        // the statistics loop as a kernel of its own: bf16(x g) and the inverse norms, then the
        // two products with the plain main loop and the SwiGLU epilogue
        u16* Xg = (u16*)((char*)split + std::max(split_bytes(MODE_GATEUP, M, F, D, kPlanCUs),
                                                 split_bytes(MODE_PLAIN, M, D, F, kPlanCUs)));
        float* rstd = (float*)((char*)Xg + align_up((size_t)M * D * 2));
        hipLaunchKernelGGL(rms_gain_rows_kernel, dim3((unsigned)M), dim3(256), 0, st, x, gg, Xg, rstd, (int)D, eps);
        BB_HIP(hipGetLastError());
        prof_mark("rms_gain_rows", st);
        if (int rc = launch_gemm<MODE_GATEUP_PRE>(Xg, (int)D, w1, w3, (int)F, H, (int)F, nullptr, rstd, nullptr,
                                                  (int)M, (int)F, (int)D, eps, pcus, st, nullptr))
            return rc;
        return launch_gemm<MODE_PLAIN>(H, (int)F, w2, nullptr, (int)D, (u16*)Y, (int)D, nullptr, nullptr, nullptr,
                                       (int)M, (int)D, (int)F, 0.f, pcus, st, split, (const u16*)R, (int)D);
    }
    if (int rc = launch_gemm<MODE_GATEUP>(x, (int)D, w1, w3, (int)F, H, (int)F, gg, nullptr, nullptr, (int)M,
                                          (int)F, (int)D, eps, pcus, st, split))
        return rc;
    return launch_gemm<MODE_PLAIN>(H, (int)F, w2, nullptr, (int)D, (u16*)Y, (int)D, nullptr, nullptr, nullptr,
                                   (int)M, (int)D, (int)F, 0.f, pcus, st, split, (const u16*)R, (int)D);
}

int ffn_t_locked(const void* X, const void* g, const void* W1t, const void* W3t, const void* W2t, void* Y,
                 int64_t M, int64_t D, int64_t F, float eps, void* stream, const void* R) {
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    if (int rc = check_fault(dev)) return rc;
    const size_t zone = zone_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F);
    if (int rc = ensure_workspace(zone + scratch_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F))) return rc;
    hipStream_t st = as_stream(stream);
    // few rows: the weight-streaming kernel for this layout (unless a tiled variant is forced)
    const int variant = read_variant();
    if (M <= kStreamTMaxM && (variant == BB_VARIANT_AUTO || variant == BB_VARIANT_STREAM)) {
        const int rc = run_stream_t((const u16*)X, (const u16*)g, (const u16*)W1t, (const u16*)W3t, (const u16*)W2t,
                                    (const u16*)R, (u16*)Y, (int)M, (int)D, (int)F, eps, dev, st);
        if (rc != BB_ERR_VARIANT) return rc;
    }
    u16* H = (u16*)((char*)g_ws.ptr + zone);
    void* split = (char*)H + align_up((size_t)M * F * 2);
    const int pcus = std::min(dev->cus, kPlanCUs);
    mark_dirty(zone);
    prof_begin(st);
    if (M >= kPrescaleMinM) {         // as AUTO does for the untransposed layout: statistics loop as its own kernel
        u16* Xg = (u16*)((char*)split + std::max(split_bytes(MODE_GATEUP, M, F, D, kPlanCUs),
                                                 split_bytes(MODE_PLAIN, M, D, F, kPlanCUs)));
        float* rstd = (float*)((char*)Xg + align_up((size_t)M * D * 2));
        hipLaunchKernelGGL(rms_gain_rows_kernel, dim3((unsigned)M), dim3(256), 0, st, (const u16*)X, (const u16*)g,
                           Xg, rstd, (int)D, eps);
        BB_HIP(hipGetLastError());
        prof_mark("rms_gain_rows", st);
        if (int rc = (launch_gemm<MODE_GATEUP_PRE, true>(Xg, (int)D, (const u16*)W1t, (const u16*)W3t, (int)D, H,
                                                         (int)F, nullptr, rstd, nullptr, (int)M, (int)F, (int)D, eps,
                                                         pcus, st, nullptr)))
            return rc;
    } else if (int rc = (launch_gemm<MODE_GATEUP, true>((const u16*)X, (int)D, (const u16*)W1t, (const u16*)W3t,
                                                        (int)D, H, (int)F, (const u16*)g, nullptr, nullptr, (int)M,
                                                        (int)F, (int)D, eps, pcus, st, split))) {
        return rc;
    }
    return launch_gemm<MODE_PLAIN, true>(H, (int)F, (const u16*)W2t, nullptr, (int)F, (u16*)Y, (int)D, nullptr,
                                         nullptr, nullptr, (int)M, (int)D, (int)F, 0.f, pcus, st, split,
                                         (const u16*)R, (int)D);
}

int ln_locked(int variant, const void* X, const void* gamma, const void* beta, const void* W, void* Y,
              int64_t M, int64_t D, int64_t N, float eps, void* stream) {
    if (variant == BB_VARIANT_UNFUSED) return ln_unfused_locked(X, gamma, beta, W, Y, M, D, N, eps, stream);
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    if (int rc = ensure_workspace(scratch_bytes(BB_OP_LAYERNORM_MATMUL, M, D, N))) return rc;
    hipStream_t st = as_stream(stream);
    mark_dirty(0);
    float* colc = (float*)g_ws.ptr;
    float* colb = (float*)((char*)g_ws.ptr + align_up((size_t)N * 4));
    prof_begin(st);
    float* part = (float*)((char*)g_ws.ptr + 2 * align_up((size_t)N * 4));
    hipLaunchKernelGGL(colvec_partial_kernel, dim3((unsigned)((N + 511) / 512), COLVEC_SPLITS), dim3(256), 0, st,
                       (const u16*)W, (const u16*)gamma, (const u16*)beta, part, (int)D, (int)N);
    BB_HIP(hipGetLastError());
    hipLaunchKernelGGL(colvec_sum_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, part, colc, colb,
                       (int)N);
    BB_HIP(hipGetLastError());
    prof_mark("colvec", st);
    if (variant == BB_VARIANT_PRESCALE) {
        // the statistics loop as a kernel of its own: bf16(x gamma), inverse standard deviations and
        // means; the product runs the plain main loop and keeps the epilogue r (P - mu c) + b
        u16* Xg = (u16*)((char*)g_ws.ptr + (2 + 2 * COLVEC_SPLITS) * align_up((size_t)N * 4));
        float* stat = (float*)((char*)Xg + align_up((size_t)M * D * 2));
        hipLaunchKernelGGL(ln_gain_rows_kernel, dim3((unsigned)M), dim3(256), 0, st, (const u16*)X,
                           (const u16*)gamma, Xg, stat, (int)D, eps);
        BB_HIP(hipGetLastError());
        prof_mark("ln_gain_rows", st);
        return launch_gemm<MODE_LN_PRE>(Xg, (int)D, (const u16*)W, nullptr, (int)N, (u16*)Y, (int)N, nullptr, colc,
                                        colb, (int)M, (int)N, (int)D, eps, dev->cus, st, nullptr, nullptr, 0, stat);
    }
    return launch_gemm<MODE_LN>((const u16*)X, (int)D, (const u16*)W, nullptr, (int)N, (u16*)Y, (int)N,
                                (const u16*)gamma, colc, colb, (int)M, (int)N, (int)D, eps, dev->cus, st);
}

}  // namespace

extern "C" {

int bb_layernorm_matmul(const void* X, const void* gamma, const void* beta, const void* W, void* Y,
                        int64_t M, int64_t D, int64_t N, float eps, void* stream) {
    if (int rc = validate_ln(X, gamma, beta, W, Y, M, D, N, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    int variant = read_variant();
    if (variant == BB_VARIANT_AUTO || variant == BB_VARIANT_STREAM || variant == BB_VARIANT_NEST)
        variant = auto_variant(BB_OP_LAYERNORM_MATMUL, M, D, N);
    return ln_locked(variant, X, gamma, beta, W, Y, M, D, N, eps, stream);
}

int bb_rmsnorm_swiglu_ffn_t(const void* X, const void* g, const void* W1t, const void* W3t, const void* W2t,
                            void* Y, int64_t M, int64_t D, int64_t F, float eps, void* stream) {
    if (int rc = validate_ffn(X, g, W1t, W3t, W2t, Y, M, D, F, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    return ffn_t_locked(X, g, W1t, W3t, W2t, Y, M, D, F, eps, stream, nullptr);
}

int bb_rmsnorm_swiglu_ffn_residual(const void* X, const void* g, const void* W1, const void* W3,
                                   const void* W2, const void* R, void* Y, int64_t M, int64_t D, int64_t F,
                                   float eps, void* stream) {
    if (int rc = validate_ffn_residual(X, g, W1, W3, W2, R, Y, M, D, F, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    int variant = read_variant();
    if (variant == BB_VARIANT_STREAM && M > kStreamMaxM) return BB_ERR_VARIANT;
    if (variant == BB_VARIANT_AUTO) variant = auto_variant(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F);
    return ffn_locked(variant, X, g, W1, W3, W2, Y, M, D, F, eps, stream, R);
}

int bb_rmsnorm_swiglu_ffn_residual_t(const void* X, const void* g, const void* W1t, const void* W3t,
                                     const void* W2t, const void* R, void* Y, int64_t M, int64_t D,
                                     int64_t F, float eps, void* stream) {
    if (int rc = validate_ffn_residual(X, g, W1t, W3t, W2t, R, Y, M, D, F, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    return ffn_t_locked(X, g, W1t, W3t, W2t, Y, M, D, F, eps, stream, R);
}

int bb_layernorm_matmul_t(const void* X, const void* gamma, const void* beta, const void* Wt, void* Y,
                          int64_t M, int64_t D, int64_t N, float eps, void* stream) {
    if (int rc = validate_ln(X, gamma, beta, Wt, Y, M, D, N, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    if (int rc = ensure_workspace(scratch_bytes(BB_OP_LAYERNORM_MATMUL, M, D, N))) return rc;
    hipStream_t st = as_stream(stream);
    mark_dirty(0);
    float* colc = (float*)g_ws.ptr;
    float* colb = (float*)((char*)g_ws.ptr + align_up((size_t)N * 4));
    prof_begin(st);
    hipLaunchKernelGGL(colvec_t_kernel, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, st, (const u16*)Wt,
                       (const u16*)gamma, (const u16*)beta, colc, colb, (int)D, (int)N);
    BB_HIP(hipGetLastError());
    prof_mark("colvec", st);
    if (M >= kPrescaleMinM) {         // as AUTO does for the untransposed layout
        u16* Xg = (u16*)((char*)g_ws.ptr + (2 + 2 * COLVEC_SPLITS) * align_up((size_t)N * 4));
        float* stat = (float*)((char*)Xg + align_up((size_t)M * D * 2));
        hipLaunchKernelGGL(ln_gain_rows_kernel, dim3((unsigned)M), dim3(256), 0, st, (const u16*)X,
                           (const u16*)gamma, Xg, stat, (int)D, eps);
        BB_HIP(hipGetLastError());
        prof_mark("ln_gain_rows", st);
        return launch_gemm<MODE_LN_PRE, true>(Xg, (int)D, (const u16*)Wt, nullptr, (int)D, (u16*)Y, (int)N, nullptr,
                                              colc, colb, (int)M, (int)N, (int)D, eps, dev->cus, st, nullptr, nullptr,
                                              0, stat);
    }
    return launch_gemm<MODE_LN, true>((const u16*)X, (int)D, (const u16*)Wt, nullptr, (int)D, (u16*)Y, (int)N,
                                      (const u16*)gamma, colc, colb, (int)M, (int)N, (int)D, eps, dev->cus, st);
}

int bb_attention(const void* Q, const void* K, const void* V, void* O, int64_t B, int64_t M, int64_t N,
                 int64_t d, int64_t dv, void* stream) {
    if (B < 0 || M < 0 || N < 1) return BB_ERR_SHAPE;
    if ((d != 64 && d != 128) || (dv != 64 && dv != 128)) return BB_ERR_SHAPE;
    if (M > (1 << 24) || N >= (1 << 24)) return BB_ERR_SHAPE;   // 32-bit byte offsets inside one problem's K and V
    if (B * ((M + 127) / 128) > 0x7ffffff0LL) return BB_ERR_SHAPE;  // one workgroup per (problem, query block)
    if (B == 0 || M == 0) return BB_OK;
    if (!Q || !K || !V || !O) return BB_ERR_NULL;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O)) return BB_ERR_ALIGN;
    const size_t no = (size_t)B * M * dv * 2;
    if (overlaps(O, no, Q, (size_t)B * M * d * 2) || overlaps(O, no, K, (size_t)B * N * d * 2) ||
        overlaps(O, no, V, (size_t)B * N * dv * 2))
        return BB_ERR_ALIAS;
    std::lock_guard<std::mutex> lk(g_mu);
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    hipStream_t st = as_stream(stream);
    AttnArgs a;
    a.Q = (const u16*)Q;
    a.K = (const u16*)K;
    a.V = (const u16*)V;
    a.O = (u16*)O;
    a.B = (int)B;
    a.M = (int)M;
    a.N = (int)N;
    if (M == 1) {
        // one query per problem: the streaming kernel (no matrix product), any N
        int64_t nsplit = 1;
        a.nt_split = attn_decode_plan(B, N, std::min(dev->cus, kPlanCUs), &nsplit);
        if (B * nsplit > 0x7fffffffLL) return BB_ERR_SHAPE;
        a.nsplit = (int)nsplit;
        a.tiles_q = 1;
        a.wgs_per_xcd = 0;
        a.c = (float)(1.4426950408889634 / std::sqrt((double)d));
        const size_t zone = attn_zone_bytes(B), pbytes = align_up((size_t)B * nsplit * dv * 4);
        if (int rc = ensure_workspace(zone + pbytes + align_up((size_t)B * nsplit * 8))) return rc;
        const size_t had = g_ws.attn_zone;
        mark_dirty(0);
        if (had < zone) {                  // counters: zero before their first use; every launch leaves them zero
            if (int rc = fill_zero(g_ws.ptr, zone, st)) return rc;
            g_ws.attn_zone = zone;
        } else {
            g_ws.attn_zone = had;
        }
        a.cnt = (unsigned*)g_ws.ptr;
        a.part = (float*)((char*)g_ws.ptr + zone);
        a.ml = (float*)((char*)g_ws.ptr + zone + pbytes);
        const dim3 grid((unsigned)(B * nsplit)), block(256);
        prof_begin(st);
        if (d == 64 && dv == 64) attn_decode_launch<64, 64>(grid, st, a);
        else if (d == 64) attn_decode_launch<64, 128>(grid, st, a);
        else if (dv == 64) attn_decode_launch<128, 64>(grid, st, a);
        else attn_decode_launch<128, 128>(grid, st, a);
        BB_HIP(hipGetLastError());
        prof_mark("attention", st);
        return BB_OK;
    }
    // few queries (decoding): split the keys over workgroups so that the chip has about two per
    // compute unit; equal numbers of key blocks per workgroup, at least two each
    const int64_t nt_all = (N + ATTN_BK - 1) / ATTN_BK;
    const int ksplit = attn_key_splits(B * ((M + 127) / 128), nt_all, std::min(dev->cus, kPlanCUs));
    // eight wavefronts (256 queries) per workgroup when that still gives every compute unit a
    // workgroup and wastes little on a ragged last query block; else four (128 queries)
    static const int forced_waves = [] { const char* e = std::getenv("BB_ATTN_WAVES"); return e ? std::atoi(e) : 0; }();
    // (measured: +2..7 % for head dimension 128, -4..8 % for 64, where the vector work per block dominates)
    int nw = d == 128 && dv == 128 && (M % 256 == 0 || M >= 2048) && B * ((M + 255) / 256) >= dev->cus ? 8 : 4;
    if (forced_waves == 4 || forced_waves == 8) nw = forced_waves;
    if (ksplit > 1) nw = 4;
    const int64_t tiles_q = (M + 32 * nw - 1) / (32 * nw);
    a.tiles_q = (int)tiles_q;
    a.wgs_per_xcd = (int)((B * tiles_q * ksplit + 7) / 8);
    a.c = (float)(1.4426950408889634 / std::sqrt((double)d));
    a.nsplit = ksplit;
    a.nt_split = (int)(nt_all / ksplit);
    a.part = nullptr;
    a.ml = nullptr;
    a.cnt = nullptr;
    if (ksplit > 1) {
        const size_t rows = (size_t)B * M;
        const size_t pbytes = align_up(rows * ksplit * dv * 4);
        if (int rc = ensure_workspace(pbytes + align_up(rows * ksplit * 8))) return rc;
        mark_dirty(0);
        a.part = (float*)g_ws.ptr;
        a.ml = (float*)((char*)g_ws.ptr + pbytes);
    }
    const dim3 grid((unsigned)(8 * a.wgs_per_xcd)), block((unsigned)(64 * nw));
    prof_begin(st);
    const int64_t nt = nt_all / ksplit;                            // key blocks per workgroup
    const int tail = nt <= 4 ? (int)nt : ((nt & 1) ? 3 : 4);     // iterations left after the main loop
    if (d == 64 && dv == 64) attn_tiled_launch<64, 64>(tail, nw, ksplit, grid, block, st, a);
    else if (d == 64) attn_tiled_launch<64, 128>(tail, nw, ksplit, grid, block, st, a);
    else if (dv == 64) attn_tiled_launch<128, 64>(tail, nw, ksplit, grid, block, st, a);
    else attn_tiled_launch<128, 128>(tail, nw, ksplit, grid, block, st, a);
    BB_HIP(hipGetLastError());
    prof_mark("attention", st);
    return BB_OK;
}

size_t bb_attention_workspace_bytes(int64_t B, int64_t M, int64_t N, int64_t d, int64_t dv) {
    if (B < 0 || M < 0 || N < 1 || (d != 64 && d != 128) || (dv != 64 && dv != 128)) return 0;
    if (B == 0 || M == 0) return 0;
    if (M == 1) {
        int64_t nsplit = 1;
        attn_decode_plan(B, N, kPlanCUs, &nsplit);
        return attn_zone_bytes(B) + align_up((size_t)B * nsplit * dv * 4) + align_up((size_t)B * nsplit * 8);
    }
    const int s = attn_key_splits(B * ((M + 127) / 128), (N + ATTN_BK - 1) / ATTN_BK, kPlanCUs);
    if (s < 2) return 0;
    const size_t rows = (size_t)B * M;
    return align_up(rows * s * dv * 4) + align_up(rows * s * 8);
}

int bb_rmsnorm_swiglu_ffn_unfused(const void* X, const void* g, const void* W1, const void* W3,
                                  const void* W2, void* Y, int64_t M, int64_t D, int64_t F, float eps,
                                  void* stream) {
    if (int rc = validate_ffn(X, g, W1, W3, W2, Y, M, D, F, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    return ffn_unfused_locked(X, g, W1, W3, W2, Y, M, D, F, eps, stream);
}

int bb_layernorm_matmul_unfused(const void* X, const void* gamma, const void* beta, const void* W, void* Y,
                                int64_t M, int64_t D, int64_t N, float eps, void* stream) {
    if (int rc = validate_ln(X, gamma, beta, W, Y, M, D, N, eps)) return rc;
    if (M == 0) return BB_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    return ln_unfused_locked(X, gamma, beta, W, Y, M, D, N, eps, stream);
}

}  // extern "C"

namespace {

int ffn_unfused_locked(const void* X, const void* g, const void* W1, const void* W3, const void* W2, void* Y,
                       int64_t M, int64_t D, int64_t F, float eps, void* stream) {
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    if (int rc = ensure_workspace(scratch_bytes(BB_OP_RMSNORM_SWIGLU_FFN_UNFUSED, M, D, F))) return rc;
    hipStream_t st = as_stream(stream);
    mark_dirty(0);
    char* base = (char*)g_ws.ptr;
    const size_t nMF = align_up((size_t)M * F * 2);
    u16* Xh = (u16*)base;
    u16* P = (u16*)(base + align_up((size_t)M * D * 2));
    u16* Q = (u16*)((char*)P + nMF);
    u16* H = (u16*)((char*)Q + nMF);
    void* split = (char*)H + nMF;
    const int pcus = std::min(dev->cus, kPlanCUs);
    prof_begin(st);
    hipLaunchKernelGGL(rmsnorm_rows_kernel, dim3((unsigned)M), dim3(256), 0, st, (const u16*)X, (const u16*)g,
                       Xh, (int)D, eps);
    BB_HIP(hipGetLastError());
    prof_mark("rmsnorm_rows", st);
    if (int rc = launch_gemm<MODE_PLAIN>(Xh, (int)D, (const u16*)W1, nullptr, (int)F, P, (int)F, nullptr,
                                         nullptr, nullptr, (int)M, (int)F, (int)D, 0.f, pcus, st, split))
        return rc;
    if (int rc = launch_gemm<MODE_PLAIN>(Xh, (int)D, (const u16*)W3, nullptr, (int)F, Q, (int)F, nullptr,
                                         nullptr, nullptr, (int)M, (int)F, (int)D, 0.f, pcus, st, split))
        return rc;
    const size_t n8 = (size_t)M * F / 8;
    hipLaunchKernelGGL(silu_mul_kernel, dim3((unsigned)std::min<size_t>((n8 + 255) / 256, 4096)), dim3(256), 0,
                       st, P, Q, H, n8);
    BB_HIP(hipGetLastError());
    prof_mark("silu_mul", st);
    return launch_gemm<MODE_PLAIN>(H, (int)F, (const u16*)W2, nullptr, (int)D, (u16*)Y, (int)D, nullptr,
                                   nullptr, nullptr, (int)M, (int)D, (int)F, 0.f, pcus, st, split);
}

int ln_unfused_locked(const void* X, const void* gamma, const void* beta, const void* W, void* Y, int64_t M,
                      int64_t D, int64_t N, float eps, void* stream) {
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    if (int rc = ensure_workspace(scratch_bytes(BB_OP_LAYERNORM_MATMUL_UNFUSED, M, D, N))) return rc;
    hipStream_t st = as_stream(stream);
    mark_dirty(0);
    u16* Z = (u16*)g_ws.ptr;
    prof_begin(st);
    hipLaunchKernelGGL(layernorm_rows_kernel, dim3((unsigned)M), dim3(256), 0, st, (const u16*)X,
                       (const u16*)gamma, (const u16*)beta, Z, (int)D, eps);
    BB_HIP(hipGetLastError());
    prof_mark("layernorm_rows", st);
    return launch_gemm<MODE_PLAIN>(Z, (int)D, (const u16*)W, nullptr, (int)N, (u16*)Y, (int)N, nullptr, nullptr,
                                   nullptr, (int)M, (int)N, (int)D, 0.f, dev->cus, st);
}

// Times fn() `reps` times on the stream after one untimed call; mean milliseconds, or < 0 on error.
template <class Fn>
int time_candidate(Fn fn, int reps, hipStream_t st, float* ms) {
    hipEvent_t e0, e1;
    BB_HIP(hipEventCreate(&e0));
    BB_HIP(hipEventCreate(&e1));
    int rc = fn();
    if (rc == BB_OK) {
        (void)hipEventRecord(e0, st);
        for (int i = 0; i < reps && rc == BB_OK; ++i) rc = fn();
        (void)hipEventRecord(e1, st);
        const hipError_t e = hipEventSynchronize(e1);
        if (rc == BB_OK && e != hipSuccess) rc = hip_fail(e);
        if (rc == BB_OK) {
            (void)hipEventElapsedTime(ms, e0, e1);
            *ms /= (float)reps;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

// Measured selection: runs every candidate program of the operator on the caller's operands, records
// the fastest for this (op, M, D, F or N) in the table AUTO consults, reports the times.
template <class Run>
int tune_locked(int op, int64_t M, int64_t D, int64_t FN, int reps, hipStream_t st, int* chosen, float* ms_out,
                Run run) {
    if (reps < 1 || reps > 1000) return BB_ERR_SHAPE;
    const bool prof = g_prof.on;
    g_prof.on = false;
    int best = 0;
    float best_ms = 0.f;
    int rc = BB_OK;
    for (int v = BB_VARIANT_STREAM; v <= BB_VARIANT_NEST && rc == BB_OK; ++v) {
        if (ms_out) ms_out[v] = -1.f;
        if (op == BB_OP_LAYERNORM_MATMUL && (v == BB_VARIANT_STREAM || v == BB_VARIANT_NEST)) continue;
        if (v == BB_VARIANT_NEST && D > NEST_MAXD) continue;
        if (v == BB_VARIANT_STREAM && M > kStreamMaxM) continue;
        if (op == BB_OP_RMSNORM_SWIGLU_FFN && v == BB_VARIANT_PRESCALE && M <= kPrescaleFloorM) continue;
        float ms = 0.f;
        rc = time_candidate([&]() { return run(v); }, reps, st, &ms);
        if (rc == BB_ERR_WORKSPACE && g_ws.user) {      // does not fit the caller's workspace: not a candidate
            rc = BB_OK;
            continue;
        }
        if (rc != BB_OK) break;
        if (ms_out) ms_out[v] = ms;
        if (!best || ms < best_ms) best = v, best_ms = ms;
    }
    g_prof.on = prof;
    if (rc != BB_OK) return rc;
    g_tuned[TuneKey{op, M, D, FN}] = best;
    if (ms_out) ms_out[0] = best_ms;
    if (chosen) *chosen = best;
    if (log_on()) std::fprintf(stderr, "[bb] tuned op %d M %lld D %lld F/N %lld -> variant %d (%.4f ms)\n", op,
                               (long long)M, (long long)D, (long long)FN, best, best_ms);
    return rc;
}

}  // namespace

extern "C" {

int bb_rmsnorm_swiglu_ffn_tune(const void* X, const void* g, const void* W1, const void* W3, const void* W2,
                               void* Y, int64_t M, int64_t D, int64_t F, float eps, void* stream, int reps,
                               int* chosen, float* ms) {
    if (int rc = validate_ffn(X, g, W1, W3, W2, Y, M, D, F, eps)) return rc;
    if (M == 0) return BB_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_mu);
    return tune_locked(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F, reps, as_stream(stream), chosen, ms,
                       [&](int v) { return ffn_locked(v, X, g, W1, W3, W2, Y, M, D, F, eps, stream); });
}

int bb_layernorm_matmul_tune(const void* X, const void* gamma, const void* beta, const void* W, void* Y,
                             int64_t M, int64_t D, int64_t N, float eps, void* stream, int reps, int* chosen,
                             float* ms) {
    if (int rc = validate_ln(X, gamma, beta, W, Y, M, D, N, eps)) return rc;
    if (M == 0) return BB_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_mu);
    return tune_locked(BB_OP_LAYERNORM_MATMUL, M, D, N, reps, as_stream(stream), chosen, ms,
                       [&](int v) { return ln_locked(v, X, gamma, beta, W, Y, M, D, N, eps, stream); });
}

int bb_tuned_variant(int op, int64_t M, int64_t D, int64_t F_or_N) {
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_tuned.find(TuneKey{op, M, D, F_or_N});
    return it == g_tuned.end() ? BB_VARIANT_AUTO : it->second;
}

int bb_tune_clear(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_tuned.clear();
    return BB_OK;
}

// ---------------------------------------------------------------- profiling
int bb_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (on && !g_prof.created) {
        for (auto& c : g_prof.ring)
            for (int i = 0; i <= kMaxProf; ++i) BB_HIP(hipEventCreate(&c.ev[i]));
        g_prof.created = true;
    }
    g_prof.on = on != 0;
    g_prof.calls = 0;
    for (auto& c : g_prof.ring) c.n = 0;
    return BB_OK;
}

int bb_profile_calls(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    return (int)std::min<long>(g_prof.calls, kProfRing);
}

int bb_profile_count_of(int back) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (back < 0 || back >= std::min<long>(g_prof.calls, kProfRing)) return 0;
    return g_prof.ring[(g_prof.calls - 1 - back) % kProfRing].n;
}

int bb_profile_get_of(int back, int i, float* ms, const char** name) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!ms) return BB_ERR_NULL;
    if (!g_prof.created || back < 0 || back >= std::min<long>(g_prof.calls, kProfRing)) return BB_ERR_SHAPE;
    ProfCall& c = g_prof.ring[(g_prof.calls - 1 - back) % kProfRing];
    if (i < 0 || i >= c.n) return BB_ERR_SHAPE;
    BB_HIP(hipEventSynchronize(c.ev[i + 1]));
    BB_HIP(hipEventElapsedTime(ms, c.ev[i], c.ev[i + 1]));
    if (name) *name = c.name[i];
    return BB_OK;
}

int bb_profile_count(void) { return bb_profile_count_of(0); }

int bb_profile_get(int i, float* ms, const char** name) { return bb_profile_get_of(0, i, ms, name); }

// ------------------------------------------------------------- calibration
int bb_calib_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst) return BB_ERR_NULL;
    if ((bytes & 15) || misaligned(src) || misaligned(dst)) return BB_ERR_ALIGN;
    if (overlaps(src, bytes, dst, bytes)) return BB_ERR_ALIAS;
    if (bytes == 0) return BB_OK;
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    hipLaunchKernelGGL(calib_copy_kernel, dim3(dev->cus * 8), dim3(256), 0, as_stream(stream),
                       (const u32x4*)src, (u32x4*)dst, bytes / 16);
    BB_HIP(hipGetLastError());
    return BB_OK;
}

int bb_calib_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink) return BB_ERR_NULL;
    if ((bytes & 15) || misaligned(src) || misaligned(sink)) return BB_ERR_ALIGN;
    if (bytes == 0) return BB_OK;
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    hipLaunchKernelGGL(calib_read_kernel, dim3(dev->cus), dim3(256), 0, as_stream(stream), (const u32x4*)src,
                       bytes / 16, (float*)sink);
    BB_HIP(hipGetLastError());
    return BB_OK;
}

int bb_calib_mfma(int workgroups, int iters, void* sink, void* stream) {
    if (!sink) return BB_ERR_NULL;
    if (workgroups <= 0 || iters <= 0 || workgroups > 65536 || iters > (1 << 22)) return BB_ERR_SHAPE;
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    hipLaunchKernelGGL(calib_mfma_kernel, dim3(workgroups), dim3(256), 0, as_stream(stream), (float*)sink, iters);
    BB_HIP(hipGetLastError());
    return BB_OK;
}

int bb_calib_mfma_data(const void* operands, int workgroups, int iters, void* sink, void* stream) {
    if (!sink || !operands) return BB_ERR_NULL;
    if (misaligned(operands) || misaligned(sink)) return BB_ERR_ALIGN;
    if (workgroups <= 0 || iters <= 0 || workgroups > 65536 || iters > (1 << 22)) return BB_ERR_SHAPE;
    const DeviceInfo* dev = nullptr;
    if (int rc = current_device_info(&dev)) return rc;
    hipLaunchKernelGGL(calib_mfma_data_kernel, dim3(workgroups), dim3(256), 0, as_stream(stream),
                       (const u32x4*)operands, (float*)sink, iters);
    BB_HIP(hipGetLastError());
    return BB_OK;
}

}  // extern "C"
