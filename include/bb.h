/*
 * bb -- fused RMSNorm -> FFN-SwiGLU and LayerNorm -> matmul for AMD MI355X
 * (gfx950), the two fused operators derived in "Blockbuster, Part 1:
 * Block-level AI Operator Fusion" (Example 3, Flash-RMSNorm+FFN-SwiGLU, and
 * Example 2, Flash-LayerNorm+Matmul).
 *
 * C ABI.  Every tensor pointer is a DEVICE pointer to bf16 elements (raw
 * 16-bit patterns), dense row-major with no strides, unless a parameter says
 * otherwise.  The caller owns every buffer; the library keeps no user pointer
 * after a call returns.  Inputs are only read, the output is only written and
 * must not overlap any input.  Calls enqueue work on `stream` (a hipStream_t
 * passed as void*, NULL = the default stream) and return without
 * synchronising; no host<->device copy is made.  No exception crosses the
 * boundary and nothing is printed unless the environment variable BB_LOG is
 * set.  Only gfx950 devices are supported.
 *
 * Every function returning int returns BB_OK (0) or a negative bb_status.
 * Argument checks happen before anything is launched, so a failed call has
 * no effect on the output buffer.
 */
#ifndef BB_H_
#define BB_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BB_VERSION 100 /* major*10000 + minor*100 + patch */

typedef enum bb_status {
    BB_OK = 0,
    BB_ERR_NULL = -1,      /* a pointer is NULL while its extent is > 0           */
    BB_ERR_SHAPE = -2,     /* M < 0, D/F/N <= 0, D/F/N not a multiple of 8, or a
                              size beyond the supported range (2^31-1 elements
                              per row-major dimension product per tile index)   */
    BB_ERR_ALIGN = -3,     /* a pointer is not 16-byte aligned                    */
    BB_ERR_EPS = -4,       /* eps negative, NaN or infinite                       */
    BB_ERR_ALIAS = -5,     /* the output overlaps an input                        */
    BB_ERR_ARCH = -6,      /* the current device is not gfx950                    */
    BB_ERR_WORKSPACE = -7, /* workspace missing, too small or misaligned          */
    BB_ERR_HIP = -8,       /* a HIP call failed; see bb_last_hip_error()          */
    BB_ERR_VARIANT = -9,   /* unknown variant, or one that cannot run this shape  */
    BB_ERR_TIMEOUT = -10,  /* a weight-streaming kernel of an EARLIER launch gave
                              up waiting for another workgroup: that launch's
                              output is invalid (see bb_check_fault)              */
    BB_ERR_INIT = -11      /* bb_rmsnorm_swiglu_ffn_static before bb_init (or any
                              other call of this library) on the current device   */
} bb_status;

/* Which fused block program of Example 3 a call of bb_rmsnorm_swiglu_ffn runs.
 * Both are the first snapshot the fusion algorithm returns (taken before any
 * map extension, so no work is replicated): row statistics, the K-map that
 * produces the hidden blocks, the N-map that reduces over them.
 *
 * BB_VARIANT_SNAPSHOT1 compute-bound form for many rows.  A norm-prologue dual
 *                      GEMM (sum x^2 and both products from one pass over X,
 *                      inverse norm after the dots, Swish*gate epilogue)
 *                      writes the hidden once as bf16 to the workspace; a
 *                      second GEMM contracts it with W2.  Two launches.  With
 *                      few rows (fewer output tiles than half the compute
 *                      units) either contraction is split over several
 *                      workgroups per tile, whose fp32 partial results a small
 *                      kernel adds in fixed order before the epilogue (Rule 3's
 *                      parallel reduction without atomics): up to four launches.
 * BB_VARIANT_STREAM    bandwidth-bound form for M <= 32 rows (transposed-weight
 *                      entry points: M <= 16).  One persistent
 *                      kernel (one workgroup per compute unit, all resident)
 *                      streams W1, W3 and then W2 exactly once; both
 *                      reductions (over the model dimension and over the
 *                      hidden dimension) run in parallel over all workgroups
 *                      (Rule 3; Example 3's epilogue proposes it for the
 *                      K-map) through per-workgroup partial-sum slots that a
 *                      short phase adds up.  The hidden block (M x F) passes
 *                      through a cache-resident scratch between the phases.
 *                      The kernel synchronises its workgroups through counters
 *                      in the workspace that only the kernels touch: a launch
 *                      carries no host-side state and, once a first call has
 *                      set up the workspace, may be captured into a HIP graph
 *                      and replayed.
 * BB_VARIANT_UNFUSED   the initial block program (what the *_unfused entry points
 *                       run); a candidate of the measured selection below.
 * BB_VARIANT_PRESCALE  (FFN with M > 16; LN -> matmul) SNAPSHOT1 with the statistics loop as a
 *                       kernel of its own, as Example 3's first snapshot has
 *                       it (a loop over the model dimension before the K-map):
 *                       a row kernel writes bf16(x g) and the inverse norms,
 *                       the dual product runs the plain main loop (no vector
 *                       work on the A operand) and applies the inverse norm,
 *                       Swish and the Hadamard product in its epilogue.  Same
 *                       arithmetic as SNAPSHOT1; costs one extra pass over X
 *                       (M D bf16 written and read).  For LN -> matmul the row
 *                       kernel writes bf16(x gamma), the means and the inverse
 *                       standard deviations (two passes over the row), the
 *                       product keeps the epilogue r (P - mu c) + b.  A
 *                       candidate of the measured selection below.
 * BB_VARIANT_NEST      (FFN with D <= 512) the LAST snapshot of Example 3, the
 *                       fully fused nest of the listing after Step 26, with one
 *                       block of output columns (N = 1: the case of the
 *                       Epilogue in which the extended maps replicate no work).
 *                       ONE launch, a workgroup per block of 16 rows: statistics
 *                       loop, then a serial loop over blocks of 128 hidden units
 *                       (both products over the whole model dimension, inverse
 *                       norm after the dots, Swish, gate, the block contracted
 *                       with its rows of W2) with the 16 x D block of outputs in
 *                       registers throughout.  The hidden never leaves the
 *                       compute unit; no workspace is touched.  BB_ERR_VARIANT
 *                       when D > 512 (the output block no longer fits).  A
 *                       candidate of the measured selection below and the
 *                       rule of thumb's choice for small weight matrices (one
 *                       compute unit per 16 rows reads all three of them
 *                       alone: it wins where six pairs of wavefronts take all
 *                       hidden blocks at once).
 * BB_VARIANT_AUTO      the measured selection for exactly this shape if
 *                       bb_*_tune has recorded one, else NEST for D <= 256,
 *                       F <= 768 and M <= 4096, else STREAM for M <= 32,
 *                       SNAPSHOT1 up to 255 rows and PRESCALE from 256 rows on
 *                       (the table measured on an MI355X for D = 4096,
 *                       F = 11008); LN -> matmul: SNAPSHOT1 up to 255 rows,
 *                       PRESCALE from 256 on.
 */
typedef enum bb_variant {
    BB_VARIANT_AUTO = 0,
    BB_VARIANT_STREAM = 1,
    BB_VARIANT_SNAPSHOT1 = 2,
    BB_VARIANT_UNFUSED = 3,
    BB_VARIANT_PRESCALE = 4,
    BB_VARIANT_NEST = 5
} bb_variant;

typedef enum bb_op {
    BB_OP_RMSNORM_SWIGLU_FFN = 0,
    BB_OP_LAYERNORM_MATMUL = 1,
    BB_OP_RMSNORM_SWIGLU_FFN_UNFUSED = 2,
    BB_OP_LAYERNORM_MATMUL_UNFUSED = 3
} bb_op;

/* ------------------------------------------------------------------------
 * Y = ( SiLU(Xh W1) (.) (Xh W3) ) W2,   Xh[i,:] = g (.) X[i,:] / sqrt(mean(X[i,:]^2) + eps)
 *
 * The array program of Example 3 ("RMSNorm and FeedForward-SwiGLU") with the
 * root MEAN square, eps inside the root and a per-column gain g; SiLU(x) =
 * x/(1+exp(-x)) acts on the W1 product.  W1, W3, W2 are the paper's W, V, U.
 *
 *   X  [M, D]  in      g  [D]  in
 *   W1 [D, F]  in      W3 [D, F]  in      W2 [F, D]  in
 *   Y  [M, D]  out (bf16, every element written)
 *
 * Arithmetic: bf16 operands, fp32 accumulation and statistics, the gained row
 * bf16(x*g) and the hidden are rounded to bf16 before they enter a matrix
 * instruction, the inverse norm is applied after the first contraction
 * (Rule 4).  M may be any value >= 0 (M == 0 returns BB_OK and launches
 * nothing); D and F must be positive multiples of 8.
 * Needs a workspace of bb_workspace_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F)
 * bytes: taken from bb_set_workspace() if one is set, otherwise allocated by
 * the library on first use (that call may synchronise the device) and cached.
 * Two calls that share the workspace must not overlap in time.
 */
int bb_rmsnorm_swiglu_ffn(const void* X, const void* g, const void* W1,
                          const void* W3, const void* W2, void* Y,
                          int64_t M, int64_t D, int64_t F, float eps,
                          void* stream);

/* ------------------------------------------------------------------------
 * Y = LN(X) W,  LN(x) = gamma (.) (x - mean(x)) / sqrt(var(x) + eps) + beta
 *
 * The array program of Example 2 ("LayerNorm and Matmul") with the biased
 * variance of its sigma formula, plus gamma, beta and eps.  Computed in the
 * fused form the paper ends with: one pass over X per output tile that
 * accumulates sum x, sum x^2 and (X diag(gamma)) W together; the mean is
 * removed after the contraction through the column vector gamma^T W (Rule 5)
 * and rows are scaled by the inverse standard deviation afterwards (Rule 4).
 *
 *   X [M, D] in   gamma [D] in   beta [D] in   W [D, N] in   Y [M, N] out
 *
 * D and N positive multiples of 8, M >= 0.  With the statistics inside the
 * product loop (BB_VARIANT_SNAPSHOT1: AUTO's choice below 256 rows) the
 * variance is the one-pass form sum(x^2)/D - mean^2 in fp32: rows whose
 * |mean|/std exceeds a few hundred lose accuracy.  BB_VARIANT_PRESCALE (AUTO
 * from 256 rows on) takes two passes over the row (mean, then the sum of
 * squared deviations) and has no such limit, so the two sides of the row
 * threshold differ on such inputs; a caller with large means selects
 * BB_VARIANT_PRESCALE or BB_VARIANT_UNFUSED for every M.  Workspace: bb_workspace_bytes(
 * BB_OP_LAYERNORM_MATMUL, M, D, N) (fp32 column vectors of length N and their
 * partial sums).
 */
int bb_layernorm_matmul(const void* X, const void* gamma, const void* beta,
                        const void* W, void* Y, int64_t M, int64_t D,
                        int64_t N, float eps, void* stream);

/* ------------------------------------------------------------------------
 * The same two operators with the weights given TRANSPOSED, which is the form
 * the paper's block programs take their inputs in (W^T, V^T, U^T; Section 2.1
 * says non-row-major inputs are transposed on their way to local memory) and
 * the layout of linear-layer checkpoints:
 *
 *   W1t [F, D], W3t [F, D], W2t [D, F]   with  W1t[f,d] = W1[d,f]  etc.
 *   Wt  [N, D]                           with  Wt[n,d]  = W[d,n]
 *
 * Everything else (arguments, arithmetic, results, workspace of the op without
 * the suffix, errors) is as for bb_rmsnorm_swiglu_ffn / bb_layernorm_matmul.
 * The contraction index is contiguous in these layouts, so the weight tiles
 * need no transposition on chip.  The FFN with at most 16 rows runs a
 * weight-streaming kernel of its own for this layout (every workgroup owns a
 * contiguous range of rows of W1t, W3t and then of W2t: no partial sums between
 * workgroups, one grid barrier), unless bb_set_variant selected a tiled variant
 * or the shape gives a workgroup more than 128 hidden units or output columns
 * (F or D above 128 times the number of compute units); more rows, and
 * bb_layernorm_matmul_t at any size, go through the tiled kernels (for few rows
 * with the split contraction, from 256 rows on with the statistics loop as a
 * kernel of its own, see BB_VARIANT_PRESCALE).
 */
int bb_rmsnorm_swiglu_ffn_t(const void* X, const void* g, const void* W1t,
                            const void* W3t, const void* W2t, void* Y,
                            int64_t M, int64_t D, int64_t F, float eps,
                            void* stream);
int bb_layernorm_matmul_t(const void* X, const void* gamma, const void* beta,
                          const void* Wt, void* Y, int64_t M, int64_t D,
                          int64_t N, float eps, void* stream);

/* ------------------------------------------------------------------------
 * The FFN operator with the residual connection of a decoder block fused into
 * the last kernel's epilogue (the operator that follows Example 3's program in
 * a Transformer block; Section 2 names fusing past operator boundaries as the
 * point of block-level fusion):
 *
 *   Y = R + ( SiLU(Xh W1) * (Xh W3) ) W2          R [M, D] bf16, row-major
 *
 * The sum is formed in fp32 before the output's one rounding to bf16.  R may be
 * X (the usual pre-norm block y = x + FFN(norm(x))).  Y may be R itself (in
 * place), and then also X; otherwise Y must overlap no input.  Variants: as
 * bb_rmsnorm_swiglu_ffn, except that a recorded or forced UNFUSED selection
 * runs SNAPSHOT1 (the unfused program has no such epilogue).  _t: transposed
 * weights as for bb_rmsnorm_swiglu_ffn_t.  Workspace and errors as for the
 * operator without the residual.
 */
int bb_rmsnorm_swiglu_ffn_residual(const void* X, const void* g, const void* W1,
                                   const void* W3, const void* W2, const void* R,
                                   void* Y, int64_t M, int64_t D, int64_t F,
                                   float eps, void* stream);
int bb_rmsnorm_swiglu_ffn_residual_t(const void* X, const void* g,
                                     const void* W1t, const void* W3t,
                                     const void* W2t, const void* R, void* Y,
                                     int64_t M, int64_t D, int64_t F, float eps,
                                     void* stream);

/* ------------------------------------------------------------------------
 * The UNFUSED block programs (Example 3 / Example 2, initial block programs):
 * one kernel per array operator, every intermediate materialised in global
 * memory.  Built from the same tile primitives; exported so that the cost of
 * not fusing can be timed.  Same arguments and results as the fused calls.
 * FFN: rmsnorm rows -> Xh (bf16) ; P = Xh W1 ; Q = Xh W3 ; H = SiLU(P)*Q ;
 * Y = H W2  (5 launches).  LN: layernorm rows -> Z ; Y = Z W (2 launches).
 * Workspace: bb_workspace_bytes(BB_OP_*_UNFUSED, ...).
 */
int bb_rmsnorm_swiglu_ffn_unfused(const void* X, const void* g, const void* W1,
                                  const void* W3, const void* W2, void* Y,
                                  int64_t M, int64_t D, int64_t F, float eps,
                                  void* stream);
int bb_layernorm_matmul_unfused(const void* X, const void* gamma,
                                const void* beta, const void* W, void* Y,
                                int64_t M, int64_t D, int64_t N, float eps,
                                void* stream);

/* ------------------------------------------------------------------------
 * Attention (Example 1; numerics of the Appendix):
 *
 *   O[b] = softmax_rows( Q[b] K[b]^T / sqrt(d) ) V[b]         b = 0 .. B-1
 *
 * as ONE kernel: the loop nest Example 1 ends with (per block of queries a
 * serial loop over key blocks that accumulates the dot with the value block
 * and the row sums of the exponentiated scores, then the division), with the
 * feature and value dimensions unsplit.  The exponentiated score blocks are
 * the Appendix's significand-exponent pairs in row-wise form: one exponent per
 * query row, accumulators rescaled to the larger exponent before a block is
 * added, so large scores neither overflow nor lose the row.  A row's exponent
 * is a running maximum of its scaled scores that moves only when a block's
 * maximum exceeds it by more than 8 binary orders of magnitude (significands
 * stay below 2^8).
 *
 *   Q [B, M, d], K [B, N, d], V [B, N, dv], O [B, M, dv]   bf16, row-major,
 *   densely packed, device pointers, 16-byte aligned; O overlaps no input.
 *
 * d and dv are 64 or 128; B, M >= 0 (zero: nothing is done), 1 <= N < 2^24,
 * M <= 2^24.  Scores are accumulated in fp32, scaled and exponentiated in
 * fp32 (base-2 exponential of score * log2(e)/sqrt(d)), rounded to bf16 as
 * the operand of the second product; output sums and row sums in fp32, the
 * quotient rounded to bf16 once.  Errors as for the other operators.
 *
 * Few queries (decoding: fewer (problem, 128-query block) pairs than half the
 * compute units, and at least 8 blocks of 64 keys): the loop over the key
 * blocks is cut into equal ranges that run in parallel workgroups (Rule 3's
 * parallel form); each stores its unnormalised output and row sum with their
 * row exponents, fp32, and a second kernel adds these significand-exponent
 * pairs (Appendix: both terms brought to the larger exponent) in a fixed
 * order and divides.
 * One query per problem (M = 1, any N): no matrix product is left; a
 * streaming kernel reads K and V once with every lane loading (fp32 dot
 * products and probabilities, Example 1's online softmax per wavefront over
 * blocks of 64 keys), workgroups share a problem's keys as above, and the
 * workgroup of a problem that finishes last adds the pairs (arrival counters
 * at the start of the workspace, which every launch leaves at zero): one
 * launch.
 * This path uses bb_attention_workspace_bytes(B, M, N, d, dv) bytes of the
 * library workspace (0 when M > 1 and the keys are not split; see
 * bb_set_workspace).
 * The entry points share the workspace: a launch captured into a HIP graph
 * (this one with M = 1, or a BB_VARIANT_STREAM one) is replayed only while
 * no other entry point of the library, and no call that needs a larger
 * workspace, has run since its capture.  The environment variable BB_ATTN_WAVES=4|8 (read once) forces
 * the number of wavefronts per workgroup (32 queries each) instead of the
 * shape-driven choice; a query row is computed by one wavefront in the same
 * order either way, so the results are bit-identical.
 */
int bb_attention(const void* Q, const void* K, const void* V, void* O,
                 int64_t B, int64_t M, int64_t N, int64_t d, int64_t dv,
                 void* stream);
size_t bb_attention_workspace_bytes(int64_t B, int64_t M, int64_t N, int64_t d,
                                    int64_t dv);

/* ------------------------------------------------------------------------
 * Measured selection (Section 4: the fusion algorithm returns several
 * snapshots of a candidate, partially and fully fused, and a selection step
 * keeps the one that runs fastest; Example 3's epilogue lists the forms).
 *
 * bb_*_tune run every candidate program of the operator on the caller's
 * operands (same arguments as the operator): STREAM (FFN, M <= 32 only),
 * SNAPSHOT1, UNFUSED, PRESCALE (for the FFN M > 16 only); each once untimed and then `reps` (1..1000) times between
 * two events on `stream`, which the call waits for.  The fastest is recorded
 * for exactly this (operator, M, D, F or N) in a process-wide table that
 * BB_VARIANT_AUTO consults, so later calls of bb_rmsnorm_swiglu_ffn /
 * bb_layernorm_matmul with that shape run it.  Y holds the result of the last
 * candidate run (all candidates compute the same operator).
 *   chosen (host, may be NULL): the recorded variant.
 *   ms (host, 6 floats, may be NULL): ms[v] = mean milliseconds of variant v,
 *     -1 where v is not a candidate; ms[0] = the fastest.
 * A candidate that does not fit a caller-provided workspace is skipped.
 * bb_set_workspace and bb_tune_clear empty the table.  bb_tuned_variant returns
 * the recorded variant of a shape, BB_VARIANT_AUTO (0) if none.
 * The *_t entry points and bb_attention have one program each and no selection.
 */
int bb_rmsnorm_swiglu_ffn_tune(const void* X, const void* g, const void* W1,
                               const void* W3, const void* W2, void* Y,
                               int64_t M, int64_t D, int64_t F, float eps,
                               void* stream, int reps, int* chosen, float* ms);
int bb_layernorm_matmul_tune(const void* X, const void* gamma,
                             const void* beta, const void* W, void* Y,
                             int64_t M, int64_t D, int64_t N, float eps,
                             void* stream, int reps, int* chosen, float* ms);
int bb_tuned_variant(int op, int64_t M, int64_t D, int64_t F_or_N);
int bb_tune_clear(void);

/* ------------------------------------------------------------------------
 * Workspace and variant control.
 *
 * bb_workspace_bytes: bytes of device scratch `op` needs for the given sizes
 *   (third size is F for the FFN ops, N for the LN ops); the maximum over
 *   STREAM, SNAPSHOT1 and PRESCALE.  The UNFUSED candidate needs
 *   bb_workspace_bytes(BB_OP_*_UNFUSED, ...): a caller who provides the
 *   workspace and wants it considered by bb_*_tune sizes for the larger of the
 *   two.  Returns 0 for invalid sizes.
 * bb_set_workspace: hand the library a device buffer (256-byte aligned) to use
 *   instead of its own allocation; (NULL, 0) returns to the internal one.  The
 *   buffer must be ZERO-FILLED when it is handed over (the streaming variant
 *   keeps all-zero accumulators between calls) and stays owned by the caller.
 * bb_set_variant / bb_get_variant: process-wide choice for
 *   bb_rmsnorm_swiglu_ffn (default BB_VARIANT_AUTO, or the BB_VARIANT
 *   environment variable: "auto", "stream", "snapshot1", "unfused", "prescale");
 *   BB_VARIANT_UNFUSED also applies to bb_layernorm_matmul.
 * bb_shutdown: frees the library's own workspace (synchronises the device).
 */
size_t bb_workspace_bytes(int op, int64_t M, int64_t D, int64_t F_or_N);
int bb_set_workspace(void* dptr, size_t bytes);
int bb_set_variant(int variant);
int bb_get_variant(void);
int bb_shutdown(void);

/* ------------------------------------------------------------------------
 * For callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.
 *
 * bb_init: sets the CURRENT device up (device properties, the 64-byte pinned
 *   host word of bb_check_fault, the address of this device's copy of the
 *   static scratch array).  The only call of this section that allocates
 *   (that host word, once per device).  Every other entry point of the library
 *   does the same on its first call on a device.  BB_OK, BB_ERR_ARCH, BB_ERR_HIP.
 * bb_rmsnorm_swiglu_ffn_static: bb_rmsnorm_swiglu_ffn (same arguments, same
 *   kernels, same variant choice, bit-identical output) with its scratch (the
 *   hidden H, partial results of split contractions, the streaming kernels'
 *   partial sums and synchronisation words) in a static device array of
 *   BB_STATIC_SCRATCH_BYTES that each device holds from the loading of the
 *   library to the end of the process.  Calls no hipMalloc, hipFree, event or
 *   stream creation; what must start at zero is cleared by a kernel on
 *   `stream` (no memset node), so the call can be captured into a HIP graph.
 *   Neither reads nor changes the workspace of bb_set_workspace.
 *   Errors: those of bb_rmsnorm_swiglu_ffn, and
 *     BB_ERR_INIT       the current device has not been set up (bb_init);
 *     BB_ERR_WORKSPACE  bb_workspace_bytes(BB_OP_RMSNORM_SWIGLU_FFN, M, D, F)
 *                       exceeds BB_STATIC_SCRATCH_BYTES: nothing is launched
 *                       (M=64 D=512 F=1408 needs 2 MiB, M=16 D=4096 F=11008
 *                       13 MiB, M=300 D=2048 F=5632 28 MiB; M=4096 D=4096
 *                       F=11008 needs 118 MiB and is rejected);
 *     BB_ERR_VARIANT    BB_VARIANT_UNFUSED is set (that program has its own,
 *                       larger scratch).
 *   All calls on one device share that device's array: calls that overlap in
 *   time on one device (different streams, or threads) race; order them.
 */
#define BB_STATIC_SCRATCH_BYTES (32u << 20)
int bb_init(void);
int bb_rmsnorm_swiglu_ffn_static(const void* X, const void* g, const void* W1,
                                 const void* W3, const void* W2, void* Y,
                                 int64_t M, int64_t D, int64_t F, float eps,
                                 void* stream);

/* ------------------------------------------------------------------------
 * Diagnostics.
 */
const char* bb_status_string(int status);
int bb_version(void);
int bb_last_hip_error(void); /* raw hipError_t of the last BB_ERR_HIP, else 0 */

/* ------------------------------------------------------------------------
 * Failure of a weight-streaming launch (BB_VARIANT_STREAM kernels, both
 * weight layouts).  Their workgroups wait for each other inside the kernel
 * (Example 3's epilogue: the parallel K-map hands partial results from
 * processor to processor), which needs every workgroup resident at once: the
 * launch must have the WHOLE device (no other kernel running beside it, on any
 * stream), and its synchronisation words in the workspace must not be
 * overwritten while it runs.  Every such wait is bounded (about two seconds).
 * A wait that gives up lets the kernel run to its end with an INVALID output
 * and sets a flag in host memory.  The flag is reported once, as
 * BB_ERR_TIMEOUT, by the next bb_rmsnorm_swiglu_ffn* call on that device (which
 * then launches nothing) or by bb_check_fault; either clears it and has the
 * synchronisation words zeroed again before the next launch.  The flag is set by
 * the kernel when it gives up, so it is seen only after that launch has run:
 * synchronise the stream before bb_check_fault to learn about the launches
 * issued so far.
 * bb_check_fault:          BB_OK, or BB_ERR_TIMEOUT once per failure.
 * bb_debug_inject_fault:   sets the flag from the host (tests of the path above).
 * bb_debug_set_spin_limit: polls after which a wait gives up (default 8000000;
 *                          0 = every wait that is not satisfied at once gives
 *                          up, for tests: every kernel still runs to its end).
 */
int bb_check_fault(void);
int bb_debug_inject_fault(void);
int bb_debug_set_spin_limit(unsigned polls);

/* ------------------------------------------------------------------------
 * Per-kernel timing of the most recent operator calls, for roofline reports.
 * While enabled, every operator call records a HIP event on its stream before
 * its first kernel and after each kernel (this serialises nothing but adds a
 * few event packets, so time whole calls with profiling off).  The last 64
 * calls are kept, so kernels can be timed inside a run of back-to-back calls
 * (a call timed alone starts on an idle chip and reads longer).
 * bb_profile_enable: switches recording on or off and forgets what was kept.
 * bb_profile_calls:  calls kept (at most 64).
 * bb_profile_count_of / bb_profile_get_of: kernels recorded by the call `back`
 *                   calls before the most recent one (0 = the most recent);
 *                   waits for kernel i of that call and returns its duration
 *                   in ms and a static name (host pointers).  BB_ERR_SHAPE for
 *                   an index out of range.
 * bb_profile_count / bb_profile_get: the same for the most recent call.
 */
int bb_profile_enable(int on);
int bb_profile_calls(void);
int bb_profile_count_of(int back);
int bb_profile_get_of(int back, int i, float* ms, const char** name);
int bb_profile_count(void);
int bb_profile_get(int i, float* ms, const char** name);

/* ------------------------------------------------------------------------
 * Calibration kernels for roofline denominators (not part of the operators).
 * bb_calib_copy:  dst[i] = src[i] for `bytes` bytes (multiple of 16), a plain
 *                 grid-stride copy; known traffic = bytes read + bytes written.
 * bb_calib_read:  streams `bytes` bytes (multiple of 16) and writes one float
 *                 per workgroup to `sink` (>= 4096 floats).
 * bb_calib_mfma:  each wave issues `iters` x 16 independent bf16
 *                 32x32x16 matrix instructions on register operands; `sink`
 *                 (>= 64 floats) is only there to keep the work alive.  Flops
 *                 issued = workgroups * 4 waves * iters * 16 * 32768.
 * bb_calib_mfma_data: the same instruction stream with operands read from
 *                 `operands` (device, 16-byte aligned, 32 KiB of bf16 values):
 *                 with random real-valued operands the matrix cores draw more
 *                 power than with constants and the clock drops, so this is
 *                 the rate attainable on real data.
 */
int bb_calib_copy(const void* src, void* dst, size_t bytes, void* stream);
int bb_calib_read(const void* src, size_t bytes, void* sink, void* stream);
int bb_calib_mfma(int workgroups, int iters, void* sink, void* stream);
int bb_calib_mfma_data(const void* operands, int workgroups, int iters, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BB_H_ */
