/*
 * lemo.h -- C ABI of the MI355X (gfx950) Contextual Token Sparsity hot path
 *           (LeMo, arXiv 2501.09767: Sec. 4.2 token elimination, Sec. 4.4 permutation-free kernels).
 *
 * One layer's path is four calls on one HIP stream:
 *
 *   lemo_score_segments   informativeness of every token from the layer's attention        (Sec. 4.2, Eq. 1-2)
 *   lemo_select_topk      which tokens of each segment (token block) to keep               (Sec. 4.2)
 *   lemo_gather_gemm      consumer GEMM that loads the kept rows straight from the input   (Sec. 4.4)
 *   lemo_scatter_grad     in-place add of per-kept-row results / gradients back into [S,C] (Sec. 4.4)
 *
 * Beside them: the paper's block-wise criterion and threshold rule (lemo_score_blocks, lemo_threshold_init,
 * lemo_select_threshold; Sec. 4.2 Eq. 2, Alg. 1 step 1), the attention block over the kept tokens with its
 * projection added back in place (lemo_kept_attention, lemo_gather_gemm_add; Sec. 4.4), and the gradients
 * of the selective-load GEMM (lemo_gather_gemm_dx, lemo_gather_gemm_dw).
 *
 * Conventions shared by every call
 *   - Pointers are DEVICE pointers unless the comment says "host".  The caller owns every buffer;
 *     the library never allocates, frees or keeps a pointer after the call returns.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null stream) and the
 *     call returns without synchronising.  Calls on one stream execute in order.
 *   - Arguments are validated on the host before anything is launched.  A negative return code
 *     means nothing was launched and no output was touched.  Nothing is printed, thrown or aborted.
 *   - bf16 is the upper half of an IEEE binary32; every reduction accumulates in binary32 and
 *     rounds to nearest-even once when a bf16 result is stored (mixed precision, Sec. 6.1).
 *   - Strides and leading dimensions are in ELEMENTS.  Base pointers and row starts must be 16-byte
 *     aligned (so strides are multiples of 8 for bf16, 4 for fp32); otherwise LEMO_ERR_ALIGN.
 *   - No global mutable state beyond one-time kernel attribute set-up: calls are re-entrant and may be
 *     issued from several host threads.  Calls that are given a workspace use it until their work on
 *     the stream has finished; two calls in flight at once need two workspaces.
 *   - The calls only launch kernels (no allocation, no memset, no host synchronisation), so a stream
 *     that carries them may be captured into a HIP graph -- once each entry point has been called
 *     for its dtype and head size outside a capture: the first such call raises the dynamic-LDS
 *     limit of its kernels (hipFuncSetAttribute), which is not a stream operation.
 */
#ifndef LEMO_H
#define LEMO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LEMO_F32 = 0, LEMO_BF16 = 1 } lemo_dtype_t;

/* flags of lemo_score_segments */
enum {
    LEMO_CAUSAL = 1u,       /* query i attends keys j <= i (autoregressive layers); else all keys   */
    LEMO_EXCLUDE_SELF = 2u  /* leave the i == j term out of a token's score, as Eq. 1 does           */
};

/* mode of lemo_scatter_grad */
enum {
    LEMO_SCATTER_ACCUMULATE = 0, /* dX[idx[m]] += G[m]; other rows untouched (padding adds zero)     */
    LEMO_SCATTER_ZERO_PAD = 1    /* dX = G zero-padded to S rows: kept rows = G[m], other rows = +0   */
};

/* return codes */
enum {
    LEMO_OK = 0,
    LEMO_ERR_NULL = -1,        /* a required pointer is NULL                                         */
    LEMO_ERR_SHAPE = -2,       /* a size, stride or count is out of range or inconsistent            */
    LEMO_ERR_DTYPE = -3,       /* dtype is not LEMO_F32 / LEMO_BF16                                  */
    LEMO_ERR_WORKSPACE = -4,   /* workspace smaller than lemo_score_workspace_bytes reports          */
    LEMO_ERR_ALIGN = -5,       /* pointer or stride breaks the 16-byte alignment rule                */
    LEMO_ERR_UNSUPPORTED = -6, /* valid request outside what the kernels are built for               */
    LEMO_ERR_HIP = -7          /* the HIP runtime refused a launch                                   */
};

/* host: text for a return code (static storage, never NULL) */
const char* lemo_strerror(int code);

/* host: kept tokens per FULL segment of length L at keep ratio `ratio`: ceil(ratio * L) clamped to
 * [1, L] (a 1e-9 slack keeps exact products such as 0.5 * 128 from rounding up).  0 if L <= 0. */
int32_t lemo_keep_k(int32_t L, double ratio);

/* host: M = total kept tokens for S tokens cut into segments of L keeping k per full segment; a
 * ragged last segment of length t keeps ceil(k * t / L), at least 1.  -1 on bad arguments. */
int64_t lemo_kept_count(int64_t S, int32_t L, int32_t k);

/* host: bytes of device workspace lemo_score_segments needs for this shape.  Linear in S (row
 * statistics and per-head column sums, 3 * H * S floats): the S x S score matrix is never stored,
 * which is the property Sec. 4.3's overhead analysis asks of the scoring kernel. */
int lemo_score_workspace_bytes(int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                               size_t* bytes /* host, out */);

/*
 * Token informativeness (Sec. 4.2).  With P^h = softmax_j(scale * Q^h K^{g(h)T}) the attention
 * probabilities of query head h (row i over the keys query i may attend; g(h) = floor(h*H_kv/H)
 * is the KV head a query head reads), the call produces
 *
 *     colsum^h[j] = sum_i P^h[i][j]                       column sums, diagonal INCLUDED
 *     diag^h[j]   = P^h[j][j]
 *     scores[j]   = (1/H) * sum_h ( colsum^h[j] - [EXCLUDE_SELF] diag^h[j] )      (Eq. 1, head mean of Eq. 2)
 *
 * The key axis is processed one segment of L tokens at a time against tiles of queries; results do
 * not depend on L beyond binary32 summation order.  Two sweeps over Q K^T are made (row
 * log-sum-exp, then column sums); both run on the matrix cores (bf16 inputs) or in true binary32
 * (fp32 inputs), accumulate in binary32, and keep probabilities in binary32.
 *
 *   Q  [S, H, d]     element (i,h,c) at Q[i*q_tok_stride + h*q_head_stride + c]   (d contiguous)
 *   K  [S, H_kv, d]  likewise with the k_ strides
 *   scale            logit scale; <= 0 selects 1/sqrt(d)
 *   scores           [S] float, out
 *   colsum_per_head  [H, S] float, out, or NULL
 *   diag_per_head    [H, S] float, out, or NULL
 *   workspace        at least lemo_score_workspace_bytes() bytes, 256-byte aligned; contents are
 *                    scratch (undefined before and after)
 *
 * Supported: d in {64, 128}, H % H_kv == 0, 1 <= S < 2^31, L >= 1.  Deterministic: the same inputs
 * give the same bits on every run (no atomics).
 */
int lemo_score_segments(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d,
                        lemo_dtype_t dt, int64_t q_tok_stride, int64_t q_head_stride,
                        int64_t k_tok_stride, int64_t k_head_stride, float scale, int32_t L,
                        uint32_t flags, float* scores, float* colsum_per_head, float* diag_per_head,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * lemo_score_segments for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the
 * same bits in `scores`; the three [H, S] float planes live in a fixed array inside the library's code object
 * instead of a workspace, so the per-head outputs are not offered.
 *
 *   Limit: H * S <= 1048576 (12 MiB of scratch, held by every GPU the library runs on until the process
 *   ends); larger shapes return LEMO_ERR_UNSUPPORTED and launch nothing.
 *   The call allocates and frees nothing.  Its first call on a device looks the array's device address up
 *   (hipGetSymbolAddress, once per device, with that device current; LEMO_ERR_HIP if that fails) -- make that
 *   first call outside a stream capture, like the first call of any entry point.
 *   All calls on one GPU share the one array: two calls whose work overlaps in time on the same GPU (different
 *   streams, or different host threads) race; calls on one stream are ordered and safe.  The array keeps the
 *   last call's contents; the kernels write every element they later read, so nothing needs clearing.
 */
int lemo_score_segments_static(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d,
                               lemo_dtype_t dt, int64_t q_tok_stride, int64_t q_head_stride,
                               int64_t k_tok_stride, int64_t k_head_stride, float scale, int32_t L,
                               uint32_t flags, float* scores, void* stream);

/*
 * The three steps lemo_score_segments runs back to back, callable one at a time (same kernels, same
 * bits) so that each can be timed or reused.  Arguments mean what they mean above.
 *
 *   lemo_score_rowstats   sweep 1: lse2[h][i] = log2 sum_j 2^(c * <Q_i^h, K_j^g(h)>) over the keys query i
 *                         may attend, c = scale * log2(e)            -> lse2 [H, S] float, out
 *   lemo_score_colsums    sweep 2: colsum^h[j], diag^h[j] from Q, K and lse2 (read-only, [H, S]);
 *                         both outputs are required here             -> [H, S] float each, out
 *   lemo_score_head_mean  scores[j] = (1/H) sum_h (colsum - [EXCLUDE_SELF] diag), heads added in
 *                         ascending order                            -> scores [S] float, out
 */
int lemo_score_rowstats(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d,
                        lemo_dtype_t dt, int64_t q_tok_stride, int64_t q_head_stride,
                        int64_t k_tok_stride, int64_t k_head_stride, float scale, uint32_t flags,
                        float* lse2, void* stream);
int lemo_score_colsums(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d,
                       lemo_dtype_t dt, int64_t q_tok_stride, int64_t q_head_stride,
                       int64_t k_tok_stride, int64_t k_head_stride, float scale, int32_t L,
                       uint32_t flags, const float* lse2, float* colsum_per_head, float* diag_per_head,
                       void* stream);
int lemo_score_head_mean(const float* colsum_per_head, const float* diag_per_head, int64_t S, int32_t H,
                         uint32_t flags, float* scores, void* stream);

/*
 * Per-segment top-k (the token-block elimination step of Sec. 4.2 with the threshold replaced by a
 * keep count).  For each segment [n*L, min((n+1)*L, S)) keep the k tokens of highest score -- a
 * ragged last segment of length t keeps ceil(k*t/L), at least 1 -- breaking ties towards the LOWER
 * token index (-0.0 ties +0.0), and write the kept token indices in ascending order, segment after
 * segment, to kept_idx[0 .. lemo_kept_count(S,L,k)).  Scores must not be NaN (then the selection is
 * unspecified but still in range).  Bit-exact and deterministic.
 *
 * Supported: 1 <= k <= L <= 32768, S < 2^31.
 */
int lemo_select_topk(const float* scores, int64_t S, int32_t L, int32_t k, int32_t* kept_idx, void* stream);

/*
 * lemo_score_head_mean and lemo_select_topk in ONE launch (Sec. 4.2: head aggregation of Eq. 2, then the token-block
 * elimination): one workgroup per segment reads its [H, L] slab of the per-head column sums and diagonals, adds the
 * heads in ascending order, writes scores[S] and selects from the same values without a round trip through memory.
 * `scores` and `kept_idx` receive exactly the bits the two separate calls produce.  Arguments as for those calls.
 * Both steps are far below one kernel launch in size (4 MB read at S = 32768, 32 heads), so halving the launches
 * is what this buys.  Supported: 1 <= k <= L <= 32768.
 */
int lemo_head_mean_select_topk(const float* colsum_per_head, const float* diag_per_head, int64_t S, int32_t H,
                               uint32_t flags, int32_t L, int32_t k, float* scores, int32_t* kept_idx, void* stream);

/* Measurement aid: enqueues one empty kernel (one wavefront) on `stream` -- the launch floor that the
 * microsecond-sized steps (head mean, selection, threshold) are reported against. */
int lemo_launch_floor(void* stream);

/* Measurement aid: the instruction mix of the scoring sweeps (Sec. 4.2, Eq. 1) with everything else taken away.  Per
 * 32 x 32 logit tile at head_dim 128 a sweep must issue a chain of 8 dependent 32x32x16 bf16 MFMAs and, per logit, one
 * fma, one exp2 and one add in binary32; this enqueues a register-only kernel that issues exactly that, two wavefronts
 * per SIMD on every compute unit, `tiles_per_wave` tiles each (even, at most 2^24).  Timed by the caller, it gives the
 * rate at which the matrix cores and the vector ALU together get through this mix on the machine at hand:
 * 8 * 32768 flops * tiles_per_wave * *waves / seconds.  `operand_seed` 0: the same small-integer operand fragments for
 * every MFMA (next to nothing switches at the matrix cores' inputs: the rate at the chip's highest clock); non-zero:
 * pseudo-random unit-scale operands drawn from the seed that change from MFMA to MFMA, as a sweep's data does (the rate
 * at the clock the chip's power management grants on such data).  `sink`: one float of device memory (not written in
 * practice); `waves` (host, out): wavefronts launched. */
int lemo_probe_sweep_issue_mix(int32_t tiles_per_wave, uint32_t operand_seed, float* sink, int32_t* waves /* host, out */, void* stream);

/*
 * Block-wise informativeness (Sec. 4.2 "Block-wise Elimination", Eq. 2, and the token-block scores of
 * "Layer-specific Threshold"):
 *
 *     mean[i][j]        = (1/H) * sum over heads h with S^h_ij > 0 of S^h_ij
 *     score_blocks[m,n] = max of mean[i][j] over i in [m*b,(m+1)*b), j in [n*b,(n+1)*b)      I(B^S_mn)
 *     token_blocks[n]   = sum over m of score_blocks[m,n]                                     B^T_n
 *
 * mode LEMO_BLOCKS_PROBABILITIES:   S^h_ij is the softmax probability (the reading of Eq. 1 used by
 *                                   lemo_score_segments; the positivity condition is then vacuous);
 * mode LEMO_BLOCKS_POSITIVE_LOGITS: S^h_ij = scale * <Q_i, K_j>, pre-softmax, positive terms only.
 * Pairs the causal mask forbids (LEMO_CAUSAL: j > i) and, with LEMO_EXCLUDE_SELF, the pairs i == j take
 * no part in the maximum; a block without an admitted pair scores 0.  nb = ceil(S / b); a ragged last
 * block is shorter.
 *
 *   Q, K, strides, scale, flags: as for lemo_score_segments.
 *   b: score-block edge in tokens, a multiple of 32 (LEMO_ERR_UNSUPPORTED otherwise).
 *   lse2 [H,S] or NULL: the row statistics lemo_score_rowstats produced for the same Q, K, scale and
 *        flags.  NULL (probabilities mode) makes this call compute them first.  Ignored for logits.
 *   score_blocks [nb,nb] fp32, row m = query block, or NULL;  token_blocks [nb] fp32.
 *   workspace: at least lemo_score_blocks_workspace_bytes(S,H) bytes, 256-byte aligned, device memory.
 *
 * fp32 arithmetic; deterministic and repeatable.  Same tolerance against an fp64 evaluation as the
 * token-wise scores (2e-3 relative).
 */
enum { LEMO_BLOCKS_PROBABILITIES = 0, LEMO_BLOCKS_POSITIVE_LOGITS = 1 };
int lemo_score_blocks_workspace_bytes(int64_t S, int32_t H, size_t* bytes);
int lemo_score_blocks(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                      int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                      float scale, int32_t b, uint32_t flags, int32_t mode, const float* lse2, float* score_blocks,
                      float* token_blocks, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Selection by threshold (Sec. 4.2 "Layer-specific Threshold"): token block n is kept iff
 * token_blocks[n] >= T; the indices of all tokens of the kept blocks are written in ascending order to
 * kept_idx[0 .. count) and count to *kept_count (both device memory; kept_idx must have room for S
 * entries, entries past count are left as they were).  T is `threshold`, or, when threshold_dev is not
 * NULL, the float it points to in device memory (so that lemo_threshold_init can feed it without a
 * host round trip).  The number of kept rows is data dependent: read *kept_count back before sizing
 * the consumer call.  Supported: ceil(S / b) <= 16384.  Bit-exact and deterministic.
 *
 * lemo_threshold_init: step 1 of Alg. 1, the layer's initial threshold = the mean of its token-block
 * scores, written to *threshold (device memory).
 */
int lemo_threshold_init(const float* token_blocks, int64_t nb, float* threshold, void* stream);
int lemo_select_threshold(const float* token_blocks, int64_t S, int32_t b, float threshold, const float* threshold_dev,
                          int32_t* kept_idx, int32_t* kept_count, void* stream);

/*
 * Selective-load GEMM (Sec. 4.4, permutation-free token movement: the consumer reads the kept rows
 * from the original [S,C] input; no compacted copy of X is made):
 *
 *     Y[m, n] = sum_c X[kept_idx[m], c] * W[n, c]  (+ bias[n])        m < M, n < N
 *
 *   X [S, C] row stride ldx;  W [N, C] row stride ldw (torch.nn.Linear weight layout);
 *   bias [N] or NULL;  Y [M, N] row stride ldy;  all of dtype dt.
 *   kept_idx [M] int32 rows of X in [0,S) (not checked on the device), or NULL for rows 0..M-1
 *   (then M <= S).  M == 0 is a no-op.
 *
 * binary32 accumulation, one rounding at the store.  The result for output row m depends only on
 * the values of X row kept_idx[m], so running on a materialised compact copy gives identical bits.
 * Supported: C % 8 == 0 (bf16) / C % 4 == 0 (fp32).  X and W follow the 16-byte rule; Y only needs
 * element alignment and any ldy >= N (4-byte aligned bf16 rows are stored two columns at a time).
 */
int lemo_gather_gemm(const void* X, int64_t S, int64_t ldx, const int32_t* kept_idx, int64_t M,
                     const void* W, int64_t ldw, const void* bias, void* Y, int64_t ldy, int32_t C,
                     int32_t N, lemo_dtype_t dt, void* stream);

/*
 * Selective-load GEMM whose result is added in place into the residual stream (Sec. 4.4: the kept rows
 * are read from the original input AND the block's output is added to the original rows, which does
 * the zero padding and the residual addition in the GEMM's own store):
 *
 *     R[out_idx[m], n] += sum_c X[kept_idx[m], c] * W[n, c]  (+ bias[n])        m < M, n < N
 *
 *   X [S, C] row stride ldx, W [N, C] row stride ldw, bias [N] or NULL as for lemo_gather_gemm;
 *   R [S_out, N] row stride ldr, read and written; all of dtype dt.
 *   kept_idx [M] rows of X, or NULL for rows 0..M-1;  out_idx [M] rows of R, or NULL for rows 0..M-1.
 *   out_idx must name each row at most once (two result rows adding into one row of R would race;
 *   not checked); a value outside [0, S_out) drops that result row.  Rows of R that out_idx does not
 *   name are not touched.  X and R may not overlap.  M == 0 is a no-op.
 *
 * binary32 accumulation; bias and then the residual are added in binary32; ONE rounding at the store.
 * Same shape, stride and alignment rules as lemo_gather_gemm (R takes the place of Y); in addition R's
 * row pitch must be below 8 MiB and R must span less than 4 GiB (LEMO_ERR_UNSUPPORTED otherwise).
 */
int lemo_gather_gemm_add(const void* X, int64_t S, int64_t ldx, const int32_t* kept_idx, int64_t M,
                         const void* W, int64_t ldw, const void* bias, void* R, int64_t ldr, int64_t S_out,
                         const int32_t* out_idx, int32_t C, int32_t N, lemo_dtype_t dt, void* stream);

/*
 * Gradients of the selective-load GEMM Y = X[kept_idx] W^T (the backward of Sec. 4.4's selective load), permutation-free
 * on this pass as well: neither a transposed copy of the weight nor transposed copies of dY and of the kept rows are made.
 *
 *   lemo_gather_gemm_dx   dX[out_idx[m], c] += sum_n dY[m, n] * W[n, c]         m < M, c < C      (input gradient)
 *   lemo_gather_gemm_dw   dW[n, c]           = sum over m < M of dY[m, n] * X[kept_idx[m], c]    (weight gradient)
 *
 *   dY [M, N] row stride ldy (compact rows, one per kept token);  W [N, C] row stride ldw, as lemo_gather_gemm takes it;
 *   dX [S_out, C] row stride lddx, read and written (rows that out_idx does not name are not touched; out_idx NULL means
 *   rows 0..M-1; each row at most once, values outside [0, S_out) drop the row);  X [S, C] row stride ldx;  dW [N, C] row
 *   stride lddw (overwritten; M == 0 writes zeros);  kept_idx [M] rows of X in [0,S) (not checked on the device) or NULL
 *   for rows 0..M-1.  All of dtype dt.
 *
 * Both products contract over an axis along which the stored operand is NOT contiguous (W over n, dY and X over the
 * tokens).  For bf16 the kernels stage the operand tiles as they lie in memory and take their matrix-core fragments with
 * the transposing LDS read of gfx950; the kept rows of X are picked inside the tile load.  binary32 accumulation, one
 * rounding at the store (for dX after the old value has been added).
 *
 * Supported: lemo_gather_gemm_dx: LEMO_BF16 only (fp32: lemo_gather_gemm_add with W^T stored as [C, N]); C % 8 == 0 and
 * N % 8 == 0; dY, W follow the 16-byte rule; row pitches below 8 MiB; dY and dX spanning less than 4 GiB, W less than
 * 2 GiB.  lemo_gather_gemm_dw: C % 8 == 0 and N % 8 == 0 (bf16) / % 4 (fp32); bf16 needs no workspace
 * (lemo_gather_gemm_dw_workspace_bytes reports 0, `workspace` may be NULL) with dY spanning less than 2 GiB and X less than
 * 4 GiB; fp32 goes through transposed copies of both operands in the workspace (256-byte aligned device memory of the
 * reported size; M below 2M tokens and N * M * 4 below 4 GiB).
 */
int lemo_gather_gemm_dx(const void* dY, int64_t ldy, int64_t M, const void* W, int64_t ldw, void* dX, int64_t lddx,
                        int64_t S_out, const int32_t* out_idx, int32_t C, int32_t N, lemo_dtype_t dt, void* stream);
int lemo_gather_gemm_dw_workspace_bytes(int64_t M, int32_t C, int32_t N, lemo_dtype_t dt, size_t* bytes);
int lemo_gather_gemm_dw(const void* dY, int64_t ldy, const void* X, int64_t S, int64_t ldx, const int32_t* kept_idx, int64_t M,
                        void* dW, int64_t lddw, int32_t C, int32_t N, lemo_dtype_t dt, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * Attention over the kept tokens, read in place (Sec. 4.4: the attention block loads the selected tokens
 * straight from the original inputs instead of from a re-permuted copy):
 *
 *     O[m, h, :] = sum_n softmax_n( scale * <Q[kept_idx[m],h,:], K[kept_idx[n],g,:]> ) * V[kept_idx[n],g,:]
 *
 * with g = floor(h * H_kv / H) and n over all M kept tokens, or with LEMO_CAUSAL over n <= m (kept_idx
 * must then be ascending, as lemo_select_topk / lemo_select_threshold write it, so that list order is
 * position order).  LEMO_EXCLUDE_SELF is not accepted here.
 *
 *   Q [S,H,d], K and V [S,H_kv,d], element strides as for lemo_score_segments (d contiguous, 16-byte rule);
 *   kept_idx [M] int32 token positions in [0,S) (not checked on the device), or NULL for the first M tokens;
 *   O [M,H,d] compact result with element strides o_tok_stride, o_head_stride (multiples of 8, d contiguous):
 *     row m belongs to token kept_idx[m]; lemo_gather_gemm_add with out_idx = kept_idx puts the block's
 *     projection back into the residual stream;
 *   workspace: lemo_kept_attention_workspace_bytes(M,H_kv,d) bytes, 256-byte aligned (holds the kept rows
 *     of V transposed, 2 bytes per kept element).
 *
 * Supported: LEMO_BF16, d in {64,128}; Q and K each spanning less than 4 GiB.  The probabilities are
 * rounded to bf16 for the second product and the normaliser is summed in binary32 from the unrounded
 * values; one rounding of the result at the store.  M == 0 is a no-op.  Deterministic.
 */
int lemo_kept_attention_workspace_bytes(int64_t M, int32_t H_kv, int32_t d, size_t* bytes);
int lemo_kept_attention(const void* Q, const void* K, const void* V, int64_t S, int32_t H, int32_t H_kv, int32_t d,
                        lemo_dtype_t dt, int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride,
                        int64_t k_head_stride, int64_t v_tok_stride, int64_t v_head_stride, const int32_t* kept_idx,
                        int64_t M, float scale, uint32_t flags, void* O, int64_t o_tok_stride, int64_t o_head_stride,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * In-place add at the kept positions (Sec. 4.4: zero padding and the residual add collapse into one
 * read-modify-write of the kept rows); also the backward of the selective load:
 *
 *     ACCUMULATE:  dX[kept_idx[m], c] = round( float(dX[kept_idx[m], c]) + float(G[m, c]) )
 *     ZERO_PAD:    dX[kept_idx[m], c] = round( float(G[m, c]) ),  every other row of dX = +0
 *
 *   G [M, C] row stride ldg, dtype g_dt;  dX [S, C] row stride lddx, dtype dx_dt.
 *   kept_idx [M] int32, in [0,S) and UNIQUE (not checked on the device); ZERO_PAD additionally
 *   requires it strictly ascending (what lemo_select_topk produces).  M == 0: ACCUMULATE is a
 *   no-op, ZERO_PAD clears dX.
 *
 * One binary32 add and one rounding per element: bit-exact and order-independent.
 * Supported: C % 8 == 0.
 */
int lemo_scatter_grad(const void* G, int64_t ldg, const int32_t* kept_idx, int64_t M, void* dX,
                      int64_t lddx, int64_t S, int32_t C, lemo_dtype_t g_dt, lemo_dtype_t dx_dt,
                      int32_t mode, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LEMO_H */
