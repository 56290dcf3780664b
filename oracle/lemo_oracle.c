/*
 * CPU oracle for the Contextual Token Sparsity hot path (LeMo, arXiv 2501.09767).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64 statement of what the
 * four operations compute, written from the paper's definitions so that a reader can check it
 * against the paper by eye.  It shares no source, header, table or helper with the HIP library and
 * must only be called from tests, the smoke check and the bench's cpu_baseline leg.
 *
 *   oracle_score            Sec. 4.2 Eq. 1 (token informativeness = column sum of attention scores,
 *                           self excluded) with the head mean of Eq. 2; attention scores are the
 *                           softmax probabilities (Sec. 4.2 states that the scores pass through a softmax).
 *   oracle_score_bruteforce same quantity through a materialised S x S matrix (tiny S only).
 *   oracle_score_blocks     Sec. 4.2 Eq. 2 (maximum of the head-aggregated score over a b x b score block)
 *                           and the token-block sums B^T_n of "Layer-specific Threshold".
 *   oracle_select_threshold keep the token blocks whose score reaches a threshold (Sec. 4.2);
 *   oracle_threshold_init   Alg. 1 step 1, the average token-block score.
 *   oracle_select_topk      per-segment top-k at a keep ratio (the selection unit is the paper's
 *                           token block, Sec. 4.2 "Layer-specific Threshold"; here the k best of
 *                           each block are kept instead of thresholding).
 *   oracle_gather_gemm      Sec. 4.4 selective load (kept rows are read from the original input):
 *                           Y[m,:] = X[idx[m],:] . W^T (+ bias).
 *   oracle_gather_gemm_add  Sec. 4.4, both halves fused: selective load on the way in, in-place add
 *                           into the residual rows on the way out.
 *   oracle_gather_gemm_dw   weight gradient of the selective-load GEMM (the gather on the contraction axis).
 *   oracle_kept_attention   Sec. 4.4: the attention block computed over the kept tokens, read in place.
 *   oracle_scatter_add      Sec. 4.4 in-place add (padding and residual add in one step):
 *                           dX[idx[m],:] += G[m,:].
 *
 * Every floating-point reduction is carried in double.  Nothing here is blocked, fused or
 * reordered beyond what the definitions state.  Parallelism (OpenMP) is over independent query rows
 * (scoring) or independent output rows (GEMM) only.
 *
 * Pins (tests/test_oracle_pins.py): softmax rows sum to one => per-head column sums total S;
 * brute-force S x S agreement; closed forms for constant logits (harmonic numbers under a causal
 * mask); shift/permutation invariances; numpy textbook softmax; argsort top-k; numpy float64
 * matmul; adjoint identity between gather and scatter.  The paper prints no worked numeric example
 * for this path, so parity against paper-printed values is unpinned; the pins above are what fixes
 * the oracle.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_CAUSAL = 1u, ORACLE_EXCLUDE_SELF = 2u };
enum { ORACLE_SCATTER_ACCUMULATE = 0, ORACLE_SCATTER_ZERO_PAD = 1 };
enum { ORACLE_OK = 0, ORACLE_ERR_ARG = -1, ORACLE_ERR_NOMEM = -2 };

/* ---------------------------------------------------------------- element access */

static float bf16_bits_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16; /* bf16 is the upper half of an IEEE binary32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static double load_elem(const void* base, int64_t index, int dtype) {
    if (dtype == ORACLE_BF16) return (double)bf16_bits_to_float(((const uint16_t*)base)[index]);
    return (double)((const float*)base)[index];
}

/* Round a double to the nearest bfloat16 (ties to even) in ONE rounding step and return its bit
 * pattern.  bf16: 1 sign, 8 exponent, 7 stored fraction bits; smallest normal 2^-126, so the
 * spacing of representable values never drops below 2^-133. */
static uint16_t double_to_bf16_bits(double x) {
    if (isnan(x)) return 0x7fc0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7f80;
    int e;
    (void)frexp(a, &e);              /* a = m * 2^e, m in [0.5, 1) */
    int q = e - 8;                   /* spacing 2^q keeps 8 significant bits */
    if (q < -133) q = -133;          /* subnormal range: fixed spacing */
    double r = nearbyint(ldexp(a, -q)); /* default rounding mode = ties to even; exact scaling */
    double v = ldexp(r, q);          /* representable in bf16 unless it overflowed */
    if (v > 3.3895313892515355e38) return sign | 0x7f80; /* beyond (2 - 2^-7) * 2^127: infinity */
    float f = (float)v;              /* exact: v has <= 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return sign | (uint16_t)(u >> 16);
}

static uint16_t float_to_bf16_bits(float x) { return double_to_bf16_bits((double)x); }

/* ---------------------------------------------------------------- host helpers */

/* k = ceil(ratio * L) kept tokens per full segment, clamped to [1, L].  A 1e-9 slack keeps exact
 * products such as 0.5 * 128 from rounding up. */
int32_t oracle_keep_k(int32_t L, double ratio) {
    if (L <= 0) return 0;
    double v = ceil(ratio * (double)L - 1e-9);
    if (v < 1.0) v = 1.0;
    if (v > (double)L) v = (double)L;
    return (int32_t)v;
}

/* tokens kept in a segment of length len when full segments of length L keep k */
static int32_t seg_keep(int64_t len, int32_t L, int32_t k) {
    if (len == (int64_t)L) return k;
    int64_t v = ((int64_t)k * len + (int64_t)L - 1) / (int64_t)L; /* ceil(k * len / L) */
    if (v < 1) v = 1;
    if (v > len) v = len;
    return (int32_t)v;
}

int64_t oracle_kept_count(int64_t S, int32_t L, int32_t k) {
    if (S <= 0 || L <= 0 || k <= 0 || k > L) return -1;
    int64_t full = S / L, tail = S % L;
    int64_t M = full * k;
    if (tail) M += seg_keep(tail, L, k);
    return M;
}

/* ---------------------------------------------------------------- scoring */

/* Widen one head's rows ([S, d] with a token stride) exactly to double. */
static double* widen_head(const void* base, int64_t S, int d, int dtype, int64_t tok_stride, int64_t head_off) {
    double* out = (double*)malloc(sizeof(double) * (size_t)S * (size_t)d);
    if (!out) return NULL;
    for (int64_t i = 0; i < S; ++i)
        for (int c = 0; c < d; ++c) out[i * d + c] = load_elem(base, i * tok_stride + head_off + c, dtype);
    return out;
}

/* One query row of one head.  Logits s_ij = scale * <Q_i, K_j> over the allowed keys (j <= i under
 * a causal mask, all j otherwise); p_ij = softmax over j; p_ij is added to column j and p_ii is
 * remembered.  `row` is an O(S) buffer; the S x S matrix never exists. */
static void score_one_row(const double* Qh, const double* Kh, int64_t S, int d, double scale, int causal,
                          int64_t i, double* row, double* col, double* dg) {
    int64_t nk = causal ? i + 1 : S;
    double mx = -INFINITY;
    for (int64_t j = 0; j < nk; ++j) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += Qh[i * d + c] * Kh[j * d + c];
        row[j] = scale * dot;
        if (row[j] > mx) mx = row[j];
    }
    double den = 0.0;
    for (int64_t j = 0; j < nk; ++j) { row[j] = exp(row[j] - mx); den += row[j]; }
    for (int64_t j = 0; j < nk; ++j) {
        double p = row[j] / den;
        col[j] += p;
        if (j == i) dg[j] = p;
    }
}

/* Q [S,H,d], K [S,H_kv,d] with element strides (d contiguous); query head h reads KV head
 * floor(h * H_kv / H).  scores[S] (float) is the head mean of (column sum - [EXCLUDE_SELF] p_jj),
 * rounded once from double.  colsum / diag, when not NULL, receive the per-head [H,S] doubles;
 * colsum always INCLUDES the diagonal term.
 *
 * Query rows are independent, so they are dealt out to OpenMP threads round-robin; each
 * thread adds into its own column array and the arrays are summed in thread order afterwards. */
int oracle_score(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype,
                 int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                 double scale, uint32_t flags, float* scores, double* colsum, double* diag) {
    if (!Q || !K || !scores || S <= 0 || H <= 0 || H_kv <= 0 || d <= 0 || H % H_kv) return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_ERR_ARG;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)d);
    const int causal = (flags & ORACLE_CAUSAL) != 0;
    const int excl = (flags & ORACLE_EXCLUDE_SELF) != 0;
    const int nthr = omp_get_max_threads();
    double* col = (double*)calloc((size_t)H * (size_t)S, sizeof(double));
    double* dg = (double*)calloc((size_t)H * (size_t)S, sizeof(double));
    double* part = (double*)malloc(sizeof(double) * (size_t)nthr * (size_t)S);  /* per-thread column sums */
    double* rows = (double*)malloc(sizeof(double) * (size_t)nthr * (size_t)S);  /* per-thread row buffers */
    if (!col || !dg || !part || !rows) { free(col); free(dg); free(part); free(rows); return ORACLE_ERR_NOMEM; }
    for (int h = 0; h < H; ++h) {
        int g = (int)(((int64_t)h * H_kv) / H);
        double* Qh = widen_head(Q, S, d, dtype, q_tok_stride, (int64_t)h * q_head_stride);
        double* Kh = widen_head(K, S, d, dtype, k_tok_stride, (int64_t)g * k_head_stride);
        if (!Qh || !Kh) { free(Qh); free(Kh); free(col); free(dg); free(part); free(rows); return ORACLE_ERR_NOMEM; }
        memset(part, 0, sizeof(double) * (size_t)nthr * (size_t)S);
#pragma omp parallel num_threads(nthr)
        {
            int t = omp_get_thread_num();
            /* interleaved rows: under a causal mask row i costs i+1 keys, so contiguous ranges would be lopsided */
            for (int64_t i = t; i < S; i += nthr)
                score_one_row(Qh, Kh, S, d, scale, causal, i, rows + (size_t)t * S, part + (size_t)t * S, dg + (size_t)h * S);
        }
        for (int t = 0; t < nthr; ++t)
            for (int64_t j = 0; j < S; ++j) col[(size_t)h * S + j] += part[(size_t)t * S + j];
        free(Qh);
        free(Kh);
    }
    free(part);
    free(rows);
    for (int64_t j = 0; j < S; ++j) {
        double acc = 0.0;
        for (int h = 0; h < H; ++h) {
            double v = col[(size_t)h * S + j];
            if (excl) v -= dg[(size_t)h * S + j];
            acc += v;
        }
        scores[j] = (float)(acc / (double)H);
    }
    if (colsum) memcpy(colsum, col, sizeof(double) * (size_t)H * (size_t)S);
    if (diag) memcpy(diag, dg, sizeof(double) * (size_t)H * (size_t)S);
    free(col);
    free(dg);
    return ORACLE_OK;
}

/* Block-wise informativeness (Sec. 4.2 "Block-wise Elimination", Eq. 2, and the token-block sum of
 * "Layer-specific Threshold"):
 *   mean[i][j]   = (1/H) * sum over heads h with S^h_ij > 0 of S^h_ij        (head aggregation, positive terms only)
 *   I(B^S_mn)    = max of mean[i][j] over the b x b score block  i in [m*b,(m+1)*b), j in [n*b,(n+1)*b)
 *   B^T_n        = sum over m of I(B^S_mn)                                    (token-block score)
 * S^h_ij is the softmax probability of Eq. 1's reading (mode 0: always positive, so the condition is
 * vacuous) or the scaled pre-softmax logit scale * <Q_i, K_j> (mode 1: the literal "only positive
 * scores" rule).  Pairs a causal mask forbids (j > i), and the pair i == j when EXCLUDE_SELF is set,
 * take no part in the maximum; a block with no admissible pair scores 0.  Ragged last blocks are
 * simply shorter.  score_blocks ([nb,nb] doubles, row m, column n; may be NULL) and token_blocks
 * ([nb] floats, one rounding from double), nb = ceil(S / b). */
/* One query i of the block-wise score: the head aggregate mean[j] over the allowed keys, folded into the
 * running maxima best[j / b] of the query's block row.  Qh[h] / Kh[g] are the heads widened to double; Qh
 * rows are indexed from q_first (a caller may have widened only the rows it needs).  `mean` and `row` are
 * O(S) buffers. */
static void score_block_query(double* const* Qh, int64_t q_first, double* const* Kh, int64_t S, int32_t H, int32_t H_kv,
                              int32_t d, double scale, int causal, int excl, int32_t b, int mode, int64_t i, double* mean,
                              double* row, double* best) {
    int64_t nk = causal ? i + 1 : S;
    for (int64_t j = 0; j < nk; ++j) mean[j] = 0.0;
    for (int h = 0; h < H; ++h) {
        const double* q = Qh[h] + (i - q_first) * d;
        const double* kk = Kh[(int)(((int64_t)h * H_kv) / H)];
        double mx = -INFINITY;
        for (int64_t j = 0; j < nk; ++j) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += q[c] * kk[j * d + c];
            row[j] = scale * dot;
            if (row[j] > mx) mx = row[j];
        }
        if (mode == 0) { /* softmax probabilities */
            double den = 0.0;
            for (int64_t j = 0; j < nk; ++j) { row[j] = exp(row[j] - mx); den += row[j]; }
            for (int64_t j = 0; j < nk; ++j) row[j] /= den;
        }
        for (int64_t j = 0; j < nk; ++j)
            if (row[j] > 0.0) mean[j] += row[j]; /* only positive scores are aggregated */
    }
    for (int64_t j = 0; j < nk; ++j) {
        if (excl && j == i) continue;
        double v = mean[j] / (double)H;
        if (v > best[j / b]) best[j / b] = v;
    }
}

int oracle_score_blocks(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype,
                        int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                        double scale, uint32_t flags, int32_t b, int mode, double* score_blocks, float* token_blocks) {
    if (!Q || !K || !token_blocks || S <= 0 || H <= 0 || H_kv <= 0 || d <= 0 || H % H_kv || b <= 0) return ORACLE_ERR_ARG;
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || (mode != 0 && mode != 1)) return ORACLE_ERR_ARG;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)d);
    const int causal = (flags & ORACLE_CAUSAL) != 0;
    const int excl = (flags & ORACLE_EXCLUDE_SELF) != 0;
    const int64_t nb = (S + b - 1) / b;
    const int nthr = omp_get_max_threads();
    double** Qh = (double**)calloc((size_t)H, sizeof(double*));
    double** Kh = (double**)calloc((size_t)H_kv, sizeof(double*));
    double* best = (double*)calloc((size_t)nb * (size_t)nb, sizeof(double));
    double* work = (double*)malloc(sizeof(double) * 2 * (size_t)nthr * (size_t)S);
    int ok = Qh && Kh && best && work;
    for (int h = 0; ok && h < H; ++h) ok = (Qh[h] = widen_head(Q, S, d, dtype, q_tok_stride, (int64_t)h * q_head_stride)) != NULL;
    for (int g = 0; ok && g < H_kv; ++g) ok = (Kh[g] = widen_head(K, S, d, dtype, k_tok_stride, (int64_t)g * k_head_stride)) != NULL;
    if (ok) {
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthr)
        for (int64_t m = nb - 1; m >= 0; --m) { /* block rows are independent; late rows are the long ones */
            double* mean = work + 2 * (size_t)omp_get_thread_num() * (size_t)S;
            int64_t i_end = (m + 1) * b < S ? (m + 1) * b : S;
            for (int64_t i = m * b; i < i_end; ++i)
                score_block_query(Qh, 0, Kh, S, H, H_kv, d, scale, causal, excl, b, mode, i, mean, mean + S, best + m * nb);
        }
        for (int64_t n = 0; n < nb; ++n) {
            double acc = 0.0;
            for (int64_t m = 0; m < nb; ++m) acc += best[m * nb + n];
            token_blocks[n] = (float)acc;
        }
        if (score_blocks) memcpy(score_blocks, best, sizeof(double) * (size_t)nb * (size_t)nb);
    }
    for (int h = 0; Qh && h < H; ++h) free(Qh[h]);
    for (int g = 0; Kh && g < H_kv; ++g) free(Kh[g]);
    free(Qh); free(Kh); free(best); free(work);
    return ok ? ORACLE_OK : ORACLE_ERR_NOMEM;
}

/* The score blocks I(B^S_mn), n < nb, of the listed block rows only (row_out is [n_rows, nb]): the same
 * arithmetic as oracle_score_blocks, for quick spot checks (the whole 32K-token, 32-head matrix takes the full routine
 * about a minute on 16 threads). */
int oracle_score_block_rows(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype,
                            int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                            double scale, uint32_t flags, int32_t b, int mode, const int64_t* rows, int32_t n_rows, double* row_out) {
    if (!Q || !K || !rows || !row_out || S <= 0 || H <= 0 || H_kv <= 0 || d <= 0 || H % H_kv || b <= 0 || n_rows < 0) return ORACLE_ERR_ARG;
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || (mode != 0 && mode != 1)) return ORACLE_ERR_ARG;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)d);
    const int64_t nb = (S + b - 1) / b;
    for (int32_t t = 0; t < n_rows; ++t)
        if (rows[t] < 0 || rows[t] >= nb) return ORACLE_ERR_ARG;
    double** Qh = (double**)calloc((size_t)H, sizeof(double*));
    double** Kh = (double**)calloc((size_t)H_kv, sizeof(double*));
    int ok = Qh && Kh;
    for (int g = 0; ok && g < H_kv; ++g) ok = (Kh[g] = widen_head(K, S, d, dtype, k_tok_stride, (int64_t)g * k_head_stride)) != NULL;
    memset(row_out, 0, sizeof(double) * (size_t)n_rows * (size_t)nb);
    for (int32_t t = 0; ok && t < n_rows; ++t) {
        const int64_t m = rows[t], first = m * b, len = ((m + 1) * b < S ? (m + 1) * b : S) - first;
        for (int h = 0; ok && h < H; ++h) /* only this block row's queries are widened */
            ok = (Qh[h] = widen_head(Q, len, d, dtype, q_tok_stride, first * q_tok_stride + (int64_t)h * q_head_stride)) != NULL;
        if (ok) {
            /* the queries of the row are independent: each thread keeps its own maxima, merged afterwards */
            const int nthr = omp_get_max_threads();
            const size_t per = (size_t)(2 * S + nb);
            double* work = (double*)calloc((size_t)nthr * per, sizeof(double));
            if (!work) ok = 0;
            if (ok) {
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthr)
                for (int64_t i = first; i < first + len; ++i) {
                    double* mine = work + (size_t)omp_get_thread_num() * per;
                    score_block_query(Qh, first, Kh, S, H, H_kv, d, scale, (flags & ORACLE_CAUSAL) != 0,
                                      (flags & ORACLE_EXCLUDE_SELF) != 0, b, mode, i, mine + nb, mine + nb + S, mine);
                }
                for (int th = 0; th < nthr; ++th)
                    for (int64_t n = 0; n < nb; ++n) {
                        double v = work[(size_t)th * per + n];
                        if (v > row_out[(size_t)t * nb + n]) row_out[(size_t)t * nb + n] = v;
                    }
            }
            free(work);
        }
        for (int h = 0; h < H; ++h) { free(Qh[h]); Qh[h] = NULL; }
    }
    for (int g = 0; Kh && g < H_kv; ++g) free(Kh[g]);
    free(Qh); free(Kh);
    return ok ? ORACLE_OK : ORACLE_ERR_NOMEM;
}

/* Selection by threshold (Sec. 4.2 "Layer-specific Threshold"): a token block is kept iff its score
 * B^T_n >= T; the tokens of kept blocks are listed in ascending order.  Returns the number of kept
 * tokens (kept_idx must have room for S), or a negative error. */
int64_t oracle_select_threshold(const float* token_blocks, int64_t S, int32_t b, double T, int32_t* kept_idx) {
    if (!token_blocks || !kept_idx || S <= 0 || b <= 0) return ORACLE_ERR_ARG;
    int64_t nb = (S + b - 1) / b, out = 0;
    for (int64_t n = 0; n < nb; ++n) {
        if (!((double)token_blocks[n] >= T)) continue;
        int64_t end = (n + 1) * b < S ? (n + 1) * b : S;
        for (int64_t j = n * b; j < end; ++j) kept_idx[out++] = (int32_t)j;
    }
    return out;
}

/* Step 1 of Alg. 1: the initial layer threshold is the average score of the layer's token blocks
 * (sum in double, in index order). */
double oracle_threshold_init(const float* token_blocks, int64_t nb) {
    if (!token_blocks || nb <= 0) return NAN;
    double acc = 0.0;
    for (int64_t n = 0; n < nb; ++n) acc += (double)token_blocks[n];
    return acc / (double)nb;
}

/* The same scores through the full S x S probability matrix of each head: all logits first, then a
 * softmax over every row, then a sum down every column with the i == j entry left out when
 * EXCLUDE_SELF is set.  Memory is quadratic, so S is limited. */
int oracle_score_bruteforce(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d,
                            int dtype, int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride,
                            int64_t k_head_stride, double scale, uint32_t flags, float* scores) {
    if (!Q || !K || !scores || S <= 0 || S > 2048 || H <= 0 || H_kv <= 0 || d <= 0 || H % H_kv) return ORACLE_ERR_ARG;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)d);
    const int causal = (flags & ORACLE_CAUSAL) != 0;
    const int excl = (flags & ORACLE_EXCLUDE_SELF) != 0;
    double* P = (double*)malloc(sizeof(double) * (size_t)S * (size_t)S);
    double* total = (double*)calloc((size_t)S, sizeof(double));
    if (!P || !total) { free(P); free(total); return ORACLE_ERR_NOMEM; }
    for (int h = 0; h < H; ++h) {
        int g = (int)(((int64_t)h * H_kv) / H);
        for (int64_t i = 0; i < S; ++i)
            for (int64_t j = 0; j < S; ++j) {
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += load_elem(Q, i * q_tok_stride + h * q_head_stride + c, dtype) *
                           load_elem(K, j * k_tok_stride + g * k_head_stride + c, dtype);
                P[i * S + j] = (causal && j > i) ? -INFINITY : scale * dot;
            }
        for (int64_t i = 0; i < S; ++i) {
            double mx = -INFINITY, den = 0.0;
            for (int64_t j = 0; j < S; ++j) if (P[i * S + j] > mx) mx = P[i * S + j];
            for (int64_t j = 0; j < S; ++j) { P[i * S + j] = exp(P[i * S + j] - mx); den += P[i * S + j]; }
            for (int64_t j = 0; j < S; ++j) P[i * S + j] /= den;
        }
        for (int64_t j = 0; j < S; ++j) {
            double c = 0.0;
            for (int64_t i = 0; i < S; ++i)
                if (!(excl && i == j)) c += P[i * S + j];
            total[j] += c;
        }
    }
    for (int64_t j = 0; j < S; ++j) scores[j] = (float)(total[j] / (double)H);
    free(P);
    free(total);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------- selection */

typedef struct { float score; int32_t index; } scored_t;

/* higher score first; equal scores (including -0.0 vs +0.0) keep the lower index first */
static int by_score_desc_then_index(const void* a, const void* b) {
    const scored_t* x = (const scored_t*)a;
    const scored_t* y = (const scored_t*)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->index > y->index) - (x->index < y->index);
}

static int by_int32(const void* a, const void* b) {
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

/* For every segment [n L, min((n+1) L, S)): order its tokens by score (descending, ties to the
 * lower index), keep the first k (a ragged last segment keeps ceil(k * len / L), at least one),
 * and append the kept token indices in ascending order. */
int oracle_select_topk(const float* scores, int64_t S, int32_t L, int32_t k, int32_t* kept_idx) {
    if (!scores || !kept_idx || S <= 0 || L <= 0 || k <= 0 || k > L) return ORACLE_ERR_ARG;
    scored_t* seg = (scored_t*)malloc(sizeof(scored_t) * (size_t)L);
    if (!seg) return ORACLE_ERR_NOMEM;
    int64_t out = 0;
    for (int64_t start = 0; start < S; start += L) {
        int64_t len = (S - start < L) ? S - start : L;
        int32_t keep = seg_keep(len, L, k);
        for (int64_t t = 0; t < len; ++t) { seg[t].score = scores[start + t]; seg[t].index = (int32_t)(start + t); }
        qsort(seg, (size_t)len, sizeof(scored_t), by_score_desc_then_index);
        for (int32_t t = 0; t < keep; ++t) kept_idx[out + t] = seg[t].index;
        qsort(kept_idx + out, (size_t)keep, sizeof(int32_t), by_int32);
        out += keep;
    }
    free(seg);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------- gather-GEMM */

/* Y[m,n] = round( sum_c X[idx[m],c] * W[n,c] + bias[n] ), sum in double, ONE rounding to the
 * output type (same type as the inputs).  idx == NULL means rows 0..M-1.  X is [S,C] with row
 * stride ldx, W is [N,C] with row stride ldw, Y is [M,N] with row stride ldy (all in elements). */
int oracle_gather_gemm(const void* X, int64_t S, int64_t ldx, const int32_t* idx, int64_t M,
                       const void* W, int64_t ldw, const void* bias, void* Y, int64_t ldy,
                       int32_t C, int32_t N, int dtype) {
    if (!X || !W || !Y || S <= 0 || M < 0 || C <= 0 || N <= 0 || ldx < C || ldw < C || ldy < N) return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_ERR_ARG;
    for (int64_t m = 0; m < M; ++m) {
        int64_t r = idx ? idx[m] : m;
        if (r < 0 || r >= S) return ORACLE_ERR_ARG;
    }
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        int64_t r = idx ? idx[m] : m;
        for (int32_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int32_t c = 0; c < C; ++c)
                acc += load_elem(X, r * ldx + c, dtype) * load_elem(W, (int64_t)n * ldw + c, dtype);
            if (bias) acc += load_elem(bias, n, dtype);
            if (dtype == ORACLE_BF16) ((uint16_t*)Y)[m * ldy + n] = double_to_bf16_bits(acc);
            else ((float*)Y)[m * ldy + n] = (float)acc;
        }
    }
    return ORACLE_OK;
}

/* Fused form of Sec. 4.4's token movement: the GEMM reads its rows through in_idx (selective load) and
 * its result is added in place into the rows out_idx of the residual stream R, which completes the
 * zero padding and the residual addition in one step:
 *   R[out_idx[m],n] = round( R[out_idx[m],n] + sum_c X[in_idx[m],c] * W[n,c] + bias[n] ),
 * everything in double, ONE rounding to the element type.  Rows of R that out_idx does not name stay
 * untouched.  in_idx == NULL reads rows 0..M-1 of X; out_idx == NULL writes rows 0..M-1 of R.
 * out_idx must be unique and within [0,S_out). */
int oracle_gather_gemm_add(const void* X, int64_t S, int64_t ldx, const int32_t* in_idx, int64_t M,
                           const void* W, int64_t ldw, const void* bias, void* R, int64_t ldr, int64_t S_out,
                           const int32_t* out_idx, int32_t C, int32_t N, int dtype) {
    if (!X || !W || !R || S <= 0 || S_out <= 0 || M < 0 || C <= 0 || N <= 0 || ldx < C || ldw < C || ldr < N) return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_ERR_ARG;
    if (!out_idx && M > S_out) return ORACLE_ERR_ARG;
    unsigned char* seen = (unsigned char*)calloc((size_t)S_out, 1);
    if (!seen) return ORACLE_ERR_NOMEM;
    for (int64_t m = 0; m < M; ++m) {
        int64_t r = in_idx ? in_idx[m] : m, o = out_idx ? out_idx[m] : m;
        if (r < 0 || r >= S || o < 0 || o >= S_out || seen[o]) { free(seen); return ORACLE_ERR_ARG; }
        seen[o] = 1;
    }
    free(seen);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        int64_t r = in_idx ? in_idx[m] : m, o = out_idx ? out_idx[m] : m;
        for (int32_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int32_t c = 0; c < C; ++c)
                acc += load_elem(X, r * ldx + c, dtype) * load_elem(W, (int64_t)n * ldw + c, dtype);
            if (bias) acc += load_elem(bias, n, dtype);
            acc += load_elem(R, o * ldr + n, dtype);
            if (dtype == ORACLE_BF16) ((uint16_t*)R)[o * ldr + n] = double_to_bf16_bits(acc);
            else ((float*)R)[o * ldr + n] = (float)acc;
        }
    }
    return ORACLE_OK;
}

/* Weight gradient of the selective-load GEMM Y = X[idx] W^T:  dW[n,c] = round( sum_m dY[m,n] * X[idx[m],c] ),
 * the contraction running over the kept tokens (the gather sits on the contraction axis), sum in double, ONE rounding.
 * dY [M,N] row stride ldy, X [S,C] row stride ldx, dW [N,C] row stride lddw; idx == NULL means rows 0..M-1. */
int oracle_gather_gemm_dw(const void* dY, int64_t ldy, const void* X, int64_t S, int64_t ldx, const int32_t* idx, int64_t M,
                          void* dW, int64_t lddw, int32_t C, int32_t N, int dtype) {
    if (!dY || !X || !dW || S <= 0 || M < 0 || C <= 0 || N <= 0 || ldy < N || ldx < C || lddw < C) return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_ERR_ARG;
    if (!idx && M > S) return ORACLE_ERR_ARG;
    for (int64_t m = 0; m < M; ++m) {
        int64_t r = idx ? idx[m] : m;
        if (r < 0 || r >= S) return ORACLE_ERR_ARG;
    }
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n)
        for (int32_t c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int64_t m = 0; m < M; ++m) {
                int64_t r = idx ? idx[m] : m;
                acc += load_elem(dY, m * ldy + n, dtype) * load_elem(X, r * ldx + c, dtype);
            }
            if (dtype == ORACLE_BF16) ((uint16_t*)dW)[(int64_t)n * lddw + c] = double_to_bf16_bits(acc);
            else ((float*)dW)[(int64_t)n * lddw + c] = (float)acc;
        }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------- attention over the kept tokens */

/* The attention block on the kept tokens only (Sec. 4.4: the block reads the selected tokens straight
 * from the original inputs; what it returns is the compact result that the in-place add then puts back):
 *   O[m,h,:] = sum_n softmax_n( scale * <Q[idx[m],h,:], K[idx[n],g,:]> ) * V[idx[n],g,:],   g = floor(h*H_kv/H),
 * n running over the kept tokens the mask allows: all of them, or with CAUSAL those whose position idx[n]
 * is not after idx[m].  Everything in double, ONE rounding to the element type.  Q [S,H,d], K and V
 * [S,H_kv,d] with element strides (d contiguous); O [M,H,d] with strides o_tok, o_head.  idx == NULL
 * means the first M tokens. */
/* one kept query m, all heads -> out_row[H*d] (o_head_stride apart); w [M] and acc [d] are scratch */
static void attention_one_query(const void* Q, const void* K, const void* V, int32_t H, int32_t H_kv, int32_t d, int dtype,
                                int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                                int64_t v_tok_stride, int64_t v_head_stride, const int32_t* idx, int64_t M, double scale, int causal,
                                int64_t m, void* O, int64_t o_base, int64_t o_head_stride, double* w, double* acc) {
    int64_t pm = idx ? idx[m] : m;
    for (int h = 0; h < H; ++h) {
        int g = (int)(((int64_t)h * H_kv) / H);
        double mx = -INFINITY;
        for (int64_t n = 0; n < M; ++n) {
            int64_t pn = idx ? idx[n] : n;
            if (causal && pn > pm) { w[n] = -INFINITY; continue; }
            double dot = 0.0;
            for (int c = 0; c < d; ++c)
                dot += load_elem(Q, pm * q_tok_stride + h * q_head_stride + c, dtype) *
                       load_elem(K, pn * k_tok_stride + g * k_head_stride + c, dtype);
            w[n] = scale * dot;
            if (w[n] > mx) mx = w[n];
        }
        double den = 0.0;
        for (int64_t n = 0; n < M; ++n) { w[n] = (w[n] == -INFINITY) ? 0.0 : exp(w[n] - mx); den += w[n]; }
        for (int c = 0; c < d; ++c) acc[c] = 0.0;
        for (int64_t n = 0; n < M; ++n) {
            if (w[n] == 0.0) continue;
            int64_t pn = idx ? idx[n] : n;
            double p = w[n] / den;
            for (int c = 0; c < d; ++c) acc[c] += p * load_elem(V, pn * v_tok_stride + g * v_head_stride + c, dtype);
        }
        for (int c = 0; c < d; ++c) {
            int64_t o = o_base + h * o_head_stride + c;
            if (dtype == ORACLE_BF16) ((uint16_t*)O)[o] = double_to_bf16_bits(acc[c]);
            else ((float*)O)[o] = (float)acc[c];
        }
    }
}

/* rows == NULL: every kept query m < M, written to O row m.  rows != NULL: only the listed kept queries, written to O
 * rows 0 .. n_rows-1 (quick spot checks; all 9856 kept queries of the 32K-token layer take about a minute on 16 threads). */
int oracle_kept_attention(const void* Q, const void* K, const void* V, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype,
                          int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                          int64_t v_tok_stride, int64_t v_head_stride, const int32_t* idx, int64_t M, double scale,
                          uint32_t flags, const int64_t* rows, int64_t n_rows, void* O, int64_t o_tok_stride, int64_t o_head_stride) {
    if (!Q || !K || !V || !O || S <= 0 || M < 0 || H <= 0 || H_kv <= 0 || d <= 0 || H % H_kv) return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_ERR_ARG;
    if (!idx && M > S) return ORACLE_ERR_ARG;
    for (int64_t m = 0; m < M; ++m) {
        int64_t r = idx ? idx[m] : m;
        if (r < 0 || r >= S) return ORACLE_ERR_ARG;
    }
    if (!rows) n_rows = M;
    for (int64_t t = 0; rows && t < n_rows; ++t)
        if (rows[t] < 0 || rows[t] >= M) return ORACLE_ERR_ARG;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)d);
    const int causal = (flags & ORACLE_CAUSAL) != 0;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = n_rows - 1; t >= 0; --t) {
        double* w = (double*)malloc(sizeof(double) * (size_t)(M > 0 ? M : 1));
        double* acc = (double*)malloc(sizeof(double) * (size_t)d);
        if (w && acc)
            attention_one_query(Q, K, V, H, H_kv, d, dtype, q_tok_stride, q_head_stride, k_tok_stride, k_head_stride, v_tok_stride,
                                v_head_stride, idx, M, scale, causal, rows ? rows[t] : t, O, t * o_tok_stride, o_head_stride, w, acc);
        else
            fail = 1;
        free(w);
        free(acc);
    }
    return fail ? ORACLE_ERR_NOMEM : ORACLE_OK;
}

/* ---------------------------------------------------------------- scatter-add */

/* dX[idx[m],c] = round_to_dx_type( float(dX[idx[m],c]) + float(G[m,c]) ): one binary32 add and one
 * rounding to the destination type per element (mixed bf16/fp32 precision, Sec. 6.1).  Rows not
 * named by idx stay untouched in ACCUMULATE mode.  ZERO_PAD mode first sets the whole [S,C]
 * destination to +0 and then accumulates, i.e. it writes the zero-padded G.  Indices must be
 * unique and within [0,S). */
int oracle_scatter_add(const void* G, int64_t ldg, const int32_t* idx, int64_t M, void* dX, int64_t lddx,
                       int64_t S, int32_t C, int g_dtype, int dx_dtype, int mode) {
    if (!G || !idx || !dX || S <= 0 || M < 0 || C <= 0 || ldg < C || lddx < C) return ORACLE_ERR_ARG;
    if ((g_dtype != ORACLE_F32 && g_dtype != ORACLE_BF16) || (dx_dtype != ORACLE_F32 && dx_dtype != ORACLE_BF16)) return ORACLE_ERR_ARG;
    if (mode != ORACLE_SCATTER_ACCUMULATE && mode != ORACLE_SCATTER_ZERO_PAD) return ORACLE_ERR_ARG;
    unsigned char* seen = (unsigned char*)calloc((size_t)S, 1);
    if (!seen) return ORACLE_ERR_NOMEM;
    for (int64_t m = 0; m < M; ++m) {
        if (idx[m] < 0 || idx[m] >= S || seen[idx[m]]) { free(seen); return ORACLE_ERR_ARG; }
        seen[idx[m]] = 1;
    }
    free(seen);
    if (mode == ORACLE_SCATTER_ZERO_PAD)
        for (int64_t r = 0; r < S; ++r)
            for (int32_t c = 0; c < C; ++c) {
                if (dx_dtype == ORACLE_BF16) ((uint16_t*)dX)[r * lddx + c] = 0;
                else ((float*)dX)[r * lddx + c] = 0.0f;
            }
    for (int64_t m = 0; m < M; ++m) {
        int64_t r = idx[m];
        for (int32_t c = 0; c < C; ++c) {
            float g = (float)load_elem(G, m * ldg + c, g_dtype);
            float x = (float)load_elem(dX, r * lddx + c, dx_dtype);
            volatile float sum = x + g; /* a single binary32 addition, never contracted or widened */
            if (dx_dtype == ORACLE_BF16) ((uint16_t*)dX)[r * lddx + c] = float_to_bf16_bits(sum);
            else ((float*)dX)[r * lddx + c] = sum;
        }
    }
    return ORACLE_OK;
}

/* threads the scoring and GEMM loops will use (for reporting beside timings) */
int oracle_num_threads(void) { return omp_get_max_threads(); }

/* exposed so tests can pin the bf16 rounding routine against an independent implementation */
uint16_t oracle_double_to_bf16_bits(double x) { return double_to_bf16_bits(x); }
