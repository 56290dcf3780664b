/*
 * Sanitizer driver for the CPU oracle (test infrastructure).  Built together with oracle/lemo_oracle.c under
 * -fsanitize=address,undefined by tests/test_oracle_sanitizers.py; it calls every oracle routine on small seeded
 * inputs chosen for their edges (one token, ragged last segment / block, grouped KV heads, strided views, empty kept
 * sets, unsorted indices) and checks return codes and a few invariants, so that an out-of-bounds access, a leak, a
 * signed overflow or a misaligned access anywhere in the oracle fails the run.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int32_t oracle_keep_k(int32_t L, double ratio);
int64_t oracle_kept_count(int64_t S, int32_t L, int32_t k);
int oracle_score(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype, int64_t qts, int64_t qhs,
                 int64_t kts, int64_t khs, double scale, uint32_t flags, float* scores, double* colsum, double* diag);
int oracle_score_bruteforce(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype, int64_t qts,
                            int64_t qhs, int64_t kts, int64_t khs, double scale, uint32_t flags, float* scores);
int oracle_score_blocks(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype, int64_t qts, int64_t qhs,
                        int64_t kts, int64_t khs, double scale, uint32_t flags, int32_t b, int mode, double* score_blocks, float* token_blocks);
int oracle_score_block_rows(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype, int64_t qts,
                            int64_t qhs, int64_t kts, int64_t khs, double scale, uint32_t flags, int32_t b, int mode, const int64_t* rows,
                            int32_t n_rows, double* row_out);
int64_t oracle_select_threshold(const float* token_blocks, int64_t S, int32_t b, double T, int32_t* kept_idx);
double oracle_threshold_init(const float* token_blocks, int64_t nb);
int oracle_select_topk(const float* scores, int64_t S, int32_t L, int32_t k, int32_t* kept_idx);
int oracle_gather_gemm(const void* X, int64_t S, int64_t ldx, const int32_t* idx, int64_t M, const void* W, int64_t ldw, const void* bias,
                       void* Y, int64_t ldy, int32_t C, int32_t N, int dtype);
int oracle_gather_gemm_add(const void* X, int64_t S, int64_t ldx, const int32_t* in_idx, int64_t M, const void* W, int64_t ldw,
                           const void* bias, void* R, int64_t ldr, int64_t S_out, const int32_t* out_idx, int32_t C, int32_t N, int dtype);
int oracle_gather_gemm_dw(const void* dY, int64_t ldy, const void* X, int64_t S, int64_t ldx, const int32_t* idx, int64_t M, void* dW,
                          int64_t lddw, int32_t C, int32_t N, int dtype);
int oracle_kept_attention(const void* Q, const void* K, const void* V, int64_t S, int32_t H, int32_t H_kv, int32_t d, int dtype, int64_t qts,
                          int64_t qhs, int64_t kts, int64_t khs, int64_t vts, int64_t vhs, const int32_t* idx, int64_t M, double scale,
                          uint32_t flags, const int64_t* rows, int64_t n_rows, void* O, int64_t ots, int64_t ohs);
int oracle_scatter_add(const void* G, int64_t ldg, const int32_t* idx, int64_t M, void* dX, int64_t lddx, int64_t S, int32_t C, int g_dtype,
                       int dx_dtype, int mode);
uint16_t oracle_double_to_bf16_bits(double x);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform(void) { /* xorshift64*, in (-1, 1) */
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (double)((rng_state * 0x2545F4914F6CDD1Dull) >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
/* exactly n elements of the given dtype (0 = float, 1 = bf16 bits): a read one element past the end is out of bounds */
static void* random_array(size_t n, int dtype, double amp) {
    void* p = malloc(n * (dtype ? 2 : 4) + (n == 0));
    for (size_t i = 0; i < n; ++i) {
        if (dtype) ((uint16_t*)p)[i] = oracle_double_to_bf16_bits(amp * uniform());
        else ((float*)p)[i] = (float)(amp * uniform());
    }
    return p;
}
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "driver: check failed at line %d: %s\n", __LINE__, #cond); exit(1); } } while (0)

static void score_cases(void) {
    const int shapes[][5] = {{1, 2, 1, 8, 4}, {7, 4, 2, 8, 3}, {33, 3, 3, 16, 5}, {50, 4, 1, 8, 7}};  /* S, H, H_kv, d, b */
    for (unsigned s = 0; s < sizeof shapes / sizeof shapes[0]; ++s)
        for (int dtype = 0; dtype < 2; ++dtype)
            for (uint32_t flags = 0; flags < 4; ++flags) {
                const int64_t S = shapes[s][0];
                const int H = shapes[s][1], Hkv = shapes[s][2], d = shapes[s][3], b = shapes[s][4];
                void* Q = random_array((size_t)S * H * d, dtype, 2.0);
                void* K = random_array((size_t)S * Hkv * d, dtype, 2.0);
                float* sc = malloc(sizeof(float) * S);
                float* sc2 = malloc(sizeof(float) * S);
                double* col = malloc(sizeof(double) * H * S);
                double* dg = malloc(sizeof(double) * H * S);
                CHECK(oracle_score(Q, K, S, H, Hkv, d, dtype, H * d, d, Hkv * d, d, 0.0, flags, sc, col, dg) == 0);
                CHECK(oracle_score_bruteforce(Q, K, S, H, Hkv, d, dtype, H * d, d, Hkv * d, d, 0.0, flags, sc2) == 0);
                for (int h = 0; h < H; ++h) {  /* rows of a softmax sum to one */
                    double tot = 0.0;
                    for (int64_t j = 0; j < S; ++j) tot += col[h * S + j];
                    CHECK(fabs(tot - (double)S) < 1e-9 * (double)S);
                }
                for (int64_t j = 0; j < S; ++j) CHECK(fabs((double)sc[j] - (double)sc2[j]) <= 1e-6 * fabs((double)sc2[j]) + 1e-7);
                const int64_t nb = (S + b - 1) / b;
                double* sb = malloc(sizeof(double) * nb * nb);
                float* tb = malloc(sizeof(float) * nb);
                for (int mode = 0; mode < 2; ++mode) {
                    CHECK(oracle_score_blocks(Q, K, S, H, Hkv, d, dtype, H * d, d, Hkv * d, d, 0.0, flags, b, mode, sb, tb) == 0);
                    int64_t rows[2] = {0, nb - 1};
                    double* ro = malloc(sizeof(double) * 2 * nb);
                    CHECK(oracle_score_block_rows(Q, K, S, H, Hkv, d, dtype, H * d, d, Hkv * d, d, 0.0, flags, b, mode, rows, 2, ro) == 0);
                    for (int64_t n = 0; n < nb; ++n) CHECK(ro[n] == sb[n] && ro[nb + n] == sb[(nb - 1) * nb + n]);
                    free(ro);
                }
                int32_t* kept = malloc(sizeof(int32_t) * S);
                const double T = oracle_threshold_init(tb, nb);
                const int64_t cnt = oracle_select_threshold(tb, S, b, T, kept);
                CHECK(cnt >= 0 && cnt <= S);
                CHECK(oracle_select_threshold(tb, S, b, -INFINITY, kept) == S);
                free(kept); free(sb); free(tb); free(Q); free(K); free(sc); free(sc2); free(col); free(dg);
            }
}

static void select_cases(void) {
    const int cases[][3] = {{1, 8, 8}, {7, 4, 3}, {100, 1, 1}, {130, 64, 20}, {64, 64, 64}, {200, 300, 150}};  /* S, L, k */
    for (unsigned c = 0; c < sizeof cases / sizeof cases[0]; ++c) {
        const int64_t S = cases[c][0];
        const int L = cases[c][1], k = cases[c][2];
        float* sc = random_array((size_t)S, 0, 1.0);
        for (int64_t j = 0; j < S; j += 3) sc[j] = 0.25f;  /* ties */
        const int64_t M = oracle_kept_count(S, L, k);
        CHECK(M > 0 && M <= S);
        int32_t* kept = malloc(sizeof(int32_t) * M);
        CHECK(oracle_select_topk(sc, S, L, k, kept) == 0);
        for (int64_t m = 0; m < M; ++m) CHECK(kept[m] >= 0 && kept[m] < S && (m == 0 || kept[m] > kept[m - 1]));
        free(kept); free(sc);
    }
    CHECK(oracle_keep_k(1024, 0.3) == 308 && oracle_keep_k(128, 0.5) == 64 && oracle_keep_k(0, 0.5) == 0);
    CHECK(oracle_kept_count(10, 4, 5) == -1);
}

static void gemm_scatter_attention_cases(void) {
    for (int dtype = 0; dtype < 2; ++dtype) {
        const int64_t S = 37, M = 11;
        const int C = 24, N = 13, H = 4, Hkv = 2, d = 8;
        int32_t idx[11] = {36, 0, 5, 17, 3, 29, 30, 8, 21, 12, 1};   /* unsorted, first and last rows included */
        int32_t sorted[11] = {0, 1, 3, 5, 8, 12, 17, 21, 29, 30, 36};
        void* X = random_array((size_t)S * C, dtype, 1.0);
        void* W = random_array((size_t)N * C, dtype, 0.1);
        void* bias = random_array((size_t)N, dtype, 1.0);
        void* Y = random_array((size_t)M * N, dtype, 0.0);
        CHECK(oracle_gather_gemm(X, S, C, idx, M, W, C, bias, Y, N, C, N, dtype) == 0);
        CHECK(oracle_gather_gemm(X, S, C, NULL, M, W, C, NULL, Y, N, C, N, dtype) == 0);       /* no index list: rows 0..M-1 */
        CHECK(oracle_gather_gemm(X, S, C, idx, 0, W, C, NULL, Y, N, C, N, dtype) == 0);       /* nothing kept */
        void* R = random_array((size_t)S * N, dtype, 1.0);
        CHECK(oracle_gather_gemm_add(X, S, C, idx, M, W, C, bias, R, N, S, sorted, C, N, dtype) == 0);
        CHECK(oracle_gather_gemm_add(X, S, C, NULL, M, W, C, NULL, R, N, S, NULL, C, N, dtype) == 0);
        void* dW = random_array((size_t)N * C, dtype, 0.0);
        CHECK(oracle_gather_gemm_dw(Y, N, X, S, C, idx, M, dW, C, C, N, dtype) == 0);
        CHECK(oracle_gather_gemm_dw(Y, N, X, S, C, idx, 0, dW, C, C, N, dtype) == 0);          /* empty sum */
        void* G = random_array((size_t)M * C, dtype, 1.0);
        for (int xdt = 0; xdt < 2; ++xdt)
            for (int mode = 0; mode < 2; ++mode) {
                void* dX = random_array((size_t)S * C, xdt, 1.0);
                CHECK(oracle_scatter_add(G, C, mode ? sorted : idx, M, dX, C, S, C, dtype, xdt, mode) == 0);
                free(dX);
            }
        void* Q = random_array((size_t)S * H * d, dtype, 2.0);
        void* K = random_array((size_t)S * Hkv * d, dtype, 2.0);
        void* V = random_array((size_t)S * Hkv * d, dtype, 1.0);
        void* O = random_array((size_t)M * H * d, dtype, 0.0);
        for (uint32_t flags = 0; flags < 2; ++flags) {
            CHECK(oracle_kept_attention(Q, K, V, S, H, Hkv, d, dtype, H * d, d, Hkv * d, d, Hkv * d, d, sorted, M, 0.0, flags, NULL, 0, O, H * d, d) == 0);
            int64_t rows[3] = {0, 10, 4};
            CHECK(oracle_kept_attention(Q, K, V, S, H, Hkv, d, dtype, H * d, d, Hkv * d, d, Hkv * d, d, sorted, M, 0.0, flags, rows, 3, O, H * d, d) == 0);
        }
        free(X); free(W); free(bias); free(Y); free(R); free(dW); free(G); free(Q); free(K); free(V); free(O);
    }
}

static void bf16_rounding_cases(void) {
    const double v[] = {0.0, -0.0, 1.0, 1.00390625, 1.0 + 1.0 / 256 + 1e-9, 3.3895313892515355e38, 3.4e38, 1e-40, 9.18e-41, 4.6e-41, -2.5, INFINITY, NAN};
    for (unsigned i = 0; i < sizeof v / sizeof v[0]; ++i) (void)oracle_double_to_bf16_bits(v[i]);
    CHECK(oracle_double_to_bf16_bits(1.0) == 0x3f80 && oracle_double_to_bf16_bits(1.00390625) == 0x3f80);  /* tie to even */
    CHECK(oracle_double_to_bf16_bits(1.0 + 1.0 / 256 + 1e-9) == 0x3f81);
}

int main(void) {
    score_cases();
    select_cases();
    gemm_scatter_attention_cases();
    bf16_rounding_cases();
    printf("oracle sanitizer driver: ok\n");
    return 0;
}
