// Host side of the C ABI declared in lemo.h: argument validation and kernel launches only.
#include <cmath>
#include <mutex>

#include "lemo_common.hpp"

using namespace lemo;

// Scratch of lemo_score_segments_static: the three [H, S] float planes (row log-sum-exp, per-head column sums,
// per-head diagonal) that lemo_score_segments takes from the caller's workspace, for H * S up to LEMO_STATIC_MAX_HS.
// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.  In host
// code the name below is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
// (No `used` attribute here: the compiler gives a static device variable external linkage in the code object -- which
// the runtime's lookup by name needs -- when it sees the host reference below; `used` would emit it earlier, local.)
constexpr long long LEMO_STATIC_MAX_HS = 1ll << 20;
static __device__ __align__(256) unsigned char scratch[3 * LEMO_STATIC_MAX_HS * sizeof(float)];

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool valid_dtype(int dt) { return dt == LEMO_F32 || dt == LEMO_BF16; }
inline int elems_per_16B(int dt) { return dt == LEMO_BF16 ? 8 : 4; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// device address of the current device's copy of `scratch`, looked up once per device
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void* scratch_address[MAX_DEVICES];

int scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return LEMO_ERR_HIP;
    std::lock_guard<std::mutex> guard(scratch_mutex);
    if (!scratch_address[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LEMO_ERR_HIP;
        scratch_address[dev] = p;
    }
    *out = scratch_address[dev];
    return LEMO_OK;
}

int32_t seg_keep(int64_t len, int32_t L, int32_t k) {
    if (len == L) return k;
    int64_t v = ((int64_t)k * len + L - 1) / L;
    if (v < 1) v = 1;
    if (v > len) v = len;
    return (int32_t)v;
}

}  // namespace

extern "C" {

const char* lemo_strerror(int code) {
    switch (code) {
        case LEMO_OK: return "ok";
        case LEMO_ERR_NULL: return "a required pointer is NULL";
        case LEMO_ERR_SHAPE: return "size, stride or count out of range";
        case LEMO_ERR_DTYPE: return "unknown dtype";
        case LEMO_ERR_WORKSPACE: return "workspace too small";
        case LEMO_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
        case LEMO_ERR_UNSUPPORTED: return "valid request the kernels are not built for";
        case LEMO_ERR_HIP: return "HIP runtime refused the launch";
        default: return "unknown error code";
    }
}

int32_t lemo_keep_k(int32_t L, double ratio) {
    if (L <= 0) return 0;
    double v = std::ceil(ratio * (double)L - 1e-9);
    if (!(v >= 1.0)) v = 1.0;
    if (v > (double)L) v = (double)L;
    return (int32_t)v;
}

int64_t lemo_kept_count(int64_t S, int32_t L, int32_t k) {
    if (S <= 0 || L <= 0 || k <= 0 || k > L) return -1;
    const int64_t full = S / L, tail = S % L;
    int64_t M = full * k;
    if (tail) M += seg_keep(tail, L, k);
    return M;
}

int lemo_score_workspace_bytes(int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt, size_t* bytes) {
    if (!bytes) return LEMO_ERR_NULL;
    if (!valid_dtype(dt)) return LEMO_ERR_DTYPE;
    if (S <= 0 || S >= (int64_t)1 << 31 || H <= 0 || H_kv <= 0 || H % H_kv) return LEMO_ERR_SHAPE;
    if (d != 64 && d != 128) return LEMO_ERR_UNSUPPORTED;
    const size_t plane = round_up((size_t)H * (size_t)S * sizeof(float), 256);
    *bytes = 3 * plane;  // row log-sum-exp, per-head column sums, per-head diagonal
    return LEMO_OK;
}

// shared validation of the Q/K description; fills the shape part of the parameter block
static int check_qk(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                    int64_t q_ts, int64_t q_hs, int64_t k_ts, int64_t k_hs, float scale, uint32_t flags, ScoreParams& p) {
    if (!Q || !K) return LEMO_ERR_NULL;
    size_t need = 0;
    const int rc = lemo_score_workspace_bytes(S, H, H_kv, d, dt, &need);
    if (rc != LEMO_OK) return rc;
    if (flags & ~(uint32_t)(LEMO_CAUSAL | LEMO_EXCLUDE_SELF)) return LEMO_ERR_SHAPE;
    if (q_ts < 0 || q_hs < 0 || k_ts < 0 || k_hs < 0 || !std::isfinite(scale)) return LEMO_ERR_SHAPE;
    if (q_ts >= (1 << 22) || k_ts >= (1 << 22)) return LEMO_ERR_UNSUPPORTED;  // token pitch must stay below 16 MiB
    const int e16 = elems_per_16B(dt);
    if (!aligned16(Q) || !aligned16(K) || q_ts % e16 || q_hs % e16 || k_ts % e16 || k_hs % e16) return LEMO_ERR_ALIGN;
    p = ScoreParams{};
    p.Q = Q;
    p.K = K;
    p.S = (int)S;
    p.H = H;
    p.H_kv = H_kv;
    p.q_ts = q_ts;
    p.q_hs = q_hs;
    p.k_ts = k_ts;
    p.k_hs = k_hs;
    const double sc = scale > 0.f ? (double)scale : 1.0 / std::sqrt((double)d);
    p.c2 = (float)(sc * 1.4426950408889634);  // log2(e): probabilities are formed with exp2
    p.L = 1;
    p.flags = flags;
    return LEMO_OK;
}

static inline int hip_rc(int e) { return e == 0 ? LEMO_OK : LEMO_ERR_HIP; }

int lemo_score_rowstats(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                        int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                        float scale, uint32_t flags, float* lse2, void* stream) {
    ScoreParams p;
    const int rc = check_qk(Q, K, S, H, H_kv, d, dt, q_tok_stride, q_head_stride, k_tok_stride, k_head_stride, scale, flags, p);
    if (rc != LEMO_OK) return rc;
    if (!lse2) return LEMO_ERR_NULL;
    p.lse2 = lse2;
    return hip_rc(launch_score(p, dt, d, 1, static_cast<hipStream_t>(stream)));
}

int lemo_score_colsums(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                       int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                       float scale, int32_t L, uint32_t flags, const float* lse2, float* colsum_per_head,
                       float* diag_per_head, void* stream) {
    ScoreParams p;
    const int rc = check_qk(Q, K, S, H, H_kv, d, dt, q_tok_stride, q_head_stride, k_tok_stride, k_head_stride, scale, flags, p);
    if (rc != LEMO_OK) return rc;
    if (!lse2 || !colsum_per_head || !diag_per_head) return LEMO_ERR_NULL;
    if (L <= 0) return LEMO_ERR_SHAPE;
    p.L = L;
    p.lse2 = const_cast<float*>(lse2);
    p.colsum = colsum_per_head;
    p.diag = diag_per_head;
    return hip_rc(launch_score(p, dt, d, 2, static_cast<hipStream_t>(stream)));
}

int lemo_score_head_mean(const float* colsum_per_head, const float* diag_per_head, int64_t S, int32_t H, uint32_t flags,
                         float* scores, void* stream) {
    if (!colsum_per_head || !diag_per_head || !scores) return LEMO_ERR_NULL;
    if (S <= 0 || S >= (int64_t)1 << 31 || H <= 0 || (flags & ~(uint32_t)(LEMO_CAUSAL | LEMO_EXCLUDE_SELF))) return LEMO_ERR_SHAPE;
    ScoreParams p{};
    p.S = (int)S;
    p.H = H;
    p.H_kv = H;
    p.L = 1;
    p.flags = flags;
    p.colsum = const_cast<float*>(colsum_per_head);
    p.diag = const_cast<float*>(diag_per_head);
    p.scores = scores;
    return hip_rc(launch_score(p, LEMO_F32, 64, 4, static_cast<hipStream_t>(stream)));
}

int lemo_score_segments(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                        int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                        float scale, int32_t L, uint32_t flags, float* scores, float* colsum_per_head,
                        float* diag_per_head, void* workspace, size_t workspace_bytes, void* stream) {
    ScoreParams p;
    const int rc = check_qk(Q, K, S, H, H_kv, d, dt, q_tok_stride, q_head_stride, k_tok_stride, k_head_stride, scale, flags, p);
    if (rc != LEMO_OK) return rc;
    if (!scores || !workspace) return LEMO_ERR_NULL;
    if (L <= 0) return LEMO_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return LEMO_ERR_ALIGN;
    size_t need = 0;
    lemo_score_workspace_bytes(S, H, H_kv, d, dt, &need);
    if (workspace_bytes < need) return LEMO_ERR_WORKSPACE;
    const size_t plane = need / 3;
    char* ws = static_cast<char*>(workspace);
    p.L = L;
    p.lse2 = reinterpret_cast<float*>(ws);
    p.colsum = colsum_per_head ? colsum_per_head : reinterpret_cast<float*>(ws + plane);
    p.diag = diag_per_head ? diag_per_head : reinterpret_cast<float*>(ws + 2 * plane);
    p.scores = scores;
    return hip_rc(launch_score(p, dt, d, 7, static_cast<hipStream_t>(stream)));  // the three steps, back to back
}

int lemo_score_segments_static(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                               int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                               float scale, int32_t L, uint32_t flags, float* scores, void* stream) {
    ScoreParams p;
    const int rc = check_qk(Q, K, S, H, H_kv, d, dt, q_tok_stride, q_head_stride, k_tok_stride, k_head_stride, scale, flags, p);
    if (rc != LEMO_OK) return rc;
    if (!scores) return LEMO_ERR_NULL;
    if (L <= 0) return LEMO_ERR_SHAPE;
    if ((long long)H * (long long)S > LEMO_STATIC_MAX_HS) return LEMO_ERR_UNSUPPORTED;  // beyond the built-in scratch
    void* base = nullptr;
    const int src = scratch_of_current_device(&base);
    if (src != LEMO_OK) return src;
    // Every element of the three planes that a later step reads is written by the step before it (row statistics
    // for all S queries, column sums and diagonals for all S keys), so nothing has to be cleared between calls.
    const size_t plane = round_up((size_t)H * (size_t)S * sizeof(float), 256);
    char* ws = static_cast<char*>(base);
    p.L = L;
    p.lse2 = reinterpret_cast<float*>(ws);
    p.colsum = reinterpret_cast<float*>(ws + plane);
    p.diag = reinterpret_cast<float*>(ws + 2 * plane);
    p.scores = scores;
    return hip_rc(launch_score(p, dt, d, 7, static_cast<hipStream_t>(stream)));
}

int lemo_select_topk(const float* scores, int64_t S, int32_t L, int32_t k, int32_t* kept_idx, void* stream) {
    if (!scores || !kept_idx) return LEMO_ERR_NULL;
    if (S <= 0 || S >= (int64_t)1 << 31 || L <= 0 || k <= 0 || k > L) return LEMO_ERR_SHAPE;
    if (L > 32768) return LEMO_ERR_UNSUPPORTED;
    return launch_select(scores, (int)S, L, k, kept_idx, static_cast<hipStream_t>(stream)) == 0 ? LEMO_OK : LEMO_ERR_HIP;
}

int lemo_head_mean_select_topk(const float* colsum_per_head, const float* diag_per_head, int64_t S, int32_t H, uint32_t flags,
                               int32_t L, int32_t k, float* scores, int32_t* kept_idx, void* stream) {
    if (!colsum_per_head || !diag_per_head || !scores || !kept_idx) return LEMO_ERR_NULL;
    if (S <= 0 || S >= (int64_t)1 << 31 || H <= 0 || (flags & ~(uint32_t)(LEMO_CAUSAL | LEMO_EXCLUDE_SELF))) return LEMO_ERR_SHAPE;
    if (L <= 0 || k <= 0 || k > L) return LEMO_ERR_SHAPE;
    if (L > 32768) return LEMO_ERR_UNSUPPORTED;
    return hip_rc(launch_head_mean_select(colsum_per_head, diag_per_head, (int)S, H, (flags & LEMO_EXCLUDE_SELF) ? 1 : 0, L, k, scores,
                                          kept_idx, static_cast<hipStream_t>(stream)));
}

int lemo_launch_floor(void* stream) { return hip_rc(launch_empty(static_cast<hipStream_t>(stream))); }

int lemo_probe_sweep_issue_mix(int32_t tiles_per_wave, uint32_t operand_seed, float* sink, int32_t* waves, void* stream) {
    if (!sink || !waves) return LEMO_ERR_NULL;
    if (tiles_per_wave <= 0 || tiles_per_wave > (1 << 24) || (tiles_per_wave & 1)) return LEMO_ERR_SHAPE;
    int w = 0;
    const int rc = launch_issue_mix(tiles_per_wave, operand_seed, sink, &w, static_cast<hipStream_t>(stream));
    if (rc != 0) return LEMO_ERR_HIP;
    *waves = w;
    return LEMO_OK;
}

int lemo_score_blocks_workspace_bytes(int64_t S, int32_t H, size_t* bytes) {
    if (!bytes) return LEMO_ERR_NULL;
    if (S <= 0 || S >= (int64_t)1 << 31 || H <= 0) return LEMO_ERR_SHAPE;
    const size_t nt32 = (size_t)((S + 31) / 32);
    *bytes = round_up((size_t)H * (size_t)S * sizeof(float), 256) + round_up(nt32 * nt32 * sizeof(float), 256);
    return LEMO_OK;
}

int lemo_score_blocks(const void* Q, const void* K, int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                      int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride, float scale,
                      int32_t b, uint32_t flags, int32_t mode, const float* lse2, float* score_blocks, float* token_blocks,
                      void* workspace, size_t workspace_bytes, void* stream) {
    ScoreParams sp;
    const int rc = check_qk(Q, K, S, H, H_kv, d, dt, q_tok_stride, q_head_stride, k_tok_stride, k_head_stride, scale, flags, sp);
    if (rc != LEMO_OK) return rc;
    if (!token_blocks || !workspace) return LEMO_ERR_NULL;
    if (mode != LEMO_BLOCKS_PROBABILITIES && mode != LEMO_BLOCKS_POSITIVE_LOGITS) return LEMO_ERR_SHAPE;
    if (b <= 0) return LEMO_ERR_SHAPE;
    if (b % 32) return LEMO_ERR_UNSUPPORTED;
    size_t need = 0;
    lemo_score_blocks_workspace_bytes(S, H, &need);
    if (workspace_bytes < need) return LEMO_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return LEMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* lse_ws = static_cast<float*>(workspace);
    float* tiles = reinterpret_cast<float*>(static_cast<char*>(workspace) + round_up((size_t)H * (size_t)S * sizeof(float), 256));
    if (mode == LEMO_BLOCKS_PROBABILITIES && !lse2) {  // sweep 1 of the token-wise score supplies the row statistics
        sp.lse2 = lse_ws;
        if (launch_score(sp, dt, d, 1, st) != 0) return LEMO_ERR_HIP;
        lse2 = lse_ws;
    }
    BlockParams p{};
    p.Q = Q;
    p.K = K;
    p.S = (int)S;
    p.H = H;
    p.H_kv = H_kv;
    p.q_ts = q_tok_stride;
    p.q_hs = q_head_stride;
    p.k_ts = k_tok_stride;
    p.k_hs = k_head_stride;
    p.c2 = sp.c2;
    const double sc = scale > 0.f ? (double)scale : 1.0 / std::sqrt((double)d);
    p.out_scale = mode == LEMO_BLOCKS_PROBABILITIES ? (float)(1.0 / H) : (float)(sc / H);
    p.flags = flags;
    p.lse2 = lse2;
    p.tilemax = tiles;
    return hip_rc(launch_score_blocks(p, dt, d, mode, b, score_blocks, token_blocks, st));
}

int lemo_threshold_init(const float* token_blocks, int64_t nb, float* threshold, void* stream) {
    if (!token_blocks || !threshold) return LEMO_ERR_NULL;
    if (nb <= 0 || nb >= (int64_t)1 << 31) return LEMO_ERR_SHAPE;
    return hip_rc(launch_block_mean(token_blocks, (int)nb, threshold, static_cast<hipStream_t>(stream)));
}

int lemo_select_threshold(const float* token_blocks, int64_t S, int32_t b, float threshold, const float* threshold_dev,
                          int32_t* kept_idx, int32_t* kept_count, void* stream) {
    if (!token_blocks || !kept_idx || !kept_count) return LEMO_ERR_NULL;
    if (S <= 0 || S >= (int64_t)1 << 31 || b <= 0) return LEMO_ERR_SHAPE;
    if (!threshold_dev && std::isnan(threshold)) return LEMO_ERR_SHAPE;
    if ((S + b - 1) / b > 16384) return LEMO_ERR_UNSUPPORTED;
    return hip_rc(launch_select_threshold(token_blocks, (int)S, b, threshold, threshold_dev, kept_idx, kept_count,
                                          static_cast<hipStream_t>(stream)));
}

int lemo_kept_attention_workspace_bytes(int64_t M, int32_t H_kv, int32_t d, size_t* bytes) {
    if (!bytes) return LEMO_ERR_NULL;
    if (M < 0 || M >= (int64_t)1 << 31 || H_kv <= 0 || d <= 0) return LEMO_ERR_SHAPE;
    const size_t Mpad = (size_t)((M + 127) / 128) * 128;
    *bytes = round_up((size_t)H_kv * (size_t)d * Mpad * 2, 256);
    if (*bytes == 0) *bytes = 256;
    return LEMO_OK;
}

int lemo_kept_attention(const void* Q, const void* K, const void* V, int64_t S, int32_t H, int32_t H_kv, int32_t d, lemo_dtype_t dt,
                        int64_t q_tok_stride, int64_t q_head_stride, int64_t k_tok_stride, int64_t k_head_stride,
                        int64_t v_tok_stride, int64_t v_head_stride, const int32_t* kept_idx, int64_t M, float scale, uint32_t flags,
                        void* O, int64_t o_tok_stride, int64_t o_head_stride, void* workspace, size_t workspace_bytes, void* stream) {
    ScoreParams sp;
    const int rc = check_qk(Q, K, S, H, H_kv, d, dt, q_tok_stride, q_head_stride, k_tok_stride, k_head_stride, scale, flags & LEMO_CAUSAL, sp);
    if (rc != LEMO_OK) return rc;
    if (flags & ~(uint32_t)LEMO_CAUSAL) return LEMO_ERR_SHAPE;  // the self pair always takes part in attention
    if (dt != LEMO_BF16) return LEMO_ERR_UNSUPPORTED;
    if (M == 0) return LEMO_OK;
    if (!V || !O || !workspace) return LEMO_ERR_NULL;
    if (M < 0 || M >= (int64_t)1 << 31 || (!kept_idx && M > S)) return LEMO_ERR_SHAPE;
    if (v_tok_stride < 0 || v_head_stride < 0 || o_tok_stride < d || o_head_stride < 0) return LEMO_ERR_SHAPE;
    if (!aligned16(V) || !aligned16(O) || v_tok_stride % 8 || v_head_stride % 8 || o_tok_stride % 8 || o_head_stride % 8) return LEMO_ERR_ALIGN;
    if (kept_idx && (reinterpret_cast<uintptr_t>(kept_idx) & 3u)) return LEMO_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return LEMO_ERR_ALIGN;
    size_t need = 0;
    lemo_kept_attention_workspace_bytes(M, H_kv, d, &need);
    if (workspace_bytes < need) return LEMO_ERR_WORKSPACE;
    // Q and K are addressed with 32-bit byte offsets
    if (((S - 1) * q_tok_stride + (int64_t)(H - 1) * q_head_stride + d) * 2 >= ((int64_t)1 << 32)) return LEMO_ERR_UNSUPPORTED;
    if (((S - 1) * k_tok_stride + (int64_t)(H_kv - 1) * k_head_stride + d) * 2 >= ((int64_t)1 << 32)) return LEMO_ERR_UNSUPPORTED;
    return hip_rc(launch_kept_attention(Q, K, V, S, H, H_kv, d, q_tok_stride, q_head_stride, k_tok_stride, k_head_stride, v_tok_stride,
                                        v_head_stride, kept_idx, M, sp.c2, flags, O, o_tok_stride, o_head_stride, workspace,
                                        static_cast<hipStream_t>(stream)));
}

int lemo_gather_gemm(const void* X, int64_t S, int64_t ldx, const int32_t* kept_idx, int64_t M, const void* W, int64_t ldw,
                     const void* bias, void* Y, int64_t ldy, int32_t C, int32_t N, lemo_dtype_t dt, void* stream) {
    if (!valid_dtype(dt)) return LEMO_ERR_DTYPE;
    if (M == 0) return LEMO_OK;  // nothing to compute; Y may be an empty allocation
    if (!X || !W || !Y) return LEMO_ERR_NULL;
    if (S <= 0 || M < 0 || C <= 0 || N <= 0 || ldx < C || ldw < C || ldy < N) return LEMO_ERR_SHAPE;
    if (!kept_idx && M > S) return LEMO_ERR_SHAPE;
    if (M >= (int64_t)1 << 31 || S >= (int64_t)1 << 31) return LEMO_ERR_SHAPE;
    const int e16 = elems_per_16B(dt);
    if (C % e16) return LEMO_ERR_UNSUPPORTED;
    if (!aligned16(X) || !aligned16(W) || ldx % e16 || ldw % e16) return LEMO_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(Y) % (dt == LEMO_BF16 ? 2 : 4)) return LEMO_ERR_ALIGN;  // Y: element alignment is enough
    if (kept_idx && (reinterpret_cast<uintptr_t>(kept_idx) & 3u)) return LEMO_ERR_ALIGN;
    const int64_t esz = dt == LEMO_BF16 ? 2 : 4;
    if (ldw * esz >= (1 << 23) || ldx * esz >= (1 << 23)) return LEMO_ERR_UNSUPPORTED;  // row pitch below 8 MiB
    if (((S - 1) * ldx + C) * esz >= ((int64_t)1 << 32)) return LEMO_ERR_UNSUPPORTED;      // X is addressed with 32-bit offsets
    const int64_t tiles = ((M + 255) / 256) * (((int64_t)N + 255) / 256);
    if (tiles >= (int64_t)1 << 28) return LEMO_ERR_UNSUPPORTED;
    return launch_gather_gemm(X, S, ldx, kept_idx, M, W, ldw, bias, Y, ldy, C, N, dt, static_cast<hipStream_t>(stream)) == 0
               ? LEMO_OK : LEMO_ERR_HIP;
}

int lemo_gather_gemm_add(const void* X, int64_t S, int64_t ldx, const int32_t* kept_idx, int64_t M, const void* W, int64_t ldw,
                         const void* bias, void* R, int64_t ldr, int64_t S_out, const int32_t* out_idx, int32_t C, int32_t N,
                         lemo_dtype_t dt, void* stream) {
    if (!valid_dtype(dt)) return LEMO_ERR_DTYPE;
    if (M == 0) return LEMO_OK;  // nothing to add
    if (!X || !W || !R) return LEMO_ERR_NULL;
    if (S <= 0 || S_out <= 0 || M < 0 || C <= 0 || N <= 0 || ldx < C || ldw < C || ldr < N) return LEMO_ERR_SHAPE;
    if ((!kept_idx && M > S) || M > S_out) return LEMO_ERR_SHAPE;  // unique output rows cannot outnumber the rows of R
    if (M >= (int64_t)1 << 31 || S >= (int64_t)1 << 31 || S_out >= (int64_t)1 << 31) return LEMO_ERR_SHAPE;
    const int e16 = elems_per_16B(dt);
    if (C % e16) return LEMO_ERR_UNSUPPORTED;
    if (!aligned16(X) || !aligned16(W) || ldx % e16 || ldw % e16) return LEMO_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(R) % (dt == LEMO_BF16 ? 2 : 4)) return LEMO_ERR_ALIGN;
    if ((kept_idx && (reinterpret_cast<uintptr_t>(kept_idx) & 3u)) || (out_idx && (reinterpret_cast<uintptr_t>(out_idx) & 3u)))
        return LEMO_ERR_ALIGN;
    const int64_t esz = dt == LEMO_BF16 ? 2 : 4;
    if (ldw * esz >= (1 << 23) || ldx * esz >= (1 << 23)) return LEMO_ERR_UNSUPPORTED;  // row pitch below 8 MiB
    if (((S - 1) * ldx + C) * esz >= ((int64_t)1 << 32)) return LEMO_ERR_UNSUPPORTED;      // X is addressed with 32-bit offsets
    if (ldr * esz >= (1 << 23) || ((S_out - 1) * ldr + N) * esz >= ((int64_t)1 << 32) - 16) return LEMO_ERR_UNSUPPORTED;  // so is R
    const int64_t tiles = ((M + 255) / 256) * (((int64_t)N + 255) / 256);
    if (tiles >= (int64_t)1 << 28) return LEMO_ERR_UNSUPPORTED;
    return launch_gather_gemm_add(X, S, ldx, kept_idx, M, W, ldw, bias, R, ldr, S_out, out_idx, C, N, dt,
                                  static_cast<hipStream_t>(stream)) == 0
               ? LEMO_OK : LEMO_ERR_HIP;
}

int lemo_gather_gemm_dx(const void* dY, int64_t ldy, int64_t M, const void* W, int64_t ldw, void* dX, int64_t lddx, int64_t S_out,
                        const int32_t* out_idx, int32_t C, int32_t N, lemo_dtype_t dt, void* stream) {
    if (!valid_dtype(dt)) return LEMO_ERR_DTYPE;
    if (M == 0) return LEMO_OK;  // nothing to add
    if (!dY || !W || !dX) return LEMO_ERR_NULL;
    if (S_out <= 0 || M < 0 || C <= 0 || N <= 0 || ldy < N || ldw < C || lddx < C) return LEMO_ERR_SHAPE;
    if (M > S_out || M >= (int64_t)1 << 31 || S_out >= (int64_t)1 << 31) return LEMO_ERR_SHAPE;
    if (dt != LEMO_BF16) return LEMO_ERR_UNSUPPORTED;  // fp32: lemo_gather_gemm_add with the transposed weight
    if (C % 8 || N % 8) return LEMO_ERR_UNSUPPORTED;
    if (!aligned16(dY) || !aligned16(W) || ldy % 8 || ldw % 8) return LEMO_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(dX) % 2 || (out_idx && (reinterpret_cast<uintptr_t>(out_idx) & 3u))) return LEMO_ERR_ALIGN;
    if (ldy * 2 >= (1 << 23) || ldw * 2 >= (1 << 23) || lddx * 2 >= (1 << 23)) return LEMO_ERR_UNSUPPORTED;  // row pitches below 8 MiB
    if (((M - 1) * ldy + N) * 2 >= ((int64_t)1 << 32)) return LEMO_ERR_UNSUPPORTED;               // dY is addressed with 32-bit offsets
    if (((int64_t)(N - 1) * ldw + C) * 2 >= ((int64_t)1 << 31)) return LEMO_ERR_UNSUPPORTED;     // W: signed 32-bit spans
    if (((S_out - 1) * lddx + C) * 2 >= ((int64_t)1 << 32) - 16) return LEMO_ERR_UNSUPPORTED;     // so is dX
    const int64_t tiles = ((M + 255) / 256) * (((int64_t)C + 255) / 256);
    if (tiles >= (int64_t)1 << 28) return LEMO_ERR_UNSUPPORTED;
    return hip_rc(launch_gather_gemm_dx(dY, ldy, M, W, ldw, dX, lddx, S_out, out_idx, C, N, static_cast<hipStream_t>(stream)));
}

// bf16 takes the kernel that reads both operands as they are stored when their spans fit its 32-bit offsets
static bool dw_direct(int64_t ldy, int64_t S, int64_t ldx, int64_t M, int32_t C, int32_t N, lemo_dtype_t dt) {
    return dt == LEMO_BF16 && ldy * 2 < (1 << 23) && ldx * 2 < (1 << 23) && ((M - 1) * ldy + N) * 2 < ((int64_t)1 << 31) &&
           ((S - 1) * ldx + C) * 2 < ((int64_t)1 << 32) - 16;
}

int lemo_gather_gemm_dw_workspace_bytes(int64_t M, int32_t C, int32_t N, lemo_dtype_t dt, size_t* bytes) {
    if (!bytes) return LEMO_ERR_NULL;
    if (!valid_dtype(dt)) return LEMO_ERR_DTYPE;
    if (M < 0 || M >= (int64_t)1 << 31 || C <= 0 || N <= 0) return LEMO_ERR_SHAPE;
    if (dt == LEMO_BF16) { *bytes = 0; return LEMO_OK; }  // both operands are read where they lie
    const size_t Mpad = (size_t)((M + 63) / 64) * 64, esz = dt == LEMO_BF16 ? 2 : 4;
    *bytes = round_up((size_t)N * Mpad * esz, 256) + round_up((size_t)C * Mpad * esz, 256);
    if (*bytes == 0) *bytes = 256;
    return LEMO_OK;
}

int lemo_gather_gemm_dw(const void* dY, int64_t ldy, const void* X, int64_t S, int64_t ldx, const int32_t* kept_idx, int64_t M, void* dW,
                        int64_t lddw, int32_t C, int32_t N, lemo_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    if (!valid_dtype(dt)) return LEMO_ERR_DTYPE;
    if (!dW || (M > 0 && (!dY || !X))) return LEMO_ERR_NULL;
    if (S <= 0 || M < 0 || C <= 0 || N <= 0 || ldy < N || ldx < C || lddw < C) return LEMO_ERR_SHAPE;
    if ((!kept_idx && M > S) || M >= (int64_t)1 << 31 || S >= (int64_t)1 << 31) return LEMO_ERR_SHAPE;
    const int e16 = elems_per_16B(dt);
    if (C % e16 || N % e16) return LEMO_ERR_UNSUPPORTED;
    if ((M > 0 && (!aligned16(dY) || !aligned16(X))) || ldy % e16 || ldx % e16) return LEMO_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(dW) % (dt == LEMO_BF16 ? 2 : 4)) return LEMO_ERR_ALIGN;
    if (kept_idx && (reinterpret_cast<uintptr_t>(kept_idx) & 3u)) return LEMO_ERR_ALIGN;
    if (M > 0 && dw_direct(ldy, S, ldx, M, C, N, dt)) {  // both operands read where they lie: no workspace
        const int64_t tiles = (((int64_t)N + 255) / 256) * (((int64_t)C + 255) / 256);
        if (tiles >= (int64_t)1 << 28) return LEMO_ERR_UNSUPPORTED;
        return hip_rc(launch_gather_gemm_dw_direct(dY, ldy, X, S, ldx, kept_idx, M, dW, lddw, C, N, static_cast<hipStream_t>(stream)));
    }
    if (M == 0) return hip_rc(launch_zero_matrix(dW, lddw, C, N, dt, static_cast<hipStream_t>(stream)));  // an empty sum: dW = 0
    if (dt == LEMO_BF16) return LEMO_ERR_UNSUPPORTED;  // operands beyond the 32-bit offsets of the kernel
    if (!workspace) return LEMO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return LEMO_ERR_ALIGN;
    const size_t Mp = (size_t)((M + 63) / 64) * 64, es = dt == LEMO_BF16 ? 2 : 4;
    const size_t need = round_up((size_t)N * Mp * es, 256) + round_up((size_t)C * Mp * es, 256);  // transposed copies of both operands
    if (workspace_bytes < need) return LEMO_ERR_WORKSPACE;
    const int64_t esz = dt == LEMO_BF16 ? 2 : 4, Mpad = (M + 63) / 64 * 64;
    if (Mpad * esz >= (1 << 23) || (int64_t)N * Mpad * esz >= ((int64_t)1 << 32)) return LEMO_ERR_UNSUPPORTED;  // limits of the GEMM on the transposed operands
    const int64_t tiles = (((int64_t)N + 255) / 256) * (((int64_t)C + 255) / 256);
    if (tiles >= (int64_t)1 << 28) return LEMO_ERR_UNSUPPORTED;
    return hip_rc(launch_gather_gemm_dw(dY, ldy, X, S, ldx, kept_idx, M, dW, lddw, C, N, dt, workspace, static_cast<hipStream_t>(stream)));
}

int lemo_scatter_grad(const void* G, int64_t ldg, const int32_t* kept_idx, int64_t M, void* dX, int64_t lddx, int64_t S,
                      int32_t C, lemo_dtype_t g_dt, lemo_dtype_t dx_dt, int32_t mode, void* stream) {
    if (!dX || (M > 0 && (!G || !kept_idx))) return LEMO_ERR_NULL;
    if (!valid_dtype(g_dt) || !valid_dtype(dx_dt)) return LEMO_ERR_DTYPE;
    if (mode != LEMO_SCATTER_ACCUMULATE && mode != LEMO_SCATTER_ZERO_PAD) return LEMO_ERR_SHAPE;
    if (S <= 0 || S >= (int64_t)1 << 31 || M < 0 || M > S || C <= 0 || ldg < C || lddx < C) return LEMO_ERR_SHAPE;
    if (C % 8) return LEMO_ERR_UNSUPPORTED;
    if (!aligned16(dX) || lddx % elems_per_16B(dx_dt)) return LEMO_ERR_ALIGN;
    if (M > 0 && (!aligned16(G) || ldg % elems_per_16B(g_dt))) return LEMO_ERR_ALIGN;
    return launch_scatter(G, ldg, kept_idx, M, dX, lddx, S, C, g_dt, dx_dt, mode, static_cast<hipStream_t>(stream)) == 0
               ? LEMO_OK : LEMO_ERR_HIP;
}

}  // extern "C"
