// Attention over the kept tokens, read in place (Sec. 4.4: the block loads the selected tokens straight from the
// original inputs; no re-permuted copy of Q or K is made).
//
//   O[m,h,:] = sum_n softmax_n(scale * <Q[idx[m],h], K[idx[n],g]>) V[idx[n],g,:]        g = floor(h * H_kv / H)
//
// A workgroup owns 256 kept queries of one head (8 waves x 32), their rows gathered through idx into MFMA fragments that
// stay in registers, and walks the kept keys in stages of 128 through two LDS stages.  Both products are computed
// transposed so that a lane owns one QUERY column throughout:
//   S^T = K Q^T       acc[key row][query col]: the 16 logits a lane holds belong to one query -> the online softmax is
//                     an in-register chain; the two half-waves (which hold the other 16 keys of the same query) agree
//                     on the running maximum with one cross-lane exchange per tile
//   O^T += V^T P^T    the B operand (P^T: 8 keys per lane for its query column) is exactly what the lane already holds:
//                     registers 8c..8c+7 of the logit tile are keys 16c + 4*half + {0..3} and 16c + 8 + 4*half + {0..3},
//                     and since a dot product does not care in which order its terms are paired, the A operand (V^T)
//                     simply supplies the same keys in the same slots.
// V^T needs the keys contiguous per value column, which the [token, head, d] layout does not offer; a small kernel first
// writes the kept rows of V transposed ([H_kv, d, M] in the workspace; 2 bytes per kept element, once per call).
// P is rounded to bf16 for the second product (as in every flash-attention kernel); the normaliser is summed from the
// unrounded values.
#include <mutex>
#include <type_traits>

#include "lemo_common.hpp"

namespace lemo {

// Eight waves per workgroup (two per SIMD: while one wave does its softmax arithmetic the other has the matrix core),
// each keeping ONE 32-query subtile: 64 accumulator registers for O^T, everything within 256 registers.  One workgroup
// per CU with two LDS stages of 128 keys: a barrier every four tiles, and a stage of K and V^T is shared by 256 queries.
#ifndef LEMO_AT_THREADS
#define LEMO_AT_THREADS 512
#endif
#ifndef LEMO_AT_NQ
#define LEMO_AT_NQ 1
#endif
#ifndef LEMO_AT_PIPE
#define LEMO_AT_PIPE 1
#endif
constexpr int AT_THREADS = LEMO_AT_THREADS;
constexpr int AT_NQ = LEMO_AT_NQ;                   // 32-query subtiles per wave
constexpr int AT_BQ = (AT_THREADS / 64) * 32 * AT_NQ;  // queries per workgroup
constexpr int AT_KT = 128;                          // keys per LDS stage
constexpr int AT_MPAD = 128;         // the transposed V is padded to a multiple of this many kept tokens

template <int D> struct AGeo {
    static constexpr int ROWB = D * 2;            // bytes per head row (bf16)
    static constexpr int NCH = ROWB / 32;         // MFMA chunks per K / Q row
    static constexpr int CPR = ROWB / 16;         // 16-byte pieces per K row
    static constexpr int KSTRIDE = ROWB + 16;     // LDS pitch of a K row
    static constexpr int VSTRIDE = AT_KT * 2 + 16;  // LDS pitch of a V^T row (128 keys)
    static constexpr int NDV = D / 32;            // 32-row tiles of the value dimension
    static constexpr int NLK = AT_KT * CPR / AT_THREADS;  // K loads per thread and stage
    static constexpr int K_RPL = AT_THREADS / CPR;        // K rows covered by one load of the workgroup
    static constexpr int VCPR = AT_KT * 2 / 16;           // 16-byte pieces per V^T row of a stage
    static constexpr int NLV = D * VCPR / AT_THREADS;     // V^T loads per thread and stage
    static constexpr int V_RPL = AT_THREADS / VCPR;       // V^T rows covered by one load of the workgroup
    static constexpr int STAGE = AT_KT * KSTRIDE + D * VSTRIDE;
    static constexpr int LDS = 2 * STAGE;
};

struct AttnParams {
    const uint16_t* Q;
    const uint16_t* K;
    const uint16_t* Vt;  // [H_kv, D, Mpad]
    const int* idx;      // [M] or null
    uint16_t* O;
    int M, Mpad, H, H_kv;
    long long q_ts, q_hs, k_ts, k_hs, o_ts, o_hs;  // element strides
    unsigned q_bytes, k_bytes;                     // spans of Q and K (32-bit buffer offsets)
    float c2;
    unsigned flags;
    int n_qblocks, heads_per_xcd;
};

// Inside every group of 16 kept tokens the transposed V is stored with its two middle quads exchanged (tokens 0-3, 8-11,
// 4-7, 12-15): the 8 key slots a lane feeds to the second MFMA are keys 4*half + {0..3} and 8 + 4*half + {0..3} of a
// 16-key chunk, and in this order they are 16 contiguous bytes.  The permutation is its own inverse.
__device__ __forceinline__ int vt_src(int pos) { return (pos & ~12) | ((pos & 4) << 1) | ((pos & 8) >> 1); }

// kept rows of V, transposed: Vt[g][c][pos] = V[idx[vt_src(pos)], g, c] for kept tokens below M, zero up to Mpad
__global__ __launch_bounds__(256) void gather_vt_kernel(const uint16_t* __restrict__ V, long long v_ts, long long v_hs, const int* __restrict__ idx,
                                                        int M, int Mpad, int D, uint16_t* __restrict__ Vt) {
    __shared__ uint16_t tile[64][128 + 2];
    const int m0 = blockIdx.x * 64, g = blockIdx.y, tid = threadIdx.x;
    // load 64 kept rows x D values: thread -> (row = tid / 16 + 16 * i, 8 values at (tid % 16) * 8)
    for (int i = 0; i < 4; ++i) {
        const int row = tid / 16 + 16 * i, c0 = (tid % 16) * 8, m = m0 + row;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (m < M && c0 < D) {
            const long long tok = idx ? idx[m] : m;
            v = *reinterpret_cast<const u32x4*>(V + tok * v_ts + (long long)g * v_hs + c0);
        }
        if (c0 < D) {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) tile[row][c0 + e] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
        }
    }
    __syncthreads();
    // store: value column c, 64 consecutive kept tokens = 128 bytes; thread -> (c = tid / 8 + 32 * i, 8 tokens at (tid % 8) * 8)
    for (int i = 0; i < 4; ++i) {
        const int c = tid / 8 + 32 * i, r0 = (tid % 8) * 8;
        if (c < D) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (uint32_t)tile[vt_src(r0 + 2 * e)][c] | ((uint32_t)tile[vt_src(r0 + 2 * e + 1)][c] << 16);
            *reinterpret_cast<u32x4*>(Vt + ((long long)g * D + c) * Mpad + m0 + r0) = u32x4{w[0], w[1], w[2], w[3]};
        }
    }
}

template <int D>
__global__ __launch_bounds__(AT_THREADS, 1) void kept_attention_kernel(AttnParams p) {
    using G = AGeo<D>;
    using T = bf16_t;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // block -> (head, query block): die b % 8 gets a contiguous range of heads; late query blocks (most keys) first
    const int b = blockIdx.x, x = b % NUM_XCD, w_ = b / NUM_XCD;
    const int slot = w_ / p.n_qblocks;
    int qb = w_ - slot * p.n_qblocks;
    const int h = x * p.heads_per_xcd + slot;
    if (h >= p.H) return;
    const bool causal = (p.flags & LEMO_CAUSAL) != 0;
    if (causal) qb = p.n_qblocks - 1 - qb;
    const int g = (int)(((long long)h * p.H_kv) / p.H);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int M = p.M;
    const float c2 = p.c2;
    const int m0 = qb * AT_BQ, mw0 = m0 + wave * 32 * AT_NQ;

    // resident operand: this wave's 64 queries (rows gathered through idx), as MFMA B fragments
    u32x4 qf[AT_NQ][G::NCH];
#pragma unroll
    for (int qs = 0; qs < AT_NQ; ++qs) {
        const int m = mw0 + qs * 32 + l32;
        const long long tok = m < M ? (p.idx ? (long long)p.idx[m] : (long long)m) : -1;
#pragma unroll
        for (int c = 0; c < G::NCH; ++c) {
            qf[qs][c] = u32x4{0u, 0u, 0u, 0u};
            if (tok >= 0) qf[qs][c] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(p.Q + tok * p.q_ts + (long long)h * p.q_hs) + c * 32 + half * 16);
        }
    }

    // O^T accumulators: o[qs][dv][r] = element (value row dv*32 + acc_row(r), query column l32 of subtile qs)
    f32x16 o[AT_NQ][G::NDV];
#pragma unroll
    for (int qs = 0; qs < AT_NQ; ++qs)
#pragma unroll
        for (int dv = 0; dv < G::NDV; ++dv) o[qs][dv] = f32x16{0};
    float mrun[AT_NQ], lrun[AT_NQ];  // reference of the exponentials (base-2 units, identical in both half-waves); this half-wave's share of the normaliser
#pragma unroll
    for (int qs = 0; qs < AT_NQ; ++qs) { mrun[qs] = -INFINITY; lrun[qs] = 0.f; }

    const int k_last = causal ? min(m0 + AT_BQ, M) - 1 : M - 1;
    const int nstage = k_last / AT_KT + 1;

    // staging.  K rows are gathered through idx (32-bit offsets into a range-checked descriptor of the whole K tensor);
    // V^T rows are contiguous in the workspace.
    const int k_row = tid / G::CPR, k_cc = tid % G::CPR;
    const int k_row_bytes = (int)p.k_ts * 2;
    const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(p.K + (long long)g * p.k_hs)), 0, (int)(p.k_bytes - (unsigned)(g * p.k_hs * 2)), 0x00020000);
    const int v_row = tid / G::VCPR, v_cc = tid % G::VCPR;
    const uint16_t* vt_head = p.Vt + (long long)g * D * p.Mpad;
    u32x4 prek[G::NLK], prev_[G::NLV];
    // Row indices run one stage ahead of the rows (tok holds the K rows of the stage about to be fetched), so a row load
    // never waits behind its own index; rows past the end repeat the last kept row (masked later).
    unsigned tok[G::NLK];
    auto fetch_idx = [&](int t) {
        const int n0 = t * AT_KT;
        if (p.idx) {
#pragma unroll
            for (int i = 0; i < G::NLK; ++i) tok[i] = (unsigned)p.idx[min(n0 + k_row + i * G::K_RPL, M - 1)];
        } else {
#pragma unroll
            for (int i = 0; i < G::NLK; ++i) tok[i] = (unsigned)min(n0 + k_row + i * G::K_RPL, M - 1);
        }
    };
    auto fetch = [&](int t) {  // needs tok = fetch_idx(t); leaves tok = fetch_idx(t + 1)
        const int n0 = t * AT_KT;
#pragma unroll
        for (int i = 0; i < G::NLK; ++i)
            prek[i] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, (int)(tok[i] * (unsigned)k_row_bytes + (unsigned)k_cc * 16u), 0, 0);
#pragma unroll
        for (int i = 0; i < G::NLV; ++i)  // the padded length is a multiple of the stage length: always in range
            prev_[i] = *reinterpret_cast<const u32x4*>(vt_head + (long long)(v_row + i * G::V_RPL) * p.Mpad + n0 + v_cc * 8);
        fetch_idx(t + 1);  // clamped to the last kept row, so any t is fine
    };
    auto stash = [&](int buf) {
        char* s = smem + buf * G::STAGE;
#pragma unroll
        for (int i = 0; i < G::NLK; ++i) *reinterpret_cast<u32x4*>(s + (k_row + i * G::K_RPL) * G::KSTRIDE + k_cc * 16) = prek[i];
#pragma unroll
        for (int i = 0; i < G::NLV; ++i) *reinterpret_cast<u32x4*>(s + AT_KT * G::KSTRIDE + (v_row + i * G::V_RPL) * G::VSTRIDE + v_cc * 16) = prev_[i];
    };

    fetch_idx(0);
    fetch(0);
    stash(0);
    for (int t = 0; t < nstage; ++t) {
        __syncthreads();  // stage t is complete; every wave is done reading stage t-1
        const bool more = t + 1 < nstage;
        if (more) fetch(t + 1);
        const int k0 = t * AT_KT;
        const char* sk = smem + (t & 1) * G::STAGE;
        const char* sv = sk + AT_KT * G::KSTRIDE;
        if (!(causal && k0 > mw0 + 32 * AT_NQ - 1)) {  // otherwise every key of the stage lies after every query of the wave
#pragma unroll 1
            for (int ks = 0; ks < AT_KT / 32; ++ks) {
                const int kmin = k0 + ks * 32;
                if (kmin >= M || (causal && kmin > mw0 + 32 * AT_NQ - 1)) break;
                u32x4 kf[G::NCH];
#pragma unroll
                for (int c = 0; c < G::NCH; ++c) kf[c] = *reinterpret_cast<const u32x4*>(&sk[(ks * 32 + l32) * G::KSTRIDE + c * 32 + half * 16]);
                // V^T fragments of this key subtile: value row dv*32 + l32, keys 16c + 4*half + {0..3} and 16c + 8 + 4*half + {0..3}
                // (contiguous in the quad-exchanged layout)
                u32x4 vf[G::NDV][2];
#pragma unroll
                for (int dv = 0; dv < G::NDV; ++dv)
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        vf[dv][c] = *reinterpret_cast<const u32x4*>(&sv[(dv * 32 + l32) * G::VSTRIDE + (ks * 32 + 16 * c + 8 * half) * 2]);
                    }
#pragma unroll
                for (int qs = 0; qs < AT_NQ; ++qs) {
                    const int qmin = mw0 + qs * 32;
                    if (causal && kmin > qmin + 31) continue;  // every key lies after every query (wave-uniform)
                    f32x16 acc = {0};
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) mma_chunk<T>(acc, kf[c], qf[qs][c]);  // acc[key row][query col]
                    const bool all_allowed = (kmin + 31 < M) && (!causal || kmin + 31 <= qmin);
                    if (!all_allowed) {
                        const int lim = causal ? min(qmin + l32, M - 1) : M - 1;  // last key this lane's query may use
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[r] = (kmin + acc_row(r, lane) <= lim) ? acc[r] : -INFINITY;
                    }
                    // online softmax of the lane's query over its 16 keys + the partner half-wave's 16
                    float t0 = fmaxf(fmaxf(acc[0], acc[1]), acc[2]), t1 = fmaxf(fmaxf(acc[3], acc[4]), acc[5]);
                    float t2 = fmaxf(fmaxf(acc[6], acc[7]), acc[8]), t3 = fmaxf(fmaxf(acc[9], acc[10]), acc[11]);
                    float t4 = fmaxf(fmaxf(acc[12], acc[13]), acc[14]);
                    float tmax = fmaxf(fmaxf(fmaxf(t0, t1), t2), fmaxf(fmaxf(t3, t4), acc[15])) * c2;
                    {  // the other half-wave holds the other 16 keys of the same query: both take the larger maximum
                        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
                        tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                    }
                    // Lazy reference: the running reference only moves when the tile's maximum exceeds it by more than 2^8
                    // (probabilities up to 256 are harmless in binary32 and bf16 keeps its relative precision), so
                    // the rescale below becomes rare instead of happening in almost every tile for some query.
                    const float mn = tmax > mrun[qs] + 8.f ? tmax : mrun[qs];
                    const float ms = mn == -INFINITY ? 0.f : mn;  // nothing allowed so far (padding rows only): keep arguments finite
                    const float corr = __builtin_amdgcn_exp2f(mrun[qs] - ms);
                    float pr[16], s0 = 0.f, s1 = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        pr[r] = __builtin_amdgcn_exp2f(fmaf(acc[r], c2, -ms));
                        if (r & 1) s1 += pr[r]; else s0 += pr[r];
                    }
                    lrun[qs] = fmaf(lrun[qs], corr, s0 + s1);
                    if (__any(mn > mrun[qs])) {  // the reference moved for some query of the wave: rescale what has been summed
#pragma unroll
                        for (int dv = 0; dv < G::NDV; ++dv)
#pragma unroll
                            for (int r = 0; r < 16; ++r) o[qs][dv][r] *= corr;
                    }
                    mrun[qs] = mn;
                    // P^T as B operand: registers 8c .. 8c+7 are this lane's 8 key slots of chunk c
                    u32x4 pb[2];
#pragma unroll
                    for (int c = 0; c < 2; ++c)
                        pb[c] = u32x4{pack_bf16x2_hw(pr[8 * c + 0], pr[8 * c + 1]), pack_bf16x2_hw(pr[8 * c + 2], pr[8 * c + 3]),
                                      pack_bf16x2_hw(pr[8 * c + 4], pr[8 * c + 5]), pack_bf16x2_hw(pr[8 * c + 6], pr[8 * c + 7])};
#pragma unroll
                    for (int dv = 0; dv < G::NDV; ++dv)
#pragma unroll
                        for (int c = 0; c < 2; ++c) mma_chunk<T>(o[qs][dv], vf[dv][c], pb[c]);  // o[value row][query col]
                }
            }
        }
        if (more) stash((t + 1) & 1);
    }

    // normalise and store: lane (query l32, half) holds value rows 8*(r/4) + 4*half + r%4 of every 32-row tile
#pragma unroll
    for (int qs = 0; qs < AT_NQ; ++qs) {
        const float ltot = lrun[qs] + __shfl_xor(lrun[qs], 32);
        const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
        const int m = mw0 + qs * 32 + l32;
        if (m >= M) continue;
        uint16_t* orow = p.O + (long long)m * p.o_ts + (long long)h * p.o_hs;
#pragma unroll
        for (int dv = 0; dv < G::NDV; ++dv)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int c0 = dv * 32 + gq * 8 + half * 4;
                uint2 v;
                v.x = pack_bf16x2_hw(o[qs][dv][gq * 4 + 0] * inv, o[qs][dv][gq * 4 + 1] * inv);
                v.y = pack_bf16x2_hw(o[qs][dv][gq * 4 + 2] * inv, o[qs][dv][gq * 4 + 3] * inv);
                *reinterpret_cast<uint2*>(orow + c0) = v;  // host guarantees 8-byte alignment of every output row
            }
    }
}


// ------------------------------------------------------------------------------------------------
// head_dim 128: the same computation with 64 queries per wave, one wave per SIMD, the overlap written out.
//
// With 32 queries per wave every K and V^T fragment read (16 x 16 bytes per lane and 32-key subtile) feeds one pair of
// MFMA chains, and at full matrix-core rate that alone is the CU's whole LDS bandwidth.  Two query subtiles per wave
// halve it, but their 128 accumulator registers leave room for one wave per SIMD only, so matrix and vector work are
// interleaved by hand.  Stages of keys that need no mask ("hot" stages) run as one branch-free stream of groups of 16
// MFMAs.  With the tiles in the order a(n) = (key subtile n, query subtile 0), b(n) = (n, 1), a(n+1), ..., group k
//   * accumulates the logits of tile k+1          (a chain of 8 MFMAs, in the even slots),
//   * multiplies the probabilities of tile k-1 into its O^T accumulators (8 MFMAs, in the odd slots),
//   * turns the logits of tile k into probabilities (vector work: one element per slot),
// so nothing inside a group waits for anything else inside it, and no two dependent MFMAs stand next to each other.
//
// A branch anywhere inside would let the compiler collect the vector work behind the MFMAs, so a hot stage has none:
// * no rescale: inside hot stages the reference of the exponentials is FROZEN at the value the stages before left
//   (the first stage, and every stage that needs a mask, run the ordinary online softmax with its running reference).
//   This is exact unless a later logit exceeds the frozen reference by more than binary32's exponent range; then a
//   normaliser comes out huge or non-finite, and a workgroup that finds one goes through its keys again with the
//   ordinary softmax in every stage, before it stores anything.
// * no "is there a next stage" test: the next stage's loads go through a descriptor of size zero when there is none.
// * no "is a tile pending" test: the run of hot stages starts with an empty pending tile (logits -inf, probabilities
//   0), carries the pending tile from stage to stage in registers, and finishes the last one after the run.
// The exponential of an element is issued in one slot and added and packed in the next, so that nothing waits on the
// transcendental unit, and every running sum is pinned where it is written (the compiler would otherwise postpone the
// additions and park each exponential in a spare register).  A wave's stages come in three runs -- the first stage,
// the hot stages, the rest -- each a loop of its own, which keeps the register allocator's view of the hot stream clean.
// Stages (128 keys: K rows and V^T rows, 64 KB) are filled by LDS-direct loads that ride on the first key subtile of
// the stage before, with the rows' indices fetched two stages ahead; rows are unpadded and piece p of row r sits at
// position p ^ (r mod 16).  The MFMAs of this file must write ordinary vector registers (their results feed vector
// arithmetic): the file is compiled with -mllvm -amdgpu-mfma-vgpr-form, without which a kernel that may use the whole
// register file gets its MFMA results in the accumulation registers and a copy around every use.
constexpr int AP_THREADS = 256;
constexpr int AP_BQ = 256;                 // queries per workgroup
constexpr int AP_TILE = 128 * 256;         // bytes of a K tile (128 keys x 256 B) and of a V^T tile (128 value rows x 128 keys)
constexpr int AP_STAGE = 2 * AP_TILE;
constexpr int AP_LDS = 2 * AP_STAGE;
constexpr int AP_NLD = 8;                  // 16-byte loads per thread, tile and stage

__device__ __forceinline__ void ap_fence() { __builtin_amdgcn_sched_barrier(0); }
// keeps an addition where it is written: without it the compiler postpones the running sums of the hot stream to the
// point where they are next read, and parks every exponential in a spare register until then
__device__ __forceinline__ void ap_pin(float& x) { asm volatile("" : "+v"(x)); }
// before a barrier that hands a stage over: this wave's LDS-direct loads have landed, its LDS reads have returned
__device__ __forceinline__ void ap_settle() {
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_waitcnt(LGKMCNT0);
}

__global__ __launch_bounds__(AP_THREADS, 1) void kept_attention_pipe_kernel(AttnParams p) {
    using T = bf16_t;
    constexpr int NCH = 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int b = blockIdx.x, x = b % NUM_XCD, w_ = b / NUM_XCD;
    const int slot = w_ / p.n_qblocks;
    int qb = w_ - slot * p.n_qblocks;
    const int h = x * p.heads_per_xcd + slot;
    if (h >= p.H) return;
    const bool causal = (p.flags & LEMO_CAUSAL) != 0;
    if (causal) qb = p.n_qblocks - 1 - qb;
    const int g = (int)(((long long)h * p.H_kv) / p.H);
    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, and known to be: what follows from it stays scalar
    const int M = p.M;
    const float c2 = p.c2;
    const int m0 = qb * AP_BQ, mw0 = m0 + wave * 64;

    // resident operand: this wave's 64 queries (rows gathered through idx), as MFMA B fragments
    u32x4 qf[2][NCH];
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
        const int m = mw0 + qs * 32 + l32;
        const long long tok = m < M ? (p.idx ? (long long)p.idx[m] : (long long)m) : -1;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            qf[qs][c] = u32x4{0u, 0u, 0u, 0u};
            if (tok >= 0) qf[qs][c] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(p.Q + tok * p.q_ts + (long long)h * p.q_hs) + c * 32 + half * 16);
        }
    }

    const int k_last = causal ? min(m0 + AP_BQ, M) - 1 : M - 1;          // last key any wave of the workgroup needs
    const int nstage = k_last / AT_KT + 1;
    const bool active = mw0 < M;                                         // the wave holds at least one query
    const int hot_last = causal ? mw0 : M - 1;                           // a stage whose last key is <= this needs no mask for this wave

    // ---- staging: LDS-direct loads, unit u = i*256 + tid -> row i*16 + tid/16, position tid%16, which holds piece (tid%16) ^ (row%16)
    const int s_row = tid >> 4, s_piece = (tid & 15) ^ (s_row & 15);
    const int k_row_bytes = (int)p.k_ts * 2;
    const u32x4 k_rsrc = raw_rsrc(reinterpret_cast<const char*>(p.K + (long long)g * p.k_hs), (long long)p.k_bytes - (long long)g * p.k_hs * 2);
    const u32x4 v_rsrc = raw_rsrc(reinterpret_cast<const char*>(p.Vt + (long long)g * 128 * p.Mpad), (long long)128 * p.Mpad * 2);
    int v_voff[AP_NLD];
#pragma unroll
    for (int i = 0; i < AP_NLD; ++i) v_voff[i] = (i * 16 + s_row) * p.Mpad * 2 + s_piece * 16;
    unsigned tok[AP_NLD], tok_next[AP_NLD];  // byte offsets of the K rows of the stage being requested / of the one after it
    auto fetch_tok = [&](int t, unsigned (&dst)[AP_NLD]) {  // rows past the end repeat the last kept row (masked later)
        const int n0 = t * AT_KT;
#pragma unroll
        for (int i = 0; i < AP_NLD; ++i) {
            const int n = min(n0 + i * 16 + s_row, M - 1);
            dst[i] = (unsigned)(p.idx ? p.idx[n] : n) * (unsigned)k_row_bytes + (unsigned)s_piece * 16u;
        }
    };
    const unsigned lds_w = lds_offset_of(smem) + (unsigned)wave * 1024u;
    // load n (0..15) of the stage that starts at key n0, into stage buffer `buf`: K rows first, then V^T rows
    auto stage_load_one = [&](int n, int buf, int n0, const u32x4& kd, const u32x4& vd) {
        const unsigned dst = lds_w + (unsigned)buf * AP_STAGE + (unsigned)(n & 7) * 4096u;
        if (n < 8) lds_direct_b128(kd, dst, (int)tok[n & 7]);
        else lds_direct_b128(vd, dst + AP_TILE, v_voff[n & 7], n0 * 2);
    };

    // ---- fragments
    const int f_swz = l32 & 15;
    auto k_frag = [&](const char* sk, int ks, int c) {
        return *reinterpret_cast<const u32x4*>(sk + (ks * 32 + l32) * 256 + (((2 * c + half) ^ f_swz) << 4));
    };
    auto v_frag = [&](const char* sv, int ks, int n) {  // n = dv*2 + c: value rows dv*32.., keys 16c + 8*half .. of the subtile (quad-exchanged order)
        return *reinterpret_cast<const u32x4*>(sv + ((n >> 1) * 32 + l32) * 256 + (((ks * 4 + 2 * (n & 1) + half) ^ f_swz) << 4));
    };

    bool frozen = true;  // workgroup-uniform: which pass this is
    f32x16 o[2][4];      // O^T accumulators: o[qs][dv][r] = element (value row dv*32 + acc_row(r), query column l32 of subtile qs)
    float ltot[2];
    for (;;) {
#pragma unroll
    for (int qs = 0; qs < 2; ++qs)
#pragma unroll
        for (int dv = 0; dv < 4; ++dv) o[qs][dv] = f32x16{0};
    float mrun[2] = {-INFINITY, -INFINITY};  // reference of the exponentials (base-2 units, identical in both half-waves)
    float la[2] = {0.f, 0.f}, lb[2] = {0.f, 0.f};  // this half-wave's share of the normaliser, in two partial sums

    // the ordinary online softmax of one 32 x 32 tile (first stage, stages that need a mask, the repair pass)
    auto slow_tile = [&](int qs, int kmin, const u32x4 (&kfr)[NCH], const u32x4 (&vfr)[8]) {
        const int qmin = mw0 + qs * 32;
        if (causal && kmin > qmin + 31) return;  // every key lies after every query (wave-uniform)
        f32x16 acc = {0};
#pragma unroll
        for (int c = 0; c < NCH; ++c) mma_chunk<T>(acc, kfr[c], qf[qs][c]);  // acc[key row][query col]
        const bool all_allowed = (kmin + 31 < M) && (!causal || kmin + 31 <= qmin);
        if (!all_allowed) {
            const int lim = causal ? min(qmin + l32, M - 1) : M - 1;  // last key this lane's query may use
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = (kmin + acc_row(r, lane) <= lim) ? acc[r] : -INFINITY;
        }
        float t0 = fmaxf(fmaxf(acc[0], acc[1]), acc[2]), t1 = fmaxf(fmaxf(acc[3], acc[4]), acc[5]);
        float t2 = fmaxf(fmaxf(acc[6], acc[7]), acc[8]), t3 = fmaxf(fmaxf(acc[9], acc[10]), acc[11]);
        float t4 = fmaxf(fmaxf(acc[12], acc[13]), acc[14]);
        float tmax = fmaxf(fmaxf(fmaxf(t0, t1), t2), fmaxf(fmaxf(t3, t4), acc[15])) * c2;
        {  // the other half-wave holds the other 16 keys of the same query: both take the larger maximum
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
            tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        }
        // lazy reference: it only moves when the tile's maximum exceeds it by more than 2^8
        const float mn = tmax > mrun[qs] + 8.f ? tmax : mrun[qs];
        const float ms = mn == -INFINITY ? 0.f : mn;  // nothing allowed so far (padding rows only): keep arguments finite
        const float corr = __builtin_amdgcn_exp2f(mrun[qs] - ms);
        float pr[16], s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            pr[r] = __builtin_amdgcn_exp2f(fmaf(acc[r], c2, -ms));
            if (r & 1) s1 += pr[r]; else s0 += pr[r];
        }
        la[qs] = fmaf(la[qs], corr, s0);
        lb[qs] = fmaf(lb[qs], corr, s1);
        if (__any(mn > mrun[qs])) {  // the reference moved for some query of the wave: rescale what has been summed
#pragma unroll
            for (int dv = 0; dv < 4; ++dv)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[qs][dv][r] *= corr;
        }
        mrun[qs] = mn;
        u32x4 pbs[2];  // P^T as B operand: registers 8c .. 8c+7 are this lane's 8 key slots of chunk c
#pragma unroll
        for (int c = 0; c < 2; ++c)
            pbs[c] = u32x4{pack_bf16x2_hw(pr[8 * c + 0], pr[8 * c + 1]), pack_bf16x2_hw(pr[8 * c + 2], pr[8 * c + 3]),
                           pack_bf16x2_hw(pr[8 * c + 4], pr[8 * c + 5]), pack_bf16x2_hw(pr[8 * c + 6], pr[8 * c + 7])};
#pragma unroll
        for (int n = 0; n < 8; ++n) mma_chunk<T>(o[qs][n >> 1], vfr[n], pbs[n & 1]);  // o[value row][query col]
    };

    // ---- state of the hot stream: the pending tile (previous subtile, Q1) -- its logits, the first half of its
    // probabilities, and the V^T fragments of its subtile
    f32x16 S0, S1;
    u32x4 pb[2][2];
    u32x4 kf[NCH], vf[8];
    float nm[2];  // minus the (finite) reference of each query subtile

    fetch_tok(0, tok);
#pragma unroll
    for (int n = 0; n < 16; ++n) stage_load_one(n, 0, 0, k_rsrc, v_rsrc);
    fetch_tok(1, tok);
    fetch_tok(2, tok_next);
    ap_settle();
    // A wave's stages come in three runs: the first stage (ordinary softmax: it sets the reference), then the stages that
    // need no mask (hot), then the rest (masked, or past the wave's last query).  Each run is a loop of its own, so that
    // the register allocator sees the hot stream alone.  Every wave passes one barrier per stage, whichever loop it is in.
    auto stage_head = [&](int t, bool& more, int& k0, int& nbuf, int& n_next, const char*& sk, const char*& sv, u32x4& kd, u32x4& vd) {
        __syncthreads();  // stage t is complete; every wave is done reading stage t-1
        more = t + 1 < nstage;
        k0 = t * AT_KT; nbuf = (t + 1) & 1; n_next = (t + 1) * AT_KT;
        sk = smem + (t & 1) * AP_STAGE;
        sv = sk + AP_TILE;
        // the next stage's loads: through descriptors of size zero when there is no next stage (nothing is read then)
        kd = k_rsrc; vd = v_rsrc;
        kd[2] = more ? kd[2] : 0u;
        vd[2] = more ? vd[2] : 0u;
    };
    auto stage_tail = [&](int t, bool more) {
        ap_settle();
        if (more) {  // after the wait, so that these index loads have the whole next stage to arrive
#pragma unroll
            for (int i = 0; i < AP_NLD; ++i) tok[i] = tok_next[i];
            fetch_tok(t + 3, tok_next);
        }
    };
    auto slow_stage = [&](int t) {
        bool more; int k0, nbuf, n_next; const char* sk; const char* sv; u32x4 kd, vd;
        stage_head(t, more, k0, nbuf, n_next, sk, sv, kd, vd);
            if (more) {
#pragma unroll
                for (int n = 0; n < 16; ++n) stage_load_one(n, nbuf, n_next, k_rsrc, v_rsrc);
            }
            if (active && !(causal && k0 > mw0 + 63)) {  // otherwise every key of the stage lies after every query of the wave
#pragma unroll 1
                for (int ks = 0; ks < 4; ++ks) {
                    const int kmin = k0 + ks * 32;
                    if (kmin >= M || (causal && kmin > mw0 + 63)) break;
                    u32x4 kfr[NCH], vfr[8];
#pragma unroll
                    for (int c = 0; c < NCH; ++c) kfr[c] = k_frag(sk, ks, c);
#pragma unroll
                    for (int n = 0; n < 8; ++n) vfr[n] = v_frag(sv, ks, n);
                    slow_tile(0, kmin, kfr, vfr);
                    slow_tile(1, kmin, kfr, vfr);
                }
            }
        stage_tail(t, more);
    };
    // The stream of exponentials of one tile: its sixteen logits become sixteen probabilities, added to the query's
    // running sums (even elements to la, odd ones to lb) and packed in pairs into the B operand pb[qs] (two chunks of
    // 16 keys).  The exponential of an element is issued in one slot and consumed (added, packed) when the next one is
    // issued, so that no instruction waits on the transcendental unit; the last element is consumed in the first slot of
    // the next group.
    struct Hold { float prev, even; };
    Hold h0{0.f, 0.f}, h1{0.f, 0.f};  // of the Q0 tiles, of the Q1 tiles
    auto consume = [&](Hold& hd, int j, int qs) {  // hd.prev is the exponential of element j (0..15)
        if (j & 1) {
            lb[qs] += hd.prev;
            ap_pin(lb[qs]);
            pb[qs][j >> 3][(j & 7) >> 1] = pack_bf16x2_hw(hd.even, hd.prev);
        } else {
            la[qs] += hd.prev;
            ap_pin(la[qs]);
            hd.even = hd.prev;
        }
    };
    auto feed = [&](Hold& hd, int j, float logit, int qs) {  // element j of the tile
        const float e = __builtin_amdgcn_exp2f(fmaf(logit, c2, nm[qs]));
        if (j > 0) consume(hd, j - 1, qs);
        hd.prev = e;
    };
    // One group of 16 slots.  Tiles in the order a(n) = (subtile n, Q0), b(n) = (subtile n, Q1), a(n+1), ...; group k
    // accumulates the logits of tile k+1 (a chain of 8 MFMAs, even slots), multiplies the probabilities of tile k-1 into
    // its O^T accumulators (8 MFMAs, odd slots, chunk-major so that neighbours differ in accumulator) and turns the logits
    // of tile k into probabilities (one element per slot).  Nothing inside a group depends on anything else inside it.
    //   EVEN(n): logits of b(n) (K fragments of subtile n, each refilled with subtile n+1's right after its use),
    //            product of b(n-1) (V^T fragments of subtile n-1, each refilled with subtile n's right after its use),
    //            exponentials of a(n)
    //   ODD(n):  logits of a(n+1), product of a(n), exponentials of b(n)
    auto group = [&](auto odd_tag, const char* sk, const char* sv, int ks, bool refill_k, auto&& ride) {
        constexpr bool ODD = decltype(odd_tag)::value;
        constexpr int QL = ODD ? 0 : 1;   // query subtile whose logits are accumulated
        constexpr int QP = ODD ? 0 : 1;   // ... whose product is taken: ODD a(n) -> Q0; EVEN b(n-1) -> Q1
        constexpr int QE = ODD ? 1 : 0;   // ... whose exponentials are formed
        f32x16& SL = ODD ? S0 : S1;
        f32x16& SE = ODD ? S1 : S0;
        Hold& hd = ODD ? h1 : h0;
        Hold& hp = ODD ? h0 : h1;         // of the tile whose product is taken: its last exponential is still to be consumed
        SL = f32x16{0};
        ap_fence();
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            mma_chunk<T>(SL, kf[c], qf[QL][c]);
            if (!ODD && refill_k) kf[c] = k_frag(sk, ks + 1, c);
            ride(2 * c);
            if (c == 0) consume(hp, 15, QP);  // completes pb[QP][1], which the group's fifth product MFMA is the first to read
            feed(hd, 2 * c, SE[2 * c], QE);
            ap_fence();
            mma_chunk<T>(o[QP][c & 3], vf[(c & 3) * 2 + (c >> 2)], pb[QP][c >> 2]);
            if (!ODD) vf[(c & 3) * 2 + (c >> 2)] = v_frag(sv, ks, (c & 3) * 2 + (c >> 2));
            ride(2 * c + 1);
            feed(hd, 2 * c + 1, SE[2 * c + 1], QE);
            ap_fence();
        }
    };
    using EvenT = std::integral_constant<bool, false>;
    using OddT = std::integral_constant<bool, true>;
    auto hot_stage = [&](int t) {
        bool more; int k0, nbuf, n_next; const char* sk; const char* sv; u32x4 kd, vd;
        stage_head(t, more, k0, nbuf, n_next, sk, sv, kd, vd);
#pragma unroll
        for (int c = 0; c < NCH; ++c) kf[c] = k_frag(sk, 0, c);
        // the next stage's sixteen loads ride on the stage's first group, one per slot, so that they have the other seven
        // groups' time to land before the stage's closing wait
        auto ride = [&](int n) { stage_load_one(n, nbuf, n_next, kd, vd); };
        auto no_ride = [&](int) {};
        group(OddT{}, sk, sv, 0, false, ride);      // ODD(4t - 1): logits of a(4t), product of a(4t-1), exponentials of b(4t-1)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            group(EvenT{}, sk, sv, ks, ks < 3, no_ride);
            if (ks < 3) group(OddT{}, sk, sv, ks, false, no_ride);
        }
        stage_tail(t, more);
    };
    // hot stages: 1 <= t < t_hot, all keys of the stage at or before the wave's first query (causal) and below M
    const int t_hot = (frozen && active) ? max(1, min(min((hot_last + 1) / AT_KT, M / AT_KT), nstage)) : 1;
    if (nstage > 0) slow_stage(0);
    if (t_hot > 1) {
        // the hot stream starts with empty tiles in flight (logits -inf, probabilities and V^T fragments zero) ...
#pragma unroll
        for (int r = 0; r < 16; ++r) S1[r] = -INFINITY;
        pb[0][0] = pb[0][1] = pb[1][0] = pb[1][1] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int n = 0; n < 8; ++n) vf[n] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int qs = 0; qs < 2; ++qs) nm[qs] = -(mrun[qs] == -INFINITY ? 0.f : mrun[qs]);
        for (int t = 1; t < t_hot; ++t) hot_stage(t);
        // ... and ends by finishing the two that are left: a(last) has its probabilities, b(last) its logits
        consume(h0, 15, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) mma_chunk<T>(o[0][i & 3], vf[(i & 3) * 2 + (i >> 2)], pb[0][i >> 2]);
#pragma unroll
        for (int j = 0; j < 16; ++j) feed(h1, j, S1[j], 1);
        consume(h1, 15, 1);
#pragma unroll
        for (int i = 0; i < 8; ++i) mma_chunk<T>(o[1][i & 3], vf[(i & 3) * 2 + (i >> 2)], pb[1][i >> 2]);
    }
    for (int t = t_hot; t < nstage; ++t) slow_stage(t);

    // the normaliser of each query; a value that is not finite or has come close to the end of binary32's range means that
    // a frozen reference was overtaken by too much: then everything is done again with the ordinary softmax throughout
    bool bad = false;
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
        const float l = la[qs] + lb[qs];
        ltot[qs] = l + __shfl_xor(l, 32);
        bad |= !(ltot[qs] < 0x1p100f);
    }
    if (!frozen || !__syncthreads_or(bad)) break;
    frozen = false;
    }

    // normalise and store: lane (query l32, half) holds value rows 8*(r/4) + 4*half + r%4 of every 32-row tile
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
        const float inv = ltot[qs] > 0.f ? 1.f / ltot[qs] : 0.f;
        const int m = mw0 + qs * 32 + l32;
        if (m >= M) continue;
        uint16_t* orow = p.O + (long long)m * p.o_ts + (long long)h * p.o_hs;
#pragma unroll
        for (int dv = 0; dv < 4; ++dv)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int c0 = dv * 32 + gq * 8 + half * 4;
                uint2 v;
                v.x = pack_bf16x2_hw(o[qs][dv][gq * 4 + 0] * inv, o[qs][dv][gq * 4 + 1] * inv);
                v.y = pack_bf16x2_hw(o[qs][dv][gq * 4 + 2] * inv, o[qs][dv][gq * 4 + 3] * inv);
                *reinterpret_cast<uint2*>(orow + c0) = v;  // host guarantees 8-byte alignment of every output row
            }
    }
}

template <int D>
static int launch_attn_t(AttnParams p, hipStream_t st) {
    using G = AGeo<D>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&kept_attention_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    p.heads_per_xcd = (p.H + NUM_XCD - 1) / NUM_XCD;
#if LEMO_AT_PIPE
    if (D == 128) {
        static std::once_flag once2;
        static hipError_t attr_err2 = hipSuccess;
        std::call_once(once2, [] {
            attr_err2 = hipFuncSetAttribute(reinterpret_cast<const void*>(&kept_attention_pipe_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, AP_LDS);
        });
        if (attr_err2 != hipSuccess) return (int)attr_err2;
        p.n_qblocks = (p.M + AP_BQ - 1) / AP_BQ;
        hipLaunchKernelGGL(kept_attention_pipe_kernel, dim3((unsigned)(NUM_XCD * p.heads_per_xcd * p.n_qblocks)), dim3(AP_THREADS), AP_LDS, st, p);
        return (int)hipGetLastError();
    }
#endif
    p.n_qblocks = (p.M + AT_BQ - 1) / AT_BQ;
    hipLaunchKernelGGL((kept_attention_kernel<D>), dim3((unsigned)(NUM_XCD * p.heads_per_xcd * p.n_qblocks)), dim3(AT_THREADS), G::LDS, st, p);
    return (int)hipGetLastError();
}

// V [S,H_kv,d] element strides v_ts, v_hs; workspace holds V^T of the kept rows: H_kv * d * Mpad bf16
int launch_kept_attention(const void* Q, const void* K, const void* V, long long S, int H, int H_kv, int d, long long q_ts, long long q_hs,
                          long long k_ts, long long k_hs, long long v_ts, long long v_hs, const int* idx, long long M, float c2,
                          unsigned flags, void* O, long long o_ts, long long o_hs, void* workspace, hipStream_t st) {
    if (M == 0) return 0;
    const int Mpad = (int)((M + AT_MPAD - 1) / AT_MPAD) * AT_MPAD;
    uint16_t* Vt = static_cast<uint16_t*>(workspace);
    hipLaunchKernelGGL(gather_vt_kernel, dim3((unsigned)(Mpad / 64), (unsigned)H_kv), dim3(256), 0, st, static_cast<const uint16_t*>(V), v_ts, v_hs,
                       idx, (int)M, Mpad, d, Vt);
    int rc = (int)hipGetLastError();
    if (rc) return rc;
    AttnParams p{};
    p.Q = static_cast<const uint16_t*>(Q);
    p.K = static_cast<const uint16_t*>(K);
    p.Vt = Vt;
    p.idx = idx;
    p.O = static_cast<uint16_t*>(O);
    p.M = (int)M;
    p.Mpad = Mpad;
    p.H = H;
    p.H_kv = H_kv;
    p.q_ts = q_ts; p.q_hs = q_hs; p.k_ts = k_ts; p.k_hs = k_hs; p.o_ts = o_ts; p.o_hs = o_hs;
    p.q_bytes = (unsigned)(((S - 1) * q_ts + (long long)(H - 1) * q_hs + d) * 2);
    p.k_bytes = (unsigned)(((S - 1) * k_ts + (long long)(H_kv - 1) * k_hs + d) * 2);
    p.c2 = c2;
    p.flags = flags;
    return d == 128 ? launch_attn_t<128>(p, st) : launch_attn_t<64>(p, st);
}

}  // namespace lemo
