// Token informativeness (Sec. 4.2, Eq. 1 with the head mean of Eq. 2) on gfx950.
//
// Column sums of softmax(Q K^T) need every row's FINAL normaliser, so Q K^T is swept twice and the
// S x S matrix is never stored (Sec. 4.3: derived online, memory linear in S):
//
//   sweep 1  rowstats_kernel   per (head, 256-query block): keys stream through LDS, the block's
//                              queries stay in registers; an online max/sum per query gives the
//                              base-2 log-sum-exp  lse2[h][i].
//   sweep 2  colsum_kernel     per (head, <=256-key block of one segment): the block's keys stay in
//                              registers, queries stream through LDS; p = exp2(s*c2 - lse2[i]) is
//                              added into per-lane column accumulators -- each column is owned by one
//                              workgroup, so there are no atomics and the result is deterministic.
//   reduce   head_mean_kernel  scores[j] = (1/H) sum_h (colsum - [exclude self] diag), fixed order.
//
// Both sweeps compute 32x32 logit tiles with MFMA (bf16: 32x32x16; fp32: 32x32x2, a true binary32
// contraction).  The product is oriented so that the axis being reduced runs along the accumulator
// REGISTERS of a lane and the axis being kept runs along LANES: sweep 1 computes K.Q^T (lane = query),
// sweep 2 computes Q.K^T (lane = key).  Row and column statistics are then plain in-register chains
// with one cross-lane step at the very end.
#include "lemo_common.hpp"

namespace lemo {

constexpr int SC_THREADS = 256;  // 4 waves
constexpr int SC_WAVES = 4;
constexpr int SC_RES = 64;       // resident rows per wave (two 32-row MFMA subtiles)
constexpr int SC_BLOCK = SC_WAVES * SC_RES;  // 256 resident rows per workgroup

template <typename T, int D> struct Geo {
    static constexpr int ROWB = D * (int)sizeof(T);  // bytes per head row
    static constexpr int NCH = ROWB / 32;            // MFMA chunks per row
    static constexpr int CPR = ROWB / 16;            // 16-byte pieces per row
    static constexpr int STRIDE = ROWB + 16;         // LDS row pitch: +16 B so that 16 consecutive rows hit 16 distinct bank groups
    static constexpr int TILE = ROWB > 256 ? 32 : 64;  // streamed rows per LDS stage
    static constexpr int NSUB = TILE / 32;           // 32-row MFMA subtiles per stage
    static constexpr int NLOAD = TILE * CPR / SC_THREADS;  // 16-byte global loads per thread per stage
    static constexpr int MIN_WG = ROWB > 256 ? 1 : 2;  // workgroups per CU the register budget is set for
    static_assert(TILE * CPR % SC_THREADS == 0, "tile must split evenly over the workgroup");
};

// block index -> (head, block-within-head).  Workgroup b runs on die b % 8; a die gets a contiguous
// range of heads (so the query heads of one GQA group share the die's L2 with their KV head) and
// walks one head's blocks in order before moving to its next head.
__device__ __forceinline__ bool decode_block(int nblk, int heads_per_xcd, int H, int& h, int& blk) {
    int b = blockIdx.x;
    int x = b % NUM_XCD, w = b / NUM_XCD;
    int slot = w / nblk;
    blk = w - slot * nblk;
    h = x * heads_per_xcd + slot;
    return h < H;
}

// 16-byte piece `c` of row `row` of a [rows, heads, D] tensor, zero beyond `nrows`
template <typename T>
__device__ __forceinline__ uint4 load_piece(const T* base, long long tok_stride, long long head_off, int row, int nrows, int byte_off) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < nrows) v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(base + (long long)row * tok_stride + head_off) + byte_off);
    return v;
}

// ------------------------------------------------------------------------------------------------
// Sweep 1: base-2 log-sum-exp of every query row.
// ------------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(SC_THREADS, (Geo<T, D>::MIN_WG)) void rowstats_kernel(ScoreParams p) {
    using G = Geo<T, D>;
    __shared__ __attribute__((aligned(16))) char sK[2][G::TILE * G::STRIDE];

    int h, qb;
    if (!decode_block(p.n_query_blocks, p.heads_per_xcd, p.H, h, qb)) return;
    const bool causal = (p.flags & LEMO_CAUSAL) != 0;
    if (causal) qb = p.n_query_blocks - 1 - qb;  // late query blocks see the most keys: start them first
    const int g = (int)(((long long)h * p.H_kv) / p.H);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const T* Qb = static_cast<const T*>(p.Q);
    const T* Kb = static_cast<const T*>(p.K);
    const long long q_off = (long long)h * p.q_hs, k_off = (long long)g * p.k_hs;
    const int S = p.S;
    const int q0 = qb * SC_BLOCK;     // first query of the workgroup
    const int qw0 = q0 + wave * SC_RES;  // first query of this wave

    // resident operand: this wave's 64 queries as MFMA B fragments
    uint4 qf[2][G::NCH];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
        for (int c = 0; c < G::NCH; ++c) qf[qt][c] = load_piece(Qb, p.q_ts, q_off, qw0 + qt * 32 + l32, S, c * 32 + half * 16);

    const int my_q[2] = {qw0 + l32, qw0 + 32 + l32};  // the two queries this lane keeps statistics for
    float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.f, 0.f};

    // key tiles [0, ntile): under a causal mask only keys up to the block's last query matter
    const int q_last = min(q0 + SC_BLOCK, S) - 1;
    const int ntile = (causal ? q_last : S - 1) / G::TILE + 1;

    uint4 pre[G::NLOAD];
    auto fetch = [&](int t) {
#pragma unroll
        for (int i = 0; i < G::NLOAD; ++i) {
            int piece = i * SC_THREADS + tid, row = piece / G::CPR, cc = piece % G::CPR;
            pre[i] = load_piece(Kb, p.k_ts, k_off, t * G::TILE + row, S, cc * 16);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < G::NLOAD; ++i) {
            int piece = i * SC_THREADS + tid, row = piece / G::CPR, cc = piece % G::CPR;
            *reinterpret_cast<uint4*>(&sK[buf][row * G::STRIDE + cc * 16]) = pre[i];
        }
    };

    fetch(0);
    stash(0);
    for (int t = 0; t < ntile; ++t) {
        __syncthreads();  // stage t is complete; every wave is done reading stage t-1
        const bool more = t + 1 < ntile;
        if (more) fetch(t + 1);
        const int k0 = t * G::TILE;
        // wave-uniform classification of this 64x64 tile against the wave's queries [qw0, qw0+63]
        const bool skip = causal && k0 > qw0 + SC_RES - 1;  // every key lies after every query
        const bool clean = causal ? (k0 + G::TILE - 1 <= qw0) : (k0 + G::TILE <= S);
        if (!skip) {
            const char* sbuf = sK[t & 1];
#pragma unroll
            for (int ks = 0; ks < G::NSUB; ++ks) {
                uint4 kf[G::NCH];
#pragma unroll
                for (int c = 0; c < G::NCH; ++c) kf[c] = *reinterpret_cast<const uint4*>(&sbuf[(ks * 32 + l32) * G::STRIDE + c * 32 + half * 16]);
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    f32x16 acc = {0};
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) mma_chunk<T>(acc, kf[c], qf[qt][c]);  // acc[key row][query col]
                    if (clean) {
                        float tmax = acc[0];
#pragma unroll
                        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, acc[r]);
                        const float mn = fmaxf(m[qt], tmax * p.c2);
                        float sum = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(acc[r], p.c2, -mn));
                        l[qt] = fmaf(l[qt], __builtin_amdgcn_exp2f(m[qt] - mn), sum);
                        m[qt] = mn;
                    } else {
                        // key j may be used by query i iff j <= lim(i): i itself under the causal mask, S-1 otherwise
                        const int lim = causal ? my_q[qt] : S - 1;
                        float tmax = -INFINITY;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = k0 + ks * 32 + acc_row(r, lane);
                            acc[r] = key <= lim ? acc[r] * p.c2 : -INFINITY;
                            tmax = fmaxf(tmax, acc[r]);
                        }
                        const float mn = fmaxf(m[qt], tmax);
                        const float ms = mn == -INFINITY ? 0.f : mn;  // nothing seen yet: keep exp2 arguments finite
                        float sum = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(acc[r] - ms);
                        l[qt] = fmaf(l[qt], __builtin_amdgcn_exp2f(m[qt] - ms), sum);
                        m[qt] = mn;
                    }
                }
            }
        }
        if (more) stash((t + 1) & 1);
    }

    // the two half-waves hold disjoint key rows of the same queries: merge, then lse2 = m + log2(l)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const float mo = __shfl_xor(m[qt], 32), lo = __shfl_xor(l[qt], 32);
        const float mt = fmaxf(m[qt], mo);
        const float ms = mt == -INFINITY ? 0.f : mt;
        const float lt = l[qt] * __builtin_amdgcn_exp2f(m[qt] - ms) + lo * __builtin_amdgcn_exp2f(mo - ms);
        if (half == 0 && my_q[qt] < S) p.lse2[(size_t)h * S + my_q[qt]] = mt + __builtin_amdgcn_logf(lt);
    }
}

// ------------------------------------------------------------------------------------------------
// Sweep 2: column sums (and the diagonal) of the probabilities, one key block per workgroup.
// ------------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(SC_THREADS, (Geo<T, D>::MIN_WG)) void colsum_kernel(ScoreParams p) {
    using G = Geo<T, D>;
    __shared__ __attribute__((aligned(16))) char sQ[2][G::TILE * G::STRIDE];
    __shared__ __attribute__((aligned(16))) float sL[2][G::TILE];

    int h, kb;
    if (!decode_block(p.n_key_blocks, p.heads_per_xcd, p.H, h, kb)) return;
    const bool causal = (p.flags & LEMO_CAUSAL) != 0;
    const int S = p.S;
    // key block -> (segment, block inside the segment); blocks never straddle a segment boundary
    const int seg = kb / p.blocks_per_seg, bis = kb - seg * p.blocks_per_seg;
    const long long seg0 = (long long)seg * p.L;
    const long long key0_ll = seg0 + (long long)bis * SC_BLOCK;
    if (key0_ll >= S) return;
    const int key0 = (int)key0_ll;
    const int kend = (int)min((long long)S, min(seg0 + p.L, key0_ll + SC_BLOCK));  // exclusive

    const int g = (int)(((long long)h * p.H_kv) / p.H);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const T* Qb = static_cast<const T*>(p.Q);
    const T* Kb = static_cast<const T*>(p.K);
    const long long q_off = (long long)h * p.q_hs, k_off = (long long)g * p.k_hs;
    const float* lse = p.lse2 + (size_t)h * S;
    const int kw0 = key0 + wave * SC_RES;  // first key of this wave

    // resident operand: this wave's 64 keys as MFMA B fragments (zero beyond the block's end)
    uint4 kf[2][G::NCH];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int c = 0; c < G::NCH; ++c) kf[kt][c] = load_piece(Kb, p.k_ts, k_off, kw0 + kt * 32 + l32, kend, c * 32 + half * 16);

    const int my_k[2] = {kw0 + l32, kw0 + 32 + l32};  // the two columns this lane accumulates
    float col[2] = {0.f, 0.f}, dg[2] = {0.f, 0.f};

    // query tiles run from the end of the sequence DOWN to the first tile that can see this block, so
    // that all key blocks of a head walk the same query rows at about the same time (shared through L2)
    const int t_hi = (S - 1) / G::TILE;
    const int t_lo = causal ? key0 / G::TILE : 0;

    uint4 pre[G::NLOAD];
    float pre_l = 0.f;
    auto fetch = [&](int t) {
#pragma unroll
        for (int i = 0; i < G::NLOAD; ++i) {
            int piece = i * SC_THREADS + tid, row = piece / G::CPR, cc = piece % G::CPR;
            pre[i] = load_piece(Qb, p.q_ts, q_off, t * G::TILE + row, S, cc * 16);
        }
        if (tid < G::TILE) {
            int q = t * G::TILE + tid;
            pre_l = q < S ? lse[q] : INFINITY;  // rows beyond S: exp2(-inf) = 0, they add nothing
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < G::NLOAD; ++i) {
            int piece = i * SC_THREADS + tid, row = piece / G::CPR, cc = piece % G::CPR;
            *reinterpret_cast<uint4*>(&sQ[buf][row * G::STRIDE + cc * 16]) = pre[i];
        }
        if (tid < G::TILE) sL[buf][tid] = pre_l;
    };

    fetch(t_hi);
    stash(0);
    int buf = 0;
    for (int t = t_hi; t >= t_lo; --t, buf ^= 1) {
        __syncthreads();
        const bool more = t > t_lo;
        if (more) fetch(t - 1);
        const int i0 = t * G::TILE;
        const bool on_diag = i0 <= kw0 + SC_RES - 1 && i0 + G::TILE - 1 >= kw0;  // tile meets the diagonal band of this wave
        const bool skip = causal && i0 + G::TILE - 1 < kw0;                     // every query lies before every key
        if (!skip) {
            const char* sbuf = sQ[buf];
            const float* lbuf = sL[buf];
#pragma unroll
            for (int qs = 0; qs < G::NSUB; ++qs) {
                uint4 qf[G::NCH];
#pragma unroll
                for (int c = 0; c < G::NCH; ++c) qf[c] = *reinterpret_cast<const uint4*>(&sbuf[(qs * 32 + l32) * G::STRIDE + c * 32 + half * 16]);
                float nl[16];  // -lse2 of the 16 query rows this lane sees
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const f32x4 v = *reinterpret_cast<const f32x4*>(&lbuf[qs * 32 + gq * 8 + half * 4]);
                    nl[gq * 4 + 0] = -v[0]; nl[gq * 4 + 1] = -v[1]; nl[gq * 4 + 2] = -v[2]; nl[gq * 4 + 3] = -v[3];
                }
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) {
                    f32x16 acc = {0};
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) mma_chunk<T>(acc, qf[c], kf[kt][c]);  // acc[query row][key col]
                    float part = 0.f;
                    if (!on_diag) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) part += __builtin_amdgcn_exp2f(fmaf(acc[r], p.c2, nl[r]));
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int q = i0 + qs * 32 + acc_row(r, lane);
                            float pr = __builtin_amdgcn_exp2f(fmaf(acc[r], p.c2, nl[r]));
                            if (causal && q < my_k[kt]) pr = 0.f;
                            if (q == my_k[kt]) dg[kt] = pr;
                            part += pr;
                        }
                    }
                    col[kt] += part;
                }
            }
        }
        if (more) stash(buf ^ 1);
    }

#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
        const float c = col[kt] + __shfl_xor(col[kt], 32);
        const float dd = dg[kt] + __shfl_xor(dg[kt], 32);
        if (half == 0 && my_k[kt] < kend) {
            p.colsum[(size_t)h * S + my_k[kt]] = c;
            p.diag[(size_t)h * S + my_k[kt]] = dd;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Head mean (Eq. 2's 1/N_head) with the self term optionally removed (Eq. 1's i != j).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void head_mean_kernel(const float* __restrict__ colsum, const float* __restrict__ diag,
                                                        float* __restrict__ scores, int S, int H, int exclude_self) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= S) return;
    float acc = 0.f;
    for (int h = 0; h < H; ++h) {
        float v = colsum[(size_t)h * S + j];
        if (exclude_self) v -= diag[(size_t)h * S + j];
        acc += v;
    }
    scores[j] = acc / (float)H;
}

// which: bit 0 = sweep 1 (row statistics), bit 1 = sweep 2 (column sums), bit 2 = head mean
template <typename T, int D>
static int launch_score_t(const ScoreParams& p, int which, hipStream_t st) {
    const unsigned g1 = (unsigned)(NUM_XCD * p.heads_per_xcd * p.n_query_blocks);
    const unsigned g2 = (unsigned)(NUM_XCD * p.heads_per_xcd * p.n_key_blocks);
    if (which & 1) hipLaunchKernelGGL((rowstats_kernel<T, D>), dim3(g1), dim3(SC_THREADS), 0, st, p);
    if (which & 2) hipLaunchKernelGGL((colsum_kernel<T, D>), dim3(g2), dim3(SC_THREADS), 0, st, p);
    if (which & 4)
        hipLaunchKernelGGL(head_mean_kernel, dim3((p.S + 255) / 256), dim3(256), 0, st, p.colsum, p.diag, p.scores, p.S, p.H,
                           (p.flags & LEMO_EXCLUDE_SELF) ? 1 : 0);
    return (int)hipGetLastError();
}

int launch_score(const ScoreParams& p_in, lemo_dtype_t dt, int d, int which, hipStream_t st) {
    ScoreParams p = p_in;
    p.heads_per_xcd = (p.H + NUM_XCD - 1) / NUM_XCD;
    p.n_query_blocks = (p.S + SC_BLOCK - 1) / SC_BLOCK;
    // Key blocks never straddle a segment boundary.  Segments shorter than a block are grouped: a block
    // then covers as many WHOLE segments as fit, which is the same as working with that longer unit.
    long long Leff = p.L;
    if (Leff < SC_BLOCK) Leff = (SC_BLOCK / Leff) * Leff;
    if (Leff > p.S) Leff = p.S;
    p.L = (int)Leff;
    p.blocks_per_seg = (int)((Leff + SC_BLOCK - 1) / SC_BLOCK);
    const long long nseg = ((long long)p.S + Leff - 1) / Leff;
    p.n_key_blocks = (int)(nseg * p.blocks_per_seg);
    if (which == 4) return launch_score_t<float, 64>(p, which, st);  // the head mean has no dtype
    if (dt == LEMO_BF16 && d == 128) return launch_score_t<bf16_t, 128>(p, which, st);
    if (dt == LEMO_BF16 && d == 64) return launch_score_t<bf16_t, 64>(p, which, st);
    if (dt == LEMO_F32 && d == 128) return launch_score_t<float, 128>(p, which, st);
    if (dt == LEMO_F32 && d == 64) return launch_score_t<float, 64>(p, which, st);
    return (int)hipErrorInvalidValue;
}

}  // namespace lemo
