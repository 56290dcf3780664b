// Token informativeness (Sec. 4.2, Eq. 1 with the head mean of Eq. 2) on gfx950.
//
// Column sums of softmax(Q K^T) need every row's FINAL normaliser, so Q K^T is swept twice and the
// S x S matrix is never stored (memory linear in S, as Sec. 4.3 requires of the scoring kernel):
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
//
// Per logit the matrix core spends as many cycles (2*d flops) as the vector ALU does on fma + exp2 + add,
// so the two must run at the same time.  Tiles that need no masking go through a software pipeline:
// while the MFMA chain of tile n runs, the exp/sum work of tile n-1 (kept in a "carry" accumulator)
// is issued between the MFMAs; the instruction order is pinned with scheduling-group barriers.
#include <mutex>

#include "lemo_common.hpp"

namespace lemo {

// resident subtiles per wave for bf16, d = 128 (2 or 4; see Geo)
#ifndef LEMO_NRT_BF16_128
#define LEMO_NRT_BF16_128 2
#endif

#ifndef LEMO_SC_WAVES
#define LEMO_SC_WAVES 4
#endif
constexpr int SC_WAVES = LEMO_SC_WAVES;
constexpr int SC_THREADS = 64 * SC_WAVES;

// Geometry of one instantiation.  NRT = 32-row MFMA subtiles of the RESIDENT operand a wave keeps in registers:
//   NRT = 2  64 resident rows per wave, 256 per workgroup, two workgroups per CU (two waves per SIMD)
//   NRT = 4  128 resident rows per wave, 512 per workgroup, one workgroup per CU: every LDS fragment read feeds
//            four MFMA chains instead of two (half the LDS traffic per flop), but a SIMD then has no second wave
//            to run while the first waits at a barrier or on LDS
// Measured on the 32K-token bf16 d=128 layer: NRT = 2 4.20 / 4.25 ms (sweep 1 / sweep 2), NRT = 4 4.45 / 4.57 ms; with
// the stages filled by LDS-direct loads NRT = 2 4.06 ms (sweep 1) against 4.93 ms for NRT = 4 (4.23 ms when NRT = 4 is
// squeezed into half the register file for two workgroups per CU).
template <typename T, int D, int NRT_> struct Geo {
    static constexpr int NRT = NRT_;
    static constexpr int RES = 32 * NRT;             // resident rows per wave
    static constexpr int BLOCK = SC_WAVES * RES;     // resident rows per workgroup
    static constexpr int ROWB = D * (int)sizeof(T);  // bytes per head row
    static constexpr int NCH = ROWB / 32;            // MFMA chunks per row
    static constexpr int CPR = ROWB / 16;            // 16-byte pieces per row
    // LDS rows are not padded (LDS-direct loads fill consecutive bytes): piece p of row r sits at position p ^ swz(r),
    // which spreads any one piece of 16 consecutive rows over 16 distinct bank groups
    static constexpr int STRIDE = ROWB;
    __device__ static constexpr int swz(int row) { return CPR >= 16 ? (row & 15) : ((row >> 1) & (CPR - 1)); }
    // byte offset inside a stage of the fragment piece (chunk c, half) of row `row`
    __device__ static constexpr int frag(int row, int c, int half) { return row * ROWB + (((2 * c + half) ^ swz(row)) << 4); }
    static constexpr int TILE = ROWB > 256 ? 64 : 128; // streamed rows per LDS stage (two stages; long enough to hide a global load)
    static constexpr int NSUB = TILE / 32;           // 32-row MFMA subtiles per stage
    static constexpr int NLOAD = TILE * CPR / SC_THREADS;  // 16-byte global loads per thread per stage
    static constexpr int ROWS_PER_LOAD = SC_THREADS / CPR; // rows covered by one load of the whole workgroup
    static constexpr int STAGE_BYTES = TILE * STRIDE;
    static constexpr int LDS_ROWSTATS = 2 * STAGE_BYTES;
    static constexpr int LDS_COLSUM = 2 * STAGE_BYTES + 2 * TILE * (int)sizeof(float);
    static constexpr int MIN_WG = (ROWB > 256 || NRT > 2 || SC_WAVES > 4) ? 1 : 2;  // workgroups per CU the register budget is set for
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

// 16 bytes at byte offset `byte_off` of row `row` of a [rows, heads, D] tensor, zero beyond `nrows`
template <typename T>
__device__ __forceinline__ u32x4 load_piece(const T* base, long long tok_stride, long long head_off, int row, int nrows, int byte_off) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (row < nrows) v = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(base + (long long)row * tok_stride + head_off) + byte_off);
    return v;
}

// Stage loads: LDS-direct (no staging registers, no LDS write instructions).  Unit u = i * SC_THREADS + tid of a stage is
// its LDS bytes [16u, 16u + 16) = row u / CPR, position u % CPR; the lane fetches the piece that belongs there.  The
// loads go through a buffer descriptor rebuilt per stage (wave-uniform base = first row of the stage, size = bytes up to
// the end of the last valid row), so pieces of rows beyond the end of the tensor arrive as zeros.
template <typename G>
__device__ __forceinline__ void stage_offsets(int (&voff)[G::NLOAD], int row_bytes, int tid) {
#pragma unroll
    for (int i = 0; i < G::NLOAD; ++i) {
        const int u = i * SC_THREADS + tid, row = u / G::CPR, piece = (u % G::CPR) ^ G::swz(row);
        voff[i] = row * row_bytes + piece * 16;
    }
}
// descriptor of the stage that starts at row0 (length zero when !live: its loads then fetch nothing)
template <typename G>
__device__ __forceinline__ u32x4 stage_desc(const char* head, int row_bytes, int row0, int nrows, bool live) {
    const long long span = (long long)(nrows - row0 - 1) * row_bytes + G::ROWB;  // bytes from row0 to the end of row nrows-1
    return raw_rsrc(head + (long long)row0 * row_bytes, !live ? 0 : span > 0x7fffffffLL ? 0x7fffffffLL : span);
}
// lds_stage: LDS byte offset of the stage plus 1024 * (wave index), wave-uniform
template <typename G>
__device__ __forceinline__ void stage_load(const int (&voff)[G::NLOAD], u32x4 rsrc, unsigned lds_stage) {
#pragma unroll
    for (int i = 0; i < G::NLOAD; ++i) lds_direct_b128(rsrc, lds_stage + i * (SC_THREADS * 16), voff[i]);
}
// the share of pipeline slot `ti` of `nslots`: issued one slot at a time, the loads do not queue up behind each other
// in the CU's vector-memory pipe (16 cycles per 1 KB instruction) while the wave stands still
template <typename G>
__device__ __forceinline__ void stage_load_slot(const int (&voff)[G::NLOAD], u32x4 rsrc, unsigned lds_stage, int ti, int nslots) {
#pragma unroll
    for (int i = 0; i < G::NLOAD; ++i)
        if (i >= ti * G::NLOAD / nslots && i < (ti + 1) * G::NLOAD / nslots) lds_direct_b128(rsrc, lds_stage + i * (SC_THREADS * 16), voff[i]);
}
// before the barrier that ends a stage: this wave's loads of the next stage have landed, its reads of this one returned
__device__ __forceinline__ void stage_settle() {
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_waitcnt(LGKMCNT0);
}
// the NCH fragments of one 32-row subtile of a stage
template <typename G>
__device__ __forceinline__ void read_frags(u32x4 (&f)[G::NCH], const char* sbuf, int sub, int l32, int half) {
#pragma unroll
    for (int c = 0; c < G::NCH; ++c) f[c] = *reinterpret_cast<const u32x4*>(&sbuf[G::frag(sub * 32 + l32, c, half)]);
}

// The scheduler may not move anything across this point: the source order of the pipeline slots below
// (a share of the carried tile's vector work, then the next MFMAs) is the order the wave issues them in.
__device__ __forceinline__ void slot_fence() { __builtin_amdgcn_sched_barrier(0); }

// ------------------------------------------------------------------------------------------------
// Sweep 1: base-2 log-sum-exp of every query row.
// ------------------------------------------------------------------------------------------------

// Online softmax update of one query's (m, l) with the 16 logits a lane holds of one tile, cut into NS
// slices so that it can be issued between the MFMAs of the next tile.  `raw` are unscaled dot products
// (-inf = masked, or "no tile at all"); everything stays finite-safe when all inputs so far are -inf.
struct RowStat {
    float mn, ms, sum0, sum1, corr;
};
template <int NS>
__device__ __forceinline__ void rowstat_slice(int c, const f32x16& raw, float c2, float m, RowStat& st) {
    if (c == 0) {
        float t0 = fmaxf(fmaxf(raw[0], raw[1]), raw[2]);  // v_max3_f32
        float t1 = fmaxf(fmaxf(raw[3], raw[4]), raw[5]);
        float t2 = fmaxf(fmaxf(raw[6], raw[7]), raw[8]);
        float t3 = fmaxf(fmaxf(raw[9], raw[10]), raw[11]);
        float t4 = fmaxf(fmaxf(raw[12], raw[13]), raw[14]);
        t0 = fmaxf(fmaxf(t0, t1), t2);
        t3 = fmaxf(fmaxf(t3, t4), raw[15]);
        st.mn = fmaxf(m, fmaxf(t0, t3) * c2);
        st.ms = st.mn == -INFINITY ? 0.f : st.mn;  // nothing seen yet: keep the exp2 arguments finite
        st.corr = __builtin_amdgcn_exp2f(m - st.ms);
        st.sum0 = 0.f;
        st.sum1 = 0.f;
    } else {
        const int lo = (c - 1) * 16 / (NS - 1), hi = c * 16 / (NS - 1);
#pragma unroll
        for (int r = lo; r < hi; ++r) {
            const float e = __builtin_amdgcn_exp2f(fmaf(raw[r], c2, -st.ms));
            if (r & 1) st.sum1 += e; else st.sum0 += e;
        }
    }
}
__device__ __forceinline__ void rowstat_finish(const RowStat& st, float& m, float& l) {
    l = fmaf(l, st.corr, st.sum0 + st.sum1);
    m = st.mn;
}
// the whole update at once (masked tiles, pipeline drain)
__device__ __forceinline__ void rowstat_update(const f32x16& raw, float c2, float& m, float& l) {
    RowStat st;
#pragma unroll
    for (int c = 0; c < 8; ++c) rowstat_slice<8>(c, raw, c2, m, st);
    rowstat_finish(st, m, l);
}
// The same sum against a FROZEN reference m (no maximum search, no rescaling): exact for any finite m as long as
// nothing overflows, which the caller checks at the end.  Slice c of NS covers elements [c*16/NS, (c+1)*16/NS).
template <int NS>
__device__ __forceinline__ void rowstat_frozen_slice(int c, const f32x16& raw, float c2, float neg_m, float& s0, float& s1) {
    const int lo = c * 16 / NS, hi = (c + 1) * 16 / NS;
#pragma unroll
    for (int r = lo; r < hi; ++r) {
        const float e = __builtin_amdgcn_exp2f(fmaf(raw[r], c2, neg_m));
        if (r & 1) s1 += e; else s0 += e;
    }
}

// First pass, frozen reference: the running maximum is tracked through the first stage (and through every masked
// tile); from then on unmasked tiles add exp2(s*c2 - m) against the maximum frozen at that point, which saves the
// maximum search and the rescale.  Should a later logit exceed the frozen reference by more than the binary32
// exponent range the sum overflows and lse2 comes out non-finite.  A workgroup that finds such a row among its own
// (normally none does) goes through its keys a second time with the running maximum everywhere, before it stores
// anything: no second launch, no extra traffic when there is nothing to repair.
template <typename T, int D, int NRT>
__global__ __launch_bounds__(SC_THREADS, (Geo<T, D, NRT>::MIN_WG)) void rowstats_kernel(ScoreParams p) {
    using G = Geo<T, D, NRT>;
    extern __shared__ __attribute__((aligned(16))) char smem[];

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
    const float c2 = p.c2;
    const int q0 = qb * G::BLOCK;        // first query of the workgroup
    const int qw0 = q0 + wave * G::RES;  // first query of this wave

    // resident operand: this wave's queries as MFMA B fragments
    u32x4 qf[NRT][G::NCH];
#pragma unroll
    for (int qt = 0; qt < NRT; ++qt)
#pragma unroll
        for (int c = 0; c < G::NCH; ++c) qf[qt][c] = load_piece(Qb, p.q_ts, q_off, qw0 + qt * 32 + l32, S, c * 32 + half * 16);

    // key stages [0, nstage): under a causal mask only keys up to the block's last query matter
    const int q_last = min(q0 + G::BLOCK, S) - 1;
    const int nstage = (causal ? q_last : S - 1) / G::TILE + 1;

    const char* k_head = reinterpret_cast<const char*>(Kb + k_off);  // wave-uniform
    const int k_row_bytes = (int)p.k_ts * (int)sizeof(T);           // host guarantees < 2^24
    int st_voff[G::NLOAD];
    stage_offsets<G>(st_voff, k_row_bytes, tid);
    const unsigned lds_w = lds_offset_of(smem) + (unsigned)__builtin_amdgcn_readfirstlane(wave) * 1024u;

    float lse[NRT];       // the result: lse2 of query qw0 + qt*32 + l32
    bool frozen = true;   // wave-uniform (in fact workgroup-uniform): which pass this is
    for (;;) {
    float m[NRT], l[NRT];  // statistics of the queries qw0 + qt*32 + l32 this lane keeps
#pragma unroll
    for (int qt = 0; qt < NRT; ++qt) { m[qt] = -INFINITY; l[qt] = 0.f; }

    // carry: the last computed tile whose statistics have not been folded in yet (it belongs to the last
    // query subtile); -inf means "none"
    f32x16 carry;
#pragma unroll
    for (int r = 0; r < 16; ++r) carry[r] = -INFINITY;

    stage_load<G>(st_voff, stage_desc<G>(k_head, k_row_bytes, 0, S, true), lds_w);
    stage_settle();
    for (int t = 0; t < nstage; ++t) {
        __syncthreads();  // stage t is complete; every wave is done reading stage t-1
        const bool more = t + 1 < nstage;
        const u32x4 next_desc = stage_desc<G>(k_head, k_row_bytes, (t + 1) * G::TILE, S, more);
        const unsigned next_lds = lds_w + ((t + 1) & 1) * G::STAGE_BYTES;
        const int k0 = t * G::TILE;
        // wave-uniform classification of this stage of keys against the wave's queries [qw0, qw0+RES-1]
        const bool skip = causal && k0 > qw0 + G::RES - 1;  // every key lies after every query
        const bool clean = causal ? (k0 + G::TILE - 1 <= qw0) : (k0 + G::TILE <= S);
        const char* sbuf = smem + (t & 1) * G::STAGE_BYTES;
        const bool hot = clean && frozen && t > 0;
        if (more && !hot) stage_load<G>(st_voff, next_desc, next_lds);  // (the hot path spreads them over its tiles)
        if (hot) {
            // pipelined, frozen reference: exp/sum of the previous tile between the MFMAs of tile (ks, qt)
            // (the sum of a query is kept in two halves, l and l2, that the exponentials are added to directly)
            float nm[NRT], l2[NRT];
#pragma unroll
            for (int q = 0; q < NRT; ++q) {
                m[q] = m[q] == -INFINITY ? 0.f : m[q];  // nothing seen yet: take 0 as the reference
                nm[q] = -m[q];
                l2[q] = 0.f;
            }
            u32x4 kf[G::NCH];
            read_frags<G>(kf, sbuf, 0, l32, half);
#pragma unroll
            for (int ks = 0; ks < G::NSUB; ++ks) {
                u32x4 kn[G::NCH];
                f32x16 prev = carry;
#pragma unroll
                for (int qt = 0; qt < NRT; ++qt) {  // tile (ks, qt) while the tile before it is summed
                    const int pq = (qt + NRT - 1) % NRT;  // query subtile of the tile before
                    f32x16 acc = {0};
                    slot_fence();
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) {
                        rowstat_frozen_slice<G::NCH>(c, prev, c2, nm[pq], l[pq], l2[pq]);
                        mma_chunk<T>(acc, kf[c], qf[qt][c]);  // acc[key row][query col]
                        if (c == 1) stage_load_slot<G>(st_voff, next_desc, next_lds, ks * NRT + qt, G::NSUB * NRT);
                        if (qt == NRT - 1 && ks + 1 < G::NSUB)
                            kn[c] = *reinterpret_cast<const u32x4*>(&sbuf[G::frag((ks + 1) * 32 + l32, c, half)]);
                        slot_fence();
                    }
                    prev = acc;
                }
                carry = prev;
                if (ks + 1 < G::NSUB) {
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) kf[c] = kn[c];
                }
            }
#pragma unroll
            for (int q = 0; q < NRT; ++q) l[q] += l2[q];
        } else if (clean) {
            // pipelined, running maximum: the statistics update of the previous tile is issued slice by slice
            // between the MFMAs of tile (ks, qt); fragments of the next key subtile are read during the last chain
            u32x4 kf[G::NCH];
            read_frags<G>(kf, sbuf, 0, l32, half);
#pragma unroll
            for (int ks = 0; ks < G::NSUB; ++ks) {
                u32x4 kn[G::NCH];
                f32x16 prev = carry;
#pragma unroll
                for (int qt = 0; qt < NRT; ++qt) {
                    const int pq = (qt + NRT - 1) % NRT;
                    f32x16 acc = {0};
                    RowStat st;
                    slot_fence();
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) {
                        rowstat_slice<G::NCH>(c, prev, c2, m[pq], st);
                        mma_chunk<T>(acc, kf[c], qf[qt][c]);
                        if (qt == NRT - 1 && ks + 1 < G::NSUB)
                            kn[c] = *reinterpret_cast<const u32x4*>(&sbuf[G::frag((ks + 1) * 32 + l32, c, half)]);
                        slot_fence();
                    }
                    rowstat_finish(st, m[pq], l[pq]);
                    prev = acc;
                }
                carry = prev;
                if (ks + 1 < G::NSUB) {
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) kf[c] = kn[c];
                }
            }
        } else if (!skip) {
            rowstat_update(carry, c2, m[NRT - 1], l[NRT - 1]);  // drain the pipeline before the masked tiles
#pragma unroll
            for (int r = 0; r < 16; ++r) carry[r] = -INFINITY;
#pragma unroll
            for (int ks = 0; ks < G::NSUB; ++ks) {
                u32x4 kf[G::NCH];
                read_frags<G>(kf, sbuf, ks, l32, half);
#pragma unroll
                for (int qt = 0; qt < NRT; ++qt) {
                    // this 32x32 tile: keys [kmin, kmin+31] against queries [qmin, qmin+31] (wave-uniform tests)
                    const int kmin = k0 + ks * 32, qmin = qw0 + qt * 32;
                    if (causal && kmin > qmin + 31) continue;  // every key lies after every query
                    f32x16 acc = {0};
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) mma_chunk<T>(acc, kf[c], qf[qt][c]);
                    const bool all_allowed = causal ? (kmin + 31 <= qmin) : (kmin + 31 < S);
                    if (!all_allowed) {
                        // key j may be used by query i iff j <= lim(i): i itself under the causal mask, S-1 otherwise
                        const int lim = causal ? qmin + l32 : S - 1;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = kmin + acc_row(r, lane);
                            acc[r] = key <= lim ? acc[r] : -INFINITY;
                        }
                    }
                    rowstat_update(acc, c2, m[qt], l[qt]);
                }
            }
        }
        stage_settle();
    }
    rowstat_update(carry, c2, m[NRT - 1], l[NRT - 1]);

    // the two half-waves hold disjoint key rows of the same queries: merge, then lse2 = m + log2(l)
    bool bad = false;
#pragma unroll
    for (int qt = 0; qt < NRT; ++qt) {
        const float mo = __shfl_xor(m[qt], 32), lo = __shfl_xor(l[qt], 32);
        const float mt = fmaxf(m[qt], mo);
        const float ms = mt == -INFINITY ? 0.f : mt;
        const float lt = l[qt] * __builtin_amdgcn_exp2f(m[qt] - ms) + lo * __builtin_amdgcn_exp2f(mo - ms);
        lse[qt] = mt + __builtin_amdgcn_logf(lt);
        bad |= qw0 + qt * 32 + l32 < S && !isfinite(lse[qt]);
    }
    // every wave is past its last read of the stages here as well, so a second pass may refill them
    if (!frozen || !__syncthreads_or(bad)) break;
    frozen = false;
    }
#pragma unroll
    for (int qt = 0; qt < NRT; ++qt) {
        const int q = qw0 + qt * 32 + l32;
        if (half == 0 && q < S) p.lse2[(size_t)h * S + q] = lse[qt];
    }
}

// ------------------------------------------------------------------------------------------------
// Sweep 2: column sums (and the diagonal) of the probabilities, one key block per workgroup.
// ------------------------------------------------------------------------------------------------

// sum over the 16 probabilities a lane holds of one tile, p = exp2(raw * c2 + nl) with nl = -lse2 of the
// row; slice c of NS covers elements [c*16/NS, (c+1)*16/NS) and adds into two partial sums
template <int NS>
__device__ __forceinline__ void colsum_slice(int c, const f32x16& raw, const float (&nl)[16], float c2, float& s0, float& s1) {
    const int lo = c * 16 / NS, hi = (c + 1) * 16 / NS;
#pragma unroll
    for (int r = lo; r < hi; ++r) {
        const float e = __builtin_amdgcn_exp2f(fmaf(raw[r], c2, nl[r]));
        if (r & 1) s1 += e; else s0 += e;
    }
}
__device__ __forceinline__ float colsum_tile(const f32x16& raw, const float (&nl)[16], float c2) {
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) colsum_slice<8>(c, raw, nl, c2, s0, s1);
    return s0 + s1;
}
// -lse2 of the 16 query rows of subtile `sub` this lane meets (rows 8g + 4*half + 0..3)
__device__ __forceinline__ void read_nl(float (&nl)[16], const float* lbuf, int sub, int half) {
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(&lbuf[sub * 32 + gq * 8 + half * 4]);
        nl[gq * 4 + 0] = v[0]; nl[gq * 4 + 1] = v[1]; nl[gq * 4 + 2] = v[2]; nl[gq * 4 + 3] = v[3];
    }
}

template <typename T, int D, int NRT>
__global__ __launch_bounds__(SC_THREADS, (Geo<T, D, NRT>::MIN_WG)) void colsum_kernel(ScoreParams p) {
    using G = Geo<T, D, NRT>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float* const sLbase = reinterpret_cast<float*>(smem + 2 * G::STAGE_BYTES);

    int h, kb;
    if (!decode_block(p.n_key_blocks, p.heads_per_xcd, p.H, h, kb)) return;
    const bool causal = (p.flags & LEMO_CAUSAL) != 0;
    const int S = p.S;
    const float c2 = p.c2;
    // key block -> (segment, block inside the segment); blocks never straddle a segment boundary
    const int seg = kb / p.blocks_per_seg, bis = kb - seg * p.blocks_per_seg;
    const long long seg0 = (long long)seg * p.L;
    const long long key0_ll = seg0 + (long long)bis * G::BLOCK;
    if (key0_ll >= S) return;
    const int key0 = (int)key0_ll;
    const int kend = (int)min((long long)S, min(seg0 + p.L, key0_ll + G::BLOCK));  // exclusive

    const int g = (int)(((long long)h * p.H_kv) / p.H);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const T* Qb = static_cast<const T*>(p.Q);
    const T* Kb = static_cast<const T*>(p.K);
    const long long q_off = (long long)h * p.q_hs, k_off = (long long)g * p.k_hs;
    const float* lse = p.lse2 + (size_t)h * S;
    const int kw0 = key0 + wave * G::RES;  // first key of this wave

    // resident operand: this wave's keys as MFMA B fragments (zero beyond the block's end)
    u32x4 kf[NRT][G::NCH];
#pragma unroll
    for (int kt = 0; kt < NRT; ++kt)
#pragma unroll
        for (int c = 0; c < G::NCH; ++c) kf[kt][c] = load_piece(Kb, p.k_ts, k_off, kw0 + kt * 32 + l32, kend, c * 32 + half * 16);

    float col[NRT], col2[NRT], dg[NRT];  // column kw0 + kt*32 + l32 (its sum kept in two halves, col and col2)
#pragma unroll
    for (int kt = 0; kt < NRT; ++kt) { col[kt] = 0.f; col2[kt] = 0.f; dg[kt] = 0.f; }

    // query stages run from the end of the sequence DOWN to the first stage that can see this block, so
    // that all key blocks of a head walk the same query rows at about the same time (shared through L2)
    const int t_hi = (S - 1) / G::TILE;
    const int t_lo = causal ? key0 / G::TILE : 0;

    const char* q_head = reinterpret_cast<const char*>(Qb + q_off);  // wave-uniform
    const int q_row_bytes = (int)p.q_ts * (int)sizeof(T);           // host guarantees < 2^24
    int st_voff[G::NLOAD];
    stage_offsets<G>(st_voff, q_row_bytes, tid);
    const unsigned lds_w = lds_offset_of(smem) + (unsigned)__builtin_amdgcn_readfirstlane(wave) * 1024u;
    float pre_l = 0.f;
    // row statistics of a stage: thread tid < TILE owns row tid; beyond the end +inf, so that p = exp2(-inf) = 0
    auto fetch_l = [&](int t) { return tid < G::TILE ? lse[min(t * G::TILE + tid, S - 1)] : 0.f; };
    auto fix_l = [&](int t, float v) { return t * G::TILE + tid < S ? -v : -INFINITY; };  // stored negated: p = exp2(s*c2 + nl)

    // carry: last computed tile not yet summed (always a tile of the last key subtile); nl = -inf means "none"
    f32x16 carry = {0};
    float carry_nl[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) carry_nl[r] = -INFINITY;

    stage_load<G>(st_voff, stage_desc<G>(q_head, q_row_bytes, t_hi * G::TILE, S, true), lds_w);
    pre_l = fetch_l(t_hi);
    if (tid < G::TILE) sLbase[tid] = fix_l(t_hi, pre_l);
    stage_settle();
    int buf = 0;
    for (int t = t_hi; t >= t_lo; --t, buf ^= 1) {
        __syncthreads();
        const bool more = t > t_lo;
        const u32x4 next_desc = stage_desc<G>(q_head, q_row_bytes, (t - 1) * G::TILE, S, more);
        const unsigned next_lds = lds_w + (buf ^ 1) * G::STAGE_BYTES;
        if (more) pre_l = fetch_l(t - 1);
        const int i0 = t * G::TILE;
        const bool on_diag = i0 <= kw0 + G::RES - 1 && i0 + G::TILE - 1 >= kw0;  // stage meets the diagonal band of this wave
        const bool skip = causal && i0 + G::TILE - 1 < kw0;                     // every query lies before every key
        const char* sbuf = smem + buf * G::STAGE_BYTES;
        const float* lbuf = sLbase + buf * G::TILE;
        const bool hot = !on_diag && !skip;
        if (more && !hot) stage_load<G>(st_voff, next_desc, next_lds);  // (the hot path spreads them over its tiles)
        if (hot) {
            // pipelined: exp/sum of the previous tile is issued slice by slice between the MFMAs of tile
            // (qs, kt); fragments and row statistics of the next query subtile are read during the last chain
            u32x4 qf[G::NCH];
            float nl[16];
            read_frags<G>(qf, sbuf, 0, l32, half);
            read_nl(nl, lbuf, 0, half);
#pragma unroll
            for (int qs = 0; qs < G::NSUB; ++qs) {
                u32x4 qn[G::NCH];
                float nn[16];
                f32x16 prev = carry;
#pragma unroll
                for (int kt = 0; kt < NRT; ++kt) {  // tile (qs, kt) while the tile before it is summed
                    const int pk = (kt + NRT - 1) % NRT;  // key subtile of the tile before
                    f32x16 acc = {0};
                    slot_fence();
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) {
                        if (kt == 0) colsum_slice<G::NCH>(c, prev, carry_nl, c2, col[pk], col2[pk]);  // the carried tile has its own rows
                        else colsum_slice<G::NCH>(c, prev, nl, c2, col[pk], col2[pk]);
                        mma_chunk<T>(acc, qf[c], kf[kt][c]);  // acc[query row][key col]
                        if (c == 1) stage_load_slot<G>(st_voff, next_desc, next_lds, qs * NRT + kt, G::NSUB * NRT);
                        if (kt == NRT - 1 && qs + 1 < G::NSUB) {
                            qn[c] = *reinterpret_cast<const u32x4*>(&sbuf[G::frag((qs + 1) * 32 + l32, c, half)]);
                            if (c < 4) {
                                const f32x4 v = *reinterpret_cast<const f32x4*>(&lbuf[(qs + 1) * 32 + c * 8 + half * 4]);
                                nn[c * 4 + 0] = v[0]; nn[c * 4 + 1] = v[1]; nn[c * 4 + 2] = v[2]; nn[c * 4 + 3] = v[3];
                            }
                        }
                        slot_fence();
                    }
                    prev = acc;
                }
                carry = prev;
#pragma unroll
                for (int r = 0; r < 16; ++r) carry_nl[r] = nl[r];
                if (qs + 1 < G::NSUB) {
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) qf[c] = qn[c];
#pragma unroll
                    for (int r = 0; r < 16; ++r) nl[r] = nn[r];
                }
            }
        } else if (!skip) {
            col[NRT - 1] += colsum_tile(carry, carry_nl, c2);  // drain the pipeline before the masked tiles
#pragma unroll
            for (int r = 0; r < 16; ++r) carry_nl[r] = -INFINITY;
#pragma unroll
            for (int qs = 0; qs < G::NSUB; ++qs) {
                u32x4 qf[G::NCH];
                float nl[16];
                read_frags<G>(qf, sbuf, qs, l32, half);
                read_nl(nl, lbuf, qs, half);
#pragma unroll
                for (int kt = 0; kt < NRT; ++kt) {
                    // this 32x32 tile: queries [qmin, qmin+31] against keys [kmin, kmin+31] (wave-uniform tests)
                    const int qmin = i0 + qs * 32, kmin = kw0 + kt * 32;
                    if (causal && qmin + 31 < kmin) continue;  // every query lies before every key
                    f32x16 acc = {0};
#pragma unroll
                    for (int c = 0; c < G::NCH; ++c) mma_chunk<T>(acc, qf[c], kf[kt][c]);
                    if (qmin > kmin + 31 || qmin + 31 < kmin) {  // off the diagonal: nothing to mask, no self term
                        col[kt] += colsum_tile(acc, nl, c2);
                    } else {
                        const int my_k = kmin + l32;
                        float part = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int q = qmin + acc_row(r, lane);
                            float pr = __builtin_amdgcn_exp2f(fmaf(acc[r], c2, nl[r]));
                            if (causal && q < my_k) pr = 0.f;
                            if (q == my_k) dg[kt] = pr;
                            part += pr;
                        }
                        col[kt] += part;
                    }
                }
            }
        }
        if (more && tid < G::TILE) sLbase[(buf ^ 1) * G::TILE + tid] = fix_l(t - 1, pre_l);
        stage_settle();
    }
    col[NRT - 1] += colsum_tile(carry, carry_nl, c2);

#pragma unroll
    for (int kt = 0; kt < NRT; ++kt) {
        col[kt] += col2[kt];
        const float c = col[kt] + __shfl_xor(col[kt], 32);
        const float dd = dg[kt] + __shfl_xor(dg[kt], 32);
        const int key = kw0 + kt * 32 + l32;
        if (half == 0 && key < kend) {
            p.colsum[(size_t)h * S + key] = c;
            p.diag[(size_t)h * S + key] = dd;
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

// which: bit 0 = sweep 1 (row statistics), bit 1 = sweep 2 (column sums)
template <typename T, int D, int NRT>
static int launch_sweeps(const ScoreParams& p_in, int which, hipStream_t st) {
    using G = Geo<T, D, NRT>;
    ScoreParams p = p_in;
    p.n_query_blocks = (p.S + G::BLOCK - 1) / G::BLOCK;
    // Key blocks never straddle a segment boundary.  Segments shorter than a block are grouped: a block
    // then covers as many WHOLE segments as fit, which is the same as working with that longer unit.
    long long Leff = p.L;
    if (Leff < G::BLOCK) Leff = (G::BLOCK / Leff) * Leff;
    if (Leff > p.S) Leff = p.S;
    p.L = (int)Leff;
    p.blocks_per_seg = (int)((Leff + G::BLOCK - 1) / G::BLOCK);
    const long long nseg = ((long long)p.S + Leff - 1) / Leff;
    p.n_key_blocks = (int)(nseg * p.blocks_per_seg);
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {  // the kernels use more dynamic LDS than the default limit
        const void* ks[2] = {reinterpret_cast<const void*>(&rowstats_kernel<T, D, NRT>),
                             reinterpret_cast<const void*>(&colsum_kernel<T, D, NRT>)};
        const int bytes[2] = {G::LDS_ROWSTATS, G::LDS_COLSUM};
        for (int i = 0; i < 2 && attr_err == hipSuccess; ++i)
            attr_err = hipFuncSetAttribute(ks[i], hipFuncAttributeMaxDynamicSharedMemorySize, bytes[i]);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    const unsigned g1 = (unsigned)(NUM_XCD * p.heads_per_xcd * p.n_query_blocks);
    const unsigned g2 = (unsigned)(NUM_XCD * p.heads_per_xcd * p.n_key_blocks);
    if (which & 1) hipLaunchKernelGGL((rowstats_kernel<T, D, NRT>), dim3(g1), dim3(SC_THREADS), G::LDS_ROWSTATS, st, p);
    if (which & 2) hipLaunchKernelGGL((colsum_kernel<T, D, NRT>), dim3(g2), dim3(SC_THREADS), G::LDS_COLSUM, st, p);
    return (int)hipGetLastError();
}

int launch_score(const ScoreParams& p_in, lemo_dtype_t dt, int d, int which, hipStream_t st) {
    ScoreParams p = p_in;
    p.heads_per_xcd = (p.H + NUM_XCD - 1) / NUM_XCD;
    int rc = 0;
    if (which & 3) {
        if (dt == LEMO_BF16 && d == 128) rc = launch_sweeps<bf16_t, 128, LEMO_NRT_BF16_128>(p, which, st);
        else if (dt == LEMO_BF16 && d == 64) rc = launch_sweeps<bf16_t, 64, 2>(p, which, st);
        else if (dt == LEMO_F32 && d == 128) rc = launch_sweeps<float, 128, 2>(p, which, st);
        else if (dt == LEMO_F32 && d == 64) rc = launch_sweeps<float, 64, 2>(p, which, st);
        else return (int)hipErrorInvalidValue;
        if (rc) return rc;
    }
    if (which & 4) {
        hipLaunchKernelGGL(head_mean_kernel, dim3((p.S + 255) / 256), dim3(256), 0, st, p.colsum, p.diag, p.scores, p.S, p.H,
                           (p.flags & LEMO_EXCLUDE_SELF) ? 1 : 0);
        rc = (int)hipGetLastError();
    }
    return rc;
}

}  // namespace lemo
