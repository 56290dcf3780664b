// Block-wise informativeness (Sec. 4.2 "Block-wise Elimination", Eq. 2; token-block sums of "Layer-specific
// Threshold"):  mean[i][j] = (1/H) sum_h S^h_ij (positive terms only),  I(B^S_mn) = max over the b x b score block,
// B^T_n = sum_m I(B^S_mn).
//
// Eq. 2 takes the head aggregate BEFORE the maximum, so the head loop has to run inside a tile: a workgroup owns a
// TT x TT (query x key) rectangle of the score matrix and walks the heads, adding each head's probabilities (or positive
// logits) into register accumulators that hold the rectangle's head sum.  Nothing is masked while accumulating -- pairs
// a causal mask forbids are simply left out of the maximum at the end.  Kernel 1 writes the maximum of every 32 x 32
// MFMA tile to a [ceil(S/32)]^2 matrix; kernel 2 folds that matrix into b x b score blocks (b a multiple of 32) and sums
// each block column.
//
// Unlike the two sweeps of the token-wise score there is no operand that stays resident across the inner loop (every
// head brings its own Q and K rows), so the kernel leans on the caches: the 256 workgroups in flight form a 16 x 16
// super-patch of rectangles (32 operand tiles for 256 rectangles), and each die works on a 4 x 8 sub-patch of it.
// Per head a workgroup moves 64 KB from L2 into LDS and 192 KB from LDS into registers for 4.2 MFLOP, so the head loop
// is one software pipeline three heads deep: head h in registers (MFMA fragments, refilled in place as soon as an
// MFMA has used them), head h + 1 complete in one LDS stage, head h + 2 arriving in the other through LDS-direct
// loads, one barrier per head.
#include <mutex>
#include <type_traits>

#include "lemo_common.hpp"

namespace lemo {

constexpr int SB_PATCH = 16;  // super-patch edge, in rectangles

template <typename T, int D> struct BGeo {
    static constexpr int ROWB = D * (int)sizeof(T);  // bytes per head row
    static constexpr int NCH = ROWB / 32;            // MFMA chunks per row
    static constexpr int CPR = ROWB / 16;            // 16-byte pieces per row
    static constexpr int TT = ROWB > 256 ? 64 : 128; // rectangle edge (queries and keys)
    // Waves: NWQ along the queries x NWK along the keys.  The LDS only reaches its bandwidth with two waves per SIMD
    // (measured: 114 B/clk/CU with four waves reading, 220 with eight), and this kernel moves 5 LDS bytes per 1000
    // flops, so the 128-row rectangle is worked by eight waves of 32 queries x 64 keys (one query subtile per wave: half
    // as many row-statistic reads as with 64 x 32).
    static constexpr int NWQ = TT == 128 ? 4 : 2;
    static constexpr int NWK = 2;
    static constexpr int THREADS = NWQ * NWK * 64;
    static constexpr int NSQ = TT / NWQ / 32;        // 32-row query subtiles per wave
    static constexpr int NSK = TT / NWK / 32;        // 32-row key subtiles per wave
    // Staging is done by LDS-direct buffer loads (the data never passes through registers): a wave instruction fills
    // 1 KB of consecutive LDS bytes, lane by lane, so rows cannot be padded.  Instead unit u (16 bytes) of a tile holds
    // row u / CPR, piece (u % CPR) ^ swz(row): 16 consecutive rows still put any one piece into 16 distinct bank groups.
    static constexpr int NLOAD = TT * CPR / THREADS; // 16-byte loads per thread, head and operand
    static constexpr int TILE_BYTES = TT * ROWB;
    static constexpr int STAGE_BYTES = 2 * TILE_BYTES;                            // Q rows, K rows
    static constexpr int LSE_BASE = 2 * STAGE_BYTES, LSE_BYTES = TT * (int)sizeof(float);  // ring of four heads' row statistics
    static constexpr int LDS = LSE_BASE + 4 * LSE_BYTES;
    static_assert(TT * CPR % THREADS == 0 && THREADS % CPR == 0, "tile must split evenly over the workgroup");
    __device__ static constexpr int swz(int row) { return CPR >= 16 ? (row & 15) : ((row >> 1) & (CPR - 1)); }
};

__device__ __forceinline__ void sb_fence() { __builtin_amdgcn_sched_barrier(0); }

// MODE 0: probabilities exp2(s * c2 - lse2_i);  MODE 1: positive part of the raw dot product (scaled at the end)
template <typename T, int D, int MODE>
__global__ __launch_bounds__((BGeo<T, D>::THREADS), 1) void tilemax_kernel(BlockParams p) {
    using G = BGeo<T, D>;
    constexpr int NSQ = G::NSQ, NSK = G::NSK;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // rectangle of this workgroup
    const bool causal = (p.flags & LEMO_CAUSAL) != 0;
    const int sp_id = blockIdx.x / (SB_PATCH * SB_PATCH), loc = blockIdx.x % (SB_PATCH * SB_PATCH);
    int spm, spn;
    if (causal) {  // super-patches on and below the diagonal, row by row
        spm = (int)((sqrtf(8.f * (float)sp_id + 1.f) - 1.f) * 0.5f);
        while ((spm + 1) * (spm + 2) / 2 <= sp_id) ++spm;
        while (spm * (spm + 1) / 2 > sp_id) --spm;
        spn = sp_id - spm * (spm + 1) / 2;
    } else {
        spm = sp_id / p.nsp;
        spn = sp_id - spm * p.nsp;
    }
    const int x = loc % NUM_XCD, w = loc / NUM_XCD;  // die, and the workgroup's slot on it
    const int tq = spm * SB_PATCH + (x >> 1) * 4 + (w & 3);
    const int tk = spn * SB_PATCH + (x & 1) * 8 + (w >> 2);
    if (tq >= p.nt || tk >= p.nt || (causal && tk > tq)) return;  // outside the matrix, or wholly above the diagonal

    const int S = p.S;
    const int q0 = tq * G::TT, k0 = tk * G::TT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int wq = wave / G::NWK, wk = wave % G::NWK;
    const float c2 = p.c2;
    const T* Qb = static_cast<const T*>(p.Q);
    const T* Kb = static_cast<const T*>(p.K);

    // staging: unit u = i * THREADS + tid of a tile goes to LDS bytes [16u, 16u + 16); the lane fetches the piece that
    // belongs there.  Range-checked loads: the descriptor starts at the rectangle's first row of the head and ends with
    // the last row of the tensor, so rows past the end arrive as zeros.
    const int q_row_bytes = (int)p.q_ts * (int)sizeof(T), k_row_bytes = (int)p.k_ts * (int)sizeof(T);  // host: < 2^24
    int q_voff[G::NLOAD], k_voff[G::NLOAD];
#pragma unroll
    for (int i = 0; i < G::NLOAD; ++i) {
        const int u = i * G::THREADS + tid, row = u / G::CPR, piece = (u % G::CPR) ^ G::swz(row);
        q_voff[i] = row * q_row_bytes + piece * 16;
        k_voff[i] = row * k_row_bytes + piece * 16;
    }
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const unsigned group = (unsigned)(p.H / p.H_kv);  // query heads per key head (the host checks divisibility)
    const unsigned lds0 = (unsigned)reinterpret_cast<unsigned long long>(smem);  // LDS byte offset of the staging area
    // Row statistics: every wave brings in 64 of the TT values (several waves the same ones: no branch in the stream).
    // Rows past the end reuse the last row's (they are masked at the end).
    const int l_voff = min(q0 + tid % G::TT, S - 1) * (int)sizeof(float);
    // A head's loads are described once (`aim`) and then issued one by one (`issue_one`), so that a computing wave can
    // spread them between its MFMAs: the CU's vector-memory pipe takes 16 cycles per 1 KB instruction, and a wave that
    // issues its share back to back stalls on the queue.
    constexpr int PER_HEAD = 2 * G::NLOAD;  // tile loads per wave and head (the row statistics are one more)
    u32x4 aim_q, aim_k, aim_l;
    unsigned aim_s = 0, aim_ls = 0;
    // Head hh goes to stage buf and to entry hh & 3 of the statistics ring.  Past the last head the descriptors have
    // length zero: the loads stay in the stream (no branch) but fetch nothing, and what they write nobody reads.
    auto aim = [&](int hh, int buf) {
        const bool live = hh < p.H;
        const int h = min(hh, p.H - 1);
        const int g = (int)((unsigned)h / group);
        const char* qh = reinterpret_cast<const char*>(Qb + (long long)h * p.q_hs) + (long long)q0 * q_row_bytes;
        const char* kh = reinterpret_cast<const char*>(Kb + (long long)g * p.k_hs) + (long long)k0 * k_row_bytes;
        const long long qspan = (long long)(S - q0 - 1) * q_row_bytes + G::ROWB, kspan = (long long)(S - k0 - 1) * k_row_bytes + G::ROWB;
        aim_q = raw_rsrc(qh, live ? qspan : 0);
        aim_k = raw_rsrc(kh, live ? kspan : 0);
        if (MODE == 0) aim_l = raw_rsrc(p.lse2 + (size_t)h * S, live ? (long long)S * 4 : 0);
        aim_s = lds0 + buf * G::STAGE_BYTES;
        aim_ls = lds0 + G::LSE_BASE + (hh & 3) * G::LSE_BYTES;
    };
    auto issue_one = [&](int n) {  // n = 0 .. PER_HEAD (compile-time after unrolling)
        if (n < PER_HEAD) {
            const int i = n >> 1;
            if (n & 1) lds_direct_b128(aim_k, aim_s + G::TILE_BYTES + wave_u * 1024 + i * G::THREADS * 16, k_voff[i]);
            else lds_direct_b128(aim_q, aim_s + wave_u * 1024 + i * G::THREADS * 16, q_voff[i]);
        } else if (MODE == 0 && n == PER_HEAD) {
            lds_direct_b32(aim_l, aim_ls + wave_u % (G::TT / 64) * 256, l_voff);
        }
    };
    auto issue = [&](int h, int buf) {
        aim(h, buf);
#pragma unroll
        for (int n = 0; n <= PER_HEAD; ++n) issue_one(n);
    };

    // head sums of this wave's NSQ x NSK tiles: sbar[qs][ks][r] = element (row acc_row(r), column l32) of tile (qs, ks)
    f32x16 sbar[NSQ][NSK];
#pragma unroll
    for (int a = 0; a < NSQ; ++a)
#pragma unroll
        for (int b = 0; b < NSK; ++b) sbar[a][b] = f32x16{0};

    // add the tile `raw` (unscaled dot products) into its accumulator; slice c of NSL covers elements [c*16/NSL, ...)
    auto accumulate = [&](f32x16& dst, const f32x16& raw, const float (&nl)[16], int c, int nsl) {
        const int lo = c * 16 / nsl, hi = (c + 1) * 16 / nsl;
        // The slice's arithmetic hangs on a scalar that an (empty) volatile statement defines here, so that instruction
        // selection cannot gather the slices of a tile in front of the first of them.
        float k = MODE == 0 ? c2 : 0.f;
        asm volatile("" : "+s"(k));
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < lo || r >= hi) continue;
            if (MODE == 0) dst[r] += __builtin_amdgcn_exp2f(fmaf(raw[r], k, -nl[r]));
            else dst[r] += fmaxf(raw[r], k);
        }
    };

    // fragments of the head being worked on (registers); refilled in place, piece by piece, with the next head's
    u32x4 qf[NSQ][G::NCH], kf[NSK][G::NCH];
    float nl[NSQ][16];  // row statistics of the head whose tiles are being accumulated
#pragma unroll
    for (int r = 0; r < 16 * NSQ; ++r) nl[r / 16][r % 16] = INFINITY;  // the first "tile before" is empty: exp2(0 - inf) = 0
    const int q_row0 = wq * NSQ * 32 + l32, k_row0 = wk * NSK * 32 + l32;  // + 32 s: swz() of the row does not depend on s
    const int q_frag = q_row0 * G::ROWB, k_frag = G::TILE_BYTES + k_row0 * G::ROWB, f_swz = G::swz(l32);
    auto read_q = [&](int buf, int s_, int c) {
        qf[s_][c] = *reinterpret_cast<const u32x4*>(&smem[buf * G::STAGE_BYTES + q_frag + s_ * 32 * G::ROWB + (((2 * c + half) ^ f_swz) << 4)]);
    };
    auto read_k = [&](int buf, int s_, int c) {
        kf[s_][c] = *reinterpret_cast<const u32x4*>(&smem[buf * G::STAGE_BYTES + k_frag + s_ * 32 * G::ROWB + (((2 * c + half) ^ f_swz) << 4)]);
    };
    auto read_nl = [&](int h) {
        if (MODE != 0) return;
        const float* sl = reinterpret_cast<const float*>(smem + G::LSE_BASE + (h & 3) * G::LSE_BYTES);
#pragma unroll
        for (int s_ = 0; s_ < NSQ; ++s_)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {  // rows 8*gq + 4*half + 0..3 of query subtile s_
                const f32x4 v = *reinterpret_cast<const f32x4*>(&sl[(wq * NSQ + s_) * 32 + gq * 8 + half * 4]);
                nl[s_][gq * 4 + 0] = v[0]; nl[s_][gq * 4 + 1] = v[1]; nl[s_][gq * 4 + 2] = v[2]; nl[s_][gq * 4 + 3] = v[3];
            }
    };

    // Prologue: head 0 into stage 0 and from there into registers, head 1 into stage 1.
    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
#pragma unroll
    for (int c = 0; c < G::NCH; ++c) {
#pragma unroll
        for (int s_ = 0; s_ < NSQ; ++s_) read_q(0, s_, c);
#pragma unroll
        for (int s_ = 0; s_ < NSK; ++s_) read_k(0, s_, c);
    }
    if (p.H > 1) issue(1, 1);
    aim(2, 0);

    // Head h: one barrier, then a single instruction stream in which every MFMA is followed by the LDS reads that refill
    // the fragments it was the last to use (with head h + 1, from stage (h+1) & 1), by this wave's next LDS-direct load
    // of head h + 2 (into stage h & 1, which nobody reads any more; row statistics into entry (h+2) & 3 of their ring) and
    // by a slice of the exponentials of the tile before -- for the first tile that is the last tile of head h - 1
    // (`carry`).  Nothing is issued in bursts and nothing is left for a tail: a wave gets one 16-byte LDS read through in
    // about 40 cycles, the CU's vector-memory pipe takes 16 cycles per 1 KB load instruction, and while a wave does
    // vector-only work at the end of a step the matrix unit of its SIMD idles.
    constexpr int NT = NSQ * NSK, NM = NT * G::NCH, NL = PER_HEAD + 1, LPM = (NL + NM - 1) / NM;  // tiles, MFMAs, loads, loads per MFMA
    constexpr int AIM_SLOT = (NL + LPM - 1) / LPM;  // the first MFMA after the step's last load: describe the next step's loads
    static_assert(NSQ == 1 && AIM_SLOT < NM, "the stream below assumes one query subtile per wave and room after the loads");
    f32x16 carry = {0};
    for (int h = 0; h < p.H; ++h) {
        // The stages are refilled by loads the compiler does not see: this wave's reads of stage h & 1 must have
        // returned, and its part of head h + 1 must have landed, before anyone passes the barrier.
        __builtin_amdgcn_s_waitcnt(LGKMCNT0);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __syncthreads();
        const int nxt = (h + 1) & 1;
        f32x16 prev = carry;
#pragma unroll
        for (int tl = 0; tl < NT; ++tl) {
            const int qs = tl / NSK, ks = tl % NSK;
            const int pq = (tl + NT - 1) % NT / NSK, pk = (tl + NT - 1) % NT % NSK;  // the tile before
            f32x16 acc = {0};
            sb_fence();
#pragma unroll
            for (int c = 0; c < G::NCH; ++c) {
                mma_chunk<T>(acc, qf[qs][c], kf[ks][c]);  // acc[query row][key col]
                if (ks == NSK - 1) read_q(nxt, qs, c);
                if (qs == NSQ - 1) read_k(nxt, ks, c);
                const int m = tl * G::NCH + c;  // loads go out with the first MFMAs: they must have landed by the end of the step
#pragma unroll
                for (int n = m * LPM; n < (m + 1) * LPM; ++n) issue_one(n);  // (issue_one ignores n past the last load)
                if (m == AIM_SLOT) aim(h + 3, nxt);
                accumulate(sbar[pq][pk], prev, nl[pq], c, G::NCH);
                // the statistics of head h - 1 have served (its last tile has just been added): bring in head h's
                if (tl == 0 && c == G::NCH - 1) read_nl(h);
                sb_fence();
            }
            prev = acc;
        }
        carry = prev;
    }
    __builtin_amdgcn_s_waitcnt(LGKMCNT0);
#pragma unroll
    for (int c = 0; c < 4; ++c) accumulate(sbar[NSQ - 1][NSK - 1], carry, nl[NSQ - 1], c, 4);

    // maximum of every 32 x 32 tile over the pairs that are admitted
    const bool excl = (p.flags & LEMO_EXCLUDE_SELF) != 0;
#pragma unroll
    for (int qs = 0; qs < NSQ; ++qs)
#pragma unroll
        for (int ks = 0; ks < NSK; ++ks) {
            const int i0 = q0 + (wq * NSQ + qs) * 32, j = k0 + (wk * NSK + ks) * 32 + l32;
            float m = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + acc_row(r, lane);
                const bool ok = (i < S) & (j < S) & (!causal | (j <= i)) & (!excl | (i != j));
                m = fmaxf(m, ok ? sbar[qs][ks][r] : 0.f);
            }
#pragma unroll
            for (int sh = 32; sh >= 1; sh >>= 1) m = fmaxf(m, __shfl_xor(m, sh));
            const int ti = i0 / 32, tj = (k0 + (wk * NSK + ks) * 32) / 32;
            if (lane == 0 && ti < p.nt32 && tj < p.nt32) p.tilemax[(size_t)ti * p.nt32 + tj] = m * p.out_scale;
        }
}

// One workgroup per block column n: I(B_mn) = max of the 32 x 32 tile maxima inside the b x b block, B^T_n = sum over m.
// Under a causal mask only tiles on or below the diagonal were written (the others are zero by definition).
__global__ __launch_bounds__(256) void block_reduce_kernel(const float* __restrict__ tilemax, int nt32, int b32, int nb, int causal,
                                                           float* __restrict__ score_blocks, float* __restrict__ token_blocks) {
    __shared__ float part[256];
    const int n = blockIdx.x, tid = threadIdx.x;
    float sum = 0.f;
    for (int m = tid; m < nb; m += 256) {
        float best = 0.f;
        if (!causal || m >= n) {
            const int ti_end = min((m + 1) * b32, nt32), tj_end = min((n + 1) * b32, nt32);
            for (int ti = m * b32; ti < ti_end; ++ti)
                for (int tj = n * b32; tj < tj_end; ++tj)
                    if (!causal || tj <= ti) best = fmaxf(best, tilemax[(size_t)ti * nt32 + tj]);
        }
        if (score_blocks) score_blocks[(size_t)m * nb + n] = best;
        sum += best;
    }
    part[tid] = sum;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {  // fixed-order tree: the result does not depend on timing
        if (tid < s) part[tid] += part[tid + s];
        __syncthreads();
    }
    if (tid == 0) token_blocks[n] = part[0];
}

template <typename T, int D, int MODE>
static int launch_tilemax_t(BlockParams p, hipStream_t st) {
    using G = BGeo<T, D>;
    p.nt = (p.S + G::TT - 1) / G::TT;
    p.nsp = (p.nt + SB_PATCH - 1) / SB_PATCH;
    const long long nsp_total = (p.flags & LEMO_CAUSAL) ? (long long)p.nsp * (p.nsp + 1) / 2 : (long long)p.nsp * p.nsp;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&tilemax_kernel<T, D, MODE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    hipLaunchKernelGGL((tilemax_kernel<T, D, MODE>), dim3((unsigned)(nsp_total * SB_PATCH * SB_PATCH)), dim3(G::THREADS), G::LDS, st, p);
    return (int)hipGetLastError();
}

// mode 0: probabilities (lse2 must hold the row statistics); mode 1: positive logits
int launch_score_blocks(const BlockParams& p_in, lemo_dtype_t dt, int d, int mode, int b, float* score_blocks, float* token_blocks,
                        hipStream_t st) {
    BlockParams p = p_in;
    p.nt32 = (p.S + 31) / 32;
    int rc;
    if (dt == LEMO_BF16 && d == 128) rc = mode ? launch_tilemax_t<bf16_t, 128, 1>(p, st) : launch_tilemax_t<bf16_t, 128, 0>(p, st);
    else if (dt == LEMO_BF16 && d == 64) rc = mode ? launch_tilemax_t<bf16_t, 64, 1>(p, st) : launch_tilemax_t<bf16_t, 64, 0>(p, st);
    else if (dt == LEMO_F32 && d == 128) rc = mode ? launch_tilemax_t<float, 128, 1>(p, st) : launch_tilemax_t<float, 128, 0>(p, st);
    else if (dt == LEMO_F32 && d == 64) rc = mode ? launch_tilemax_t<float, 64, 1>(p, st) : launch_tilemax_t<float, 64, 0>(p, st);
    else return (int)hipErrorInvalidValue;
    if (rc) return rc;
    const int nb = (p.S + b - 1) / b;
    hipLaunchKernelGGL(block_reduce_kernel, dim3((unsigned)nb), dim3(256), 0, st, p.tilemax, p.nt32, b / 32, nb,
                       (p.flags & LEMO_CAUSAL) ? 1 : 0, score_blocks, token_blocks);
    return (int)hipGetLastError();
}

}  // namespace lemo
