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
#include <mutex>
#include <type_traits>

#include "lemo_common.hpp"

namespace lemo {

constexpr int SB_PATCH = 16;  // super-patch edge, in rectangles

template <typename T, int D> struct BGeo {
    static constexpr int ROWB = D * (int)sizeof(T);  // bytes per head row
    static constexpr int NCH = ROWB / 32;            // MFMA chunks per row
    static constexpr int CPR = ROWB / 16;            // 16-byte pieces per row
    static constexpr int STRIDE = ROWB + 16;         // LDS row pitch (16 consecutive rows -> 16 distinct bank groups)
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
    static constexpr int ROWS_PER_LOAD = THREADS / CPR;
    static constexpr int NLOAD = TT / ROWS_PER_LOAD; // 16-byte loads per thread, head and operand
    static constexpr int STAGE_BYTES = 2 * TT * STRIDE + TT * (int)sizeof(float);  // Q rows, K rows, -lse2 of the Q rows
    static constexpr int LDS = 2 * STAGE_BYTES;
    static_assert(TT % ROWS_PER_LOAD == 0, "tile must split evenly over the workgroup");
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

    // staging: thread owns the 16-byte piece (tid % CPR) of rows tid / CPR + i * ROWS_PER_LOAD of both operands
    const int st_row = tid / G::CPR, st_cc = tid % G::CPR;
    const int q_row_bytes = (int)p.q_ts * (int)sizeof(T), k_row_bytes = (int)p.k_ts * (int)sizeof(T);  // host: < 2^24
    const int q_voff = st_row * q_row_bytes + st_cc * 16, k_voff = st_row * k_row_bytes + st_cc * 16;
    const int st_off = st_row * G::STRIDE + st_cc * 16;
    u32x4 preq[G::NLOAD], prek[G::NLOAD];
    float pre_l = 0.f;
    // Range-checked loads: the descriptor starts at the rectangle's first row of the head and ends with the last row
    // of the tensor, so rows past the end read as zero.
    auto fetch = [&](int h) {
        const int g = (int)(((long long)h * p.H_kv) / p.H);
        const char* qh = reinterpret_cast<const char*>(Qb + (long long)h * p.q_hs) + (long long)q0 * q_row_bytes;
        const char* kh = reinterpret_cast<const char*>(Kb + (long long)g * p.k_hs) + (long long)k0 * k_row_bytes;
        const long long qspan = (long long)(S - q0 - 1) * q_row_bytes + G::ROWB, kspan = (long long)(S - k0 - 1) * k_row_bytes + G::ROWB;
        const __amdgpu_buffer_rsrc_t qr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(qh), 0, (int)min(qspan, 0x7fffffffLL), 0x00020000);
        const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kh), 0, (int)min(kspan, 0x7fffffffLL), 0x00020000);
#pragma unroll
        for (int i = 0; i < G::NLOAD; ++i) {
            preq[i] = __builtin_amdgcn_raw_buffer_load_b128(qr, q_voff, i * G::ROWS_PER_LOAD * q_row_bytes, 0);
            prek[i] = __builtin_amdgcn_raw_buffer_load_b128(kr, k_voff, i * G::ROWS_PER_LOAD * k_row_bytes, 0);
        }
        if (MODE == 0 && tid < G::TT) pre_l = p.lse2[(size_t)h * S + min(q0 + tid, S - 1)];
    };
    auto stash = [&](int buf) {
        char* s = smem + buf * G::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < G::NLOAD; ++i) {
            *reinterpret_cast<u32x4*>(s + st_off + i * G::ROWS_PER_LOAD * G::STRIDE) = preq[i];
            *reinterpret_cast<u32x4*>(s + G::TT * G::STRIDE + st_off + i * G::ROWS_PER_LOAD * G::STRIDE) = prek[i];
        }
        // stored negated (p = exp2(s*c2 + nl)); rows past the end get -inf, i.e. probability 0
        if (MODE == 0 && tid < G::TT) reinterpret_cast<float*>(s + 2 * G::TT * G::STRIDE)[tid] = q0 + tid < S ? -pre_l : -INFINITY;
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
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < lo || r >= hi) continue;
            if (MODE == 0) dst[r] += __builtin_amdgcn_exp2f(fmaf(raw[r], c2, nl[r]));
            else dst[r] += fmaxf(raw[r], 0.f);
        }
    };

    // carry: the last tile of the previous head, added while this head's fragments arrive from LDS
    f32x16 carry = {0};
    float carry_nl[16];
    bool have_carry = false;
#pragma unroll
    for (int r = 0; r < 16; ++r) carry_nl[r] = -INFINITY;

    fetch(0);
    stash(0);
    for (int h = 0; h < p.H; ++h) {
        __syncthreads();  // stage h is complete; every wave is done reading stage h-1
        const bool more = h + 1 < p.H;
        if (more) fetch(h + 1);
        const char* sq = smem + (h & 1) * G::STAGE_BYTES;
        const char* sk = sq + G::TT * G::STRIDE;
        const float* sl = reinterpret_cast<const float*>(sq + 2 * G::TT * G::STRIDE);
        u32x4 qf[NSQ][G::NCH], kf[NSK][G::NCH];
        float nl[NSQ][16] = {};
#pragma unroll
        for (int c = 0; c < G::NCH; ++c) {
#pragma unroll
            for (int s = 0; s < NSQ; ++s) qf[s][c] = *reinterpret_cast<const u32x4*>(&sq[((wq * NSQ + s) * 32 + l32) * G::STRIDE + c * 32 + half * 16]);
#pragma unroll
            for (int s = 0; s < NSK; ++s) kf[s][c] = *reinterpret_cast<const u32x4*>(&sk[((wk * NSK + s) * 32 + l32) * G::STRIDE + c * 32 + half * 16]);
        }
        if (MODE == 0) {
#pragma unroll
            for (int s = 0; s < NSQ; ++s)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {  // rows 8*gq + 4*half + 0..3 of query subtile s
                    const f32x4 v = *reinterpret_cast<const f32x4*>(&sl[(wq * NSQ + s) * 32 + gq * 8 + half * 4]);
                    nl[s][gq * 4 + 0] = v[0]; nl[s][gq * 4 + 1] = v[1]; nl[s][gq * 4 + 2] = v[2]; nl[s][gq * 4 + 3] = v[3];
                }
        }
        if (have_carry) {  // vector work that covers the LDS latency of the reads above
#pragma unroll
            for (int c = 0; c < 4; ++c) accumulate(sbar[NSQ - 1][NSK - 1], carry, carry_nl, c, 4);
        }
        // tiles of this head in the order (0,0), (0,1), ..: the accumulation of one tile is issued slice by slice
        // between the MFMAs of the next
        f32x16 prev = {0};
#pragma unroll
        for (int t = 0; t < NSQ * NSK; ++t) {
            const int qs = t / NSK, ks = t % NSK;
            const int pq = (t + NSQ * NSK - 1) % (NSQ * NSK) / NSK, pk = (t + NSQ * NSK - 1) % (NSQ * NSK) % NSK;  // the tile before
            f32x16 acc = {0};
            sb_fence();
#pragma unroll
            for (int c = 0; c < G::NCH; ++c) {
                if (t > 0) accumulate(sbar[pq][pk], prev, nl[pq], c, G::NCH);
                mma_chunk<T>(acc, qf[qs][c], kf[ks][c]);  // acc[query row][key col]
                sb_fence();
            }
            prev = acc;
        }
        carry = prev;
#pragma unroll
        for (int r = 0; r < 16; ++r) carry_nl[r] = nl[NSQ - 1][r];
        have_carry = true;
        if (more) stash((h + 1) & 1);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) accumulate(sbar[NSQ - 1][NSK - 1], carry, carry_nl, c, 4);

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
