// Selective-load GEMM (Sec. 4.4): Y[m,:] = X[kept_idx[m],:] . W^T (+ bias).  The kept rows are read
// straight from the [S,C] input inside the A-tile load -- a kept row is C contiguous elements, so the
// indexed load is as coalesced as a dense one and no compacted copy of X ever exists.
//
// 256 x 256 output tile per workgroup, 4 waves in a 2 x 2 grid, each wave 128 x 128 = 4 x 4 MFMA tiles
// of 32 x 32 (256 accumulator registers per lane).  K advances 128 bytes per stage (64 bf16 / 32 fp32)
// through two LDS stages; the next stage's global loads are issued before the current stage's MFMAs.
// Both operands are K-contiguous in memory (X rows, nn.Linear weight rows), which is exactly the
// per-lane 16-byte fragment the 32x32 MFMAs take, so neither needs a transpose.
#include <mutex>
#include <type_traits>

#include "lemo_common.hpp"

namespace lemo {

constexpr int GG_THREADS = 256;
constexpr int GG_BM = 256, GG_BN = 256;
constexpr int GG_KB = 128;               // bytes of the contraction axis per stage and row
constexpr int GG_STRIDE = GG_KB + 16;    // LDS row pitch (16 consecutive rows -> 16 distinct bank groups)
constexpr int GG_NCH = GG_KB / 32;       // MFMA chunks per stage
constexpr int GG_CPR = GG_KB / 16;       // 16-byte pieces per row per stage
constexpr int GG_STAGE = (GG_BM + GG_BN) * GG_STRIDE;
constexpr int GG_LDS = 2 * GG_STAGE;     // 147456 bytes of the CU's 160 KB
constexpr int GG_NLD = GG_BM * GG_CPR / GG_THREADS;  // 8 loads per thread per operand per stage
#ifndef LEMO_GG_GROUP_M
#define LEMO_GG_GROUP_M 4
#endif
#ifndef LEMO_GG_EARLY_BARRIER
#define LEMO_GG_EARLY_BARRIER 1
#endif
constexpr int GG_GROUP_M = LEMO_GG_GROUP_M;  // tile rows walked together (4 keeps a die's 32 tiles to a 4 x 8 patch)

// How the operands lie in memory (an MFMA lane always wants 8 consecutive contraction elements of one operand row):
//   GG_NT  A rows and B rows run along the contraction (X[idx] [M,C] against an nn.Linear weight [N,C]); 16-byte reads.
//   GG_NN  A as above; B is stored contraction-major, [C, N] (the same weight used the other way round, as the input
//          gradient needs it).  Its slabs go to LDS as they are, 64 contraction rows x 256 columns, and the fragments
//          come out through the transposing LDS read (ds_read_b64_tr_b16: inside a group of 16 lanes, lane l receives
//          element l % 4 of the 8 bytes addressed by lanes l / 4, 4 + l / 4, 8 + l / 4 and 12 + l / 4 -- with lane
//          4 j + q pointed at row j, column quad q of a 4-row x 16-column block, lane l gets 4 consecutive rows of
//          column l).  Two such reads make one 16-byte fragment: the same bytes from LDS as before, no transposed copy
//          anywhere.
//   GG_TN  both operands contraction-major: A [C, M], B [C, N] with B's rows picked by idx (the weight gradient: the
//          contraction runs over the kept tokens).  bf16 only for GG_NN and GG_TN.
enum { GG_NT = 0, GG_NN = 1, GG_TN = 2 };
constexpr int GG_KROWS = 64;             // contraction rows per slab of a contraction-major operand
constexpr int GG_KPITCH = 512 + 32;      // LDS pitch of such a row (256 columns + pad): 136 dwords, so the 4 rows x 4 column
                                         // quads one 16-lane group reads fall into 32 distinct banks
static_assert(GG_KROWS * GG_KPITCH <= GG_BM * GG_STRIDE, "a contraction-major slab must fit the operand's LDS region");
typedef __attribute__((ext_vector_type(4))) short s16x4;

// exchange with the neighbouring lane (l ^ 1) inside a quad: DPP quad_perm [1,0,3,2]
__device__ __forceinline__ float swap_with_neighbour(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
}

// ADD = false: Y[m,:] = result row m.
// ADD = true:  Y is the residual stream [out_rows, N]; result row m is ADDED in place to row oidx[m] (row m when
//              oidx is null) -- the zero padding and the residual addition of Sec. 4.4 in one step, one rounding.
// GG_TN: `w_bytes_all` is the span of the whole B tensor (its rows are picked by idx); unused otherwise.
template <typename T, bool ADD, int LAYOUT>
__global__ __launch_bounds__(GG_THREADS, 1) void gather_gemm_kernel(const T* __restrict__ X, long long ldx,
                                                                    const int* __restrict__ idx, long long M,
                                                                    const T* __restrict__ W, long long ldw,
                                                                    const T* __restrict__ bias, T* __restrict__ Y,
                                                                    long long ldy, int C, int N, int tiles_m, int tiles_n,
                                                                    unsigned x_bytes, const int* __restrict__ oidx,
                                                                    long long out_rows, unsigned r_bytes, unsigned w_bytes_all) {
    static_assert(LAYOUT == GG_NT || sizeof(T) == 2, "the contraction-major layouts are built for 16-bit elements");
    constexpr bool A_KMAJOR = LAYOUT == GG_TN, B_KMAJOR = LAYOUT != GG_NT;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // tile assignment: die x = b % 8 takes a contiguous run of tiles in grouped order (GROUP_M tile rows
    // at a time, column by column), so the tiles resident on one die share X rows and W rows through L2
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + NUM_XCD - 1) / NUM_XCD;
    const int b = blockIdx.x;
    const int tile = (b % NUM_XCD) * per_xcd + b / NUM_XCD;
    if (b / NUM_XCD >= per_xcd || tile >= total) return;
    const int group = tile / (GG_GROUP_M * tiles_n);
    const int first_m = group * GG_GROUP_M;
    const int rows_in_group = min(GG_GROUP_M, tiles_m - first_m);
    const int within = tile - group * GG_GROUP_M * tiles_n;
    const int tm = first_m + within % rows_in_group, tn = within / rows_in_group;
    const long long m0 = (long long)tm * GG_BM;
    const int n0 = tn * GG_BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int wm = wave >> 1, wn = wave & 1;
    const int cbytes = C * (int)sizeof(T);

    // rows this thread stages: piece i*256+tid -> tile row i*32 + tid/8, 16-byte piece tid%8.
    // Both operands are read through buffer descriptors (X: the whole [S,C] tensor, rows picked by kept_idx;
    // W: this tile's rows): a 32-bit per-thread offset plus a scalar offset per load, no vector address
    // arithmetic, so the steady state has no branches.  The hardware range check compares the PER-THREAD offset
    // (plus the immediate) with the descriptor's size and ignores the scalar offset, so everything that can run
    // past the end -- the row -- sits in the per-thread offset: W rows at or past N are answered with zeros and
    // touch no memory.  The scalar offset only carries the slab's position inside a row, and a slab that does not
    // lie entirely inside C is never requested through it (see `slab`).  Rows past M are clamped to the last kept
    // row (computed, never stored).
    const int prow = tid >> 3, pcc = tid & 7;
    const int ldx_bytes = (int)ldx * (int)sizeof(T), ldw_bytes = (int)ldw * (int)sizeof(T);  // host: both < 2^23
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(X)), 0, (int)x_bytes, 0x00020000);
    // A contraction-major operand is staged slab by slab as it lies in memory: piece i*256+tid -> contraction row
    // i*8 + tid/32 of the slab, 16-byte piece tid%32 of the tile's 256 columns.  Its descriptor is rebuilt per slab: it
    // starts at the slab's first row (and the tile's first column) and ends with the operand's last row, so rows past
    // the end of the contraction are refused by the range check and arrive as zeros, and a slab past the end gets a
    // descriptor of size zero.  (Columns past the operand's width are only refused in the last row; elsewhere they
    // read the neighbouring row's first elements, which only ever reach output columns that are not stored.)
    const int krow = tid >> 5, kpiece = tid & 31;
    auto kmajor_rsrc = [&](const T* base, long long ld, long long col0, long long ncols, int kslab) {
        const long long k0 = (long long)kslab * GG_KROWS;
        long long span = k0 < C ? ((C - k0 - 1) * ld + (ncols - col0)) * (long long)sizeof(T) : 0;  // host: the operand spans < 2^31 bytes
        if (span < 0) span = 0;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(reinterpret_cast<const char*>(base + k0 * ld + col0)), 0, (int)span, 0x00020000);
    };
    unsigned a_voff[GG_NLD];
#pragma unroll
    for (int i = 0; i < GG_NLD; ++i) {
        if constexpr (A_KMAJOR) {
            a_voff[i] = (unsigned)(i * 8 + krow) * (unsigned)ldx_bytes + kpiece * 16;
        } else {
            const long long m = min(m0 + i * 32 + prow, M - 1);
            const unsigned row = idx ? (unsigned)idx[m] : (unsigned)m;
            a_voff[i] = row * (unsigned)ldx_bytes + pcc * 16;  // host guarantees S * ldx * sizeof(T) < 2^32
        }
    }
    const int b_rows = min(GG_BN, N - n0);
    const int w_bytes = (b_rows - 1) * ldw_bytes + cbytes;  // (GG_NT) this tile's rows of W, up to the end of the last one
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(W + (LAYOUT == GG_NT ? (long long)n0 * ldw : 0ll))), 0,
        LAYOUT == GG_TN ? (int)w_bytes_all : w_bytes, 0x00020000);
    int b_voff[GG_NLD];
#pragma unroll
    for (int i = 0; i < GG_NLD; ++i) {
        if constexpr (LAYOUT == GG_NT) b_voff[i] = (i * 32 + prow) * ldw_bytes + pcc * 16;  // at or past w_bytes for rows >= b_rows
        else if constexpr (LAYOUT == GG_NN) b_voff[i] = (i * 8 + krow) * ldw_bytes + kpiece * 16;
        else b_voff[i] = (int)w_bytes_all;  // GG_TN: set per slab from the kept rows' indices (refused until then)
    }
    // GG_TN: the rows of B are the kept tokens of the slab, idx[slab * 64 + i*8 + krow]; their indices are fetched one
    // slab ahead of the rows (tokn holds those of the slab that is requested next), tokens past the end are refused
    unsigned tokn[LAYOUT == GG_TN ? GG_NLD : 1];
    auto load_tokens = [&](int kslab) {
        if constexpr (LAYOUT == GG_TN) {
#pragma unroll
            for (int i = 0; i < GG_NLD; ++i) {
                const long long m = (long long)kslab * GG_KROWS + i * 8 + krow;
                const long long mc = min(m, (long long)C - 1);
                const unsigned row = idx ? (unsigned)idx[mc] : (unsigned)mc;
                tokn[i] = m < C ? row * (unsigned)ldw_bytes + (unsigned)n0 * 2u + (unsigned)kpiece * 16u : w_bytes_all;
            }
        }
    };
    auto take_tokens = [&]() {
        if constexpr (LAYOUT == GG_TN) {
#pragma unroll
            for (int i = 0; i < GG_NLD; ++i) b_voff[i] = (int)tokn[i];
        }
    };

    // Global loads take longer than one slab of MFMAs, so two slabs are kept in flight: the pieces of slab s
    // live in register set s & 1 from the moment they are requested (during slab s-2) until they are written
    // to LDS (during slab s-1).
    u32x4 pa[2][GG_NLD], pb[2][GG_NLD];
    // pieces of one slab, all at once (prologue and the ragged last slab: pieces past C are zero in BOTH operands)
    auto fetch = [&](int kslab, auto set_tag) {  // GG_TN: b_voff must hold the slab's rows (take_tokens)
        constexpr int SET = decltype(set_tag)::value;
        const int kbyte = kslab * GG_KB;
        const bool in_k = kbyte + pcc * 16 + 16 <= cbytes;  // C is a multiple of 16 bytes: a piece is all in or all out
        const __amdgpu_buffer_rsrc_t a_k = kmajor_rsrc(X, ldx, m0, M, kslab), b_k = kmajor_rsrc(W, ldw, n0, N, kslab);
#pragma unroll
        for (int i = 0; i < GG_NLD; ++i) {
            pa[SET][i] = u32x4{0u, 0u, 0u, 0u};
            pb[SET][i] = u32x4{0u, 0u, 0u, 0u};
            if constexpr (A_KMAJOR) pa[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(a_k, (int)a_voff[i], 0, 0);
            else if (in_k) pa[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)a_voff[i], kbyte, 0);
            if constexpr (LAYOUT == GG_NN) pb[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(b_k, b_voff[i], 0, 0);
            else if constexpr (LAYOUT == GG_TN) pb[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, b_voff[i], 0, 0);
            else if (in_k) pb[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, b_voff[i], kbyte, 0);
        }
    };
    // where this thread's pieces go in an operand's LDS region
    const int st_off = prow * GG_STRIDE + pcc * 16;        // + i * 32 rows: row-major along the contraction
    const int st_koff = krow * GG_KPITCH + kpiece * 16;    // + i * 8 rows: contraction-major
    auto a_store = [&](char* stage, int i, const u32x4& v) {
        if constexpr (A_KMAJOR) *reinterpret_cast<u32x4*>(stage + st_koff + i * 8 * GG_KPITCH) = v;
        else *reinterpret_cast<u32x4*>(stage + st_off + i * 32 * GG_STRIDE) = v;
    };
    auto b_store = [&](char* stage, int i, const u32x4& v) {
        if constexpr (B_KMAJOR) *reinterpret_cast<u32x4*>(stage + GG_BM * GG_STRIDE + st_koff + i * 8 * GG_KPITCH) = v;
        else *reinterpret_cast<u32x4*>(stage + GG_BM * GG_STRIDE + st_off + i * 32 * GG_STRIDE) = v;
    };
    // fragment (32-row subtile i of the wave's 128 rows, chunk c of the slab) of an operand
    const int tr_off = (8 * half + ((l32 & 15) >> 2)) * GG_KPITCH + ((l32 >> 4) * 16 + (l32 & 3) * 4) * 2;  // this lane's corner of a 4 x 16 block
    auto tr_frag = [&](const char* region, int col0, int c) {
        const char* at = region + tr_off + c * 16 * GG_KPITCH + col0 * 2;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(at));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(at + 4 * GG_KPITCH));
        const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
        return u32x4{l2.x, l2.y, h2.x, h2.y};
    };
    auto a_frag = [&](const char* stage, int i, int c) {
        if constexpr (A_KMAJOR) return tr_frag(stage, wm * 128 + i * 32, c);
        else return *reinterpret_cast<const u32x4*>(stage + (wm * 128 + l32) * GG_STRIDE + half * 16 + i * 32 * GG_STRIDE + c * 32);
    };
    auto b_frag = [&](const char* stage, int j, int c) {
        if constexpr (B_KMAJOR) return tr_frag(stage + GG_BM * GG_STRIDE, wn * 128 + j * 32, c);
        else return *reinterpret_cast<const u32x4*>(stage + GG_BM * GG_STRIDE + (wn * 128 + l32) * GG_STRIDE + half * 16 + j * 32 * GG_STRIDE + c * 32);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x16{0};

    // Main loop.  One wave per SIMD, so the overlap is written out: the source order below is the issue
    // order (scheduling fences), one memory instruction between consecutive MFMAs.
    //   every third MFMA of chunks 0-2: one global load of the slab after next (almost two slabs to arrive)
    //   the MFMA after it: one LDS write of the next slab (requested during the previous slab)
    //   chunks 0-2: LDS reads of the next chunk's fragments;  after chunk 3: barrier, then the next slab's first chunk
    const int nk = (cbytes + GG_KB - 1) / GG_KB;
    const int nfull = cbytes / GG_KB;  // slabs that lie entirely inside C
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    load_tokens(0);
    take_tokens();
    load_tokens(1);
    fetch(0, I0{});
#pragma unroll
    for (int i = 0; i < GG_NLD; ++i) {
        a_store(smem, i, pa[0][i]);
        b_store(smem, i, pb[0][i]);
    }
    take_tokens();
    load_tokens(2);
    fetch(1, I1{});  // slab 1 (all zero if there is none)
    __syncthreads();
    u32x4 fa[4], fb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        fa[i] = a_frag(smem, i, 0);
        fb[i] = b_frag(smem, i, 0);
    }
    // One slab kt of the contraction, kt & 1 == PAR.  It always moves set PAR^1 (slab kt+1) to the other LDS
    // stage and always requests slab kt+2 into set PAR.  When slab kt+1 does not exist the writes land in a
    // stage nobody reads again.  When slab kt+2 does not lie entirely inside C (it is the ragged last slab, which
    // `fetch` brings in with its pieces past C zeroed, or there is none) the requests go through descriptors of
    // size zero: they are answered with zeros and read nothing, neither past the end of a row nor past the end
    // of X or W.
    auto slab = [&](int kt, auto par_tag) {
        constexpr int PAR = decltype(par_tag)::value;
        const char* cur = smem + PAR * GG_STAGE;
        char* nxt = smem + (PAR ^ 1) * GG_STAGE;
        const int kbyte = (kt + 2) * GG_KB;
        const bool live = kt + 2 < nfull;
        const __amdgpu_buffer_rsrc_t a_req = A_KMAJOR ? kmajor_rsrc(X, ldx, m0, M, kt + 2) : __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char*>(reinterpret_cast<const char*>(X)), 0, live ? (int)x_bytes : 0, 0x00020000);
        const __amdgpu_buffer_rsrc_t b_req = LAYOUT == GG_NN ? kmajor_rsrc(W, ldw, n0, N, kt + 2) : LAYOUT == GG_TN ? b_rsrc : __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char*>(reinterpret_cast<const char*>(W + (long long)n0 * ldw)), 0, live ? w_bytes : 0, 0x00020000);
        const int a_soff = A_KMAJOR ? 0 : kbyte, b_soff = B_KMAJOR ? 0 : kbyte;
        take_tokens();         // GG_TN: the rows of slab kt+2, fetched during the slab before
        load_tokens(kt + 3);
#pragma unroll
        for (int c = 0; c < GG_NCH; ++c) {
            u32x4 nb[4];
            __builtin_amdgcn_sched_barrier(0);
#if LEMO_GG_EARLY_BARRIER
            // The slab's one barrier stands before its LAST chunk: by then this thread's LDS writes of slab kt+1 (the
            // last one follows MFMA 46 of 64) and its reads of this stage (the last chunk's fragments, read during the
            // chunk before) have been issued, and the barrier waits for them.  The last chunk's MFMAs then cover the
            // reads of the next slab's first fragments, which would otherwise stand between the barrier and an MFMA.
            if (c == GG_NCH - 1) {
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
#endif
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int q = i * 4 + j;  // position of this MFMA in the chunk
                    mma_chunk<T>(acc[i][j], fa[i], fb[j]);
                    // global loads and LDS writes are spread over the slab, one every third MFMA each: issued
                    // back to back by all four waves they would outrun the vector-memory and LDS pipes
                    const int g = c * 16 + q, slot = g / 3;
                    if (g % 3 == 0 && slot < 16) {  // request piece `slot` of slab kt+2: A pieces first, then B pieces
                        if (slot < 8) pa[PAR][slot] = __builtin_amdgcn_raw_buffer_load_b128(a_req, (int)a_voff[slot], a_soff, 0);
                        else pb[PAR][slot - 8] = __builtin_amdgcn_raw_buffer_load_b128(b_req, b_voff[slot - 8], b_soff, 0);
                    }
                    if (g % 3 == 1 && slot < 16) {  // move piece `slot` of slab kt+1 (requested during the previous slab) to LDS
                        if (slot < 8) a_store(nxt, slot, pa[PAR ^ 1][slot]);
                        else b_store(nxt, slot - 8, pb[PAR ^ 1][slot - 8]);
                    }
                    if (c < GG_NCH - 1) {
                        // fragments of the next chunk: row i of A is done after its fourth MFMA and is refilled in
                        // place; the B fragments are live to the end of the chunk, so they go to a second set
                        if (j == 3) fa[i] = a_frag(cur, i, c + 1);
                        if (i == 2) nb[j] = b_frag(cur, j, c + 1);
                    }
#if LEMO_GG_EARLY_BARRIER
                    else {  // behind the barrier: the first fragments of the next slab
                        if (j == 3) fa[i] = a_frag(nxt, i, 0);
                        if (i == 2) nb[j] = b_frag(nxt, j, 0);
                    }
#endif
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (LEMO_GG_EARLY_BARRIER || c < GG_NCH - 1) {
#pragma unroll
                for (int j = 0; j < 4; ++j) fb[j] = nb[j];
            }
        }
#if !LEMO_GG_EARLY_BARRIER
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[i] = a_frag(nxt, i, 0);
            fb[i] = b_frag(nxt, i, 0);
        }
#endif
    };
    // the ragged last slab (if any) is slab nfull; it must be fetched with zero fill once its register set is free
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        slab(kt, I0{});
        if (!A_KMAJOR && kt + 2 == nfull && nfull < nk) fetch(kt + 2, I0{});  // (never GG_TN: its b_voff runs ahead, and rows past the end are refused anyway)
        slab(kt + 1, I1{});
        if (!A_KMAJOR && kt + 3 == nfull && nfull < nk) fetch(kt + 3, I1{});
    }
    if (kt < nk) slab(kt, I0{});

    // epilogue of the in-place-add form.  Output row of result row m: oidx[m] (m itself without a list); rows whose
    // index falls outside [0, out_rows) are dropped.
    auto add_epilogue = [&]() {
        if constexpr (sizeof(T) == 2) {
            // The wave's 128 x 128 block goes through LDS in two halves of 64 rows, as binary32 (the residual is
            // added before the only rounding).  A lane then owns 8 consecutive columns of a row (16 lanes cover a
            // row's 256 bytes): two 16-byte LDS reads, the residual's 16 bytes, one 16-byte store.  The residual
            // rows are requested ahead -- half 0 before anything is staged, half 1 before half 0 is consumed -- so
            // that their latency is covered by the staging.
            constexpr int EPF = 128 * 4 + 16;  // LDS pitch of one staged row of 128 floats
            char* region = smem + wave * 64 * EPF;
            const bool vec_ok = ((ldy & 7) == 0) && ((reinterpret_cast<uintptr_t>(Y) & 15u) == 0);
            const int piece = lane & 15, rsub = lane >> 4;
            const int ncol = n0 + wn * 128 + piece * 8;
            const bool col_vec = vec_ok && ncol + 8 <= N;
            float bv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + wn * 128 + j * 32 + l32;
                bv[j] = (bias && n < N) ? bf16_to_f32(reinterpret_cast<const uint16_t*>(bias)[n]) : 0.f;
            }
            // Byte offset in R of this lane's piece of row (ih*64 + rr*4 + rsub), or NONE if it is not to be written.
            // All 32 row indices are fetched in one batch, and the residual is read through a range-checked buffer
            // descriptor (a NONE offset lies past its end and reads as zero), so nothing here branches or waits
            // between the loads.
            const unsigned NONE = r_bytes;
            const int ldy_bytes = (int)ldy * 2;
            const __amdgpu_buffer_rsrc_t r_rsrc = __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<char*>(Y), 0, (int)r_bytes, 0x00020000);
            int orow[2][16];
#pragma unroll
            for (int ih = 0; ih < 2; ++ih)
#pragma unroll
                for (int rr = 0; rr < 16; ++rr) {
                    const long long m = min(m0 + wm * 128 + ih * 64 + rr * 4 + rsub, M - 1);
                    orow[ih][rr] = oidx ? oidx[m] : (int)m;
                }
            unsigned roff[2][16];
#pragma unroll
            for (int ih = 0; ih < 2; ++ih)
#pragma unroll
                for (int rr = 0; rr < 16; ++rr) {
                    const long long m = m0 + wm * 128 + ih * 64 + rr * 4 + rsub;
                    const bool ok = (m < M) & (ncol < N) & (orow[ih][rr] >= 0) & (orow[ih][rr] < out_rows);  // no short circuit: no branches
                    roff[ih][rr] = ok ? (unsigned)orow[ih][rr] * (unsigned)ldy_bytes + (unsigned)ncol * 2u : NONE;
                }
            auto prefetch = [&](int ih, u32x4 (&old)[16]) {
#pragma unroll
                for (int rr = 0; rr < 16; ++rr)
                    old[rr] = __builtin_amdgcn_raw_buffer_load_b128(r_rsrc, (int)(col_vec ? roff[ih][rr] : NONE), 0, 0);
            };
            auto stage = [&](int ih) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    char* colp = region + (4 * half) * EPF + (j * 32 + l32) * 4;
#pragma unroll
                    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            *reinterpret_cast<float*>(colp + (ii * 32 + 8 * (r >> 2) + (r & 3)) * EPF) = acc[ih * 2 + ii][j][r] + bv[j];
                }
            };
            auto consume = [&](int ih, const u32x4 (&old)[16]) {
#pragma unroll
                for (int rr = 0; rr < 16; ++rr) {
                    const int row = rr * 4 + rsub;
                    const f32x4 lo = *reinterpret_cast<const f32x4*>(region + row * EPF + piece * 32);
                    const f32x4 hi = *reinterpret_cast<const f32x4*>(region + row * EPF + piece * 32 + 16);
                    if (roff[ih][rr] == NONE) continue;
                    uint16_t* dst = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(Y) + roff[ih][rr]);
                    const float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    if (col_vec) {
                        u32x4 out;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            out[e] = pack_bf16x2_hw(v[2 * e] + __uint_as_float(old[rr][e] << 16),
                                                    v[2 * e + 1] + __uint_as_float(old[rr][e] & 0xffff0000u));
                        *reinterpret_cast<u32x4*>(dst) = out;
                    } else {  // ragged right edge or unaligned rows: element by element
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (ncol + e < N) dst[e] = (uint16_t)(pack_bf16x2_hw(v[e] + bf16_to_f32(dst[e]), 0.f) & 0xffffu);
                    }
                }
            };
            u32x4 old0[16], old1[16];
            prefetch(0, old0);
            stage(0);
            prefetch(1, old1);
            consume(0, old0);
            stage(1);
            consume(1, old1);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + wn * 128 + j * 32 + l32;
                const float bv = (bias && n < N) ? reinterpret_cast<const float*>(bias)[n] : 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const long long mbase = m0 + wm * 128 + i * 32;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const long long m = mbase + acc_row(r, lane);
                        if (m < M && n < N) {
                            const long long orow = oidx ? (long long)oidx[m] : m;
                            if (orow >= 0 && orow < out_rows) {
                                float* dst = reinterpret_cast<float*>(Y) + orow * ldy + n;
                                *dst = *dst + (acc[i][j][r] + bv);
                            }
                        }
                    }
                }
            }
        }
    };

    // epilogue: acc[i][j][r] is Y[m0 + wm*128 + i*32 + acc_row(r), n0 + wn*128 + j*32 + l32]
    if constexpr (ADD) {
        add_epilogue();
    } else if constexpr (sizeof(T) == 2) {
        // bf16: a lane holds ONE column of 16 rows, so storing from the accumulators would write 2-4 bytes per
        // lane into many rows.  Each wave instead lays its 128 x 128 block out in LDS (its own region; the
        // main loop's stages are dead after the last barrier) and writes whole 256-byte row segments.
        constexpr int EP = 128 * 2 + 16;  // LDS pitch of one staged row
        char* region = smem + wave * 128 * EP;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn * 128 + j * 32 + l32;
            const float bv = (bias && n < N) ? bf16_to_f32(reinterpret_cast<const uint16_t*>(bias)[n]) : 0.f;
            char* colp = region + (4 * half) * EP + (j * 32 + l32) * 2;  // this lane's column, first of its rows
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    // registers r and r+1 are two consecutive rows of this lane's column: one conversion
                    // instruction rounds both, the two halves go to the two rows
                    const uint32_t word = pack_bf16x2_hw(acc[i][j][r] + bv, acc[i][j][r + 1] + bv);
                    const int row = i * 32 + 8 * (r >> 2) + (r & 3);
                    *reinterpret_cast<uint16_t*>(colp + row * EP) = (uint16_t)(word & 0xffffu);
                    *reinterpret_cast<uint16_t*>(colp + (row + 1) * EP) = (uint16_t)(word >> 16);
                }
            }
        }
        // the region is private to the wave; its LDS writes are complete before its own reads (same wave, in order)
        const bool vec_ok = ((ldy & 7) == 0) && ((reinterpret_cast<uintptr_t>(Y) & 15u) == 0);
        const int piece = lane & 15, rsub = lane >> 4;
        const int ncol = n0 + wn * 128 + piece * 8;
#pragma unroll 4
        for (int rr = 0; rr < 32; ++rr) {
            const int row = rr * 4 + rsub;
            const long long m = m0 + wm * 128 + row;
            const u32x4 v = *reinterpret_cast<const u32x4*>(region + row * EP + piece * 16);
            if (m < M) {
                uint16_t* dst = reinterpret_cast<uint16_t*>(Y) + m * ldy + ncol;
                if (vec_ok && ncol + 8 <= N) {
                    *reinterpret_cast<u32x4*>(dst) = v;
                } else {  // ragged right edge or unaligned rows: element stores
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (ncol + e < N) dst[e] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
                }
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn * 128 + j * 32 + l32;
            const float bv = (bias && n < N) ? reinterpret_cast<const float*>(bias)[n] : 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const long long mbase = m0 + wm * 128 + i * 32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long long m = mbase + acc_row(r, lane);
                    if (m < M && n < N) reinterpret_cast<float*>(Y)[m * ldy + n] = acc[i][j][r] + bv;
                }
            }
        }
    }
}

template <typename T, bool ADD, int LAYOUT = GG_NT>
static int launch_gg_t(const void* X, long long S, long long ldx, const int* idx, long long M, const void* W, long long ldw,
                       const void* bias, void* Y, long long ldy, int C, int N, const int* oidx, long long out_rows, hipStream_t st,
                       unsigned w_bytes_all = 0) {
    const unsigned x_bytes = (unsigned)(((S - 1) * ldx + (LAYOUT == GG_TN ? M : (long long)C)) * (long long)sizeof(T));  // host checked: fits 32 bits
    const unsigned r_bytes = ADD ? (unsigned)(((out_rows - 1) * ldy + N) * (long long)sizeof(T)) : 0u;  // likewise
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_gemm_kernel<T, ADD, LAYOUT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, GG_LDS);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    const int tiles_m = (int)((M + GG_BM - 1) / GG_BM), tiles_n = (N + GG_BN - 1) / GG_BN;
    const int per_xcd = (tiles_m * tiles_n + NUM_XCD - 1) / NUM_XCD;
    hipLaunchKernelGGL((gather_gemm_kernel<T, ADD, LAYOUT>), dim3((unsigned)(per_xcd * NUM_XCD)), dim3(GG_THREADS), GG_LDS, st,
                       static_cast<const T*>(X), ldx, idx, M, static_cast<const T*>(W), ldw, static_cast<const T*>(bias),
                       static_cast<T*>(Y), ldy, C, N, tiles_m, tiles_n, x_bytes, oidx, out_rows, r_bytes, w_bytes_all);
    return (int)hipGetLastError();
}

int launch_gather_gemm(const void* X, long long S, long long ldx, const int* idx, long long M, const void* W, long long ldw,
                       const void* bias, void* Y, long long ldy, int C, int N, lemo_dtype_t dt, hipStream_t st) {
    if (M == 0) return 0;
    if (dt == LEMO_BF16) return launch_gg_t<bf16_t, false>(X, S, ldx, idx, M, W, ldw, bias, Y, ldy, C, N, nullptr, 0, st);
    return launch_gg_t<float, false>(X, S, ldx, idx, M, W, ldw, bias, Y, ldy, C, N, nullptr, 0, st);
}

int launch_gather_gemm_add(const void* X, long long S, long long ldx, const int* idx, long long M, const void* W, long long ldw,
                           const void* bias, void* R, long long ldr, long long out_rows, const int* oidx, int C, int N,
                           lemo_dtype_t dt, hipStream_t st) {
    if (M == 0) return 0;
    if (dt == LEMO_BF16) return launch_gg_t<bf16_t, true>(X, S, ldx, idx, M, W, ldw, bias, R, ldr, C, N, oidx, out_rows, st);
    return launch_gg_t<float, true>(X, S, ldx, idx, M, W, ldw, bias, R, ldr, C, N, oidx, out_rows, st);
}

// Input gradient of Y = X[idx] W^T:  dX[oidx[m], c] += sum_n dY[m, n] W[n, c], W as stored ([N, C], contraction-major
// for this product).  bf16.  dY [M, N] compact rows; dX [out_rows, C].
int launch_gather_gemm_dx(const void* dY, long long ldy, long long M, const void* W, long long ldw, void* dX, long long lddx, long long out_rows,
                          const int* oidx, int C, int N, hipStream_t st) {
    if (M == 0) return 0;
    return launch_gg_t<bf16_t, true, GG_NN>(dY, M, ldy, nullptr, M, W, ldw, nullptr, dX, lddx, /*contraction*/ N, /*columns*/ C, oidx, out_rows, st);
}

// Weight gradient dW[n, c] = sum_m dY[m, n] X[idx[m], c], both operands read as they are stored (contraction-major),
// the kept rows of X picked inside the B-tile load.  bf16.
int launch_gather_gemm_dw_direct(const void* dY, long long ldy, const void* X, long long S, long long ldx, const int* idx, long long M, void* dW,
                                 long long lddw, int C, int N, hipStream_t st) {
    const unsigned x_span = (unsigned)(((S - 1) * ldx + C) * 2);  // host checked: fits 32 bits
    return launch_gg_t<bf16_t, false, GG_TN>(dY, M, ldy, idx, /*output rows*/ N, X, ldx, nullptr, dW, lddw, /*contraction*/ (int)M, /*columns*/ C, nullptr, 0, st,
                                             x_span);
}

}  // namespace lemo
