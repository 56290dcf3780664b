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
constexpr int GG_GROUP_M = 4;            // tile rows walked together (keeps a die's 32 tiles to a 4 x 8 patch)

// exchange with the neighbouring lane (l ^ 1) inside a quad: DPP quad_perm [1,0,3,2]
__device__ __forceinline__ float swap_with_neighbour(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
}

template <typename T>
__global__ __launch_bounds__(GG_THREADS, 1) void gather_gemm_kernel(const T* __restrict__ X, long long ldx,
                                                                    const int* __restrict__ idx, long long M,
                                                                    const T* __restrict__ W, long long ldw,
                                                                    const T* __restrict__ bias, T* __restrict__ Y,
                                                                    long long ldy, int C, int N, int tiles_m, int tiles_n) {
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

    // rows this thread stages: piece i*256+tid -> tile row i*32 + tid/8, 16-byte piece tid%8
    const int prow = tid >> 3, pcc = tid & 7;
    const char* a_ptr[GG_NLD];
    const char* b_ptr[GG_NLD];
#pragma unroll
    for (int i = 0; i < GG_NLD; ++i) {
        const long long m = m0 + i * 32 + prow;
        a_ptr[i] = nullptr;
        if (m < M) {
            const long long row = idx ? (long long)idx[m] : m;
            a_ptr[i] = reinterpret_cast<const char*>(X + row * ldx) + pcc * 16;
        }
        const int n = n0 + i * 32 + prow;
        b_ptr[i] = n < N ? reinterpret_cast<const char*>(W + (long long)n * ldw) + pcc * 16 : nullptr;
    }

    u32x4 pa[GG_NLD], pb[GG_NLD];
    auto fetch = [&](int kbyte) {
        const bool in_k = kbyte + pcc * 16 + 16 <= cbytes;  // C is a multiple of 16 bytes: a piece is all in or all out
#pragma unroll
        for (int i = 0; i < GG_NLD; ++i) {
            pa[i] = u32x4{0u, 0u, 0u, 0u};
            pb[i] = u32x4{0u, 0u, 0u, 0u};
            if (in_k && a_ptr[i]) pa[i] = *reinterpret_cast<const u32x4*>(a_ptr[i] + kbyte);
            if (in_k && b_ptr[i]) pb[i] = *reinterpret_cast<const u32x4*>(b_ptr[i] + kbyte);
        }
    };
    auto stash = [&](int buf) {
        char* sA = smem + buf * GG_STAGE;
        char* sB = sA + GG_BM * GG_STRIDE;
#pragma unroll
        for (int i = 0; i < GG_NLD; ++i) {
            *reinterpret_cast<u32x4*>(sA + (i * 32 + prow) * GG_STRIDE + pcc * 16) = pa[i];
            *reinterpret_cast<u32x4*>(sB + (i * 32 + prow) * GG_STRIDE + pcc * 16) = pb[i];
        }
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x16{0};

    const int nk = (cbytes + GG_KB - 1) / GG_KB;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) fetch((kt + 1) * GG_KB);
        const char* sA = smem + (kt & 1) * GG_STAGE + (wm * 128 + l32) * GG_STRIDE + half * 16;
        const char* sB = smem + (kt & 1) * GG_STAGE + GG_BM * GG_STRIDE + (wn * 128 + l32) * GG_STRIDE + half * 16;
#pragma unroll
        for (int c = 0; c < GG_NCH; ++c) {
            u32x4 af[4], bf[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const u32x4*>(sA + i * 32 * GG_STRIDE + c * 32);
#pragma unroll
            for (int j = 0; j < 4; ++j) bf[j] = *reinterpret_cast<const u32x4*>(sB + j * 32 * GG_STRIDE + c * 32);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) mma_chunk<T>(acc[i][j], af[i], bf[j]);
        }
        if (more) stash((kt + 1) & 1);  // the other stage: last read before the barrier that ended iteration kt-1
        __syncthreads();
    }

    // epilogue: acc[i][j][r] is Y[m0 + wm*128 + i*32 + acc_row(r), n0 + wn*128 + j*32 + l32]
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n = n0 + wn * 128 + j * 32 + l32;
        float bv = 0.f;
        if (bias && n < N) {
            if constexpr (sizeof(T) == 2) bv = bf16_to_f32(reinterpret_cast<const uint16_t*>(bias)[n]);
            else bv = reinterpret_cast<const float*>(bias)[n];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const long long mbase = m0 + wm * 128 + i * 32;
            if constexpr (sizeof(T) == 2) {
                // neighbouring lanes hold neighbouring columns: trade one value so that each lane owns two
                // adjacent columns of ONE row and can store 4 bytes (even lane: row r, odd lane: row r+1)
                const bool odd = lane & 1;
                const int n_even = n & ~1;
                const bool pair_ok = ((ldy & 1) == 0) && ((reinterpret_cast<uintptr_t>(Y) & 3u) == 0);  // rows 4-byte aligned
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float v0 = acc[i][j][r] + bv, v1 = acc[i][j][r + 1] + bv;
                    const float got = swap_with_neighbour(odd ? v0 : v1);
                    const long long m = mbase + acc_row(odd ? r + 1 : r, lane);
                    const uint32_t word = odd ? pack_bf16x2(got, v1) : pack_bf16x2(v0, got);
                    if (m < M) {
                        uint16_t* dst = reinterpret_cast<uint16_t*>(Y) + m * ldy + n_even;
                        if (pair_ok && n_even + 1 < N) {
                            *reinterpret_cast<uint32_t*>(dst) = word;
                        } else {  // odd row pitch or last column of an odd N: element stores
                            if (n_even < N) dst[0] = (uint16_t)(word & 0xffffu);
                            if (n_even + 1 < N) dst[1] = (uint16_t)(word >> 16);
                        }
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long long m = mbase + acc_row(r, lane);
                    if (m < M && n < N) reinterpret_cast<float*>(Y)[m * ldy + n] = acc[i][j][r] + bv;
                }
            }
        }
    }
}

template <typename T>
static int launch_gg_t(const void* X, long long ldx, const int* idx, long long M, const void* W, long long ldw,
                       const void* bias, void* Y, long long ldy, int C, int N, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_gemm_kernel<T>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, GG_LDS);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    const int tiles_m = (int)((M + GG_BM - 1) / GG_BM), tiles_n = (N + GG_BN - 1) / GG_BN;
    const int per_xcd = (tiles_m * tiles_n + NUM_XCD - 1) / NUM_XCD;
    hipLaunchKernelGGL((gather_gemm_kernel<T>), dim3((unsigned)(per_xcd * NUM_XCD)), dim3(GG_THREADS), GG_LDS, st,
                       static_cast<const T*>(X), ldx, idx, M, static_cast<const T*>(W), ldw, static_cast<const T*>(bias),
                       static_cast<T*>(Y), ldy, C, N, tiles_m, tiles_n);
    return (int)hipGetLastError();
}

int launch_gather_gemm(const void* X, long long S, long long ldx, const int* idx, long long M, const void* W, long long ldw,
                       const void* bias, void* Y, long long ldy, int C, int N, lemo_dtype_t dt, hipStream_t st) {
    (void)S;
    if (M == 0) return 0;
    if (dt == LEMO_BF16) return launch_gg_t<bf16_t>(X, ldx, idx, M, W, ldw, bias, Y, ldy, C, N, st);
    return launch_gg_t<float>(X, ldx, idx, M, W, ldw, bias, Y, ldy, C, N, st);
}

}  // namespace lemo
