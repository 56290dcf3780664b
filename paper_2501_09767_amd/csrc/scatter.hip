// In-place add at the kept positions (Sec. 4.4: padding and residual addition in one step); also the
// backward of the selective load.  HBM-bound: every byte of G is read once and every kept row of dX is
// read and written once, in 16-byte pieces, one workgroup per kept row.
//
// ZERO_PAD writes the zero-padded G instead: workgroup m also clears the rows strictly between
// kept_idx[m-1] and kept_idx[m] (the last one clears the tail), which needs kept_idx ascending.
#include "lemo_common.hpp"

namespace lemo {

constexpr int SCAT_THREADS = 256;

// eight consecutive elements as binary32
template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
        const uint4 u = *reinterpret_cast<const uint4*>(p);
        v[0] = bf16lo_to_f32(u.x); v[1] = bf16hi_to_f32(u.x); v[2] = bf16lo_to_f32(u.y); v[3] = bf16hi_to_f32(u.y);
        v[4] = bf16lo_to_f32(u.z); v[5] = bf16hi_to_f32(u.z); v[6] = bf16lo_to_f32(u.w); v[7] = bf16hi_to_f32(u.w);
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
        uint4 u;
        u.x = pack_bf16x2(v[0], v[1]); u.y = pack_bf16x2(v[2], v[3]); u.z = pack_bf16x2(v[4], v[5]); u.w = pack_bf16x2(v[6], v[7]);
        *reinterpret_cast<uint4*>(p) = u;
    }
};
template <> struct Vec8<float> {
    static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
        const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
        reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
        reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
    }
};

template <typename TG, typename TX, bool ZERO_PAD>
__global__ __launch_bounds__(SCAT_THREADS) void scatter_rows_kernel(const TG* __restrict__ G, long long ldg,
                                                                    const int* __restrict__ idx, long long M,
                                                                    TX* __restrict__ dX, long long lddx, long long S, int C) {
    const long long m = blockIdx.x;  // ACCUMULATE: grid = M;  ZERO_PAD: grid = M + 1 (the extra one clears the tail)
    const int nvec = C >> 3;
    if (ZERO_PAD) {
        const long long lo = m == 0 ? 0 : (long long)idx[m - 1] + 1;
        const long long hi = m < M ? (long long)idx[m] : S;
        const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (long long r = lo; r < hi; ++r)
            for (int v = threadIdx.x; v < nvec; v += SCAT_THREADS) Vec8<TX>::store(dX + r * lddx + (long long)v * 8, z);
        if (m >= M) return;
    }
    const long long row = idx[m];
    const TG* g = G + m * ldg;
    TX* x = dX + row * lddx;
    for (int v = threadIdx.x; v < nvec; v += SCAT_THREADS) {
        float a[8], b[8];
        Vec8<TG>::load(g + (long long)v * 8, a);
        if (ZERO_PAD) {
#pragma unroll
            for (int e = 0; e < 8; ++e) b[e] = 0.f + a[e];  // the same add the accumulate path does on a +0 row
        } else {
            Vec8<TX>::load(x + (long long)v * 8, b);
#pragma unroll
            for (int e = 0; e < 8; ++e) b[e] = b[e] + a[e];
        }
        Vec8<TX>::store(x + (long long)v * 8, b);
    }
}

template <typename TG, typename TX>
static int launch_scatter_t(const void* G, long long ldg, const int* idx, long long M, void* dX, long long lddx, long long S,
                            int C, int mode, hipStream_t st) {
    if (mode == LEMO_SCATTER_ZERO_PAD)
        hipLaunchKernelGGL((scatter_rows_kernel<TG, TX, true>), dim3((unsigned)(M + 1)), dim3(SCAT_THREADS), 0, st,
                           static_cast<const TG*>(G), ldg, idx, M, static_cast<TX*>(dX), lddx, S, C);
    else if (M > 0)
        hipLaunchKernelGGL((scatter_rows_kernel<TG, TX, false>), dim3((unsigned)M), dim3(SCAT_THREADS), 0, st,
                           static_cast<const TG*>(G), ldg, idx, M, static_cast<TX*>(dX), lddx, S, C);
    return (int)hipGetLastError();
}

int launch_scatter(const void* G, long long ldg, const int* idx, long long M, void* dX, long long lddx, long long S, int C,
                   lemo_dtype_t g_dt, lemo_dtype_t dx_dt, int mode, hipStream_t st) {
    if (g_dt == LEMO_BF16 && dx_dt == LEMO_BF16) return launch_scatter_t<bf16_t, bf16_t>(G, ldg, idx, M, dX, lddx, S, C, mode, st);
    if (g_dt == LEMO_BF16 && dx_dt == LEMO_F32) return launch_scatter_t<bf16_t, float>(G, ldg, idx, M, dX, lddx, S, C, mode, st);
    if (g_dt == LEMO_F32 && dx_dt == LEMO_BF16) return launch_scatter_t<float, bf16_t>(G, ldg, idx, M, dX, lddx, S, C, mode, st);
    return launch_scatter_t<float, float>(G, ldg, idx, M, dX, lddx, S, C, mode, st);
}

}  // namespace lemo
