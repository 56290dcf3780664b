// Per-segment top-k (token-block elimination of Sec. 4.2 with a keep count instead of a threshold).
//
// One workgroup per segment.  The k-th largest score is found by an MSB-first radix select over the
// order-preserving uint32 image of the floats (4 passes of 8 bits, LDS histogram); the kept set is
// then { key > pivot } plus the first (k - #greater) elements with key == pivot in index order, which
// is exactly "ties go to the lower index".  A block-wide prefix sum in index order gives every kept
// element its output slot, so the indices come out ascending without a sort.  Integer work only:
// bit-exact and deterministic.
#include <mutex>

#include "lemo_common.hpp"

namespace lemo {

constexpr int SEL_THREADS = 256;

// monotone map float -> uint32 (larger float <=> larger key); -0.0 and +0.0 share a key
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// inclusive prefix sum over the 64 lanes of a wave (DPP-free: five shuffles and a last one across the halves)
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t u = __shfl_up(v, off);
        if (lane >= off) v += u;
    }
    return v;
}

// The selection proper, shared by the two kernels below: `keys` [len] (LDS) hold the order keys of one segment, the
// `keep` kept token indices go to kept[out0 ...) in ascending order.  T = threads of the workgroup (a multiple of 256);
// every thread of the workgroup must call it.  Scans run inside wavefronts (shuffles) with one pass through LDS for
// the wave totals, so a radix pass costs four barriers and the compaction two.
template <int T>
__device__ __forceinline__ void select_from_keys(const uint32_t* keys, int len, int keep, long long out0, int start,
                                                 int* __restrict__ kept) {
    constexpr int NW = T / 64;
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_total[NW];
    __shared__ uint32_t sh_prefix, sh_need;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { sh_prefix = 0u; sh_need = (uint32_t)keep; }
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();

    // radix select: after the pass for `shift`, sh_prefix holds the top bits of the pivot and sh_need how
    // many elements must still be taken among those sharing that prefix
#pragma unroll 1
    for (int shift = 24; shift >= 0; shift -= 8) {
        const uint32_t prefix = sh_prefix, need = sh_need;
        const uint32_t himask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
        for (int t = tid; t < len; t += T) {
            const uint32_t key = keys[t];
            if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        // suffix sums over the 256 digits: ge = number of candidates whose digit is >= tid.  Waves 0..3 hold the
        // digits in DESCENDING order (thread t holds digit 255 - t), so a prefix sum over threads is the suffix sum.
        uint32_t incl = 0;
        if (tid < 256) {
            incl = wave_inclusive_scan(hist[255 - tid], lane);
            if (lane == 63) wave_total[wave] = incl;
        }
        __syncthreads();
        if (tid < 256) {
            for (int w = 0; w < wave; ++w) incl += wave_total[w];
            const uint32_t ge = incl, gt = incl - hist[255 - tid];
            hist[255 - tid] = 0u;  // cleared for the next pass (every thread is past its atomics)
            if (gt < need && need <= ge) {  // exactly one digit satisfies this
                sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
                sh_need = need - gt;
            }
        }
        __syncthreads();
    }
    const uint32_t pivot = sh_prefix;   // key of the k-th largest element
    const uint32_t need_eq = sh_need;   // how many elements equal to the pivot are kept (lowest indices first)

    // compaction in index order: thread t owns the contiguous range [t*per, (t+1)*per)
    const int per = (len + T - 1) / T;
    const int lo = min(len, tid * per), hi = min(len, lo + per);
    uint32_t ngt = 0, neq = 0;
    for (int t = lo; t < hi; ++t) {
        const uint32_t key = keys[t];
        ngt += key > pivot;
        neq += key == pivot;
    }
    // len <= 32768 so both counts fit 16 bits, as do their prefix sums: one scan carries both
    uint32_t incl = wave_inclusive_scan(ngt | (neq << 16), lane);
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    for (int w = 0; w < wave; ++w) incl += wave_total[w];
    uint32_t gt_before = (incl & 0xffffu) - ngt, eq_before = (incl >> 16) - neq;
    for (int t = lo; t < hi; ++t) {
        const uint32_t key = keys[t];
        if (key > pivot) {
            kept[out0 + gt_before + min(eq_before, need_eq)] = start + t;
            ++gt_before;
        } else if (key == pivot) {
            if (eq_before < need_eq) kept[out0 + gt_before + eq_before] = start + t;
            ++eq_before;
        }
    }
}

// tokens kept in a segment of length len when full segments of length L keep k
__device__ __forceinline__ int segment_keep(int len, int L, int k) {
    if (len == L) return k;
    const long long v = ((long long)k * len + L - 1) / L;
    return (int)max(1ll, min((long long)len, v));
}

__global__ __launch_bounds__(SEL_THREADS) void select_topk_kernel(const float* __restrict__ scores, int S, int L, int k,
                                                                  int* __restrict__ kept) {
    extern __shared__ uint32_t keys[];  // [len]
    const int seg = blockIdx.x, tid = threadIdx.x;
    const int start = seg * L;  // host guarantees start < S and no overflow
    const int len = min(L, S - start);
    for (int t = tid; t < len; t += SEL_THREADS) keys[t] = order_key(scores[start + t]);
    select_from_keys<SEL_THREADS>(keys, len, segment_keep(len, L, k), (long long)seg * k /* every earlier segment is full */, start, kept);
}

// Head mean and selection in one launch (one workgroup per segment): the segment's [H, len] slab of per-head column
// sums and diagonals is read once, coalesced along the tokens, the heads are added in ascending order exactly as
// head_mean_kernel adds them (same bits), the scores are written out and their order keys go straight to LDS for the
// selection.  Saves one launch and the round trip of the scores through memory.
constexpr int FUSED_THREADS = 1024;
__global__ __launch_bounds__(FUSED_THREADS) void head_mean_select_kernel(const float* __restrict__ colsum, const float* __restrict__ diag,
                                                                         int S, int H, int exclude_self, int L, int k,
                                                                         float* __restrict__ scores, int* __restrict__ kept) {
    extern __shared__ uint32_t keys[];  // [len]
    const int seg = blockIdx.x, tid = threadIdx.x;
    const int start = seg * L;
    const int len = min(L, S - start);
    for (int t = tid; t < len; t += FUSED_THREADS) {
        const float* c = colsum + start + t;
        const float* g = diag + start + t;
        float acc = 0.f;
        int h = 0;
        for (; h + 8 <= H; h += 8) {  // eight heads' loads in flight at a time; the additions stay in head order
            float cv[8], gv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) cv[u] = c[(size_t)(h + u) * S];
            if (exclude_self) {
#pragma unroll
                for (int u = 0; u < 8; ++u) gv[u] = g[(size_t)(h + u) * S];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                float v = cv[u];
                if (exclude_self) v -= gv[u];
                acc += v;
            }
        }
        for (; h < H; ++h) {
            float v = c[(size_t)h * S];
            if (exclude_self) v -= g[(size_t)h * S];
            acc += v;
        }
        const float sc = acc / (float)H;
        scores[start + t] = sc;
        keys[t] = order_key(sc);
    }
    select_from_keys<FUSED_THREADS>(keys, len, segment_keep(len, L, k), (long long)seg * k, start, kept);
}

// nothing: the cost of one launch on a stream (what the microsecond-sized steps of the path are measured against)
__global__ void empty_kernel() {}

// ------------------------------------------------------------------------------------------------
// Threshold selection over token blocks (Sec. 4.2 "Layer-specific Threshold"; Alg. 1 step 1).
// ------------------------------------------------------------------------------------------------

// mean of the token-block scores: one workgroup, per-thread partial sums in index order, fixed-order tree
__global__ __launch_bounds__(256) void block_mean_kernel(const float* __restrict__ token_blocks, int nb, float* __restrict__ out) {
    __shared__ float part[256];
    const int tid = threadIdx.x;
    float s = 0.f;
    for (int n = tid; n < nb; n += 256) s += token_blocks[n];
    part[tid] = s;
    __syncthreads();
    for (int k = 128; k >= 1; k >>= 1) {
        if (tid < k) part[tid] += part[tid + k];
        __syncthreads();
    }
    if (tid == 0) out[0] = part[0] / (float)nb;
}

// One workgroup.  Phase 1: start[n] = number of kept tokens in blocks before n (prefix sum over the kept blocks'
// lengths, carried from chunk to chunk of 1024 blocks).  Phase 2: every token of a kept block writes its own index.
constexpr int THR_THREADS = 1024;
__global__ __launch_bounds__(THR_THREADS) void select_threshold_kernel(const float* __restrict__ token_blocks, int S, int b, int nb,
                                                                       float t_host, const float* __restrict__ t_dev,
                                                                       int* __restrict__ kept, int* __restrict__ kept_count) {
    extern __shared__ int start[];  // [nb]; -1 marks a dropped block
    __shared__ int scan[THR_THREADS];
    __shared__ int base;
    const int tid = threadIdx.x;
    const float T = t_dev ? t_dev[0] : t_host;
    if (tid == 0) base = 0;
    __syncthreads();
    for (int n0 = 0; n0 < nb; n0 += THR_THREADS) {
        const int n = n0 + tid;
        int len = 0;
        if (n < nb && token_blocks[n] >= T) len = min(b, S - n * b);
        scan[tid] = len;
        __syncthreads();
        for (int off = 1; off < THR_THREADS; off <<= 1) {
            const int v = tid >= off ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += v;
            __syncthreads();
        }
        if (n < nb) start[n] = len ? base + scan[tid] - len : -1;
        __syncthreads();
        if (tid == 0) base += scan[THR_THREADS - 1];
        __syncthreads();
    }
    if (tid == 0) kept_count[0] = base;
    for (int j = tid; j < S; j += THR_THREADS) {
        const int n = j / b;
        if (start[n] >= 0) kept[start[n] + (j - n * b)] = j;
    }
}

int launch_block_mean(const float* token_blocks, int nb, float* out, hipStream_t st) {
    hipLaunchKernelGGL(block_mean_kernel, dim3(1), dim3(256), 0, st, token_blocks, nb, out);
    return (int)hipGetLastError();
}

int launch_select_threshold(const float* token_blocks, int S, int b, float t_host, const float* t_dev, int* kept, int* kept_count,
                            hipStream_t st) {
    const int nb = (S + b - 1) / b;  // host checked: nb <= 16384
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {  // 16384 block offsets are 64 KB of dynamic LDS on top of the kernel's static 4 KB: above the default limit
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_threshold_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 16384 * 4);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    hipLaunchKernelGGL(select_threshold_kernel, dim3(1), dim3(THR_THREADS), (size_t)nb * sizeof(int), st, token_blocks, S, b, nb, t_host,
                       t_dev, kept, kept_count);
    return (int)hipGetLastError();
}

int launch_empty(hipStream_t st) {
    hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, st);
    return (int)hipGetLastError();
}

int launch_head_mean_select(const float* colsum, const float* diag, int S, int H, int exclude_self, int L, int k, float* scores, int* kept,
                            hipStream_t st) {
    const int Leff = L < S ? L : S;
    const int nseg = (S + L - 1) / L;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {  // a 32768-token segment needs 128 KB of dynamic LDS
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&head_mean_select_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 32768 * 4);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    hipLaunchKernelGGL(head_mean_select_kernel, dim3(nseg), dim3(FUSED_THREADS), (size_t)Leff * sizeof(uint32_t), st, colsum, diag, S, H,
                       exclude_self, L, k, scores, kept);
    return (int)hipGetLastError();
}

int launch_select(const float* scores, int S, int L, int k, int* kept, hipStream_t st) {
    const int Leff = L < S ? L : S;
    const int nseg = (S + L - 1) / L;  // L <= 32768 here (keys of one segment live in LDS), no overflow
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {  // a 32768-token segment needs 128 KB of dynamic LDS
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_topk_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 32768 * 4);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    hipLaunchKernelGGL(select_topk_kernel, dim3(nseg), dim3(SEL_THREADS), (size_t)Leff * sizeof(uint32_t), st, scores, S, L, k, kept);
    return (int)hipGetLastError();
}

}  // namespace lemo
