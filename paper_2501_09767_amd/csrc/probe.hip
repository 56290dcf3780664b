// Measurement aid: the instruction mix of the scoring sweeps with everything else taken away.
//
// Per 32 x 32 logit tile at head_dim 128 the sweeps (Sec. 4.2, Eq. 1) cannot issue less than a chain of 8 dependent
// 32x32x16 bf16 MFMAs plus, for each of the 16 logits a lane holds, one fma (scale and reference), one exp2 and one add
// in binary32.  This kernel issues exactly that -- the vector work of one tile between the MFMAs of the next, two
// accumulators ping-ponging, operands in registers, no LDS, no memory -- with two wavefronts per SIMD, as the sweeps
// run.  Its rate, quoted as the MFMA flops of the tiles it "computes", is what the matrix cores and the vector ALU
// deliver together on this mix: the ceiling the sweeps are reported against beside the published MFMA peak.
#include "lemo_common.hpp"

namespace lemo {

// NOPS operand fragments per side rotate through the chain: 1 = the same pair for every MFMA (nothing switches at the
// matrix cores' inputs), 4 = a different pair for every MFMA of four in a row, as in the sweeps
template <int NOPS>
__device__ __forceinline__ void mix_tile(f32x16& dst, const f32x16& src, const bf16x8 (&a)[NOPS], const bf16x8 (&b)[NOPS], int turn,
                                         const float (&nl)[16], float c2, float& s0, float& s1) {
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        s0 += __builtin_amdgcn_exp2f(fmaf(src[2 * c], c2, nl[2 * c]));
        s1 += __builtin_amdgcn_exp2f(fmaf(src[2 * c + 1], c2, nl[2 * c + 1]));
        const bf16x8& af = a[(c + turn) % NOPS];
        const bf16x8& bf = b[(3 * c + turn) % NOPS];
        // written as assembly so that the chain stays a chain: the first MFMA of a tile starts from zero
        if (c == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(dst) : "v"(af), "v"(bf));
        else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(dst) : "v"(af), "v"(bf));
        __builtin_amdgcn_sched_barrier(0);
    }
}

// a reproducible value in [-2, 2) from a counter (xorshift-multiply hash): stands in for a unit-scale operand element
__device__ __forceinline__ float mix_value(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return (float)(int)(x >> 8) * (1.0f / 4194304.0f) - 2.0f;
}

template <int NOPS>
__global__ __launch_bounds__(256, 2) void issue_mix_kernel(int tiles, float c2, unsigned seed, float* sink) {
    bf16x8 a[NOPS], b[NOPS];
#pragma unroll
    for (int f = 0; f < NOPS; ++f)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (NOPS == 1) {
                a[f][i] = (__bf16)(float)((int)(threadIdx.x + i) % 3 - 1);
                b[f][i] = (__bf16)(float)((int)(threadIdx.x * 7 + i) % 3 - 1);
            } else {
                a[f][i] = (__bf16)mix_value(seed + (blockIdx.x * 256u + threadIdx.x) * 64u + f * 8u + i);
                b[f][i] = (__bf16)mix_value(seed * 3u + (blockIdx.x * 256u + threadIdx.x) * 64u + 32u + f * 8u + i);
            }
        }
    f32x16 accA, accB;
    float nl[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        accA[r] = (float)(threadIdx.x % 5) * 0.1f;
        accB[r] = (float)(threadIdx.x % 3) * 0.1f;
        nl[r] = -1.0f - r * 0.01f;
    }
    float s0 = 0.f, s1 = 0.f;
    for (int t = 0; t < tiles; t += 2) {  // a fixed trip count: every wave finishes
        mix_tile<NOPS>(accA, accB, a, b, 0, nl, c2, s0, s1);
        mix_tile<NOPS>(accB, accA, a, b, 1, nl, c2, s0, s1);
    }
    float s = s0 + s1;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += accA[r] + accB[r];
    if (s == 1234567.0f) sink[0] = s;  // never true in practice; keeps the work alive
}

// two workgroups of four waves per compute unit = two waves per SIMD
int launch_issue_mix(int tiles, unsigned operand_seed, float* sink, int* waves_out, hipStream_t st) {
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess || cus <= 0) return (int)(e != hipSuccess ? e : hipErrorInvalidDevice);
    // c2 = 0.02 keeps the exponentials of unit-scale dot products over 128 terms (|s| up to a few tens) well inside range
    if (operand_seed == 0) hipLaunchKernelGGL(issue_mix_kernel<1>, dim3(2 * cus), dim3(256), 0, st, tiles, 0.127f, 0u, sink);
    else hipLaunchKernelGGL(issue_mix_kernel<4>, dim3(2 * cus), dim3(256), 0, st, tiles, 0.02f, operand_seed, sink);
    *waves_out = 2 * cus * 4;
    return (int)hipGetLastError();
}

}  // namespace lemo
