// Shared device-side vocabulary of the gfx950 kernels: MFMA fragment types, the 32x32 accumulator
// layout, bf16 conversion, and the parameter blocks the host entry points fill in.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lemo.h"

namespace lemo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;  // one 16-byte piece; a native vector, so copies are plain loads/stores

struct bf16_t { uint16_t bits; };  // storage tag for bfloat16 (upper half of a binary32)

constexpr int WAVE = 64;
constexpr int NUM_XCD = 8;  // MI355X: 8 accelerator dies, workgroup b is dispatched to die b % 8

// ---- one 32x32 MFMA "chunk": 32 bytes of the contraction axis per operand row ---------------------
// Every lane supplies 16 bytes per operand: lane l holds row (l % 32), bytes [16*(l/32), +16) of the
// chunk.  bf16: one v_mfma_f32_32x32x16_bf16 (16 elements).  fp32: four v_mfma_f32_32x32x2_f32, step t
// contracting element t of the lower half with element 4+t of the upper half; A and B use the same
// assignment, and a dot product does not care in which order its terms are paired off.
template <typename T> __device__ __forceinline__ void mma_chunk(f32x16& acc, const u32x4& a, const u32x4& b);

template <> __device__ __forceinline__ void mma_chunk<bf16_t>(f32x16& acc, const u32x4& a, const u32x4& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <> __device__ __forceinline__ void mma_chunk<float>(f32x16& acc, const u32x4& a, const u32x4& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// Accumulator layout of the 32x32 MFMAs (checked on hardware): register r of lane l is the element in
//   row = 8*(r/4) + 4*(l/32) + (r%4)   (A-operand row),   col = l % 32   (B-operand row).
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// ---- LDS-direct loads ----------------------------------------------------------------------------
// Every lane fetches 16 (or 4) bytes at its own byte offset `voff` (+ the wave-uniform `soff`) into the buffer; the
// wave's 64 pieces land in consecutive LDS bytes starting at the wave-uniform LDS byte offset `lds_off`.  No registers
// and no LDS write instructions are involved.  Written as assembly so that the compiler does not make every later LDS
// read wait for them; a kernel that uses them awaits completion itself (vmcnt, they complete in issue order) before
// the barrier that publishes the data, and makes sure (lgkmcnt) that its own reads of the target have returned before
// the barrier that releases it.  The LDS offset travels in M0, which is set inside the same statement that uses it (the
// compiler keeps no value of its own in M0 across statements).
__device__ __forceinline__ void lds_direct_b128(u32x4 rsrc, unsigned lds_off, int voff, int soff = 0) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(lds_off), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ __forceinline__ void lds_direct_b32(u32x4 rsrc, unsigned lds_off, int voff, int soff = 0) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, %3 offen lds" ::"s"(lds_off), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
// raw buffer descriptor over [base, base + bytes): offsets at or past `bytes` read as zero
__device__ __forceinline__ u32x4 raw_rsrc(const void* base, long long bytes) {
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    u32x4 r;
    r[0] = (unsigned)a;
    r[1] = (unsigned)(a >> 32) & 0xffffu;
    r[2] = (unsigned)(bytes < 0xffffffffLL ? (bytes > 0 ? bytes : 0) : 0xffffffffLL);
    r[3] = 0x00020000u;
    return r;
}
// s_waitcnt immediates that wait on one counter only (gfx9 layout: vmcnt in bits 3:0 and 15:14, lgkmcnt in 11:8)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }
constexpr int LGKMCNT0 = 0xC07F;
// LDS byte offset of a pointer into the workgroup's LDS
__device__ __forceinline__ unsigned lds_offset_of(const void* p) { return (unsigned)reinterpret_cast<unsigned long long>(p); }

// ---- bf16 <-> binary32 ----------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// round to nearest, ties to even; NaN stays NaN (quiet)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) { return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16); }
// the same rounding done by the conversion instruction of gfx950 (v_cvt_pk_bf16_f32, nearest-even): one
// instruction for two values, used where conversions are on the critical path
__device__ __forceinline__ uint32_t pack_bf16x2_hw(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// ---- parameter blocks -----------------------------------------------------------------------------
struct ScoreParams {
    const void* Q;
    const void* K;
    int S, H, H_kv;
    long long q_ts, q_hs, k_ts, k_hs;  // element strides
    float c2;                          // scale * log2(e): logits are handled in base-2 units
    int L;                             // segment length (key axis is cut per segment)
    int blocks_per_seg;                // key blocks per segment
    int n_key_blocks;                  // total key blocks
    int n_query_blocks;
    int heads_per_xcd;
    unsigned flags;
    float* lse2;    // [H,S] base-2 log-sum-exp of every query row
    float* colsum;  // [H,S]
    float* diag;    // [H,S]
    float* scores;  // [S]
};

struct BlockParams {
    const void* Q;
    const void* K;
    int S, H, H_kv;
    long long q_ts, q_hs, k_ts, k_hs;  // element strides
    float c2;           // probabilities: scale * log2(e)
    float out_scale;    // probabilities: 1/H;  positive logits: scale / H
    unsigned flags;
    const float* lse2;  // [H,S] row statistics (probabilities only)
    float* tilemax;     // [nt32, nt32] maxima of the 32 x 32 tiles
    int nt32;           // ceil(S / 32)
    int nt;             // rectangles per side
    int nsp;            // super-patches per side
};

// kernel launchers (defined next to their kernels; return hipError_t as int)
int launch_score(const ScoreParams& p, lemo_dtype_t dt, int d, int which, hipStream_t st);  // which: 1 row stats | 2 column sums | 4 head mean
int launch_score_blocks(const BlockParams& p, lemo_dtype_t dt, int d, int mode, int b, float* score_blocks, float* token_blocks,
                        hipStream_t st);  // mode 0: probabilities (p.lse2 filled), 1: positive logits
int launch_select(const float* scores, int S, int L, int k, int* kept, hipStream_t st);
int launch_head_mean_select(const float* colsum, const float* diag, int S, int H, int exclude_self, int L, int k, float* scores, int* kept,
                            hipStream_t st);
int launch_empty(hipStream_t st);
int launch_issue_mix(int tiles, unsigned operand_seed, float* sink, int* waves_out, hipStream_t st);
int launch_block_mean(const float* token_blocks, int nb, float* out, hipStream_t st);
int launch_select_threshold(const float* token_blocks, int S, int b, float t_host, const float* t_dev, int* kept, int* kept_count,
                            hipStream_t st);
int launch_gather_gemm_dw(const void* dY, long long ldy, const void* X, long long S, long long ldx, const int* idx, long long M, void* dW,
                          long long lddw, int C, int N, lemo_dtype_t dt, void* workspace, hipStream_t st);
int launch_zero_matrix(void* p, long long pitch, int row_elems, int rows, lemo_dtype_t dt, hipStream_t st);  // pitch in elements
int launch_kept_attention(const void* Q, const void* K, const void* V, long long S, int H, int H_kv, int d, long long q_ts, long long q_hs,
                          long long k_ts, long long k_hs, long long v_ts, long long v_hs, const int* idx, long long M, float c2,
                          unsigned flags, void* O, long long o_ts, long long o_hs, void* workspace, hipStream_t st);
int launch_scatter(const void* G, long long ldg, const int* idx, long long M, void* dX, long long lddx, long long S,
                   int C, lemo_dtype_t g_dt, lemo_dtype_t dx_dt, int mode, hipStream_t st);
int launch_gather_gemm(const void* X, long long S, long long ldx, const int* idx, long long M, const void* W,
                       long long ldw, const void* bias, void* Y, long long ldy, int C, int N, lemo_dtype_t dt,
                       hipStream_t st);
int launch_gather_gemm_dx(const void* dY, long long ldy, long long M, const void* W, long long ldw, void* dX, long long lddx, long long out_rows,
                          const int* oidx, int C, int N, hipStream_t st);
int launch_gather_gemm_dw_direct(const void* dY, long long ldy, const void* X, long long S, long long ldx, const int* idx, long long M, void* dW,
                                 long long lddw, int C, int N, hipStream_t st);
int launch_gather_gemm_add(const void* X, long long S, long long ldx, const int* idx, long long M, const void* W,
                           long long ldw, const void* bias, void* R, long long ldr, long long out_rows, const int* oidx,
                           int C, int N, lemo_dtype_t dt, hipStream_t st);

}  // namespace lemo
