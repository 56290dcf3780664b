// Weight gradient of the selective-load GEMM (backward of the selective load of Sec. 4.4):
//   dW[n,c] = sum_m dY[m,n] * X[idx[m],c]
// The contraction runs over the kept tokens, i.e. over the ROW index of both operands, while the MFMA wants each operand
// contiguous along the contraction.  Both operands are therefore first written transposed into the workspace -- dY^T
// [N, Mpad] and X[idx]^T [C, Mpad], the gather folded into that pass (the kept rows are read in place, no compact copy of
// X in its original orientation is made) -- and the product is then the forward kernel's  A . B^T  with A = dY^T, B = X^T.
#include "lemo_common.hpp"

namespace lemo {

// out[c][m] = in[row(m)][c] for m < M (row(m) = idx[m], or m without a list), zero for M <= m < Mpad.  Bits are moved,
// never interpreted: U is an unsigned integer of the element's size.
template <typename U>
__global__ __launch_bounds__(256) void gather_transpose_kernel(const U* __restrict__ in, long long ld_in, const int* __restrict__ idx, int M,
                                                               int ncols, U* __restrict__ out, long long ld_out) {
    constexpr int EPV = 16 / (int)sizeof(U);  // elements per 16 bytes
    constexpr int TC = 16 * EPV;              // columns of `in` per tile
    constexpr int PPC = 64 / EPV;             // 16-byte pieces per output row segment of 64 tokens
    __shared__ U tile[64][TC + 4 / (int)sizeof(U)];
    const int m0 = blockIdx.x * 64, c0 = blockIdx.y * TC, tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = tid / 16 + 16 * i, cc = (tid % 16) * EPV, m = m0 + row;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (m < M && c0 + cc < ncols) {
            const long long r = idx ? (long long)idx[m] : (long long)m;
            v = *reinterpret_cast<const u32x4*>(in + r * ld_in + c0 + cc);
        }
        U e[EPV];
        __builtin_memcpy(e, &v, 16);
#pragma unroll
        for (int k = 0; k < EPV; ++k) tile[row][cc + k] = e[k];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TC * PPC / 256; ++i) {
        const int c = tid / PPC + (256 / PPC) * i, r0 = (tid % PPC) * EPV;
        if (c0 + c < ncols) {
            U e[EPV];
#pragma unroll
            for (int k = 0; k < EPV; ++k) e[k] = tile[r0 + k][c];
            u32x4 v;
            __builtin_memcpy(&v, e, 16);
            *reinterpret_cast<u32x4*>(out + (long long)(c0 + c) * ld_out + m0 + r0) = v;
        }
    }
}

template <typename U>
static int launch_transpose(const void* in, long long ld_in, const int* idx, long long M, long long Mpad, int ncols, void* out, hipStream_t st) {
    constexpr int TC = 16 * (16 / (int)sizeof(U));
    hipLaunchKernelGGL((gather_transpose_kernel<U>), dim3((unsigned)(Mpad / 64), (unsigned)((ncols + TC - 1) / TC)), dim3(256), 0, st,
                       static_cast<const U*>(in), ld_in, idx, (int)M, ncols, static_cast<U*>(out), Mpad);
    return (int)hipGetLastError();
}

// workspace: dY^T [N, Mpad] then X[idx]^T [C, Mpad], Mpad = M rounded up to 64, each block rounded up to 256 bytes
// rows x row_elems elements of U set to zero (row pitch in elements): a kernel rather than a memset, so that a caller may
// capture the call in a HIP graph
template <typename U>
__global__ __launch_bounds__(256) void zero_matrix_kernel(U* __restrict__ p, long long pitch, int row_elems) {
    U* row = p + (long long)blockIdx.x * pitch;
    for (int c = threadIdx.x; c < row_elems; c += 256) row[c] = 0;
}
int launch_zero_matrix(void* p, long long pitch, int row_elems, int rows, lemo_dtype_t dt, hipStream_t st) {
    if (rows <= 0 || row_elems <= 0) return 0;
    if (dt == LEMO_BF16) hipLaunchKernelGGL(zero_matrix_kernel<uint16_t>, dim3((unsigned)rows), dim3(256), 0, st, static_cast<uint16_t*>(p), pitch, row_elems);
    else hipLaunchKernelGGL(zero_matrix_kernel<uint32_t>, dim3((unsigned)rows), dim3(256), 0, st, static_cast<uint32_t*>(p), pitch, row_elems);
    return (int)hipGetLastError();
}

int launch_gather_gemm_dw(const void* dY, long long ldy, const void* X, long long S, long long ldx, const int* idx, long long M, void* dW,
                          long long lddw, int C, int N, lemo_dtype_t dt, void* workspace, hipStream_t st) {
    const long long Mpad = (M + 63) / 64 * 64;
    const size_t esz = dt == LEMO_BF16 ? 2 : 4;
    char* dYt = static_cast<char*>(workspace);
    char* Xt = dYt + (((size_t)N * (size_t)Mpad * esz + 255) / 256) * 256;
    int rc = dt == LEMO_BF16 ? launch_transpose<uint16_t>(dY, ldy, nullptr, M, Mpad, N, dYt, st)
                             : launch_transpose<uint32_t>(dY, ldy, nullptr, M, Mpad, N, dYt, st);
    if (rc) return rc;
    rc = dt == LEMO_BF16 ? launch_transpose<uint16_t>(X, ldx, idx, M, Mpad, C, Xt, st) : launch_transpose<uint32_t>(X, ldx, idx, M, Mpad, C, Xt, st);
    if (rc) return rc;
    // dW [N, C] = dY^T [N, Mpad] . (X^T [C, Mpad])^T : the forward kernel with the padded token axis as contraction
    return launch_gather_gemm(dYt, N, Mpad, nullptr, N, Xt, Mpad, nullptr, dW, lddw, (int)Mpad, C, dt, st);
}

}  // namespace lemo
