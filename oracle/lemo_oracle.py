"""ctypes front end of the C oracle.  TEST INFRASTRUCTURE ONLY (see lemo_oracle.c).

bf16 tensors cross this boundary as numpy ``uint16`` arrays holding the raw bit patterns, so the
oracle sees exactly the bits handed to the GPU.  fp32 tensors are ``float32`` arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

F32, BF16 = 0, 1
CAUSAL, EXCLUDE_SELF = 1, 2
SCATTER_ACCUMULATE, SCATTER_ZERO_PAD = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lemo_oracle.c")
_LIB = os.path.join(_HERE, "liblemo_oracle.so")
# a prebuilt library to load instead (the sanitizer run of the test suite points this at an instrumented build)
_OVERRIDE = os.environ.get("LEMO_ORACLE_LIB")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile lemo_oracle.c into liblemo_oracle.so beside it (gcc -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                        "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(_OVERRIDE if _OVERRIDE else build())
            i64, i32, u32, dbl, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_double, ctypes.c_void_p
            lib.oracle_keep_k.restype = i32
            lib.oracle_keep_k.argtypes = [i32, dbl]
            lib.oracle_kept_count.restype = i64
            lib.oracle_kept_count.argtypes = [i64, i32, i32]
            lib.oracle_score.restype = ctypes.c_int
            lib.oracle_score.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, dbl, u32, vp, vp, vp]
            lib.oracle_score_bruteforce.restype = ctypes.c_int
            lib.oracle_score_bruteforce.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, dbl, u32, vp]
            lib.oracle_score_blocks.restype = ctypes.c_int
            lib.oracle_score_blocks.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, dbl, u32, i32, ctypes.c_int, vp, vp]
            lib.oracle_score_block_rows.restype = ctypes.c_int
            lib.oracle_score_block_rows.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, dbl, u32, i32, ctypes.c_int, vp, i32, vp]
            lib.oracle_select_threshold.restype = i64
            lib.oracle_select_threshold.argtypes = [vp, i64, i32, dbl, vp]
            lib.oracle_threshold_init.restype = dbl
            lib.oracle_threshold_init.argtypes = [vp, i64]
            lib.oracle_select_topk.restype = ctypes.c_int
            lib.oracle_select_topk.argtypes = [vp, i64, i32, i32, vp]
            lib.oracle_gather_gemm.restype = ctypes.c_int
            lib.oracle_gather_gemm.argtypes = [vp, i64, i64, vp, i64, vp, i64, vp, vp, i64, i32, i32, ctypes.c_int]
            lib.oracle_gather_gemm_add.restype = ctypes.c_int
            lib.oracle_gather_gemm_add.argtypes = [vp, i64, i64, vp, i64, vp, i64, vp, vp, i64, i64, vp, i32, i32, ctypes.c_int]
            lib.oracle_gather_gemm_dw.restype = ctypes.c_int
            lib.oracle_gather_gemm_dw.argtypes = [vp, i64, vp, i64, i64, vp, i64, vp, i64, i32, i32, ctypes.c_int]
            lib.oracle_kept_attention.restype = ctypes.c_int
            lib.oracle_kept_attention.argtypes = [vp, vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, i64, i64, vp, i64, dbl, u32, vp, i64, vp, i64, i64]
            lib.oracle_scatter_add.restype = ctypes.c_int
            lib.oracle_scatter_add.argtypes = [vp, i64, vp, i64, vp, i64, i64, i32, ctypes.c_int, ctypes.c_int, ctypes.c_int]
            lib.oracle_num_threads.restype = ctypes.c_int
            lib.oracle_num_threads.argtypes = []
            lib.oracle_double_to_bf16_bits.restype = ctypes.c_uint16
            lib.oracle_double_to_bf16_bits.argtypes = [dbl]
            _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or uint16 (bf16 bits) arrays, got {a.dtype}")


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what} failed with oracle error {rc}")


# ------------------------------------------------------------------ bf16 bit helpers (marshalling)

def bf16_bits_to_float32(bits: np.ndarray) -> np.ndarray:
    """Widen raw bf16 bit patterns exactly to float32."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def float32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bf16 (ties to even) and return the bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    lib = _load()
    flat = x.reshape(-1)
    out = np.empty(flat.shape, dtype=np.uint16)
    for n, v in enumerate(flat):  # scalar routine; only used on small test arrays
        out[n] = lib.oracle_double_to_bf16_bits(float(v))
    return out.reshape(x.shape)


def double_to_bf16_bits(x: float) -> int:
    return int(_load().oracle_double_to_bf16_bits(float(x)))


# ------------------------------------------------------------------ the four operations

def num_threads() -> int:
    """OpenMP threads the oracle's parallel loops use."""
    return int(_load().oracle_num_threads())


def keep_k(L: int, ratio: float) -> int:
    return int(_load().oracle_keep_k(L, ratio))


def kept_count(S: int, L: int, k: int) -> int:
    return int(_load().oracle_kept_count(S, L, k))


def _qk_layout(Q, K):
    if Q.ndim != 3 or K.ndim != 3:
        raise ValueError("Q must be [S,H,d] and K [S,H_kv,d]")
    if Q.strides[2] != Q.itemsize or K.strides[2] != K.itemsize:
        raise ValueError("head_dim must be contiguous")
    S, H, d = Q.shape
    if K.shape[0] != S or K.shape[2] != d:
        raise ValueError("Q/K shape mismatch")
    return S, H, K.shape[1], d, Q.strides[0] // Q.itemsize, Q.strides[1] // Q.itemsize, K.strides[0] // K.itemsize, K.strides[1] // K.itemsize


def score(Q: np.ndarray, K: np.ndarray, flags: int = CAUSAL | EXCLUDE_SELF, scale: float = 0.0,
          per_head: bool = False):
    """Token informativeness (Sec. 4.2 Eq. 1, head mean of Eq. 2) -> float32 [S].

    With ``per_head=True`` also returns the float64 [H,S] column sums (diagonal included) and the
    float64 [H,S] diagonal probabilities.
    """
    S, H, Hkv, d, qts, qhs, kts, khs = _qk_layout(Q, K)
    dt = _dtype_code(Q)
    if _dtype_code(K) != dt:
        raise TypeError("Q and K must share a dtype")
    scores = np.empty(S, dtype=np.float32)
    col = np.empty((H, S), dtype=np.float64) if per_head else None
    dg = np.empty((H, S), dtype=np.float64) if per_head else None
    _check(_load().oracle_score(_ptr(Q), _ptr(K), S, H, Hkv, d, dt, qts, qhs, kts, khs, float(scale), flags,
                                _ptr(scores), _ptr(col), _ptr(dg)), "oracle_score")
    return (scores, col, dg) if per_head else scores


def score_bruteforce(Q: np.ndarray, K: np.ndarray, flags: int = CAUSAL | EXCLUDE_SELF, scale: float = 0.0):
    """Same scores via the materialised S x S probability matrix (S <= 2048)."""
    S, H, Hkv, d, qts, qhs, kts, khs = _qk_layout(Q, K)
    dt = _dtype_code(Q)
    scores = np.empty(S, dtype=np.float32)
    _check(_load().oracle_score_bruteforce(_ptr(Q), _ptr(K), S, H, Hkv, d, dt, qts, qhs, kts, khs, float(scale),
                                           flags, _ptr(scores)), "oracle_score_bruteforce")
    return scores


PROBABILITIES, POSITIVE_LOGITS = 0, 1


def score_blocks(Q: np.ndarray, K: np.ndarray, b: int, flags: int = CAUSAL | EXCLUDE_SELF, scale: float = 0.0,
                 mode: int = PROBABILITIES):
    """Block-wise informativeness (Sec. 4.2 Eq. 2) -> (score_blocks float64 [nb,nb], token_blocks float32 [nb])."""
    S, H, Hkv, d, qts, qhs, kts, khs = _qk_layout(Q, K)
    dt = _dtype_code(Q)
    if _dtype_code(K) != dt:
        raise TypeError("Q and K must share a dtype")
    nb = (S + b - 1) // b
    sb = np.empty((nb, nb), dtype=np.float64)
    tb = np.empty(nb, dtype=np.float32)
    _check(_load().oracle_score_blocks(_ptr(Q), _ptr(K), S, H, Hkv, d, dt, qts, qhs, kts, khs, float(scale), flags, b, mode,
                                       _ptr(sb), _ptr(tb)), "oracle_score_blocks")
    return sb, tb


def score_block_rows(Q: np.ndarray, K: np.ndarray, b: int, rows, flags: int = CAUSAL | EXCLUDE_SELF, scale: float = 0.0,
                     mode: int = PROBABILITIES) -> np.ndarray:
    """Rows `rows` of the score-block matrix only -> float64 [len(rows), nb] (spot checks at large S)."""
    S, H, Hkv, d, qts, qhs, kts, khs = _qk_layout(Q, K)
    dt = _dtype_code(Q)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    out = np.empty((len(rows), (S + b - 1) // b), dtype=np.float64)
    _check(_load().oracle_score_block_rows(_ptr(Q), _ptr(K), S, H, Hkv, d, dt, qts, qhs, kts, khs, float(scale), flags, b, mode,
                                           _ptr(rows), len(rows), _ptr(out)), "oracle_score_block_rows")
    return out


def select_threshold(token_blocks: np.ndarray, S: int, b: int, T: float) -> np.ndarray:
    """Tokens of the token blocks whose score is >= T, ascending -> int32 [M]."""
    token_blocks = np.ascontiguousarray(token_blocks, dtype=np.float32)
    if token_blocks.shape != ((S + b - 1) // b,):
        raise ValueError("token_blocks must be [ceil(S/b)]")
    out = np.empty(S, dtype=np.int32)
    n = _load().oracle_select_threshold(_ptr(token_blocks), S, b, float(T), _ptr(out))
    if n < 0:
        raise ValueError(f"oracle_select_threshold failed with oracle error {n}")
    return out[:n].copy()


def threshold_init(token_blocks: np.ndarray) -> float:
    """Alg. 1 step 1: the mean token-block score."""
    token_blocks = np.ascontiguousarray(token_blocks, dtype=np.float32)
    return float(_load().oracle_threshold_init(_ptr(token_blocks), token_blocks.shape[0]))


def select_topk(scores: np.ndarray, L: int, k: int) -> np.ndarray:
    """Per-segment top-k (ties to the lower index), kept indices ascending -> int32 [M]."""
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    S = scores.shape[0]
    M = kept_count(S, L, k)
    if M < 0:
        raise ValueError("bad S/L/k")
    out = np.empty(M, dtype=np.int32)
    _check(_load().oracle_select_topk(_ptr(scores), S, L, k, _ptr(out)), "oracle_select_topk")
    return out


def gather_gemm(X: np.ndarray, idx, W: np.ndarray, bias=None) -> np.ndarray:
    """Y[m,:] = X[idx[m],:] @ W.T (+ bias), fp64 accumulate, one rounding to the input dtype."""
    X = np.ascontiguousarray(X)
    W = np.ascontiguousarray(W)
    dt = _dtype_code(X)
    if _dtype_code(W) != dt:
        raise TypeError("X and W must share a dtype")
    S, C = X.shape
    N = W.shape[0]
    if W.shape[1] != C:
        raise ValueError("W must be [N,C]")
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        M = idx.shape[0]
    else:
        M = S
    if bias is not None:
        bias = np.ascontiguousarray(bias)
        if _dtype_code(bias) != dt or bias.shape != (N,):
            raise TypeError("bias must be [N] of the input dtype")
    Y = np.empty((M, N), dtype=X.dtype)
    _check(_load().oracle_gather_gemm(_ptr(X), S, C, _ptr(idx), M, _ptr(W), C, _ptr(bias), _ptr(Y), N, C, N, dt),
           "oracle_gather_gemm")
    return Y


def gather_gemm_add(X: np.ndarray, in_idx, W: np.ndarray, R: np.ndarray, out_idx, bias=None) -> np.ndarray:
    """In place: R[out_idx[m],:] += X[in_idx[m],:] @ W.T (+ bias), fp64, one rounding.  Returns R."""
    X = np.ascontiguousarray(X)
    W = np.ascontiguousarray(W)
    dt = _dtype_code(X)
    if _dtype_code(W) != dt or _dtype_code(R) != dt:
        raise TypeError("X, W and R must share a dtype")
    if not R.flags.c_contiguous:
        raise ValueError("R must be C-contiguous (it is updated in place)")
    S, C = X.shape
    N = W.shape[0]
    if W.shape[1] != C or R.shape[1] != N:
        raise ValueError("W must be [N,C] and R [S_out,N]")
    if in_idx is not None:
        in_idx = np.ascontiguousarray(in_idx, dtype=np.int32)
    if out_idx is not None:
        out_idx = np.ascontiguousarray(out_idx, dtype=np.int32)
    M = in_idx.shape[0] if in_idx is not None else (out_idx.shape[0] if out_idx is not None else S)
    if out_idx is not None and out_idx.shape[0] != M:
        raise ValueError("in_idx and out_idx must have the same length")
    if bias is not None:
        bias = np.ascontiguousarray(bias)
        if _dtype_code(bias) != dt or bias.shape != (N,):
            raise TypeError("bias must be [N] of the input dtype")
    _check(_load().oracle_gather_gemm_add(_ptr(X), S, C, _ptr(in_idx), M, _ptr(W), C, _ptr(bias), _ptr(R), N, R.shape[0],
                                          _ptr(out_idx), C, N, dt), "oracle_gather_gemm_add")
    return R


def gather_gemm_dw(dY: np.ndarray, X: np.ndarray, idx) -> np.ndarray:
    """dW[n,c] = sum_m dY[m,n] * X[idx[m],c] (fp64, one rounding) -> [N,C] of the input dtype."""
    dY = np.ascontiguousarray(dY)
    X = np.ascontiguousarray(X)
    dt = _dtype_code(X)
    if _dtype_code(dY) != dt:
        raise TypeError("dY and X must share a dtype")
    M, N = dY.shape
    S, C = X.shape
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        if idx.shape[0] != M:
            raise ValueError("idx must have one entry per row of dY")
    dW = np.empty((N, C), dtype=X.dtype)
    _check(_load().oracle_gather_gemm_dw(_ptr(dY), N, _ptr(X), S, C, _ptr(idx), M, _ptr(dW), C, C, N, dt), "oracle_gather_gemm_dw")
    return dW


def kept_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, idx, flags: int = CAUSAL, scale: float = 0.0, rows=None) -> np.ndarray:
    """Attention over the kept tokens (rows idx of Q, K, V; None = all) -> compact O [M,H,d] of the input dtype.
    With ``rows`` (kept-query numbers) only those queries are computed -> [len(rows),H,d]."""
    S, H, Hkv, d, qts, qhs, kts, khs = _qk_layout(Q, K)
    dt = _dtype_code(Q)
    if _dtype_code(K) != dt or _dtype_code(V) != dt or V.shape != K.shape or V.strides[2] != V.itemsize:
        raise TypeError("K and V must be [S,H_kv,d] of Q's dtype, head_dim contiguous")
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        M = idx.shape[0]
    else:
        M = S
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
    n_rows = M if rows is None else len(rows)
    O = np.empty((n_rows, H, d), dtype=Q.dtype)
    _check(_load().oracle_kept_attention(_ptr(Q), _ptr(K), _ptr(V), S, H, Hkv, d, dt, qts, qhs, kts, khs,
                                         V.strides[0] // V.itemsize, V.strides[1] // V.itemsize, _ptr(idx), M, float(scale), flags,
                                         _ptr(rows), n_rows, _ptr(O), H * d, d), "oracle_kept_attention")
    return O


def scatter_add(G: np.ndarray, idx: np.ndarray, dX: np.ndarray, mode: int = SCATTER_ACCUMULATE) -> np.ndarray:
    """In place: dX[idx[m],:] += G[m,:] (one binary32 add, one rounding).  Returns dX."""
    G = np.ascontiguousarray(G)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if not dX.flags.c_contiguous:
        raise ValueError("dX must be C-contiguous (it is updated in place)")
    M, C = G.shape
    S = dX.shape[0]
    if dX.shape[1] != C or idx.shape[0] != M:
        raise ValueError("shape mismatch")
    _check(_load().oracle_scatter_add(_ptr(G), C, _ptr(idx), M, _ptr(dX), C, S, C, _dtype_code(G), _dtype_code(dX), mode),
           "oracle_scatter_add")
    return dX
