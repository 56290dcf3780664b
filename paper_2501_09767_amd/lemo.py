"""Thin binding over the C-ABI HIP library (include/lemo.h).  Argument marshalling only.

Every function takes torch tensors that live on the GPU, passes their ``data_ptr()`` and the current
HIP stream to the library call of the same name, and raises ``LemoError`` on a negative return code.
No arithmetic of the method happens here, and there is NO fallback: if ``liblemo_hip.so`` has not
been built the import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

F32, BF16 = 0, 1
CAUSAL, EXCLUDE_SELF = 1, 2
SCATTER_ACCUMULATE, SCATTER_ZERO_PAD = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblemo_hip.so")

EXPORTS = ("lemo_strerror", "lemo_keep_k", "lemo_kept_count", "lemo_score_workspace_bytes",
           "lemo_score_segments", "lemo_score_segments_static", "lemo_score_rowstats", "lemo_score_colsums", "lemo_score_head_mean",
           "lemo_select_topk", "lemo_head_mean_select_topk", "lemo_launch_floor", "lemo_probe_sweep_issue_mix", "lemo_gather_gemm", "lemo_gather_gemm_add", "lemo_scatter_grad",
           "lemo_score_blocks_workspace_bytes", "lemo_score_blocks", "lemo_threshold_init", "lemo_select_threshold",
           "lemo_kept_attention_workspace_bytes", "lemo_kept_attention",
           "lemo_gather_gemm_dw_workspace_bytes", "lemo_gather_gemm_dw", "lemo_gather_gemm_dx")


class LemoError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {_lib.lemo_strerror(code).decode()} ({code})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2501_09767_amd.build). "
                          "There is no CPU fallback for the hot path.")
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, u32, vp, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_float
    lib.lemo_strerror.restype = ctypes.c_char_p
    lib.lemo_strerror.argtypes = [ctypes.c_int]
    lib.lemo_keep_k.restype = i32
    lib.lemo_keep_k.argtypes = [i32, ctypes.c_double]
    lib.lemo_kept_count.restype = i64
    lib.lemo_kept_count.argtypes = [i64, i32, i32]
    lib.lemo_score_workspace_bytes.restype = ctypes.c_int
    lib.lemo_score_workspace_bytes.argtypes = [i64, i32, i32, i32, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.lemo_score_segments.restype = ctypes.c_int
    lib.lemo_score_segments.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, f32, i32, u32,
                                        vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.lemo_score_segments_static.restype = ctypes.c_int
    lib.lemo_score_segments_static.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, f32, i32, u32, vp, vp]
    lib.lemo_score_rowstats.restype = ctypes.c_int
    lib.lemo_score_rowstats.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, f32, u32, vp, vp]
    lib.lemo_score_colsums.restype = ctypes.c_int
    lib.lemo_score_colsums.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, f32, i32, u32, vp, vp, vp, vp]
    lib.lemo_score_head_mean.restype = ctypes.c_int
    lib.lemo_score_head_mean.argtypes = [vp, vp, i64, i32, u32, vp, vp]
    lib.lemo_score_blocks_workspace_bytes.restype = ctypes.c_int
    lib.lemo_score_blocks_workspace_bytes.argtypes = [i64, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.lemo_score_blocks.restype = ctypes.c_int
    lib.lemo_score_blocks.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, f32, i32, u32, i32,
                                      vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.lemo_threshold_init.restype = ctypes.c_int
    lib.lemo_threshold_init.argtypes = [vp, i64, vp, vp]
    lib.lemo_select_threshold.restype = ctypes.c_int
    lib.lemo_select_threshold.argtypes = [vp, i64, i32, f32, vp, vp, vp, vp]
    lib.lemo_kept_attention_workspace_bytes.restype = ctypes.c_int
    lib.lemo_kept_attention_workspace_bytes.argtypes = [i64, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.lemo_kept_attention.restype = ctypes.c_int
    lib.lemo_kept_attention.argtypes = [vp, vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, i64, i64, vp, i64, f32, u32,
                                        vp, i64, i64, vp, ctypes.c_size_t, vp]
    lib.lemo_gather_gemm_dw_workspace_bytes.restype = ctypes.c_int
    lib.lemo_gather_gemm_dw_workspace_bytes.argtypes = [i64, i32, i32, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.lemo_gather_gemm_dw.restype = ctypes.c_int
    lib.lemo_gather_gemm_dw.argtypes = [vp, i64, vp, i64, i64, vp, i64, vp, i64, i32, i32, ctypes.c_int, vp, ctypes.c_size_t, vp]
    lib.lemo_head_mean_select_topk.restype = ctypes.c_int
    lib.lemo_head_mean_select_topk.argtypes = [vp, vp, i64, i32, u32, i32, i32, vp, vp, vp]
    lib.lemo_launch_floor.restype = ctypes.c_int
    lib.lemo_launch_floor.argtypes = [vp]
    lib.lemo_probe_sweep_issue_mix.restype = ctypes.c_int
    lib.lemo_probe_sweep_issue_mix.argtypes = [i32, u32, vp, ctypes.POINTER(i32), vp]
    lib.lemo_gather_gemm_dx.restype = ctypes.c_int
    lib.lemo_gather_gemm_dx.argtypes = [vp, i64, i64, vp, i64, vp, i64, i64, vp, i32, i32, ctypes.c_int, vp]
    lib.lemo_select_topk.restype = ctypes.c_int
    lib.lemo_select_topk.argtypes = [vp, i64, i32, i32, vp, vp]
    lib.lemo_gather_gemm.restype = ctypes.c_int
    lib.lemo_gather_gemm.argtypes = [vp, i64, i64, vp, i64, vp, i64, vp, vp, i64, i32, i32, ctypes.c_int, vp]
    lib.lemo_gather_gemm_add.restype = ctypes.c_int
    lib.lemo_gather_gemm_add.argtypes = [vp, i64, i64, vp, i64, vp, i64, vp, vp, i64, i64, vp, i32, i32, ctypes.c_int, vp]
    lib.lemo_scatter_grad.restype = ctypes.c_int
    lib.lemo_scatter_grad.argtypes = [vp, i64, vp, i64, vp, i64, i64, i32, ctypes.c_int, ctypes.c_int, i32, vp]
    return lib


_lib = _load()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"expected float32 or bfloat16, got {t.dtype}")


def _dev(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("tensors must live on the GPU")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, what: str):
    if rc != 0:
        raise LemoError(rc, what)


# --------------------------------------------------------------------------------- host helpers

def lemo_keep_k(L: int, ratio: float) -> int:
    return int(_lib.lemo_keep_k(L, ratio))


def lemo_kept_count(S: int, L: int, k: int) -> int:
    return int(_lib.lemo_kept_count(S, L, k))


def lemo_score_workspace_bytes(S: int, H: int, H_kv: int, d: int, dtype: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.lemo_score_workspace_bytes(S, H, H_kv, d, dtype, ctypes.byref(n)), "lemo_score_workspace_bytes")
    return int(n.value)


# --------------------------------------------------------------------------------- the four calls

def lemo_score_segments(Q: torch.Tensor, K: torch.Tensor, L: int, flags: int = CAUSAL | EXCLUDE_SELF,
                        scale: float = 0.0, scores: Optional[torch.Tensor] = None,
                        colsum_per_head: Optional[torch.Tensor] = None, diag_per_head: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Q [S,H,d], K [S,H_kv,d] (last dim contiguous) -> scores [S] float32."""
    _dev(Q, K, scores, colsum_per_head, diag_per_head, workspace)
    if Q.dim() != 3 or K.dim() != 3 or Q.stride(2) != 1 or K.stride(2) != 1:
        raise ValueError("Q must be [S,H,d] and K [S,H_kv,d] with head_dim contiguous")
    S, H, d = Q.shape
    if K.shape[0] != S or K.shape[2] != d or _dt(K) != _dt(Q):
        raise ValueError("Q/K mismatch")
    Hkv = K.shape[1]
    if scores is None:
        scores = torch.empty(S, dtype=torch.float32, device=Q.device)
    need = lemo_score_workspace_bytes(S, H, Hkv, d, _dt(Q))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    for o, shape in ((scores, (S,)), (colsum_per_head, (H, S)), (diag_per_head, (H, S))):
        if o is not None and (o.dtype != torch.float32 or tuple(o.shape) != shape or not o.is_contiguous()):
            raise ValueError("output tensors must be contiguous float32 of shape [S] / [H,S]")
    _check(_lib.lemo_score_segments(_ptr(Q), _ptr(K), S, H, Hkv, d, _dt(Q), Q.stride(0), Q.stride(1), K.stride(0),
                                    K.stride(1), float(scale), int(L), int(flags), _ptr(scores), _ptr(colsum_per_head),
                                    _ptr(diag_per_head), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream()), "lemo_score_segments")
    return scores


def lemo_score_segments_static(Q: torch.Tensor, K: torch.Tensor, L: int, scores: torch.Tensor,
                               flags: int = CAUSAL | EXCLUDE_SELF, scale: float = 0.0) -> torch.Tensor:
    """lemo_score_segments without a workspace (the library's built-in scratch; H*S <= 2**20).  Allocates nothing:
    `scores` [S] float32 must be passed in."""
    a = _qk_args(Q, K)
    _dev(scores)
    if scores.dtype != torch.float32 or tuple(scores.shape) != (a[2],) or not scores.is_contiguous():
        raise ValueError("scores must be contiguous float32 [S]")
    _check(_lib.lemo_score_segments_static(*a, float(scale), int(L), int(flags), _ptr(scores), _stream()),
           "lemo_score_segments_static")
    return scores


def _qk_args(Q: torch.Tensor, K: torch.Tensor):
    _dev(Q, K)
    if Q.dim() != 3 or K.dim() != 3 or Q.stride(2) != 1 or K.stride(2) != 1:
        raise ValueError("Q must be [S,H,d] and K [S,H_kv,d] with head_dim contiguous")
    S, H, d = Q.shape
    if K.shape[0] != S or K.shape[2] != d or _dt(K) != _dt(Q):
        raise ValueError("Q/K mismatch")
    return (_ptr(Q), _ptr(K), S, H, K.shape[1], d, _dt(Q), Q.stride(0), Q.stride(1), K.stride(0), K.stride(1))


def _plane(t: Optional[torch.Tensor], H: int, S: int, device) -> torch.Tensor:
    if t is None:
        return torch.empty((H, S), dtype=torch.float32, device=device)
    _dev(t)
    if t.dtype != torch.float32 or tuple(t.shape) != (H, S) or not t.is_contiguous():
        raise ValueError("per-head planes must be contiguous float32 [H,S]")
    return t


def lemo_score_rowstats(Q: torch.Tensor, K: torch.Tensor, flags: int = CAUSAL | EXCLUDE_SELF, scale: float = 0.0,
                        lse2: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Sweep 1 of the scoring: base-2 log-sum-exp of every query row -> [H,S] float32."""
    a = _qk_args(Q, K)
    lse2 = _plane(lse2, a[3], a[2], Q.device)
    _check(_lib.lemo_score_rowstats(*a, float(scale), int(flags), _ptr(lse2), _stream()), "lemo_score_rowstats")
    return lse2


def lemo_score_colsums(Q: torch.Tensor, K: torch.Tensor, L: int, lse2: torch.Tensor, flags: int = CAUSAL | EXCLUDE_SELF,
                       scale: float = 0.0, colsum_per_head: Optional[torch.Tensor] = None,
                       diag_per_head: Optional[torch.Tensor] = None):
    """Sweep 2 of the scoring: per-head column sums and diagonal -> two [H,S] float32 tensors."""
    a = _qk_args(Q, K)
    lse2 = _plane(lse2, a[3], a[2], Q.device)
    col = _plane(colsum_per_head, a[3], a[2], Q.device)
    dg = _plane(diag_per_head, a[3], a[2], Q.device)
    _check(_lib.lemo_score_colsums(*a, float(scale), int(L), int(flags), _ptr(lse2), _ptr(col), _ptr(dg), _stream()),
           "lemo_score_colsums")
    return col, dg


def lemo_score_head_mean(colsum_per_head: torch.Tensor, diag_per_head: torch.Tensor, flags: int = CAUSAL | EXCLUDE_SELF,
                         scores: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Head mean of (column sums - [EXCLUDE_SELF] diagonal) -> scores [S] float32."""
    H, S = colsum_per_head.shape
    col = _plane(colsum_per_head, H, S, colsum_per_head.device)
    dg = _plane(diag_per_head, H, S, colsum_per_head.device)
    if scores is None:
        scores = torch.empty(S, dtype=torch.float32, device=col.device)
    elif scores.dtype != torch.float32 or tuple(scores.shape) != (S,) or not scores.is_contiguous() or not scores.is_cuda:
        raise ValueError("scores must be contiguous float32 [S] on the GPU")
    _check(_lib.lemo_score_head_mean(_ptr(col), _ptr(dg), S, H, int(flags), _ptr(scores), _stream()), "lemo_score_head_mean")
    return scores


BLOCKS_PROBABILITIES, BLOCKS_POSITIVE_LOGITS = 0, 1


def lemo_score_blocks_workspace_bytes(S: int, H: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.lemo_score_blocks_workspace_bytes(S, H, ctypes.byref(n)), "lemo_score_blocks_workspace_bytes")
    return int(n.value)


def lemo_score_blocks(Q: torch.Tensor, K: torch.Tensor, b: int, flags: int = CAUSAL | EXCLUDE_SELF, scale: float = 0.0,
                      mode: int = BLOCKS_PROBABILITIES, lse2: Optional[torch.Tensor] = None, want_score_blocks: bool = True,
                      score_blocks: Optional[torch.Tensor] = None, token_blocks: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None):
    """Block-wise informativeness -> (score_blocks [nb,nb] float32 or None, token_blocks [nb] float32), nb = ceil(S/b)."""
    a = _qk_args(Q, K)
    S, H = a[2], a[3]
    nb = (S + b - 1) // b if b > 0 else 0
    if lse2 is not None:
        lse2 = _plane(lse2, H, S, Q.device)
    if score_blocks is None and want_score_blocks:
        score_blocks = torch.empty((nb, nb), dtype=torch.float32, device=Q.device)
    if token_blocks is None:
        token_blocks = torch.empty(nb, dtype=torch.float32, device=Q.device)
    for o, shape in ((score_blocks, (nb, nb)), (token_blocks, (nb,))):
        if o is not None:
            _dev(o)
            if o.dtype != torch.float32 or tuple(o.shape) != shape or not o.is_contiguous():
                raise ValueError("score_blocks / token_blocks must be contiguous float32 [nb,nb] / [nb]")
    if workspace is None:
        workspace = torch.empty(lemo_score_blocks_workspace_bytes(S, H), dtype=torch.uint8, device=Q.device)
    _dev(workspace)
    _check(_lib.lemo_score_blocks(*a, float(scale), int(b), int(flags), int(mode), _ptr(lse2), _ptr(score_blocks), _ptr(token_blocks),
                                  _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()), "lemo_score_blocks")
    return score_blocks, token_blocks


def lemo_threshold_init(token_blocks: torch.Tensor, threshold: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Mean token-block score (Alg. 1 step 1) -> float32 [1] on the GPU."""
    _dev(token_blocks, threshold)
    if token_blocks.dtype != torch.float32 or token_blocks.dim() != 1 or not token_blocks.is_contiguous():
        raise ValueError("token_blocks must be contiguous float32 [nb]")
    if threshold is None:
        threshold = torch.empty(1, dtype=torch.float32, device=token_blocks.device)
    elif threshold.dtype != torch.float32 or threshold.numel() != 1:
        raise ValueError("threshold must be one float32")
    _check(_lib.lemo_threshold_init(_ptr(token_blocks), token_blocks.numel(), _ptr(threshold), _stream()), "lemo_threshold_init")
    return threshold


def lemo_select_threshold(token_blocks: torch.Tensor, S: int, b: int, threshold, kept_idx: Optional[torch.Tensor] = None,
                          kept_count: Optional[torch.Tensor] = None):
    """Tokens of the blocks with score >= threshold (a float, or a float32 GPU tensor of one element)
    -> (kept_idx int32 [S], of which the first kept_count[0] entries are valid, kept_count int32 [1])."""
    _dev(token_blocks, kept_idx, kept_count)
    if token_blocks.dtype != torch.float32 or token_blocks.dim() != 1 or not token_blocks.is_contiguous() \
            or (b > 0 and token_blocks.numel() != (S + b - 1) // b):
        raise ValueError("token_blocks must be contiguous float32 [ceil(S/b)]")
    if kept_idx is None:
        kept_idx = torch.empty(S, dtype=torch.int32, device=token_blocks.device)
    elif kept_idx.dtype != torch.int32 or kept_idx.numel() < S or not kept_idx.is_contiguous():
        raise ValueError("kept_idx must be contiguous int32 with room for S entries")
    if kept_count is None:
        kept_count = torch.empty(1, dtype=torch.int32, device=token_blocks.device)
    elif kept_count.dtype != torch.int32 or kept_count.numel() != 1:
        raise ValueError("kept_count must be one int32")
    t_dev = None
    t_host = 0.0
    if isinstance(threshold, torch.Tensor):
        _dev(threshold)
        if threshold.dtype != torch.float32 or threshold.numel() != 1:
            raise ValueError("a device threshold must be one float32")
        t_dev = threshold
    else:
        t_host = float(threshold)
    _check(_lib.lemo_select_threshold(_ptr(token_blocks), int(S), int(b), t_host, _ptr(t_dev), _ptr(kept_idx), _ptr(kept_count),
                                      _stream()), "lemo_select_threshold")
    return kept_idx, kept_count


def lemo_select_topk(scores: torch.Tensor, L: int, k: int, kept_idx: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores [S] float32 -> kept_idx [M] int32, ascending."""
    _dev(scores, kept_idx)
    if scores.dtype != torch.float32 or scores.dim() != 1 or not scores.is_contiguous():
        raise ValueError("scores must be contiguous float32 [S]")
    S = scores.shape[0]
    M = lemo_kept_count(S, L, k)
    if M < 0:
        raise LemoError(-2, "lemo_kept_count")
    if kept_idx is None:
        kept_idx = torch.empty(M, dtype=torch.int32, device=scores.device)
    elif kept_idx.dtype != torch.int32 or kept_idx.numel() != M or not kept_idx.is_contiguous():
        raise ValueError("kept_idx must be contiguous int32 [M]")
    _check(_lib.lemo_select_topk(_ptr(scores), S, int(L), int(k), _ptr(kept_idx), _stream()), "lemo_select_topk")
    return kept_idx


def lemo_head_mean_select_topk(colsum_per_head: torch.Tensor, diag_per_head: torch.Tensor, L: int, k: int,
                               flags: int = CAUSAL | EXCLUDE_SELF, scores: Optional[torch.Tensor] = None,
                               kept_idx: Optional[torch.Tensor] = None):
    """Head mean + per-segment top-k in one launch -> (scores [S] float32, kept_idx [M] int32)."""
    H, S = colsum_per_head.shape
    col = _plane(colsum_per_head, H, S, colsum_per_head.device)
    dg = _plane(diag_per_head, H, S, colsum_per_head.device)
    M = lemo_kept_count(S, L, k)
    if M < 0:
        raise LemoError(-2, "lemo_kept_count")
    if scores is None:
        scores = torch.empty(S, dtype=torch.float32, device=col.device)
    elif scores.dtype != torch.float32 or tuple(scores.shape) != (S,) or not scores.is_contiguous() or not scores.is_cuda:
        raise ValueError("scores must be contiguous float32 [S] on the GPU")
    if kept_idx is None:
        kept_idx = torch.empty(M, dtype=torch.int32, device=col.device)
    elif kept_idx.dtype != torch.int32 or kept_idx.numel() != M or not kept_idx.is_contiguous() or not kept_idx.is_cuda:
        raise ValueError("kept_idx must be contiguous int32 [M] on the GPU")
    _check(_lib.lemo_head_mean_select_topk(_ptr(col), _ptr(dg), S, H, int(flags), int(L), int(k), _ptr(scores), _ptr(kept_idx), _stream()),
           "lemo_head_mean_select_topk")
    return scores, kept_idx


def lemo_launch_floor() -> None:
    """One empty kernel on the current stream (measurement aid)."""
    _check(_lib.lemo_launch_floor(_stream()), "lemo_launch_floor")


def lemo_probe_sweep_issue_mix(tiles_per_wave: int, sink: torch.Tensor, operand_seed: int = 0) -> int:
    """Enqueue the register-only instruction mix of the scoring sweeps (measurement aid) -> wavefronts launched.
    operand_seed 0: constant operands; non-zero: pseudo-random operands that change from MFMA to MFMA."""
    _dev(sink)
    if sink.dtype != torch.float32 or sink.numel() < 1:
        raise ValueError("sink must hold one float32")
    waves = ctypes.c_int32(0)
    _check(_lib.lemo_probe_sweep_issue_mix(int(tiles_per_wave), int(operand_seed) & 0xffffffff, _ptr(sink), ctypes.byref(waves), _stream()), "lemo_probe_sweep_issue_mix")
    return int(waves.value)


def lemo_gather_gemm(X: torch.Tensor, kept_idx: Optional[torch.Tensor], W: torch.Tensor,
                     bias: Optional[torch.Tensor] = None, Y: Optional[torch.Tensor] = None,
                     M: Optional[int] = None) -> torch.Tensor:
    """Y[m,:] = X[kept_idx[m],:] @ W.T (+ bias).  X [S,C], W [N,C], rows contiguous."""
    _dev(X, kept_idx, W, bias, Y)
    if X.dim() != 2 or W.dim() != 2 or X.stride(1) != 1 or W.stride(1) != 1 or X.shape[1] != W.shape[1] or _dt(X) != _dt(W):
        raise ValueError("X must be [S,C], W [N,C], same dtype, rows contiguous")
    S, C = X.shape
    N = W.shape[0]
    if kept_idx is not None:
        if kept_idx.dtype != torch.int32 or kept_idx.dim() != 1 or not kept_idx.is_contiguous():
            raise ValueError("kept_idx must be contiguous int32 [M]")
        M = kept_idx.numel() if M is None else M
    elif M is None:
        M = S
    if bias is not None and (bias.dtype != X.dtype or tuple(bias.shape) != (N,) or not bias.is_contiguous()):
        raise ValueError("bias must be [N] of the input dtype")
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    elif Y.dtype != X.dtype or Y.dim() != 2 or Y.shape[0] < M or Y.shape[1] != N or Y.stride(1) != 1:
        raise ValueError("Y must be [M,N] of the input dtype, rows contiguous")
    _check(_lib.lemo_gather_gemm(_ptr(X), S, X.stride(0), _ptr(kept_idx), M, _ptr(W), W.stride(0), _ptr(bias), _ptr(Y),
                                 Y.stride(0) if M > 0 else N, C, N, _dt(X), _stream()), "lemo_gather_gemm")
    return Y


def lemo_gather_gemm_add(X: torch.Tensor, kept_idx: Optional[torch.Tensor], W: torch.Tensor, R: torch.Tensor,
                         out_idx: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                         M: Optional[int] = None) -> torch.Tensor:
    """In place: R[out_idx[m],:] += X[kept_idx[m],:] @ W.T (+ bias).  X [S,C], W [N,C], R [S_out,N], rows contiguous."""
    _dev(X, kept_idx, W, bias, R, out_idx)
    if X.dim() != 2 or W.dim() != 2 or X.stride(1) != 1 or W.stride(1) != 1 or X.shape[1] != W.shape[1] or _dt(X) != _dt(W):
        raise ValueError("X must be [S,C], W [N,C], same dtype, rows contiguous")
    S, C = X.shape
    N = W.shape[0]
    for name, ix in (("kept_idx", kept_idx), ("out_idx", out_idx)):
        if ix is not None:
            if ix.dtype != torch.int32 or ix.dim() != 1 or not ix.is_contiguous():
                raise ValueError(f"{name} must be contiguous int32 [M]")
            if M is None:
                M = ix.numel()
            elif ix.numel() < M:
                raise ValueError(f"{name} is shorter than M")
    if M is None:
        M = S
    if bias is not None and (bias.dtype != X.dtype or tuple(bias.shape) != (N,) or not bias.is_contiguous()):
        raise ValueError("bias must be [N] of the input dtype")
    if R.dtype != X.dtype or R.dim() != 2 or R.shape[1] != N or R.stride(1) != 1:
        raise ValueError("R must be [S_out,N] of the input dtype, rows contiguous")
    _check(_lib.lemo_gather_gemm_add(_ptr(X), S, X.stride(0), _ptr(kept_idx), M, _ptr(W), W.stride(0), _ptr(bias), _ptr(R),
                                     R.stride(0), R.shape[0], _ptr(out_idx), C, N, _dt(X), _stream()), "lemo_gather_gemm_add")
    return R


def lemo_kept_attention_workspace_bytes(M: int, H_kv: int, d: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.lemo_kept_attention_workspace_bytes(M, H_kv, d, ctypes.byref(n)), "lemo_kept_attention_workspace_bytes")
    return int(n.value)


def lemo_kept_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, kept_idx: Optional[torch.Tensor], flags: int = CAUSAL,
                        scale: float = 0.0, O: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                        M: Optional[int] = None) -> torch.Tensor:
    """Attention over the kept rows of Q [S,H,d], K, V [S,H_kv,d] -> compact O [M,H,d]."""
    a = _qk_args(Q, K)
    _dev(V, kept_idx, O, workspace)
    S, H, Hkv, d = a[2], a[3], a[4], a[5]
    if V.dim() != 3 or tuple(V.shape) != tuple(K.shape) or V.stride(2) != 1 or V.dtype != K.dtype:
        raise ValueError("V must match K: [S,H_kv,d], head_dim contiguous")
    if kept_idx is not None:
        if kept_idx.dtype != torch.int32 or kept_idx.dim() != 1 or not kept_idx.is_contiguous():
            raise ValueError("kept_idx must be contiguous int32 [M]")
        M = kept_idx.numel() if M is None else M
    elif M is None:
        M = S
    if O is None:
        O = torch.empty((M, H, d), dtype=Q.dtype, device=Q.device)
    elif O.dtype != Q.dtype or O.dim() != 3 or O.shape[0] < M or O.shape[1] != H or O.shape[2] != d or O.stride(2) != 1:
        raise ValueError("O must be [M,H,d] of the input dtype, head_dim contiguous")
    if workspace is None:
        workspace = torch.empty(lemo_kept_attention_workspace_bytes(M, Hkv, d), dtype=torch.uint8, device=Q.device)
    _check(_lib.lemo_kept_attention(a[0], a[1], _ptr(V), *a[2:11], V.stride(0), V.stride(1), _ptr(kept_idx), M, float(scale), int(flags), _ptr(O),
                                    O.stride(0) if M > 0 else H * d, O.stride(1) if M > 0 else d, _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream()), "lemo_kept_attention")
    return O


def lemo_gather_gemm_dx(dY: torch.Tensor, W: torch.Tensor, dX: torch.Tensor, out_idx: Optional[torch.Tensor]) -> torch.Tensor:
    """In place: dX[out_idx[m],:] += dY[m,:] @ W.  dY [M,N], W [N,C] (as stored for the forward), dX [S_out,C]."""
    _dev(dY, W, dX, out_idx)
    if dY.dim() != 2 or W.dim() != 2 or dX.dim() != 2 or _dt(dY) != _dt(W) or _dt(dX) != _dt(W) or W.stride(1) != 1 or dX.stride(1) != 1 \
            or dY.shape[1] != W.shape[0] or dX.shape[1] != W.shape[1] or (dY.shape[0] > 0 and dY.stride(1) != 1):
        raise ValueError("dY must be [M,N], W [N,C], dX [S_out,C], same dtype, rows contiguous")
    M, N = dY.shape
    C = W.shape[1]
    if out_idx is not None and (out_idx.dtype != torch.int32 or out_idx.dim() != 1 or out_idx.numel() != M or not out_idx.is_contiguous()):
        raise ValueError("out_idx must be contiguous int32 [M]")
    _check(_lib.lemo_gather_gemm_dx(_ptr(dY), dY.stride(0) if M > 0 else N, M, _ptr(W), W.stride(0), _ptr(dX), dX.stride(0), dX.shape[0],
                                    _ptr(out_idx), C, N, _dt(W), _stream()), "lemo_gather_gemm_dx")
    return dX


def lemo_gather_gemm_dw_workspace_bytes(M: int, C: int, N: int, dtype: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.lemo_gather_gemm_dw_workspace_bytes(M, C, N, dtype, ctypes.byref(n)), "lemo_gather_gemm_dw_workspace_bytes")
    return int(n.value)


def lemo_gather_gemm_dw(dY: torch.Tensor, X: torch.Tensor, kept_idx: Optional[torch.Tensor], dW: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dW[n,c] = sum_m dY[m,n] * X[kept_idx[m],c].  dY [M,N], X [S,C] -> dW [N,C]."""
    _dev(dY, X, kept_idx, dW, workspace)
    if dY.dim() != 2 or X.dim() != 2 or _dt(dY) != _dt(X) or X.stride(1) != 1 or (dY.shape[0] > 0 and dY.stride(1) != 1):
        raise ValueError("dY must be [M,N] and X [S,C], same dtype, rows contiguous")
    M, N = dY.shape
    S, C = X.shape
    if kept_idx is not None and (kept_idx.dtype != torch.int32 or kept_idx.dim() != 1 or kept_idx.numel() != M or not kept_idx.is_contiguous()):
        raise ValueError("kept_idx must be contiguous int32 [M]")
    if dW is None:
        dW = torch.empty((N, C), dtype=X.dtype, device=X.device)
    elif dW.dtype != X.dtype or tuple(dW.shape) != (N, C) or dW.stride(1) != 1:
        raise ValueError("dW must be [N,C] of the input dtype, rows contiguous")
    if workspace is None:
        need = lemo_gather_gemm_dw_workspace_bytes(M, C, N, _dt(X))
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device) if need else None
    _check(_lib.lemo_gather_gemm_dw(_ptr(dY), dY.stride(0) if M > 0 else N, _ptr(X), S, X.stride(0), _ptr(kept_idx), M, _ptr(dW),
                                    dW.stride(0), C, N, _dt(X), _ptr(workspace),
                                    workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                    _stream()), "lemo_gather_gemm_dw")
    return dW


def lemo_scatter_grad(G: torch.Tensor, kept_idx: torch.Tensor, dX: torch.Tensor, mode: int = SCATTER_ACCUMULATE) -> torch.Tensor:
    """In place: dX[kept_idx[m],:] += G[m,:] (ACCUMULATE) or dX = zero-padded G (ZERO_PAD)."""
    _dev(G, kept_idx, dX)
    if G.dim() != 2 or dX.dim() != 2 or G.shape[1] != dX.shape[1] or dX.stride(1) != 1 or (G.shape[0] > 0 and G.stride(1) != 1):
        raise ValueError("G must be [M,C] and dX [S,C], rows contiguous")
    if kept_idx.dtype != torch.int32 or kept_idx.dim() != 1 or kept_idx.numel() != G.shape[0] or not kept_idx.is_contiguous():
        raise ValueError("kept_idx must be contiguous int32 [M]")
    M, C = G.shape
    _check(_lib.lemo_scatter_grad(_ptr(G), G.stride(0) if M > 0 else C, _ptr(kept_idx), M, _ptr(dX), dX.stride(0),
                                  dX.shape[0], C, _dt(G), _dt(dX), int(mode), _stream()), "lemo_scatter_grad")
    return dX
