"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, its host
helpers agree with the oracle, and bad arguments are turned into error codes before any launch."""
import ctypes
import os
import re

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2501_09767_amd", "liblemo_hip.so")
HEADER = os.path.join(ROOT, "include", "lemo.h")

i64, i32, u32, vp, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_float


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("liblemo_hip.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB)
    L.lemo_strerror.restype = ctypes.c_char_p
    L.lemo_strerror.argtypes = [ctypes.c_int]
    L.lemo_keep_k.restype = i32
    L.lemo_keep_k.argtypes = [i32, ctypes.c_double]
    L.lemo_kept_count.restype = i64
    L.lemo_kept_count.argtypes = [i64, i32, i32]
    L.lemo_score_workspace_bytes.argtypes = [i64, i32, i32, i32, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    L.lemo_score_segments.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, f32, i32, u32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.lemo_select_topk.argtypes = [vp, i64, i32, i32, vp, vp]
    L.lemo_gather_gemm.argtypes = [vp, i64, i64, vp, i64, vp, i64, vp, vp, i64, i32, i32, ctypes.c_int, vp]
    L.lemo_scatter_grad.argtypes = [vp, i64, vp, i64, vp, i64, i64, i32, ctypes.c_int, ctypes.c_int, i32, vp]
    return L


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lemo_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_calls():
    names = declared_functions()
    for need in ("lemo_score_segments", "lemo_select_topk", "lemo_gather_gemm", "lemo_scatter_grad"):
        assert need in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in lemo.h but not exported"


def test_binding_lists_the_same_symbols():
    src = open(os.path.join(ROOT, "paper_2501_09767_amd", "lemo.py")).read()
    for name in declared_functions():
        assert name in src


def test_host_helpers_agree_with_oracle(lib):
    for L, r in [(128, 0.5), (512, 0.4), (1024, 0.3), (1024, 0.5), (7, 0.01), (7, 1.5), (100, 0.999)]:
        assert lib.lemo_keep_k(L, r) == oracle.keep_k(L, r)
    for S, L, k in [(1024, 128, 64), (8192, 512, 205), (32768, 1024, 308), (1000, 128, 64), (5, 8, 8), (1, 1, 1), (10, 4, 5), (0, 4, 2)]:
        assert lib.lemo_kept_count(S, L, k) == oracle.kept_count(S, L, k)


def test_workspace_is_linear_in_sequence_length(lib):
    n1, n2 = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.lemo_score_workspace_bytes(16384, 32, 8, 128, 1, ctypes.byref(n1)) == 0
    assert lib.lemo_score_workspace_bytes(32768, 32, 8, 128, 1, ctypes.byref(n2)) == 0
    assert n2.value == 2 * n1.value == 3 * 32 * 32768 * 4   # 12 MiB at S=32K, nowhere near S*S
    assert lib.lemo_score_workspace_bytes(1024, 32, 8, 96, 1, ctypes.byref(n1)) == -6   # head_dim not built
    assert lib.lemo_score_workspace_bytes(1024, 32, 5, 128, 1, ctypes.byref(n1)) == -2  # H % H_kv
    assert lib.lemo_score_workspace_bytes(1024, 32, 8, 128, 7, ctypes.byref(n1)) == -3
    assert lib.lemo_score_workspace_bytes(1024, 32, 8, 128, 1, None) == -1


A, B, C_, D = 0x10000, 0x20000, 0x30000, 0x40000  # fake, aligned device addresses: never dereferenced on these paths


def test_score_argument_errors(lib):
    ok = dict(Q=A, K=B, S=1024, H=4, Hkv=4, d=64, dt=0, qts=256, qhs=64, kts=256, khs=64, scale=0.0, L=128, flags=3,
              scores=C_, col=None, dg=None, ws=D, wsb=3 * 4 * 1024 * 4, st=None)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.lemo_score_segments(a["Q"], a["K"], a["S"], a["H"], a["Hkv"], a["d"], a["dt"], a["qts"], a["qhs"], a["kts"],
                                       a["khs"], a["scale"], a["L"], a["flags"], a["scores"], a["col"], a["dg"], a["ws"], a["wsb"], a["st"])
    assert call(Q=None) == -1 and call(scores=None) == -1 and call(ws=None) == -1
    assert call(S=0) == -2 and call(L=0) == -2 and call(flags=8) == -2 and call(Hkv=3) == -2
    assert call(dt=2) == -3
    assert call(wsb=100) == -4
    assert call(Q=A + 4) == -5 and call(qts=258) == -5 and call(ws=D + 16) == -5
    assert call(d=80) == -6


def test_select_gemm_scatter_argument_errors(lib):
    assert lib.lemo_select_topk(None, 100, 10, 5, B, None) == -1
    assert lib.lemo_select_topk(A, 100, 10, 11, B, None) == -2
    assert lib.lemo_select_topk(A, 0, 10, 5, B, None) == -2
    assert lib.lemo_select_topk(A, 100000, 40000, 5, B, None) == -6
    g = lambda **kw: lib.lemo_gather_gemm(*[dict(dict(X=A, S=100, ldx=64, idx=B, M=10, W=C_, ldw=64, bias=None, Y=D, ldy=32, C=64, N=32, dt=1, st=None), **kw)[k]
                                            for k in ("X", "S", "ldx", "idx", "M", "W", "ldw", "bias", "Y", "ldy", "C", "N", "dt", "st")])
    assert g(X=None) == -1 and g(Y=None) == -1
    assert g(dt=5) == -3
    assert g(ldx=32) == -2 and g(ldy=16) == -2 and g(M=-1) == -2 and g(idx=None, M=101) == -2
    assert g(C=60, ldx=64) == -6
    assert g(ldx=68) == -5 and g(X=A + 2) == -5
    s = lambda **kw: lib.lemo_scatter_grad(*[dict(dict(G=A, ldg=64, idx=B, M=10, dX=C_, lddx=64, S=100, C=64, gdt=1, xdt=1, mode=0, st=None), **kw)[k]
                                             for k in ("G", "ldg", "idx", "M", "dX", "lddx", "S", "C", "gdt", "xdt", "mode", "st")])
    assert s(dX=None) == -1 and s(G=None) == -1 and s(idx=None) == -1
    assert s(gdt=9) == -3
    assert s(mode=2) == -2 and s(M=101) == -2 and s(ldg=32) == -2
    assert s(C=60) == -6
    assert s(lddx=68) == -5
    assert lib.lemo_strerror(-4) == b"workspace too small" and lib.lemo_strerror(0) == b"ok"


def _caller(fn, order, ok):
    return lambda **kw: fn(*[dict(ok, **kw)[k] for k in order])


def test_block_score_threshold_attention_and_gradient_argument_errors(lib):
    """The later entry points refuse bad arguments on the host, before any launch (fake addresses are never touched)."""
    E = 0x50000
    lib.lemo_score_blocks.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, f32, i32, u32, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.lemo_score_blocks_workspace_bytes.argtypes = [i64, i32, ctypes.POINTER(ctypes.c_size_t)]
    n = ctypes.c_size_t()
    assert lib.lemo_score_blocks_workspace_bytes(32768, 32, ctypes.byref(n)) == 0
    assert n.value == 32 * 32768 * 4 + 1024 * 1024 * 4  # row statistics + one float per 32 x 32 tile
    sb = _caller(lib.lemo_score_blocks, ("Q", "K", "S", "H", "Hkv", "d", "dt", "qts", "qhs", "kts", "khs", "scale", "b", "flags", "mode", "lse", "sb", "tb",
                                         "ws", "wsb", "st"),
                 dict(Q=A, K=B, S=1024, H=4, Hkv=4, d=64, dt=1, qts=256, qhs=64, kts=256, khs=64, scale=0.0, b=64, flags=3, mode=0, lse=None, sb=None,
                      tb=C_, ws=D, wsb=1 << 20, st=None))
    assert sb(tb=None) == -1 and sb(ws=None) == -1 and sb(Q=None) == -1
    assert sb(mode=2) == -2 and sb(b=0) == -2 and sb(flags=4) == -2
    assert sb(b=48) == -6 and sb(d=96) == -6
    assert sb(wsb=1000) == -4 and sb(ws=D + 64) == -5

    lib.lemo_select_threshold.argtypes = [vp, i64, i32, f32, vp, vp, vp, vp]
    lib.lemo_threshold_init.argtypes = [vp, i64, vp, vp]
    assert lib.lemo_select_threshold(None, 1024, 64, 0.5, None, B, C_, None) == -1
    assert lib.lemo_select_threshold(A, 1024, 64, 0.5, None, B, None, None) == -1
    assert lib.lemo_select_threshold(A, 0, 64, 0.5, None, B, C_, None) == -2
    assert lib.lemo_select_threshold(A, 1024, 64, float("nan"), None, B, C_, None) == -2
    assert lib.lemo_select_threshold(A, 1 << 20, 32, 0.5, None, B, C_, None) == -6  # more than 16384 token blocks
    assert lib.lemo_threshold_init(A, 0, B, None) == -2 and lib.lemo_threshold_init(None, 4, B, None) == -1

    lib.lemo_kept_attention.argtypes = [vp, vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, i64, i64, vp, i64, f32, u32, vp, i64, i64, vp,
                                        ctypes.c_size_t, vp]
    at = _caller(lib.lemo_kept_attention, ("Q", "K", "V", "S", "H", "Hkv", "d", "dt", "qts", "qhs", "kts", "khs", "vts", "vhs", "idx", "M", "scale", "flags",
                                           "O", "ots", "ohs", "ws", "wsb", "st"),
                 dict(Q=A, K=B, V=C_, S=1024, H=4, Hkv=2, d=128, dt=1, qts=512, qhs=128, kts=256, khs=128, vts=256, vhs=128, idx=D, M=100, scale=0.0,
                      flags=1, O=E, ots=512, ohs=128, ws=0x60000, wsb=1 << 20, st=None))
    assert at(V=None) == -1 and at(O=None) == -1 and at(ws=None) == -1
    assert at(dt=0) == -6 and at(d=96) == -6
    assert at(flags=3) == -2 and at(idx=None, M=2000) == -2 and at(ots=64) == -2
    assert at(vts=260) == -5 and at(O=E + 8) == -5
    assert at(wsb=100) == -4
    assert at(M=0, O=None, V=None) == 0  # nothing to do

    lib.lemo_gather_gemm_add.argtypes = [vp, i64, i64, vp, i64, vp, i64, vp, vp, i64, i64, vp, i32, i32, ctypes.c_int, vp]
    ga = _caller(lib.lemo_gather_gemm_add, ("X", "S", "ldx", "idx", "M", "W", "ldw", "bias", "R", "ldr", "So", "oidx", "C", "N", "dt", "st"),
                 dict(X=A, S=100, ldx=64, idx=B, M=10, W=C_, ldw=64, bias=None, R=D, ldr=32, So=50, oidx=E, C=64, N=32, dt=1, st=None))
    assert ga(R=None) == -1 and ga(X=None) == -1
    assert ga(M=60) == -2 and ga(ldr=16) == -2 and ga(So=0) == -2
    assert ga(C=60) == -6 and ga(oidx=E + 2) == -5 and ga(dt=3) == -3
    assert ga(M=0) == 0

    lib.lemo_gather_gemm_dw.argtypes = [vp, i64, vp, i64, i64, vp, i64, vp, i64, i32, i32, ctypes.c_int, vp, ctypes.c_size_t, vp]
    lib.lemo_gather_gemm_dw_workspace_bytes.argtypes = [i64, i32, i32, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    assert lib.lemo_gather_gemm_dw_workspace_bytes(100, 64, 32, 1, ctypes.byref(n)) == 0 and n.value == 0   # bf16: operands read in place
    assert lib.lemo_gather_gemm_dw_workspace_bytes(100, 64, 32, 0, ctypes.byref(n)) == 0 and n.value == (32 + 64) * 128 * 4
    dw = _caller(lib.lemo_gather_gemm_dw, ("dY", "ldy", "X", "S", "ldx", "idx", "M", "dW", "lddw", "C", "N", "dt", "ws", "wsb", "st"),
                 dict(dY=A, ldy=32, X=B, S=100, ldx=64, idx=C_, M=10, dW=D, lddw=64, C=64, N=32, dt=0, ws=E, wsb=1 << 20, st=None))
    assert dw(dW=None) == -1 and dw(dY=None) == -1 and dw(ws=None) == -1
    assert dw(ldy=16) == -2 and dw(idx=None, M=200) == -2
    assert dw(N=34, ldy=40) == -6 and dw(ldx=66) == -5 and dw(wsb=64) == -4 and dw(dt=2) == -3
    assert dw(dt=1, N=36, ldy=40) == -6 and dw(dt=1, ldx=68) == -5 and dw(dt=1, dW=None) == -1
    lib.lemo_gather_gemm_dx.argtypes = [vp, i64, i64, vp, i64, vp, i64, i64, vp, i32, i32, ctypes.c_int, vp]
    dx = _caller(lib.lemo_gather_gemm_dx, ("dY", "ldy", "M", "W", "ldw", "dX", "lddx", "So", "oidx", "C", "N", "dt", "st"),
                 dict(dY=A, ldy=32, M=10, W=B, ldw=64, dX=C_, lddx=64, So=100, oidx=D, C=64, N=32, dt=1, st=None))
    assert dx(dY=None) == -1 and dx(W=None) == -1 and dx(dX=None) == -1
    assert dx(ldy=16) == -2 and dx(ldw=32) == -2 and dx(M=101) == -2 and dx(So=0) == -2
    assert dx(dt=0) == -6 and dx(dt=4) == -3 and dx(C=60, ldw=64) == -6 and dx(N=36, ldy=40) == -6
    assert dx(ldw=68) == -5 and dx(oidx=D + 2) == -5
    assert dx(M=0) == 0


def test_static_scratch_and_fused_select_argument_errors(lib):
    """lemo_score_segments_static and lemo_head_mean_select_topk refuse bad arguments on the host (no GPU needed: every
    case returns before the first HIP call)."""
    lib.lemo_score_segments_static.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, i64, i64, i64, i64, f32, i32, u32, vp, vp]
    st = _caller(lib.lemo_score_segments_static, ("Q", "K", "S", "H", "Hkv", "d", "dt", "qts", "qhs", "kts", "khs", "scale", "L", "flags", "scores", "st"),
                 dict(Q=A, K=B, S=1024, H=4, Hkv=4, d=64, dt=0, qts=256, qhs=64, kts=256, khs=64, scale=0.0, L=128, flags=3, scores=C_, st=None))
    assert st(Q=None) == -1 and st(scores=None) == -1
    assert st(S=0) == -2 and st(L=0) == -2 and st(Hkv=3) == -2
    assert st(dt=2) == -3 and st(qts=258) == -5 and st(d=80) == -6
    assert st(S=(1 << 20) // 4 + 1) == -6          # H * S beyond the built-in scratch
    assert st(S=32769, H=32, Hkv=32, qts=2048, kts=2048) == -6
    lib.lemo_head_mean_select_topk.argtypes = [vp, vp, i64, i32, u32, i32, i32, vp, vp, vp]
    hs = _caller(lib.lemo_head_mean_select_topk, ("col", "dg", "S", "H", "flags", "L", "k", "scores", "kept", "st"),
                 dict(col=A, dg=B, S=1024, H=4, flags=3, L=128, k=64, scores=C_, kept=D, st=None))
    assert hs(col=None) == -1 and hs(dg=None) == -1 and hs(scores=None) == -1 and hs(kept=None) == -1
    assert hs(S=0) == -2 and hs(H=0) == -2 and hs(flags=4) == -2 and hs(k=0) == -2 and hs(k=129) == -2 and hs(L=0) == -2
    assert hs(L=40000, k=5) == -6
