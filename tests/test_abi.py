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
