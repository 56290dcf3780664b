"""The entry point that allocates nothing (lemo_score_segments_static) against lemo_score_segments, through the C ABI:
identical bits, on two calls in a row that share the library's built-in scratch, the second on a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2501_09767_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _score_static(lib, Q, K, L, flags, scores):
    S, H, d = Q.shape
    rc = lib.lemo_score_segments_static(ctypes.c_void_p(Q.data_ptr()), ctypes.c_void_p(K.data_ptr()), S, H, K.shape[1], d,
                                        1 if Q.dtype == torch.bfloat16 else 0, Q.stride(0), Q.stride(1), K.stride(0), K.stride(1),
                                        0.0, L, flags, ctypes.c_void_p(scores.data_ptr()),
                                        ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc


def test_static_scratch_entry_point_matches_the_workspace_one():
    from paper_2501_09767_amd import lemo
    lib = lemo._lib
    cases = [(3000, 8, 2, 128, "bf16", 512, 3), (700, 4, 4, 64, "f32", 128, 1)]  # the second call is the smaller one
    for n, (S, H, Hkv, d, dtype, L, flags) in enumerate(cases):
        print(f"[static] call {n}: S={S} H={H}/{Hkv} d={d} {dtype} L={L} flags={flags}", flush=True)
        Q, K = wl.tiny_qk(S, H, Hkv, d, dtype, seed=100 + n, heavy=6)
        Qd, Kd = Q.cuda(), K.cuda()
        want = lemo.lemo_score_segments(Qd, Kd, L, flags=flags)
        got = torch.full((S,), -1.0, dtype=torch.float32, device="cuda")
        assert _score_static(lib, Qd, Kd, L, flags, got) == 0
        torch.cuda.synchronize()
        np.testing.assert_array_equal(got.cpu().numpy(), want.cpu().numpy())
    # beyond the built-in scratch: refused on the host, nothing launched, the output untouched
    S, H = 40000, 32
    Qb = torch.zeros((S, H, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.full((S,), 7.0, dtype=torch.float32, device="cuda")
    assert _score_static(lib, Qb, Qb, 1024, 3, out) == -6
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    # the binding of the same name
    Q, K = wl.tiny_qk(500, 2, 1, 128, "bf16", seed=3)
    got = lemo.lemo_score_segments_static(Q.cuda(), K.cuda(), 100, torch.empty(500, dtype=torch.float32, device="cuda"))
    assert torch.equal(got, lemo.lemo_score_segments(Q.cuda(), K.cuda(), 100))
