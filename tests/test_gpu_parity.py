"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars: scores |gpu - oracle| <= 2e-3 * |oracle| + 1e-6; kept-index sets bit-exact when
fed the oracle's own scores, and equal up to swaps inside the 2e-3 band around the cut when fed the
GPU's scores; gather bit-exact and the GEMM within one bf16 step plus the binary32 accumulation bound; scatter bit-exact.
"""
import sys

import math

import numpy as np
import pytest
import torch

import oracle
from paper_2501_09767_amd import workloads as wl

pytestmark = pytest.mark.gpu

RTOL, ATOL = 2e-3, 1e-6


@pytest.fixture(scope="module")
def lemo():
    from paper_2501_09767_amd import lemo as m  # fails loudly if the HIP library is not built
    return m


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def assert_scores_close(got, want, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want)
    tol = RTOL * np.abs(want) + ATOL
    bad = np.nonzero(err > tol)[0]
    assert bad.size == 0, f"{what}: {bad.size} of {want.size} outside tolerance; worst at {bad[:5]}: got {got[bad[:5]]}, want {want[bad[:5]]}"
    return float((err / (np.abs(want) + 1e-30))[np.abs(want) > 1e-3].max(initial=0.0))


def assert_selection_equivalent(kept_gpu, scores_oracle, L, k):
    """Kept sets from GPU scores may differ from the oracle's only by elements whose ORACLE score lies
    within the score tolerance of the segment's cut value."""
    kept_ref = oracle.select_topk(scores_oracle, L, k)
    assert len(kept_gpu) == len(kept_ref)
    assert np.all(np.diff(kept_gpu) > 0)
    S = len(scores_oracle)
    out = 0
    nswap = 0
    for s0 in range(0, S, L):
        seg = scores_oracle[s0:s0 + L].astype(np.float64)
        kk = k if len(seg) == L else max(1, min(len(seg), -(-k * len(seg) // L)))
        a = set(kept_gpu[out:out + kk].tolist())
        b = set(kept_ref[out:out + kk].tolist())
        assert all(s0 <= i < s0 + len(seg) for i in a)
        out += kk
        if a == b:
            continue
        cut = np.sort(seg)[::-1][kk - 1]
        band = 2 * (RTOL * abs(cut) + ATOL)
        for i in a ^ b:
            assert abs(seg[i - s0] - cut) <= band, f"token {i}: oracle score {seg[i - s0]} is not within {band} of the cut {cut}"
            nswap += 1
    return nswap


def run_score(lemo, Q, K, L, flags, per_head=True, scale=0.0):
    S, H, _ = Q.shape
    Qd, Kd = Q.cuda(), K.cuda()
    col = torch.empty((H, S), dtype=torch.float32, device="cuda") if per_head else None
    dg = torch.empty((H, S), dtype=torch.float32, device="cuda") if per_head else None
    s = lemo.lemo_score_segments(Qd, Kd, L, flags=flags, scale=scale, colsum_per_head=col, diag_per_head=dg)
    torch.cuda.synchronize()
    return s.cpu().numpy(), (col.cpu().numpy() if per_head else None), (dg.cpu().numpy() if per_head else None)


# ------------------------------------------------------------------------------------ scoring

SCORE_CASES = [
    # S, H, Hkv, d, dtype, L
    (1, 2, 1, 64, "f32", 8), (2, 2, 2, 128, "bf16", 1), (7, 4, 2, 64, "bf16", 4), (64, 2, 2, 128, "bf16", 64),
    (129, 3, 3, 64, "f32", 50), (1000, 4, 2, 128, "bf16", 128), (777, 8, 2, 64, "bf16", 300), (600, 2, 1, 128, "f32", 256),
    (1500, 9, 3, 128, "bf16", 512),
]


@pytest.mark.parametrize("flags", [0, 1, 2, 3])
@pytest.mark.parametrize("S,H,Hkv,d,dtype,L", SCORE_CASES)
def test_score_small_shapes(lemo, S, H, Hkv, d, dtype, L, flags):
    say(f"[score] S={S} H={H}/{Hkv} d={d} {dtype} L={L} flags={flags}")
    Q, K = wl.tiny_qk(S, H, Hkv, d, dtype, seed=S * 31 + H + flags, heavy=max(1, S // 64))
    got, col, dg = run_score(lemo, Q, K, L, flags)
    want, wcol, wdg = oracle.score(wl.as_numpy(Q), wl.as_numpy(K), flags=flags, per_head=True)
    assert_scores_close(col.ravel(), wcol.ravel(), "colsum_per_head")
    assert_scores_close(dg.ravel(), wdg.ravel(), "diag_per_head")
    assert_scores_close(got, want, "scores")
    # rows of a softmax sum to one: every head's column sums total S (diagonal included)
    np.testing.assert_allclose(col.astype(np.float64).sum(axis=1), S, rtol=1e-4)
    if flags == 3:
        assert got[-1] == 0.0  # last token under causal + exclude-self: its column holds only its own diagonal


def test_score_config_C1_fp32(lemo):
    cfg = wl.CONFIGS["C1"]
    lay = wl.make_layer(cfg)
    for flags in (3, 0):
        say(f"[score] C1 flags={flags}")
        got, col, _ = run_score(lemo, lay["Q"], lay["K"], cfg.L, flags)
        want = oracle.score(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]), flags=flags)
        worst = assert_scores_close(got, want, "C1 scores")
        say(f"    worst relative error {worst:.2e}")
    # soft sanity: the 16 heavy-key tokens are all kept
    got, _, _ = run_score(lemo, lay["Q"], lay["K"], cfg.L, 3, per_head=False)
    kept = lemo.lemo_select_topk(torch.from_numpy(got).cuda(), cfg.L, cfg.k).cpu().numpy()
    heavy = np.nonzero(lay["mult"].numpy() > 1)[0]
    assert np.isin(heavy, kept).all()


def test_score_independent_of_segment_length_and_deterministic(lemo):
    Q, K = wl.tiny_qk(1100, 4, 2, 128, "bf16", seed=77, heavy=8)
    base, _, _ = run_score(lemo, Q, K, 128, 3, per_head=False)
    again, _, _ = run_score(lemo, Q, K, 128, 3, per_head=False)
    np.testing.assert_array_equal(base, again)  # no atomics: bitwise repeatable
    for L in (1, 100, 256, 333, 1024, 5000):
        say(f"[score] L-independence L={L}")
        other, _, _ = run_score(lemo, Q, K, L, 3, per_head=False)
        np.testing.assert_allclose(other, base, rtol=2e-5, atol=1e-7)  # only the fp32 summation order moves


def test_score_strided_views_and_scale(lemo):
    S, H, Hkv, d = 300, 4, 2, 64
    Q, K = wl.tiny_qk(S, H, Hkv, d, "bf16", seed=5, heavy=4)
    big = torch.zeros((S, H + 2, d + 64), dtype=torch.bfloat16)
    big[:, 1:H + 1, 64:] = Q
    say("[score] strided Q view")
    Qd = big.cuda()[:, 1:H + 1, 64:]
    s1 = lemo.lemo_score_segments(Qd, K.cuda(), 128, scale=0.2)
    s2 = lemo.lemo_score_segments(Q.cuda(), K.cuda(), 128, scale=0.2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(s1.cpu().numpy(), s2.cpu().numpy())
    want = oracle.score(wl.as_numpy(Q), wl.as_numpy(K), scale=0.2)
    assert_scores_close(s2.cpu().numpy(), want, "scale=0.2")


def test_score_steps_compose_to_the_full_call(lemo):
    """lemo_score_rowstats -> lemo_score_colsums -> lemo_score_head_mean is what lemo_score_segments runs."""
    say("[score] three steps vs one call")
    Q, K = wl.tiny_qk(900, 6, 2, 128, "bf16", seed=41, heavy=8)
    Qd, Kd = Q.cuda(), K.cuda()
    for flags in (3, 0):
        whole = lemo.lemo_score_segments(Qd, Kd, 256, flags=flags)
        lse2 = lemo.lemo_score_rowstats(Qd, Kd, flags=flags)
        col, dg = lemo.lemo_score_colsums(Qd, Kd, 256, lse2, flags=flags)
        parts = lemo.lemo_score_head_mean(col, dg, flags=flags)
        torch.cuda.synchronize()
        assert torch.equal(whole, parts)
        # lse2 is the base-2 log-sum-exp of each row: check a few rows against numpy
        q = Q.float().numpy().astype(np.float64)
        k = K.float().numpy().astype(np.float64)
        for h, i in ((0, 0), (3, 450), (5, 899)):
            n = i + 1 if flags & 1 else 900
            logits = (k[:n, h // 3] @ q[i, h]) / np.sqrt(128.0)
            want = (logits.max() + np.log(np.exp(logits - logits.max()).sum())) / np.log(2.0)
            assert abs(float(lse2[h, i]) - want) < 1e-4 * max(1.0, abs(want))


@pytest.mark.parametrize("dominant", [450, 690, 3])
def test_score_reference_overflow_is_repaired(lemo, dominant):
    """Sweep 1 freezes its reference maximum after the first stage of keys; a key far later whose logit exceeds that
    reference by more than the binary32 exponent range overflows the frozen sum, and the workgroup must then go through
    its keys again with a running maximum.  Logits of ~360 nats against a first-stage maximum near 0 force that path.
    dominant = 450: unmasked stages of the later query blocks overflow (causal), or of every block (full attention), and
    the block [256, 512) holds rows that overflow next to rows that do not; 690: under the causal mask the key is only
    ever met in masked diagonal tiles, which track the maximum, so nothing overflows there; 3: the key lies in the first
    stage, whose maximum is tracked, so the frozen reference already covers it."""
    say(f"[score] frozen-reference overflow -> second pass, dominant key {dominant}")
    S, H, d = 700, 2, 128
    rng = np.random.default_rng(123)
    q = np.full((S, H, d), 4.0, dtype=np.float32)
    q[:300] = rng.standard_normal((300, H, d)).astype(np.float32)      # ordinary rows as well
    k = (rng.standard_normal((S, H, d)) * 0.05).astype(np.float32)
    k[dominant] = 8.0                                                  # scale * <q, k> = 128*32/sqrt(128) = 362
    k[611] = -8.0
    Q = torch.from_numpy(q).to(torch.bfloat16)
    K = torch.from_numpy(k).to(torch.bfloat16)
    for flags in (3, 0):
        got, col, dg = run_score(lemo, Q, K, 256, flags)
        assert np.isfinite(got).all() and np.isfinite(col).all()
        want, wcol, wdg = oracle.score(wl.as_numpy(Q), wl.as_numpy(K), flags=flags, per_head=True)
        assert_scores_close(col.ravel(), wcol.ravel(), "colsum after repair")
        assert_scores_close(got, want, "scores after repair")
        if dominant < S - 20 or flags == 0:
            assert want[dominant] > 5  # the dominant key really collects the later queries


def test_score_config_C2_full(lemo):
    """Llama2-7B-shaped layer, S=4096, all 32 heads, against the full oracle."""
    cfg = wl.CONFIGS["C2"]
    lay = wl.make_layer(cfg, want_gemm=False)
    say("[score] C2 full: GPU")
    got, col, dg = run_score(lemo, lay["Q"], lay["K"], cfg.L, 3)
    say("[score] C2 full: oracle")
    want, wcol, wdg = oracle.score(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]), flags=3, per_head=True)
    worst = assert_scores_close(got, want, "C2 scores")
    assert_scores_close(col.ravel(), wcol.ravel(), "C2 colsum")
    say(f"    worst relative error {worst:.2e}")
    kept = lemo.lemo_select_topk(torch.from_numpy(got).cuda(), cfg.L, cfg.k).cpu().numpy()
    nswap = assert_selection_equivalent(kept, want, cfg.L, cfg.k)
    say(f"    kept sets equal up to {nswap} in-band swaps")
    heavy = np.nonzero(lay["mult"].numpy() > 1)[0]
    say(f"    heavy-key tokens kept: {int(np.isin(heavy, kept).sum())} of {len(heavy)}")


def assert_gemm_close_by_rows(got_bits, want_bits, Xrows, W, rows_per_chunk=1024):
    """assert_gemm_close over every output, a block of rows at a time (the magnitude matrix of the accumulation bound is
    float64 [rows, N]); returns the share of outputs whose bits equal the oracle's."""
    same = 0
    for r0 in range(0, got_bits.shape[0], rows_per_chunk):
        r1 = min(got_bits.shape[0], r0 + rows_per_chunk)
        assert_gemm_close(got_bits[r0:r1], want_bits[r0:r1], Xrows[r0:r1], W)
        same += int((got_bits[r0:r1] == want_bits[r0:r1]).sum())
    return same / got_bits.size


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
def test_config_whole_path_full_size(lemo, name):
    """The large configurations exactly as bench.py launches them -- full sequence, ALL heads, the consumer GEMM at its
    real width -- every output of every stage against the oracle: scores, per-head column sums and diagonals element
    by element; the kept set from the GPU's own scores equal to the oracle's up to swaps inside the tolerance band at
    the cut; every element of the gathered GEMM on that kept set; the backward scatter bit for bit (configurations
    that have one)."""
    cfg = wl.CONFIGS[name]
    say(f"[config] {name} S={cfg.S} H={cfg.H}/{cfg.H_kv} N={cfg.N} L={cfg.L} k={cfg.k} M={cfg.M}: inputs")
    lay = wl.make_layer(cfg, device="cuda")
    Qn, Kn, Xn, Wn = (wl.as_numpy(lay[n]) for n in ("Q", "K", "X", "W"))
    say(f"[config] {name}: GPU score (all {cfg.H} heads)")
    got, col, dg = run_score(lemo, lay["Q"], lay["K"], cfg.L, 3)
    np.testing.assert_allclose(col.astype(np.float64).sum(axis=1), cfg.S, rtol=1e-4)
    assert got[-1] == 0.0
    say(f"[config] {name}: oracle score on {oracle.num_threads()} threads")
    want, wcol, wdg = oracle.score(Qn, Kn, flags=3, per_head=True)
    worst = assert_scores_close(got, want, f"{name} scores")
    assert_scores_close(col.ravel(), wcol.ravel(), f"{name} colsum")
    assert_scores_close(dg.ravel(), wdg.ravel(), f"{name} diag")
    del col, dg, wcol, wdg
    say(f"    worst relative score error {worst:.2e}")
    scores_d = torch.from_numpy(got).cuda()
    kept_d = lemo.lemo_select_topk(scores_d, cfg.L, cfg.k)
    kept = kept_d.cpu().numpy()
    assert len(kept) == cfg.M
    np.testing.assert_array_equal(kept, oracle.select_topk(got, cfg.L, cfg.k))   # the selection itself is bit-exact
    nswap = assert_selection_equivalent(kept, want, cfg.L, cfg.k)                 # and valid against the oracle's scores
    heavy = np.nonzero(lay["mult"].numpy() >= 4)[0]
    say(f"    kept set equals the oracle's up to {nswap} in-band swaps; x4-key tokens kept: {int(np.isin(heavy, kept).sum())} of {len(heavy)}")
    say(f"[config] {name}: GPU gather-GEMM on the kept set")
    Y = lemo.lemo_gather_gemm(lay["X"], kept_d, lay["W"])
    torch.cuda.synchronize()
    Yb = wl.to_bf16_bits(Y)
    del Y
    say(f"[config] {name}: oracle gather-GEMM, all {cfg.M} x {cfg.N} outputs")
    want_Y = oracle.gather_gemm(Xn, kept, Wn)
    share = assert_gemm_close_by_rows(Yb, want_Y, Xn[kept], Wn)
    say(f"    {100 * share:.2f} % of the GEMM outputs carry the oracle's bits, the rest are within one bf16 step")
    del Yb, want_Y
    if cfg.backward:
        say(f"[config] {name}: backward scatter of G [{cfg.M},{cfg.C}] at the kept rows")
        R = torch.from_numpy(np.random.default_rng(cfg.seed + 9).standard_normal((cfg.S, cfg.C), dtype=np.float32)).to(torch.bfloat16)
        for init in (torch.zeros_like(R), R):
            Dd = init.cuda()
            lemo.lemo_scatter_grad(lay["G"], kept_d, Dd)
            torch.cuda.synchronize()
            want_D = wl.as_numpy(init).copy()
            oracle.scatter_add(wl.as_numpy(lay["G"]), kept, want_D)
            np.testing.assert_array_equal(wl.as_numpy(Dd), want_D)


# ------------------------------------------------------------------------------------ selection

@pytest.mark.parametrize("S,L,k", [(1024, 128, 64), (1000, 128, 64), (7, 4, 3), (1, 8, 8), (8192, 512, 205), (32768, 1024, 308),
                                   (16384, 1024, 512), (300, 100, 1), (300, 100, 100), (20000, 8192, 3000), (513, 512, 205), (100, 1, 1),
                                   (32768, 32768, 9831), (70000, 20000, 7000)])
def test_select_bit_exact(lemo, S, L, k):
    say(f"[select] S={S} L={L} k={k}")
    rng = np.random.default_rng(S + L + k)
    scores = rng.random(S).astype(np.float32)
    scores[rng.integers(0, S, S // 3)] = np.float32(0.25)        # many exact ties
    scores[rng.integers(0, S, max(1, S // 50))] *= np.float32(-1.0)  # some negatives
    scores[rng.integers(0, S, max(1, S // 100))] = np.float32(-0.0)
    scores[rng.integers(0, S, max(1, S // 100))] = np.float32(0.0)
    got = lemo.lemo_select_topk(torch.from_numpy(scores).cuda(), L, k).cpu().numpy()
    np.testing.assert_array_equal(got, oracle.select_topk(scores, L, k))


def test_select_all_equal_and_extremes(lemo):
    say("[select] ties and extremes")
    const = torch.full((4096,), 0.5, dtype=torch.float32)
    got = lemo.lemo_select_topk(const.cuda(), 1024, 300).cpu().numpy()
    np.testing.assert_array_equal(got, oracle.select_topk(const.numpy(), 1024, 300))
    ext = np.array([np.inf, -np.inf, 3.4e38, -3.4e38, 1e-45, -1e-45, 0.0, -0.0] * 16, dtype=np.float32)
    for k in (1, 17, 64, 128):
        got = lemo.lemo_select_topk(torch.from_numpy(ext).cuda(), 128, k).cpu().numpy()
        np.testing.assert_array_equal(got, oracle.select_topk(ext, 128, k))


@pytest.mark.parametrize("S,H,L,k,flags", [(1024, 4, 128, 64, 3), (1000, 3, 128, 64, 1), (7, 1, 4, 3, 2), (8192, 32, 512, 205, 3), (32768, 32, 1024, 308, 3),
                                           (20000, 9, 8192, 3000, 0), (32768, 8, 32768, 9831, 3), (513, 17, 512, 205, 3), (70000, 2, 20000, 7000, 2)])
def test_head_mean_and_select_in_one_launch(lemo, S, H, L, k, flags):
    """lemo_head_mean_select_topk == lemo_score_head_mean followed by lemo_select_topk, bit for bit (scores and kept
    indices), and its kept set is the oracle's selection on those scores."""
    say(f"[fused select] S={S} H={H} L={L} k={k} flags={flags}")
    rng = np.random.default_rng(S + H + L)
    col = rng.random((H, S)).astype(np.float32) * 3
    dg = (rng.random((H, S)).astype(np.float32) * 0.5)
    col[:, rng.integers(0, S, S // 4)] = np.float32(0.75)   # columns with equal sums in every head: exact ties after the mean
    dg[:, rng.integers(0, S, S // 4)] = np.float32(0.25)
    cold, dgd = torch.from_numpy(col).cuda(), torch.from_numpy(dg).cuda()
    want_scores = lemo.lemo_score_head_mean(cold, dgd, flags=flags)
    want_kept = lemo.lemo_select_topk(want_scores, L, k)
    scores = torch.full((S,), -3.0, dtype=torch.float32, device="cuda")
    kept = torch.full((lemo.lemo_kept_count(S, L, k),), -1, dtype=torch.int32, device="cuda")
    lemo.lemo_head_mean_select_topk(cold, dgd, L, k, flags=flags, scores=scores, kept_idx=kept)
    torch.cuda.synchronize()
    assert torch.equal(scores, want_scores) and torch.equal(kept, want_kept)
    np.testing.assert_array_equal(kept.cpu().numpy(), oracle.select_topk(scores.cpu().numpy(), L, k))
    # the head mean itself: float32 adds in head order, as numpy does them
    ref = np.zeros(S, dtype=np.float32)
    for h in range(H):
        ref = ref + ((col[h] - dg[h]) if flags & 2 else col[h])
    np.testing.assert_array_equal(scores.cpu().numpy(), ref / np.float32(H))


# ------------------------------------------------------------------------------------ block-wise informativeness, thresholds

def assert_blocks_close(got, want, what="", atol=1e-6):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, what
    assert np.isfinite(got).all(), what
    bad = np.abs(got - want) > 2e-3 * np.abs(want) + atol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond tolerance, worst {np.abs(got - want).max():.3e}"


BLOCK_CASES = [(300, 4, 2, 64, "bf16", 32), (257, 2, 2, 128, "bf16", 64), (1000, 8, 2, 128, "bf16", 128), (129, 2, 1, 64, "f32", 32),
               (200, 2, 2, 128, "f32", 64), (2100, 4, 4, 128, "bf16", 96), (31, 1, 1, 64, "bf16", 32),
               # head counts around the depth of the kernel's head pipeline (three heads in flight, a ring of four statistics)
               (150, 3, 3, 128, "bf16", 32), (150, 5, 1, 64, "f32", 32), (140, 6, 3, 128, "f32", 32), (130, 7, 7, 64, "bf16", 32)]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("flags", [0, 1, 2, 3])
@pytest.mark.parametrize("S,H,Hkv,d,dtype,b", BLOCK_CASES)
def test_score_blocks_small_shapes(lemo, S, H, Hkv, d, dtype, b, flags, mode):
    say(f"[blocks] S={S} H={H}/{Hkv} d={d} {dtype} b={b} flags={flags} mode={mode}")
    Q, K = wl.tiny_qk(S, H, Hkv, d, dtype, seed=S + b)
    sb, tb = lemo.lemo_score_blocks(Q.cuda(), K.cuda(), b, flags=flags, mode=mode)
    torch.cuda.synchronize()
    want_sb, want_tb = oracle.score_blocks(wl.as_numpy(Q), wl.as_numpy(K), b, flags=flags, mode=mode)
    atol = 1e-6 if mode == 0 else 1e-5
    assert_blocks_close(sb.cpu().numpy(), want_sb, "score blocks", atol)
    assert_blocks_close(tb.cpu().numpy(), want_tb, "token blocks", atol)


def test_score_blocks_options_and_determinism(lemo):
    say("[blocks] options")
    Q, K = wl.tiny_qk(700, 4, 2, 128, "bf16", seed=5)
    Qd, Kd = Q.cuda(), K.cuda()
    sb, tb = lemo.lemo_score_blocks(Qd, Kd, 64)
    # row statistics handed in == computed inside; no score-block matrix wanted; run twice == same bits
    lse2 = lemo.lemo_score_rowstats(Qd, Kd)
    sb2, tb2 = lemo.lemo_score_blocks(Qd, Kd, 64, lse2=lse2)
    none, tb3 = lemo.lemo_score_blocks(Qd, Kd, 64, want_score_blocks=False)
    torch.cuda.synchronize()
    assert none is None
    assert torch.equal(sb, sb2) and torch.equal(tb, tb2) and torch.equal(tb, tb3)
    # strided views (a fused QKV buffer) and an explicit scale
    qkv = torch.zeros((700, 8, 128), dtype=torch.bfloat16, device="cuda")
    qkv[:, :4] = Qd
    qkv[:, 4:6] = Kd
    _, tb4 = lemo.lemo_score_blocks(qkv[:, :4], qkv[:, 4:6], 64, scale=1.0 / math.sqrt(128))
    assert_blocks_close(tb4.cpu().numpy(), tb.cpu().numpy(), "strided", 1e-7)
    # b must be a multiple of 32
    with pytest.raises(lemo.LemoError) as e:
        lemo.lemo_score_blocks(Qd, Kd, 48)
    assert e.value.code == -6


def test_score_blocks_config_C1_fp32(lemo):
    cfg = wl.CONFIGS["C1"]
    lay = wl.make_layer(cfg, want_gemm=False)
    say("[blocks] C1")
    for flags in (0, 3):
        sb, tb = lemo.lemo_score_blocks(lay["Q"].cuda(), lay["K"].cuda(), 64, flags=flags)
        want_sb, want_tb = oracle.score_blocks(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]), 64, flags=flags)
        assert_blocks_close(sb.cpu().numpy(), want_sb, "C1 score blocks")
        assert_blocks_close(tb.cpu().numpy(), want_tb, "C1 token blocks")


def test_score_blocks_config_C2_heads_subset(lemo):
    """4096 tokens, 8 of the 32 heads (the oracle's cost is linear in the head count), b = 64: every score block."""
    cfg = wl.CONFIGS["C2"]
    lay = wl.make_layer(cfg, want_gemm=False, heads=list(range(8)), device="cuda")
    say("[blocks] C2, 8 heads: GPU")
    sb, tb = lemo.lemo_score_blocks(lay["Q"].cuda(), lay["K"].cuda(), 64)
    torch.cuda.synchronize()
    say("[blocks] C2, 8 heads: oracle")
    want_sb, want_tb = oracle.score_blocks(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]), 64)
    assert_blocks_close(sb.cpu().numpy(), want_sb, "C2 score blocks")
    assert_blocks_close(tb.cpu().numpy(), want_tb, "C2 token blocks")


def test_score_blocks_full_size(lemo):
    """The 32K-token, 32-head configuration in the launch shape the bench times (b = 64): EVERY score block and token
    block against the oracle, plus what holds by construction: blocks above the diagonal are 0, every other block lies
    in (0, 1], and the token-block scores are the column sums of the matrix."""
    cfg = wl.CONFIGS["C5"]
    lay = wl.make_layer(cfg, want_gemm=False, device="cuda")
    say("[blocks] C5: GPU")
    sb, tb = lemo.lemo_score_blocks(lay["Q"].cuda(), lay["K"].cuda(), 64)
    torch.cuda.synchronize()
    sbn, tbn = sb.cpu().numpy(), tb.cpu().numpy()
    nb = cfg.S // 64
    assert sbn.shape == (nb, nb)
    assert not np.triu(sbn, 1).any()
    low = sbn[np.tril_indices(nb)]
    assert (low > 0).all() and (low <= 1.0 + 1e-6).all()
    np.testing.assert_allclose(tbn, sbn.astype(np.float64).sum(axis=0), rtol=1e-5)
    say(f"[blocks] C5: oracle, all {nb} x {nb} score blocks, {oracle.num_threads()} threads")
    want_sb, want_tb = oracle.score_blocks(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]), 64)
    assert_blocks_close(sbn, want_sb, "C5 score blocks")
    assert_blocks_close(tbn, want_tb, "C5 token blocks")


@pytest.mark.parametrize("S,b", [(1000, 32), (4096, 64), (40000, 32), (77, 128), (32768, 1024), (16384, 1), (49150, 3)])  # the last two: the largest block count the kernel takes
def test_select_threshold_bit_exact(lemo, S, b):
    say(f"[threshold] S={S} b={b}")
    rng = np.random.default_rng(S + b)
    nb = -(-S // b)
    tb = rng.random(nb).astype(np.float32)
    tbd = torch.from_numpy(tb).cuda()
    for T in (float(np.sort(tb)[nb // 2]), -np.inf, np.inf, 0.25):
        kept, count = lemo.lemo_select_threshold(tbd, S, b, T)
        want = oracle.select_threshold(tb, S, b, T)
        n = int(count.item())
        assert n == len(want)
        np.testing.assert_array_equal(kept.cpu().numpy()[:n], want)
    # Alg. 1 step 1 on the device feeding the selection without a host round trip
    T0 = lemo.lemo_threshold_init(tbd)
    kept, count = lemo.lemo_select_threshold(tbd, S, b, T0)
    t0 = float(T0.item())
    assert t0 == pytest.approx(oracle.threshold_init(tb), rel=1e-5)
    want = oracle.select_threshold(tb, S, b, t0)
    assert int(count.item()) == len(want)
    np.testing.assert_array_equal(kept.cpu().numpy()[:len(want)], want)


def test_threshold_path_feeds_the_consumer(lemo):
    """Block scores -> initial threshold -> kept tokens -> selective-load GEMM with the data-dependent row count."""
    say("[threshold] whole path")
    cfg = wl.scaled(wl.CONFIGS["C2"], S=2048, H=4, H_kv=4, C=256, N=320)
    lay = wl.make_layer(cfg)
    Qd, Kd = lay["Q"].cuda(), lay["K"].cuda()
    _, tb = lemo.lemo_score_blocks(Qd, Kd, 64, want_score_blocks=False)
    T0 = lemo.lemo_threshold_init(tb)
    kept, count = lemo.lemo_select_threshold(tb, cfg.S, 64, T0)
    M = int(count.item())
    assert 0 < M < cfg.S and M % 64 == 0
    Y = lemo.lemo_gather_gemm(lay["X"].cuda(), kept[:M].contiguous(), lay["W"].cuda())
    torch.cuda.synchronize()
    # the GPU's block scores are close to the oracle's; its selection is exact on its own scores
    _, want_tb = oracle.score_blocks(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]), 64)
    assert_blocks_close(tb.cpu().numpy(), want_tb, "token blocks")
    idx = oracle.select_threshold(tb.cpu().numpy(), cfg.S, 64, float(T0.item()))
    np.testing.assert_array_equal(kept.cpu().numpy()[:M], idx)
    want = oracle.gather_gemm(wl.as_numpy(lay["X"]), idx, wl.as_numpy(lay["W"]))
    assert_gemm_close(wl.to_bf16_bits(Y), want, wl.as_numpy(lay["X"])[idx], wl.as_numpy(lay["W"]))


# ------------------------------------------------------------------------------------ gather-GEMM

def widen(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def assert_gemm_close(got_bits, want_bits, Xrows, W, bias=None):
    """GPU = RNE_bf16(binary32 accumulation), oracle = RNE_bf16(exact).  The two roundings can land one
    bf16 step apart, and the binary32 accumulation over C terms adds an error of about
    sqrt(C) * 2^-24 * sum_c |x_c w_c| (4x that is allowed), which matters only where the terms cancel."""
    g = widen(got_bits).astype(np.float64)
    o = widen(want_bits).astype(np.float64)
    C = Xrows.shape[1]
    mag = np.abs(widen(Xrows).astype(np.float64)) @ np.abs(widen(W).astype(np.float64)).T
    if bias is not None:
        mag = mag + np.abs(widen(bias).astype(np.float64))
    ulp = np.maximum(np.abs(g), np.abs(o))
    ulp = np.where(ulp > 0, 2.0 ** (np.floor(np.log2(np.maximum(ulp, 1e-300))) - 7), 0.0)
    tol = ulp + 2 * 4 * np.sqrt(C) * 2.0 ** -24 * mag
    bad = np.abs(g - o) > tol
    assert not bad.any(), f"{bad.sum()} of {bad.size} outputs beyond one bf16 step + accumulation bound"
    assert (got_bits == want_bits).mean() > 0.98


@pytest.mark.parametrize("S,C,N,M,bias", [(300, 64, 40, 130, False), (1000, 256, 300, 517, True), (513, 1000, 257, 513, False),
                                          (64, 8, 2, 1, True), (700, 4096, 512, 300, False)])
def test_gather_gemm_bf16(lemo, S, C, N, M, bias):
    say(f"[gemm] bf16 S={S} C={C} N={N} M={M} bias={bias}")
    rng = np.random.default_rng(S + C + N)
    X = torch.from_numpy(rng.standard_normal((S, C)).astype(np.float32)).to(torch.bfloat16)
    W = torch.from_numpy((rng.standard_normal((N, C)) * 0.02).astype(np.float32)).to(torch.bfloat16)
    b = torch.from_numpy(rng.standard_normal(N).astype(np.float32)).to(torch.bfloat16) if bias else None
    idx = np.sort(rng.choice(S, M, replace=False)).astype(np.int32)
    Xd, Wd, idxd = X.cuda(), W.cuda(), torch.from_numpy(idx).cuda()
    Y = lemo.lemo_gather_gemm(Xd, idxd, Wd, b.cuda() if bias else None)
    # the same kernel on a materialised compact copy must give identical bits (the gather is exact)
    Yc = lemo.lemo_gather_gemm(Xd[idxd.long()].contiguous(), None, Wd, b.cuda() if bias else None)
    torch.cuda.synchronize()
    got = wl.to_bf16_bits(Y)
    np.testing.assert_array_equal(got, wl.to_bf16_bits(Yc))
    want = oracle.gather_gemm(wl.as_numpy(X), idx, wl.as_numpy(W), wl.as_numpy(b) if bias else None)
    assert_gemm_close(got, want, wl.as_numpy(X)[idx], wl.as_numpy(W), wl.as_numpy(b) if bias else None)


def test_gather_gemm_identity_weight_is_a_bit_exact_gather(lemo):
    say("[gemm] identity weight")
    rng = np.random.default_rng(3)
    S, C, M = 500, 256, 333
    X = torch.from_numpy(rng.standard_normal((S, C)).astype(np.float32)).to(torch.bfloat16)
    idx = rng.permutation(S)[:M].astype(np.int32)  # unsorted on purpose: any row order is a valid gather
    Y = lemo.lemo_gather_gemm(X.cuda(), torch.from_numpy(idx).cuda(), torch.eye(C, dtype=torch.bfloat16).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(wl.to_bf16_bits(Y), wl.to_bf16_bits(X)[idx])


def test_gather_gemm_fp32_config_C1(lemo):
    cfg = wl.CONFIGS["C1"]
    lay = wl.make_layer(cfg)
    say("[gemm] C1 fp32")
    s = oracle.score(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]))
    idx = oracle.select_topk(s, cfg.L, cfg.k)
    Y = lemo.lemo_gather_gemm(lay["X"].cuda(), torch.from_numpy(idx).cuda(), lay["W"].cuda()).cpu().numpy()
    want = oracle.gather_gemm(wl.as_numpy(lay["X"]), idx, wl.as_numpy(lay["W"]))
    np.testing.assert_allclose(Y, want, rtol=1e-5, atol=1e-6)  # fp32 accumulation over C=256 vs fp64
    # strided output and M == 0
    Ybig = torch.zeros((cfg.M, cfg.N + 64), dtype=torch.float32, device="cuda")
    lemo.lemo_gather_gemm(lay["X"].cuda(), torch.from_numpy(idx).cuda(), lay["W"].cuda(), Y=Ybig[:, :cfg.N])
    np.testing.assert_array_equal(Ybig[:, :cfg.N].cpu().numpy(), Y)
    assert not Ybig[:, cfg.N:].any()
    empty = lemo.lemo_gather_gemm(lay["X"].cuda(), torch.empty(0, dtype=torch.int32, device="cuda"), lay["W"].cuda())
    assert empty.shape == (0, cfg.N)


# ------------------------------------------------------------------------------------ fused gather-GEMM + in-place add

def assert_gemm_add_close(got_bits, want_bits, before_bits, Xrows, W, out_rows, bias=None):
    """Rows named by out_rows: same bar as the plain GEMM with the residual's magnitude added to the accumulation
    bound.  Every other row must keep its bits."""
    untouched = np.setdiff1d(np.arange(got_bits.shape[0]), out_rows)
    np.testing.assert_array_equal(got_bits[untouched], before_bits[untouched])
    g = widen(got_bits[out_rows]).astype(np.float64)
    o = widen(want_bits[out_rows]).astype(np.float64)
    C = Xrows.shape[1]
    mag = np.abs(widen(Xrows).astype(np.float64)) @ np.abs(widen(W).astype(np.float64)).T + np.abs(widen(before_bits[out_rows]))
    if bias is not None:
        mag = mag + np.abs(widen(bias).astype(np.float64))
    ulp = np.maximum(np.abs(g), np.abs(o))
    ulp = np.where(ulp > 0, 2.0 ** (np.floor(np.log2(np.maximum(ulp, 1e-300))) - 7), 0.0)
    tol = ulp + 2 * 4 * np.sqrt(C) * 2.0 ** -24 * mag
    bad = np.abs(g - o) > tol
    assert not bad.any(), f"{bad.sum()} of {bad.size} outputs beyond one bf16 step + accumulation bound"
    assert (got_bits[out_rows] == want_bits[out_rows]).mean() > 0.98


@pytest.mark.parametrize("S,S_out,C,N,M,bias,pad", [(300, 300, 64, 40, 130, False, 0), (1000, 700, 256, 304, 517, True, 8),
                                                    (513, 513, 1000, 257, 513, False, 3), (64, 9, 8, 2, 1, True, 0),
                                                    (700, 900, 4096, 512, 300, False, 0)])
def test_gather_gemm_add_bf16(lemo, S, S_out, C, N, M, bias, pad):
    say(f"[gemm+add] bf16 S={S} S_out={S_out} C={C} N={N} M={M} bias={bias} pad={pad}")
    rng = np.random.default_rng(S + C + N + 1)
    X = torch.from_numpy(rng.standard_normal((S, C)).astype(np.float32)).to(torch.bfloat16)
    W = torch.from_numpy((rng.standard_normal((N, C)) * 0.02).astype(np.float32)).to(torch.bfloat16)
    b = torch.from_numpy(rng.standard_normal(N).astype(np.float32)).to(torch.bfloat16) if bias else None
    R = torch.from_numpy(rng.standard_normal((S_out, N)).astype(np.float32)).to(torch.bfloat16)
    in_idx = rng.permutation(S)[:M].astype(np.int32)
    out_idx = rng.permutation(S_out)[:M].astype(np.int32)  # unsorted, unrelated to in_idx
    Rbig = torch.full((S_out, N + pad), 7.0, dtype=torch.bfloat16, device="cuda")  # padded leading dimension
    Rd = Rbig[:, :N]
    Rd.copy_(R)
    lemo.lemo_gather_gemm_add(X.cuda(), torch.from_numpy(in_idx).cuda(), W.cuda(), Rd, torch.from_numpy(out_idx).cuda(),
                              b.cuda() if bias else None)
    torch.cuda.synchronize()
    assert (Rbig[:, N:] == 7.0).all()
    before = wl.as_numpy(R)
    want = oracle.gather_gemm_add(wl.as_numpy(X), in_idx, wl.as_numpy(W), before.copy(), out_idx, wl.as_numpy(b) if bias else None)
    assert_gemm_add_close(wl.to_bf16_bits(Rd.contiguous()), want, before, wl.as_numpy(X)[in_idx], wl.as_numpy(W), out_idx,
                          wl.as_numpy(b) if bias else None)


def test_gather_gemm_add_exact_cases(lemo):
    """Values on a dyadic grid (every partial sum representable in binary32): bit-exact against the oracle, bf16 and
    fp32, with and without the index lists; zero residual + identity weights = zero-padded rows (token padding)."""
    say("[gemm+add] exact cases")
    rng = np.random.default_rng(21)
    S, C, N, M = 400, 128, 264, 290
    Xf = (rng.integers(-8, 9, (S, C)) / 4.0).astype(np.float32)
    Wf = (rng.integers(-8, 9, (N, C)) / 8.0).astype(np.float32)
    Rf = (rng.integers(-64, 65, (S, N)) / 4.0).astype(np.float32)
    bf = (rng.integers(-8, 9, N) / 2.0).astype(np.float32)
    in_idx = rng.permutation(S)[:M].astype(np.int32)
    out_idx = rng.permutation(S)[:M].astype(np.int32)
    for dtype in (torch.bfloat16, torch.float32):
        X, W, R, b = (torch.from_numpy(a).to(dtype) for a in (Xf, Wf, Rf, bf))
        for ii, oi in ((in_idx, out_idx), (None, out_idx), (in_idx, None), (None, None)):
            got = lemo.lemo_gather_gemm_add(X.cuda(), None if ii is None else torch.from_numpy(ii).cuda(), W.cuda(), R.clone().cuda(),
                                            None if oi is None else torch.from_numpy(oi).cuda(), b.cuda(), M=M)
            torch.cuda.synchronize()
            want = oracle.gather_gemm_add(wl.as_numpy(X), np.arange(M, dtype=np.int32) if ii is None else ii, wl.as_numpy(W),
                                          wl.as_numpy(R).copy(), np.arange(M, dtype=np.int32) if oi is None else oi, wl.as_numpy(b))
            np.testing.assert_array_equal(wl.as_numpy(got.cpu()), want)
    X = torch.from_numpy(rng.standard_normal((S, C)).astype(np.float32)).to(torch.bfloat16)
    idx = np.sort(in_idx)
    pad = lemo.lemo_gather_gemm_add(X.cuda(), torch.from_numpy(idx).cuda(), torch.eye(C, dtype=torch.bfloat16).cuda(),
                                    torch.zeros((S, C), dtype=torch.bfloat16, device="cuda"), torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    padn = wl.to_bf16_bits(pad)
    np.testing.assert_array_equal(padn[idx], wl.to_bf16_bits(X)[idx])
    assert not padn[np.setdiff1d(np.arange(S), idx)].any()
    # out-of-range output rows are dropped, M == 0 is a no-op
    R0 = torch.from_numpy(Rf).to(torch.bfloat16).cuda()
    oob = out_idx.copy(); oob[::3] = S + 5; oob[1::3] = -2
    got = lemo.lemo_gather_gemm_add(torch.from_numpy(Xf).to(torch.bfloat16).cuda(), torch.from_numpy(in_idx).cuda(),
                                    torch.from_numpy(Wf).to(torch.bfloat16).cuda(), R0.clone(), torch.from_numpy(oob).cuda())
    keep = np.arange(M)[2::3]
    want = oracle.gather_gemm_add(bf16(Xf), in_idx[keep], bf16(Wf), wl.to_bf16_bits(R0).copy(), out_idx[keep])
    np.testing.assert_array_equal(wl.to_bf16_bits(got), want)
    same = lemo.lemo_gather_gemm_add(X.cuda(), torch.empty(0, dtype=torch.int32, device="cuda"), torch.eye(C, dtype=torch.bfloat16).cuda(),
                                     R0[:, :C].contiguous(), torch.empty(0, dtype=torch.int32, device="cuda"))
    np.testing.assert_array_equal(wl.to_bf16_bits(same), wl.to_bf16_bits(R0[:, :C].contiguous()))


def test_gather_gemm_add_as_backward_of_the_selective_load(lemo):
    """Backward of Y = X[idx] W^T with respect to X: dX[idx[m],:] += dY[m,:] W.  With the weight's transpose stored as a
    [C,N] matrix this is the same call (compact rows in, indexed rows out); bit-exact against the oracle on a dyadic grid."""
    say("[gemm+add] backward form")
    rng = np.random.default_rng(23)
    S, C, N, M = 300, 96, 160, 120
    dY = (rng.integers(-8, 9, (M, N)) / 4.0).astype(np.float32)
    W = (rng.integers(-8, 9, (N, C)) / 8.0).astype(np.float32)
    dX = (rng.integers(-64, 65, (S, C)) / 4.0).astype(np.float32)
    idx = np.sort(rng.permutation(S)[:M]).astype(np.int32)
    Wt = torch.from_numpy(W).to(torch.bfloat16).t().contiguous()  # [C,N]
    want = oracle.gather_gemm_add(bf16(dY), None, wl.as_numpy(Wt), bf16(dX).copy(), idx)
    got = lemo.lemo_gather_gemm_add(torch.from_numpy(dY).to(torch.bfloat16).cuda(), None, Wt.cuda(),
                                    torch.from_numpy(dX).to(torch.bfloat16).cuda(), torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(wl.to_bf16_bits(got), want)


def bf16(x):
    return wl.to_bf16_bits(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16))


def test_gather_gemm_add_output_projection_shape_sampled(lemo):
    """The attention block's output projection at the 32K-token configuration (Sec. 4.4): M = 9856 kept rows,
    C = N = 4096, added into the [32768, 4096] residual stream at the kept positions.  Sampled rows against the
    oracle (all columns), every row that is not kept must keep its bits."""
    cfg = wl.CONFIGS["C5"]
    say("[gemm+add] C5 output projection: inputs")
    rng = np.random.default_rng(cfg.seed + 200)
    A = torch.from_numpy(rng.standard_normal((cfg.M, cfg.C), dtype=np.float32)).to(torch.bfloat16)       # compact block output
    W = torch.from_numpy(rng.standard_normal((cfg.C, cfg.C), dtype=np.float32) * np.float32(0.02)).to(torch.bfloat16)
    R = torch.from_numpy(rng.standard_normal((cfg.S, cfg.C), dtype=np.float32)).to(torch.bfloat16)
    idx = oracle.select_topk(rng.random(cfg.S).astype(np.float32), cfg.L, cfg.k)
    say("[gemm+add] C5 output projection: GPU")
    Rd = R.cuda()
    lemo.lemo_gather_gemm_add(A.cuda(), None, W.cuda(), Rd, torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    got = wl.to_bf16_bits(Rd)
    before = wl.as_numpy(R)
    mask = np.ones(cfg.S, dtype=bool); mask[idx] = False
    np.testing.assert_array_equal(got[mask], before[mask])
    rows = np.unique(np.concatenate([[0, 127, 128, 255, 256, cfg.M - 257, cfg.M - 129, cfg.M - 1], rng.integers(0, cfg.M, 16)]))
    say(f"[gemm+add] C5 output projection: oracle on {len(rows)} rows")
    want = oracle.gather_gemm_add(wl.as_numpy(A), rows.astype(np.int32), wl.as_numpy(W), before.copy(), idx[rows])
    sel = idx[rows]
    g, o = got[sel], want[sel]
    mag = np.abs(widen(wl.as_numpy(A)[rows]).astype(np.float64)) @ np.abs(widen(wl.as_numpy(W)).astype(np.float64)).T + np.abs(widen(before[sel]))
    gv, ov = widen(g).astype(np.float64), widen(o).astype(np.float64)
    ulp = np.maximum(np.abs(gv), np.abs(ov))
    ulp = np.where(ulp > 0, 2.0 ** (np.floor(np.log2(np.maximum(ulp, 1e-300))) - 7), 0.0)
    assert np.all(np.abs(gv - ov) <= ulp + 8 * np.sqrt(cfg.C) * 2.0 ** -24 * mag)
    assert (g == o).mean() > 0.98


# ------------------------------------------------------------------------------------ input gradient of the selective-load GEMM

@pytest.mark.parametrize("S,C,N,M,pad", [(300, 64, 40, 130, 0), (1000, 256, 304, 517, 8), (513, 1000, 264, 513, 0), (64, 8, 8, 1, 0),
                                         (700, 512, 4096, 300, 0), (900, 520, 72, 900, 16), (400, 264, 1000, 257, 0)])
def test_gather_gemm_dx_bf16(lemo, S, C, N, M, pad):
    """dX[idx[m],:] += dY[m,:] W with W as stored [N,C]: against the oracle's fused GEMM + in-place add fed the transposed
    weight (a host-side copy of the same bits); rows that idx does not name keep their bits; padded leading dimensions."""
    say(f"[gemm dX] bf16 S={S} C={C} N={N} M={M} pad={pad}")
    rng = np.random.default_rng(S + C + N + 3)
    dY = torch.from_numpy((rng.standard_normal((M, N)) * 0.5).astype(np.float32)).to(torch.bfloat16)
    W = torch.from_numpy((rng.standard_normal((N, C)) * 0.05).astype(np.float32)).to(torch.bfloat16)
    R = torch.from_numpy(rng.standard_normal((S, C)).astype(np.float32)).to(torch.bfloat16)
    idx = rng.permutation(S)[:M].astype(np.int32)
    Wbig = torch.full((N, C + pad), 3.0, dtype=torch.bfloat16, device="cuda")
    Wbig[:, :C] = W.cuda()
    Rbig = torch.full((S, C + pad), 7.0, dtype=torch.bfloat16, device="cuda")
    Rd = Rbig[:, :C]
    Rd.copy_(R)
    lemo.lemo_gather_gemm_dx(dY.cuda(), Wbig[:, :C], Rd, torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    assert (Rbig[:, C:] == 7.0).all()
    before = wl.as_numpy(R)
    Wt = np.ascontiguousarray(wl.as_numpy(W).T)  # [C,N]: the same bits, the other way round
    want = oracle.gather_gemm_add(wl.as_numpy(dY), None, Wt, before.copy(), idx)
    assert_gemm_add_close(wl.to_bf16_bits(Rd.contiguous()), want, before, wl.as_numpy(dY), Wt, idx)


def test_gather_gemm_dx_exact_and_edge_cases(lemo):
    say("[gemm dX] exact cases")
    rng = np.random.default_rng(31)
    S, C, N, M = 300, 96, 160, 120
    dY = (rng.integers(-8, 9, (M, N)) / 4.0).astype(np.float32)
    W = (rng.integers(-8, 9, (N, C)) / 8.0).astype(np.float32)
    dX = (rng.integers(-64, 65, (S, C)) / 4.0).astype(np.float32)
    idx = np.sort(rng.permutation(S)[:M]).astype(np.int32)
    Wb = torch.from_numpy(W).to(torch.bfloat16)
    for oi in (idx, None):
        want = oracle.gather_gemm_add(bf16(dY), None, np.ascontiguousarray(wl.as_numpy(Wb).T), bf16(dX).copy(), oi)
        got = lemo.lemo_gather_gemm_dx(torch.from_numpy(dY).to(torch.bfloat16).cuda(), Wb.cuda(), torch.from_numpy(dX).to(torch.bfloat16).cuda(),
                                       None if oi is None else torch.from_numpy(oi).cuda())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(wl.to_bf16_bits(got), want)   # dyadic grid: every partial sum is exact
    # the same bits as the transposed-weight form of the in-place-add GEMM on non-dyadic data is NOT promised (other
    # summation order); but it equals that form on the dyadic grid above.  No kept rows: nothing happens.
    D0 = torch.from_numpy(dX).to(torch.bfloat16).cuda()
    same = lemo.lemo_gather_gemm_dx(torch.empty((0, N), dtype=torch.bfloat16, device="cuda"), Wb.cuda(), D0.clone(), torch.empty(0, dtype=torch.int32, device="cuda"))
    assert torch.equal(same, D0)
    with pytest.raises(lemo.LemoError) as e:  # fp32 is served by lemo_gather_gemm_add with the transposed weight
        lemo.lemo_gather_gemm_dx(torch.zeros((M, N), device="cuda"), torch.zeros((N, C), device="cuda"), torch.zeros((S, C), device="cuda"), None)
    assert e.value.code == -6


def test_gather_gemm_dx_bench_shape_sampled(lemo):
    """The 32K layer's consumer GEMM backward with respect to the input: M = 9856 kept rows, N = 11008, C = 4096, added into
    dX [32768, 4096]; sampled kept rows (all columns) against the oracle, every other row untouched."""
    cfg = wl.CONFIGS["C5"]
    say("[gemm dX] C5 shape: inputs")
    rng = np.random.default_rng(cfg.seed + 500)
    dY = torch.from_numpy(rng.standard_normal((cfg.M, cfg.N), dtype=np.float32) * np.float32(0.05)).to(torch.bfloat16)
    W = torch.from_numpy(rng.standard_normal((cfg.N, cfg.C), dtype=np.float32) * np.float32(0.02)).to(torch.bfloat16)
    R = torch.from_numpy(rng.standard_normal((cfg.S, cfg.C), dtype=np.float32)).to(torch.bfloat16)
    idx = oracle.select_topk(rng.random(cfg.S).astype(np.float32), cfg.L, cfg.k)
    say("[gemm dX] C5 shape: GPU")
    Rd = R.cuda()
    lemo.lemo_gather_gemm_dx(dY.cuda(), W.cuda(), Rd, torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    got, before = wl.to_bf16_bits(Rd), wl.as_numpy(R)
    mask = np.ones(cfg.S, dtype=bool); mask[idx] = False
    np.testing.assert_array_equal(got[mask], before[mask])
    rows = np.unique(np.concatenate([[0, 127, 128, 255, 256, cfg.M - 257, cfg.M - 129, cfg.M - 1], rng.integers(0, cfg.M, 24)]))
    say(f"[gemm dX] C5 shape: oracle on {len(rows)} rows")
    Wt = np.ascontiguousarray(wl.as_numpy(W).T)
    sub = before[idx[rows]].copy()
    want = oracle.gather_gemm_add(wl.as_numpy(dY), rows.astype(np.int32), Wt, sub, None)
    assert_gemm_add_close(got[idx[rows]], want, before[idx[rows]], wl.as_numpy(dY)[rows], Wt, np.arange(len(rows)))


# ------------------------------------------------------------------------------------ weight gradient of the selective-load GEMM

@pytest.mark.parametrize("S,C,N,M", [(300, 64, 40, 130), (1000, 256, 304, 517), (513, 1000, 264, 513), (64, 8, 8, 1), (700, 512, 4096, 300)])
def test_gather_gemm_dw_bf16(lemo, S, C, N, M):
    say(f"[gemm dW] bf16 S={S} C={C} N={N} M={M}")
    rng = np.random.default_rng(S + C + N + 2)
    X = torch.from_numpy(rng.standard_normal((S, C)).astype(np.float32)).to(torch.bfloat16)
    dY = torch.from_numpy((rng.standard_normal((M, N)) * 0.1).astype(np.float32)).to(torch.bfloat16)
    idx = rng.permutation(S)[:M].astype(np.int32)
    dW = lemo.lemo_gather_gemm_dw(dY.cuda(), X.cuda(), torch.from_numpy(idx).cuda())
    # the gather folded into the transpose == the same call on a materialised compact copy
    dWc = lemo.lemo_gather_gemm_dw(dY.cuda(), X.cuda()[torch.from_numpy(idx).cuda().long()].contiguous(), None)
    torch.cuda.synchronize()
    got = wl.to_bf16_bits(dW)
    np.testing.assert_array_equal(got, wl.to_bf16_bits(dWc))
    want = oracle.gather_gemm_dw(wl.as_numpy(dY), wl.as_numpy(X), idx)
    assert_gemm_close(got, want, np.ascontiguousarray(wl.as_numpy(dY).T), np.ascontiguousarray(wl.as_numpy(X)[idx].T))


def test_gather_gemm_dw_exact_and_edge_cases(lemo):
    say("[gemm dW] exact cases")
    rng = np.random.default_rng(24)
    S, C, N, M = 200, 72, 48, 101
    Xf = (rng.integers(-8, 9, (S, C)) / 4.0).astype(np.float32)
    dYf = (rng.integers(-8, 9, (M, N)) / 8.0).astype(np.float32)
    idx = rng.permutation(S)[:M].astype(np.int32)
    want = dYf.astype(np.float64).T @ Xf[idx].astype(np.float64)
    for dtype in (torch.bfloat16, torch.float32):
        X, dY = torch.from_numpy(Xf).to(dtype), torch.from_numpy(dYf).to(dtype)
        # padded output rows, and a second call into the same buffer (dW is overwritten, not accumulated)
        big = torch.full((N, C + 8), 3.0, dtype=dtype, device="cuda")
        for _ in range(2):
            lemo.lemo_gather_gemm_dw(dY.cuda(), X.cuda(), torch.from_numpy(idx).cuda(), dW=big[:, :C])
        torch.cuda.synchronize()
        assert (big[:, C:] == 3.0).all()
        got = big[:, :C].contiguous()
        if dtype == torch.bfloat16:
            np.testing.assert_array_equal(wl.to_bf16_bits(got), bf16(want))
        else:
            np.testing.assert_array_equal(got.cpu().numpy(), want.astype(np.float32))
    # no kept tokens: an empty sum
    z = lemo.lemo_gather_gemm_dw(torch.empty((0, N), dtype=torch.bfloat16, device="cuda"), torch.from_numpy(Xf).to(torch.bfloat16).cuda(),
                                 torch.empty(0, dtype=torch.int32, device="cuda"))
    assert z.shape == (N, C) and not z.any()
    for dtype in (torch.bfloat16, torch.float32):  # strided output: the columns beside it stay as they are
        big = torch.full((N, C + 8), 3.0, dtype=dtype, device="cuda")
        lemo.lemo_gather_gemm_dw(torch.empty((0, N), dtype=dtype, device="cuda"), torch.from_numpy(Xf).to(dtype).cuda(),
                                 torch.empty(0, dtype=torch.int32, device="cuda"), dW=big[:, :C])
        torch.cuda.synchronize()
        assert not big[:, :C].any() and (big[:, C:] == 3.0).all()
    with pytest.raises(lemo.LemoError) as e:  # N must be a multiple of 8 for bf16
        lemo.lemo_gather_gemm_dw(torch.zeros((M, 44), dtype=torch.bfloat16, device="cuda"), torch.from_numpy(Xf).to(torch.bfloat16).cuda(),
                                 torch.from_numpy(idx).cuda())
    assert e.value.code == -6


def test_gather_gemm_dw_bench_shape_sampled(lemo):
    """The 32K layer's consumer GEMM backward: M = 9856 kept rows, C = 4096, N = 11008; sampled weight rows (all columns)."""
    cfg = wl.CONFIGS["C5"]
    say("[gemm dW] C5 shape: inputs")
    rng = np.random.default_rng(cfg.seed + 400)
    X = torch.from_numpy(rng.standard_normal((cfg.S, cfg.C), dtype=np.float32)).to(torch.bfloat16)
    dY = torch.from_numpy(rng.standard_normal((cfg.M, cfg.N), dtype=np.float32) * np.float32(0.05)).to(torch.bfloat16)
    idx = oracle.select_topk(rng.random(cfg.S).astype(np.float32), cfg.L, cfg.k)
    say("[gemm dW] C5 shape: GPU")
    dW = lemo.lemo_gather_gemm_dw(dY.cuda(), X.cuda(), torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 255, 256, cfg.N - 1], rng.integers(0, cfg.N, 4)]))
    say(f"[gemm dW] C5 shape: oracle on {len(rows)} weight rows")
    dYs = np.ascontiguousarray(wl.as_numpy(dY)[:, rows])
    want = oracle.gather_gemm_dw(dYs, wl.as_numpy(X), idx)
    assert_gemm_close(wl.to_bf16_bits(dW)[rows], want, np.ascontiguousarray(dYs.T), np.ascontiguousarray(wl.as_numpy(X)[idx].T))


# ------------------------------------------------------------------------------------ attention over the kept tokens

def assert_attention_close(got_bits, want_bits, V_kept_bits):
    """GPU: probabilities rounded to bf16 before the second product (2^-9 each, weights summing to one, so at most
    2^-9 * max|V| in the output) and one output rounding (2^-9 relative); the test allows twice that."""
    g = widen(got_bits).astype(np.float64)
    o = widen(want_bits).astype(np.float64)
    vmax = np.abs(widen(V_kept_bits)).max()
    assert np.isfinite(g).all()
    bad = np.abs(g - o) > 2.0 ** -7 * np.abs(o) + 2.0 ** -8 * vmax
    assert not bad.any(), f"{bad.sum()} of {bad.size} outputs beyond tolerance, worst {np.abs(g - o).max():.3e}"
    assert np.sqrt(np.mean((g - o) ** 2)) < 2.0 ** -9 * vmax  # and on average far inside it


ATTN_CASES = [(300, 4, 2, 128, 130), (1000, 8, 2, 128, 517), (700, 2, 2, 64, 300), (64, 1, 1, 128, 1), (2000, 4, 4, 128, 1000),
              (513, 4, 1, 64, 513)]


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("S,H,Hkv,d,M", ATTN_CASES)
def test_kept_attention_small_shapes(lemo, S, H, Hkv, d, M, causal):
    say(f"[attention] S={S} H={H}/{Hkv} d={d} M={M} causal={causal}")
    Q, K = wl.tiny_qk(S, H, Hkv, d, "bf16", seed=S + M, heavy=5)
    V = torch.from_numpy(np.random.default_rng(S).standard_normal((S, Hkv, d)).astype(np.float32)).to(torch.bfloat16)
    idx = np.sort(np.random.default_rng(M).permutation(S)[:M]).astype(np.int32)
    flags = lemo.CAUSAL if causal else 0
    O = lemo.lemo_kept_attention(Q.cuda(), K.cuda(), V.cuda(), torch.from_numpy(idx).cuda(), flags=flags)
    torch.cuda.synchronize()
    want = oracle.kept_attention(wl.as_numpy(Q), wl.as_numpy(K), wl.as_numpy(V), idx, flags=flags)
    assert_attention_close(wl.to_bf16_bits(O), want, wl.as_numpy(V)[idx])


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("M", [127, 128, 129, 255, 256, 257, 320, 384, 385, 511, 512, 513, 640, 769, 1024])
def test_kept_attention_stage_and_block_edges(lemo, M, causal):
    """128-wide heads, kept counts around the kernel's granularities (32-key subtiles, 64-query waves, 128-key stages,
    256-query workgroups): the last stage is ragged or exactly full, waves of the last workgroup hold no query at all, the
    run of stages that need no mask is empty, one stage long, or ends exactly at a workgroup's first query."""
    say(f"[attention] edges M={M} causal={causal}")
    S, H, Hkv, d = M + 37, 4, 2, 128
    Q, K = wl.tiny_qk(S, H, Hkv, d, "bf16", seed=1000 + M, heavy=3)
    V = torch.from_numpy(np.random.default_rng(M).standard_normal((S, Hkv, d)).astype(np.float32)).to(torch.bfloat16)
    idx = np.sort(np.random.default_rng(M + 1).permutation(S)[:M]).astype(np.int32)
    flags = lemo.CAUSAL if causal else 0
    O = lemo.lemo_kept_attention(Q.cuda(), K.cuda(), V.cuda(), torch.from_numpy(idx).cuda(), flags=flags)
    torch.cuda.synchronize()
    want = oracle.kept_attention(wl.as_numpy(Q), wl.as_numpy(K), wl.as_numpy(V), idx, flags=flags)
    assert_attention_close(wl.to_bf16_bits(O), want, wl.as_numpy(V)[idx])


@pytest.mark.parametrize("dominant", [500, 840, 30])
def test_kept_attention_reference_overflow_is_repaired(lemo, dominant):
    """With 128-wide heads the attention kernel freezes the reference of its exponentials in the stages of keys that need
    no mask; a key far later whose logit exceeds that reference by more than the binary32 exponent range overflows the
    normaliser, and the workgroup must then go through its keys again with the ordinary running reference.  A logit of
    ~360 nats against a first-stage maximum near 0 forces that path.  dominant = 500: met in unmasked stages by the later
    query blocks (by every block without the mask), next to rows that never overflow; 840: under the causal mask only
    ever met in masked stages, which keep a running reference; 30: inside the first stage, whose maximum is tracked."""
    say(f"[attention] frozen-reference overflow -> second pass, dominant key {dominant}")
    S, H, d = 900, 2, 128
    rng = np.random.default_rng(321)
    q = np.full((S, H, d), 4.0, dtype=np.float32)
    q[:300] = rng.standard_normal((300, H, d)).astype(np.float32)      # ordinary rows as well
    k = (rng.standard_normal((S, H, d)) * 0.05).astype(np.float32)
    k[dominant] = 8.0                                                  # scale * <q, k> = 128*32/sqrt(128) = 362
    k[777] = -8.0
    Q = torch.from_numpy(q).to(torch.bfloat16)
    K = torch.from_numpy(k).to(torch.bfloat16)
    V = torch.from_numpy(rng.standard_normal((S, H, d)).astype(np.float32)).to(torch.bfloat16)
    for flags in (lemo.CAUSAL, 0):
        O = lemo.lemo_kept_attention(Q.cuda(), K.cuda(), V.cuda(), None, flags=flags)
        torch.cuda.synchronize()
        want = oracle.kept_attention(wl.as_numpy(Q), wl.as_numpy(K), wl.as_numpy(V), np.arange(S, dtype=np.int32), flags=flags)
        assert_attention_close(wl.to_bf16_bits(O), want, wl.as_numpy(V))
        # a row that sees the dominant key is that key's value row
        if flags == 0 or dominant < S - 1:
            np.testing.assert_array_equal(wl.to_bf16_bits(O)[S - 1], np.broadcast_to(wl.as_numpy(V)[dominant], (H, d)))


def test_kept_attention_options(lemo):
    say("[attention] options")
    S, H, Hkv, d, M = 600, 4, 2, 128, 333
    Q, K = wl.tiny_qk(S, H, Hkv, d, "bf16", seed=9)
    V = torch.from_numpy(np.random.default_rng(9).standard_normal((S, Hkv, d)).astype(np.float32)).to(torch.bfloat16)
    idx = np.sort(np.random.default_rng(10).permutation(S)[:M]).astype(np.int32)
    Qd, Kd, Vd, idxd = Q.cuda(), K.cuda(), V.cuda(), torch.from_numpy(idx).cuda()
    O = lemo.lemo_kept_attention(Qd, Kd, Vd, idxd)
    # gathered in place == the same kernel on materialised compact copies (the gather is exact), and repeatable
    Oc = lemo.lemo_kept_attention(Qd[idxd.long()].contiguous(), Kd[idxd.long()].contiguous(), Vd[idxd.long()].contiguous(), None)
    O2 = lemo.lemo_kept_attention(Qd, Kd, Vd, idxd)
    torch.cuda.synchronize()
    assert torch.equal(O, Oc) and torch.equal(O, O2)
    # strided views of a fused QKV buffer, strided output, explicit scale
    qkv = torch.zeros((S, H + 2 * Hkv, d), dtype=torch.bfloat16, device="cuda")
    qkv[:, :H] = Qd; qkv[:, H:H + Hkv] = Kd; qkv[:, H + Hkv:] = Vd
    Obig = torch.zeros((M, H + 1, d), dtype=torch.bfloat16, device="cuda")
    lemo.lemo_kept_attention(qkv[:, :H], qkv[:, H:H + Hkv], qkv[:, H + Hkv:], idxd, scale=1.0 / math.sqrt(d), O=Obig[:, :H])
    torch.cuda.synchronize()
    assert torch.equal(Obig[:, :H], O) and not Obig[:, H].any()
    # dropped tokens have no influence
    Q2, K2, V2 = Qd.clone(), Kd.clone(), Vd.clone()
    drop = torch.from_numpy(np.setdiff1d(np.arange(S), idx)).cuda()
    Q2[drop] += 3.0; K2[drop] -= 2.0; V2[drop] *= 5.0
    assert torch.equal(lemo.lemo_kept_attention(Q2, K2, V2, idxd), O)
    # refused: fp32 inputs, the self-exclusion flag; M == 0 is a no-op
    with pytest.raises(lemo.LemoError) as e:
        lemo.lemo_kept_attention(Qd.float(), Kd.float(), Vd.float(), idxd)
    assert e.value.code == -6
    with pytest.raises(lemo.LemoError):
        lemo.lemo_kept_attention(Qd, Kd, Vd, idxd, flags=lemo.CAUSAL | lemo.EXCLUDE_SELF)
    assert lemo.lemo_kept_attention(Qd, Kd, Vd, torch.empty(0, dtype=torch.int32, device="cuda")).shape == (0, H, d)


def test_kept_attention_full_size(lemo):
    """The 32K-token layer with its 9856 kept tokens and all 32 heads, as the bench runs it: EVERY kept query (all heads,
    all value columns) against the oracle."""
    cfg = wl.CONFIGS["C5"]
    lay = wl.make_layer(cfg, want_gemm=False, device="cuda")
    say("[attention] C5: inputs")
    rng = np.random.default_rng(cfg.seed + 300)
    V = torch.from_numpy(rng.standard_normal((cfg.S, cfg.H_kv, cfg.d), dtype=np.float32)).to(torch.bfloat16)
    idx = oracle.select_topk(rng.random(cfg.S).astype(np.float32), cfg.L, cfg.k)
    say("[attention] C5: GPU")
    O = lemo.lemo_kept_attention(lay["Q"], lay["K"], V.cuda(), torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    got = wl.to_bf16_bits(O)
    assert np.isfinite(widen(got)).all()
    say(f"[attention] C5: oracle on all {cfg.M} kept queries, {oracle.num_threads()} threads")
    Vn = wl.as_numpy(V)
    want = oracle.kept_attention(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]), Vn, idx)
    assert_attention_close(got, want, Vn[idx])


# ------------------------------------------------------------------------------------ scatter-add

@pytest.mark.parametrize("gdt,xdt", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32"), ("f32", "bf16")])
@pytest.mark.parametrize("S,C,M", [(100, 8, 37), (1000, 4096, 400), (513, 264, 513), (50, 64, 0)])
@pytest.mark.parametrize("mode", [0, 1])
def test_scatter_bit_exact(lemo, S, C, M, gdt, xdt, mode):
    say(f"[scatter] S={S} C={C} M={M} {gdt}->{xdt} mode={mode}")
    rng = np.random.default_rng(S + C + M)
    tg = torch.bfloat16 if gdt == "bf16" else torch.float32
    tx = torch.bfloat16 if xdt == "bf16" else torch.float32
    G = torch.from_numpy(rng.standard_normal((M, C)).astype(np.float32)).to(tg)
    D = torch.from_numpy(rng.standard_normal((S, C)).astype(np.float32)).to(tx)
    idx = np.sort(rng.choice(S, M, replace=False)).astype(np.int32)
    Dd = D.cuda()
    lemo.lemo_scatter_grad(G.cuda(), torch.from_numpy(idx).cuda(), Dd, mode=mode)
    torch.cuda.synchronize()
    want = wl.as_numpy(D).copy()
    oracle.scatter_add(wl.as_numpy(G), idx, want, mode=mode)
    np.testing.assert_array_equal(wl.as_numpy(Dd), want)


def test_scatter_unsorted_indices_and_strided_rows(lemo):
    say("[scatter] unsorted indices, padded leading dimension")
    rng = np.random.default_rng(12)
    S, C, M = 400, 128, 150
    G = torch.from_numpy(rng.standard_normal((M, C)).astype(np.float32)).to(torch.bfloat16)
    D = torch.from_numpy(rng.standard_normal((S, C + 32)).astype(np.float32)).to(torch.bfloat16)
    idx = rng.permutation(S)[:M].astype(np.int32)
    Dd = D.cuda()
    lemo.lemo_scatter_grad(G.cuda(), torch.from_numpy(idx).cuda(), Dd[:, :C])
    torch.cuda.synchronize()
    want = np.ascontiguousarray(wl.as_numpy(D)[:, :C])
    oracle.scatter_add(wl.as_numpy(G), idx, want)
    got = wl.as_numpy(Dd)
    np.testing.assert_array_equal(got[:, :C], want)
    np.testing.assert_array_equal(got[:, C:], wl.as_numpy(D)[:, C:])  # the padding columns are not touched


def test_scatter_config_C3_backward(lemo):
    """C3's backward: G ~ N(0,1) [3280,4096] bf16 scatter-added into a zero buffer and into a residual."""
    cfg = wl.CONFIGS["C3"]
    say("[scatter] C3 backward")
    rng = np.random.default_rng(cfg.seed)
    G = torch.from_numpy(rng.standard_normal((cfg.M, cfg.C), dtype=np.float32)).to(torch.bfloat16)
    R = torch.from_numpy(rng.standard_normal((cfg.S, cfg.C), dtype=np.float32)).to(torch.bfloat16)
    idx = oracle.select_topk(rng.random(cfg.S).astype(np.float32), cfg.L, cfg.k)
    idxd = torch.from_numpy(idx).cuda()
    for init in (torch.zeros_like(R), R):
        Dd = init.cuda()
        lemo.lemo_scatter_grad(G.cuda(), idxd, Dd)
        Dd2 = init.cuda()
        lemo.lemo_scatter_grad(G.cuda(), idxd, Dd2)
        torch.cuda.synchronize()
        want = wl.as_numpy(init).copy()
        oracle.scatter_add(wl.as_numpy(G), idx, want)
        np.testing.assert_array_equal(wl.as_numpy(Dd), want)
        assert torch.equal(Dd, Dd2)
    # gather(scatter(G)) on a zero buffer returns G (via an identity-weight-free check: plain row read)
    Z = torch.zeros_like(R).cuda()
    lemo.lemo_scatter_grad(G.cuda(), idxd, Z, mode=1)
    assert torch.equal(Z[idxd.long()].cpu(), G)


def test_scatter_config_C5_backward(lemo):
    """C5's backward at full size (G [9856,4096] bf16 into dX [32768,4096]), the launch bench.py times: bit-exact."""
    cfg = wl.CONFIGS["C5"]
    say("[scatter] C5 backward")
    rng = np.random.default_rng(cfg.seed + 7)
    G = torch.from_numpy(rng.standard_normal((cfg.M, cfg.C), dtype=np.float32)).to(torch.bfloat16)
    R = torch.from_numpy(rng.standard_normal((cfg.S, cfg.C), dtype=np.float32)).to(torch.bfloat16)
    idx = oracle.select_topk(rng.random(cfg.S).astype(np.float32), cfg.L, cfg.k)
    Dd = R.cuda()
    lemo.lemo_scatter_grad(G.cuda(), torch.from_numpy(idx).cuda(), Dd)
    torch.cuda.synchronize()
    want = wl.as_numpy(R).copy()
    oracle.scatter_add(wl.as_numpy(G), idx, want)
    np.testing.assert_array_equal(wl.as_numpy(Dd), want)


def test_error_codes_leave_outputs_untouched(lemo):
    """Bad arguments are refused on the host: an exception with the library's code, nothing launched, outputs as before."""
    say("[errors] refused calls")
    X = torch.randn(64, 64, device="cuda").to(torch.bfloat16)
    W = torch.randn(32, 64, device="cuda").to(torch.bfloat16)
    Y = torch.full((10, 32), 7.0, device="cuda", dtype=torch.bfloat16)
    bad_idx = torch.arange(10, device="cuda", dtype=torch.int32)
    with pytest.raises(lemo.LemoError) as e:
        lemo.lemo_gather_gemm(X[:, :60], bad_idx, W[:, :60], Y=Y)  # C = 60 is not a multiple of 8
    assert e.value.code == -6
    with pytest.raises(lemo.LemoError) as e:
        lemo.lemo_select_topk(torch.zeros(100, device="cuda"), 40000, 5000)  # segment longer than the kernel supports
    assert e.value.code == -6
    Q = torch.randn(100, 2, 96, device="cuda").to(torch.bfloat16)
    with pytest.raises(lemo.LemoError) as e:
        lemo.lemo_score_segments(Q, Q, 64)  # head_dim 96 is not built
    assert e.value.code == -6
    torch.cuda.synchronize()
    assert torch.all(Y == 7.0)


# ------------------------------------------------------------------------------------ whole path

def test_whole_path_small_layer(lemo):
    """score -> select -> gather-GEMM -> scatter on a small bf16 layer, each stage against the oracle fed
    with the oracle's own upstream result."""
    cfg = wl.scaled(wl.CONFIGS["C2"], S=1536, H=8, H_kv=8, C=512, N=768, L=512, ratio=0.4, backward=True)
    say("[path] small layer")
    lay = wl.make_layer(cfg)
    Q, K, X, W, G = (lay[n].cuda() for n in ("Q", "K", "X", "W", "G"))
    scores = lemo.lemo_score_segments(Q, K, cfg.L)
    kept = lemo.lemo_select_topk(scores, cfg.L, cfg.k)
    Y = lemo.lemo_gather_gemm(X, kept, W)
    dX = torch.zeros_like(X)
    lemo.lemo_scatter_grad(G, kept, dX)
    torch.cuda.synchronize()
    o_scores = oracle.score(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]))
    assert_scores_close(scores.cpu().numpy(), o_scores, "path scores")
    kept_np = kept.cpu().numpy()
    assert_selection_equivalent(kept_np, o_scores, cfg.L, cfg.k)
    # downstream stages are compared on the GPU's own kept set (it is valid by the check above)
    assert_gemm_close(wl.to_bf16_bits(Y), oracle.gather_gemm(wl.as_numpy(lay["X"]), kept_np, wl.as_numpy(lay["W"])),
                      wl.as_numpy(lay["X"])[kept_np], wl.as_numpy(lay["W"]))
    want = np.zeros((cfg.S, cfg.C), dtype=np.uint16)
    oracle.scatter_add(wl.as_numpy(lay["G"]), kept_np, want)
    np.testing.assert_array_equal(wl.as_numpy(dX), want)


def test_attention_block_flow(lemo):
    """The attention block of Sec. 4.4 end to end on a small layer: score -> select -> attention over the kept tokens
    (rows read in place) -> output projection added in place into the residual rows; each stage against the oracle fed
    with the GPU's upstream result, and the dropped tokens' residual rows untouched."""
    cfg = wl.scaled(wl.CONFIGS["C2"], S=1024, H=4, H_kv=2, C=512, N=512, L=256, ratio=0.5)
    say("[flow] attention block")
    lay = wl.make_layer(cfg)
    rng = np.random.default_rng(77)
    V = torch.from_numpy(rng.standard_normal((cfg.S, cfg.H_kv, cfg.d), dtype=np.float32)).to(torch.bfloat16)
    Wo = torch.from_numpy(rng.standard_normal((cfg.C, cfg.H * cfg.d), dtype=np.float32) * np.float32(0.02)).to(torch.bfloat16)
    R = torch.from_numpy(rng.standard_normal((cfg.S, cfg.C), dtype=np.float32)).to(torch.bfloat16)
    Q, K = lay["Q"].cuda(), lay["K"].cuda()
    scores = lemo.lemo_score_segments(Q, K, cfg.L)
    kept = lemo.lemo_select_topk(scores, cfg.L, cfg.k)
    O = lemo.lemo_kept_attention(Q, K, V.cuda(), kept)                       # [M, H, d], compact
    Rd = R.cuda()
    lemo.lemo_gather_gemm_add(O.view(cfg.M, cfg.H * cfg.d), None, Wo.cuda(), Rd, kept)
    torch.cuda.synchronize()
    kept_np = kept.cpu().numpy()
    assert_selection_equivalent(kept_np, oracle.score(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"])), cfg.L, cfg.k)
    want_O = oracle.kept_attention(wl.as_numpy(lay["Q"]), wl.as_numpy(lay["K"]), wl.as_numpy(V), kept_np)
    assert_attention_close(wl.to_bf16_bits(O), want_O, wl.as_numpy(V)[kept_np])
    O2 = wl.to_bf16_bits(O).reshape(cfg.M, cfg.H * cfg.d)
    before = wl.as_numpy(R)
    want_R = oracle.gather_gemm_add(O2, None, wl.as_numpy(Wo), before.copy(), kept_np)
    assert_gemm_add_close(wl.to_bf16_bits(Rd), want_R, before, O2, wl.as_numpy(Wo), kept_np)


# ------------------------------------------------------------------------------------ randomised sweep over every entry point

def test_randomised_shapes_every_entry_point(lemo):
    """Seeded random shapes, flags, segment / block sizes and index sets for all entry points against the oracle, each to
    the bar of its own section above (odd sizes, ragged tails, GQA ratios, empty and full kept sets come up by chance)."""
    rng = np.random.default_rng(2025)
    bf = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    for it in range(24):
        S = int(rng.integers(1, 1200)); H = int(rng.choice([1, 2, 4, 8])); Hkv = int(rng.choice([h for h in (1, 2, 4, 8) if H % h == 0]))
        d = int(rng.choice([64, 128])); dtype = str(rng.choice(["bf16", "f32"])); flags = int(rng.integers(0, 4)); L = int(rng.integers(1, 600))
        k = int(rng.integers(1, L + 1)); b = int(rng.choice([32, 64, 96, 128])); mode = int(rng.integers(0, 2))
        C = int(rng.choice([8, 64, 136, 256, 520])); N = int(rng.choice([8, 40, 264, 512])); M = int(rng.integers(0, S + 1))
        say(f"[random] it={it} S={S} H={H}/{Hkv} d={d} {dtype} flags={flags} L={L} k={k} b={b} mode={mode} C={C} N={N} M={M}")
        Q, K = wl.tiny_qk(S, H, Hkv, d, dtype, seed=int(rng.integers(1 << 30)), heavy=3)
        Qn, Kn = wl.as_numpy(Q), wl.as_numpy(K)
        scores, col, dg = run_score(lemo, Q, K, L, flags)
        o_s, o_col, o_dg = oracle.score(Qn, Kn, flags=flags, per_head=True)
        assert_scores_close(scores, o_s, "scores"); assert_scores_close(col, o_col, "column sums"); assert_scores_close(dg, o_dg, "diagonal")
        sc = rng.choice([-1.0, 0.0, 0.5, 0.5, 2.0, 1e-20], size=S).astype(np.float32) if it % 2 else rng.standard_normal(S).astype(np.float32)
        np.testing.assert_array_equal(lemo.lemo_select_topk(torch.from_numpy(sc).cuda(), L, k).cpu().numpy(), oracle.select_topk(sc, L, k))
        sb, tb = lemo.lemo_score_blocks(Q.cuda(), K.cuda(), b, flags=flags, mode=mode)
        w_sb, w_tb = oracle.score_blocks(Qn, Kn, b, flags=flags, mode=mode)
        atol = 1e-6 if mode == 0 else 1e-5
        assert_blocks_close(sb.cpu().numpy(), w_sb, "score blocks", atol); assert_blocks_close(tb.cpu().numpy(), w_tb, "token blocks", atol)
        T0 = float(np.sort(w_tb)[len(w_tb) // 2])
        kept_t, cnt = lemo.lemo_select_threshold(tb, S, b, T0)
        np.testing.assert_array_equal(kept_t.cpu().numpy()[:int(cnt.item())], oracle.select_threshold(tb.cpu().numpy(), S, b, T0))
        if M == 0:
            continue
        X, W, idx = bf(rng.standard_normal((S, C))), bf(rng.standard_normal((N, C)) * 0.05), rng.permutation(S)[:M].astype(np.int32)
        Xn, Wn, idxd = wl.as_numpy(X), wl.as_numpy(W), torch.from_numpy(idx).cuda()
        assert_gemm_close(wl.to_bf16_bits(lemo.lemo_gather_gemm(X.cuda(), idxd, W.cuda())), oracle.gather_gemm(Xn, idx, Wn), Xn[idx], Wn)
        So = int(rng.integers(M, M + 50)); R = bf(rng.standard_normal((So, N))); oidx = rng.permutation(So)[:M].astype(np.int32)
        Rd = R.cuda()
        lemo.lemo_gather_gemm_add(X.cuda(), idxd, W.cuda(), Rd, torch.from_numpy(oidx).cuda())
        before = wl.as_numpy(R)
        assert_gemm_add_close(wl.to_bf16_bits(Rd), oracle.gather_gemm_add(Xn, idx, Wn, before.copy(), oidx), before, Xn[idx], Wn, oidx)
        dY = bf(rng.standard_normal((M, N)) * 0.1)
        assert_gemm_close(wl.to_bf16_bits(lemo.lemo_gather_gemm_dw(dY.cuda(), X.cuda(), idxd)), oracle.gather_gemm_dw(wl.as_numpy(dY), Xn, idx),
                          np.ascontiguousarray(wl.as_numpy(dY).T), np.ascontiguousarray(Xn[idx].T))
        G, dX = bf(rng.standard_normal((M, C))), bf(rng.standard_normal((S, C)))
        dXd = dX.cuda()
        lemo.lemo_scatter_grad(G.cuda(), idxd, dXd)
        np.testing.assert_array_equal(wl.as_numpy(dXd), oracle.scatter_add(wl.as_numpy(G), idx, wl.as_numpy(dX).copy()))
        if dtype == "bf16":
            V, sidx, causal = bf(rng.standard_normal((S, Hkv, d))), np.sort(idx), flags & 1
            O = lemo.lemo_kept_attention(Q.cuda(), K.cuda(), V.cuda(), torch.from_numpy(sidx).cuda(), flags=causal)
            assert_attention_close(wl.to_bf16_bits(O), oracle.kept_attention(Qn, Kn, wl.as_numpy(V), sidx, flags=causal), wl.as_numpy(V)[sidx])
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------ the path replayed from a HIP graph

def test_hot_path_replayed_from_a_hip_graph(lemo):
    """The calls only launch kernels on the caller's stream, so the whole path can be captured once and replayed.
    Every replay runs on new inputs (written in place by ordinary eager work between the replays) and must give the
    bits of the same calls issued eagerly."""
    S, H, Hkv, d, L, k, C, N = 1500, 4, 2, 128, 256, 100, 256, 264
    M = lemo.lemo_kept_count(S, L, k)
    say(f"[graph] S={S} H={H}/{Hkv} d={d} L={L} k={k} C={C} N={N} M={M}")
    g = torch.Generator(device="cuda").manual_seed(7)
    rnd = lambda *shape: torch.randn(shape, device="cuda", dtype=torch.float32, generator=g)
    Q, K = rnd(S, H, d).to(torch.bfloat16), rnd(S, Hkv, d).to(torch.bfloat16)
    X, W, G = rnd(S, C).to(torch.bfloat16), (rnd(N, C) * 0.05).to(torch.bfloat16), rnd(M, C).to(torch.bfloat16)
    scores = torch.empty(S, dtype=torch.float32, device="cuda")
    ws = torch.empty(lemo.lemo_score_workspace_bytes(S, H, Hkv, d, lemo.BF16), dtype=torch.uint8, device="cuda")
    kept = torch.empty(M, dtype=torch.int32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((S, C), dtype=torch.bfloat16, device="cuda")

    col = torch.empty((H, S), dtype=torch.float32, device="cuda")
    dg = torch.empty((H, S), dtype=torch.float32, device="cuda")
    scores2 = torch.empty(S, dtype=torch.float32, device="cuda")
    scores3 = torch.empty(S, dtype=torch.float32, device="cuda")
    kept2 = torch.empty(M, dtype=torch.int32, device="cuda")

    def path():
        lemo.lemo_score_segments(Q, K, L, scores=scores, colsum_per_head=col, diag_per_head=dg, workspace=ws)
        lemo.lemo_select_topk(scores, L, k, kept_idx=kept)
        lemo.lemo_head_mean_select_topk(col, dg, L, k, scores=scores2, kept_idx=kept2)   # the same two steps in one launch
        lemo.lemo_score_segments_static(Q, K, L, scores3)                                  # the scoring without a workspace
        lemo.lemo_gather_gemm(X, kept, W, Y=Y)
        lemo.lemo_scatter_grad(G, kept, dX, mode=lemo.SCATTER_ZERO_PAD)

    def outputs():
        torch.cuda.synchronize()
        assert torch.equal(scores, scores2) and torch.equal(kept, kept2) and torch.equal(scores, scores3)
        return [t.clone() for t in (scores, kept, Y, dX)]

    path()  # eager first: the first call of an entry point sets kernel attributes, which is not a stream operation
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    for rep in range(3):
        say(f"[graph] replay {rep}")
        Q.copy_(rnd(S, H, d))  # eager work between the replays
        X.copy_(rnd(S, C))
        for t in (scores, scores2, scores3, Y, dX):
            t.fill_(7.0)
        kept.fill_(-1)
        kept2.fill_(-1)
        graph.replay()
        replayed = outputs()
        for t in (scores, scores2, scores3, Y, dX):
            t.fill_(5.0)
        kept.fill_(-2)
        kept2.fill_(-2)
        path()
        eager = outputs()
        for a, b, what in zip(replayed, eager, ("scores", "kept_idx", "Y", "dX")):
            assert torch.equal(a, b), f"replay {rep}: {what} differs from the eager calls"
