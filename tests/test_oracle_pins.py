"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without any GPU.

The paper prints no worked numeric example for scoring / selection / gather / scatter, so the
oracle is pinned by: a hand-derived two-token example (tests/golden), the textbook dense softmax
written with numpy, closed forms (harmonic numbers under a causal mask), invariances of softmax,
an argsort reference for top-k, numpy float64 matmul, and the gather/scatter adjoint identity.
Each test is chosen so that a plausible slip in the oracle (dropped diagonal, wrong GQA head,
transposed operand, wrong tie rule, double rounding) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import BF16, CAUSAL, EXCLUDE_SELF, F32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16_bits(x):
    """Independent bf16 rounding (torch's) of a float32/float64 numpy array -> uint16 bits."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def widen(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def textbook_scores(Q, K, flags, scale=None):
    """Dense numpy statement of Eq. 1-2 (Sec. 4.2): softmax(QK^T * scale) per head, column sums with
    the diagonal optionally left out, mean over heads.  Q [S,H,d], K [S,H_kv,d] float64."""
    S, H, d = Q.shape
    Hkv = K.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    total = np.zeros(S)
    per_head = np.zeros((H, S))
    for h in range(H):
        g = (h * Hkv) // H
        logits = scale * (Q[:, h, :] @ K[:, g, :].T)
        if flags & CAUSAL:
            logits = np.where(np.tri(S, dtype=bool), logits, -np.inf)
        logits = logits - logits.max(axis=1, keepdims=True)
        P = np.exp(logits)
        P /= P.sum(axis=1, keepdims=True)
        per_head[h] = P.sum(axis=0)
        if flags & EXCLUDE_SELF:
            P = P - np.diag(np.diag(P))
        total += P.sum(axis=0)
    return total / H, per_head


def rand_qk(S, H, Hkv, d, seed, dtype="f32"):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((S, H, d)).astype(np.float32)
    k = rng.standard_normal((S, Hkv, d)).astype(np.float32)
    k[rng.choice(S, size=max(1, S // 16), replace=False)] *= 4.0
    if dtype == "bf16":
        return bf16_bits(q), bf16_bits(k)
    return q, k


def f64(a):
    return (widen(a) if a.dtype == np.uint16 else a).astype(np.float64)


# ------------------------------------------------------------------------------ scoring

def test_golden_two_token_example():
    """Hand-derived example (tests/golden/score_two_tokens.txt): d=1, scale=1, q=(1,1), k=(0, ln 3)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "score_two_tokens.txt")) if l.strip() and not l.startswith("#")]
    want = {r[0]: [float(v) for v in r[1:]] for r in rows}
    Q = np.ones((2, 1, 1), dtype=np.float32)
    K = np.array([0.0, math.log(3.0)], dtype=np.float32).reshape(2, 1, 1)
    # float32(ln 3) is not exactly ln 3; the fixture is exact to ~1e-7, so compare to 1e-6
    s, col, dg = oracle.score(Q, K, flags=CAUSAL | EXCLUDE_SELF, scale=1.0, per_head=True)
    np.testing.assert_allclose(col[0], want["colsum_causal"], rtol=1e-6)
    np.testing.assert_allclose(dg[0], want["diag_causal"], rtol=1e-6)
    np.testing.assert_allclose(s, want["score_causal_exclude_self"], rtol=1e-6, atol=1e-12)
    s = oracle.score(Q, K, flags=CAUSAL, scale=1.0)
    np.testing.assert_allclose(s, want["score_causal"], rtol=1e-6)
    s = oracle.score(Q, K, flags=0, scale=1.0)
    np.testing.assert_allclose(s, want["score_full"], rtol=1e-6)
    s = oracle.score(Q, K, flags=EXCLUDE_SELF, scale=1.0)
    np.testing.assert_allclose(s, want["score_full_exclude_self"], rtol=1e-6)


@pytest.mark.parametrize("flags", [0, CAUSAL, EXCLUDE_SELF, CAUSAL | EXCLUDE_SELF])
@pytest.mark.parametrize("S,H,Hkv,d,dtype", [(37, 4, 2, 16, "f32"), (64, 2, 2, 64, "bf16"), (129, 8, 2, 32, "bf16"), (1, 2, 1, 8, "f32")])
def test_score_matches_textbook_softmax(S, H, Hkv, d, dtype, flags):
    Q, K = rand_qk(S, H, Hkv, d, seed=S * 7 + H, dtype=dtype)
    s, col, dg = oracle.score(Q, K, flags=flags, per_head=True)
    want, want_col = textbook_scores(f64(Q), f64(K), flags)
    np.testing.assert_allclose(col, want_col, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(s, want.astype(np.float32), rtol=2e-7, atol=1e-12)


@pytest.mark.parametrize("flags", [0, CAUSAL, EXCLUDE_SELF, CAUSAL | EXCLUDE_SELF])
def test_score_rowwise_equals_bruteforce_matrix(flags):
    Q, K = rand_qk(200, 4, 2, 32, seed=5, dtype="bf16")
    a = oracle.score(Q, K, flags=flags)
    b = oracle.score_bruteforce(Q, K, flags=flags)
    np.testing.assert_allclose(a, b, rtol=3e-7, atol=1e-12)


@pytest.mark.parametrize("flags", [0, CAUSAL])
def test_per_head_column_sums_total_the_query_count(flags):
    """Every softmax row sums to one, so each head's column sums (diagonal included) total S."""
    Q, K = rand_qk(301, 6, 3, 32, seed=11)
    _, col, _ = oracle.score(Q, K, flags=flags, per_head=True)
    np.testing.assert_allclose(col.sum(axis=1), 301.0, rtol=1e-12)
    # and the mean-over-heads score (diagonal included) totals S as well
    s = oracle.score(Q, K, flags=flags)
    assert abs(float(s.astype(np.float64).sum()) - 301.0) < 1e-3


def test_closed_form_constant_logits():
    """Q == 0 makes every allowed probability uniform: non-causal columns are 1; causal column j is
    sum_{i>=j} 1/(i+1) = H_S - H_j, minus 1/(j+1) when the self term is excluded."""
    S, H, d = 97, 3, 16
    Q = np.zeros((S, H, d), dtype=np.float32)
    K = np.random.default_rng(0).standard_normal((S, H, d)).astype(np.float32)
    harm = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, S + 1))])  # harm[n] = H_n
    np.testing.assert_allclose(oracle.score(Q, K, flags=0), np.ones(S), rtol=1e-6)
    np.testing.assert_allclose(oracle.score(Q, K, flags=EXCLUDE_SELF), np.full(S, 1.0 - 1.0 / S), rtol=1e-6)
    j = np.arange(S)
    np.testing.assert_allclose(oracle.score(Q, K, flags=CAUSAL), harm[S] - harm[j], rtol=1e-6)
    np.testing.assert_allclose(oracle.score(Q, K, flags=CAUSAL | EXCLUDE_SELF), harm[S] - harm[j + 1], rtol=1e-6, atol=1e-7)


def test_causal_edges():
    Q, K = rand_qk(50, 2, 2, 16, seed=3)
    s, col, dg = oracle.score(Q, K, flags=CAUSAL | EXCLUDE_SELF, per_head=True)
    assert np.all(col[:, 0] >= 1.0)          # token 0 gets all of query 0's mass
    np.testing.assert_array_equal(col[:, -1], dg[:, -1])  # last column holds only its own diagonal
    assert s[-1] == 0.0                       # ... so with the self term excluded it scores exactly 0
    np.testing.assert_array_equal(dg[:, 0], 1.0)


def test_key_shift_invariance():
    """Adding one vector v to every key shifts each query's logits by the constant <q_i, v>:
    softmax, and hence every score, is unchanged.  Values sit on a dyadic grid so the shift is exact."""
    rng = np.random.default_rng(8)
    S, H, d = 40, 2, 8
    Q = (rng.integers(-8, 9, (S, H, d)) / 4.0).astype(np.float32)
    K = (rng.integers(-8, 9, (S, H, d)) / 4.0).astype(np.float32)
    v = (rng.integers(-8, 9, (1, H, d)) / 4.0).astype(np.float32)
    for flags in (0, CAUSAL | EXCLUDE_SELF):
        a = oracle.score(Q, K, flags=flags)
        b = oracle.score(Q, K + v, flags=flags)
        np.testing.assert_allclose(a, b, rtol=1e-6, atol=1e-9)


def test_permutation_equivariance_noncausal():
    Q, K = rand_qk(60, 3, 3, 16, seed=21)
    rng = np.random.default_rng(2)
    pk, pq = rng.permutation(60), rng.permutation(60)
    base = oracle.score(Q, K, flags=0)
    np.testing.assert_allclose(oracle.score(Q, K[pk], flags=0), base[pk], rtol=1e-6)      # keys permute scores
    np.testing.assert_allclose(oracle.score(Q[pq], K, flags=0), base, rtol=1e-6)          # queries do not


def test_dominant_key_collects_all_queries():
    """A key hugely aligned with a direction every query shares takes ~all mass of every allowed query."""
    S, H, d = 64, 2, 8
    rng = np.random.default_rng(4)
    Q = rng.standard_normal((S, H, d)).astype(np.float32) * 0.1
    Q[..., 0] = 1.0
    K = rng.standard_normal((S, H, d)).astype(np.float32) * 0.1
    j = 17
    K[j, :, 0] = 1e3
    s = oracle.score(Q, K, flags=0)
    assert abs(s[j] - S) < 1e-3
    s = oracle.score(Q, K, flags=CAUSAL)
    assert abs(s[j] - (S - j)) < 1e-3


def test_gqa_head_mapping_and_strides():
    """Query head h reads KV head floor(h*H_kv/H); strided (non-contiguous) Q/K views are honoured."""
    S, H, Hkv, d = 33, 6, 2, 16
    Q, K = rand_qk(S, H, Hkv, d, seed=9)
    Kexp = np.repeat(K, H // Hkv, axis=1)  # explicit expansion: head h -> K[:, h // 3]
    np.testing.assert_array_equal(oracle.score(Q, K), oracle.score(Q, Kexp))
    big = np.zeros((S, H + 2, d + 8), dtype=np.float32)
    big[:, 1:H + 1, :d] = Q
    np.testing.assert_array_equal(oracle.score(big[:, 1:H + 1, :d], K), oracle.score(Q, K))
    # a wrong mapping (h % H_kv) would differ:
    Kwrong = K[:, [h % Hkv for h in range(H)]]
    assert not np.allclose(oracle.score(Q, Kwrong), oracle.score(Q, K), rtol=1e-4)


def test_scale_argument():
    Q, K = rand_qk(20, 2, 2, 16, seed=1)
    np.testing.assert_array_equal(oracle.score(Q, K, scale=0.0), oracle.score(Q, K, scale=0.25))
    want, _ = textbook_scores(f64(Q), f64(K), CAUSAL | EXCLUDE_SELF, scale=0.7)
    np.testing.assert_allclose(oracle.score(Q, K, scale=0.7), want, rtol=3e-7, atol=1e-12)


# ------------------------------------------------------------------------------ bf16 rounding

def test_bf16_rounding_against_torch():
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(2000).astype(np.float32),
        (rng.standard_normal(500) * 1e-39).astype(np.float32),  # subnormal range
        (rng.standard_normal(500) * 1e38).astype(np.float32),   # near overflow
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 1.005859375, 3.3895314e38, 3.4e38, np.inf, -np.inf,
                  2 ** -133, 2 ** -134, 1.5 * 2 ** -133, 2 ** -126], dtype=np.float32),
    ])
    # exact ties: 8 significant bits + a half-ulp
    ties = (np.arange(128, 256, dtype=np.float64) + 0.5) / 128.0
    vals = np.concatenate([vals, ties.astype(np.float32), -ties.astype(np.float32)])
    want = bf16_bits(vals)
    got = np.array([oracle.double_to_bf16_bits(float(v)) for v in vals], dtype=np.uint16)
    np.testing.assert_array_equal(got, want)


def test_bf16_rounding_is_single_step_from_double():
    """1 + 2^-8 + 2^-30 lies above the tie between 1 and 1+2^-7, so it rounds UP; rounding to float32
    first would land exactly on the tie and go down (to even)."""
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert oracle.double_to_bf16_bits(x) == 0x3F81
    assert oracle.double_to_bf16_bits(1.0 + 2.0 ** -8) == 0x3F80


# ------------------------------------------------------------------------------ selection

def argsort_topk(scores, L, k):
    S = len(scores)
    out = []
    for s0 in range(0, S, L):
        seg = scores[s0:s0 + L].astype(np.float64)
        seg = np.where(seg == 0.0, 0.0, seg)  # -0.0 == +0.0
        n = len(seg)
        kk = k if n == L else max(1, min(n, -(-k * n // L)))
        order = np.lexsort((np.arange(n), -seg))  # primary: score descending; secondary: index ascending
        out.extend(sorted(s0 + order[:kk]))
    return np.array(out, dtype=np.int32)


@pytest.mark.parametrize("S,L,k", [(1024, 128, 64), (1000, 128, 64), (7, 4, 3), (1, 8, 8), (513, 512, 205), (300, 100, 1), (300, 100, 100)])
def test_select_against_argsort(S, L, k):
    rng = np.random.default_rng(S + L + k)
    scores = rng.random(S).astype(np.float32)
    scores[rng.integers(0, S, S // 3)] = np.float32(0.25)  # many exact ties
    got = oracle.select_topk(scores, L, k)
    np.testing.assert_array_equal(got, argsort_topk(scores, L, k))
    assert len(got) == oracle.kept_count(S, L, k)
    assert np.all(np.diff(got) > 0)


def test_select_special_cases():
    S, L = 256, 64
    rng = np.random.default_rng(1)
    scores = rng.standard_normal(S).astype(np.float32)
    np.testing.assert_array_equal(oracle.select_topk(scores, L, L), np.arange(S))                  # k = L: identity
    first_argmax = [s0 + int(np.argmax(scores[s0:s0 + L])) for s0 in range(0, S, L)]
    np.testing.assert_array_equal(oracle.select_topk(scores, L, 1), first_argmax)                  # k = 1: argmax
    const = np.full(S, 0.5, dtype=np.float32)
    want = np.concatenate([np.arange(s0, s0 + 10) for s0 in range(0, S, L)])
    np.testing.assert_array_equal(oracle.select_topk(const, L, 10), want)                          # ties: lowest indices
    z = np.array([-0.0, 0.0, -0.0, 0.0, -1.0, -1.0], dtype=np.float32)
    np.testing.assert_array_equal(oracle.select_topk(z, 6, 2), [0, 1])                             # -0.0 ties +0.0
    dup = np.array([1.0, 3.0, 3.0, 2.0, 3.0, 0.0], dtype=np.float32)
    np.testing.assert_array_equal(oracle.select_topk(dup, 6, 2), [1, 2])
    np.testing.assert_array_equal(oracle.select_topk(dup, 6, 4), [1, 2, 3, 4])


def test_select_kept_dominate_dropped():
    rng = np.random.default_rng(3)
    S, L, k = 2000, 256, 77
    scores = rng.standard_normal(S).astype(np.float32)
    kept = oracle.select_topk(scores, L, k)
    mask = np.zeros(S, bool)
    mask[kept] = True
    for s0 in range(0, S, L):
        seg, m = scores[s0:s0 + L], mask[s0:s0 + L]
        assert seg[m].min() >= seg[~m].max()


def test_keep_k_and_kept_count():
    assert oracle.keep_k(128, 0.5) == 64
    assert oracle.keep_k(512, 0.4) == 205     # ceil(204.8)
    assert oracle.keep_k(1024, 0.3) == 308    # ceil(307.2)
    assert oracle.keep_k(1024, 0.5) == 512
    assert oracle.keep_k(10, 0.0) == 1 and oracle.keep_k(10, 2.0) == 10
    assert oracle.kept_count(8192, 512, 205) == 3280
    assert oracle.kept_count(32768, 1024, 308) == 9856
    assert oracle.kept_count(1000, 128, 64) == 7 * 64 + 52  # tail of 104 keeps ceil(64*104/128) = 52
    assert oracle.kept_count(10, 4, 5) == -1


# ------------------------------------------------------------------------------ block-wise informativeness, thresholds

def dense_blocks(Q, K, b, flags, scale=None, mode=0):
    """Dense numpy statement of Eq. 2 and the token-block sum (Sec. 4.2): per-head scores, positive terms summed over
    heads and divided by the head count, zero where a pair is not admitted, padded to whole blocks, maximum over every
    b x b block, column sums of the block matrix.  Q [S,H,d], K [S,H_kv,d] float64."""
    S, H, d = Q.shape
    Hkv = K.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    i, j = np.meshgrid(np.arange(S), np.arange(S), indexing="ij")
    allowed = (j <= i) if flags & CAUSAL else np.ones((S, S), dtype=bool)
    mean = np.zeros((S, S))
    for h in range(H):
        logits = scale * (Q[:, h, :] @ K[:, h * Hkv // H, :].T)
        if mode == 0:
            z = np.where(allowed, logits, -np.inf)
            e = np.exp(z - z.max(axis=1, keepdims=True))
            sc = e / e.sum(axis=1, keepdims=True)
        else:
            sc = logits
        mean += np.where(allowed & (sc > 0), sc, 0.0)
    mean /= H
    admitted = allowed & ~((i == j) if flags & EXCLUDE_SELF else np.zeros((S, S), dtype=bool))
    mean = np.where(admitted, mean, 0.0)
    nb = -(-S // b)
    padded = np.zeros((nb * b, nb * b))
    padded[:S, :S] = mean
    blocks = padded.reshape(nb, b, nb, b).max(axis=(1, 3))
    return blocks, blocks.sum(axis=0)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("flags", [0, CAUSAL, EXCLUDE_SELF, CAUSAL | EXCLUDE_SELF])
@pytest.mark.parametrize("S,H,Hkv,d,b,dtype", [(37, 2, 2, 8, 8, "f32"), (64, 4, 2, 16, 16, "bf16"), (50, 3, 1, 4, 7, "f32"),
                                               (33, 1, 1, 8, 32, "bf16"), (20, 2, 1, 8, 1, "f32")])
def test_blocks_against_dense_numpy(S, H, Hkv, d, b, dtype, flags, mode):
    rng = np.random.default_rng(S * 7 + b)
    Q = rng.standard_normal((S, H, d)).astype(np.float32)
    K = (rng.standard_normal((S, Hkv, d)) * 1.5).astype(np.float32)
    if dtype == "bf16":
        Qin, Kin = bf16_bits(Q), bf16_bits(K)
        Q, K = widen(Qin), widen(Kin)
    else:
        Qin, Kin = Q, K
    want_sb, want_tb = dense_blocks(Q.astype(np.float64), K.astype(np.float64), b, flags, mode=mode)
    sb, tb = oracle.score_blocks(Qin, Kin, b, flags=flags, mode=mode)
    np.testing.assert_allclose(sb, want_sb, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(tb, want_tb, rtol=1e-6, atol=1e-12)
    rows = [0, sb.shape[0] - 1, sb.shape[0] // 2]  # the spot-check routine is the same arithmetic, row by row
    np.testing.assert_array_equal(oracle.score_block_rows(Qin, Kin, b, rows, flags=flags, mode=mode), sb[rows])
    if mode == 1:  # a scale argument multiplies the logit variant through
        sb2, _ = oracle.score_blocks(Qin, Kin, b, flags=flags, mode=1, scale=0.5)
        np.testing.assert_allclose(sb2, want_sb * 0.5 * math.sqrt(d), rtol=1e-12, atol=1e-15)


def test_blocks_golden_four_token_example():
    """Hand-derived example (tests/golden/score_blocks_four_tokens.txt): zero queries, causal, one head, b = 2."""
    rows = {l.split()[0]: [float(x) for x in l.split()[1:]]
            for l in open(os.path.join(GOLDEN, "score_blocks_four_tokens.txt")) if l.strip() and not l.startswith("#")}
    Q = np.zeros((4, 1, 4), dtype=np.float32)
    K = np.random.default_rng(1).standard_normal((4, 1, 4)).astype(np.float32)
    sb, tb = oracle.score_blocks(Q, K, 2, flags=CAUSAL)
    np.testing.assert_allclose(sb.ravel(), rows["score_blocks_causal"], rtol=1e-15)
    np.testing.assert_allclose(tb, rows["token_blocks_causal"], rtol=1e-7)
    sb, tb = oracle.score_blocks(Q, K, 2, flags=CAUSAL | EXCLUDE_SELF)
    np.testing.assert_allclose(sb.ravel(), rows["score_blocks_causal_exclude_self"], rtol=1e-15)
    np.testing.assert_allclose(tb, rows["token_blocks_causal_exclude_self"], rtol=1e-7)
    for flags in (0, EXCLUDE_SELF):
        np.testing.assert_allclose(oracle.score_blocks(Q, K, 2, flags=flags)[1], rows["token_blocks_full"], rtol=1e-7)


def test_blocks_special_cases():
    rng = np.random.default_rng(31)
    S, H, d = 96, 4, 16
    Q = rng.standard_normal((S, H, d)).astype(np.float32)
    K = rng.standard_normal((S, 2, d)).astype(np.float32)
    for flags in (0, CAUSAL, CAUSAL | EXCLUDE_SELF):
        # blocks of one token: the token-block score is Eq. 1's column sum (head mean), already pinned above
        np.testing.assert_allclose(oracle.score_blocks(Q, K, 1, flags=flags)[1], oracle.score(Q, K, flags=flags), rtol=1e-6, atol=1e-9)
        # one block holding everything: its score is the largest admitted head-mean probability
        sb, tb = oracle.score_blocks(Q, K, S, flags=flags)
        assert sb.shape == (1, 1) and np.float32(sb[0, 0]) == tb[0]
        assert sb[0, 0] == pytest.approx(dense_blocks(Q.astype(np.float64), K.astype(np.float64), 1, flags)[0].max(), rel=1e-12)
    # closed form for constant logits under a causal mask: row i holds 1/(i+1) on its allowed keys, so a score block
    # below the diagonal is worth 1/(m*b+1), the diagonal one 1/(n*b+1) (1/(n*b+2) once self pairs are left out)
    b, nb = 8, S // 8
    Z = np.zeros_like(Q)
    _, tb = oracle.score_blocks(Z, K, b, flags=CAUSAL)
    want = [sum(1.0 / (m * b + 1) for m in range(n, nb)) for n in range(nb)]
    np.testing.assert_allclose(tb, want, rtol=1e-6)
    _, tb = oracle.score_blocks(Z, K, b, flags=CAUSAL | EXCLUDE_SELF)
    want = [1.0 / (n * b + 2) + sum(1.0 / (m * b + 1) for m in range(n + 1, nb)) for n in range(nb)]
    np.testing.assert_allclose(tb, want, rtol=1e-6)
    # logit variant: only positive logits count, so negating K flips which pairs contribute; all-negative logits give 0
    Qp, Kp = np.abs(Q), np.abs(K)
    assert not oracle.score_blocks(Qp, -Kp, b, flags=0, mode=1)[1].any()
    assert (oracle.score_blocks(Qp, Kp, b, flags=0, mode=1)[1] > 0).all()
    # head order does not matter; a KV head shared by two query heads is the same as two equal KV heads
    perm = [2, 3, 0, 1]
    np.testing.assert_allclose(oracle.score_blocks(Q[:, perm], K[:, [1, 0]], b)[1], oracle.score_blocks(Q, K, b)[1], rtol=1e-6)
    np.testing.assert_array_equal(oracle.score_blocks(Q, np.repeat(K, 2, axis=1), b)[1], oracle.score_blocks(Q, K, b)[1])


def test_threshold_selection_and_initial_threshold():
    rng = np.random.default_rng(32)
    for S, b in ((100, 8), (64, 16), (7, 32), (33, 1)):
        nb = -(-S // b)
        tb = rng.random(nb).astype(np.float32)
        T = float(np.sort(tb)[nb // 2])  # a value that occurs: equality keeps the block
        want = np.nonzero(np.repeat(tb >= np.float32(T), b)[:S])[0]
        got = oracle.select_threshold(tb, S, b, T)
        np.testing.assert_array_equal(got, want)
        assert got.dtype == np.int32
        assert len(oracle.select_threshold(tb, S, b, -np.inf)) == S
        assert len(oracle.select_threshold(tb, S, b, np.inf)) == 0
        assert oracle.threshold_init(tb) == pytest.approx(float(np.mean(tb.astype(np.float64))), rel=1e-12)
    # Alg. 1 step 1 on real block scores: the mean threshold keeps some blocks and drops some
    Q = rng.standard_normal((128, 2, 8)).astype(np.float32)
    K = rng.standard_normal((128, 2, 8)).astype(np.float32)
    K[40:48] *= 4.0
    _, tb = oracle.score_blocks(Q, K, 8)
    kept = oracle.select_threshold(tb, 128, 8, oracle.threshold_init(tb))
    assert 0 < len(kept) < 128 and len(kept) % 8 == 0
    assert set(range(40, 48)) <= set(kept.tolist())  # the block with the strong keys survives


# ------------------------------------------------------------------------------ gather-GEMM

def test_gemm_exact_on_dyadic_grid():
    """Inputs on a coarse dyadic grid make every dot product exactly representable, so the result
    must equal numpy's float64 matmul rounded once to bf16 (torch's rounding), bit for bit."""
    rng = np.random.default_rng(5)
    S, C, N, M = 50, 64, 24, 31
    X = (rng.integers(-8, 9, (S, C)) / 4.0).astype(np.float32)
    W = (rng.integers(-8, 9, (N, C)) / 8.0).astype(np.float32)
    b = (rng.integers(-8, 9, N) / 2.0).astype(np.float32)
    idx = np.sort(rng.choice(S, M, replace=False)).astype(np.int32)
    want = X[idx].astype(np.float64) @ W.astype(np.float64).T + b
    got = oracle.gather_gemm(bf16_bits(X), idx, bf16_bits(W), bf16_bits(b))
    np.testing.assert_array_equal(got, bf16_bits(want))
    got32 = oracle.gather_gemm(X, idx, W, b)
    np.testing.assert_array_equal(got32, want.astype(np.float32))
    # W (not W^T) would be a shape error here; a transposed square W must change the answer:
    Wsq = (rng.integers(-8, 9, (C, C)) / 8.0).astype(np.float32)
    assert not np.array_equal(oracle.gather_gemm(X, idx, Wsq), oracle.gather_gemm(X, idx, np.ascontiguousarray(Wsq.T)))


def test_gemm_random_within_one_ulp_and_identity_cases():
    rng = np.random.default_rng(6)
    S, C, N = 40, 96, 33
    X = bf16_bits(rng.standard_normal((S, C)))
    W = bf16_bits(rng.standard_normal((N, C)) * 0.02)
    idx = rng.permutation(S)[:25].astype(np.int32)
    want = widen(X)[idx].astype(np.float64) @ widen(W).astype(np.float64).T
    got = oracle.gather_gemm(X, idx, W)
    wb = bf16_bits(want)  # float64 -> float32 -> bf16: may differ from single rounding by one ulp at most
    assert np.max(np.abs(got.astype(np.int32) - wb.astype(np.int32))) <= 1
    assert np.mean(got == wb) > 0.999
    # identity indices == plain GEMM; identity weights == row gather, bit-exact
    np.testing.assert_array_equal(oracle.gather_gemm(X, None, W), oracle.gather_gemm(X, np.arange(S, dtype=np.int32), W))
    eye = bf16_bits(np.eye(C))
    np.testing.assert_array_equal(oracle.gather_gemm(X, idx, eye), X[idx])


# ------------------------------------------------------------------------------ fused gather-GEMM + in-place add

def test_gemm_add_exact_on_dyadic_grid():
    """Sec. 4.4 in one step: on a dyadic grid every sum is exact, so the fused call must equal the naive chain
    (gather rows, float64 matmul, zero-pad to the full sequence, add the residual), rounded once, bit for bit;
    rows outside out_idx must keep their bits."""
    rng = np.random.default_rng(15)
    S, C, N, M = 50, 64, 24, 31
    X = (rng.integers(-8, 9, (S, C)) / 4.0).astype(np.float32)
    W = (rng.integers(-8, 9, (N, C)) / 8.0).astype(np.float32)
    b = (rng.integers(-8, 9, N) / 2.0).astype(np.float32)
    R = (rng.integers(-64, 65, (S, N)) / 4.0).astype(np.float32)
    in_idx = rng.permutation(S)[:M].astype(np.int32)
    out_idx = rng.permutation(S)[:M].astype(np.int32)  # a different, unsorted set of rows
    padded = np.zeros((S, N))
    padded[out_idx] = X[in_idx].astype(np.float64) @ W.astype(np.float64).T + b
    want = R.astype(np.float64) + padded
    got = oracle.gather_gemm_add(bf16_bits(X), in_idx, bf16_bits(W), bf16_bits(R), out_idx, bf16_bits(b))
    np.testing.assert_array_equal(got, bf16_bits(want))
    untouched = np.setdiff1d(np.arange(S), out_idx)
    np.testing.assert_array_equal(got[untouched], bf16_bits(R)[untouched])
    got32 = oracle.gather_gemm_add(X, in_idx, W, R.copy(), out_idx, b)
    np.testing.assert_array_equal(got32, want.astype(np.float32))
    # swapping the roles of the two index lists must change the answer (each is used on its own side)
    assert not np.array_equal(oracle.gather_gemm_add(X, out_idx, W, R.copy(), in_idx, b), got32)


def test_gemm_add_single_rounding_and_special_cases():
    rng = np.random.default_rng(16)
    S, C, N, M = 40, 96, 33, 25
    X = bf16_bits(rng.standard_normal((S, C)))
    W = bf16_bits(rng.standard_normal((N, C)) * 0.1)
    R0 = bf16_bits(rng.standard_normal((S, N)))
    idx = np.sort(rng.permutation(S)[:M]).astype(np.int32)
    # against float64 numpy, rounded through float32 by torch: at most one step apart, almost always equal
    want = widen(R0).astype(np.float64)
    want[idx] += widen(X)[idx].astype(np.float64) @ widen(W).astype(np.float64).T
    got = oracle.gather_gemm_add(X, idx, W, R0.copy(), idx)
    wb = bf16_bits(want)
    assert np.max(np.abs(got.astype(np.int32) - wb.astype(np.int32))) <= 1
    assert np.mean(got == wb) > 0.999
    # ONE rounding: the two-step chain (GEMM rounded to bf16, then added and rounded again) differs somewhere
    two_step = R0.copy()
    oracle.scatter_add(oracle.gather_gemm(X, idx, W), idx, two_step)
    y = np.abs(widen(X)[idx].astype(np.float64) @ widen(W).astype(np.float64).T)
    slack = np.zeros((S, N))
    slack[idx] = 2.0 ** -8 * y  # the chain's extra rounding of Y: at most half a bf16 step of |Y| ...
    final = 2.0 ** -7 * np.maximum(np.abs(widen(got)), np.abs(widen(two_step)))  # ... plus half a step of each final result
    assert np.all(np.abs(widen(got).astype(np.float64) - widen(two_step)) <= slack + final)
    assert not np.array_equal(got, two_step)
    # zero weights leave R as it was; a zero residual and identity weights give the zero-padded rows (token padding)
    np.testing.assert_array_equal(oracle.gather_gemm_add(X, idx, np.zeros_like(W), R0.copy(), idx), R0)
    eye = bf16_bits(np.eye(C))
    pad = oracle.gather_gemm_add(X, idx, eye, np.zeros((S, C), dtype=np.uint16), idx)
    np.testing.assert_array_equal(pad[idx], X[idx])
    assert not pad[np.setdiff1d(np.arange(S), idx)].any()
    # no index lists at all == dense GEMM with a residual
    dense = oracle.gather_gemm_add(X, None, W, R0.copy(), None)
    np.testing.assert_array_equal(dense, oracle.gather_gemm_add(X, np.arange(S, dtype=np.int32), W, R0.copy(), np.arange(S, dtype=np.int32)))
    # duplicate or out-of-range output rows are refused
    with pytest.raises(ValueError):
        oracle.gather_gemm_add(X, idx, W, R0.copy(), np.full(M, 3, dtype=np.int32))
    bad = idx.copy(); bad[0] = S
    with pytest.raises(ValueError):
        oracle.gather_gemm_add(X, idx, W, R0.copy(), bad)


# ------------------------------------------------------------------------------ weight gradient of the selective-load GEMM

def test_gemm_dw_against_numpy_and_adjoint():
    """dW = dY^T X[idx]: exact against numpy float64 on a dyadic grid (bf16 and fp32); and the adjoint identity that
    ties it to the forward oracle: <dY, X[idx] W^T> == <dY^T X[idx], W> for any W."""
    rng = np.random.default_rng(51)
    S, C, N, M = 50, 24, 20, 31
    X = (rng.integers(-8, 9, (S, C)) / 4.0).astype(np.float32)
    dY = (rng.integers(-8, 9, (M, N)) / 8.0).astype(np.float32)
    idx = rng.permutation(S)[:M].astype(np.int32)
    want = dY.astype(np.float64).T @ X[idx].astype(np.float64)
    np.testing.assert_array_equal(oracle.gather_gemm_dw(bf16_bits(dY), bf16_bits(X), idx), bf16_bits(want))
    np.testing.assert_array_equal(oracle.gather_gemm_dw(dY, X, idx), want.astype(np.float32))
    np.testing.assert_array_equal(oracle.gather_gemm_dw(dY, X[:M], None), oracle.gather_gemm_dw(dY, X, np.arange(M, dtype=np.int32)))
    # a transposed result or a gather on the wrong operand changes the answer
    assert oracle.gather_gemm_dw(dY, X, idx).shape == (N, C)
    assert not np.array_equal(oracle.gather_gemm_dw(dY, X, idx), oracle.gather_gemm_dw(dY, X, np.sort(idx)))
    # adjoint identity with random (non-dyadic) data, fp32 oracle outputs, float64 inner products
    Xr = rng.standard_normal((S, C)).astype(np.float32)
    Wr = rng.standard_normal((N, C)).astype(np.float32)
    dYr = rng.standard_normal((M, N)).astype(np.float32)
    lhs = np.sum(dYr.astype(np.float64) * oracle.gather_gemm(Xr, idx, Wr))
    rhs = np.sum(oracle.gather_gemm_dw(dYr, Xr, idx).astype(np.float64) * Wr)
    assert lhs == pytest.approx(rhs, rel=1e-5)


# ------------------------------------------------------------------------------ attention over the kept tokens

def dense_attention(Q, K, V, idx, causal, scale=None):
    """Textbook attention on the gathered rows, float64 numpy: gather, logits, mask by token position, softmax, P @ V."""
    S, H, d = Q.shape
    Hkv = K.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    q, k, v = Q[idx].astype(np.float64), K[idx].astype(np.float64), V[idx].astype(np.float64)
    out = np.zeros((len(idx), H, d))
    allowed = (idx[None, :] <= idx[:, None]) if causal else np.ones((len(idx), len(idx)), dtype=bool)
    for h in range(H):
        g = h * Hkv // H
        z = np.where(allowed, scale * (q[:, h] @ k[:, g].T), -np.inf)
        e = np.exp(z - z.max(axis=1, keepdims=True))
        out[:, h] = (e / e.sum(axis=1, keepdims=True)) @ v[:, g]
    return out


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("S,H,Hkv,d,M,dtype", [(40, 2, 2, 8, 17, "f32"), (64, 4, 2, 16, 64, "bf16"), (50, 3, 1, 4, 1, "f32"),
                                                (33, 4, 4, 8, 20, "bf16")])
def test_kept_attention_against_dense_numpy_and_torch(S, H, Hkv, d, M, dtype, causal):
    rng = np.random.default_rng(S + M)
    Q = rng.standard_normal((S, H, d)).astype(np.float32)
    K = (rng.standard_normal((S, Hkv, d)) * 1.5).astype(np.float32)
    V = rng.standard_normal((S, Hkv, d)).astype(np.float32)
    idx = np.sort(rng.permutation(S)[:M]).astype(np.int32)
    if dtype == "bf16":
        Qin, Kin, Vin = bf16_bits(Q), bf16_bits(K), bf16_bits(V)
        Q, K, V = widen(Qin), widen(Kin), widen(Vin)
    else:
        Qin, Kin, Vin = Q, K, V
    want = dense_attention(Q, K, V, idx, causal)
    got = oracle.kept_attention(Qin, Kin, Vin, idx, flags=CAUSAL if causal else 0)
    if dtype == "bf16":
        wb = bf16_bits(want)  # through float32: at most one step from the single rounding
        assert np.max(np.abs(got.astype(np.int32) - wb.astype(np.int32))) <= 1 and np.mean(got == wb) > 0.99
        got = widen(got)
    else:
        np.testing.assert_allclose(got, want, rtol=1e-6, atol=1e-7)
    # the library routine on the same gathered rows (ascending positions make the position mask the usual triangle)
    rep = H // Hkv
    tq = torch.from_numpy(Q[idx]).double().permute(1, 0, 2)
    tk = torch.from_numpy(np.repeat(K[idx], rep, axis=1)).double().permute(1, 0, 2)
    tv = torch.from_numpy(np.repeat(V[idx], rep, axis=1)).double().permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, ref, rtol=2e-2 if dtype == "bf16" else 1e-6, atol=1e-2 if dtype == "bf16" else 1e-7)


def test_kept_attention_special_cases():
    rng = np.random.default_rng(41)
    S, H, Hkv, d, M = 60, 4, 2, 8, 25
    Q = rng.standard_normal((S, H, d)).astype(np.float32)
    K = rng.standard_normal((S, Hkv, d)).astype(np.float32)
    V = rng.standard_normal((S, Hkv, d)).astype(np.float32)
    idx = np.sort(rng.permutation(S)[:M]).astype(np.int32)
    # zero queries: every allowed key weighs the same, so the output is a mean of V rows (running mean under the mask)
    Z = np.zeros_like(Q)
    got = oracle.kept_attention(Z, K, V, idx, flags=CAUSAL)
    for h in range(H):
        want = np.cumsum(V[idx, h * Hkv // H].astype(np.float64), axis=0) / np.arange(1, M + 1)[:, None]
        np.testing.assert_allclose(got[:, h], want, rtol=1e-6, atol=1e-7)
    got = oracle.kept_attention(Z, K, V, idx, flags=0)
    np.testing.assert_allclose(got[3, 1], V[idx, 0].astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-7)
    # a list of queries computes just those rows of the full result
    full = oracle.kept_attention(Q, K, V, idx)
    np.testing.assert_array_equal(oracle.kept_attention(Q, K, V, idx, rows=[0, 7, M - 1]), full[[0, 7, M - 1]])
    # no index list == the first M tokens; all tokens kept == ordinary attention; first kept token attends to itself only
    np.testing.assert_array_equal(oracle.kept_attention(Q, K, V, None), oracle.kept_attention(Q, K, V, np.arange(S, dtype=np.int32)))
    first = oracle.kept_attention(Q, K, V, idx, flags=CAUSAL)[0]
    np.testing.assert_allclose(first, np.repeat(V[idx[0]], H // Hkv, axis=0), rtol=1e-6)
    # tokens that are not kept have no influence: changing them changes nothing
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    drop = np.setdiff1d(np.arange(S), idx)
    Q2[drop] += 3.0; K2[drop] -= 2.0; V2[drop] *= 5.0
    np.testing.assert_array_equal(oracle.kept_attention(Q2, K2, V2, idx), oracle.kept_attention(Q, K, V, idx))
    # one key far stronger than the rest takes all the weight of the queries that may see it
    Kd = K.copy(); Kd[idx[5]] = 0.0
    Qd = np.abs(Q)
    Kd[idx[5]] = 50.0
    got = oracle.kept_attention(Qd, Kd, V, idx, flags=CAUSAL)
    np.testing.assert_allclose(got[5:, 0], np.broadcast_to(V[idx[5], 0], (M - 5, d)), rtol=1e-5, atol=1e-6)
    # the scale argument; an explicit 1/sqrt(d) equals the default
    np.testing.assert_allclose(oracle.kept_attention(Q, K, V, idx, scale=1.0 / math.sqrt(d)), oracle.kept_attention(Q, K, V, idx), rtol=1e-6)
    assert not np.allclose(oracle.kept_attention(Q, K, V, idx, scale=1.0), oracle.kept_attention(Q, K, V, idx))


# ------------------------------------------------------------------------------ scatter-add

@pytest.mark.parametrize("gdt,xdt", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32"), ("f32", "bf16")])
def test_scatter_against_numpy(gdt, xdt):
    rng = np.random.default_rng(7)
    S, C, M = 60, 40, 23
    G = rng.standard_normal((M, C)).astype(np.float32)
    D = rng.standard_normal((S, C)).astype(np.float32)
    Gin = bf16_bits(G) if gdt == "bf16" else G
    Din = bf16_bits(D) if xdt == "bf16" else D.copy()
    idx = np.sort(rng.choice(S, M, replace=False)).astype(np.int32)
    before = Din.copy()
    got = oracle.scatter_add(Gin, idx, Din)
    g32 = widen(Gin) if gdt == "bf16" else Gin
    d32 = widen(before) if xdt == "bf16" else before
    want32 = d32.copy()
    want32[idx] = d32[idx] + g32  # numpy float32 add: one binary32 addition
    want = bf16_bits(want32) if xdt == "bf16" else want32
    np.testing.assert_array_equal(got, want)
    untouched = np.setdiff1d(np.arange(S), idx)
    np.testing.assert_array_equal(got[untouched], before[untouched])


def test_scatter_zero_pad_roundtrip_and_adjoint():
    rng = np.random.default_rng(9)
    S, C, M = 70, 16, 30
    G = bf16_bits(rng.standard_normal((M, C)))
    idx = np.sort(rng.choice(S, M, replace=False)).astype(np.int32)
    D = bf16_bits(rng.standard_normal((S, C)))  # garbage that ZERO_PAD must overwrite
    oracle.scatter_add(G, idx, D, mode=oracle.SCATTER_ZERO_PAD)
    np.testing.assert_array_equal(D[idx], G)                                   # gather(scatter(G)) == G
    assert not D[np.setdiff1d(np.arange(S), idx)].any()                        # padding rows are +0
    # adjoint: <scatter(G), X> == <G, gather(X)>, in float64 on exactly widened values
    X = rng.standard_normal((S, C))
    lhs = float((widen(D).astype(np.float64) * X).sum())
    rhs = float((widen(G).astype(np.float64) * X[idx]).sum())
    assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(lhs))


def test_scatter_rejects_duplicate_or_out_of_range_indices():
    G = np.zeros((2, 4), np.float32)
    D = np.zeros((5, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.scatter_add(G, np.array([1, 1], np.int32), D)
    with pytest.raises(ValueError):
        oracle.scatter_add(G, np.array([1, 5], np.int32), D)


# ------------------------------------------------------------------------------ randomised cross-checks (hypothesis)

from hypothesis import given, settings, strategies as st  # noqa: E402


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 300), st.integers(1, 64), st.data())
def test_select_topk_randomised_against_lexsort(S, L, data):
    """Any length, segment size, keep count and score multiset (many ties on purpose): the oracle's kept set equals the
    first k entries of a (score descending, index ascending) lexicographic sort, per segment, listed ascending."""
    k = data.draw(st.integers(1, L))
    vals = data.draw(st.lists(st.sampled_from([-1.5, -0.0, 0.0, 0.25, 0.25, 1.0, 3.0, 1e-30]), min_size=S, max_size=S))
    scores = np.array(vals, dtype=np.float32)
    got = oracle.select_topk(scores, L, k)
    want = []
    for s0 in range(0, S, L):
        seg = scores[s0:s0 + L]
        keep = k if len(seg) == L else max(1, min(len(seg), -(-k * len(seg) // L)))
        order = np.lexsort((np.arange(len(seg)), -(seg + np.float32(0.0))))  # +0.0 folds -0.0 into +0.0
        want.extend(sorted(s0 + order[:keep]))
    np.testing.assert_array_equal(got, np.array(want, dtype=np.int32))


@settings(max_examples=40, deadline=None)
@given(st.integers(1, 40), st.integers(1, 12), st.data())
def test_scatter_then_gather_round_trip_randomised(S, C, data):
    """ZERO_PAD scatter followed by a row gather returns the source rows bit for bit, every other row is +0."""
    M = data.draw(st.integers(0, S))
    rng = np.random.default_rng(data.draw(st.integers(0, 2 ** 31)))
    idx = np.sort(rng.permutation(S)[:M]).astype(np.int32)
    G = bf16_bits(rng.standard_normal((M, C)))
    D = bf16_bits(rng.standard_normal((S, C)))
    oracle.scatter_add(G, idx, D, mode=oracle.SCATTER_ZERO_PAD)
    np.testing.assert_array_equal(D[idx], G)
    assert not D[np.setdiff1d(np.arange(S), idx)].any()


@settings(max_examples=40, deadline=None)
@given(st.integers(1, 200), st.integers(1, 40), st.floats(-1.0, 2.0))
def test_threshold_selection_randomised(S, b, T):
    rng = np.random.default_rng(S * 41 + b)
    nb = -(-S // b)
    tb = rng.random(nb).astype(np.float32)
    want = np.nonzero(np.repeat(tb.astype(np.float64) >= T, b)[:S])[0]
    np.testing.assert_array_equal(oracle.select_threshold(tb, S, b, T), want)
