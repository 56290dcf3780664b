#!/usr/bin/env python3
"""Benchmark of the Contextual Token Sparsity hot path on one MI355X.

A step is one pass of the whole path over one synthetic layer, through the C ABI:
    lemo_score_rowstats -> lemo_score_colsums -> lemo_head_mean_select_topk (head mean + per-segment top-k, one launch)
    -> lemo_gather_gemm -> lemo_scatter_grad (when the configuration has a backward)
with every input already resident in HBM.  HIP events recorded between the calls, on the stream the
kernels run on, give each kernel's share of the timed region.  Prints ONE JSON line: the 32K-token layer as the
headline, the 16K-token layer (the other half of the metric) under "secondary", measured ceilings of the same
machine in the same run (a library GEMM of the consumer's shape, a 1 GiB device copy, an empty launch) under
"ceilings", and the CPU oracle on a bounded sample under "cpu_baseline".

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C5] [--secondary C4] [--no-cpu-baseline]
"""
import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published

# HBM-side bytes per launch (reads + writes behind L2) of each hot-path kernel on the 32K-token configuration, from two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE), each scaled by what the same counter reads for a 1 GiB device copy
# (2.000 and 1.000 KiB per counter unit); the runs and the raw figures are in profiles/C5_hotpath_kernels.md.
# The figures belong to the kernel sources they were measured on: "sources" is sources_digest() at that time, and the
# bench reports traffic as null when the sources have changed since.
MEASURED_TRAFFIC_BYTES = {
    "sources": "c7e7cdca3b2de7e5",
    "C5:rowstats": 2084561862, "C5:colsum": 2093587592, "C5:head_mean_select": 8641864,
    "C5:gather_gemm": 1687025269, "C5:scatter": 242876820,
}


HOT_PATH_SOURCES = ("lemo_common.hpp", "score.hip", "select.hip", "gather_gemm.hip", "scatter.hip")


def sources_digest() -> str:
    """sha256 over the sources of the timed step's kernels (what the measured traffic figures are tied to)."""
    h = hashlib.sha256()
    for name in HOT_PATH_SOURCES:
        path = os.path.join(ROOT, "paper_2501_09767_amd", "csrc", name)
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(key: str):
    if MEASURED_TRAFFIC_BYTES.get("sources") != sources_digest():
        return None
    return MEASURED_TRAFFIC_BYTES.get(key)


class HipEvents:
    """hipEvent_t handles created straight from the HIP runtime, recorded on a given stream."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        e = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(e))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        return e

    def record(self, e, stream):
        rc = self.hip.hipEventRecord(e, ctypes.c_void_p(stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def elapsed_ms(self, a, b) -> float:
        self.hip.hipEventSynchronize(b)
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)


def algorithmic_work(cfg):
    """Work the method must do per launch (not what an implementation happens to move)."""
    S, H, d, C, N, M = cfg.S, cfg.H, cfg.d, cfg.C, cfg.N, cfg.M
    esz = 2 if cfg.dtype == "bf16" else 4
    pairs = H * S * (S + 1) // 2          # causal: allowed (query, key) pairs over all heads
    return {
        "rowstats": {"flops": 2.0 * d * pairs},
        "colsum": {"flops": 2.0 * d * pairs},
        "head_mean": {"bytes": 2.0 * H * S * 4 + S * 4},
        "select": {"bytes": S * 4.0 + M * 4.0},
        "head_mean_select": {"bytes": 2.0 * H * S * 4 + S * 4 + M * 4.0},
        "gather_gemm": {"flops": 2.0 * M * C * N, "bytes": (M * C + N * C + M * N) * float(esz)},
        "scatter": {"bytes": 3.0 * M * C * esz + 4.0 * M},
    }


def cpu_baseline(cfg, lay, wl, steps_note=""):
    """The oracle, as it stands, timed on this host on a bounded sample of the same workload."""
    import numpy as np

    import oracle
    group = cfg.H // cfg.H_kv
    S1 = min(cfg.S, 16384)                                  # queries [0, S1): under the causal mask they only see keys < S1
    H1 = max(group, min(cfg.H, 16) // group * group)        # a few whole GQA groups
    Q = wl.as_numpy(lay["Q"][:S1, :H1].cpu())
    K = wl.as_numpy(lay["K"][:S1, :max(1, H1 // group)].cpu())
    t0 = time.perf_counter()
    sc = oracle.score(Q, K, flags=oracle.CAUSAL | oracle.EXCLUDE_SELF)
    t_score_s = time.perf_counter() - t0
    frac = (H1 * S1 * (S1 + 1)) / (cfg.H * cfg.S * (cfg.S + 1))
    t_score = t_score_s / frac
    scores_full = np.resize(sc, cfg.S).astype(np.float32)   # any scores do for timing the selection
    t0 = time.perf_counter()
    kept = oracle.select_topk(scores_full, cfg.L, cfg.k)
    t_select = time.perf_counter() - t0
    M1 = min(len(kept), 512)
    X = wl.as_numpy(lay["X"].cpu())
    W = wl.as_numpy(lay["W"].cpu())
    t0 = time.perf_counter()
    oracle.gather_gemm(X, kept[:M1], W)
    t_gemm_s = time.perf_counter() - t0
    t_gemm = t_gemm_s * (len(kept) / M1)
    t_scatter = 0.0
    if cfg.backward:
        G = wl.as_numpy(lay["G"].cpu())
        dX = np.zeros((cfg.S, cfg.C), dtype=G.dtype)
        t0 = time.perf_counter()
        oracle.scatter_add(G, kept, dX)
        t_scatter = time.perf_counter() - t0
    total = t_score + t_select + t_gemm + t_scatter
    return {
        "value": cfg.S / total, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": (f"score: queries [0,{S1}) x {H1} of {cfg.H} heads = {frac:.4f} of the causal pairs, {t_score_s:.2f} s, scaled by 1/fraction; "
                   f"select: all {cfg.S} tokens; gather-GEMM: {M1} of {len(kept)} kept rows, scaled; "
                   f"scatter: all {len(kept)} rows" + ("" if cfg.backward else " (not in this configuration)")),
        "est_seconds_per_step": total,
        "seconds": {"score": t_score, "select": t_select, "gather_gemm": t_gemm, "scatter": t_scatter},
        "measured_seconds_unscaled": {"score": t_score_s, "select": t_select, "gather_gemm": t_gemm_s, "scatter": t_scatter},
    }


def measure_fused_output_projection(cfg, lemo, ev, stream, kept, reps=10):
    """Outside the timed step: the attention block's output projection (C -> C) over the M kept rows, added into
    the [S, C] residual stream at the kept positions (Sec. 4.4's in-place add).  Fused = one lemo_gather_gemm_add;
    unfused = lemo_gather_gemm into a compact [M, C] buffer, then lemo_scatter_grad.  Timed alternately."""
    import torch
    S, C, M = cfg.S, cfg.C, cfg.M
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    g = torch.Generator(device="cuda").manual_seed(7)
    A = torch.randn((M, C), device="cuda", dtype=torch.float32, generator=g).to(dt)
    Wo = (torch.randn((C, C), device="cuda", dtype=torch.float32, generator=g) * 0.02).to(dt)
    R = torch.randn((S, C), device="cuda", dtype=torch.float32, generator=g).to(dt)
    Y = torch.empty((M, C), device="cuda", dtype=dt)

    def unfused():
        lemo.lemo_gather_gemm(A, None, Wo, Y=Y)
        lemo.lemo_scatter_grad(Y, kept, R)

    t_fused, t_unfused = timed_alternately(ev, stream, [lambda: lemo.lemo_gather_gemm_add(A, None, Wo, R, kept), unfused], reps)
    flops = 2.0 * M * C * C
    esz = 2 if cfg.dtype == "bf16" else 4
    return {"what": f"output projection {C}->{C} over M={M} kept rows added into the [{S},{C}] residual rows",
            "fused_ms": round(t_fused, 5), "fused_tflops": round(flops / t_fused * 1e-9, 2),
            "unfused_ms": round(t_unfused, 5), "bytes_saved": 2.0 * M * C * esz}


def measure_gather_fold(cfg, lemo, ev, stream, X, W, kept, Y, reps=10):
    """Outside the timed step: what folding the gather into the GEMM's A-tile load saves (Sec. 4.4, selective
    load).  Unfolded = materialise the kept rows (torch.index_select, one read and one
    write of M x C) and run the same GEMM kernel on the compact copy.  Timed alternately."""
    import torch
    kept64 = kept.long()
    Xc = torch.empty((cfg.M, cfg.C), dtype=X.dtype, device=X.device)

    def unfolded():
        torch.index_select(X, 0, kept64, out=Xc)
        lemo.lemo_gather_gemm(Xc, None, W, Y=Y)

    t_fold, t_unf = timed_alternately(ev, stream, [lambda: lemo.lemo_gather_gemm(X, kept, W, Y=Y), unfolded], reps)
    esz = 2 if cfg.dtype == "bf16" else 4
    return {"what": "consumer GEMM reading the kept rows in place vs torch.index_select into a compact copy + the same GEMM",
            "folded_ms": round(t_fold, 5), "unfolded_ms": round(t_unf, 5), "bytes_saved": 2.0 * cfg.M * cfg.C * esz}


def measure_gemm_backward(cfg, lemo, ev, stream, X, W, kept, reps=5):
    """Outside the timed step: both gradients of the consumer GEMM Y = X[kept] W^T at the layer's shape, neither with a
    transposed copy of anything: dX[kept] += dY W with W as stored, and dW = dY^T X[kept] with the kept rows read in place."""
    import torch
    M, C, N = cfg.M, cfg.C, cfg.N
    g = torch.Generator(device="cuda").manual_seed(13)
    dY = (torch.randn((M, N), device="cuda", dtype=torch.float32, generator=g) * 0.05).to(X.dtype)
    dX = torch.zeros_like(X)
    dW = torch.empty((N, C), dtype=X.dtype, device="cuda")
    dt = lemo.BF16 if cfg.dtype == "bf16" else lemo.F32
    need = lemo.lemo_gather_gemm_dw_workspace_bytes(M, C, N, dt)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
    if cfg.dtype == "bf16":
        t_dx = timed_calls(ev, stream, lambda: lemo.lemo_gather_gemm_dx(dY, W, dX, kept), reps)
    else:
        Wt = W.t().contiguous()
        t_dx = timed_calls(ev, stream, lambda: lemo.lemo_gather_gemm_add(dY, None, Wt, dX, kept), reps)
    t_dw = timed_calls(ev, stream, lambda: lemo.lemo_gather_gemm_dw(dY, X, kept, dW=dW, workspace=ws), reps)
    flops = 2.0 * M * C * N
    return {"what": f"gradients of the consumer GEMM, M={M} C={C} N={N}, operands read as stored", "dX_ms": round(t_dx, 5),
            "dX_tflops": round(flops / t_dx * 1e-9, 2), "dW_ms": round(t_dw, 5), "dW_tflops": round(flops / t_dw * 1e-9, 2),
            "dW_workspace_bytes": need}


def measure_kept_attention(cfg, lemo, ev, stream, Q, K, kept, reps=5):
    """Outside the timed step: causal attention over the M kept tokens of the layer, Q/K rows read in place through
    kept_idx (Sec. 4.4).  4*d flops per allowed (query, key) pair and head (both products)."""
    import torch
    M, H, d = cfg.M, cfg.H, cfg.d
    g = torch.Generator(device="cuda").manual_seed(11)
    V = torch.randn(tuple(K.shape), device="cuda", dtype=torch.float32, generator=g).to(K.dtype)
    O = torch.empty((M, H, d), dtype=Q.dtype, device="cuda")
    ws = torch.empty(lemo.lemo_kept_attention_workspace_bytes(M, cfg.H_kv, d), dtype=torch.uint8, device="cuda")
    fn = lambda: lemo.lemo_kept_attention(Q, K, V, kept, O=O, workspace=ws)
    fn()
    marks = [ev.create() for _ in range(reps + 1)]
    ev.record(marks[0], stream)
    for i in range(reps):
        fn()
        ev.record(marks[i + 1], stream)
    torch.cuda.synchronize()
    ms = sum(ev.elapsed_ms(marks[i], marks[i + 1]) for i in range(reps)) / reps
    flops = 4.0 * d * H * M * (M + 1) / 2
    return {"what": f"causal attention over the M={M} kept tokens, {H} heads, rows read in place", "ms": round(ms, 5),
            "tflops": round(flops / ms * 1e-9, 2)}


def measure_block_scoring(cfg, lemo, ev, stream, Q, K, lse2, flags, b=64, reps=5):
    """Outside the timed step: the paper's own criterion (Sec. 4.2 Eq. 2): block-wise informativeness with b x b score
    blocks from the row statistics sweep 1 already produced, then the initial threshold of Alg. 1 and the threshold
    selection.  Same flop count as one sweep of the token-wise score (every allowed pair, every head, once)."""
    import torch
    S, H = cfg.S, cfg.H
    nb = (S + b - 1) // b
    tb = torch.empty(nb, dtype=torch.float32, device="cuda")
    ws = torch.empty(lemo.lemo_score_blocks_workspace_bytes(S, H), dtype=torch.uint8, device="cuda")
    T0 = torch.empty(1, dtype=torch.float32, device="cuda")
    kept = torch.empty(S, dtype=torch.int32, device="cuda")
    count = torch.empty(1, dtype=torch.int32, device="cuda")

    def run(marks=None):
        if marks: ev.record(marks[0], stream)
        lemo.lemo_score_blocks(Q, K, b, flags=flags, lse2=lse2, want_score_blocks=False, token_blocks=tb, workspace=ws)
        if marks: ev.record(marks[1], stream)
        lemo.lemo_threshold_init(tb, T0)
        lemo.lemo_select_threshold(tb, S, b, T0, kept_idx=kept, kept_count=count)
        if marks: ev.record(marks[2], stream)

    run()
    marks = [[ev.create() for _ in range(3)] for _ in range(reps)]
    for i in range(reps):
        run(marks[i])
    torch.cuda.synchronize()
    t_blocks = sum(ev.elapsed_ms(m[0], m[1]) for m in marks) / reps
    t_sel = sum(ev.elapsed_ms(m[1], m[2]) for m in marks) / reps
    flops = 2.0 * cfg.d * H * S * (S + 1) / 2
    return {"what": f"block-wise informativeness, {b}x{b} score blocks, all {H} heads, then mean threshold + threshold selection",
            "score_blocks_ms": round(t_blocks, 5), "score_blocks_tflops": round(flops / t_blocks * 1e-9, 2),
            "threshold_select_ms": round(t_sel, 5), "kept_tokens": int(count.item())}


def timed_calls(ev, stream, fn, reps):
    """Mean milliseconds of `fn` over `reps` back-to-back calls, from HIP events on the launch stream (one warm-up call)."""
    import torch
    fn()
    marks = [ev.create() for _ in range(reps + 1)]
    ev.record(marks[0], stream)
    for i in range(reps):
        fn()
        ev.record(marks[i + 1], stream)
    torch.cuda.synchronize()
    return sum(ev.elapsed_ms(marks[i], marks[i + 1]) for i in range(reps)) / reps


def timed_alternately(ev, stream, fns, reps):
    """Mean milliseconds of each of `fns`, called in turn (a, b, a, b, ...) so that all of them see the same clocks and
    temperatures; one warm-up round."""
    import torch
    for fn in fns:
        fn()
    marks = [[ev.create() for _ in range(len(fns) + 1)] for _ in range(reps)]
    for r in range(reps):
        ev.record(marks[r][0], stream)
        for i, fn in enumerate(fns):
            fn()
            ev.record(marks[r][i + 1], stream)
    torch.cuda.synchronize()
    return [sum(ev.elapsed_ms(marks[r][i], marks[r][i + 1]) for r in range(reps)) / reps for i in range(len(fns))]


class LayerRun:
    """One synthetic layer resident in HBM and the step that runs the hot path over it."""

    def __init__(self, cfg, lemo, wl, ev, stream):
        import torch
        self.cfg, self.lemo, self.ev, self.stream = cfg, lemo, ev, stream
        self.flags = lemo.CAUSAL | lemo.EXCLUDE_SELF
        print(f"[bench] building synthetic layer {cfg.name}: S={cfg.S} H={cfg.H}/{cfg.H_kv} d={cfg.d} C={cfg.C} N={cfg.N} "
              f"L={cfg.L} k={cfg.k} M={cfg.M} {cfg.dtype}", file=sys.stderr, flush=True)
        self.lay = lay = wl.make_layer(cfg, device="cuda")
        self.Q, self.K, self.X, self.W = lay["Q"], lay["K"], lay["X"], lay["W"]
        dev, S, H = self.Q.device, cfg.S, cfg.H
        self.lse2 = torch.empty((H, S), dtype=torch.float32, device=dev)
        self.col = torch.empty((H, S), dtype=torch.float32, device=dev)
        self.dg = torch.empty((H, S), dtype=torch.float32, device=dev)
        self.scores = torch.empty(S, dtype=torch.float32, device=dev)
        self.kept = torch.empty(cfg.M, dtype=torch.int32, device=dev)
        self.Y = torch.empty((cfg.M, cfg.N), dtype=self.X.dtype, device=dev)
        self.phases = ["rowstats", "colsum", "head_mean_select", "gather_gemm"] + (["scatter"] if cfg.backward else [])
        # the HBM-bound scatter rotates between two sets of buffers (G, dX), so that no step finds the rows of the step
        # before in a cache: its rate is an HBM rate by construction
        self.sets = []
        if cfg.backward:
            G = lay["G"]
            self.sets = [(G, torch.zeros((S, cfg.C), dtype=self.X.dtype, device=dev)),
                         (G.clone(), torch.zeros((S, cfg.C), dtype=self.X.dtype, device=dev))]
        self.n = 0

    def step(self, m=None):
        lemo, cfg, ev, st = self.lemo, self.cfg, self.ev, self.stream
        if m: ev.record(m[0], st)
        lemo.lemo_score_rowstats(self.Q, self.K, flags=self.flags, lse2=self.lse2)
        if m: ev.record(m[1], st)
        lemo.lemo_score_colsums(self.Q, self.K, cfg.L, self.lse2, flags=self.flags, colsum_per_head=self.col, diag_per_head=self.dg)
        if m: ev.record(m[2], st)
        lemo.lemo_head_mean_select_topk(self.col, self.dg, cfg.L, cfg.k, flags=self.flags, scores=self.scores, kept_idx=self.kept)
        if m: ev.record(m[3], st)
        lemo.lemo_gather_gemm(self.X, self.kept, self.W, Y=self.Y)
        if m: ev.record(m[4], st)
        if self.sets:
            G, dX = self.sets[self.n & 1]
            self.n += 1
            lemo.lemo_scatter_grad(G, self.kept, dX)
            if m: ev.record(m[5], st)

    def run(self, steps, warmup):
        """W untimed steps, then exactly K timed steps between two synchronisations -> (ms per step, per-phase report)."""
        import torch
        ev = self.ev
        marks = [[ev.create() for _ in range(len(self.phases) + 1)] for _ in range(steps)]
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(marks[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / steps
        work = algorithmic_work(self.cfg)
        peak_tflops = PEAK_BF16_TFLOPS if self.cfg.dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS
        report = {}
        for pi, name in enumerate(self.phases):
            ts = sorted(ev.elapsed_ms(marks[i][pi], marks[i][pi + 1]) for i in range(steps))
            ms = sum(ts) / len(ts)
            w = work[name]
            r = {"ms": round(ms, 5), "ms_median": round(ts[len(ts) // 2], 5), "ms_min": round(ts[0], 5)}
            if "flops" in w:
                r["tflops"] = round(w["flops"] / (ms * 1e-3) * 1e-12, 2)
                r["frac_mfma_peak"] = round(r["tflops"] / peak_tflops, 4)
            if "bytes" in w:
                r["gbs"] = round(w["bytes"] / (ms * 1e-3) * 1e-9, 2)
                r["frac_hbm_peak"] = round(r["gbs"] / PEAK_HBM_GBS, 5)
            report[name] = r
        return ms_per_step, report

    def workload(self):
        cfg = self.cfg
        return (f"{cfg.name}: one Llama-shaped layer, S={cfg.S}, {cfg.H}x{cfg.d} heads ({cfg.H_kv} KV), hidden {cfg.C}, "
                f"consumer GEMM {cfg.C}->{cfg.N}, segment {cfg.L}, keep ratio {cfg.ratio} (k={cfg.k}, M={cfg.M}), causal, "
                f"self term excluded" + (", backward scatter-add included" if cfg.backward else ""))


def measure_ceilings(cfg, ev, stream, X, W, kept, lemo):
    """What this machine delivers, in this run, on the plainest form of each bound: the library GEMM (torch.matmul) on
    a pre-compacted copy of the consumer's operands, a 1 GiB device-to-device copy, and an empty kernel launch."""
    import torch
    Xc = X[kept.long()].contiguous()
    Wt = W.t()
    out = torch.empty((cfg.M, cfg.N), dtype=X.dtype, device=X.device)
    t_mm = timed_calls(ev, stream, lambda: torch.matmul(Xc, Wt, out=out), 10)
    del Xc, out
    a = torch.ones(1 << 29, dtype=torch.bfloat16, device=X.device)  # 1 GiB read + 1 GiB written per copy
    b = torch.empty_like(a)
    t_cp = timed_calls(ev, stream, lambda: b.copy_(a), 10)
    del a, b
    t_empty = timed_calls(ev, stream, lemo.lemo_launch_floor, 200)
    sink = torch.zeros(1, dtype=torch.float32, device=X.device)
    tiles, waves = 40000, [0]

    def mix():
        waves[0] = lemo.lemo_probe_sweep_issue_mix(tiles, sink)

    def mix_random():
        waves[0] = lemo.lemo_probe_sweep_issue_mix(tiles, sink, operand_seed=20250109)

    t_mix = timed_calls(ev, stream, mix, 3)
    mix_tflops = 8 * 32768.0 * tiles * waves[0] / t_mix * 1e-9
    t_mixr = timed_calls(ev, stream, mix_random, 3)
    mixr_tflops = 8 * 32768.0 * tiles * waves[0] / t_mixr * 1e-9
    return {"what": "same machine, same run: torch.matmul (library GEMM) on a compact copy of the consumer GEMM's operands; "
                    "1 GiB device copy (read + write counted); one empty kernel launch, back to back on the stream; "
                    "sweep_issue_mix = the sweeps' minimal instruction mix per 32x32 logit tile (8 dependent MFMAs + 16 x (fma, exp2, add), "
                    "two waves per SIMD) from registers only, quoted as the MFMA flops of the tiles, once with the same operand fragments for every MFMA "
                    "and once with pseudo-random operands that change from MFMA to MFMA (what the clock is when the matrix cores' inputs switch)",
            "library_gemm_ms": round(t_mm, 5), "library_gemm_tflops": round(2.0 * cfg.M * cfg.C * cfg.N / t_mm * 1e-9, 2),
            "device_copy_gbs": round(2.0 * (1 << 30) / t_cp * 1e-6, 1), "empty_launch_us": round(t_empty * 1e3, 3),
            "sweep_issue_mix_tflops": round(mix_tflops, 1), "sweep_issue_mix_random_operands_tflops": round(mixr_tflops, 1)}


def measure_constant_operands(cfg, lemo, ev, stream, run):
    """The step's three MFMA kernels on operands of all ones, same shapes, same launches, timed in runs of six calls
    beside the same on the step's own data.  The instruction streams are the same; what differs is how much of the chip's datapath switches, and
    with it the clock the power management grants.  The gap between the two is what the kernels lose to that, not to
    their schedule."""
    import torch
    Q1, K1 = torch.ones_like(run.Q), torch.ones_like(run.K)
    X1, W1 = torch.ones_like(run.X), torch.ones_like(run.W)
    lse2 = torch.empty_like(run.lse2)
    col, dg = torch.empty_like(run.col), torch.empty_like(run.dg)
    lemo.lemo_score_rowstats(Q1, K1, flags=run.flags, lse2=lse2)
    flops_sweep = float(cfg.d) * cfg.H * cfg.S * (cfg.S + 1)
    flops_gemm = 2.0 * cfg.M * cfg.C * cfg.N
    res = {"what": "the step's MFMA kernels on all-ones operands of the same shapes, six calls in a row, beside six on the step's data: "
                   "same instruction streams, less switching, higher granted clock"}
    pairs = {
        "rowstats": (lambda: lemo.lemo_score_rowstats(run.Q, run.K, flags=run.flags, lse2=run.lse2),
                     lambda: lemo.lemo_score_rowstats(Q1, K1, flags=run.flags, lse2=lse2), flops_sweep),
        "colsum": (lambda: lemo.lemo_score_colsums(run.Q, run.K, cfg.L, run.lse2, flags=run.flags, colsum_per_head=run.col, diag_per_head=run.dg),
                   lambda: lemo.lemo_score_colsums(Q1, K1, cfg.L, lse2, flags=run.flags, colsum_per_head=col, diag_per_head=dg), flops_sweep),
        "gather_gemm": (lambda: lemo.lemo_gather_gemm(run.X, run.kept, run.W, Y=run.Y),
                        lambda: lemo.lemo_gather_gemm(X1, run.kept, W1, Y=run.Y), flops_gemm),
    }
    for name, (real, const, flops) in pairs.items():
        t_real, t_const = timed_calls(ev, stream, real, 6), timed_calls(ev, stream, const, 6)
        res[name] = {"step_data_ms": round(t_real, 5), "ones_ms": round(t_const, 5),
                     "ones_tflops": round(flops / t_const * 1e-9, 2), "ones_frac_mfma_peak": round(flops / t_const * 1e-9 / PEAK_BF16_TFLOPS, 4)}
    lemo.lemo_gather_gemm(run.X, run.kept, run.W, Y=run.Y)  # leave the step's own output behind
    return res


def measure_select(cfg, lemo, ev, stream, col, dg, flags, batch=128):
    """Outside the timed step: head mean + selection as two launches and as one, against the empty-launch floor, and the
    same kernels on `batch` independent score sets in one launch (segments are independent, so a batch is simply a
    sequence `batch` times as long): the rate the kernels reach once the launch is amortised."""
    import torch
    S, H, L, k, M = cfg.S, cfg.H, cfg.L, cfg.k, cfg.M
    scores = torch.empty(S, dtype=torch.float32, device=col.device)
    kept = torch.empty(M, dtype=torch.int32, device=col.device)

    def two():
        lemo.lemo_score_head_mean(col, dg, flags=flags, scores=scores)
        lemo.lemo_select_topk(scores, L, k, kept_idx=kept)

    t_two = timed_calls(ev, stream, two, 50)
    t_one = timed_calls(ev, stream, lambda: lemo.lemo_head_mean_select_topk(col, dg, L, k, flags=flags, scores=scores, kept_idx=kept), 50)
    t_sel = timed_calls(ev, stream, lambda: lemo.lemo_select_topk(scores, L, k, kept_idx=kept), 50)
    Sb = S * batch
    g = torch.Generator(device="cuda").manual_seed(5)
    colb = torch.rand((H, Sb), device="cuda", dtype=torch.float32, generator=g)
    dgb = torch.rand((H, Sb), device="cuda", dtype=torch.float32, generator=g) * 0.1
    scb = torch.empty(Sb, dtype=torch.float32, device="cuda")
    kb = torch.empty(M * batch, dtype=torch.int32, device="cuda")
    t_oneb = timed_calls(ev, stream, lambda: lemo.lemo_head_mean_select_topk(colb, dgb, L, k, flags=flags, scores=scb, kept_idx=kb), 5)
    t_selb = timed_calls(ev, stream, lambda: lemo.lemo_select_topk(scb, L, k, kept_idx=kb), 5)
    del colb, dgb
    bytes_one = 2.0 * H * S * 4 + S * 4 + M * 4
    bytes_sel = S * 4.0 + M * 4.0
    return {"what": f"head mean + per-segment top-k at S={S}, {H} heads: two launches vs one; then {batch} independent score sets per launch",
            "two_launches_us": round(t_two * 1e3, 3), "one_launch_us": round(t_one * 1e3, 3), "select_alone_us": round(t_sel * 1e3, 3),
            "batched": {"sets": batch, "fused_ms": round(t_oneb, 5), "fused_gbs": round(bytes_one * batch / t_oneb * 1e-6, 1),
                        "fused_frac_hbm_peak": round(bytes_one * batch / t_oneb * 1e-6 / PEAK_HBM_GBS, 4),
                        "select_ms": round(t_selb, 5), "select_gbs": round(bytes_sel * batch / t_selb * 1e-6, 1),
                        "select_frac_hbm_peak": round(bytes_sel * batch / t_selb * 1e-6 / PEAK_HBM_GBS, 4)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C5", help="C1..C5 (default C5: S=32768 Llama2-7B-shaped layer with backward scatter)")
    ap.add_argument("--secondary", default="C4", help="a second configuration timed the same way after the first and reported "
                                                      "under 'secondary' (default C4: the S=16384 half of the metric); 'none' to skip")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (torch copy_) so that a counter profile of this command "
                         "contains a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--step-only", action="store_true",
                    help="time the step of --config and nothing else (no secondary configuration, no ceilings, none of the "
                         "measurements outside the timed step), so that a profile of this command holds the step's kernels only")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU (the path has no cross-GPU step: heads, segments and sequences shard without communication beyond one small all-reduce); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2501_09767_amd import lemo, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    ev = HipEvents()
    stream = torch.cuda.current_stream().cuda_stream
    cfg = wl.CONFIGS[args.config]
    run = LayerRun(cfg, lemo, wl, ev, stream)

    if args.copy_calibration:
        a = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda")  # 1 GiB read + 1 GiB written per copy
        b = torch.empty_like(a)
        for _ in range(2):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    ms_per_step, report = run.run(args.steps, args.warmup)

    work = algorithmic_work(cfg)
    peak_tflops = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS
    dominant = max(run.phases, key=lambda n: report[n]["ms"])
    traffic = measured_traffic(f"{cfg.name}:{dominant}")  # null when unprofiled, or profiled on other kernel sources
    if "flops" in work[dominant]:
        roof = {"bound": "mfma", "kernel": dominant, "achieved": report[dominant]["tflops"], "peak": peak_tflops,
                "unit": "TFLOP/s", "frac": round(report[dominant]["tflops"] / peak_tflops, 4), "traffic": traffic}
    else:
        roof = {"bound": "hbm", "kernel": dominant, "achieved": report[dominant]["gbs"], "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "frac": round(report[dominant]["gbs"] / PEAK_HBM_GBS, 4), "traffic": traffic}
    roof["traffic_measured_on_sources"] = MEASURED_TRAFFIC_BYTES["sources"]
    roof["sources"] = sources_digest()

    out = {
        "metric": "tokens scored+selected+gathered/sec per layer",
        "value": round(cfg.S / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": run.workload(),
                   "S": cfg.S, "H": cfg.H, "H_kv": cfg.H_kv, "d": cfg.d, "C": cfg.C, "N": cfg.N, "L": cfg.L, "k": cfg.k, "M": cfg.M},
        "roofline": roof,
        "phases": report,
    }
    if not args.step_only:
        Q, K, X, W, kept, flags = run.Q, run.K, run.X, run.W, run.kept, run.flags
        out["ceilings"] = measure_ceilings(cfg, ev, stream, X, W, kept, lemo)
        ceil = out["ceilings"]
        for name in ("rowstats", "colsum", "gather_gemm"):
            if "tflops" in report.get(name, {}):
                report[name]["frac_library_gemm"] = round(report[name]["tflops"] / ceil["library_gemm_tflops"], 4)
        for name in ("rowstats", "colsum"):
            if "tflops" in report.get(name, {}):
                report[name]["frac_sweep_issue_mix"] = round(report[name]["tflops"] / ceil["sweep_issue_mix_tflops"], 4)
                report[name]["frac_sweep_issue_mix_random_operands"] = round(report[name]["tflops"] / ceil["sweep_issue_mix_random_operands_tflops"], 4)
        if "scatter" in report:
            report["scatter"]["frac_device_copy"] = round(report["scatter"]["gbs"] / ceil["device_copy_gbs"], 4)
        out["constant_operands"] = measure_constant_operands(cfg, lemo, ev, stream, run)
        out["select"] = measure_select(cfg, lemo, ev, stream, run.col, run.dg, flags)
        out["gather_fold"] = measure_gather_fold(cfg, lemo, ev, stream, X, W, kept, run.Y)
        out["fused_in_place_add"] = measure_fused_output_projection(cfg, lemo, ev, stream, kept)
        out["gemm_backward"] = measure_gemm_backward(cfg, lemo, ev, stream, X, W, kept)
        if cfg.dtype == "bf16":
            out["kept_attention"] = measure_kept_attention(cfg, lemo, ev, stream, Q, K, kept)
        out["block_wise"] = measure_block_scoring(cfg, lemo, ev, stream, Q, K, run.lse2, flags)
    if not args.no_cpu_baseline and not args.step_only:
        print("[bench] timing the CPU oracle on a bounded sample", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(cfg, run.lay, wl)
    if not args.step_only and args.secondary.lower() != "none" and args.secondary != args.config:
        del run
        torch.cuda.empty_cache()
        cfg2 = wl.CONFIGS[args.secondary]
        run2 = LayerRun(cfg2, lemo, wl, ev, stream)
        ms2, rep2 = run2.run(args.steps, args.warmup)
        out["secondary"] = {"workload": run2.workload(), "value": round(cfg2.S / (ms2 * 1e-3), 1), "unit": "tokens/s",
                            "ms_per_step": round(ms2, 4), "steps": args.steps, "warmup": args.warmup, "dtype": cfg2.dtype, "phases": rep2}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
