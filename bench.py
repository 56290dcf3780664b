#!/usr/bin/env python3
"""Benchmark of the Contextual Token Sparsity hot path on one MI355X.

A step is one pass of the whole path over one synthetic layer, through the C ABI:
    lemo_score_rowstats -> lemo_score_colsums -> lemo_score_head_mean   (= lemo_score_segments)
    -> lemo_select_topk -> lemo_gather_gemm -> lemo_scatter_grad (when the configuration has a backward)
with every input already resident in HBM.  HIP events recorded between the calls, on the stream the
kernels run on, give each kernel's share of the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C5] [--no-cpu-baseline]
"""
import argparse
import ctypes
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
MEASURED_TRAFFIC_BYTES = {
    "C5:rowstats": 2129783382, "C5:colsum": 2228509924, "C5:head_mean": 8542739, "C5:select": 229023,
    "C5:gather_gemm": 1732136254, "C5:scatter": 242876184,
}


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
    t_gemm = (time.perf_counter() - t0) * (len(kept) / M1)
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
    }


def measure_fused_output_projection(cfg, lemo, ev, stream, kept, reps=10):
    """Outside the timed step: the attention block's output projection (C -> C) over the M kept rows, added into
    the [S, C] residual stream at the kept positions (Sec. 4.4's in-place add).  Fused = one lemo_gather_gemm_add;
    unfused = lemo_gather_gemm into a compact [M, C] buffer, then lemo_scatter_grad."""
    import torch
    S, C, M = cfg.S, cfg.C, cfg.M
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    g = torch.Generator(device="cuda").manual_seed(7)
    A = torch.randn((M, C), device="cuda", dtype=torch.float32, generator=g).to(dt)
    Wo = (torch.randn((C, C), device="cuda", dtype=torch.float32, generator=g) * 0.02).to(dt)
    R = torch.randn((S, C), device="cuda", dtype=torch.float32, generator=g).to(dt)
    Y = torch.empty((M, C), device="cuda", dtype=dt)

    def timed(fn):
        fn()
        marks = [ev.create() for _ in range(reps + 1)]
        ev.record(marks[0], stream)
        for i in range(reps):
            fn()
            ev.record(marks[i + 1], stream)
        torch.cuda.synchronize()
        return sum(ev.elapsed_ms(marks[i], marks[i + 1]) for i in range(reps)) / reps

    def unfused():
        lemo.lemo_gather_gemm(A, None, Wo, Y=Y)
        lemo.lemo_scatter_grad(Y, kept, R)

    t_fused = timed(lambda: lemo.lemo_gather_gemm_add(A, None, Wo, R, kept))
    t_unfused = timed(unfused)
    flops = 2.0 * M * C * C
    esz = 2 if cfg.dtype == "bf16" else 4
    return {"what": f"output projection {C}->{C} over M={M} kept rows added into the [{S},{C}] residual rows",
            "fused_ms": round(t_fused, 5), "fused_tflops": round(flops / t_fused * 1e-9, 2),
            "unfused_ms": round(t_unfused, 5), "bytes_saved": 2.0 * M * C * esz}


def measure_gather_fold(cfg, lemo, ev, stream, X, W, kept, Y, reps=10):
    """Outside the timed step: what folding the gather into the GEMM's A-tile load saves (Sec. 4.4, "directly loads the
    selected tokens from original inputs").  Unfolded = materialise the kept rows (torch.index_select, one read and one
    write of M x C) and run the same GEMM kernel on the compact copy."""
    import torch
    kept64 = kept.long()
    Xc = torch.empty((cfg.M, cfg.C), dtype=X.dtype, device=X.device)

    def timed(fn):
        fn()
        marks = [ev.create() for _ in range(reps + 1)]
        ev.record(marks[0], stream)
        for i in range(reps):
            fn()
            ev.record(marks[i + 1], stream)
        torch.cuda.synchronize()
        return sum(ev.elapsed_ms(marks[i], marks[i + 1]) for i in range(reps)) / reps

    def unfolded():
        torch.index_select(X, 0, kept64, out=Xc)
        lemo.lemo_gather_gemm(Xc, None, W, Y=Y)

    t_fold = timed(lambda: lemo.lemo_gather_gemm(X, kept, W, Y=Y))
    t_unf = timed(unfolded)
    esz = 2 if cfg.dtype == "bf16" else 4
    return {"what": "consumer GEMM reading the kept rows in place vs torch.index_select into a compact copy + the same GEMM",
            "folded_ms": round(t_fold, 5), "unfolded_ms": round(t_unf, 5), "bytes_saved": 2.0 * cfg.M * cfg.C * esz}


def measure_gemm_backward(cfg, lemo, ev, stream, X, W, kept, reps=5):
    """Outside the timed step: both gradients of the consumer GEMM Y = X[kept] W^T at the layer's shape.
    dX[kept] += dY W  (the in-place-add GEMM with W^T kept as a [C,N] matrix) and dW = dY^T X[kept]."""
    import torch
    M, C, N = cfg.M, cfg.C, cfg.N
    g = torch.Generator(device="cuda").manual_seed(13)
    dY = (torch.randn((M, N), device="cuda", dtype=torch.float32, generator=g) * 0.05).to(X.dtype)
    Wt = W.t().contiguous()
    dX = torch.zeros_like(X)
    dW = torch.empty((N, C), dtype=X.dtype, device="cuda")
    ws = torch.empty(lemo.lemo_gather_gemm_dw_workspace_bytes(M, C, N, lemo.BF16 if cfg.dtype == "bf16" else lemo.F32), dtype=torch.uint8, device="cuda")

    def timed(fn):
        fn()
        marks = [ev.create() for _ in range(reps + 1)]
        ev.record(marks[0], stream)
        for i in range(reps):
            fn()
            ev.record(marks[i + 1], stream)
        torch.cuda.synchronize()
        return sum(ev.elapsed_ms(marks[i], marks[i + 1]) for i in range(reps)) / reps

    t_dx = timed(lambda: lemo.lemo_gather_gemm_add(dY, None, Wt, dX, kept))
    t_dw = timed(lambda: lemo.lemo_gather_gemm_dw(dY, X, kept, dW=dW, workspace=ws))
    flops = 2.0 * M * C * N
    return {"what": f"gradients of the consumer GEMM, M={M} C={C} N={N}", "dX_ms": round(t_dx, 5), "dX_tflops": round(flops / t_dx * 1e-9, 2),
            "dW_ms": round(t_dw, 5), "dW_tflops": round(flops / t_dw * 1e-9, 2)}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C5", help="C1..C5 (default C5: S=32768 Llama2-7B-shaped layer with backward scatter)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (torch copy_) so that a counter profile of this command "
                         "contains a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--step-only", action="store_true",
                    help="skip the measurements outside the timed step (gather_fold, fused_in_place_add, gemm_backward, "
                         "kept_attention, block_wise), so that a profile of this command holds the step's kernels only")
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
    cfg = wl.CONFIGS[args.config]
    flags = lemo.CAUSAL | lemo.EXCLUDE_SELF
    print(f"[bench] building synthetic layer {cfg.name}: S={cfg.S} H={cfg.H}/{cfg.H_kv} d={cfg.d} C={cfg.C} N={cfg.N} "
          f"L={cfg.L} k={cfg.k} M={cfg.M} {cfg.dtype}", file=sys.stderr, flush=True)
    lay = wl.make_layer(cfg, device="cuda")
    Q, K, X, W, G = lay["Q"], lay["K"], lay["X"], lay["W"], lay.get("G")
    dev = Q.device
    S, H = cfg.S, cfg.H
    lse2 = torch.empty((H, S), dtype=torch.float32, device=dev)
    col = torch.empty((H, S), dtype=torch.float32, device=dev)
    dg = torch.empty((H, S), dtype=torch.float32, device=dev)
    scores = torch.empty(S, dtype=torch.float32, device=dev)
    kept = torch.empty(cfg.M, dtype=torch.int32, device=dev)
    Y = torch.empty((cfg.M, cfg.N), dtype=X.dtype, device=dev)
    dX = torch.zeros((S, cfg.C), dtype=X.dtype, device=dev)
    do_scatter = cfg.backward

    phases = ["rowstats", "colsum", "head_mean", "select", "gather_gemm"] + (["scatter"] if do_scatter else [])
    ev = HipEvents()
    stream = torch.cuda.current_stream().cuda_stream
    marks = [[ev.create() for _ in range(len(phases) + 1)] for _ in range(args.steps)]

    def step(m=None):
        if m: ev.record(m[0], stream)
        lemo.lemo_score_rowstats(Q, K, flags=flags, lse2=lse2)
        if m: ev.record(m[1], stream)
        lemo.lemo_score_colsums(Q, K, cfg.L, lse2, flags=flags, colsum_per_head=col, diag_per_head=dg)
        if m: ev.record(m[2], stream)
        lemo.lemo_score_head_mean(col, dg, flags=flags, scores=scores)
        if m: ev.record(m[3], stream)
        lemo.lemo_select_topk(scores, cfg.L, cfg.k, kept_idx=kept)
        if m: ev.record(m[4], stream)
        lemo.lemo_gather_gemm(X, kept, W, Y=Y)
        if m: ev.record(m[5], stream)
        if do_scatter:
            lemo.lemo_scatter_grad(G, kept, dX)
            ev.record(m[6], stream) if m else None

    if args.copy_calibration:
        a = torch.ones(1 << 29, dtype=torch.bfloat16, device=dev)  # 1 GiB read + 1 GiB written per copy
        b = torch.empty_like(a)
        for _ in range(2):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(marks[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    work = algorithmic_work(cfg)
    phase_ms, phase_min, phase_med = {}, {}, {}
    for pi, name in enumerate(phases):
        ts = sorted(ev.elapsed_ms(marks[i][pi], marks[i][pi + 1]) for i in range(args.steps))
        phase_ms[name] = sum(ts) / len(ts)
        phase_min[name], phase_med[name] = ts[0], ts[len(ts) // 2]
    peak_tflops = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS
    report = {}
    for name in phases:
        ms = phase_ms[name]
        w = work[name]
        r = {"ms": round(ms, 5), "ms_median": round(phase_med[name], 5), "ms_min": round(phase_min[name], 5)}
        if "flops" in w:
            r["tflops"] = round(w["flops"] / (ms * 1e-3) * 1e-12, 2)
            r["frac_mfma_peak"] = round(r["tflops"] / peak_tflops, 4)
        if "bytes" in w:
            r["gbs"] = round(w["bytes"] / (ms * 1e-3) * 1e-9, 2)
            r["frac_hbm_peak"] = round(r["gbs"] / PEAK_HBM_GBS, 5)
        report[name] = r

    dominant = max(phases, key=lambda n: phase_ms[n])
    traffic = MEASURED_TRAFFIC_BYTES.get(f"{cfg.name}:{dominant}")  # null for configurations that were not profiled
    if "flops" in work[dominant]:
        roof = {"bound": "mfma", "kernel": dominant, "achieved": report[dominant]["tflops"], "peak": peak_tflops,
                "unit": "TFLOP/s", "frac": round(report[dominant]["tflops"] / peak_tflops, 4), "traffic": traffic}
    else:
        roof = {"bound": "hbm", "kernel": dominant, "achieved": report[dominant]["gbs"], "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "frac": round(report[dominant]["gbs"] / PEAK_HBM_GBS, 4), "traffic": traffic}

    out = {
        "metric": "tokens scored+selected+gathered/sec per layer",
        "value": round(S / (ms_per_step * 1e-3), 1),
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
        "config": {"workload": f"{cfg.name}: one Llama-shaped layer, S={S}, {cfg.H}x{cfg.d} heads ({cfg.H_kv} KV), hidden {cfg.C}, "
                               f"consumer GEMM {cfg.C}->{cfg.N}, segment {cfg.L}, keep ratio {cfg.ratio} (k={cfg.k}, M={cfg.M}), causal, "
                               f"self term excluded" + (", backward scatter-add included" if do_scatter else ""),
                   "S": S, "H": cfg.H, "H_kv": cfg.H_kv, "d": cfg.d, "C": cfg.C, "N": cfg.N, "L": cfg.L, "k": cfg.k, "M": cfg.M},
        "roofline": roof,
        "phases": report,
    }
    if not args.step_only:
        out["gather_fold"] = measure_gather_fold(cfg, lemo, ev, stream, X, W, kept, Y)
        out["fused_in_place_add"] = measure_fused_output_projection(cfg, lemo, ev, stream, kept)
        out["gemm_backward"] = measure_gemm_backward(cfg, lemo, ev, stream, X, W, kept)
        if cfg.dtype == "bf16":
            out["kept_attention"] = measure_kept_attention(cfg, lemo, ev, stream, Q, K, kept)
        out["block_wise"] = measure_block_scoring(cfg, lemo, ev, stream, Q, K, lse2, flags)
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle on a bounded sample", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(cfg, lay, wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
