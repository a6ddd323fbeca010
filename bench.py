#!/usr/bin/env python3
"""Benchmark of the hybrid delta attention hot path on one MI355X.

One "step" = one pass of the whole prefill path (delta scan, compaction, hybrid attention) over one
synthetic batch already resident in HBM.  Headline workload: the 8K-token long-context
configuration (batch 4, 20 query / 5 KV heads, head_dim 128, window 512) at the ~60 % delta
sparsity point with 5 % jump rate.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5|C3|C2] [--mode gather|rebase]
                    [--no-decode] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_MFMA_BF16_TFLOPS = 2500.0  # dense bf16 MFMA
PEAK_VALU_F32_TFLOPS = 157.3    # published: 256 CU x 4 SIMD x 32 fp32 multiply-adds per cycle x 2 flop x 2.4 GHz
# The prefill kernel's gather loop multiplies with v_fma_mix_f32 (fp16 x fp32 + fp32), which issues once per 4 cycles per
# SIMD: 256 CU x 4 SIMD x 64 lanes / 4 cycles x 2 flop x 2.4 GHz (a register-only loop of that instruction measured
# 63 - 71 TFLOP/s at the kernel's 2 waves per SIMD).  The published 157.3 counts two fp32 multiply-adds per lane and
# 2 cycles (packed or dual-rate fp32), the plain single-rate figure is half of it.
FMA_MIX_ISSUE_TFLOPS = 78.6

PROFILE_TRAFFIC = os.path.join(ROOT, "profiles", "prefill_C5_and_decode_C4_hbm_traffic.md")


def measured_traffic(path=PROFILE_TRAFFIC):
    """HBM-side bytes per launch of the dominant kernels (fetch + write), as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE and written down in the profile summary (its table, MiB per launch, already scaled by the copy
    calibration), and the commit the counters were taken at.  Counters cannot be read from inside this process, so
    the bench line quotes the summary; workloads it does not cover report null."""
    rows, commit = {}, None
    labels = {"prefill attention, gather mode": ("C5/p05/s60", "gather"),
              "prefill attention, telescoped mode": ("C5/p05/s60", "rebase"),
              "decode step kernel": ("C4/p05/s57", "decode")}
    try:
        text = open(path).read()
    except OSError:
        return rows, commit
    for line in text.splitlines():
        if line.startswith("Counters taken at commit"):
            commit = line.split("`")[1]
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        for label, key in labels.items():
            if len(cells) >= 4 and cells[0].startswith(label):
                rows[key] = (float(cells[2]) + float(cells[3])) * 2 ** 20
    return rows, commit


MEASURED_TRAFFIC_BYTES, TRAFFIC_FROM_COMMIT = measured_traffic()


def outside_rows(n, W, sliding=False):
    """rows_out[j]: number of query rows for which key column j lies outside the exact window
    (rows below the column's square, or rows i >= j + W for the band)."""
    import numpy as np
    j = np.arange(n)
    if sliding:
        return np.maximum(0, n - np.minimum(n, j + W))
    return np.maximum(0, n - np.minimum(n, (j // W + 1) * W))


def prefill_bench(args, da, wl, torch, np, mode_name, data=None, workload=None):
    w = workload or {"C5": wl.c5(args.sparsity, args.p_jump), "C3": wl.C3, "C2": wl.C2}[args.workload]
    mode = da.DA_SCORE_GATHER if mode_name == "gather" else da.DA_SCORE_REBASE
    wmode = da.DA_WINDOW_SLIDING if args.window_mode == "sliding" else da.DA_WINDOW_BLOCK
    theta = wl.theta_for(w)
    tdt = torch.bfloat16
    if data is None:
        x = wl.generate(w)
        Q, K, V = (torch.from_numpy(x[k]).to(tdt).cuda().contiguous() for k in "QKV")
    else:
        x, (Q, K, V) = data
    B, Hq, n, d = Q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    p = da.make_params(Q, K, w.window, theta, 0.0, mode, wmode)
    ws = torch.empty(da.delta_attn_prefill_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    out = (torch.empty_like(Q), torch.empty((B, Hkv, n, d // 32), dtype=torch.int32, device="cuda"),
           torch.empty((B, Hkv), dtype=torch.int64, device="cuda"))

    pieces = max(1, args.chunks)
    if pieces > 1:   # chunked prefill onto a growing cache: same rows, same results, `pieces` calls per step
        cache = da.Cache(B, Hq, Hkv, d, n, max(w.window, 64), theta, tdt)
        cuts = [n * i // pieces for i in range(pieces + 1)]
        parts = [tuple(t[:, :, cuts[i]:cuts[i + 1]].contiguous() for t in (Q, K, V)) for i in range(pieces)]

    def step():
        if pieces == 1:
            da.delta_attn_prefill(Q, K, V, theta, w.window, score_mode=mode, workspace=ws, out=out, window_mode=wmode)
            return
        cache.reset()
        for q_, k_, v_ in parts:
            o_, _, nz_ = da.delta_attn_prefill_append(cache, q_, k_, v_, theta, w.window, score_mode=mode,
                                                      window_mode=wmode)
        out[2].copy_(cache.nnz())

    if args.calibrate_copy:   # a plain copy of known size, to scale the profiler's byte counters
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    use_graph = args.graph and pieces == 1
    if use_graph:   # the call allocates nothing and records no memset: replay it from a HIP graph (no launch gaps)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        step = graph.replay
        step()
        torch.cuda.synchronize()
    da.delta_attn_stage_timing_enable(not use_graph)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stages = da.delta_attn_stage_timing_read()
    da.delta_attn_stage_timing_enable(False)

    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = B * n / (dt / args.steps)
    s_m, s_c = da.delta_attn_sparsity(out[2], n, d, w.window)

    # algorithmic work of the attention kernel (dominant kernel)
    mask = (out[1] if pieces == 1 else cache.mask_rows()).cpu().numpy().view(np.uint32)
    nnz_col = np.bitwise_count(mask).sum(axis=-1).astype(np.int64)   # [B, Hkv, n]
    rows_out = outside_rows(n, w.window, args.window_mode == "sliding")
    sparse_macs = float((nnz_col * rows_out[None, None, :]).sum()) * g
    # of which in columns the gather kernel re-bases on the matrix cores instead of gathering: full columns (more than
    # d - 8 surviving entries) of whole 32-column blocks that have at least four of them
    nb = n // 32
    full = (nnz_col[..., :nb * 32] > d - 8).reshape(B, Hkv, nb, 32)
    routed = full & (full.sum(axis=-1, keepdims=True) >= 4)
    rebased_macs = float((nnz_col[..., :nb * 32] * routed.reshape(B, Hkv, nb * 32) * rows_out[None, None, :nb * 32]).sum()) * g
    if mode != da.DA_SCORE_GATHER or w.dtype != "bf16" or d not in (64, 128):
        rebased_macs = 0.0
    outside_pairs = float(rows_out.sum()) * B * Hq
    causal_pairs = n * (n + 1) / 2.0 * B * Hq
    window_pairs = causal_pairs - outside_pairs
    # per step: one launch, or one per piece; under a graph no per-kernel events exist: the whole step stands in
    attn_ms = stages["attn"][0] / args.steps if not use_graph else dt / args.steps * 1e3
    if mode == da.DA_SCORE_GATHER:
        alu_flops = 2.0 * sparse_macs
        mfma_flops = 2.0 * (window_pairs + causal_pairs) * d
        roof = {"bound": "alu", "achieved": alu_flops / (attn_ms * 1e-3) / 1e12, "peak": PEAK_VALU_F32_TFLOPS,
                "unit": "TFLOP/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof["sparse_gmac_rebased_on_matrix_cores"] = rebased_macs / 1e9
        roof["achieved_on_vector_alu"] = 2.0 * (sparse_macs - rebased_macs) / (attn_ms * 1e-3) / 1e12
        roof["single_rate_issue_peak"] = FMA_MIX_ISSUE_TFLOPS
        roof["frac_of_single_rate_issue_peak"] = roof["achieved"] / FMA_MIX_ISSUE_TFLOPS
    else:
        alu_flops = 0.0
        mfma_flops = 2.0 * (2.0 * causal_pairs) * d
        roof = {"bound": "mfma", "achieved": mfma_flops / (attn_ms * 1e-3) / 1e12, "peak": PEAK_MFMA_BF16_TFLOPS,
                "unit": "TFLOP/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
    es = 2
    hbm_bytes = (2 * B * Hq * n * d + 2 * B * Hkv * n * d) * es + B * Hkv * n * d / 8
    roof.update({"traffic": MEASURED_TRAFFIC_BYTES.get((w.key(), "gather" if mode == da.DA_SCORE_GATHER else "rebase"))
                 if args.window_mode == "block" and pieces == 1 else None,
                 "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE)",
                 "traffic_from": f"profiles/{os.path.basename(PROFILE_TRAFFIC)} at commit {TRAFFIC_FROM_COMMIT}",
                 "kernel": "prefill attention", "kernel_ms": attn_ms,
                 "algorithmic_sparse_gmac": sparse_macs / 1e9, "row_weighted_density": sparse_macs / max(outside_pairs * d, 1),
                 "mfma_tflops": mfma_flops / (attn_ms * 1e-3) / 1e12,
                 "mfma_frac": mfma_flops / (attn_ms * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS,
                 "hbm_gbs": hbm_bytes / (attn_ms * 1e-3) / 1e9, "hbm_frac": hbm_bytes / (attn_ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
    res = {
        "metric": "hybrid delta-attention tokens/s per layer at ~60% sparsity",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.key()}: prefill B{B} Hq{Hq} Hkv{Hkv} n{n} d{d} W{w.window} theta={theta:.6g} "
                               f"p_jump={w.p_jump}", "score_mode": mode_name, "window_mode": args.window_mode, "pieces": pieces, "hip_graph": bool(use_graph), "s_m": s_m, "s_c": s_c},
        "stage_ms": {k: (v[0] / v[1] if v[1] else 0.0) for k, v in stages.items() if v[1]},
        "roofline": roof,
    }
    return res, (w, x, theta, (Q, K, V))


def cpu_baseline(w, x, theta, np):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: every query row and
    every query head of batch entry 0 (one of w.batch entries)."""
    from oracle import delta_oracle as orc
    n, g = w.seq_len, w.n_q_heads // w.n_kv_heads
    t0 = time.perf_counter()
    for hk in range(w.n_kv_heads):
        _, dK, _, _ = orc.delta_scan(x["K"][0, hk], theta)
        for h in range(hk * g, (hk + 1) * g):
            orc.hybrid_rows(x["Q"][0, h], x["K"][0, hk], x["V"][0, hk], dK, w.window, 0, None, 0, (0, n))
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"batch entry 0 of {w.batch}: all {n} query rows x all {w.n_q_heads} query heads of the same "
                      f"workload, fp64, {dt:.1f} s"}


def decode_bench(args, da, wl, torch, np):
    w = wl.C4
    theta = wl.theta_for(w)
    x = wl.generate(w)
    tdt = torch.bfloat16
    Q, K, V = (torch.from_numpy(x[k]).to(tdt).cuda().contiguous() for k in "QKV")
    del x
    B, Hq, L, d = Q.shape
    Hkv, n, steps = K.shape[1], w.seq_len, w.decode_steps
    # Several independent copies of the cache are stepped in turn, so that the bytes a step reads were last touched
    # ~0.5 GB of traffic ago: well beyond the 256 MB last-level cache, as in a model whose other layers run between
    # two steps of this one.  (One cache stepped alone stays resident there and measures 10-14 % faster.)
    ncopies = 4
    caches = [da.Cache(B, Hq, Hkv, d, L, w.window, theta, tdt) for _ in range(ncopies)]
    cache = caches[0]
    qs = [Q[:, :, t].contiguous() for t in range(n, L)]
    ks = [K[:, :, t].contiguous() for t in range(n, L)]
    vs = [V[:, :, t].contiguous() for t in range(n, L)]
    Qp, Kp, Vp = Q[:, :, :n].contiguous(), K[:, :, :n].contiguous(), V[:, :, :n].contiguous()
    o = torch.empty_like(qs[0])
    mrow = torch.empty((B, Hkv, d // 32), dtype=torch.int32, device="cuda")

    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def run(stage_timing, used):
        for c in used:
            c.reset()
            da.delta_attn_prefill(Qp, Kp, Vp, theta, w.window, cache=c)
        torch.cuda.synchronize()
        da.delta_attn_stage_timing_enable(stage_timing)
        t0 = time.perf_counter()
        ev0.record()
        for i in range(steps):
            for c in used:
                da.delta_attn_decode(c, qs[i], ks[i], vs[i], out=o, mask_row=mrow)
        ev1.record()
        t1 = time.perf_counter()
        torch.cuda.synchronize()
        k = len(used)
        return (time.perf_counter() - t0) / k, (t1 - t0) / k, ev0.elapsed_time(ev1) / k

    run(False, caches)
    dt, enqueue, dev_ms = run(False, caches)   # the reported rate: no per-stage events in the stream
    _, _, warm_ms = run(False, caches[:1])     # one cache alone: resident in the last-level cache
    run(True, caches)                          # per-kernel durations from HIP events around each launch
    stages = da.delta_attn_stage_timing_read()
    da.delta_attn_stage_timing_enable(False)
    nnz = int(cache.nnz().sum())
    s_m, s_c = da.delta_attn_sparsity(cache.nnz(), L, d, w.window)
    units = B * Hkv
    t_avg = n + (steps - 1) / 2.0 + 1
    # algorithmic bytes per step: V of every cached row; mask bits and surviving key values (bf16) of the
    # rows left of the decode window; raw keys of the window rows; q and o
    hist = t_avg - w.window
    bytes_step = units * (t_avg * d * 2 + hist * d / 8 + (nnz / units) * (hist / L) * 2 + w.window * d * 2) \
        + 2 * B * Hq * d * 2
    # The step is one launch (work groups merge on chip), so the device time of the whole loop (one HIP event pair
    # on the launch stream around all steps) divided by the steps is that kernel's average duration plus the launch
    # gaps; the per-stage event pairs add about 2 us to a 24 us kernel and are reported separately.
    chunk_ms = dev_ms / steps
    for c in caches:
        c.close()
    return {"workload": f"{w.key()}: decode B{B} Hq{Hq} Hkv{Hkv} d{d} cached {n} + {steps} steps W_d{w.window} "
                        f"theta={theta:.6g}", "value": B * steps / dt, "unit": "tokens/s",
            "ms_per_step": dt / steps * 1e3, "host_enqueue_ms_per_step": enqueue / steps * 1e3,
            "cache_copies_stepped_in_turn": ncopies, "ms_per_step_one_cache_resident_in_llc": warm_ms / steps,
            "s_m": s_m, "s_c": s_c,
            "stage_ms_with_event_pairs": {k: v[0] / v[1] for k, v in stages.items() if v[1]},
            "roofline": {"bound": "hbm", "kernel": "decode step", "kernel_ms": chunk_ms,
                         "achieved": bytes_step / (chunk_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": bytes_step / (chunk_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                         "traffic": MEASURED_TRAFFIC_BYTES.get((w.key(), "decode")),
                         "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE)",
                         "traffic_from": f"profiles/{os.path.basename(PROFILE_TRAFFIC)} at commit {TRAFFIC_FROM_COMMIT}",
                         "algorithmic_mb_per_step": bytes_step / 1e6}}


def c5_sweep(args, da, wl, torch, np):
    """The 12-point C5 sweep (threshold for S_m ~ 0, 0.4, 0.6, 0.8 x jump rate 1, 5, 20 %), both score modes."""
    rows = []
    for p_jump in (0.01, 0.05, 0.20):
        for sp in (0.0, 0.40, 0.60, 0.80):
            args.sparsity, args.p_jump = sp, p_jump
            r, (w, x, theta, dev) = prefill_bench(args, da, wl, torch, np, "gather")
            r2, _ = prefill_bench(args, da, wl, torch, np, "rebase", data=(x, dev))
            rows.append({"workload": w.key(), "theta": theta, "s_m": r["config"]["s_m"],
                         "row_weighted_density": r["roofline"]["row_weighted_density"],
                         "sparse_gmac": r["roofline"]["algorithmic_sparse_gmac"],
                         "gather_attn_ms": r["roofline"]["kernel_ms"], "gather_tokens_per_s": r["value"],
                         "gather_alu_tflops": r["roofline"]["achieved"],
                         "gather_gmac_rebased_on_matrix_cores": r["roofline"]["sparse_gmac_rebased_on_matrix_cores"],
                         "rebase_attn_ms": r2["roofline"]["kernel_ms"], "rebase_tokens_per_s": r2["value"],
                         "rebase_mfma_frac": r2["roofline"]["frac"]})
            sys.stderr.write(json.dumps(rows[-1]) + "\n")
            sys.stderr.flush()
            del x, dev
            torch.cuda.empty_cache()
    return rows


def eq5_sweep(args, da, wl, torch, np):
    """Prompt lengths 64 .. 8192 with the window of Eq. 5 (gamma as given, W_max = 512): the C5 head shape,
    generator and threshold at every length (the paper's own regime is the short end, windows of 2 - 10 keys)."""
    import dataclasses
    base = wl.c5(0.60, 0.05)
    theta = wl.theta_for(base)
    rows = []
    for n in (64, 128, 256, 512, 1024, 2048, 4096, 8192):
        W = da.delta_attn_window_from_gamma(n, args.gamma, 512)
        w = dataclasses.replace(base, seq_len=n, window=W, theta=theta, target_sparsity=None)
        r, (_, x, _, dev) = prefill_bench(args, da, wl, torch, np, "gather", workload=w)
        r2, _ = prefill_bench(args, da, wl, torch, np, "rebase", data=(x, dev), workload=w)
        rows.append({"n": n, "window": W, "s_m": r["config"]["s_m"], "s_c": r["config"]["s_c"],
                     "gather_ms_per_step": r["ms_per_step"], "gather_tokens_per_s": r["value"],
                     "gather_stage_ms": r["stage_ms"],
                     "rebase_ms_per_step": r2["ms_per_step"], "rebase_tokens_per_s": r2["value"],
                     "rebase_stage_ms": r2["stage_ms"]})
        sys.stderr.write(json.dumps(rows[-1]) + "\n")
        sys.stderr.flush()
        del x, dev
    return rows


def decode_sweep(args, da, wl, torch, np):
    """Decode step time over head sizes and unit counts (batch x KV heads), 2048 cached tokens, decode window 128,
    C4's generator at a fixed threshold: one work group per unit (waves merge on chip) against single-wave work
    groups plus a merge launch - the measurements behind the default launch plan."""
    rows = []
    theta, n, steps, Wd = 0.11, 2048, 40, 128
    for d in (64, 128):
        for B, Hq, Hkv in ((8, 32, 8), (16, 32, 8), (32, 20, 5), (24, 32, 8), (32, 32, 8), (64, 32, 8)):
            L = n + steps
            Q, K, V = (torch.from_numpy(wl.round_to_dtype(
                wl.ar1_jump(9, name, list(range(B)), H, L, d, 0.05, True), "bf16")).to(torch.bfloat16).cuda()
                for name, H in (("Q", Hq), ("K", Hkv), ("V", Hkv)))
            qs = [Q[:, :, t].contiguous() for t in range(n, L)]
            ks = [K[:, :, t].contiguous() for t in range(n, L)]
            vs = [V[:, :, t].contiguous() for t in range(n, L)]
            Qp, Kp, Vp = Q[:, :, :n].contiguous(), K[:, :, :n].contiguous(), V[:, :, :n].contiguous()
            # copies of the cache stepped in turn: 0.6 GB between two steps of the same copy, so that the 256 MB
            # last-level cache cannot serve them
            ncopies = max(2, int(np.ceil(600e6 / (B * Hkv * n * d * 2.9))))
            row = {"head_dim": d, "units": B * Hkv, "cache_copies": ncopies}
            for name, plan in (("one_group_per_unit_us", (1, 0)), ("single_wave_groups_us", (0, 0)), ("default_us", (-1, 0))):
                caches = [da.Cache(B, Hq, Hkv, d, L, Wd, theta, torch.bfloat16) for _ in range(ncopies)]
                for cache in caches:
                    cache.set_launch_plan(*plan)
                    da.delta_attn_prefill(Qp, Kp, Vp, theta, 512, score_mode=da.DA_SCORE_REBASE, cache=cache)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                for i in range(8):
                    for cache in caches:
                        da.delta_attn_decode(cache, qs[i], ks[i], vs[i])
                e0.record()
                for i in range(8, steps):
                    for cache in caches:
                        da.delta_attn_decode(cache, qs[i], ks[i], vs[i])
                e1.record()
                torch.cuda.synchronize()
                row[name] = e0.elapsed_time(e1) / ((steps - 8) * ncopies) * 1e3
                if plan[0] < 0:
                    s_m, _ = da.delta_attn_sparsity(caches[0].nnz(), L, d, Wd)
                    t_avg = n + steps / 2
                    row["algorithmic_mb_per_step"] = B * Hkv * t_avg * d * (2 + 1 / 8 + 2 * (1 - s_m)) / 1e6
                    row["default_tb_per_s"] = row["algorithmic_mb_per_step"] / row[name]
                for cache in caches:
                    cache.close()
            rows.append(row)
            sys.stderr.write(json.dumps(row) + "\n")
            sys.stderr.flush()
            del Q, K, V, qs, ks, vs, Qp, Kp, Vp
            torch.cuda.empty_cache()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C5", choices=["C5", "C3", "C2"])
    ap.add_argument("--mode", default="gather", choices=["gather", "rebase"])
    ap.add_argument("--sparsity", type=float, default=0.60, help="C5 only: 0, 0.4, 0.6 or 0.8 (tuned theta)")
    ap.add_argument("--p-jump", type=float, default=0.05, help="C5 only: 0.01, 0.05 or 0.20")
    ap.add_argument("--window-mode", default="block", choices=["block", "sliding"],
                    help="exact region of the prefill: squares of side W on the diagonal (the paper's prefill stage, "
                         "the headline) or the band of the W newest keys")
    ap.add_argument("--chunks", type=int, default=1,
                    help="prefill the sequence in this many equal pieces onto a growing cache (delta_attn_prefill_append)")
    ap.add_argument("--graph", action="store_true",
                    help="prefill: capture one call into a HIP graph and time replays (short prompts are launch-bound)")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-other-mode", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (profiling aid for scaling FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--eq5-sweep", action="store_true",
                    help="only run prompt lengths 64..8192 with the window of Eq. 5 (see --gamma) and exit")
    ap.add_argument("--gamma", type=float, default=0.05, help="Eq. 5 scaling factor for --eq5-sweep")
    ap.add_argument("--sweep", action="store_true",
                    help="only run the 12-point C5 sweep (threshold x jump rate), both score modes, and exit")
    ap.add_argument("--decode-sweep", action="store_true",
                    help="decode step time over head sizes and unit counts under both launch plans")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build is a single-GPU kernel library; run with --gpus 1\n")
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2507_19608_amd import binding as da
    from paper_2507_19608_amd import workloads as wl
    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible; the library has no CPU path\n")
        sys.exit(1)
    da.lib()
    if args.decode_sweep:
        print(json.dumps({"decode_sweep": decode_sweep(args, da, wl, torch, np)}))
        return
    if args.eq5_sweep:
        print(json.dumps({"eq5_sweep": eq5_sweep(args, da, wl, torch, np), "gamma": args.gamma, "w_max": 512,
                          "steps": args.steps, "warmup": args.warmup, "window_mode": args.window_mode}))
        return
    if args.sweep:
        print(json.dumps({"c5_sweep": c5_sweep(args, da, wl, torch, np), "steps": args.steps, "warmup": args.warmup,
                          "window_mode": args.window_mode}))
        return
    res, (w, x, theta, dev) = prefill_bench(args, da, wl, torch, np, args.mode)
    if not args.no_other_mode:
        # the same workload through the other score mode (same results; see include/delta_attn.h)
        other = "rebase" if args.mode == "gather" else "gather"
        r2, _ = prefill_bench(args, da, wl, torch, np, other, data=(x, dev))
        res["other_score_mode"] = {k: r2[k] for k in ("value", "unit", "ms_per_step", "stage_ms", "roofline")}
        res["other_score_mode"]["score_mode"] = other
    del dev
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_baseline(w, x, theta, np)
    del x
    torch.cuda.empty_cache()
    if not args.no_decode:
        res["decode"] = decode_bench(args, da, wl, torch, np)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
