#!/usr/bin/env python3
"""Benchmark of the DynamicRad attention hot path on one MI355X.

One "step" is one attention call of the whole path on the headline workload (cfg4:
B=1, H=40, d=128, 21 frames x 45x80 tokens = 75 600 tokens, block 128, static-ratio
selection at >= 85 % effective sparsity, lambda = 0.5, fused-head scores, bf16):

    dr_block_scores -> dr_build_mask -> dr_sparse_attn_fwd

Inputs are synthetic (workloads/generate.py), resident in HBM before the timed region.
Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

NOMINAL_MHZ = 2400.0
PEAK_BF16_TFLOPS = 2500.0          # MI355X published dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def generate_on_device(wl, heads, device):
    """Q, K, V [1, len(heads), N, d] in the run dtype on the GPU; heads generated on host threads."""
    import torch
    from workloads.generate import make_head, round_to_dtype
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    out = [torch.empty((wl.B, len(heads), wl.N, wl.d), dtype=tdt, device=device) for _ in range(3)]
    host = {}

    def one(i):
        q, k, v = make_head(wl, 0, heads[i])
        return i, [round_to_dtype(x, wl.dtype) for x in (q, k, v)]

    workers = min(12, max(1, (os.cpu_count() or 8) - 2), len(heads))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        for i, tensors in ex.map(one, range(len(heads))):
            for dst, src in zip(out, tensors):
                dst[0, i].copy_(src)
            if heads[i] < 2 or heads[i] == heads[-1]:
                host[heads[i]] = tensors
    return out, host


def algorithmic_flop(rowptr, colidx, wl, H):
    """4 d sum over kept (query block, key block) pairs of n_q n_k, times heads and batch."""
    import numpy as np
    Sb, Bs, N = wl.Sb, wl.Bs, wl.N
    n_blk = np.minimum(N, (np.arange(Sb) + 1) * Bs) - np.arange(Sb) * Bs
    pairs = 0
    for qb in range(Sb):
        cols = colidx[rowptr[qb]:rowptr[qb + 1]]
        pairs += int(n_blk[qb]) * int(n_blk[cols].sum())
    return 4.0 * wl.d * pairs * H * wl.B


def read_traffic(kernel_tag):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary (or None)."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_pmc.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(wl, host_heads, mode, par, kept_blocks_total, H, O, rp_gpu, ci_gpu, budget_s=15.0):
    """Times the CPU oracle (scores + geometry + selection in full, attention on a sample of query blocks) and compares
    every attention row it computes with the output O of the launch that was timed.  Returns (cpu_baseline, parity)."""
    import numpy as np
    import torch
    from oracle import dynamicrad_oracle as o
    f64 = lambda t: t.to(torch.float64).numpy()
    Q = np.stack([f64(host_heads[h][0]) for h in (0, 1)])[None]
    K = np.stack([f64(host_heads[h][1]) for h in (0, 1)])[None]
    t0 = time.perf_counter()
    sc = o.block_scores(Q, K, wl.Bs, 2)
    tab = o.frame_table(wl.Nf, wl.Nt, wl.Bs, 1.0, wl.lam)
    cls = o.classify_blocks(wl.N, wl.Nt, wl.Bs, tab, 0.15, 0.60)
    o.build_mask(sc.astype(np.float32), cls, mode, par)
    t_front = time.perf_counter() - t0
    # the attention rows are taken under the mask the GPU emitted (the mask itself is compared bit for bit in the
    # tests, where the oracle selects from the GPU's own fp32 scores)
    rp, ci = rp_gpu.astype(np.int64), ci_gpu.astype(np.int64)
    worst, checked = 0.0, 0

    def check(hd_index, hd, qb, want):
        nonlocal worst, checked
        got = O[0, hd_index, qb * wl.Bs: qb * wl.Bs + want.shape[0]].to(torch.float64).cpu().numpy()
        worst = max(worst, float(np.abs(got - want).max()))
        checked += want.shape[0]

    rng = np.random.default_rng(7)
    done_blocks, rows, t_attn = 0, 0, 0.0
    for hd in (0, 1):
        Vh = f64(host_heads[hd][2])
        for qb in rng.permutation(wl.Sb):
            t1 = time.perf_counter()
            want = o.masked_attention(Q[0, hd], K[0, hd], Vh, rp, ci, wl.Bs, rows=[int(qb)])
            t_attn += time.perf_counter() - t1
            check(hd, hd, int(qb), want[int(qb)])
            done_blocks += int(rp[qb + 1] - rp[qb])
            rows += 1
            if t_attn > budget_s:
                break
        if t_attn > budget_s:
            break
    # the last head sits at the far end of the launch's work-item order (the last XCD's run): first, last, and a few
    # random query blocks of it (untimed)
    last = max(host_heads)
    if last >= 2:
        Ql, Kl, Vl = (f64(t) for t in host_heads[last])
        picks = sorted({0, wl.Sb - 1, wl.Sb - 2, *rng.integers(0, wl.Sb, 13).tolist()})
        want = o.masked_attention(Ql, Kl, Vl, rp, ci, wl.Bs, rows=picks)
        for qb in picks:
            check(H - 1, last, qb, want[qb])
    est_ms = (t_front + t_attn * (kept_blocks_total * H / max(1, done_blocks))) * 1e3
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    tol = 2e-2 if wl.dtype == "bf16" else 1e-4
    base = {"value": est_ms, "unit": "ms per attention call (extrapolated)", "cores": int(cores), "kind": "oracle",
            "sample": (f"block scores, geometry and selection in full ({t_front:.2f} s); fp64 masked attention on {rows} "
                       f"query-block rows of heads 0-1 ({done_blocks} kept key blocks, {t_attn:.2f} s) scaled by "
                       f"kept blocks x heads = {kept_blocks_total * H}")}
    parity = {"rows": checked, "heads": sorted({0, 1, H - 1}), "max_abs_err": worst, "tol": tol,
              "what": "output of the timed launch configuration against the fp64 oracle, element by element"}
    return base, parity


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=6)          # the shader clock settles over the first ~5 attention launches of a train
    ap.add_argument("--config", default="cfg4")
    ap.add_argument("--heads", type=int, default=0, help="use only the first H heads (0 = the workload's own count)")
    ap.add_argument("--block-size", type=int, default=0, help="override the workload's block size Bs (32, 64 or 128)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run three plain 1 GiB device copies (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (the path shards by head with no exchange inside it); "
            "--gpus must be 1")
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2604_20470_amd as dr
    from workloads import CONFIGS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "3 x copy of 1 GiB (reads 1048576 KiB, writes 1048576 KiB per copy)"}))
        return
    wl = CONFIGS[args.config]
    if args.block_size:
        import dataclasses
        wl = dataclasses.replace(wl, Bs=args.block_size)
    H = args.heads or wl.H
    dev = "cuda:0"
    t0 = time.time()
    (Q, K, V), host_heads = generate_on_device(wl, list(range(H)), dev)
    log(f"[bench] generated {args.config}: H={H} N={wl.N} d={wl.d} in {time.time() - t0:.1f}s")

    ctx = dr.Context(0)
    shape = dr.shape_of(Q, wl.Nf, wl.Hg, wl.Wg, wl.Bs)
    params = dr.MaskParams(head_fuse=wl.head_fuse)
    Sb = wl.Sb
    cap, _ = dr.dr_mask_capacity(ctx, shape, wl.lam, params)
    scores = torch.empty((wl.B, 1, Sb, Sb), dtype=torch.float32, device=dev)
    rowptr = torch.empty((wl.B, 1, Sb + 1), dtype=torch.int32, device=dev)
    colidx = torch.empty((wl.B, 1, cap), dtype=torch.int32, device=dev)
    nnz = torch.empty((wl.B, 1), dtype=torch.int64, device=dev)
    O = torch.empty_like(Q)

    # selection parameter: static ratio from the geometry alone (largest rho on a 1e-3 grid reaching the target)
    if wl.mode == "static":
        mode = dr.MODE_STATIC
        if wl.ratio is not None:
            par = wl.ratio
        else:
            par, _ = dr.dr_static_ratio_for_sparsity(ctx, shape, wl.lam, params, wl.target_sparsity)
    else:
        mode, par = dr.MODE_DYNAMIC, wl.tau

    def step(ev=None):
        if ev: ev[0].record()
        dr.dr_block_scores(ctx, shape, Q, K, wl.head_fuse, scores)
        if ev: ev[1].record()
        dr.dr_build_mask(ctx, shape, mode, par, wl.lam, params, scores, rowptr, colidx, cap, nnz)
        if ev: ev[2].record()
        dr.dr_sparse_attn_fwd(ctx, shape, Q, K, V, rowptr, colidx, 1, cap, O)
        if ev: ev[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    st = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in evs])
    ms_scores, ms_mask, ms_attn = st.mean(axis=0).tolist()
    st_median, st_min = np.median(st, axis=0).tolist(), st.min(axis=0).tolist()

    n_kept = int(nnz[0, 0].item())
    assert n_kept <= cap
    rp = rowptr[0, 0].cpu().numpy()
    ci = colidx[0, 0, :n_kept].cpu().numpy()
    flop = algorithmic_flop(rp, ci, wl, H)
    dense_flop = 4.0 * wl.B * H * float(wl.N) ** 2 * wl.d
    sparsity = 1.0 - n_kept / float(Sb * Sb)
    eff_tflops = flop / (ms_attn * 1e-3) / 1e12
    assert torch.isfinite(O[0, 0, :256].float()).all()

    result = {
        "metric": "ms per attention call (block scores + mask + block-sparse attention) at 75.6k tokens; "
                  "effective TFLOP/s of the attention kernel in roofline",
        "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{args.config}: B={wl.B} H={H} d={wl.d} Nf={wl.Nf} grid={wl.Hg}x{wl.Wg} N={wl.N} "
                               f"Bs={wl.Bs} {wl.mode} par={par:.3f} lambda={wl.lam} head_fuse={wl.head_fuse}",
                   "effective_sparsity": round(sparsity, 5), "kept_blocks": n_kept, "candidate_blocks": cap},
        "stages_ms": {"block_scores": round(ms_scores, 4), "build_mask": round(ms_mask, 4),
                      "sparse_attn_fwd": round(ms_attn, 4)},
        "stages_ms_median": {"block_scores": round(st_median[0], 4), "build_mask": round(st_median[1], 4),
                             "sparse_attn_fwd": round(st_median[2], 4)},
        "stages_ms_min": {"block_scores": round(st_min[0], 4), "build_mask": round(st_min[1], 4),
                          "sparse_attn_fwd": round(st_min[2], 4)},
        "effective_tflops": round(eff_tflops, 1),
        "effective_tflops_whole_call": round(flop / (ms_per_step * 1e-3) / 1e12, 1),      # scores + mask + attention
        "dense_equivalent_tflops": round(dense_flop / (ms_attn * 1e-3) / 1e12, 1),
        "pct_bf16_mfma_peak": round(100.0 * eff_tflops / PEAK_BF16_TFLOPS, 2),
        "paper_context": "paper reports 1.7x-2.5x end-to-end speedup at >80% sparsity on NVIDIA H100 (not comparable)",
        "roofline": {"kernel": ({128: "k_attn_mfma_pair", 64: "k_attn_mfma_quad", 32: "k_attn_mfma_oct"}[wl.Bs]
                                if (wl.dtype == "bf16" and wl.d == 128) else "k_attn_generic"), "bound": "mfma", "achieved": round(eff_tflops, 1),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(eff_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": read_traffic(f"k_attn_mfma_pair_{args.config}") if wl.Bs == 128 else None,
                     "traffic_source": (f"profiles/k_attn_mfma_pair_{args.config}_pmc.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                        "runs of this command, scaled by a plain copy; not measured in this run"),
                     "flop_per_launch": flop, "avg_launch_ms": round(ms_attn, 4)},
    }
    # Shader clock while the attention kernel runs (separate, untimed pass): a one-wave probe on a side stream
    # spans ~60 % of a train of attention launches.  The MFMA peak is quoted at 2400 MHz; under this load the chip
    # holds less, so the roofline fraction is also given against the peak at the measured clock.
    def probe_clock(load_reps):
        clk = torch.zeros(2, dtype=torch.int64, device=dev)
        side = torch.cuda.Stream()
        window_us = max(2000, int(0.6 * load_reps * ms_attn * 1e3)) if load_reps else 20000
        torch.cuda.synchronize()
        if load_reps:
            dr.dr_sparse_attn_fwd(ctx, shape, Q, K, V, rowptr, colidx, 1, cap, O)
        dr.dr_clock_probe(ctx, window_us, clk, stream=side)
        for _ in range(load_reps):
            dr.dr_sparse_attn_fwd(ctx, shape, Q, K, V, rowptr, colidx, 1, cap, O)
        torch.cuda.synchronize()
        ticks, ref = (int(x) for x in clk.tolist())
        return 100.0 * ticks / max(ref, 1)
    mhz_load = probe_clock(max(4, int(round(150.0 / ms_attn))))
    mhz_idle = probe_clock(0)
    result["clock"] = {"nominal_mhz": NOMINAL_MHZ, "under_attention_mhz": round(mhz_load, 1),
                       "idle_probe_mhz": round(mhz_idle, 1),
                       "roofline_frac_at_measured_clock": round(eff_tflops / (PEAK_BF16_TFLOPS * mhz_load / NOMINAL_MHZ), 4)}
    # MFMA-only loops on this device: the matrix cores with constant and with random register operands (same shader
    # clock probe running beside them).  The roofline denominator stays the published peak; these say how much of
    # it the device can sustain at all.
    def mfma_only(shape, random_operands):
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        clk = torch.zeros(2, dtype=torch.int64, device=dev)
        side = torch.cuda.Stream()
        iters = 40000 if shape == 32 else 80000                         # ~10 ms per launch
        dr.dr_mfma_probe(ctx, shape, 512, 2000, random_operands, sink)  # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        flop = 0.0
        dr.dr_mfma_probe(ctx, shape, 512, iters, random_operands, sink)  # fills the chip before the clock window opens
        dr.dr_clock_probe(ctx, 40000, clk, stream=side)
        e0.record()
        for _ in range(6):
            flop += dr.dr_mfma_probe(ctx, shape, 512, iters, random_operands, sink)
        e1.record()
        torch.cuda.synchronize()
        ticks, ref = (int(v) for v in clk.tolist())
        return {"tflops": round(flop / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1), "clock_mhz": round(100.0 * ticks / max(ref, 1), 1)}
    result["mfma_only"] = {"32x32x16": {"constant_operands": mfma_only(32, False), "random_operands": mfma_only(32, True)},
                           "16x16x32": {"constant_operands": mfma_only(16, False), "random_operands": mfma_only(16, True)}}
    result["roofline"]["frac_of_measured_mfma_only_random"] = round(
        eff_tflops / result["mfma_only"]["32x32x16"]["random_operands"]["tflops"], 4)
    # The same matrix instruction, one wave per SIMD, with one exponential and two fp32 instructions per slot: what a
    # loop with the attention loop's kind of vector work beside every matrix instruction sustains with no memory
    # traffic at all (matrix flop only are counted).
    def mfma_mix():
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        dr.dr_mfma_mix_probe(ctx, 256, 2000, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        flop = 0.0
        dr.dr_mfma_mix_probe(ctx, 256, 80000, sink)                      # ~15 ms per launch; the chip is at its working clock when timing starts
        e0.record()
        for _ in range(4):
            flop += dr.dr_mfma_mix_probe(ctx, 256, 80000, sink)
        e1.record()
        torch.cuda.synchronize()
        return {"tflops": round(flop / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1),
                "per_slot": "1 v_mfma_f32_32x32x16_bf16 + 1 v_exp_f32 + 2 v_fma_f32, random operands, one wave per SIMD"}
    result["mfma_with_vector_mix"] = mfma_mix()
    result["roofline"]["frac_of_measured_mfma_with_vector_mix"] = round(eff_tflops / result["mfma_with_vector_mix"]["tflops"], 4)
    # The scoring and mask stages are HBM/latency bound; with fused-head scoring (2 of 40 heads) they move only a few
    # MB, so their bandwidth is shown on the per-head variant (head_fuse = 0: every head scored, one mask per head).
    def timed(fn, iters=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters
    ph = dr.MaskParams(head_fuse=0)
    sc_h = torch.empty((wl.B, H, Sb, Sb), dtype=torch.float32, device=dev)
    rp_h = torch.empty((wl.B, H, Sb + 1), dtype=torch.int32, device=dev)
    ci_h = torch.empty((wl.B, H, cap), dtype=torch.int32, device=dev)
    nz_h = torch.empty((wl.B, H), dtype=torch.int64, device=dev)
    ms_sc = timed(lambda: dr.dr_block_scores(ctx, shape, Q, K, 0, sc_h))
    ms_mk = timed(lambda: dr.dr_build_mask(ctx, shape, mode, par, wl.lam, ph, sc_h, rp_h, ci_h, cap, nz_h))
    es = 2 if wl.dtype == "bf16" else 4
    bytes_sc = 2.0 * wl.B * H * wl.N * wl.d * es + 4.0 * wl.B * H * Sb * Sb
    bytes_mk = wl.B * H * (4.0 * Sb * Sb + Sb * Sb + 4.0 * (Sb + 1)) + 4.0 * float(nz_h.sum().item())
    result["hbm_stages_per_head_variant"] = {
        "block_scores": {"ms": round(ms_sc, 4), "algorithmic_bytes": bytes_sc,
                         "GBps": round(bytes_sc / ms_sc / 1e6, 1), "frac_of_8TBps": round(bytes_sc / ms_sc / 1e6 / PEAK_HBM_GBS, 4)},
        "build_mask": {"ms": round(ms_mk, 4), "algorithmic_bytes": bytes_mk,
                       "GBps": round(bytes_mk / ms_mk / 1e6, 1), "frac_of_8TBps": round(bytes_mk / ms_mk / 1e6 / PEAK_HBM_GBS, 4)},
    }
    del sc_h, rp_h, ci_h, nz_h
    # build_mask alone in each selection rule (fused-head scores, one mask): latency-bound launches
    pz = dr.MaskParams(head_fuse=wl.head_fuse, tau_far=0.8, seed=1)
    result["build_mask_ms_by_rule"] = {
        "static_topk": round(timed(lambda: dr.dr_build_mask(ctx, shape, dr.MODE_STATIC, 0.05, wl.lam, params, scores, rowptr, colidx, cap, nnz)), 4),
        "cumulative_mass": round(timed(lambda: dr.dr_build_mask(ctx, shape, dr.MODE_DYNAMIC, 0.9, wl.lam, params, scores, rowptr, colidx, cap, nnz)), 4),
        "zscore_threshold": round(timed(lambda: dr.dr_build_mask(ctx, shape, dr.MODE_ZSCORE, 0.3, wl.lam, pz, scores, rowptr, colidx, cap, nnz)), 4),
        "uniform_sample": round(timed(lambda: dr.dr_build_mask(ctx, shape, dr.MODE_UNIFORM, 0.05, wl.lam, pz, None, rowptr, colidx, cap, nnz)), 4),
    }
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a bounded sample and comparing it with the timed launch's output ...")
        mode_name = "static" if mode == dr.MODE_STATIC else "dynamic"
        result["cpu_baseline"], result["parity_in_bench"] = cpu_baseline(wl, host_heads, mode_name, par, n_kept, H, O, rp, ci)
    else:
        result["cpu_baseline"], result["parity_in_bench"] = None, None
    print(json.dumps(result), flush=True)
    pib = result.get("parity_in_bench")
    if pib and not (pib["max_abs_err"] <= pib["tol"]):
        log(f"[bench] PARITY FAILURE: max abs error {pib['max_abs_err']:.3e} above {pib['tol']:.0e}")
        sys.exit(1)


if __name__ == "__main__":
    main()
