#!/usr/bin/env python3
"""Benchmark of the AnchorAttention prefill path on one MI355X.

A step is one pass of the whole hot path (anchor computation -> stripe
identification -> gathered sparse attention) over one attention layer of the
128k-token GQA workload (32 query / 8 KV heads, d = 128, bf16), inputs already
resident in HBM.  One JSON line is printed:

  value / ms_per_step : ms per layer of the fused entry point
  effective_tflops    : 4 * d * attended (q,k) pairs / time
  stage_ms            : per-stage times (the same kernels through the stage-wise entry
                        points, HIP events between the launches, same stream)
  roofline            : stage-3 kernel (the dominant one) against the bf16 MFMA peak
  dense_flash_ms      : the from-scratch dense causal flash kernel on the same GPU
  recall              : mean exp(lse_sparse - lse_dense), attention mass kept
  calibrated          : the same measurements with the planted magnitudes in scaled-logit
                        units (signal="logit"), the regime where the threshold separates
                        stripes from background
  peaked              : the same with the planted magnitudes times three and the threshold
                        scaled with them (signal="peaked"): the planted columns then hold most
                        of a row's attention mass, as in real heads, so high sparsity and high
                        recall occur together
  cpu_baseline        : the fp64 CPU oracle timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15   # MI355X dense bf16, FLOP/s
HBM_PEAK = 8.0e12         # B/s


def load_inputs(torch, synth, wl, signal, log=None):
    t0 = time.time()
    seq = synth.make_sequence(wl, 0, signal=signal)
    qkv = tuple(torch.from_numpy(seq[n]).to(torch.bfloat16)[None].cuda() for n in ("q", "k", "v"))
    if log:
        log("inputs %s/%s ready in %.1fs" % (wl.name, signal, time.time() - t0))
    return qkv


def measure(api, torch, synth, wl, signal, step, steps, warmup, theta=None, dense_steps=2, log=None):
    cfg = api.Config(block=wl.block, n_init=wl.n_init, window=wl.window, step=step,
                     theta=wl.theta if theta is None else theta)
    q, k, v = load_inputs(torch, synth, wl, signal, log)
    out = torch.empty_like(q)
    p = api.make_params(cfg, q, k, v, out)
    sz = api.anchor_sizes(p)
    ws = torch.empty(sz.prefill_ws_bytes, dtype=torch.uint8, device="cuda")
    lse = torch.empty(sz.rows, dtype=torch.float32, device="cuda")
    stats = torch.zeros(4, dtype=torch.int64, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)

    # ---- fused entry point: the timed step
    for _ in range(warmup):
        api.anchor_attention_prefill(p, q, k, v, out, lse, stats, ws)
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(steps):
        api.anchor_attention_prefill(p, q, k, v, out, lse, stats, ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    pairs, selected = int(stats[0]), int(stats[1])
    if log:
        log("fused: %.3f ms/layer, pairs %.4g" % (ms, pairs))

    # ---- per-stage times: same kernels through the stage-wise entry points
    B = api.alloc_stage_buffers(p)
    marks = [[ev() for _ in range(4)] for _ in range(steps)]
    api.anchor_compute(p, q, k, v, B["M"], B["L"], B["Acc"], B["xa"])
    api.stripe_select(p, q, k, B["xa"], B["counts"], B["offsets"], B["idx"], B["flag"], B["ws"])
    api.sparse_attn(p, q, k, v, B["M"], B["L"], B["Acc"], B["counts"], B["offsets"], B["idx"], out, B["lse"])
    torch.cuda.synchronize()
    for m in marks:
        m[0].record()
        api.anchor_compute(p, q, k, v, B["M"], B["L"], B["Acc"], B["xa"])
        m[1].record()
        api.stripe_select(p, q, k, B["xa"], B["counts"], B["offsets"], B["idx"], B["flag"], B["ws"])
        m[2].record()
        api.sparse_attn(p, q, k, v, B["M"], B["L"], B["Acc"], B["counts"], B["offsets"], B["idx"], out, B["lse"])
        m[3].record()
    torch.cuda.synchronize()
    stage = [sum(m[i].elapsed_time(m[i + 1]) for m in marks) / steps for i in range(3)]
    assert int(B["flag"]) == 0
    list_pairs = int((B["counts"].to(torch.int64).view(-1, sz.grp_cap) *
                      torch.tensor([min(wl.block * step, wl.seqlens[0] - g * wl.block * step)
                                    for g in range(sz.grp_cap)], device="cuda")).sum())
    sparse_lse = B["lse"].clone()
    # which of the two bf16 engines stage 3 ran in: the library decides on the device from the total
    # padded list length (mean list of 48 tiles of 64 entries per group or more: 256-row engine)
    pair_engine = step % 2 == 0 and int(B["offsets"][-1]) >= 48 * 64 * sz.groups
    del B

    # ---- dense causal flash on the same GPU
    dlse = torch.empty(sz.rows, dtype=torch.float32, device="cuda")
    dout = torch.empty_like(q)
    api.dense_causal_flash(p, q, k, v, dout, dlse)
    torch.cuda.synchronize()
    d0, d1 = ev(), ev()
    d0.record()
    for _ in range(dense_steps):
        api.dense_causal_flash(p, q, k, v, dout, dlse)
    d1.record()
    torch.cuda.synchronize()
    dense_ms = d0.elapsed_time(d1) / dense_steps
    recall = float(torch.exp(sparse_lse - dlse).double().mean())
    N, Hq, d = wl.seqlens[0], wl.Hq, wl.d
    causal_pairs = Hq * N * (N + 1) // 2
    res = dict(
        ms_per_layer=ms, attended_pairs=pairs, selected_entries=selected,
        sparsity=1.0 - pairs / causal_pairs,
        effective_tflops=4.0 * d * pairs / (ms * 1e-3) / 1e12,
        stage_ms=dict(anchor=stage[0], select=stage[1], sparse=stage[2]),
        stage3_list_pairs=list_pairs,
        stage3_kernel="engine_bf16_pp_kernel" if pair_engine else "engine_bf16_kernel",
        stage3_tflops=4.0 * d * list_pairs / (stage[2] * 1e-3) / 1e12 if list_pairs else 0.0,
        dense_flash_ms=dense_ms, dense_flash_tflops=4.0 * d * causal_pairs / (dense_ms * 1e-3) / 1e12,
        speedup_vs_dense=dense_ms / ms, recall=recall, theta=cfg.theta, step=step, signal=signal,
    )
    if log:
        log(json.dumps(res))
    return res, (q, k, v)


def theta_sweep(api, torch, synth, wl, signal, step, steps, warmup, thetas, granularity=0, log=None):
    """Rows of (theta, anchor on/off) -> sparsity, recall, ms per layer of the fused entry point
    on one set of inputs: the columns of the paper's threshold ablation (Table 4)."""
    q, k, v = load_inputs(torch, synth, wl, signal, log)
    out = torch.empty_like(q)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    p = api.make_params(api.Config(block=wl.block, n_init=wl.n_init, window=wl.window, step=step, theta=0.0,
                                   granularity=granularity), q, k, v, out)
    sz = api.anchor_sizes(p)
    ws = torch.empty(sz.prefill_ws_bytes, dtype=torch.uint8, device="cuda")
    lse = torch.empty(sz.rows, dtype=torch.float32, device="cuda")
    dlse = torch.empty_like(lse)
    stats = torch.zeros(4, dtype=torch.int64, device="cuda")
    api.dense_causal_flash(p, q, k, v, out, dlse)
    e0, e1 = ev(), ev()
    e0.record()
    api.dense_causal_flash(p, q, k, v, out, dlse)
    e1.record()
    torch.cuda.synchronize()
    dense_ms = e0.elapsed_time(e1)
    N = wl.seqlens[0]
    causal_pairs = wl.Hq * N * (N + 1) // 2
    rows = []
    for use_anchor in (True, False):
        for th in thetas:
            cfg = api.Config(block=wl.block, n_init=wl.n_init, window=wl.window, step=step, theta=th,
                             use_anchor=use_anchor, granularity=granularity)
            p = api.make_params(cfg, q, k, v, out)
            for _ in range(warmup):
                api.anchor_attention_prefill(p, q, k, v, out, lse, stats, ws)
            e0.record()
            for _ in range(steps):
                api.anchor_attention_prefill(p, q, k, v, out, lse, stats, ws)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / steps
            rows.append(dict(use_anchor=use_anchor, theta=th, sparsity=1.0 - int(stats[0]) / causal_pairs,
                             recall=float(torch.exp(lse - dlse).double().mean()), ms_per_layer=ms,
                             speedup_vs_dense=dense_ms / ms))
            if log:
                log(json.dumps(rows[-1]))
    return dict(workload=wl.name, signal=signal, step=step, granularity=["stripe", "block"][granularity],
                dense_flash_ms=dense_ms, rows=rows)


def cpu_baseline(synth, wl, step, signal, budget_s=12.0):
    """Oracle (as it stands) on host cores, on whole (head 0, group) units of the same workload:
    groups are taken from the end of the sequence until about budget_s of CPU time is spent."""
    from oracle import anchor_oracle as ao
    N = wl.seqlens[0]
    span = wl.block * step
    seq = synth.make_sequence(wl, 0, signal=signal, heads_kv=[0])
    op = ao.OracleParams(b_q=wl.block, n_init=wl.n_init, w=wl.window, step=step, theta=wl.theta)
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    ngrp = (N + span - 1) // span
    t0, pairs, groups = time.time(), 0, []
    for g in range(ngrp - 1, -1, -1):
        r = ao.run_group(seq["q"][0], seq["k"][0], seq["v"][0], op, g)
        pairs += r["pairs"]
        groups.append(g)
        if time.time() - t0 > budget_s:
            break
    return dict(seconds=time.time() - t0, pairs=pairs, groups=groups, cores=cores)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="gqa_128k")
    ap.add_argument("--step", type=int, default=16, help="query blocks sharing one list (paper default 16)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-calibrated", action="store_true")
    ap.add_argument("--signal", default="literal", choices=["literal", "logit", "peaked"])
    ap.add_argument("--granularity", default="stripe", choices=["stripe", "block"],
                    help="with --theta-sweep: identification per key column (the method) or per key block")
    ap.add_argument("--theta-sweep", default=None, metavar="T1,T2,...",
                    help="instead of the benchmark line: one JSON object with sparsity / recall / ms per "
                         "threshold, with and without the anchor (use with --signal logit)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only (the path shards by heads with no exchange step; "
                 "this build has no multi-GPU code): run with --gpus 1")

    import torch
    from paper_2505_23520_amd import api, synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = synth.workloads()[args.workload]
    if wl.packed or wl.dtype != "bf16":
        sys.exit("bench.py times the single-sequence bf16 workloads (gqa_8k, gqa_32k, gqa_128k); "
                 "the packed and fp32 workloads are parity-test cases")
    log = lambda s: print("[bench] " + s, file=sys.stderr, flush=True)

    if args.theta_sweep:
        thetas = [float(t) for t in args.theta_sweep.split(",")]
        print(json.dumps(theta_sweep(api, torch, synth, wl, args.signal, args.step, args.steps, args.warmup,
                                     thetas, granularity=["stripe", "block"].index(args.granularity), log=log)),
              flush=True)
        return

    main_res, tensors = measure(api, torch, synth, wl, args.signal, args.step, args.steps, args.warmup, log=log)
    del tensors
    torch.cuda.empty_cache()
    calibrated, peaked = None, None
    if not args.no_calibrated and args.signal == "literal":
        calibrated, t2 = measure(api, torch, synth, wl, "logit", args.step, args.steps, args.warmup, log=log)
        del t2
        torch.cuda.empty_cache()
        # planted magnitudes times three, threshold scaled with them
        peaked, t2 = measure(api, torch, synth, wl, "peaked", args.step, args.steps, args.warmup,
                             theta=3.0 * wl.theta, log=log)
        del t2
        torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu:
        c = cpu_baseline(synth, wl, args.step, args.signal)
        layer_ms = c["seconds"] * 1e3 * main_res["attended_pairs"] / max(1, c["pairs"])
        cpu = dict(value=layer_ms, unit="ms/layer (sample time scaled by attended pairs)", cores=c["cores"],
                   kind="oracle",
                   sample="query head 0, groups %d..%d (%d rows each) of %s: %.1f s for %.3g pairs" % (
                       c["groups"][-1], c["groups"][0], wl.block * args.step, wl.name, c["seconds"], c["pairs"]))
        log(json.dumps(cpu))

    # rates this GPU sustains at its actual clock: register-only MFMA loop, 1 GiB device copies
    # (the copies are also the dispatches of known size that scale the FETCH_SIZE / WRITE_SIZE
    # counters of a rocprofv3 --pmc run of this same command)
    scratch = torch.empty(1 << 18, dtype=torch.float32, device="cuda")
    api.anchor_probe_mfma(200, scratch)
    torch.cuda.synchronize()
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record()
    flop = api.anchor_probe_mfma(10000, scratch)
    p1.record()
    torch.cuda.synchronize()
    mfma_sustained = flop / (p0.elapsed_time(p1) * 1e-3)
    cp_src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    torch.cuda.synchronize()
    p0.record()
    for _ in range(4):
        cp_dst.copy_(cp_src)
    p1.record()
    torch.cuda.synchronize()
    hbm_sustained = 4 * 2 * cp_src.numel() * 4 / (p0.elapsed_time(p1) * 1e-3)
    del cp_src, cp_dst
    log("sustained: MFMA %.0f TFLOP/s, copy %.2f TB/s" % (mfma_sustained / 1e12, hbm_sustained / 1e12))

    N, d = wl.seqlens[0], wl.d
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "%s_stage3_%s_%s_traffic.txt" % (
        main_res["stage3_kernel"].replace("_kernel", ""), wl.name, args.signal))
    if os.path.exists(tpath):
        for ln in open(tpath):
            if ln.startswith("traffic_bytes_per_launch="):
                traffic = float(ln.split("=")[1])
    s3 = main_res["stage_ms"]["sparse"] * 1e-3
    flops3 = 4.0 * d * main_res["stage3_list_pairs"]
    line = {
        "metric": "prefill attention ms/layer at 128k GQA32/8 d128 bf16 (effective TFLOPS over attended pairs, recall alongside)",
        "value": main_res["ms_per_layer"], "unit": "ms/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_res["ms_per_layer"], "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s (B=1, Hq=%d, Hkv=%d, N=%d, d=%d, block %d, n_init %d, window %d, step %d, theta %.4f, signal %s)" % (
            wl.name, wl.Hq, wl.Hkv, N, d, wl.block, wl.n_init, wl.window, args.step, wl.theta, args.signal)},
        "effective_tflops": main_res["effective_tflops"], "sparsity": main_res["sparsity"],
        "recall": main_res["recall"], "stage_ms": main_res["stage_ms"],
        "dense_flash_ms": main_res["dense_flash_ms"], "dense_flash_tflops": main_res["dense_flash_tflops"],
        "speedup_vs_dense": main_res["speedup_vs_dense"],
        "mfma_peak_frac_whole_path": main_res["effective_tflops"] * 1e12 / MFMA_BF16_PEAK,
        "roofline": {"kernel": "%s (stage 3, gathered sparse attention)" % main_res["stage3_kernel"], "bound": "mfma",
                     "achieved": flops3 / s3 / 1e12 if flops3 else 0.0, "peak": MFMA_BF16_PEAK / 1e12,
                     "unit": "TFLOP/s", "frac": flops3 / s3 / MFMA_BF16_PEAK if flops3 else 0.0, "traffic": traffic,
                     "hbm_achieved_GBps": (traffic / s3 / 1e9) if traffic else None,
                     "hbm_frac_of_peak": (traffic / s3 / HBM_PEAK) if traffic else None,
                     "sustained_mfma_TFLOPs_this_gpu": mfma_sustained / 1e12,
                     "frac_of_sustained_mfma": flops3 / s3 / mfma_sustained if flops3 else 0.0,
                     "sustained_copy_TBps_this_gpu": hbm_sustained / 1e12},
        "calibrated": calibrated,
        "peaked": peaked,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
