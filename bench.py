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
  roofline            : the dominant kernel of the primary workload against its roof, plus
                        `stages`: every stage against both roofs (MFMA rate over its
                        algorithmic FLOP, HBM rate over its compulsory bytes)
  dense_flash_ms      : the from-scratch dense causal flash kernel on the same GPU
  recall              : mean exp(lse_sparse - lse_dense), attention mass kept
  calibrated          : the same measurements (with their own `roofline`) with the planted
                        magnitudes in scaled-logit units (signal="logit"), the regime where the
                        threshold separates stripes from background
  peaked              : the same with the planted magnitudes times three and the threshold
                        scaled with them (signal="peaked"): the planted columns then hold most
                        of a row's attention mass, as in real heads, so high sparsity and high
                        recall occur together
  normalisers         : what this GPU sustains in the same run (register-only MFMA loop, 1 GiB
                        copies, the dense flash kernel): boxes of one pool differ by up to 10 %
  cpu_baseline        : the fp64 CPU oracle timed on a bounded sample of the same workload

`--workload varlen_mixed` times the packed batch of four sequences (16k / 48k / 96k / 128k tokens,
no planted structure: the low-sparsity worst case) and reports, besides the above, the imbalance of
the index lists and the index storage actually used.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15   # MI355X dense bf16, FLOP/s
HBM_PEAK = 8.0e12         # B/s


def kernel_sources_sha256():
    """Digest of the kernel sources of this tree: counter summaries under profiles/ carry the digest
    of the build they were measured on, and are quoted only when it is this one."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2505_23520_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def load_inputs(torch, synth, wl, signal, log=None):
    """Device tensors of the workload: [1, H, N, d] for one sequence, packed [H, total, d] plus
    cu_seqlens for several."""
    t0 = time.time()
    seqs = [synth.make_sequence(wl, s, signal=signal) for s in range(wl.B)]
    if wl.packed:
        import numpy as np
        qkv = tuple(torch.cat([torch.from_numpy(s[n]).to(torch.bfloat16) for s in seqs], 1).cuda()
                    for n in ("q", "k", "v"))
        cu = torch.from_numpy(np.concatenate([[0], np.cumsum(wl.seqlens)]).astype(np.int32)).cuda()
    else:
        qkv = tuple(torch.from_numpy(seqs[0][n]).to(torch.bfloat16)[None].cuda() for n in ("q", "k", "v"))
        cu = None
    if log:
        log("inputs %s/%s ready in %.1fs" % (wl.name, signal, time.time() - t0))
    return qkv, cu


def region_pairs(wl, step):
    """Per query head: (row, key) pairs of the anchor regions, of the (pooled row, candidate key)
    products of stage 2, and of dense causal attention; rows per group for the list pairs."""
    import numpy as np
    span = wl.block * step
    anchor = pooled = causal = 0
    rows_per_group = []
    for n in wl.seqlens:
        r = np.arange(n, dtype=np.int64)
        g = r // span
        W = np.maximum(wl.n_init, g * span - wl.window)
        anchor += int((np.minimum(wl.n_init, r + 1) + np.maximum(0, r - W + 1)).sum())
        nblk = (n + wl.block - 1) // wl.block
        gb = np.arange(nblk, dtype=np.int64) // step
        pooled += int((np.maximum(wl.n_init, gb * span - wl.window) - wl.n_init).sum())
        causal += n * (n + 1) // 2
        ng = (n + span - 1) // span
        rows_per_group.append([min(span, n - gi * span) for gi in range(ng)])
    return anchor, pooled, causal, rows_per_group


def list_analysis(torch, wl, sz, B, rows_per_group, grp):
    """From the device lists: list pairs of stage 3, distinct gathered K/V rows, padded entries,
    and the imbalance figures (per group and per sequence)."""
    Hq = wl.Hq
    counts = B["counts"].to(torch.int64).view(Hq, sz.grp_cap)
    offsets = B["offsets"][:-1].view(Hq, sz.grp_cap)
    rows = torch.tensor([r for seq in rows_per_group for r in seq], device="cuda", dtype=torch.int64)
    ngr = rows.numel()                                   # groups that exist (packed: grp_cap may be larger)
    counts = counts[:, :ngr]
    list_pairs = int((counts * rows[None, :]).sum())
    padded = (counts + 63) // 64 * 64
    # distinct (KV head, sequence, key) rows that some list names
    seq_of_group = torch.tensor([b for b, seq in enumerate(rows_per_group) for _ in seq], device="cuda")
    tok0 = torch.tensor([sum(wl.seqlens[:b]) for b in range(wl.B)], device="cuda", dtype=torch.int64)
    total_tok = sum(wl.seqlens)
    flat_counts = counts.reshape(-1)
    nent = int(flat_counts.sum())
    distinct = 0
    if nent:
        start = offsets[:, :ngr].reshape(-1)
        grp_id = torch.repeat_interleave(torch.arange(flat_counts.numel(), device="cuda"), flat_counts)
        first = torch.cumsum(flat_counts, 0) - flat_counts
        pos = start[grp_id] + (torch.arange(nent, device="cuda") - first[grp_id])
        keys = B["idx"][pos].to(torch.int64)
        hk = (grp_id // ngr) // grp
        sq = seq_of_group[grp_id % ngr]
        seen = torch.zeros(wl.Hkv * total_tok, dtype=torch.bool, device="cuda")
        seen[hk * total_tok + tok0[sq] + keys] = True
        distinct = int(seen.sum())
        del grp_id, first, pos, keys, hk, sq, seen
    per_seq, g0 = [], 0
    for b, seq in enumerate(rows_per_group):
        c = padded[:, g0:g0 + len(seq)].double()
        per_seq.append(dict(tokens=wl.seqlens[b], groups=len(seq), mean_list=float(c.mean()), max_list=float(c.max()),
                            entries=int(c.sum())))
        g0 += len(seq)
    pf = padded.double()
    imbalance = dict(
        mean_list_per_group=float(pf.mean()), max_list_per_group=float(pf.max()),
        max_over_mean_per_group=float(pf.max() / pf.mean()) if float(pf.mean()) else None,
        max_over_mean_per_sequence=(max(s["mean_list"] for s in per_seq) / (sum(s["entries"] for s in per_seq) /
                                    (Hq * ngr))) if nent else None,
        per_sequence=per_seq)
    return list_pairs, distinct, int(padded.sum()), imbalance


def stage_rooflines(wl, res, sustained):
    """Every stage against both roofs.  FLOP are algorithmic (what the method defines), bytes are
    compulsory (each tensor once): achieved rate = that / the stage's measured time."""
    d, Hq, Hkv = wl.d, wl.Hq, wl.Hkv
    tok = sum(wl.seqlens)
    nblk = sum((n + wl.block - 1) // wl.block for n in wl.seqlens)
    qb, kvb = Hq * tok * d * 2, Hkv * tok * d * 2
    acc, vec = Hq * tok * d * 4, Hq * tok * 4
    t1, t2, t3 = (res["stage_ms"][k] * 1e-3 for k in ("anchor", "select", "sparse"))
    idxb = 4 * res["padded_entries"]
    bits = res["groups"] * ((max(wl.seqlens) + 31) // 32) * 4
    f1 = 4.0 * d * res["anchor_pairs"]
    b1 = qb + 2 * kvb + acc + 2 * vec + Hq * nblk * 4
    f2 = 2.0 * d * res["pooled_pairs"]
    b2 = qb + kvb + 4 * Hq * nblk * d * 2 + 2 * bits + idxb
    f3 = 4.0 * d * res["stage3_list_pairs"]
    b3 = 2 * qb + acc + 3 * vec + idxb + res["distinct_gathered_rows"] * 2 * d * 2

    def entry(kernel, flop, nbytes, t, note):
        return dict(kernel=kernel, ms=t * 1e3, flop=flop, bytes=nbytes,
                    mfma_TFLOPs=flop / t / 1e12, mfma_frac=flop / t / MFMA_BF16_PEAK,
                    mfma_frac_of_sustained=flop / t / sustained["mfma"],
                    hbm_GBps=nbytes / t / 1e9, hbm_frac=nbytes / t / HBM_PEAK,
                    hbm_frac_of_sustained_copy=nbytes / t / sustained["copy"], note=note)

    return dict(
        anchor=entry("engine_bf16_kernel<anchor region, store state>", f1, b1, t1,
                     "FLOP = 4 d x anchor-region pairs; bytes = Q + K + V + Acc + M + L + pooled anchor"),
        select=entry("pool_q + mask_bf16 + count + scan + fill", f2, b2, t2,
                     "FLOP = 2 d x (pooled row, candidate key) pairs (the kernel issues up to twice that: "
                     "bf16 hi and lo parts of the pooled query); bytes = Q + K + pooled queries + bit words "
                     "(written, read) + index lists"),
        sparse=entry(res["stage3_kernel"] + "<list, load state, store out>", f3, b3, t3,
                     "FLOP = 4 d x list pairs; bytes = Q + O + Acc + M + L + lse + index lists + distinct "
                     "gathered K and V rows"))


def measure(api, torch, synth, wl, signal, step, steps, warmup, sustained, theta=None, dense_steps=2, log=None):
    cfg = api.Config(block=wl.block, n_init=wl.n_init, window=wl.window, step=step,
                     theta=wl.theta if theta is None else theta)
    (q, k, v), cu = load_inputs(torch, synth, wl, signal, log)
    out = torch.empty_like(q)
    pk = dict(cu_seqlens=cu, max_seqlen=max(wl.seqlens)) if wl.packed else {}
    p = api.make_params(cfg, q, k, v, out, **pk)
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
    del ws
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
    anchor_pairs, pooled_pairs, causal_pairs, rows_per_group = region_pairs(wl, step)
    list_pairs, distinct, padded_entries, imbalance = list_analysis(torch, wl, sz, B, rows_per_group, wl.Hq // wl.Hkv)
    assert wl.Hq * anchor_pairs + list_pairs == pairs, "attended pairs do not add up"
    sparse_lse = B["lse"].clone()
    # which of the two bf16 engines stage 3 ran in: the library decides on the device from the total
    # padded list length (mean list of 48 tiles of 64 entries per group or more: 256-row engine)
    total_padded = int(B["offsets"][-1])
    pair_engine = step % 2 == 0 and total_padded >= 48 * 64 * sz.groups
    del B
    torch.cuda.empty_cache()

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
    Hq, d = wl.Hq, wl.d
    res = dict(
        ms_per_layer=ms, attended_pairs=pairs, selected_entries=selected,
        sparsity=1.0 - pairs / (Hq * causal_pairs),
        effective_tflops=4.0 * d * pairs / (ms * 1e-3) / 1e12,
        stage_ms=dict(anchor=stage[0], select=stage[1], sparse=stage[2]),
        anchor_pairs=Hq * anchor_pairs, pooled_pairs=Hq * pooled_pairs, stage3_list_pairs=list_pairs,
        distinct_gathered_rows=distinct, padded_entries=padded_entries, groups=int(sz.groups),
        idx_bytes_used=4 * total_padded, idx_bytes_capacity=4 * int(sz.idx_capacity_max),
        list_imbalance=imbalance,
        stage3_kernel="engine_bf16_pp_kernel" if pair_engine else "engine_bf16_kernel",
        stage3_tflops=4.0 * d * list_pairs / (stage[2] * 1e-3) / 1e12 if list_pairs else 0.0,
        dense_flash_ms=dense_ms, dense_flash_tflops=4.0 * d * Hq * causal_pairs / (dense_ms * 1e-3) / 1e12,
        speedup_vs_dense=dense_ms / ms, recall=recall, theta=cfg.theta, step=step, signal=signal,
    )
    res["roofline"] = dict(stages=stage_rooflines(wl, res, sustained),
                           normalised_by="mfma_frac / hbm_frac: nominal peaks (2.5 PFLOP/s, 8 TB/s); *_of_sustained: "
                                         "the register-only MFMA loop and the 1 GiB copy of this run (`normalisers`)")
    if not wl.packed:
        del res["list_imbalance"]["per_sequence"]
    if log:
        log(json.dumps({k_: v_ for k_, v_ in res.items() if k_ not in ("roofline", "list_imbalance")}))
    return res, (q, k, v, cu, p)


def dense_per_sequence(api, torch, wl, q, k, v, steps=2):
    """Dense causal flash on each sequence of a packed batch by itself (views into the packed tensors)."""
    out = []
    off = 0
    for n in wl.seqlens:
        qs, ks, vs = (t[None, :, off:off + n] for t in (q, k, v))
        o = torch.empty((1, wl.Hq, n, wl.d), dtype=q.dtype, device="cuda")
        cfg = api.Config(block=wl.block, n_init=wl.n_init, window=wl.window, step=wl.step, theta=wl.theta)
        p = api.make_params(cfg, qs, ks, vs, o)
        api.dense_causal_flash(p, qs, ks, vs, o, None)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            api.dense_causal_flash(p, qs, ks, vs, o, None)
        e1.record()
        torch.cuda.synchronize()
        out.append(dict(tokens=n, dense_flash_ms=e0.elapsed_time(e1) / steps))
        off += n
    return out


def theta_sweep(api, torch, synth, wl, signal, step, steps, warmup, thetas, granularity=0, log=None):
    """Rows of (theta, anchor on/off) -> sparsity, recall, ms per layer of the fused entry point
    on one set of inputs: the columns of the paper's threshold ablation (Table 4)."""
    (q, k, v), _ = load_inputs(torch, synth, wl, signal, log)
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
    """Oracle (as it stands) on host cores, on whole (head 0, group) units of the workload's longest
    sequence: groups are taken from its end until about budget_s of CPU time is spent."""
    from oracle import anchor_oracle as ao
    b = max(range(wl.B), key=lambda i: wl.seqlens[i])
    N = wl.seqlens[b]
    span = wl.block * step
    seq = synth.make_sequence(wl, b, signal=signal, heads_kv=[0])
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
    return dict(seconds=time.time() - t0, pairs=pairs, groups=groups, cores=cores, seq=b)


def sustained_rates(api, torch, log):
    """Rates this GPU sustains at its actual clock: register-only MFMA loop, 1 GiB device copies
    (the copies are also the dispatches of known size that scale the FETCH_SIZE / WRITE_SIZE
    counters of a rocprofv3 --pmc run of this same command)."""
    from paper_2505_23520_amd import probe
    scratch = torch.empty(1 << 18, dtype=torch.float32, device="cuda")
    probe.mfma_probe(200, scratch)
    torch.cuda.synchronize()
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record()
    flop = probe.mfma_probe(10000, scratch)
    p1.record()
    torch.cuda.synchronize()
    mfma = flop / (p0.elapsed_time(p1) * 1e-3)
    cp_src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    torch.cuda.synchronize()
    p0.record()
    for _ in range(4):
        cp_dst.copy_(cp_src)
    p1.record()
    torch.cuda.synchronize()
    copy = 4 * 2 * cp_src.numel() * 4 / (p0.elapsed_time(p1) * 1e-3)
    del cp_src, cp_dst
    torch.cuda.empty_cache()
    log("sustained: MFMA %.0f TFLOP/s, copy %.2f TB/s" % (mfma / 1e12, copy / 1e12))
    return dict(mfma=mfma, copy=copy)


def counter_traffic(kernel, wl_name, signal):
    """HBM bytes per launch of the dominant kernel from the rocprofv3 --pmc summary under profiles/,
    quoted only if that summary was measured on a build of these same kernel sources."""
    path = os.path.join(ROOT, "profiles", "%s_stage3_%s_%s_traffic.txt" % (kernel.replace("_kernel", ""), wl_name, signal))
    prov = dict(source=os.path.relpath(path, ROOT), kernel_sources_sha256=kernel_sources_sha256())
    if not os.path.exists(path):
        return None, dict(prov, status="no counter summary for this kernel and workload")
    kv = dict(ln.strip().split("=", 1) for ln in open(path) if "=" in ln)
    prov.update(measured_on_sources=kv.get("kernel_sources_sha256"), measured=kv.get("measured"))
    if kv.get("kernel_sources_sha256") != prov["kernel_sources_sha256"]:
        return None, dict(prov, status="summary is from another build of the kernels: not quoted")
    return float(kv["traffic_bytes_per_launch"]), dict(prov, status="same kernel sources; another run of this command "
                                                       "under rocprofv3 --pmc, divided by this run's time")


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
    ap.add_argument("--theta-sweep", default=None, metavar="T1,T2,...|config",
                    help="instead of the benchmark line: one JSON object with sparsity / recall / ms per "
                         "threshold, with and without the anchor; `config` takes the workload's own list")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only (the path shards by heads with no exchange step; "
                 "this build has no multi-GPU code): run with --gpus 1")

    import torch
    from paper_2505_23520_amd import api, synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = synth.workloads()[args.workload]
    if wl.dtype != "bf16":
        sys.exit("bench.py times the bf16 workloads (gqa_8k, gqa_32k, gqa_128k, varlen_mixed); "
                 "the tiny fp32 workload is a parity-test case")
    log = lambda s: print("[bench] " + s, file=sys.stderr, flush=True)

    if args.theta_sweep:
        if wl.packed:
            sys.exit("--theta-sweep runs on the single-sequence workloads")
        thetas = wl.extra["theta_sweep"] if args.theta_sweep == "config" else [float(t) for t in args.theta_sweep.split(",")]
        print(json.dumps(theta_sweep(api, torch, synth, wl, args.signal, args.step, args.steps, args.warmup,
                                     thetas, granularity=["stripe", "block"].index(args.granularity), log=log)),
              flush=True)
        return

    sustained = sustained_rates(api, torch, log)
    main_res, tensors = measure(api, torch, synth, wl, args.signal, args.step, args.steps, args.warmup, sustained, log=log)
    per_seq_dense = None
    if wl.packed:
        per_seq_dense = dense_per_sequence(api, torch, wl, *tensors[:3])
        for row, extra in zip(main_res["list_imbalance"]["per_sequence"], per_seq_dense):
            row.update(extra)
    del tensors
    torch.cuda.empty_cache()
    calibrated, peaked = None, None
    if not args.no_calibrated and args.signal == "literal" and not wl.packed:
        calibrated, t2 = measure(api, torch, synth, wl, "logit", args.step, args.steps, args.warmup, sustained, log=log)
        del t2
        torch.cuda.empty_cache()
        # planted magnitudes times three, threshold scaled with them
        peaked, t2 = measure(api, torch, synth, wl, "peaked", args.step, args.steps, args.warmup, sustained,
                             theta=3.0 * wl.theta, log=log)
        del t2
        torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu:
        c = cpu_baseline(synth, wl, args.step, args.signal)
        layer_ms = c["seconds"] * 1e3 * main_res["attended_pairs"] / max(1, c["pairs"])
        cpu = dict(value=layer_ms, unit="ms/layer (sample time scaled by attended pairs)", cores=c["cores"],
                   kind="oracle",
                   sample="query head 0, groups %d..%d (%d rows each) of sequence %d (%d tokens) of %s: %.1f s for %.3g pairs" % (
                       c["groups"][-1], c["groups"][0], wl.block * args.step, c["seq"], wl.seqlens[c["seq"]], wl.name,
                       c["seconds"], c["pairs"]))
        log(json.dumps(cpu))

    d = wl.d
    traffic, provenance = counter_traffic(main_res["stage3_kernel"], wl.name, args.signal)
    s3 = main_res["stage_ms"]["sparse"] * 1e-3
    flops3 = 4.0 * d * main_res["stage3_list_pairs"]
    shape = ("B=%d packed, lengths %s" % (wl.B, "/".join(map(str, wl.seqlens)))) if wl.packed else "B=1, N=%d" % wl.seqlens[0]
    line = {
        "metric": "prefill attention ms/layer at 128k GQA32/8 d128 bf16 (effective TFLOPS over attended pairs, recall alongside)",
        "value": main_res["ms_per_layer"], "unit": "ms/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_res["ms_per_layer"], "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s (%s, Hq=%d, Hkv=%d, d=%d, block %d, n_init %d, window %d, step %d, theta %.4f, signal %s)" % (
            wl.name, shape, wl.Hq, wl.Hkv, d, wl.block, wl.n_init, wl.window, args.step, wl.theta, args.signal)},
        "effective_tflops": main_res["effective_tflops"], "sparsity": main_res["sparsity"],
        "recall": main_res["recall"], "stage_ms": main_res["stage_ms"],
        "dense_flash_ms": main_res["dense_flash_ms"], "dense_flash_tflops": main_res["dense_flash_tflops"],
        "speedup_vs_dense": main_res["speedup_vs_dense"],
        "mfma_peak_frac_whole_path": main_res["effective_tflops"] * 1e12 / MFMA_BF16_PEAK,
        "roofline": {"kernel": "%s (stage 3, gathered sparse attention)" % main_res["stage3_kernel"], "bound": "mfma",
                     "achieved": flops3 / s3 / 1e12 if flops3 else 0.0, "peak": MFMA_BF16_PEAK / 1e12,
                     "unit": "TFLOP/s", "frac": flops3 / s3 / MFMA_BF16_PEAK if flops3 else 0.0, "traffic": traffic,
                     "traffic_provenance": provenance,
                     "hbm_achieved_GBps": (traffic / s3 / 1e9) if traffic else None,
                     "hbm_frac_of_peak": (traffic / s3 / HBM_PEAK) if traffic else None,
                     "frac_of_sustained_mfma": flops3 / s3 / sustained["mfma"] if flops3 else 0.0,
                     "stages": main_res["roofline"]["stages"],
                     "normalised_by": main_res["roofline"]["normalised_by"]},
        "normalisers": {"sustained_mfma_TFLOPs_this_gpu": sustained["mfma"] / 1e12,
                        "sustained_copy_TBps_this_gpu": sustained["copy"] / 1e12,
                        "dense_flash_ms_this_gpu": main_res["dense_flash_ms"],
                        "note": "GPUs of one pool differ by up to 10 % at the same build: compare runs through the "
                                "ratio to these, measured in this same run"},
        "lists": {k_: main_res[k_] for k_ in ("selected_entries", "padded_entries", "idx_bytes_used", "idx_bytes_capacity",
                                              "distinct_gathered_rows", "list_imbalance")},
        "calibrated": calibrated,
        "peaked": peaked,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
