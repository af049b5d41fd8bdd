"""Shared GPU-vs-oracle comparison used by the gpu tests, the smoke check and the benchmark.

The GPU side goes through the C ABI binding only; the expected values come from
``oracle/`` only.  Inputs are the seeded synthetic tensors of ``synth``.
"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch

from oracle import anchor_oracle as ao

BAND = 1e-3        # selection may differ only where |xbar - s - theta| <= BAND
ENGINE = None      # a test fixture may force one of the two bf16 tile engines for every DeviceRun


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)          # exact: values are already bf16-representable
    return t.cuda()


class DeviceRun:
    """Runs the stage-wise entry points and the fused one on a batch of sequences."""

    def __init__(self, api, seqs, cfg, dtype, packed=None, want_acc=True):
        if ENGINE is not None and cfg.engine == 0:
            cfg = dataclasses.replace(cfg, engine=ENGINE)
        self.api, self.cfg, self.dtype = api, cfg, dtype
        self.seqs = seqs
        self.lens = [s["q"].shape[1] for s in seqs]
        self.packed = (len(seqs) > 1 and len(set(self.lens)) > 1) if packed is None else packed
        Hq, d = seqs[0]["q"].shape[0], seqs[0]["q"].shape[2]
        self.Hq, self.Hkv, self.d = Hq, seqs[0]["k"].shape[0], d
        if self.packed:
            self.q = to_device(np.concatenate([s["q"] for s in seqs], 1), dtype)
            self.k = to_device(np.concatenate([s["k"] for s in seqs], 1), dtype)
            self.v = to_device(np.concatenate([s["v"] for s in seqs], 1), dtype)
            cu = np.concatenate([[0], np.cumsum(self.lens)]).astype(np.int32)
            self.cu_host = cu
            self.cu = torch.from_numpy(cu).cuda()
            self.out = torch.zeros_like(self.q)
            self.p = api.make_params(cfg, self.q, self.k, self.v, self.out, cu_seqlens=self.cu,
                                     max_seqlen=max(self.lens))
        else:
            self.q = to_device(np.stack([s["q"] for s in seqs]), dtype)
            self.k = to_device(np.stack([s["k"] for s in seqs]), dtype)
            self.v = to_device(np.stack([s["v"] for s in seqs]), dtype)
            self.cu_host = None
            self.out = torch.zeros_like(self.q)
            self.p = api.make_params(cfg, self.q, self.k, self.v, self.out)
        self.buf = api.alloc_stage_buffers(self.p, want_acc=want_acc)
        self.sizes = self.buf["sizes"]

    # ---- index helpers mirroring the layouts documented in include/anchor_attention.h
    def row_index(self, b, h, r):
        if self.packed:
            return h * int(self.p.total_tokens) + int(self.cu_host[b]) + r
        return (b * self.Hq + h) * self.lens[0] + r

    def blk_index(self, b, h, i):
        bq = self.cfg.block
        if self.packed:
            base = sum((n + bq - 1) // bq for n in self.lens[:b])
            return h * self.sizes.blk_cap + base + i
        return (b * self.Hq + h) * self.sizes.blk_cap + i

    def grp_index(self, b, h, g):
        span = self.cfg.block * self.cfg.step
        if self.packed:
            base = sum((n + span - 1) // span for n in self.lens[:b])
            return h * self.sizes.grp_cap + base + g
        return (b * self.Hq + h) * self.sizes.grp_cap + g

    def out_rows(self, out, b, h, r0, r1):
        if self.packed:
            o = int(self.cu_host[b])
            return out[h, o + r0:o + r1]
        return out[b, h, r0:r1]

    def acc_rows(self, b, h, g, nrows):
        """Acc of group g's rows as float64 [nrows, d], from the layout include/anchor_attention.h documents."""
        d, A = self.d, self.buf["Acc"]
        if self.dtype != "bf16":
            ri0 = self.row_index(b, h, g * self.cfg.block * self.cfg.step)
            return A[ri0 * d:(ri0 + nrows) * d].cpu().numpy().astype(np.float64).reshape(-1, d)
        nb = (nrows + 127) // 128
        bi0 = self.blk_index(b, h, g * self.cfg.step)
        slabs = A[bi0 * 16384:(bi0 + nb) * 16384].cpu().numpy().astype(np.float64)
        # [block, tile w, column block c/32, (c%32)/8, (c%8)/4, row n, c%4] -> [block, w, n, columns]
        t = slabs.reshape(nb, 4, 4, 4, 2, 32, 4).transpose(0, 1, 5, 2, 3, 4, 6)
        return t.reshape(nb * 128, 128)[:nrows]

    # ---- GPU calls
    def stages(self):
        api, p, B = self.api, self.p, self.buf
        api.anchor_compute(p, self.q, self.k, self.v, B["M"], B["L"], B["Acc"], B["xa"])
        api.stripe_select(p, self.q, self.k, B["xa"], B["counts"], B["offsets"], B["idx"], B["flag"], B["ws"])
        api.sparse_attn(p, self.q, self.k, self.v, B["M"], B["L"], B["Acc"], B["counts"], B["offsets"],
                        B["idx"], self.out, B["lse"])
        torch.cuda.synchronize()
        return self

    def fused(self):
        api, p = self.api, self.p
        ws = torch.empty(self.sizes.prefill_ws_bytes, dtype=torch.uint8, device="cuda")
        out = torch.zeros_like(self.q)
        lse = torch.empty(self.sizes.rows, dtype=torch.float32, device="cuda")
        stats = torch.zeros(4, dtype=torch.int64, device="cuda")
        api.anchor_attention_prefill(p, self.q, self.k, self.v, out, lse, stats, ws)
        torch.cuda.synchronize()
        return out, lse, stats.cpu().numpy()

    def dense(self):
        out = torch.zeros_like(self.q)
        lse = torch.empty(self.sizes.rows, dtype=torch.float32, device="cuda")
        self.api.dense_causal_flash(self.p, self.q, self.k, self.v, out, lse)
        torch.cuda.synchronize()
        return out, lse

    def group_list(self, b, h, g):
        t = self.grp_index(b, h, g)
        c = int(self.buf["counts"][t])
        o = int(self.buf["offsets"][t])
        return self.buf["idx"][o:o + c].cpu().numpy().astype(np.int64), o, c


def oracle_params(cfg, d):
    return ao.OracleParams(b_q=cfg.block, n_init=cfg.n_init, w=cfg.window, step=cfg.step,
                           theta=float(cfg.theta), sigma=(cfg.softmax_scale or None),
                           b_kv=cfg.block if getattr(cfg, "granularity", 0) == 1 else 0)


def tolerances(dtype):
    if dtype == "fp32":
        return dict(M=2e-5, L=2e-5, accn=1e-5, xa=2e-5, O=1e-5, lse=2e-5)
    return dict(M=2e-4, L=4e-3, accn=2e-2, xa=2e-4, O=2e-2, lse=4e-3)


def check_groups(run: DeviceRun, samples, check_state=True, out=None, lse=None):
    """Compare GPU results with the oracle for (b, h, g) samples.  Returns summary stats."""
    cfg, d, tol = run.cfg, run.d, tolerances(run.dtype)
    op = oracle_params(cfg, d)
    grp = run.Hq // run.Hkv
    out = run.out if out is None else out
    lse = run.buf["lse"] if lse is None else lse
    M_all, L_all, xa_all = run.buf["M"], run.buf["L"], run.buf["xa"]
    worst = dict(M=0.0, L=0.0, accn=0.0, xa=0.0, O=0.0, lse=0.0, band_diffs=0, selected=0, candidates=0)
    for (b, h, g) in samples:
        s = run.seqs[b]
        q, k, v = s["q"][h], s["k"][h // grp], s["v"][h // grp]
        N = q.shape[0]
        ref = ao.run_group(q, k, v, op, g, want_acc=check_state, attend=False, zero_anchor=not cfg.use_anchor)
        r0, r1 = ref["rows"]
        ri0 = run.row_index(b, h, r0)
        if check_state:
            Mg = M_all[ri0:ri0 + (r1 - r0)].cpu().numpy().astype(np.float64)
            Lg = L_all[ri0:ri0 + (r1 - r0)].cpu().numpy().astype(np.float64)
            worst["M"] = max(worst["M"], np.abs(Mg - ref["M"]).max())
            worst["L"] = max(worst["L"], (np.abs(Lg - ref["L"]) / ref["L"]).max())
            if run.buf["Acc"] is not None:
                Ag = run.acc_rows(b, h, g, r1 - r0)
                worst["accn"] = max(worst["accn"], np.abs(Ag / Lg[:, None] - ref["Acc"] / ref["L"][:, None]).max())
            nb = ref["xbar"].size
            bi0 = run.blk_index(b, h, g * cfg.step)
            xg = xa_all[bi0:bi0 + nb].cpu().numpy().astype(np.float64)
            worst["xa"] = max(worst["xa"], np.abs(xg - ref["xbar"]).max())
        # ---- stage 2: sets bit-exact outside the band
        lst, off, cnt = run.group_list(b, h, g)
        assert off % 64 == 0
        assert np.all(np.diff(lst) > 0), "list not strictly ascending"
        assert lst.size == 0 or (lst[0] >= cfg.n_init and lst[-1] < ref["W"])
        gsel = np.zeros(N, np.uint8)
        gsel[lst] = 1
        diff = np.nonzero(gsel != ref["sel"])[0]
        if diff.size:
            bad = diff[np.abs(ref["margin"][diff]) > BAND]
            assert bad.size == 0, "selection differs outside the band at columns %s (margins %s)" % (
                bad[:8], ref["margin"][bad[:8]])
        worst["band_diffs"] += int(diff.size)
        worst["selected"] += int(cnt)
        worst["candidates"] += max(0, ref["W"] - cfg.n_init)
        if cnt % 64:                                   # padding repeats the last entry
            pad = run.buf["idx"][off + cnt: off + (cnt + 63) // 64 * 64].cpu().numpy()
            assert np.all(pad == lst[-1])
        # ---- stage 3 against the oracle on the GPU's own (verified) set
        att = ao.attend_group(q, k, v, op, g, gsel)
        Og = run.out_rows(out, b, h, r0, r1).float().cpu().numpy().astype(np.float64)
        worst["O"] = max(worst["O"], np.abs(Og - att["O"]).max())
        lg = lse[ri0:ri0 + (r1 - r0)].cpu().numpy().astype(np.float64)
        worst["lse"] = max(worst["lse"], np.abs(lg - att["lse"]).max())
    for key in ("M", "L", "accn", "xa", "O", "lse"):
        assert worst[key] <= tol[key], "%s error %.3e exceeds %.1e (%s)" % (key, worst[key], tol[key], worst)
    return worst
