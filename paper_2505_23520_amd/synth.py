"""Seeded synthetic Q/K/V for the AnchorAttention prefill workloads.

This module only draws inputs.  It contains none of the method's arithmetic
(no scores, no softmax, no selection) and is the one piece shared by the GPU
tests, the benchmark and the CPU oracle's tests.

The inputs stand in for the activations the paper measures on (an 8B-class GQA
model, 32 query / 8 KV heads, d=128, on 8k...128k-token prompts, Section 4.1):
i.i.d. N(0,1) entries plus the structure the paper reports for real heads
(Section 2.2) -- an attention sink on the first keys and a sparse set of
"stripe" key columns that many queries attend to -- planted along one unit
direction per KV head.

``signal`` chooses the unit of the planted magnitudes:
  * "literal": a planted key gets  m * u  and queries get  u  (|u| = 1), as the
    workload descriptions are worded.  The scaled logit moves by only m/sqrt(d).
  * "logit":   keys get m * d**0.25 * u and queries d**0.25 * u, so the scaled
    logit q.k/sqrt(d) moves by m.  This is the regime in which the threshold
    separates stripes from background (the paper's 89-97 % sparsity range).
  * "peaked":  as "logit" with every planted magnitude (stripes and sink) times
    three.  With i.i.d. Gaussian background keys a 128k-token row spreads about
    N * e^(1/2) of softmax mass over ordinary columns; only at these magnitudes
    do the planted columns hold most of a row's mass, as the stripes and sinks
    of real heads do (Section 2.2), so that recall near one and high sparsity
    can occur together.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Workload:
    name: str
    dtype: str              # "fp32" | "bf16"
    seqlens: tuple          # one entry per sequence (B = len)
    Hq: int
    Hkv: int
    d: int
    block: int              # b_q = b_kv
    n_init: int
    window: int
    step: int
    theta: float
    seed: int
    n_planted: int = 0      # planted stripe columns per KV head and sequence
    planted_mag: tuple = (0.0, 0.0)   # (lo, hi): magnitude ~ U(lo, hi); lo == hi -> constant
    sink_keys: int = 0      # keys 0..sink_keys-1 get sink_mag * u
    sink_mag: float = 0.0
    q_shift: bool = True    # add u to every query of the KV group
    ar1: float = 0.0        # AR(1) coefficient along the sequence for query rows
    extra: dict = field(default_factory=dict)

    @property
    def B(self):
        return len(self.seqlens)

    @property
    def packed(self):
        return len(self.seqlens) > 1


LN = np.log


def workloads() -> dict:
    """The five workload recipes (tiny fp32; 8k / 32k / 128k bf16 GQA; packed mixed lengths)."""
    return {
        "tiny_fp32": Workload("tiny_fp32", "fp32", (1024,), 1, 1, 64, 64, 16, 64, 1, float(LN(16.0)), 0,
                              n_planted=8, planted_mag=(3.0, 3.0)),
        "gqa_8k": Workload("gqa_8k", "bf16", (8192,), 32, 8, 128, 128, 128, 128, 16, float(LN(32.0)), 1,
                           n_planted=64, planted_mag=(2.5, 2.5), sink_keys=4, sink_mag=4.0),
        "gqa_32k": Workload("gqa_32k", "bf16", (32768,), 32, 8, 128, 128, 128, 128, 16, float(LN(32.0)), 2,
                            n_planted=256, planted_mag=(2.5, 2.5), sink_keys=4, sink_mag=4.0, ar1=0.3,
                            extra={"theta_sweep": [float(LN(8.0)), float(LN(32.0)), float(LN(128.0))]}),
        "gqa_128k": Workload("gqa_128k", "bf16", (131072,), 32, 8, 128, 128, 128, 128, 16, float(LN(32.0)), 3,
                             n_planted=1024, planted_mag=(1.5, 3.5), sink_keys=4, sink_mag=4.0),
        "varlen_mixed": Workload("varlen_mixed", "bf16", (16384, 49152, 98304, 131072), 32, 8, 128, 128, 128,
                                 128, 16, float(LN(32.0)), 4, q_shift=False),
    }


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def make_sequence(wl: Workload, seq: int, N: int | None = None, signal: str = "literal",
                  heads_kv=None) -> dict:
    """Q [Hq', N, d], K, V [Hkv', N, d] float32 for sequence ``seq`` of the workload.

    ``heads_kv`` restricts generation to some KV heads (and their query heads),
    with exactly the values the full tensor would hold: every (sequence, KV head)
    has its own random stream.  ``N`` overrides the length (shorter parity cases
    of the same recipe).  Values are bf16-representable when wl.dtype == "bf16".
    """
    if signal not in ("literal", "logit", "peaked"):
        raise ValueError("signal must be 'literal', 'logit' or 'peaked'")
    N = int(wl.seqlens[seq] if N is None else N)
    d, grp = wl.d, wl.Hq // wl.Hkv
    hk_list = list(range(wl.Hkv)) if heads_kv is None else list(heads_kv)
    amp = 1.0 if signal == "literal" else float(d) ** 0.25
    gain = 3.0 if signal == "peaked" else 1.0       # on the planted magnitudes
    Q = np.empty((len(hk_list) * grp, N, d), np.float32)
    K = np.empty((len(hk_list), N, d), np.float32)
    V = np.empty((len(hk_list), N, d), np.float32)
    planted = []
    for a, hk in enumerate(hk_list):
        rng = np.random.default_rng([wl.seed, seq, hk])
        u = rng.standard_normal(d)
        u /= np.linalg.norm(u)
        k = rng.standard_normal((N, d), dtype=np.float32)
        v = rng.standard_normal((N, d), dtype=np.float32)
        cols = np.sort(rng.choice(N, size=min(wl.n_planted, N), replace=False)) if wl.n_planted else np.empty(0, int)
        lo, hi = wl.planted_mag
        mags = rng.uniform(lo, hi, size=cols.size) if hi > lo else np.full(cols.size, lo)
        if cols.size:
            k[cols] += (amp * gain * mags[:, None] * u[None, :]).astype(np.float32)
        if wl.sink_keys:
            k[: wl.sink_keys] += (amp * gain * wl.sink_mag * u).astype(np.float32)
        planted.append((cols, mags))
        for t in range(grp):
            qh = rng.standard_normal((N, d), dtype=np.float32)
            if wl.ar1:
                rho, c = np.float32(wl.ar1), np.float32(np.sqrt(1.0 - wl.ar1 ** 2))
                for r in range(1, N):
                    qh[r] = rho * qh[r - 1] + c * qh[r]
            if wl.q_shift and (wl.n_planted or wl.sink_keys):
                qh += (amp * u).astype(np.float32)
            Q[a * grp + t] = qh
        K[a], V[a] = k, v
    if wl.dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    return dict(q=Q, k=K, v=V, planted=planted, N=N, heads_kv=hk_list)
