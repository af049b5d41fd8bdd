"""Python face of the fp64 CPU oracle -- TEST INFRASTRUCTURE ONLY.

Loads ``anchor_oracle.c`` (compiled with gcc into ``libanchor_oracle.so`` next
to this file) and walks it over batches, GQA heads and groups.  Only
``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this module; the GPU library never does, and this module never imports
the GPU package.

The per-head pipeline follows arXiv 2505.23520 Section 3 / Algorithms 1-3:
anchor state -> block pooling -> difference-aware selection -> attention over
anchor region plus selected columns.  Heads are independent; query head h reads
KV head h // (Hq // Hkv).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "anchor_oracle.c")
_LIB = os.path.join(_HERE, "libanchor_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (strict IEEE arithmetic, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("N", ctypes.c_int64),
        ("d", ctypes.c_int32),
        ("b_q", ctypes.c_int32),
        ("n_init", ctypes.c_int32),
        ("w", ctypes.c_int32),
        ("step", ctypes.c_int32),
        ("sigma", ctypes.c_double),
        ("theta", ctypes.c_double),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        # ANCHOR_ORACLE_LIB: a library built elsewhere from (a copy of) anchor_oracle.c; the test that
        # checks that the pins notice planted mistakes loads its altered copies this way
        lib = ctypes.CDLL(os.environ.get("ANCHOR_ORACLE_LIB") or build())
        P = ctypes.c_void_p
        I64 = ctypes.c_int64
        lib.ao_window_start.restype = I64
        lib.ao_window_start.argtypes = [P, I64]
        lib.ao_anchor_rows.restype = None
        lib.ao_anchor_rows.argtypes = [P, P, P, P, I64, I64, P, P, P]
        lib.ao_pool_block.restype = None
        lib.ao_pool_block.argtypes = [P, P, P, I64, P, P]
        lib.ao_select_group.restype = I64
        lib.ao_select_group.argtypes = [P, P, I64, ctypes.c_int, P, P, P, P]
        lib.ao_select_group_blocks.restype = I64
        lib.ao_select_group_blocks.argtypes = [P, P, I64, ctypes.c_int, P, P, ctypes.c_int32, P, P]
        lib.ao_attend_rows.restype = I64
        lib.ao_attend_rows.argtypes = [P, P, P, P, I64, I64, P, P, P]
        _lib = lib
    return _lib


@dataclass
class OracleParams:
    """Method parameters (Alg. 1-3 REQUIRE lines), token units."""

    b_q: int
    n_init: int
    w: int
    step: int
    theta: float
    sigma: float | None = None  # None -> 1/sqrt(d)
    b_kv: int = 0               # 0: stripe granularity (b_q, 1); > 0: block granularity (b_q, b_kv)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _cfg(N: int, d: int, p: OracleParams) -> _Cfg:
    sigma = p.sigma if p.sigma is not None else 1.0 / np.sqrt(float(d))
    return _Cfg(N, d, p.b_q, p.n_init, p.w, p.step, float(sigma), float(p.theta))


def window_start(N: int, d: int, p: OracleParams, g: int) -> int:
    c = _cfg(N, d, p)
    return int(_load().ao_window_start(ctypes.byref(c), g))


def n_groups(N: int, p: OracleParams) -> int:
    span = p.b_q * p.step
    return (N + span - 1) // span


def run_group(q, k, v, p: OracleParams, g: int, want_acc: bool = False, attend: bool = True,
              zero_anchor: bool = False):
    """Whole pipeline for group ``g`` of one head.  q,k,v: float32 [N,d], C order.

    Returns a dict: rows (r0,r1), M, L, (Acc), xbar[nb], qbar[nb,d], sel (uint8[N]),
    margin (float64[N]), idx (ascending int64), O, lse, pairs.
    p.b_kv > 0 switches the selection to block granularity (one decision per key block).
    zero_anchor: selection compares against an anchor of zero (the "Without Anchor" rows of
    Table 4); M, L, Acc and xbar are still the true anchor state.
    """
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float32)
    k = np.ascontiguousarray(k, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    N, d = q.shape
    c = _cfg(N, d, p)
    cp = ctypes.byref(c)
    span = p.b_q * p.step
    r0, r1 = g * span, min(N, (g + 1) * span)
    n = r1 - r0
    M = np.empty(n, np.float64)
    L = np.empty(n, np.float64)
    Acc = np.empty((n, d), np.float64) if want_acc else None
    lib.ao_anchor_rows(cp, _ptr(q), _ptr(k), _ptr(v), r0, r1, _ptr(M), _ptr(L), _ptr(Acc))
    nb = (n + p.b_q - 1) // p.b_q
    xbar = np.empty(nb, np.float64)
    qbar = np.empty((nb, d), np.float64)
    for b in range(nb):
        i = g * p.step + b
        xb = ctypes.c_double()
        lib.ao_pool_block(cp, _ptr(q), _ptr(M[b * p.b_q:]), i, ctypes.byref(xb), _ptr(qbar[b]))
        xbar[b] = xb.value
    sel = np.empty(N, np.uint8)
    margin = np.empty(N, np.float64)
    xsel = np.zeros_like(xbar) if zero_anchor else xbar
    if p.b_kv:
        cnt = lib.ao_select_group_blocks(cp, _ptr(k), g, nb, _ptr(xsel), _ptr(qbar), p.b_kv, _ptr(sel), _ptr(margin))
        if cnt < 0:
            raise ValueError("block granularity needs n_init and the window start to be multiples of b_kv")
    else:
        cnt = lib.ao_select_group(cp, _ptr(k), g, nb, _ptr(xsel), _ptr(qbar), _ptr(sel), _ptr(margin))
    idx = np.nonzero(sel)[0].astype(np.int64)
    assert cnt == idx.size
    out = dict(rows=(r0, r1), M=M, L=L, Acc=Acc, xbar=xbar, qbar=qbar, sel=sel, margin=margin,
               idx=idx, W=window_start(N, d, p, g))
    if attend:
        O = np.empty((n, d), np.float64)
        lse = np.empty(n, np.float64)
        pairs = lib.ao_attend_rows(cp, _ptr(q), _ptr(k), _ptr(v), r0, r1, _ptr(sel), _ptr(O), _ptr(lse))
        out.update(O=O, lse=lse, pairs=int(pairs))
    return out


def run_head(q, k, v, p: OracleParams, groups=None, want_acc: bool = False, attend: bool = True):
    """Pipeline over the listed groups (default: all) of one head; concatenates rows."""
    N = q.shape[0]
    gs = list(range(n_groups(N, p))) if groups is None else list(groups)
    res = [run_group(q, k, v, p, g, want_acc=want_acc, attend=attend) for g in gs]
    out = dict(groups=gs, per_group=res)
    if groups is None and res:
        out["M"] = np.concatenate([r["M"] for r in res])
        out["L"] = np.concatenate([r["L"] for r in res])
        out["xbar"] = np.concatenate([r["xbar"] for r in res])
        out["qbar"] = np.concatenate([r["qbar"] for r in res])
        if want_acc:
            out["Acc"] = np.concatenate([r["Acc"] for r in res])
        if attend:
            out["O"] = np.concatenate([r["O"] for r in res])
            out["lse"] = np.concatenate([r["lse"] for r in res])
            out["pairs"] = sum(r["pairs"] for r in res)
    return out


def dense_params(b_q: int) -> OracleParams:
    """theta=+inf: every candidate is selected, so P(r) = [0, r] (dense causal attention)."""
    return OracleParams(b_q=b_q, n_init=0, w=0, step=1, theta=float("inf"))


def attend_group(q, k, v, p: OracleParams, g: int, sel: np.ndarray):
    """Attention of group ``g``'s rows over A(r) plus the columns marked in ``sel`` (uint8[N])."""
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float32)
    k = np.ascontiguousarray(k, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    N, d = q.shape
    c = _cfg(N, d, p)
    span = p.b_q * p.step
    r0, r1 = g * span, min(N, (g + 1) * span)
    sel = np.ascontiguousarray(sel, dtype=np.uint8)
    assert sel.shape == (N,)
    O = np.empty((r1 - r0, d), np.float64)
    lse = np.empty(r1 - r0, np.float64)
    pairs = lib.ao_attend_rows(ctypes.byref(c), _ptr(q), _ptr(k), _ptr(v), r0, r1, _ptr(sel), _ptr(O), _ptr(lse))
    return dict(rows=(r0, r1), O=O, lse=lse, pairs=int(pairs))
