"""Thin ctypes binding over libanchor_attention.so (see include/anchor_attention.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
torch supplies device memory and the stream.  Importing this module fails if
the library has not been built (run ``python -m paper_2505_23520_amd.build``
or ``__graft_entry__.build()``); there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import math
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libanchor_attention.so")

AA_FP32, AA_BF16 = 0, 1
AA_STRIPE, AA_BLOCK = 0, 1
AA_ENGINE_AUTO, AA_ENGINE_128, AA_ENGINE_256 = 0, 1, 2
AA_OK, AA_EINVAL, AA_EUNSUPPORTED, AA_EWORKSPACE, AA_EHIP = 0, -1, -2, -3, -4


class aa_params(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("N", ctypes.c_int32), ("d", ctypes.c_int32),
        ("block_q", ctypes.c_int32), ("block_kv", ctypes.c_int32),
        ("n_init", ctypes.c_int32), ("window", ctypes.c_int32), ("step", ctypes.c_int32),
        ("theta", ctypes.c_float), ("softmax_scale", ctypes.c_float),
        ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32), ("use_anchor", ctypes.c_int32),
        ("granularity", ctypes.c_int32), ("engine", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
        ("v_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3),
        ("cu_seqlens", ctypes.c_void_p), ("total_tokens", ctypes.c_int64),
    ]


class aa_sizes(ctypes.Structure):
    _fields_ = [
        ("rows", ctypes.c_int64), ("acc_elems", ctypes.c_int64), ("blk_cap", ctypes.c_int64),
        ("blocks", ctypes.c_int64), ("grp_cap", ctypes.c_int64), ("groups", ctypes.c_int64),
        ("idx_capacity_max", ctypes.c_int64),
        ("select_ws_bytes", ctypes.c_size_t), ("prefill_ws_bytes", ctypes.c_size_t),
    ]


_P = ctypes.c_void_p
_PP = ctypes.POINTER(aa_params)
_SIGNATURES = {
    "anchor_sizes": (ctypes.c_int, [_PP, ctypes.POINTER(aa_sizes)]),
    "anchor_workspace_bytes": (ctypes.c_int, [_PP, ctypes.POINTER(ctypes.c_size_t)]),
    "anchor_compute": (ctypes.c_int, [_PP, _P, _P, _P, _P, _P, _P, _P, _P]),
    "stripe_select": (ctypes.c_int, [_PP, _P, _P, _P, _P, _P, _P, ctypes.c_int64, _P, _P, ctypes.c_size_t, _P]),
    "stripe_select_noalloc": (ctypes.c_int, [_PP, _P, _P, _P, _P, _P, _P, ctypes.c_int64, _P, _P]),
    "sparse_attn": (ctypes.c_int, [_PP, _P, _P, _P, _P, _P, _P, _P, _P, _P, ctypes.c_int64, _P, _P, _P]),
    "anchor_attention_prefill": (ctypes.c_int, [_PP, _P, _P, _P, _P, _P, _P, _P, ctypes.c_size_t, _P]),
    "dense_causal_flash": (ctypes.c_int, [_PP, _P, _P, _P, _P, _P, _P]),
    "anchor_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "anchor_last_hip_error": (ctypes.c_char_p, []),
}
EXPORTS = tuple(_SIGNATURES)


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    """dlopen the built library and declare its signatures; ImportError if it is not there."""
    if not os.path.exists(path):
        raise ImportError(
            "libanchor_attention.so is not built (%s). Build it with "
            "`python -m paper_2505_23520_amd.build`; there is no fallback path." % path)
    lib = ctypes.CDLL(path)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = load_library()


class AnchorError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        msg = _lib.anchor_strerror(code).decode()
        if code == AA_EHIP:
            msg += ": " + _lib.anchor_last_hip_error().decode()
        super().__init__("anchor_attention error %d (%s)" % (code, msg))


def _check(rc: int):
    if rc != AA_OK:
        raise AnchorError(rc)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


@dataclass
class Config:
    """Method parameters (Algorithms 1-3 REQUIRE lines), token units."""
    block: int = 128
    n_init: int = 128
    window: int = 128
    step: int = 16
    theta: float = 12.0
    softmax_scale: float = 0.0
    use_anchor: bool = True
    causal: bool = True
    granularity: int = AA_STRIPE     # AA_BLOCK: one decision per key block (Sec. 2.1.2, Table 1)
    engine: int = AA_ENGINE_AUTO     # testing / tuning aid: force one of the two bf16 tile engines


def _strides(t: torch.Tensor, packed: bool):
    if packed:       # [H, total, d]
        assert t.dim() == 3 and t.stride(2) == 1
        return (0, t.stride(0), t.stride(1))
    assert t.dim() == 4 and t.stride(3) == 1   # [B, H, N, d]
    return (t.stride(0), t.stride(1), t.stride(2))


def make_params(cfg: Config, q, k, v, out=None, cu_seqlens=None, max_seqlen=None, total_tokens=None) -> aa_params:
    """Describe tensors q [B,Hq,N,d] / k,v [B,Hkv,N,d] (any strides with d contiguous), or,
    with cu_seqlens (device int32 [B+1]), packed q [Hq,total,d] / k,v [Hkv,total,d]."""
    packed = cu_seqlens is not None
    p = aa_params()
    if packed:
        p.B = cu_seqlens.numel() - 1
        p.Hq, p.Hkv, p.d = q.shape[0], k.shape[0], q.shape[2]
        p.N = int(max_seqlen)
        p.total_tokens = int(q.shape[1] if total_tokens is None else total_tokens)
        p.cu_seqlens = cu_seqlens.data_ptr()
    else:
        p.B, p.Hq, p.N, p.d = q.shape
        p.Hkv = k.shape[1]
        p.cu_seqlens = None
        p.total_tokens = 0
    p.block_q = p.block_kv = cfg.block
    p.n_init, p.window, p.step = cfg.n_init, cfg.window, cfg.step
    p.theta, p.softmax_scale = cfg.theta, cfg.softmax_scale
    p.causal, p.use_anchor = int(cfg.causal), int(cfg.use_anchor)
    p.granularity = int(cfg.granularity)
    p.engine = int(cfg.engine)
    p.dtype = {torch.float32: AA_FP32, torch.bfloat16: AA_BF16}[q.dtype]
    o = q if out is None else out
    for name, t in (("q_stride", q), ("k_stride", k), ("v_stride", v), ("o_stride", o)):
        setattr(p, name, (ctypes.c_int64 * 3)(*_strides(t, packed)))
    return p


def anchor_sizes(p: aa_params) -> aa_sizes:
    s = aa_sizes()
    _check(_lib.anchor_sizes(ctypes.byref(p), ctypes.byref(s)))
    return s


def anchor_workspace_bytes(p: aa_params) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.anchor_workspace_bytes(ctypes.byref(p), ctypes.byref(n)))
    return int(n.value)


def anchor_compute(p, q, k, v, M, L, Acc, xa_pooled, stream=None):
    _check(_lib.anchor_compute(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(M), _ptr(L), _ptr(Acc),
                               _ptr(xa_pooled), _stream(stream)))


def stripe_select(p, q, k, xa_pooled, counts, offsets, idx, overflow_flag, ws, stream=None, idx_capacity=None):
    cap = idx.numel() if idx_capacity is None else idx_capacity
    _check(_lib.stripe_select(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(xa_pooled), _ptr(counts), _ptr(offsets),
                              _ptr(idx), cap, _ptr(overflow_flag), _ptr(ws),
                              0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))


def stripe_select_noalloc(p, q, k, xa_pooled, counts, offsets, idx, overflow_flag, stream=None, idx_capacity=None):
    """stripe_select with the library's own static scratch: no workspace argument, no allocation."""
    cap = idx.numel() if idx_capacity is None else idx_capacity
    _check(_lib.stripe_select_noalloc(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(xa_pooled), _ptr(counts),
                                      _ptr(offsets), _ptr(idx), cap, _ptr(overflow_flag), _stream(stream)))


def sparse_attn(p, q, k, v, M, L, Acc, counts, offsets, idx, out, lse=None, stream=None, idx_capacity=None):
    cap = idx.numel() if idx_capacity is None else idx_capacity
    _check(_lib.sparse_attn(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(M), _ptr(L), _ptr(Acc), _ptr(counts),
                            _ptr(offsets), _ptr(idx), cap, _ptr(out), _ptr(lse), _stream(stream)))


def anchor_attention_prefill(p, q, k, v, out, lse, stats, ws, stream=None):
    _check(_lib.anchor_attention_prefill(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
                                         _ptr(stats), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                         _stream(stream)))


def dense_causal_flash(p, q, k, v, out, lse=None, stream=None):
    _check(_lib.dense_causal_flash(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
                                   _stream(stream)))


def alloc_stage_buffers(p: aa_params, device="cuda", want_acc=True, idx_capacity=None) -> dict:
    """torch allocations sized by anchor_sizes() for the stage-wise entry points."""
    s = anchor_sizes(p)
    f32 = dict(dtype=torch.float32, device=device)
    cap = s.idx_capacity_max if idx_capacity is None else idx_capacity
    return dict(
        sizes=s,
        M=torch.empty(s.rows, **f32), L=torch.empty(s.rows, **f32),
        Acc=torch.empty(s.acc_elems, **f32) if want_acc else None,
        xa=torch.empty(s.blocks, **f32),
        counts=torch.empty(s.groups, dtype=torch.int32, device=device),
        offsets=torch.empty(s.groups + 1, dtype=torch.int64, device=device),
        idx=torch.empty(max(cap, 64), dtype=torch.int32, device=device),
        flag=torch.zeros(1, dtype=torch.int32, device=device),
        ws=torch.empty(max(s.select_ws_bytes, 256), dtype=torch.uint8, device=device),
        lse=torch.empty(s.rows, **f32),
    )


def default_scale(d: int) -> float:
    return 1.0 / math.sqrt(d)
