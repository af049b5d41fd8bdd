"""ctypes binding of libanchor_probe.so, bench.py's measurement aid (a register-only MFMA loop).

Not part of the attention library or of its ABI: it only tells what matrix rate the GPU at hand
sustains at its actual clock.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libanchor_probe.so")
EXPORTS = ("anchor_probe_mfma", "anchor_probe_mfma_flop")


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise ImportError("libanchor_probe.so is not built (%s). Build it with "
                          "`python -m paper_2505_23520_amd.build`." % path)
    lib = ctypes.CDLL(path)
    lib.anchor_probe_mfma.restype = ctypes.c_int
    lib.anchor_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.anchor_probe_mfma_flop.restype = ctypes.c_double
    lib.anchor_probe_mfma_flop.argtypes = [ctypes.c_int]
    return lib


_lib = load_library()


def mfma_probe(iters: int, scratch: torch.Tensor, stream=None) -> float:
    """Enqueue the loop on `stream` (default: torch's current stream); returns the FLOP it performs.
    scratch: device tensor of at least 1 MiB."""
    assert scratch.is_cuda and scratch.numel() * scratch.element_size() >= (1 << 20)
    st = torch.cuda.current_stream() if stream is None else stream
    rc = _lib.anchor_probe_mfma(int(iters), ctypes.c_void_p(scratch.data_ptr()), ctypes.c_void_p(st.cuda_stream))
    if rc != 0:
        raise RuntimeError("anchor_probe_mfma failed (%d)" % rc)
    return float(_lib.anchor_probe_mfma_flop(int(iters)))
