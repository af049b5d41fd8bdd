"""Host-only checks of the C ABI: the library loads, exports every declared symbol,
and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def api():
    from paper_2505_23520_amd import api as _api
    return _api


def _params(api, **kw):
    p = api.aa_params()
    p.B, p.Hq, p.Hkv, p.N, p.d = 1, 32, 8, 8192, 128
    p.block_q = p.block_kv = 128
    p.n_init, p.window, p.step = 128, 128, 16
    p.theta, p.softmax_scale, p.causal, p.dtype, p.use_anchor = 3.0, 0.0, 1, api.AA_BF16, 1
    for name, H in (("q_stride", 32), ("k_stride", 8), ("v_stride", 8), ("o_stride", 32)):
        setattr(p, name, (ctypes.c_int64 * 3)(H * 8192 * 128, 8192 * 128, 128))
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_header_symbols_are_exported(api):
    hdr = open(os.path.join(ROOT, "include", "anchor_attention.h")).read()
    declared = set(re.findall(r"^(?:int|const char \*)\s*\*?(\w+)\(", hdr, flags=re.M))
    assert declared == set(api.EXPORTS)
    lib = ctypes.CDLL(api.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


def test_sizes_arithmetic(api):
    s = api.anchor_sizes(_params(api))
    assert s.rows == 32 * 8192 and s.acc_elems == s.rows * 128
    assert s.blk_cap == 64 and s.blocks == 32 * 64 and s.grp_cap == 4 and s.groups == 128
    # candidates per head: groups start at 0, 2048, 4096, 6144 -> W = 128, 1920, 3968, 6016
    assert s.idx_capacity_max == 32 * ((1920 - 128) + (3968 - 128) + (6016 - 128))
    assert s.prefill_ws_bytes > s.select_ws_bytes > 0
    s1 = api.anchor_sizes(_params(api, step=1))
    assert s1.groups == 32 * 64
    # block granularity adds the pooled keys (8 KV heads x 64 blocks x 128 floats) to the workspace
    sb = api.anchor_sizes(_params(api, granularity=api.AA_BLOCK))
    assert sb.select_ws_bytes == s.select_ws_bytes + 8 * 64 * 128 * 4


@pytest.mark.parametrize("kw,code", [
    (dict(Hkv=5), -1), (dict(N=0), -1), (dict(step=0), -1), (dict(block_kv=64), -1), (dict(n_init=-1), -1),
    (dict(theta=float("nan")), -1), (dict(dtype=7), -1), (dict(granularity=2), -1),
    (dict(granularity=1, n_init=64), -1), (dict(granularity=1, window=100), -1),
    (dict(causal=0), -2), (dict(d=64), -2), (dict(step=129), -2), (dict(block_q=64, block_kv=64), -2),
    (dict(B=4096, Hq=32, Hkv=8), -2),      # heads x sequences beyond a launch grid's y / z range
])
def test_rejects_bad_params(api, kw, code):
    with pytest.raises(api.AnchorError) as e:
        api.anchor_sizes(_params(api, **kw))
    assert e.value.code == code


def test_set_engine_accepts_only_known_modes(api):
    for mode in (1, 2, 0):
        api.anchor_set_engine(mode)
    with pytest.raises(api.AnchorError):
        api.anchor_set_engine(3)


def test_null_pointers_and_workspace_are_rejected_on_host(api):
    p = _params(api)
    lib = ctypes.CDLL(api.LIB_PATH)
    lib.anchor_compute.restype = ctypes.c_int
    P = ctypes.c_void_p
    lib.anchor_compute.argtypes = [ctypes.POINTER(api.aa_params)] + [P] * 8
    assert lib.anchor_compute(ctypes.byref(p), None, None, None, None, None, None, None, None) == api.AA_EINVAL
    lib.anchor_attention_prefill.restype = ctypes.c_int
    lib.anchor_attention_prefill.argtypes = [ctypes.POINTER(api.aa_params)] + [P] * 7 + [ctypes.c_size_t, P]
    fake = P(4096)          # aligned, never dereferenced: the size check fails first
    assert lib.anchor_attention_prefill(ctypes.byref(p), fake, fake, fake, fake, None, None, fake, 16, None) \
        == api.AA_EWORKSPACE
    assert lib.anchor_attention_prefill(ctypes.byref(p), P(4097), fake, fake, fake, None, None, fake, 16, None) \
        == api.AA_EINVAL
    assert api._lib.anchor_strerror(-3) == b"workspace too small"
