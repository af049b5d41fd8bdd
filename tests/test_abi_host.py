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


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 on its own, and the structs the binding
    declares have the sizes and field offsets the C compiler gives them."""
    import subprocess
    src = tmp_path / "hdr.c"
    from paper_2505_23520_amd import api as _api
    structs = (("aa_params", _api.aa_params), ("aa_sizes", _api.aa_sizes))
    prints = "".join('printf("%%zu\\n", sizeof(%s));\n' % name for name, _ in structs)
    prints += "".join('printf("%%zu\\n", offsetof(%s, %s));\n' % (name, f[0]) for name, t in structs for f in t._fields_)
    src.write_text('#include "anchor_attention.h"\n#include <stddef.h>\n#include <stdio.h>\n'
                   'int main(void) {\n' + prints + 'return 0; }\n')
    exe = tmp_path / "hdr"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror",
                           "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)], text=True).split()]
    want = [ctypes.sizeof(t) for _, t in structs] + [getattr(t, f[0]).offset for _, t in structs for f in t._fields_]
    assert got == want


def test_probe_library_is_separate_from_the_product(api):
    """bench.py's MFMA-rate probe lives in its own shared object; the attention library does not export it."""
    from paper_2505_23520_amd import probe
    lib = ctypes.CDLL(probe.LIB_PATH)
    for name in probe.EXPORTS:
        assert getattr(lib, name) is not None
        assert not hasattr(ctypes.CDLL(api.LIB_PATH), name)
    assert probe._lib.anchor_probe_mfma_flop(3) == 1024 * 4 * 3 * 16 * 32768.0
    assert probe._lib.anchor_probe_mfma(0, None, None) == -1        # rejected on the host, nothing launched


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


def test_engine_field_accepts_only_known_modes(api):
    for mode in (api.AA_ENGINE_AUTO, api.AA_ENGINE_128, api.AA_ENGINE_256):
        api.anchor_sizes(_params(api, engine=mode))
    for mode in (3, -1):
        with pytest.raises(api.AnchorError) as e:
            api.anchor_sizes(_params(api, engine=mode))
        assert e.value.code == api.AA_EINVAL


def test_workspace_bytes_is_the_prefill_workspace(api):
    for kw in (dict(), dict(step=1), dict(granularity=api.AA_BLOCK)):
        p = _params(api, **kw)
        assert api.anchor_workspace_bytes(p) == api.anchor_sizes(p).prefill_ws_bytes
    with pytest.raises(api.AnchorError):
        api.anchor_workspace_bytes(_params(api, causal=0))


def _needed_idx_entries(lens, Hq, bq, step, n_init, window):
    """Entries the lists of a packed batch need when every candidate is selected (64-entry padding)."""
    span, tot = bq * step, 0
    for n in lens:
        for g in range((n + span - 1) // span):
            W = max(n_init, g * span - window)
            tot += (W - n_init + 63) // 64 * 64
    return Hq * tot


def test_idx_capacity_max_covers_every_split_of_a_packed_batch(api):
    """idx_capacity_max promises room for any outcome.  A group counts in full once it has one row,
    so the worst split of total_tokens is not the one with the longest sequences: brute force over
    random splits (and the extreme ones: every sequence one row into its last group)."""
    import numpy as np
    rng = np.random.default_rng(7)
    cases = [((1537, 1537, 2047), 4, 128, 128), ((129025, 129025, 131072), 16, 128, 128)]
    for _ in range(300):
        step = int(rng.choice([1, 2, 3, 4, 16]))
        span = 128 * step
        B = int(rng.integers(1, 6))
        kind = int(rng.integers(3))
        if kind == 0:
            lens = [int(rng.integers(1, 9 * span)) for _ in range(B)]
        elif kind == 1:                              # one row into the last group
            lens = [int(rng.integers(1, 9)) * span + 1 for _ in range(B)]
        else:                                        # exact multiples
            lens = [int(rng.integers(1, 9)) * span for _ in range(B)]
        cases.append((tuple(lens), step, int(rng.choice([0, 64, 128, 200])), int(rng.choice([0, 128, 300]))))
    for lens, step, n_init, window in cases:
        total, N = sum(lens), max(lens)
        p = _params(api, B=len(lens), N=N, step=step, n_init=n_init, window=window, total_tokens=total,
                    cu_seqlens=4096)                 # any non-null value: host arithmetic only
        for name, H in (("q_stride", 32), ("k_stride", 8), ("v_stride", 8), ("o_stride", 32)):
            setattr(p, name, (ctypes.c_int64 * 3)(0, total * 128, 128))
        s = api.anchor_sizes(p)
        need = _needed_idx_entries(lens, 32, 128, step, n_init, window)
        assert s.idx_capacity_max >= need, (lens, step, n_init, window, s.idx_capacity_max, need)


def test_idx_capacity_max_exhaustive_small(api):
    """Every split of a small packed batch (fp32, block 16) into three sequences: the capacity covers
    all of them, and some split needs more than half of it (the bound is not idle slack)."""
    bq, Hq = 16, 2
    for step, total, N, n_init, window in ((1, 150, 100, 16, 16), (2, 170, 90, 0, 16), (3, 200, 150, 8, 40)):
        worst = 0
        for a in range(1, N + 1):
            for b in range(1, N + 1):
                c = total - a - b
                if 1 <= c <= N and max(a, b, c) == N:
                    worst = max(worst, _needed_idx_entries((a, b, c), Hq, bq, step, n_init, window))
        p = api.aa_params()
        p.B, p.Hq, p.Hkv, p.N, p.d = 3, Hq, 1, N, 32
        p.block_q = p.block_kv = bq
        p.n_init, p.window, p.step = n_init, window, step
        p.theta, p.causal, p.dtype, p.use_anchor = 1.0, 1, api.AA_FP32, 1
        p.total_tokens, p.cu_seqlens = total, 4096
        for name in ("q_stride", "k_stride", "v_stride", "o_stride"):
            setattr(p, name, (ctypes.c_int64 * 3)(0, total * 32, 32))
        cap = api.anchor_sizes(p).idx_capacity_max
        assert cap >= worst and 2 * worst > cap, (step, total, N, cap, worst)


def test_null_pointers_and_workspace_are_rejected_on_host(api):
    p = _params(api)
    lib = ctypes.CDLL(api.LIB_PATH)
    lib.anchor_compute.restype = ctypes.c_int
    P = ctypes.c_void_p
    lib.anchor_compute.argtypes = [ctypes.POINTER(api.aa_params)] + [P] * 8
    lib.sparse_attn.restype = ctypes.c_int
    lib.sparse_attn.argtypes = [ctypes.POINTER(api.aa_params)] + [P] * 9 + [ctypes.c_int64] + [P] * 3
    ok = P(4096)
    assert lib.sparse_attn(ctypes.byref(p), ok, ok, ok, None, None, None, ok, ok, ok, -1, ok, None, None) == api.AA_EINVAL
    assert lib.sparse_attn(ctypes.byref(p), ok, ok, ok, ok, None, None, ok, ok, ok, 64, ok, None, None) == api.AA_EINVAL
    assert lib.anchor_compute(ctypes.byref(p), None, None, None, None, None, None, None, None) == api.AA_EINVAL
    lib.anchor_attention_prefill.restype = ctypes.c_int
    lib.anchor_attention_prefill.argtypes = [ctypes.POINTER(api.aa_params)] + [P] * 7 + [ctypes.c_size_t, P]
    fake = P(4096)          # aligned, never dereferenced: the size check fails first
    assert lib.anchor_attention_prefill(ctypes.byref(p), fake, fake, fake, fake, None, None, fake, 16, None) \
        == api.AA_EWORKSPACE
    assert lib.anchor_attention_prefill(ctypes.byref(p), P(4097), fake, fake, fake, None, None, fake, 16, None) \
        == api.AA_EINVAL
    assert api._lib.anchor_strerror(-3) == b"workspace too small"
