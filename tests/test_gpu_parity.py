"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle.

Index sets must match bit for bit except for columns whose pooled difference lies
within 1e-3 of the threshold; outputs within 1e-5 (fp32) / 2e-2 (bf16) max-abs.
"""
import math

import numpy as np
import pytest
import torch

from paper_2505_23520_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_2505_23520_amd import api as _api
    assert torch.cuda.is_available()
    return _api


@pytest.fixture(autouse=True, params=[0, 1, 2], ids=["engine-auto", "engine-128", "engine-256"])
def engine_mode(request, api):
    """Every test runs with the bf16 engine chosen per launch and with each of the two engines forced
    (the 256-row engine falls back to the 128-row one where it does not apply)."""
    import parity_util
    parity_util.ENGINE = request.param
    yield request.param
    parity_util.ENGINE = None


def _wl(name, dtype, lens, Hq, Hkv, d, block, seed, n_planted, mag=(2.5, 2.5), sink=4, q_shift=True, ar1=0.0):
    return synth.Workload(name, dtype, tuple(lens), Hq, Hkv, d, block, 0, 0, 1, 0.0, seed, n_planted=n_planted,
                          planted_mag=mag, sink_keys=sink, sink_mag=4.0, q_shift=q_shift, ar1=ar1)


def _all_samples(run):
    span = run.cfg.block * run.cfg.step
    return [(b, h, g) for b, n in enumerate(run.lens) for h in range(run.Hq) for g in range((n + span - 1) // span)]


def _run_and_check(api, wl, cfg, signal="logit", samples=None, packed=None, edit=None):
    from parity_util import DeviceRun, check_groups
    seqs = [synth.make_sequence(wl, s, signal=signal) for s in range(wl.B)]
    if edit is not None:
        edit(seqs)
    run = DeviceRun(api, seqs, cfg, wl.dtype, packed=packed).stages()
    assert int(run.buf["flag"]) == 0
    smp = _all_samples(run) if samples is None else samples
    worst = check_groups(run, smp)
    # the fused entry point runs the same kernels: identical bits
    out, lse, stats = run.fused()
    assert torch.equal(out, run.out)
    for (b, h, g) in smp[:8]:
        r0 = g * cfg.block * cfg.step
        ri = run.row_index(b, h, r0)
        assert torch.equal(lse[ri:ri + 16], run.buf["lse"][ri:ri + 16])
    # stats: attended pairs and selected entries, from the lists themselves
    counts = run.buf["counts"].cpu().numpy().astype(np.int64)
    tot_sel, tot_pairs = 0, 0
    span = cfg.block * cfg.step
    for b, n in enumerate(run.lens):
        for h in range(run.Hq):
            for g in range((n + span - 1) // span):
                c = int(counts[run.grp_index(b, h, g)])
                W = max(cfg.n_init, g * span - cfg.window)
                rows = np.arange(g * span, min(n, (g + 1) * span))
                tot_sel += c
                tot_pairs += int((np.minimum(cfg.n_init, rows + 1) + np.maximum(0, rows - W + 1) + c).sum())
    assert int(stats[0]) == tot_pairs and int(stats[1]) == tot_sel
    return run, worst


# ------------------------------------------------------------------ fp32, the tiny configuration
def test_fp32_tiny_config(api):
    wl = synth.workloads()["tiny_fp32"]
    cfg = api.Config(block=wl.block, n_init=wl.n_init, window=wl.window, step=wl.step, theta=wl.theta)
    run, worst = _run_and_check(api, wl, cfg, signal="literal")
    assert 0 < worst["selected"] <= worst["candidates"]


@pytest.mark.parametrize("step,theta", [(1, 3.5), (2, 5.0), (4, 4.0)])
def test_fp32_logit_signal_steps(api, step, theta):
    wl = _wl("t", "fp32", [1024], 2, 1, 64, 64, 21, 24)
    cfg = api.Config(block=64, n_init=16, window=64, step=step, theta=theta)
    run, worst = _run_and_check(api, wl, cfg)
    assert 0 < worst["selected"] < worst["candidates"]


def test_fp32_ragged_and_other_shapes(api):
    wl = _wl("t", "fp32", [777], 2, 2, 32, 48, 22, 16)
    cfg = api.Config(block=48, n_init=10, window=30, step=3, theta=5.0)
    _run_and_check(api, wl, cfg)
    wl = _wl("t", "fp32", [200], 1, 1, 128, 128, 23, 8)
    cfg = api.Config(block=128, n_init=0, window=0, step=1, theta=5.0)
    _run_and_check(api, wl, cfg)


# ------------------------------------------------------------------ bf16 MFMA path
@pytest.mark.parametrize("N,step,n_init,window,theta", [
    (2048, 1, 128, 128, 3.5),
    (2048, 2, 128, 128, 5.0),        # threshold in the bulk of the background: many near-threshold columns
    (4096, 16, 128, 128, 4.0),
    (1000, 1, 128, 128, 3.5),        # ragged last block
    (1500, 4, 64, 192, 5.0),         # ragged, sub-block sink, wider window
    (1280, 3, 0, 0, 4.0),            # no sink, no extra window, step not a power of two
    (640, 5, 200, 100, 3.0),
])
def test_bf16_pipeline(api, N, step, n_init, window, theta):
    wl = _wl("t", "bf16", [N], 4, 2, 128, 128, 30 + step, max(8, N // 64))
    cfg = api.Config(block=128, n_init=n_init, window=window, step=step, theta=theta)
    run, worst = _run_and_check(api, wl, cfg)
    if N >= 1024:
        assert 0 < worst["selected"] < worst["candidates"]


def test_bf16_short_sequences(api):
    for N in (1, 50, 128, 129):
        wl = _wl("t", "bf16", [N], 2, 1, 128, 128, 40 + N, 0)
        cfg = api.Config(block=128, n_init=128, window=128, step=2, theta=2.0)
        _run_and_check(api, wl, cfg)


@pytest.mark.parametrize("theta", [float("inf"), float("-inf")])
def test_bf16_theta_extremes(api, theta):
    from parity_util import DeviceRun
    wl = _wl("t", "bf16", [1536], 4, 2, 128, 128, 50, 16)
    cfg = api.Config(block=128, n_init=128, window=128, step=2, theta=theta)
    run, worst = _run_and_check(api, wl, cfg)
    if theta > 0:       # everything selected: the sparse path equals the dense kernel's result
        assert worst["selected"] == worst["candidates"]
        dense, dlse = run.dense()
        assert (dense.float() - run.out.float()).abs().max().item() <= 2e-2
        assert (dlse - run.buf["lse"]).abs().max().item() <= 4e-3
    else:
        assert worst["selected"] == 0


def test_dense_flash_matches_oracle(api):
    from oracle import anchor_oracle as ao
    from parity_util import DeviceRun
    for dtype, d, block, N, tolO in (("bf16", 128, 128, 1100, 2e-2), ("fp32", 64, 64, 700, 1e-5)):
        wl = _wl("t", dtype, [N], 2, 1, d, block, 60, 8)
        seqs = [synth.make_sequence(wl, 0, signal="logit")]
        cfg = api.Config(block=block, n_init=block, window=block, step=1, theta=1.0)
        run = DeviceRun(api, seqs, cfg, dtype)
        out, lse = run.dense()
        for h in range(2):
            ref = ao.run_head(seqs[0]["q"][h], seqs[0]["k"][0], seqs[0]["v"][0], ao.dense_params(block))
            assert np.abs(out[0, h].float().cpu().numpy() - ref["O"]).max() <= tolO
            assert np.abs(lse[h * N:(h + 1) * N].cpu().numpy() - ref["lse"]).max() <= (4e-3 if dtype == "bf16" else 2e-5)


def test_bf16_recompute_anchor_in_stage3(api):
    """sparse_attn with M = L = Acc = NULL computes the anchor region itself: O and lse against the
    oracle (on the lists of the cached-state run, which check_groups verifies as well)."""
    from parity_util import DeviceRun, check_groups
    wl = _wl("t", "bf16", [2048], 4, 2, 128, 128, 70, 32)
    cfg = api.Config(block=128, n_init=128, window=128, step=2, theta=4.5)
    seqs = [synth.make_sequence(wl, 0, signal="logit")]
    run = DeviceRun(api, seqs, cfg, "bf16").stages()
    out2 = torch.zeros_like(run.out)
    lse2 = torch.empty_like(run.buf["lse"])
    B = run.buf
    api.sparse_attn(run.p, run.q, run.k, run.v, None, None, None, B["counts"], B["offsets"], B["idx"], out2, lse2)
    torch.cuda.synchronize()
    worst = check_groups(run, _all_samples(run), check_state=False, out=out2, lse=lse2)
    assert worst["selected"] > 0


def _plant_columns(wl, cols, mag):
    """Input edit: every query gets d^(1/4) u and the key columns `cols` get mag d^(1/4) u along a
    fixed unit direction u, so that these columns' logits sit about mag above the background's."""
    def edit(seqs):
        u = np.random.default_rng(99).standard_normal(wl.d)
        u /= np.linalg.norm(u)
        for s in seqs:
            s["q"] += (wl.d ** 0.25 * u).astype(np.float32)
            s["k"][:, cols] += (mag * wl.d ** 0.25 * u).astype(np.float32)
            s["q"], s["k"] = synth.round_to_bf16(s["q"]), synth.round_to_bf16(s["k"])
    return edit


@pytest.mark.parametrize("N,step,theta,long_lists", [(2560, 2, 6.0, False), (2560, 4, 6.0, False),
                                                     (16384, 2, 4.0, True)])
def test_bf16_listed_columns_far_above_the_anchor(api, N, step, theta, long_lists):
    """Rows whose maximum lies outside the anchor region (Sec. 2.2.2): no sink, and in the first half
    of the sequence planted columns whose logits exceed the anchor of the later rows by more than
    ten nats; even step.  Stage 3 then has to raise the reference of its exponentials above the
    cached anchor and rescale the cached state (the m' = max(m, max(qk)) update of Algorithm 3) --
    in both tile engines, and, with lists of 48 tiles and more per group, in the engine the
    automatic choice picks for long lists."""
    from oracle import anchor_oracle as ao
    from parity_util import DeviceRun, check_groups, oracle_params
    wl = _wl("t", "bf16", [N], 2, 1, 128, 128, 77, 0, sink=0)
    cfg = api.Config(block=128, n_init=128, window=128, step=step, theta=theta)
    seqs = [synth.make_sequence(wl, 0, signal="logit")]
    _plant_columns(wl, np.arange(130, N // 2 - 64, 53 if N < 8192 else 61), 22.0)(seqs)
    run = DeviceRun(api, seqs, cfg, "bf16").stages()
    assert int(run.buf["flag"]) == 0
    span = 128 * step
    ng = N // span
    if long_lists:
        mean_tiles = int(run.buf["offsets"][-1]) / 64 / run.sizes.groups
        assert mean_tiles >= 48, mean_tiles          # the automatic choice runs the 256-row engine
        samples = [(0, 0, 1), (0, 1, ng // 2), (0, 1, ng - 2), (0, 0, ng - 1)]
    else:
        samples = _all_samples(run)
    check_groups(run, samples)
    # the case is what it claims: in the last group the selected columns lift most rows' maximum
    # ten nats and more above their anchor
    q, k, v = seqs[0]["q"][0], seqs[0]["k"][0], seqs[0]["v"][0]
    ref = ao.run_group(q, k, v, oracle_params(run.cfg, 128), ng - 1)
    assert ref["M"].max() < 8.0
    rows_above = int((ref["lse"] - ref["M"] >= 10.0).sum())
    assert rows_above >= 0.75 * ref["M"].size, rows_above


def test_packed_batch_needing_the_whole_idx_capacity(api):
    """Packed sequences that each reach one row into their last group, theta = +inf: every candidate
    of every group is selected, which needs exactly the capacity anchor_sizes() promises (a group
    counts in full once it has one row).  Through the fused entry point, against dense attention."""
    from parity_util import DeviceRun
    lens = [1537, 1537, 2047]
    wl = _wl("t", "bf16", lens, 4, 2, 128, 128, 35, 8)
    cfg = api.Config(block=128, n_init=128, window=128, step=4, theta=float("inf"))
    seqs = [synth.make_sequence(wl, s, signal="logit") for s in range(3)]
    run = DeviceRun(api, seqs, cfg, "bf16", packed=True).stages()
    assert int(run.buf["flag"]) == 0
    span = 128 * 4
    need = 0
    counts = run.buf["counts"].cpu().numpy()
    for b, n in enumerate(lens):
        for h in range(4):
            for g in range((n + span - 1) // span):
                cand = max(128, g * span - 128) - 128
                assert counts[run.grp_index(b, h, g)] == cand
                need += (cand + 63) // 64 * 64
    assert need == run.sizes.idx_capacity_max == int(run.buf["offsets"][-1])
    out, lse, stats = run.fused()
    assert torch.equal(out, run.out)
    dense, dlse = run.dense()
    assert (dense.float() - out.float()).abs().max().item() <= 2e-2
    assert (dlse - lse).abs().max().item() <= 4e-3
    assert int(stats[0]) == 4 * sum(n * (n + 1) // 2 for n in lens)


@pytest.mark.parametrize("dtype,d,block", [("bf16", 128, 128), ("fp32", 64, 64)])
def test_without_anchor_variant(api, dtype, d, block):
    """use_anchor = 0: the pooled scores are compared against a zero anchor (Table 4, "Without Anchor")."""
    wl = _wl("t", dtype, [1536], 2, 1, d, block, 75, 24)
    cfg = api.Config(block=block, n_init=block, window=block, step=2, theta=-1.5, use_anchor=False)
    run, worst = _run_and_check(api, wl, cfg)
    assert 0 < worst["selected"] < worst["candidates"]


def _shift_key_blocks(wl, blocks, mag=2.0):
    """Input edit: whole key blocks get a mean shift along the direction the queries share, so that
    pooled keys differ from block to block (inputs only; rounded back to bf16 where needed)."""
    def edit(seqs):
        grp = wl.Hq // wl.Hkv
        for s in seqs:
            for hk in range(wl.Hkv):
                u = s["q"][hk * grp:(hk + 1) * grp].mean(axis=(0, 1)).astype(np.float64)
                u /= np.linalg.norm(u)
                for J in blocks:
                    if (J + 1) * wl.block <= s["k"].shape[1]:
                        s["k"][hk, J * wl.block:(J + 1) * wl.block] += (mag * wl.d ** 0.25 * u).astype(np.float32)
            if wl.dtype == "bf16":
                s["k"] = synth.round_to_bf16(s["k"])
    return edit


@pytest.mark.parametrize("dtype,d,block,step,theta", [("bf16", 128, 128, 1, 4.0), ("bf16", 128, 128, 2, 4.0),
                                                      ("fp32", 64, 32, 1, 4.0), ("fp32", 64, 32, 2, 4.0),
                                                      ("fp32", 64, 32, 1, 5.1), ("fp32", 32, 16, 3, 4.0)])
def test_block_granularity_variant(api, dtype, d, block, step, theta):
    """granularity = AA_BLOCK: one decision per key block on the block's mean key (Sec. 2.1.2, Table 1)."""
    wl = _wl("t", dtype, [block * 16], 2, 1, d, block, 33, 0)
    cfg = api.Config(block=block, n_init=block, window=block, step=step, theta=theta, granularity=api.AA_BLOCK)
    run, worst = _run_and_check(api, wl, cfg, edit=_shift_key_blocks(wl, [2, 5, 6, 11]))
    assert 0 < worst["selected"] < worst["candidates"]
    assert worst["selected"] % block == 0                     # whole blocks only
    for (b, h, g) in _all_samples(run):
        lst, _, _ = run.group_list(b, h, g)
        assert np.array_equal(np.unique(lst // block).repeat(block) * block + np.tile(np.arange(block), lst.size // block), lst)


def test_block_granularity_packed_and_errors(api):
    from paper_2505_23520_amd.api import AnchorError
    wl = _wl("t", "bf16", [1024, 2048, 384], 4, 2, 128, 128, 34, 0)
    cfg = api.Config(block=128, n_init=128, window=128, step=2, theta=4.0, granularity=api.AA_BLOCK)
    run, worst = _run_and_check(api, wl, cfg, packed=True, edit=_shift_key_blocks(wl, [1, 3, 4, 9]))
    assert worst["selected"] > 0
    bad = api.Config(block=128, n_init=16, window=128, step=2, theta=4.0, granularity=api.AA_BLOCK)
    with pytest.raises(AnchorError) as e:
        api.anchor_sizes(api.make_params(bad, run.q, run.k, run.v, run.out, cu_seqlens=run.cu, max_seqlen=2048))
    assert e.value.code == api.AA_EINVAL


def test_packed_varlen(api):
    for dtype, d, block, lens in (("bf16", 128, 128, [300, 1024, 129, 2000]), ("fp32", 64, 32, [100, 333, 64])):
        wl = _wl("t", dtype, lens, 4, 2, d, block, 80, 12)
        cfg = api.Config(block=block, n_init=block, window=block, step=2, theta=4.5)
        run, worst = _run_and_check(api, wl, cfg, packed=True)
        assert worst["selected"] > 0


def test_packed_batch_with_empty_sequences(api):
    """cu_seqlens may repeat a value: such a sequence owns no rows, blocks or groups, and the others
    are laid out and computed as if it were not there (first, middle and last position)."""
    for dtype, d, block, lens in (("bf16", 128, 128, [0, 700, 0, 0, 1500, 0]), ("fp32", 64, 32, [0, 200, 0, 333])):
        wl = _wl("t", dtype, lens, 4, 2, d, block, 82, 12)
        cfg = api.Config(block=block, n_init=block, window=block, step=2, theta=4.5)
        run, worst = _run_and_check(api, wl, cfg, packed=True)
        assert worst["selected"] > 0
        # the same sequences without the empty ones: identical output rows
        keep = [s for s in range(len(lens)) if lens[s] > 0]
        wl2 = _wl("t", dtype, lens, 4, 2, d, block, 82, 12)
        from parity_util import DeviceRun
        seqs = [synth.make_sequence(wl2, s, signal="logit") for s in keep]
        run2 = DeviceRun(api, seqs, cfg, dtype, packed=True).stages()
        assert torch.equal(run.out, run2.out)
        assert torch.equal(run.buf["lse"], run2.buf["lse"])


def test_packed_many_sequences_some_without_candidates(api):
    """Six packed sequences, three of them too short to have any candidate column (the mask kernel
    deals only the work items that exist to its work-groups and has to step over such sequences)."""
    lens = [100, 5000, 64, 3000, 129, 2600]
    wl = _wl("t", "bf16", lens, 4, 2, 128, 128, 81, 24)
    cfg = api.Config(block=128, n_init=128, window=128, step=2, theta=4.5)
    run, worst = _run_and_check(api, wl, cfg, packed=True)
    assert 0 < worst["selected"] < worst["candidates"]
    counts = run.buf["counts"].cpu().numpy()
    for b in (0, 2, 4):                              # one group, no candidates: empty lists
        for h in range(4):
            assert counts[run.grp_index(b, h, 0)] == 0


def test_fixed_batch_and_strided_layout(api):
    """B = 2 fixed-length batch; tensors given as [B, N, H, d] views (token-major memory)."""
    from parity_util import DeviceRun, check_groups
    wl = _wl("t", "bf16", [1024, 1024], 4, 2, 128, 128, 90, 16)
    cfg = api.Config(block=128, n_init=128, window=128, step=2, theta=4.5)
    seqs = [synth.make_sequence(wl, s, signal="logit") for s in range(2)]
    run = DeviceRun(api, seqs, cfg, "bf16", packed=False)
    for name in ("q", "k", "v", "out"):
        t = getattr(run, name)
        setattr(run, name, t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3))   # same values, other strides
    run.p = api.make_params(cfg, run.q, run.k, run.v, run.out)
    assert run.p.q_stride[2] == 4 * 128
    run.stages()
    check_groups(run, _all_samples(run))


def test_overflow_flag_and_capacity(api):
    from parity_util import DeviceRun
    wl = _wl("t", "bf16", [2048], 2, 1, 128, 128, 95, 64)
    cfg = api.Config(block=128, n_init=128, window=128, step=1, theta=float("inf"))
    seqs = [synth.make_sequence(wl, 0, signal="logit")]
    run = DeviceRun(api, seqs, cfg, "bf16")
    B = run.buf
    api.anchor_compute(run.p, run.q, run.k, run.v, B["M"], B["L"], B["Acc"], B["xa"])
    small = torch.full((1024 + 64,), -7, dtype=torch.int32, device="cuda")
    api.stripe_select(run.p, run.q, run.k, B["xa"], B["counts"], B["offsets"], small, B["flag"], B["ws"],
                      idx_capacity=1024)
    torch.cuda.synchronize()
    assert int(B["flag"]) == 1
    assert torch.all(small[1024:] == -7)            # nothing written past the capacity
    assert int(B["offsets"][-1]) == run.sizes.idx_capacity_max   # offsets stay exact
    # lists that did not fit are incomplete: stage 3 must not read them (nor past the buffer) and
    # leaves the output alone
    sentinel = torch.full_like(run.out, 3.0)
    lse = torch.full_like(B["lse"], -5.0)
    api.sparse_attn(run.p, run.q, run.k, run.v, B["M"], B["L"], B["Acc"], B["counts"], B["offsets"], small, sentinel,
                    lse, idx_capacity=1024)
    torch.cuda.synchronize()
    assert torch.all(sentinel == 3.0) and torch.all(lse == -5.0)


def test_determinism(api):
    from parity_util import DeviceRun
    wl = _wl("t", "bf16", [3000], 4, 2, 128, 128, 97, 40)
    cfg = api.Config(block=128, n_init=128, window=128, step=4, theta=5.0)
    seqs = [synth.make_sequence(wl, 0, signal="logit")]
    run = DeviceRun(api, seqs, cfg, "bf16").stages()
    o1, i1, c1 = run.out.clone(), run.buf["idx"].clone(), run.buf["counts"].clone()
    run.stages()
    tot = int(run.buf["offsets"][-1])
    assert torch.equal(o1, run.out) and torch.equal(c1, run.buf["counts"]) and torch.equal(i1[:tot], run.buf["idx"][:tot])


# ------------------------------------------------------------------ seeded random configurations
def _random_cases():
    rng = np.random.default_rng(20250523)
    cases = []
    for i in range(14):
        bf16 = i % 7 != 6                       # twelve bf16 cases, two fp32 cases
        block = 128 if bf16 else int(rng.choice([16, 32, 48, 64]))
        d = 128 if bf16 else int(rng.choice([32, 64, 128]))
        heads = [(2, 1), (4, 2), (4, 4), (8, 2), (3, 1)][int(rng.integers(5))]
        nseq = int(rng.integers(1, 4))
        hi = 5000 if bf16 else 700
        lens = [int(rng.integers(1, hi)) for _ in range(nseq)]
        step = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16]))
        n_init = int(rng.integers(0, 3 * block))
        window = int(rng.integers(0, 3 * block))
        theta = float(rng.uniform(2.0, 5.5))
        cases.append(("bf16" if bf16 else "fp32", d, block, heads, lens, step, n_init, window, theta, 300 + i))
    return cases


@pytest.mark.parametrize("case", _random_cases(), ids=lambda c: "%s-N%s-s%d-i%d-w%d" % (c[0], "_".join(map(str, c[4])), c[5], c[6], c[7]))
def test_random_configurations(api, case):
    """Shapes nobody picked by hand: lengths, step, sink and window sizes, GQA ratio and batch
    drawn from a fixed seed; packed when there is more than one sequence."""
    dtype, d, block, (Hq, Hkv), lens, step, n_init, window, theta, seed = case
    wl = _wl("rnd", dtype, lens, Hq, Hkv, d, block, seed, max(4, max(lens) // 48))
    cfg = api.Config(block=block, n_init=n_init, window=window, step=step, theta=theta)
    _run_and_check(api, wl, cfg, packed=(len(lens) > 1) or None)


def test_prefill_under_graph_capture(api, engine_mode):
    """The fused entry point only enqueues kernels (no allocation, no synchronisation, no memset), so
    it can be captured into a HIP graph: replays, with eager work of the same library between them,
    reproduce the eager result bit for bit, also after the inputs change in place."""
    from parity_util import DeviceRun
    wl = _wl("t", "bf16", [3000], 4, 2, 128, 128, 61, 48)
    cfg = api.Config(block=128, n_init=128, window=128, step=2, theta=4.0)
    seqs = [synth.make_sequence(wl, 0, signal="logit")]
    run = DeviceRun(api, seqs, cfg, "bf16")
    sz = run.sizes
    ws = torch.empty(sz.prefill_ws_bytes, dtype=torch.uint8, device="cuda")
    lse = torch.empty(sz.rows, dtype=torch.float32, device="cuda")
    stats = torch.zeros(4, dtype=torch.int64, device="cuda")
    out = torch.zeros_like(run.q)

    def eager():
        o = torch.zeros_like(run.q)
        l = torch.empty_like(lse)
        st = torch.zeros_like(stats)
        w = torch.empty_like(ws)
        api.anchor_attention_prefill(run.p, run.q, run.k, run.v, o, l, st, w)
        torch.cuda.synchronize()
        return o, l, st

    ref_o, ref_l, ref_st = eager()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up on the capture stream
        api.anchor_attention_prefill(run.p, run.q, run.k, run.v, out, lse, stats, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        api.anchor_attention_prefill(run.p, run.q, run.k, run.v, out, lse, stats, ws)
    for rep in range(3):
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_o) and torch.equal(lse, ref_l) and torch.equal(stats, ref_st), rep
        eager()                                         # the library's own eager work between replays
    # new inputs in the same buffers: the replay follows them
    run.q.copy_(run.q.flip(2).contiguous())
    ref_o, ref_l, ref_st = eager()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, ref_o) and torch.equal(lse, ref_l) and torch.equal(stats, ref_st)
