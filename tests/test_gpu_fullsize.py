"""GPU parity at the full workload sizes, in the launch configuration bench.py times
(same entry points, same parameters), on sampled (sequence, head, group) units that the
oracle computes one by one.  Units are independent, so a sampled comparison is exact."""
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


def _cfg(api, wl, **kw):
    d = dict(block=wl.block, n_init=wl.n_init, window=wl.window, step=wl.step, theta=wl.theta)
    d.update(kw)
    return api.Config(**d)


def _run(api, wl, cfg, signal, samples, packed=None):
    from parity_util import DeviceRun, check_groups
    seqs = [synth.make_sequence(wl, s, signal=signal) for s in range(wl.B)]
    run = DeviceRun(api, seqs, cfg, wl.dtype, packed=packed).stages()
    assert int(run.buf["flag"]) == 0
    worst = check_groups(run, samples)
    out, lse, stats = run.fused()
    assert torch.equal(out, run.out)
    del seqs
    return run, worst, stats


@pytest.mark.parametrize("signal", ["literal", "logit"])
def test_gqa_8k_all_groups_of_sampled_heads(api, signal):
    wl = synth.workloads()["gqa_8k"]
    samples = [(0, h, g) for h in (0, 5, 18, 31) for g in range(4)]
    run, worst, stats = _run(api, wl, _cfg(api, wl), signal, samples)
    if signal == "literal":     # unit planted magnitudes: practically every candidate passes
        assert worst["selected"] > 0.99 * worst["candidates"]
    else:
        assert 0 < worst["selected"] < 0.2 * worst["candidates"]


def test_gqa_8k_step1(api):
    wl = synth.workloads()["gqa_8k"]
    samples = [(0, h, g) for h in (3, 28) for g in (0, 1, 2, 17, 40, 63)]
    _run(api, wl, _cfg(api, wl, step=1, theta=4.5), "logit", samples)


def test_gqa_32k_theta_sweep(api):
    wl = synth.workloads()["gqa_32k"]
    prev = -1
    for theta in wl.extra["theta_sweep"]:
        samples = [(0, 9, 3), (0, 22, 15), (0, 0, 8)]
        run, worst, stats = _run(api, wl, _cfg(api, wl, theta=theta), "logit", samples)
        assert worst["selected"] >= prev          # selections are nested in theta
        prev = worst["selected"]
        del run
        torch.cuda.empty_cache()


@pytest.mark.parametrize("signal", ["literal", "logit", "peaked"])
def test_gqa_128k_sampled(api, signal):
    wl = synth.workloads()["gqa_128k"]
    # groups 1..3 are the first with candidates (less than one key chunk of the mask kernel)
    samples = [(0, 0, 0), (0, 7, 1), (0, 20, 2), (0, 3, 3), (0, 13, 20), (0, 26, 41), (0, 31, 63)]
    theta = 3.0 * wl.theta if signal == "peaked" else wl.theta     # as bench.py runs it
    run, worst, stats = _run(api, wl, _cfg(api, wl, theta=theta), signal, samples)
    if signal == "peaked":      # the planted columns before a group's window are kept, little else
        assert 0 < worst["selected"] < 0.05 * worst["candidates"]
    N, Hq = wl.seqlens[0], wl.Hq
    assert 0 < stats[0] <= Hq * N * (N + 1) // 2
    del run
    torch.cuda.empty_cache()


def test_varlen_mixed_packed(api):
    wl = synth.workloads()["varlen_mixed"]
    samples = [(0, 2, 7), (1, 11, 0), (1, 30, 23), (2, 17, 47), (3, 5, 63), (3, 31, 30)]
    run, worst, stats = _run(api, wl, _cfg(api, wl), "literal", samples, packed=True)
    assert worst["selected"] > 0.99 * worst["candidates"]   # no planted structure: nearly dense
    del run
    torch.cuda.empty_cache()


@pytest.mark.parametrize("step", [3, 16])
def test_long_packed_every_key_chunk_of_every_row_tile(api, step):
    """Sequences long enough for several tiles of pooled rows in the bf16 mask kernel (its grid pairs
    a short row tile with a long one, per sequence: 4, 3 and 1 tiles here; 126 or 128 rows per tile).
    theta = +inf must select every candidate of every group and theta = -inf none (a key chunk that no
    work-group visits, or visits for the wrong tile, shows as a wrong count); at a finite theta
    sampled groups from both ends of every row tile are compared with the oracle."""
    from parity_util import DeviceRun, check_groups
    lens = (50000, 33000, 3000)
    wl = synth.Workload("long_packed", "bf16", lens, 2, 1, 128, 128, 128, 128, step, 4.5, 123, n_planted=96,
                        planted_mag=(2.5, 2.5), sink_keys=4, sink_mag=4.0)
    seqs = [synth.make_sequence(wl, s, signal="logit") for s in range(wl.B)]
    span = 128 * step
    for theta in (float("inf"), float("-inf")):
        run = DeviceRun(api, seqs, _cfg(api, wl, theta=theta), "bf16", packed=True, want_acc=False)
        B = run.buf
        api.anchor_compute(run.p, run.q, run.k, run.v, B["M"], B["L"], None, B["xa"])
        api.stripe_select(run.p, run.q, run.k, B["xa"], B["counts"], B["offsets"], B["idx"], B["flag"], B["ws"])
        torch.cuda.synchronize()
        assert int(B["flag"]) == 0
        counts = B["counts"].cpu().numpy()
        for b, n in enumerate(lens):
            for h in range(wl.Hq):
                for g in range((n + span - 1) // span):
                    cand = max(0, max(wl.n_init, g * span - wl.window) - wl.n_init)
                    assert counts[run.grp_index(b, h, g)] == (cand if theta > 0 else 0), (theta, b, h, g)
        del run, B
        torch.cuda.empty_cache()
    rows_per_tile = (128 - 128 % step) // step          # groups per row tile
    samples = []
    for b, n in enumerate(lens):
        ng = (n + span - 1) // span
        edge = sorted({g for t in range(0, ng, rows_per_tile) for g in (t, min(ng - 1, t + rows_per_tile - 1))})
        samples += [(b, (b + i) % wl.Hq, g) for i, g in enumerate(edge)]
    run = DeviceRun(api, seqs, _cfg(api, wl), "bf16", packed=True).stages()
    assert int(run.buf["flag"]) == 0
    worst = check_groups(run, samples)
    assert 0 < worst["selected"] < worst["candidates"]


def test_256k_tokens_two_heads(api):
    """Twice the headline length (more than 64 list segments and 16 mask row tiles per head): every
    candidate at theta = +inf (and the output then equals dense attention), sampled groups against
    the oracle at the workload's theta."""
    from parity_util import DeviceRun, check_groups
    N, step = 262144, 16
    wl = synth.Workload("gqa_256k_2h", "bf16", (N,), 2, 1, 128, 128, 128, 128, step, float(np.log(32.0)), 77,
                        n_planted=2048, planted_mag=(1.5, 3.5), sink_keys=4, sink_mag=4.0)
    seqs = [synth.make_sequence(wl, 0, signal="logit")]
    span = 128 * step
    run = DeviceRun(api, seqs, _cfg(api, wl, theta=float("inf")), "bf16").stages()
    assert int(run.buf["flag"]) == 0
    counts = run.buf["counts"].cpu().numpy()
    for h in range(2):
        for g in range(N // span):
            assert counts[run.grp_index(0, h, g)] == max(0, max(128, g * span - 128) - 128), (h, g)
    dense, dlse = run.dense()
    rows = torch.tensor([0, 1, 127, 128, 4095, 131071, 131072, 200000, N - 1], device="cuda")
    for h in range(2):
        assert (dense[0, h, rows].float() - run.out[0, h, rows].float()).abs().max().item() <= 2e-2
    del run, dense, dlse
    torch.cuda.empty_cache()
    run = DeviceRun(api, seqs, _cfg(api, wl), "bf16").stages()
    assert int(run.buf["flag"]) == 0
    worst = check_groups(run, [(0, 0, 0), (0, 1, 1), (0, 0, 64), (0, 1, 127)])
    assert 0 < worst["selected"] < 0.1 * worst["candidates"]
