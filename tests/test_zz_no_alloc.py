"""stripe_select_noalloc (scratch inside the library, no workspace argument, no allocation) must
produce what stripe_select produces with a caller workspace: counts, offsets, lists and flag,
bit for bit, on two calls in a row, the second on a smaller input (the shared scratch then still
holds the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2505_23520_amd import synth

pytestmark = pytest.mark.gpu


def _select_both_ways(api, N, Hq, Hkv, step, theta, seed):
    from parity_util import DeviceRun
    wl = synth.Workload("na", "bf16", (N,), Hq, Hkv, 128, 128, 128, 128, step, theta, seed, n_planted=max(8, N // 64),
                        planted_mag=(2.5, 2.5), sink_keys=4, sink_mag=4.0)
    cfg = api.Config(block=128, n_init=128, window=128, step=step, theta=theta)
    run = DeviceRun(api, [synth.make_sequence(wl, 0, signal="logit")], cfg, "bf16", want_acc=False)
    B = run.buf
    api.anchor_compute(run.p, run.q, run.k, run.v, B["M"], B["L"], None, B["xa"])
    api.stripe_select(run.p, run.q, run.k, B["xa"], B["counts"], B["offsets"], B["idx"], B["flag"], B["ws"])
    counts2, offsets2 = torch.full_like(B["counts"], -1), torch.full_like(B["offsets"], -1)
    idx2, flag2 = torch.full_like(B["idx"], -1), torch.full_like(B["flag"], -1)
    api.stripe_select_noalloc(run.p, run.q, run.k, B["xa"], counts2, offsets2, idx2, flag2)
    torch.cuda.synchronize()
    total = int(B["offsets"][-1])
    assert int(B["flag"]) == 0 and int(flag2) == 0
    assert torch.equal(counts2, B["counts"]) and torch.equal(offsets2, B["offsets"])
    assert torch.equal(idx2[:total], B["idx"][:total])
    assert torch.all(idx2[total:] == -1)                      # nothing written beyond the lists
    return int(B["counts"].sum()), total


def test_noalloc_matches_workspace_variant_twice_in_a_row():
    from paper_2505_23520_amd import api
    assert torch.cuda.is_available()
    sel1, tot1 = _select_both_ways(api, 12288, 8, 2, 4, 4.5, 501)    # several mask row tiles and list segments
    sel2, tot2 = _select_both_ways(api, 3000, 4, 2, 2, 4.0, 502)     # smaller, ragged: stale scratch behind it
    assert sel1 > sel2 > 0


def test_noalloc_rejects_what_does_not_fit():
    from paper_2505_23520_amd import api
    wl = synth.workloads()["gqa_128k"]
    q = torch.empty(1, 32, 8, 128, dtype=torch.bfloat16, device="cuda")   # never read: the size check fails first
    p = api.make_params(api.Config(step=1), q, q[:, :8], q[:, :8])
    p.N = 131072                                                          # step 1 at 128k needs 1 GiB of bit words
    for name in ("q_stride", "k_stride", "v_stride", "o_stride"):
        getattr(p, name)[0] = 32 * 131072 * 128
        getattr(p, name)[1] = 131072 * 128
    assert api.anchor_sizes(p).select_ws_bytes > 64 << 20
    one = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(api.AnchorError) as e:
        api.stripe_select_noalloc(p, q, q, one.float(), one, one.long(), one, one)
    assert e.value.code == api.AA_EWORKSPACE
