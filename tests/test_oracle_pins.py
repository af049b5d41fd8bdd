"""Pins for the fp64 CPU oracle: each test ties it to something other than itself.

  * theta = +inf  -> dense causal attention, checked against a library routine
    (torch scaled_dot_product_attention in fp64) and logsumexp.
  * theta = -inf  -> initial tokens + local window only; window ranges come from
    a hand-derived table of Algorithm 1's range lines (tests/golden).
  * constant keys -> closed forms: lse_r = S_r + ln|P(r)|, O_r = mean of V over P(r).
  * a d=1 example worked by hand (tests/golden), including the <= boundary.
  * an independent mask-based brute force (full N x N matrices) on tiny inputs,
    for step in {1, 2, 4} and a ragged tail.
  * invariants: rows of the softmax sum to one, selections are nested in theta and
    lie in the candidate range, recall = exp(lse_sparse - lse_full) equals the
    directly summed attention mass.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import anchor_oracle as ao


def _rand(N, d, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, d)).astype(np.float32),
            rng.standard_normal((N, d)).astype(np.float32),
            rng.standard_normal((N, d)).astype(np.float32))


# ----------------------------------------------------------------- theta = +inf
@pytest.mark.parametrize("N,d,bq,ninit,w,step", [(300, 32, 64, 16, 64, 2), (257, 16, 32, 32, 32, 1),
                                                  (96, 8, 16, 0, 0, 3)])
def test_theta_inf_is_dense_causal_attention(N, d, bq, ninit, w, step):
    q, k, v = _rand(N, d, 11)
    p = ao.OracleParams(b_q=bq, n_init=ninit, w=w, step=step, theta=float("inf"))
    res = ao.run_head(q, k, v, p)
    tq, tk, tv = (torch.from_numpy(x).double()[None, None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0, 0].numpy()
    np.testing.assert_allclose(res["O"], ref, rtol=0, atol=1e-12)
    s = (tq[0, 0] @ tk[0, 0].T) / math.sqrt(d)
    s = s.masked_fill(torch.triu(torch.ones(N, N, dtype=torch.bool), 1), float("-inf"))
    np.testing.assert_allclose(res["lse"], torch.logsumexp(s, -1).numpy(), rtol=0, atol=1e-12)
    assert res["pairs"] == N * (N + 1) // 2


# ------------------------------------------ theta = -inf and Algorithm 1's window
def _golden_window_rows(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "alg1_window_ranges.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            i, js, je, first, last = line.split()
            rows.append((int(i), None if first == "-" else int(first), None if last == "-" else int(last)))
    return rows


def test_window_ranges_match_algorithm1_table(golden_dir):
    """|A(r)| read off lse with constant keys must equal the hand-derived ranges."""
    bq, step, N, d = 4, 2, 40, 4
    p = ao.OracleParams(b_q=bq, n_init=4, w=4, step=step, theta=float("-inf"), sigma=1.0)
    rng = np.random.default_rng(5)
    q = rng.standard_normal((N, d)).astype(np.float32)
    k = np.tile(rng.standard_normal((1, d)).astype(np.float32), (N, 1))
    v = rng.standard_normal((N, d)).astype(np.float32)
    res = ao.run_head(q, k, v, p)
    s_r = (q.astype(np.float64) @ k[0].astype(np.float64))
    for i, first, last in _golden_window_rows(golden_dir):
        for r in range((i - 1) * bq, i * bq):
            keys = set(j for j in range(4) if j <= r)
            if first is not None:
                keys |= set(j for j in range(first, last + 1) if j <= r)
            assert abs(res["lse"][r] - (s_r[r] + math.log(len(keys)))) < 1e-12
            np.testing.assert_allclose(res["O"][r], v[sorted(keys)].astype(np.float64).mean(0), atol=1e-12)
            g = (i - 1) // step
            if first is not None:
                assert ao.window_start(N, d, p, g) == first
    assert all(len(r["idx"]) == 0 for r in res["per_group"])


def test_theta_neg_inf_is_sink_plus_window_band():
    N, d, bq, ninit, w, step = 200, 16, 16, 8, 16, 2
    q, k, v = _rand(N, d, 3)
    p = ao.OracleParams(b_q=bq, n_init=ninit, w=w, step=step, theta=float("-inf"))
    res = ao.run_head(q, k, v, p)
    S = (q.astype(np.float64) @ k.astype(np.float64).T) / math.sqrt(d)
    r = np.arange(N)[:, None]
    j = np.arange(N)[None, :]
    gstart = (r // (bq * step)) * (bq * step)
    band = (j <= r) & ((j < ninit) | (j >= gstart - w))
    Sm = np.where(band, S, -np.inf)
    P = np.exp(Sm - Sm.max(1, keepdims=True))
    ref = (P / P.sum(1, keepdims=True)) @ v.astype(np.float64)
    np.testing.assert_allclose(res["O"], ref, atol=1e-12)
    np.testing.assert_allclose(res["M"], Sm.max(1), atol=1e-13)
    np.testing.assert_allclose(res["L"], P.sum(1), atol=1e-12)
    assert res["pairs"] == int(band.sum())


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("theta,all_selected", [(1.0, True), (-1.0, False)])
def test_constant_keys_closed_form(theta, all_selected):
    """All keys equal: every score of a row is the same, the pooled difference is 0,
    so theta >= 0 selects every candidate and theta < 0 none."""
    N, d, bq, ninit, w, step = 150, 8, 10, 3, 20, 2
    rng = np.random.default_rng(9)
    q = rng.standard_normal((N, d)).astype(np.float32)
    k = np.tile(rng.standard_normal((1, d)).astype(np.float32), (N, 1))
    v = rng.standard_normal((N, d)).astype(np.float32)
    p = ao.OracleParams(b_q=bq, n_init=ninit, w=w, step=step, theta=theta)
    res = ao.run_head(q, k, v, p)
    s_r = (q.astype(np.float64) @ k[0].astype(np.float64)) / math.sqrt(d)
    for r in range(N):
        G = (r // (bq * step)) * bq * step
        W = max(ninit, G - w)
        n_anchor = min(ninit, r + 1) + max(0, r - W + 1)
        n = r + 1 if all_selected else n_anchor
        assert abs(res["lse"][r] - (s_r[r] + math.log(n))) < 1e-12
        assert abs(res["M"][r] - s_r[r]) < 1e-13
        assert abs(res["L"][r] - n_anchor) < 1e-10
    for gr in res["per_group"]:
        cand = np.arange(ninit, gr["W"])
        np.testing.assert_array_equal(gr["idx"], cand if all_selected else cand[:0])
        np.testing.assert_allclose(gr["margin"][ninit:gr["W"]], -theta, atol=1e-12)


# ------------------------------------------------------- hand-worked d=1 example
def test_hand_worked_example(golden_dir):
    q = np.array([1, 1, 1, 1, 1, 1, 3, 1], np.float32)[:, None]
    k = np.array([5, 0, 1, 4.5, 2, 0, 3, 1], np.float32)[:, None]
    v = np.arange(8, dtype=np.float32)[:, None]
    with open(os.path.join(golden_dir, "hand_example_d1.txt")) as f:
        cases = [ln for ln in f if ln.startswith("theta")]
    assert len(cases) == 4
    for ln in cases:
        left, right = ln.split(":")
        theta = float(left.split()[1])
        want = [int(x) for x in right.split()]
        p = ao.OracleParams(b_q=2, n_init=1, w=2, step=1, theta=theta, sigma=0.5)
        g = ao.run_group(q, k, v, p, 3)
        assert g["W"] == 4
        np.testing.assert_array_equal(g["M"], [7.5, 2.5])
        assert g["xbar"][0] == 5.0 and g["qbar"][0, 0] == 2.0
        assert list(g["idx"]) == want
        # a key block of one column is a stripe: block granularity has the same boundary (<=)
        gb = ao.run_group(q, k, v, ao.OracleParams(b_q=2, n_init=1, w=2, step=1, theta=theta, sigma=0.5, b_kv=1), 3)
        assert list(gb["idx"]) == want
        # row 6 attends {0,4,5,6} + selected columns; scores 0.5*3*k
        keys = sorted(set([0, 4, 5, 6]) | set(want))
        e = np.array([math.exp(1.5 * float(k[j, 0])) for j in keys])
        assert abs(g["O"][0, 0] - float((e * np.array(keys)).sum() / e.sum())) < 1e-12
        assert abs(g["lse"][0] - math.log(e.sum())) < 1e-12


# ----------------------------------------------------------- brute force (tiny N)
def _brute(q, k, v, bq, ninit, w, step, theta, sigma):
    """Mask-based statement with full N x N matrices; shares nothing with the oracle."""
    q, k, v = (x.astype(np.float64) for x in (q, k, v))
    N = q.shape[0]
    S = sigma * (q @ k.T)
    rows, cols = np.arange(N)[:, None], np.arange(N)[None, :]
    blk = rows // bq
    grp = blk // step
    Wrow = np.maximum(ninit, grp * step * bq - w)
    anchor = (cols <= rows) & ((cols < ninit) | (cols >= Wrow))
    M = np.where(anchor, S, -np.inf).max(1)
    nblk = (N + bq - 1) // bq
    xbar = np.array([M[i * bq:(i + 1) * bq].mean() for i in range(nblk)])
    qbar = np.stack([q[i * bq:(i + 1) * bq].mean(0) for i in range(nblk)])
    diff = xbar[:, None] - sigma * (qbar @ k.T)                 # [nblk, N]
    ngrp = (nblk + step - 1) // step
    selg = np.zeros((ngrp, N), bool)
    for i in range(nblk):
        g = i // step
        Wg = max(ninit, g * step * bq - w)
        cand = (np.arange(N) >= ninit) & (np.arange(N) < Wg)
        selg[g] |= cand & (diff[i] <= theta)
    mask = anchor | selg[grp[:, 0]]
    Sm = np.where(mask, S, -np.inf)
    mx = Sm.max(1, keepdims=True)
    P = np.exp(Sm - mx)
    O = (P / P.sum(1, keepdims=True)) @ v
    lse = mx[:, 0] + np.log(P.sum(1))
    return dict(O=O, lse=lse, M=M, xbar=xbar, qbar=qbar, sel=selg, pairs=int(mask.sum()))


@pytest.mark.parametrize("step", [1, 2, 4])
@pytest.mark.parametrize("N", [256, 203])
def test_matches_mask_based_brute_force(step, N):
    d, bq, ninit, w = 16, 16, 4, 16
    q, k, v = _rand(N, d, 100 + step)
    u = np.zeros(d, np.float32)
    u[0] = 1.0
    q += 2.0 * u
    k[::7] += 3.0 * u                      # some columns that pass the threshold
    theta, sigma = 2.0, 1.0 / math.sqrt(d)
    p = ao.OracleParams(b_q=bq, n_init=ninit, w=w, step=step, theta=theta)
    res = ao.run_head(q, k, v, p, want_acc=True)
    ref = _brute(q, k, v, bq, ninit, w, step, theta, sigma)
    np.testing.assert_allclose(res["M"], ref["M"], atol=1e-13)
    np.testing.assert_allclose(res["xbar"], ref["xbar"], atol=1e-13)
    np.testing.assert_allclose(res["qbar"], ref["qbar"], atol=1e-14)
    for g, gr in enumerate(res["per_group"]):
        np.testing.assert_array_equal(gr["sel"].astype(bool), ref["sel"][g])
    frac = np.mean([gr["sel"][ninit:gr["W"]].mean() for gr in res["per_group"] if gr["W"] > ninit])
    assert 0.05 < frac < 0.95             # the case is discriminating: neither empty nor full
    np.testing.assert_allclose(res["O"], ref["O"], atol=1e-12)
    np.testing.assert_allclose(res["lse"], ref["lse"], atol=1e-12)
    assert res["pairs"] == ref["pairs"]
    # cached state: Acc / L is the attention over the anchor set alone
    p0 = ao.OracleParams(b_q=bq, n_init=ninit, w=w, step=step, theta=float("-inf"))
    only_anchor = ao.run_head(q, k, v, p0)
    np.testing.assert_allclose(res["Acc"] / res["L"][:, None], only_anchor["O"], atol=1e-12)


# -------------------------------------------------------------------- invariants
def test_invariants_nested_rowsum_recall():
    N, d, bq, ninit, w, step = 320, 16, 32, 8, 32, 2
    q, k, v = _rand(N, d, 77)
    k[::5, 0] += 4.0
    q[:, 0] += 2.0
    ones = np.ones_like(v)
    full = ao.run_head(q, k, ones, ao.OracleParams(bq, ninit, w, step, float("inf")))
    S = (q.astype(np.float64) @ k.astype(np.float64).T) / math.sqrt(d)
    S = np.where(np.tril(np.ones((N, N), bool)), S, -np.inf)
    Pfull = np.exp(S - full["lse"][:, None])
    prev_sets, prev_recall, prev_pairs = None, -1.0, -1
    for theta in (-1e9, 0.5, 1.5, 3.0, 1e9):
        res = ao.run_head(q, k, ones, ao.OracleParams(bq, ninit, w, step, theta))
        np.testing.assert_allclose(res["O"], 1.0, atol=1e-12)          # softmax rows sum to one
        sets = [set(gr["idx"].tolist()) for gr in res["per_group"]]
        for gr in res["per_group"]:
            assert np.all(gr["idx"] >= ninit) and np.all(gr["idx"] < gr["W"])
            assert np.all(np.diff(gr["idx"]) > 0)
        if prev_sets is not None:
            assert all(a <= b for a, b in zip(prev_sets, sets))         # nested in theta
        recall = np.exp(res["lse"] - full["lse"])
        assert np.all(recall <= 1 + 1e-12) and np.all(recall > 0)
        # recall equals the directly summed mass of full attention over P(r)
        for gr in res["per_group"]:
            r0, r1 = gr["rows"]
            for r in range(r0, r1, 13):
                keep = np.zeros(N, bool)
                keep[:min(ninit, r + 1)] = True
                keep[gr["W"]:r + 1] = True
                keep |= gr["sel"].astype(bool)
                assert abs(Pfull[r, keep].sum() - recall[r]) < 1e-12
        assert recall.mean() >= prev_recall - 1e-15 and res["pairs"] >= prev_pairs
        assert np.all(res["lse"] >= res["M"] + np.log(res["L"]) - 1e-12)  # stage 3 only adds keys
        prev_sets, prev_recall, prev_pairs = sets, recall.mean(), res["pairs"]
    assert prev_pairs == N * (N + 1) // 2 and abs(prev_recall - 1.0) < 1e-12


def test_zero_anchor_variant_selects_on_pooled_score_alone():
    """Table 4's "Without Anchor" rows set the anchor to zero: column j is kept iff
    -sigma * <qbar_i, k_j> <= theta for some block of the group."""
    N, d, bq, ninit, w, step, theta = 192, 8, 16, 4, 16, 2, -0.3
    q, k, v = _rand(N, d, 5)
    p = ao.OracleParams(bq, ninit, w, step, theta)
    sigma = 1.0 / math.sqrt(d)
    for g in range(ao.n_groups(N, p)):
        res = ao.run_group(q, k, v, p, g, attend=False, zero_anchor=True)
        want = np.zeros(N, bool)
        for b in range(step):
            i = g * step + b
            if i * bq >= N:
                break
            qbar = q[i * bq:(i + 1) * bq].astype(np.float64).mean(0)
            s = sigma * (k.astype(np.float64) @ qbar)
            want |= (-s <= theta)
        want[:ninit] = False
        want[res["W"]:] = False
        np.testing.assert_array_equal(res["sel"].astype(bool), want)


# ------------------------------------------- block granularity (Sec. 2.1.2, Table 1)
def test_block_granularity_with_unit_blocks_is_stripe_granularity():
    """A key block of one column is a stripe: both tests must keep the same columns."""
    N, d, bq, ninit, w, step, theta = 160, 8, 16, 4, 16, 2, 1.2
    q, k, v = _rand(N, d, 21)
    k[::6, 0] += 3.0
    q[:, 0] += 2.0
    stripe = ao.run_head(q, k, v, ao.OracleParams(bq, ninit, w, step, theta))
    block = ao.run_head(q, k, v, ao.OracleParams(bq, ninit, w, step, theta, b_kv=1))
    picked = 0
    for a, b in zip(stripe["per_group"], block["per_group"]):
        np.testing.assert_array_equal(a["sel"], b["sel"])
        np.testing.assert_allclose(a["margin"], b["margin"], atol=1e-13)
        picked += int(a["sel"].sum())
    assert picked > 0
    np.testing.assert_allclose(stripe["O"], block["O"], atol=1e-13)


def test_block_margin_is_mean_of_stripe_margins_for_one_query_block():
    """The pooled score is linear in the key, so with step = 1 (a single xbar, no min over blocks)
    the block margin equals the mean of the stripe margins of the block's columns."""
    N, d, bq, ninit, w, theta = 256, 16, 32, 32, 32, 0.7
    q, k, v = _rand(N, d, 31)
    for g in (3, 5, 7):
        s = ao.run_group(q, k, v, ao.OracleParams(bq, ninit, w, 1, theta), g, attend=False)
        b = ao.run_group(q, k, v, ao.OracleParams(bq, ninit, w, 1, theta, b_kv=32), g, attend=False)
        for J in range(ninit // 32, s["W"] // 32):
            blk = slice(32 * J, 32 * J + 32)
            assert np.all(b["margin"][blk] == b["margin"][32 * J])
            assert abs(b["margin"][32 * J] - s["margin"][blk].mean()) < 1e-13
            assert np.all(b["sel"][blk] == (b["margin"][32 * J] <= 0))
        assert not b["sel"][:ninit].any() and not b["sel"][s["W"]:].any()


def test_block_granularity_on_blockwise_constant_keys_equals_stripe():
    """If every key of a block equals the block mean, the two granularities see the same scores."""
    N, d, bq, ninit, w, step, theta, bkv = 256, 8, 16, 16, 16, 2, 0.4, 16
    q, _, v = _rand(N, d, 41)
    rng = np.random.default_rng(42)
    k = np.repeat(rng.standard_normal((N // bkv, d)).astype(np.float32), bkv, axis=0)
    stripe = ao.run_head(q, k, v, ao.OracleParams(bq, ninit, w, step, theta), attend=False)
    block = ao.run_head(q, k, v, ao.OracleParams(bq, ninit, w, step, theta, b_kv=bkv), attend=False)
    sizes = []
    for a, b in zip(stripe["per_group"], block["per_group"]):
        np.testing.assert_array_equal(a["sel"], b["sel"])
        sizes.append(a["sel"][ninit:a["W"]].mean() if a["W"] > ninit else np.nan)
    assert 0.05 < np.nanmean(sizes) < 0.95


@pytest.mark.parametrize("step", [1, 3])
def test_block_granularity_matches_brute_force(step):
    """Independent statement with full matrices: pooled queries x pooled keys, OR over the group."""
    N, d, bq, bkv, ninit, w, theta = 288, 8, 16, 16, 16, 32, 2.2
    q, k, v = _rand(N, d, 51 + step)
    k[64:80] += 1.5                                  # two whole key blocks with a shifted mean
    k[160:176] += 1.5
    q += 0.5
    sigma = 1.0 / math.sqrt(d)
    res = ao.run_head(q, k, v, ao.OracleParams(bq, ninit, w, step, theta, b_kv=bkv))
    q64, k64, v64 = (x.astype(np.float64) for x in (q, k, v))
    S = sigma * (q64 @ k64.T)
    rows, cols = np.arange(N)[:, None], np.arange(N)[None, :]
    grp_of_row = (rows // bq) // step
    Wrow = np.maximum(ninit, grp_of_row * step * bq - w)
    anchor = (cols <= rows) & ((cols < ninit) | (cols >= Wrow))
    M = np.where(anchor, S, -np.inf).max(1)
    nblk = N // bq
    xbar = M.reshape(nblk, bq).mean(1)
    qbar = q64.reshape(nblk, bq, d).mean(1)
    kbar = k64.reshape(N // bkv, bkv, d).mean(1)
    diff = xbar[:, None] - sigma * (qbar @ kbar.T)   # [query block, key block]
    mask = anchor.copy()
    some = 0
    for g, gr in enumerate(res["per_group"]):
        Wg = max(ninit, g * step * bq - w)
        blocks = diff[g * step:(g + 1) * step].min(0) <= theta
        want = np.repeat(blocks, bkv)
        want[:ninit] = False
        want[Wg:] = False
        np.testing.assert_array_equal(gr["sel"].astype(bool), want)
        some += int(want.sum())
        r0, r1 = gr["rows"]
        mask[r0:r1] |= want[None, :]
    assert 0 < some < res["pairs"]
    Sm = np.where(mask, S, -np.inf)
    mx = Sm.max(1, keepdims=True)
    P = np.exp(Sm - mx)
    np.testing.assert_allclose(res["O"], (P / P.sum(1, keepdims=True)) @ v64, atol=1e-12)
    assert res["pairs"] == int(mask.sum())


def test_block_granularity_rejects_unaligned_regions():
    q, k, v = _rand(128, 8, 61)
    with pytest.raises(ValueError):
        ao.run_group(q, k, v, ao.OracleParams(16, 4, 16, 1, 0.0, b_kv=16), 4, attend=False)
