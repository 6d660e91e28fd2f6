"""Pins for the oracle's beam-search tree (Sec. 4.3's comparison topology), CPU only.

Hand-worked cases, the greedy chain (width 1) against numpy's argmax and cumulative product, the full lattice
(width at least V^depth), per-depth selection against numpy's stable sort of explicitly enumerated extensions, and
Prop. 3.3: no beam tree beats the best-first tree of the same size under the surrogate.
"""
import json
import os

import numpy as np
import pytest

from paper_2605_29727_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_cases(oracle):
    g = json.load(open(os.path.join(GOLD, "beam_hand_2x3.json")))
    marg = np.array(g["marginals"], dtype=np.float32)
    for c in g["cases"]:
        t = oracle.tree_build_beam(marg, c["width"], c["depth"])
        assert t["n"] == len(c["parent"])
        assert t["parent"].tolist() == c["parent"] and t["token"].tolist() == c["token"]
        assert t["depth"].tolist() == c["node_depth"] and t["rho"].tolist() == c["rho"]
        assert t["ahat"] == c["ahat"]


@pytest.mark.parametrize("seed", range(4))
def test_width_one_is_the_greedy_chain(oracle, seed):
    B, V = 16, 997
    marg = synth.marginals(500 + seed, B, V, 3.0)
    t = oracle.tree_build_beam(marg, 1, B)
    assert t["n"] == B and t["parent"].tolist() == list(range(-1, B - 1))
    assert t["token"].tolist() == marg.argmax(axis=1).tolist()             # numpy: first index on ties, as here
    best = marg.max(axis=1)
    assert np.array_equal(t["rho"], np.cumprod(best, dtype=np.float32))     # one fp32 multiply per edge, in order
    assert t["ahat"] == pytest.approx(1.0 + np.cumprod(best, dtype=np.float32).astype(np.float64).sum(), rel=1e-12)


def test_full_width_is_the_whole_lattice(oracle):
    B, V, d = 3, 3, 3
    marg = synth.marginals(7, B, V, 1.0)
    t = oracle.tree_build_beam(marg, V ** d, d)
    assert t["n"] == V + V ** 2 + V ** 3
    assert np.bincount(t["depth"])[1:].tolist() == [V, V ** 2, V ** 3]
    # every node has each token exactly once among its children
    for p in range(-1, V + V ** 2):
        kids = t["token"][t["parent"] == p]
        assert sorted(kids.tolist()) == list(range(V))
    # sum of rho over a full depth = product of the row sums (each close to 1)
    for k in range(1, d + 1):
        want = np.prod(marg[:k].astype(np.float64).sum(axis=1))
        assert t["rho"][t["depth"] == k].astype(np.float64).sum() == pytest.approx(want, rel=1e-5)


@pytest.mark.parametrize("V,width,depth", [(5, 2, 4), (7, 3, 5), (4, 4, 3), (50, 6, 6), (3, 8, 4), (200, 16, 8)])
def test_each_depth_keeps_the_top_extensions(oracle, V, width, depth):
    """The definition, depth by depth, with numpy: all extensions of the kept prefixes, stable sort by -rho (ties
    then fall to the flattened index = parent's place * V + rank)."""
    for seed in range(3):
        marg = synth.marginals(600 + seed, depth, V, [0.5, 2.0, 5.0][seed])
        order = oracle.rank_tokens(marg)
        t = oracle.tree_build_beam(marg, width, depth)
        prev_rho, prev_ids, n = np.ones(1, dtype=np.float32), np.array([-1]), 0
        for k in range(depth):
            qs = marg[k, order[k]]                                        # probabilities by rank
            ext = (prev_rho[:, None] * qs[None, :]).astype(np.float32)    # fp32 products
            flat = np.argsort(-ext.ravel(), kind="stable")[:width]
            pp, rk = flat // V, flat % V
            m = len(flat)
            assert t["parent"][n:n + m].tolist() == prev_ids[pp].tolist()
            assert t["rank"][n:n + m].tolist() == rk.tolist()
            assert t["token"][n:n + m].tolist() == order[k, rk].tolist()
            assert np.array_equal(t["rho"][n:n + m], ext.ravel()[flat])
            assert np.all(t["depth"][n:n + m] == k + 1)
            prev_rho, prev_ids, n = ext.ravel()[flat], np.arange(n, n + m), n + m
        assert t["n"] == n
        assert t["ahat"] == pytest.approx(1.0 + t["rho"].astype(np.float64).sum(), rel=1e-12)


@pytest.mark.parametrize("width,depth", [(4, 4), (4, 15), (2, 8), (8, 8), (16, 16), (1, 16)])
def test_best_first_is_at_least_as_good(oracle, width, depth):
    """Prop. 3.3: the best-first tree maximises the surrogate among prefix-closed trees of its size; a beam tree is
    one of them (Sec. 4.3 compares the two at a matched budget, beam 4 x 15 against N = 61 with the root)."""
    for seed, sigma in enumerate([1.0, 3.0, 5.0]):
        marg = synth.marginals(700 + seed, 16, 4096, sigma)
        b = oracle.tree_build_beam(marg, width, depth)
        f = oracle.tree_build(marg, b["n"])
        assert f["ahat"] >= b["ahat"] - 1e-9
        # the beam tree is prefix-closed and rectangular
        assert np.all(b["parent"] < np.arange(b["n"]))
        assert np.bincount(b["depth"])[1:].tolist() == [width] * depth
        for i in range(b["n"]):
            assert b["depth"][i] == (1 if b["parent"][i] < 0 else b["depth"][b["parent"][i]] + 1)


def test_bad_arguments(oracle):
    marg = synth.marginals(1, 4, 8, 1.0)
    for w, d in [(0, 2), (2, 0), (2, 5)]:
        with pytest.raises(ValueError):
            oracle.tree_build_beam(marg, w, d)


def test_fig4_ordering_on_drafter_like_marginals(oracle):
    """The shape of the Sec. 4.3 comparison by the surrogate alone: at a matched budget best-first is ahead of the
    4 x 15 beam, and both are ahead of the single chain of 16 (which is not budget-matched)."""
    for seed in range(3):
        marg = synth.marginals_drafter_like(seed, 16, 4096)
        assert np.allclose(marg.sum(axis=1), 1.0, atol=1e-5) and marg.min() >= 0.0
        assert np.allclose(marg.max(axis=1), 0.9 * 0.93 ** np.arange(16), rtol=1e-5)
        bf = oracle.tree_build(marg, 60)["ahat"]
        beam = oracle.tree_build_beam(marg, 4, 15)["ahat"]
        chain = oracle.tree_build_beam(marg, 1, 16)["ahat"]
        assert bf > beam > chain > 1.0
