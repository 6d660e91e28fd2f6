"""Pins for the oracle's adaptive budget controller (Algorithm 1, Sec. 3.4) and verifier cost model (App. E).  CPU only.

The controller is checked against hand-worked stops, against the fixed-budget builder (the adaptive tree must be
a prefix of the best-first order, Prop. 3.3), and against Prop. 3.4: for a convex cost the first decrease of the
estimated speedup is its global maximum, found here by evaluating every budget from the fixed-budget scores.
The cost model (sums of the per-module tables) is checked against the appendix's closed-form totals and limits.
"""
import json
import os

import numpy as np
import pytest

from paper_2605_29727_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_stops(oracle):
    g = json.load(open(os.path.join(GOLD, "adaptive_hand_2x3.json")))
    marg = np.array(g["marginals"], dtype=np.float32)
    for case in g["cases"]:
        cost = case["cost_offset"] + case["cost_slope"] * np.arange(1, g["N_max"] + 1, dtype=np.float64)
        t = oracle.tree_build_adaptive(marg, g["N_max"], cost, case["L_AR"])
        assert t["n"] == case["n_star"], case["_derivation"]
        assert t["s_best"] == pytest.approx(case["s_star"], rel=1e-15)
        assert t["ahat"] == case["ahat"]


@pytest.mark.parametrize("sigma,seed", [(1.0, 1), (2.0, 2), (3.0, 3), (5.0, 4), (8.0, 5)])
def test_is_a_prefix_of_the_fixed_budget_tree(oracle, sigma, seed):
    marg = synth.marginals(seed, 8, 500, sigma)
    N_max = 200
    full = oracle.tree_build(marg, N_max)
    cost = 3.0 + 0.05 * np.arange(1, N_max + 1) + 2e-4 * np.arange(1, N_max + 1) ** 2
    t = oracle.tree_build_adaptive(marg, N_max, cost, 1.0)
    n = t["n"]
    assert 1 <= n <= N_max
    for k in ("parent", "token", "depth", "rank"):
        assert np.array_equal(t[k], full[k][:n]), k
    assert np.array_equal(t["rho"].view(np.uint32), full["rho"][:n].view(np.uint32))
    assert t["ahat"] == pytest.approx(1.0 + full["rho"][:n].astype(np.float64).sum(), rel=1e-14)


@pytest.mark.parametrize("sigma,seed", [(1.0, 11), (2.0, 12), (3.0, 13), (5.0, 14)])
@pytest.mark.parametrize("curve", ["affine", "quadratic", "kink"])
def test_first_decrease_is_the_global_maximum_for_convex_cost(oracle, sigma, seed, curve):
    """Prop. 3.4: Ahat concave and non-decreasing (it always is: Eq. 5), C convex and positive => the first budget
    at which S decreases maximises S.  The maximum is found by brute force over all budgets."""
    marg = synth.marginals(seed, 6, 300, sigma)
    N_max = 150
    N = np.arange(1, N_max + 1, dtype=np.float64)
    cost = {"affine": 2.0 + 0.07 * N,
            "quadratic": 5.0 + 0.01 * N + 5e-4 * N ** 2,
            "kink": np.maximum(4.0 + 0.001 * N, 0.2 * N - 3.0)}[curve]     # roofline-like: flat, then linear
    full = oracle.tree_build(marg, N_max)
    ahat = 1.0 + np.cumsum(full["rho"].astype(np.float64))
    S = ahat[:full["n"]] / cost[:full["n"]]
    best = int(np.argmax(S)) + 1                                          # smallest maximiser
    t = oracle.tree_build_adaptive(marg, N_max, cost, 1.0)
    if t["margin"] > 1e-12:                                              # no comparison was a near-tie
        assert t["n"] == best
        assert t["s_best"] == pytest.approx(S[best - 1], rel=1e-13)
    assert np.all(np.diff(S[:t["n"]]) > -1e-15)                           # non-decreasing up to the stop


def test_speedup_scales_with_the_ar_latency_and_stop_does_not(oracle):
    marg = synth.marginals(21, 5, 200, 3.0)
    cost = 1.0 + 0.03 * np.arange(1, 101)
    a = oracle.tree_build_adaptive(marg, 100, cost, 1.0)
    b = oracle.tree_build_adaptive(marg, 100, cost, 7.5)
    assert a["n"] == b["n"]
    assert b["s_best"] == pytest.approx(7.5 * a["s_best"], rel=1e-14)


def test_budget_exhausts_the_lattice(oracle):
    marg = np.array([[0.6, 0.4]], dtype=np.float32)                       # two prefixes in all
    t = oracle.tree_build_adaptive(marg, 10, np.ones(10), 1.0)
    assert t["n"] == 2 and t["ahat"] == pytest.approx(2.0, rel=1e-7)


def test_bad_arguments_are_refused(oracle):
    marg = synth.marginals(1, 2, 8, 1.0)
    with pytest.raises(ValueError):
        oracle.tree_build_adaptive(marg, 4, np.array([1.0, 0.0, 1.0, 1.0]), 1.0)     # non-positive cost
    with pytest.raises(ValueError):
        oracle.tree_build_adaptive(marg, 4, np.ones(4), 0.0)                         # non-positive L_AR


# ---- cost model (App. E) ------------------------------------------------------------------------------------
def _totals(s, c, L, h, nq, nkv, d, hffn, V, bp):
    """The appendix's closed-form totals (its two displayed equations), as printed."""
    hq, hkv = nq * d, nkv * d
    flops = L * (4 * s * h * hq + 4 * s * h * hkv + 4 * s * (c + s) * hq + 6 * s * h * hffn) + 2 * s * h * V
    byts = bp * (2 * V * h + s * (h + V) + L * (2 * h * (hq + hkv) + 3 * h * hffn + 2 * hkv * (c + 2 * s)
                                                + 4 * s * (h + hq + hffn) + 2 * nq * s * (c + s)))
    return float(flops), float(byts)


@pytest.mark.parametrize("cfg", [
    dict(s=64, c=8192, L=32, h=4096, nq=32, nkv=8, d=128, hffn=14336, V=128256, bp=2),       # Llama-3-8B shape
    dict(s=128, c=32768, L=80, h=8192, nq=64, nkv=8, d=128, hffn=28672, V=128256, bp=2),     # 70B shape
    dict(s=1, c=10, L=2, h=8, nq=2, nkv=1, d=4, hffn=16, V=50, bp=4),
    dict(s=7, c=0, L=3, h=12, nq=3, nkv=3, d=4, hffn=20, V=33, bp=1),
])
def test_module_sums_equal_the_printed_totals(oracle, cfg):
    r = oracle.verify_cost(cfg["s"], cfg["c"], cfg["L"], cfg["h"], cfg["nq"], cfg["nkv"], cfg["d"], cfg["hffn"], cfg["V"],
                           cfg["bp"], 1e15, 1e12)
    flops, byts = _totals(**cfg)
    assert r["flops"] == pytest.approx(flops, rel=1e-14)
    assert r["bytes"] == pytest.approx(byts, rel=1e-14)
    assert r["roofline_s"] == pytest.approx(max(flops / 1e15, byts / 1e12), rel=1e-14)


def test_small_configuration_by_hand(oracle):
    """s=1, c=2, one layer, h=2, one 2-wide head for Q and for KV, hffn=3, V=5, 1 byte per element.
    FLOPs: Q 2*1*2*2=8, KV 4*1*2*2=16, scores 2*1*3*2=12, PV 12, out 8, gate/up 4*1*2*3=24, down 2*1*3*2=12, LM head
    2*1*2*5=20: 112.  Elements: weights 2*5*2=20 + attention 2*2*2+2*2*2=16 + FFN 3*2*3=18; KV read 2*2*2=8, write
    2*1*2=4; activations attention 2*1*2+4*1*2+2*1*2+2*1*1*3=22, FFN 2*1*2+4*1*3=16, LM head 1*2+1*5=7: 111."""
    r = oracle.verify_cost(1, 2, 1, 2, 1, 1, 2, 3, 5, 1, 56.0, 37.0, 2.0, 0.5)
    assert r["flops"] == 112.0 and r["bytes"] == 111.0
    assert r["roofline_s"] == pytest.approx(3.0)            # max(112/56, 111/37) = max(2, 3)
    assert r["latency_s"] == pytest.approx(6.5)             # 2 * 3 + 0.5


def test_limits(oracle):
    base = dict(c=4096, L=4, h=256, nq=4, nkv=2, d=64, hffn=512, V=1000, bp=2)
    z = oracle.verify_cost(0, peak_flops=1e12, bandwidth=1e11, layers=base["L"], **{k: v for k, v in base.items() if k != "L"})
    assert z["flops"] == 0.0                                 # nothing to verify: no arithmetic,
    hkv = base["nkv"] * base["d"]; hq = base["nq"] * base["d"]
    weights = 2 * base["V"] * base["h"] + base["L"] * (2 * base["h"] * (hq + hkv) + 3 * base["h"] * base["hffn"])
    assert z["bytes"] == pytest.approx(base["bp"] * (weights + base["L"] * 2 * base["c"] * hkv))   # weights + KV read
    # Memory-bound at small s (weights dominate: about 2s/bp flop per byte), compute-bound at large s on a machine
    # whose ridge (10 flop/B here) lies below the model's asymptotic intensity 2d/bp = 64 flop/B (the score matrix
    # of the non-fused attention is counted as traffic): the roofline switches sides.
    small = oracle.verify_cost(1, peak_flops=1e13, bandwidth=1e12, layers=4, **{k: v for k, v in base.items() if k != "L"})
    large = oracle.verify_cost(100000, peak_flops=1e13, bandwidth=1e12, layers=4, **{k: v for k, v in base.items() if k != "L"})
    assert small["roofline_s"] == pytest.approx(small["bytes"] / 1e12)
    assert large["roofline_s"] == pytest.approx(large["flops"] / 1e13)
