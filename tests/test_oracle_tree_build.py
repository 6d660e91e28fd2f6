"""Pins for the oracle's best-first tree build (CPU only).

Each test checks the C oracle against something other than itself: exhaustive enumeration
(Prop. 3.3), a hand-worked example (Eq. 1), closed forms, and the Monte-Carlo meaning of the
surrogate (Prop. 3.2 / Lemma 3.1).
"""
import json
import os

import numpy as np
import pytest

from oracle import bruteforce as bf
from paper_2605_29727_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _same_tree(a, b):
    for k in ("parent", "token", "depth", "rank"):
        assert np.array_equal(a[k], b[k]), k
    assert np.array_equal(a["rho"].view(np.uint32), b["rho"].view(np.uint32)), "rho bits"


def test_hand_worked_example(oracle):
    g = json.load(open(os.path.join(GOLD, "tree_build_hand_2x3.json")))
    marg = np.array(g["marginals"], dtype=np.float32)
    t = oracle.tree_build(marg, g["N"])
    assert t["n"] == g["N"]
    assert t["rho"].tolist() == g["rho"]
    assert t["depth"].tolist() == g["depth"]
    assert t["token"].tolist() == g["token"]
    assert t["parent"].tolist() == g["parent"]
    for n, a in g["ahat_by_N"].items():
        assert oracle.tree_build(marg, int(n))["ahat"] == a


@pytest.mark.parametrize("B,V", [(2, 3), (3, 3), (2, 5), (4, 3), (3, 4), (2, 6)])
@pytest.mark.parametrize("sigma", [0.5, 2.0, 5.0])
def test_equals_exhaustive_enumeration(oracle, B, V, sigma):
    """Prop. 3.3 + proof step 2: best-first = the top-N prefixes of the whole lattice, in order."""
    lattice = sum(V ** d for d in range(1, B + 1))
    for seed in range(3):
        marg = synth.marginals(100 + seed, B, V, sigma)
        for N in sorted({1, 2, V, V + 1, lattice // 2, lattice - 1, lattice, lattice + 5}):
            t = oracle.tree_build(marg, N)
            ref = bf.tree_build_bruteforce(marg, N)
            assert t["n"] == ref["n"] == min(N, lattice)
            _same_tree(t, ref)
            assert abs(t["ahat"] - ref["ahat"]) < 1e-12


def test_exhaustive_on_ties_zeros_and_one_hot(oracle):
    """Adversarial marginals: exact ties, a one-hot position (q=1) and zeros."""
    cases = [
        np.array([[0.25, 0.25, 0.25, 0.25], [0.25, 0.25, 0.25, 0.25], [0.5, 0.5, 0.0, 0.0]], dtype=np.float32),
        np.array([[0.0, 1.0, 0.0], [0.5, 0.5, 0.0], [0.0, 0.0, 1.0]], dtype=np.float32),
        np.array([[0.5, 0.5], [0.5, 0.5], [0.5, 0.5], [0.5, 0.5]], dtype=np.float32),
        np.array([[0.7, 0.2, 0.1], [0.1, 0.2, 0.7]], dtype=np.float32),
    ]
    for marg in cases:
        B, V = marg.shape
        lattice = sum(V ** d for d in range(1, B + 1))
        for N in range(1, lattice + 1):
            _same_tree(oracle.tree_build(marg, N), bf.tree_build_bruteforce(marg, N))


def test_config1_equals_exhaustive_enumeration(oracle):
    """The tiny benchmark configuration (B=4, V=64, N=16): full lattice has ~1.7e7 prefixes; the
    enumeration is pruned to tokens of rank < N at each position, which is lossless because a rank-j
    sibling is preceded by its j earlier siblings."""
    w = synth.C1
    marg = synth.marginals(w.seed, w.B, w.V, w.marg_sigma)
    t = oracle.tree_build(marg, w.N)
    order = oracle.rank_tokens(marg)
    keep = w.N + 1   # 17 + 17^2 + 17^3 + 17^4 = 88740 prefixes; ranks >= N can never be emitted
    assert int(t["rank"].max()) < keep - 1
    sub = np.stack([marg[k, order[k, :keep]] for k in range(w.B)])
    ref = bf.tree_build_bruteforce(sub, w.N)
    assert np.array_equal(ref["parent"], t["parent"]) and np.array_equal(ref["rank"], t["rank"])
    assert np.array_equal(ref["rho"].view(np.uint32), t["rho"].view(np.uint32))
    assert np.array_equal(order[t["depth"] - 1, t["rank"]], t["token"])


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5])
def test_optimal_among_all_prefix_closed_trees(oracle, N):
    """Prop. 3.3 as stated: T_N maximises sum rho over ALL size-N prefix-closed trees."""
    for seed, (B, V) in enumerate([(2, 3), (3, 2), (2, 4)]):
        marg = synth.marginals(200 + seed, B, V, 1.5)
        t = oracle.tree_build(marg, N)
        best = bf.best_surrogate_any_tree(marg, N)
        assert abs((t["ahat"] - 1.0) - best) < 1e-6
        assert t["ahat"] - 1.0 >= best - 1e-6


@pytest.mark.parametrize("seed", range(4))
def test_invariants_large_vocab(oracle, seed):
    """Eq. 4 (path monotonicity), Eq. 5 (rho non-increasing => concave Ahat), nestedness and
    prefix-closure (proof step 3), at a vocabulary where enumeration is impossible."""
    B, V = 16, 4096
    marg = synth.marginals(300 + seed, B, V, [1.0, 3.0, 5.0, 8.0][seed])
    big = oracle.tree_build(marg, 256)
    p, rho, d, tok, rk = big["parent"], big["rho"], big["depth"], big["token"], big["rank"]
    assert np.all(np.diff(rho) <= 0)
    assert np.all(p < np.arange(len(p))) and np.all(p >= -1)
    order = oracle.rank_tokens(marg)
    for i in range(len(p)):
        prho = np.float32(1.0) if p[i] < 0 else rho[p[i]]
        assert d[i] == (1 if p[i] < 0 else d[p[i]] + 1) and d[i] <= B
        assert tok[i] == order[d[i] - 1, rk[i]]
        assert rho[i] == np.float32(prho * marg[d[i] - 1, tok[i]])      # Eq. 1, one fp32 multiply per edge
        assert rho[i] <= prho                                             # Eq. 4
        if rk[i] > 0:   # previous sibling is in the tree and came earlier
            sib = [j for j in range(i) if p[j] == p[i] and rk[j] == rk[i] - 1]
            assert len(sib) == 1
    for n in (1, 7, 64, 255):
        small = oracle.tree_build(marg, n)
        for k in ("parent", "token", "depth", "rank"):
            assert np.array_equal(small[k], big[k][:n])
        assert abs(small["ahat"] - (1.0 + rho[:n].astype(np.float64).sum())) < 1e-9   # Eq. 3


def test_beats_beam_and_random_trees(oracle):
    """Prop. 3.3 against two feasible competitors of equal size: a width x depth beam rectangle
    (Sec. 3.3: beam allocation is mismatched) and random prefix-closed trees."""
    B, V, w, dep = 8, 512, 4, 4
    for seed in range(5):
        marg = synth.marginals(400 + seed, B, V, 3.0)
        order = oracle.rank_tokens(marg)
        # beam search: keep the w best prefixes per depth
        beams = [((), 1.0)]
        total, count = 0.0, 0
        for k in range(dep):
            cand = [(rp + (r,), s * float(marg[k, order[k, r]])) for rp, s in beams for r in range(w)]
            cand.sort(key=lambda c: -c[1])
            beams = cand[:w]
            total += sum(s for _, s in beams); count += len(beams)
        t = oracle.tree_build(marg, count)
        assert t["ahat"] - 1.0 >= total - 1e-6
        # random prefix-closed trees of the same size
        rnd = synth.raw_u64(seed, "rand_tree", 4 * count)
        nodes, frontier, s = [], [((0,), float(marg[0, order[0, 0]]))], 0.0
        for i in range(count):
            j = int(rnd[i] % np.uint64(len(frontier)))
            rp, sc = frontier.pop(j)
            nodes.append(rp); s += sc
            if len(rp) < B:
                frontier.append((rp + (0,), sc * float(marg[len(rp), order[len(rp), 0]])))
            if rp[-1] + 1 < V:
                par = sc / float(marg[len(rp) - 1, order[len(rp) - 1, rp[-1]]])
                frontier.append((rp[:-1] + (rp[-1] + 1,), par * float(marg[len(rp) - 1, order[len(rp) - 1, rp[-1] + 1]])))
        assert t["ahat"] - 1.0 >= s - 1e-6


def test_closed_forms(oracle):
    B, V = 4, 5
    # every position one-hot: the chain has rho = 1, everything else rho = 0 in (depth, rank path) order
    marg = np.zeros((B, V), dtype=np.float32)
    hot = [3, 0, 4, 1]
    for k in range(B):
        marg[k, hot[k]] = 1.0
    t = oracle.tree_build(marg, 12)
    assert t["token"][:B].tolist() == hot and t["parent"][:B].tolist() == [-1, 0, 1, 2]
    assert t["rho"][:B].tolist() == [1.0] * B and np.all(t["rho"][B:] == 0.0)
    assert t["ahat"] == 1.0 + B
    assert t["depth"][B:].tolist() == [1, 1, 1, 1, 2, 2, 2, 2]          # zeros: shallow first
    assert t["token"][B:B + 4].tolist() == [0, 1, 2, 4]                    # then token id ascending
    # every position uniform: pure breadth-first order by (depth, rank path)
    marg = np.full((3, 4), 0.25, dtype=np.float32)
    t = oracle.tree_build(marg, 4 + 16 + 5)
    assert t["depth"].tolist() == [1] * 4 + [2] * 16 + [3] * 5
    assert t["token"][:4].tolist() == [0, 1, 2, 3]
    assert t["parent"][4:20].tolist() == [i // 4 for i in range(16)]
    assert t["token"][4:20].tolist() == [i % 4 for i in range(16)]
    assert t["parent"][20:].tolist() == [4] * 4 + [5]
    # budget larger than the lattice: everything is emitted, nothing more
    t = oracle.tree_build(np.array([[0.6, 0.4]], dtype=np.float32), 10)
    assert t["n"] == 2 and t["token"].tolist() == [0, 1]


def test_surrogate_is_expected_self_verified_length(oracle):
    """Prop. 3.2 with Lemma 3.1: draw X_k ~ q_k independently; the committed length (root included)
    is the number of tree nodes whose path equals the sample's prefix; its mean is 1 + sum rho."""
    B, V, N, S = 6, 32, 40, 100_000
    marg = synth.marginals(7, B, V, 2.0)
    t = oracle.tree_build(marg, N)
    cdf = np.cumsum(marg.astype(np.float64), axis=1)
    u = synth.uniform(7, "mc", (S, B))
    X = np.stack([np.minimum(np.searchsorted(cdf[k], u[:, k] * cdf[k, -1], side="right"), V - 1) for k in range(B)], axis=1)
    children = {}
    for i in range(N):
        children[(int(t["parent"][i]), int(t["token"][i]))] = i
    lengths = np.empty(S)
    for s in range(S):
        cur, n = -1, 1
        for k in range(B):
            nxt = children.get((cur, int(X[s, k])))
            if nxt is None:
                break
            cur, n = nxt, n + 1
        lengths[s] = n
    se = lengths.std() / np.sqrt(S)
    assert abs(lengths.mean() - t["ahat"]) < 4 * se + 1e-9


def test_rank_tokens_tie_order(oracle):
    marg = np.array([[0.2, 0.3, 0.2, 0.3]], dtype=np.float32)
    assert oracle.rank_tokens(marg)[0].tolist() == [1, 3, 0, 2]
