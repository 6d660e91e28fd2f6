"""Pins for the oracle's acceptance walks (CPU only)."""
import numpy as np
import pytest

from oracle import bruteforce as bf
from paper_2605_29727_amd import synth


def _depths(parent):
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(len(parent)):
        d[i] = 1 if parent[i] < 0 else d[parent[i]] + 1
    return d


# ---------------------------------------------------------------- greedy ----

def test_argmax_lowest_index_on_ties(oracle):
    x = np.array([[1, 5, 5, 2], [7, 7, 7, 7], [-3, -1, -1, -2], [0, 0, 1, 1]], dtype=np.float32)
    assert oracle.row_argmax(x).tolist() == [1, 0, 1, 2]
    big, _ = synth.target_logits(1, 5, 4096, 1.0, "bf16")
    f = synth.bf16_bits_to_f32(big)
    assert np.array_equal(oracle.row_argmax(f), np.argmax(f, axis=1))   # numpy: first maximal index


@pytest.mark.parametrize("kind", ["chain", "star", "binary", "caterpillar", "random", "deep"])
def test_greedy_equals_scoring_every_path(oracle, kind):
    """App. C 'Acceptance': the walk equals scoring every root-to-node path and keeping the longest match."""
    N, V = 40, 50
    parent = synth.tree_parents(21, N, kind)
    token = synth.sibling_distinct_tokens(21, parent, V)
    _, logits = synth.target_logits(22, N + 1, V, 1.0, "fp32", tag=kind)
    depth = _depths(parent)
    leaves = [-1] + [int(i) for i in np.argsort(-depth)[:3]] + [0, N // 2]
    for leaf in leaves:
        x = synth.plant_path(logits, parent, token, leaf)
        got = oracle.accept_greedy(x, parent, token)
        ref = bf.accept_greedy_bruteforce(np.argmax(x, axis=1), parent, token)
        assert got["n_acc"] == ref["n_acc"] and np.array_equal(got["path"], ref["path"]) and got["bonus"] == ref["bonus"]
        if leaf >= 0:
            assert got["n_acc"] >= depth[leaf]            # the planted path is accepted at least to its leaf
            assert got["path"][depth[leaf] - 1] == leaf


def test_greedy_all_miss_and_full_chain(oracle):
    N, V = 6, 10
    parent = synth.tree_parents(0, N, "chain")
    token = np.arange(N, dtype=np.int32) + 1
    x = np.zeros((N + 1, V), dtype=np.float32)
    x[:, 0] = 1.0                                            # target always says token 0: nothing matches
    r = oracle.accept_greedy(x, parent, token)
    assert r["n_acc"] == 0 and r["bonus"] == 0 and len(r["path"]) == 0
    x = np.zeros((N + 1, V), dtype=np.float32)
    for i in range(N):
        x[i, token[i]] = 1.0                                 # row of the parent predicts the child's token
    x[N, 9] = 1.0
    r = oracle.accept_greedy(x, parent, token)
    assert r["n_acc"] == N and r["path"].tolist() == list(range(N)) and r["bonus"] == 9


def test_greedy_with_oracle_tree_monte_carlo(oracle):
    """Prop. 3.2 through build + accept together: one-hot 'target logits' that put a drafter sample X
    along the path give accepted length + 1 with mean 1 + sum rho."""
    B, V, N, S = 5, 16, 30, 4000
    marg = synth.marginals(31, B, V, 1.5)
    t = oracle.tree_build(marg, N)
    cdf = np.cumsum(marg.astype(np.float64), axis=1)
    u = synth.uniform(31, "mc", (S, B))
    tot = np.empty(S)
    for s in range(S):
        X = [min(int(np.searchsorted(cdf[k], u[s, k] * cdf[k, -1], side="right")), V - 1) for k in range(B)]
        x = np.zeros((N + 1, V), dtype=np.float32)
        x[0, X[0]] = 1.0
        for i in range(N):
            d = int(t["depth"][i])
            if d < B:
                x[i + 1, X[d]] = 1.0                        # the verifier at a depth-d node says X_{d+1}
        tot[s] = oracle.accept_greedy(x, t["parent"], t["token"])["n_acc"] + 1
    assert abs(tot.mean() - t["ahat"]) < 4 * tot.std() / np.sqrt(S)


# ------------------------------------------------------------ stochastic ----

def _softmax64(x):
    e = np.exp(x.astype(np.float64) - x.max())
    return e / e.sum()


def test_stochastic_u_zero_accepts_first_children(oracle):
    B, V, N = 4, 32, 20
    marg = synth.marginals(41, B, V, 2.0)
    t = oracle.tree_build(marg, N)
    _, logits = synth.target_logits(42, N + 1, V, 1.0, "fp32")
    r = oracle.accept_stochastic(logits, marg, t["parent"], t["token"], t["depth"], np.zeros(N + 1, dtype=np.float32))
    # with u = 0 the first child of every node is accepted (p > 0 everywhere): follow child-0 links
    cur, path = -1, []
    while True:
        ch = [i for i in range(N) if t["parent"][i] == cur]
        if not ch:
            break
        cur = ch[0]; path.append(cur)
    assert r["path"].tolist() == path and r["n_acc"] == len(path)
    assert r["n_uniforms"] == len(path) + 1
    # bonus with u = 0: first token with positive mass of the last row's distribution = token 0
    assert r["bonus"] == 0


def test_stochastic_p_equals_q_always_accepts(oracle):
    B, V, N = 3, 16, 10
    marg = synth.marginals(43, B, V, 1.0)
    t = oracle.tree_build(marg, N)
    logits = np.zeros((N + 1, V), dtype=np.float32)
    for i in range(-1, N):
        d = 0 if i < 0 else int(t["depth"][i])
        if d < B:
            logits[i + 1] = np.log(marg[d].astype(np.float64)).astype(np.float32)
    u = np.full(N + 1, 0.999, dtype=np.float32)
    r = oracle.accept_stochastic(logits, marg, t["parent"], t["token"], t["depth"], u)
    # ratio p/q = 1 up to the fp32 rounding of log q: u = 0.999 accepts the first child at each level
    assert r["n_acc"] >= 1 and r["path"][0] == 0


def test_stochastic_rejects_when_p_below_q_on_tree_tokens(oracle):
    B, V, N = 2, 8, 5
    marg = synth.marginals(44, B, V, 1.0)
    t = oracle.tree_build(marg, N)
    logits = np.zeros((N + 1, V), dtype=np.float32)
    logits[:, :] = np.log(marg[0].astype(np.float64))
    for c in range(N):
        if t["parent"][c] < 0:
            logits[0, t["token"][c]] = -60.0                  # target gives (almost) no mass to tried tokens
    u = np.full(N + 1, 0.5, dtype=np.float32)
    r = oracle.accept_stochastic(logits, marg, t["parent"], t["token"], t["depth"], u)
    assert r["n_acc"] == 0
    tried = {int(t["token"][c]) for c in range(N) if t["parent"][c] < 0}
    assert r["bonus"] not in tried
    assert r["n_uniforms"] == len(tried) + 1


@pytest.mark.parametrize("n_children", [1, 2, 3])
def test_stochastic_preserves_target_distribution(oracle, n_children):
    """Textbook speculative sampling (Sec. 2.1): if the children are DRAWN from q (without replacement,
    each from the renormalised remainder), the emitted token is distributed exactly as the target p.
    Chi-square test of the empirical distribution of the first emitted token over many draws."""
    V, S = 8, 60_000
    marg = synth.marginals(51, 1, V, 1.0)
    _, logits = synth.target_logits(52, n_children + 1, V, 1.5, "fp32")
    p = _softmax64(logits[0])
    us = synth.uniform(53 + n_children, "accept", (S, n_children + 1)).astype(np.float32)
    ud = synth.uniform(54 + n_children, "draft", (S, n_children))
    counts = np.zeros(V)
    parent = np.full(n_children, -1, dtype=np.int32)
    depth = np.ones(n_children, dtype=np.int32)
    for s in range(S):
        q = marg[0].astype(np.float64).copy()
        toks = []
        for j in range(n_children):
            c = np.cumsum(q / q.sum())
            x = min(int(np.searchsorted(c, ud[s, j], side="right")), V - 1)
            toks.append(x); q[x] = 0.0
        r = oracle.accept_stochastic(logits, marg, parent, np.array(toks, dtype=np.int32), depth, us[s])
        first = int(toks[int(r["path"][0])]) if r["n_acc"] else r["bonus"]
        counts[first] += 1
    chi2 = float(((counts - S * p) ** 2 / (S * p)).sum())
    assert chi2 < 29.9, (chi2, counts / S, p)      # chi-square, 7 dof, p = 1e-4


def test_stochastic_accept_probability_closed_form(oracle):
    """Single child x: accepted iff u < min(1, p(x)/q(x)); on rejection the bonus is drawn from
    norm(max(p - q, 0)) by inverse CDF."""
    V = 6
    marg = np.array([[0.4, 0.3, 0.1, 0.1, 0.05, 0.05]], dtype=np.float32)
    p = np.array([0.1, 0.2, 0.3, 0.2, 0.1, 0.1])
    logits = np.log(p).astype(np.float32)[None].repeat(2, 0)
    pp = _softmax64(logits[0])
    parent, depth = np.array([-1], dtype=np.int32), np.array([1], dtype=np.int32)
    for x in range(V):
        ratio = min(1.0, pp[x] / float(marg[0, x]))
        for u in (0.0, ratio * 0.98, min(ratio * 1.02, 0.99999), 0.99):
            r = oracle.accept_stochastic(logits, marg, parent, np.array([x], dtype=np.int32), depth,
                                         np.array([u, 0.5], dtype=np.float32))
            assert (r["n_acc"] == 1) == (np.float32(u) * float(marg[0, x]) < pp[x])
            if r["n_acc"] == 0:
                res = np.maximum(pp - marg[0].astype(np.float64), 0.0)
                res /= res.sum()
                assert r["bonus"] == int(np.searchsorted(np.cumsum(res), 0.5, side="right"))
