"""Pins for the oracle's LM-head argmax (App. E LM head followed by App. C top-1), CPU only.

Checked against a library matrix product in fp64 (numpy), planted winners on an orthogonal basis, exact ties and
the greedy walk that consumes the tokens.
"""
import numpy as np
import pytest

from paper_2605_29727_amd import synth


@pytest.mark.parametrize("R,h,V", [(5, 48, 37), (1, 7, 3), (9, 16, 200), (3, 130, 1)])
def test_equals_library_product_and_argmax(oracle, R, h, V):
    for seed in range(3):
        _, xf, _, wf = synth.lm_head(seed, R, h, V, "bf16")
        got = oracle.lm_head_argmax(xf, wf)
        z = xf.astype(np.float64) @ wf.astype(np.float64).T          # [R, V]: row r against every W row
        assert np.array_equal(got["argmax"], z.argmax(axis=1))
        if V > 1:
            top2 = np.sort(z, axis=1)[:, -2:]
            assert np.allclose(got["margin"], top2[:, 1] - top2[:, 0], rtol=1e-9, atol=1e-12)


def test_planted_winners_on_an_orthogonal_basis(oracle):
    """W rows = distinct scaled basis vectors: logit[r, v] = scale[v] * x[r, axis[v]], so the winner is readable
    from the inputs without any product."""
    h, V = 12, 12
    axis = synth.permutation(3, "axis", V)
    scale = 1.0 + 0.25 * np.arange(V)
    W = np.zeros((V, h), dtype=np.float32)
    W[np.arange(V), axis] = scale
    X = np.zeros((4, h), dtype=np.float32)
    X[0, axis[5]] = 1.0                         # only token 5 sees a non-zero logit
    X[1, :] = 1.0                               # every logit = scale[v]: the largest scale wins
    X[2, :] = -1.0                              # every logit = -scale[v]: the smallest scale wins
    X[3, axis[2]] = 3.0; X[3, axis[9]] = 1.0    # 3 * scale[2] = 4.5 against scale[9] = 3.25
    got = oracle.lm_head_argmax(X, W)
    assert got["argmax"].tolist() == [5, V - 1, 0, 2]
    assert got["margin"][0] == pytest.approx(scale[5]) and got["margin"][3] == pytest.approx(4.5 - 3.25)


def test_ties_go_to_the_lowest_token(oracle):
    W = np.array([[1, 0], [2, 0], [2, 0], [0, 5], [2, 0]], dtype=np.float32)
    X = np.array([[1, 0], [0, 0], [-1, 0]], dtype=np.float32)
    got = oracle.lm_head_argmax(X, W)
    assert got["argmax"].tolist() == [1, 0, 3]       # tokens 1, 2, 4 tie at 2; all logits zero; 0 beats the negatives
    assert got["margin"].tolist() == [0.0, 0.0, 1.0]


def test_feeds_the_greedy_walk(oracle):
    """Hidden states turned towards the LM-head rows of a planted path make the greedy walk accept that path."""
    R, h, V, N = 17, 64, 300, 16
    parent = synth.tree_parents(11, N, "random")
    token = synth.sibling_distinct_tokens(11, parent, V)
    _, xf, _, wf = synth.lm_head(11, R, h, V, "bf16")
    leaf = 9
    xp = synth.plant_hidden(xf, wf, parent, token, leaf).astype(np.float32)
    t = oracle.lm_head_argmax(xp, wf)["argmax"]
    logits = (xp.astype(np.float64) @ wf.astype(np.float64).T).astype(np.float32)
    ref = oracle.accept_greedy(logits, parent, token)
    want = []
    i = leaf
    while i >= 0:
        want.append(i); i = int(parent[i])
    assert ref["path"].tolist()[:len(want)] == want[::-1]
    assert np.array_equal(ref["argmax"], t)
