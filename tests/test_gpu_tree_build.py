"""Bit-exact parity of the HIP best-first tree build with the CPU oracle (topology, tokens, depth, rho bits)."""
import numpy as np
import pytest

from paper_2605_29727_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _check(G, oracle, marg, N):
    """The library's own choice of expansion, then each of the two expansions forced."""
    ref = oracle.tree_build(marg, N)
    for algo in (0, 1, 2):
        got = G.run_tree_build(marg, N, algo)
        assert got["n"] == ref["n"], algo
        for k in ("parent", "token", "depth"):
            assert np.array_equal(got[k], ref[k]), (k, algo)
        assert np.array_equal(got["rho"].view(np.uint32), ref["rho"].view(np.uint32)), algo
        assert abs(got["ahat"] - ref["ahat"]) <= 1e-5 * ref["ahat"], algo
    return ref


def test_config1(G, oracle):
    w = synth.C1
    _check(G, oracle, synth.marginals(w.seed, w.B, w.V, w.marg_sigma), w.N)


@pytest.mark.parametrize("sigma,seed", [(3.0, 2), (5.0, 3), (1.0, 4), (8.0, 9)])
@pytest.mark.parametrize("N", [1, 16, 64, 100, 256])
def test_full_vocabulary(G, oracle, sigma, seed, N):
    marg = synth.marginals(seed, 16, 128256, sigma)
    ref = _check(G, oracle, marg, N)
    if sigma == 1.0 and N == 256:
        assert ref["depth"].max() == 1          # flat marginals: the tree is a depth-1 star
    if sigma >= 5.0 and N >= 64:
        assert ref["depth"].max() >= 3          # sharp marginals: deep chains


@pytest.mark.parametrize("B,V,N", [(1, 1, 1), (2, 3, 12), (4, 64, 200), (16, 2049, 256), (3, 5000, 77), (16, 300, 256)])
def test_small_and_ragged_vocabularies(G, oracle, B, V, N):
    for seed in range(3):
        _check(G, oracle, synth.marginals(50 + seed, B, V, 2.5), N)


def test_ties_zeros_one_hot_and_budget_beyond_lattice(G, oracle):
    cases = [
        np.full((4, 8), 0.125, dtype=np.float32),                                   # everything ties
        np.array([[0.0, 1.0, 0.0], [0.5, 0.5, 0.0], [0.0, 0.0, 1.0]], dtype=np.float32),
        np.array([[0.5, 0.25, 0.25], [0.75, 0.25, 0.0]], dtype=np.float32),
        np.array([[0.6, 0.4]], dtype=np.float32),                                   # lattice of 2 prefixes
    ]
    for marg in cases:
        for N in (1, 2, 5, 12, 40, 256):
            _check(G, oracle, marg, N)
    # many exact ties in a large vocabulary: probabilities quantised to multiples of 2^-12
    marg = synth.marginals(77, 8, 4096, 2.0)
    marg = (np.floor(marg * 4096) / 4096).astype(np.float32)
    _check(G, oracle, marg, 256)


def test_tiny_scores_keep_their_bits(G, oracle):
    """Products deep in the tree reach the subnormal range; rho must still match bit for bit."""
    marg = np.full((16, 4), 1e-3, dtype=np.float32)
    marg[:, 0] = 3e-3
    _check(G, oracle, marg, 256)


def test_more_candidates_than_the_selection_keeps(G, oracle):
    """Rows whose probabilities tie heavily, or grow with the token id, defeat the cheap bound of the top-K
    selection (most of the row stays a candidate): the exact byte-wise selection must take over."""
    V = 20000
    uniform = np.full((3, V), 1.0 / V, dtype=np.float32)                         # every key ties on the probability
    ramp = np.tile(np.arange(1, V + 1, dtype=np.float64), (2, 1))                 # best tokens at the highest ids
    ramp = (ramp / ramp.sum(axis=1, keepdims=True)).astype(np.float32)
    steps = np.repeat(np.arange(1, 6, dtype=np.float64), V // 5)[None, :]        # five plateaus of 4000 equal values
    steps = np.tile(steps / steps.sum(), (4, 1)).astype(np.float32)
    mixed = synth.marginals(91, 4, V, 2.0)
    mixed[1] = uniform[0]                                                         # only one row takes the slow path
    for marg in (uniform, ramp, steps, mixed):
        for N in (7, 64, 256):
            _check(G, oracle, marg, N)
