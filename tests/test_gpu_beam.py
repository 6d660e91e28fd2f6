"""GPU parity of the beam-search tree (Sec. 4.3's comparison topology) with the oracle: bit-exact node lists, and
the two topologies driven through the same attention and acceptance kernels."""
import numpy as np
import pytest

from paper_2605_29727_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _same(ref, got):
    assert got["status"] == 0 and got["n"] == ref["n"]
    for k in ("parent", "token", "depth"):
        assert np.array_equal(got[k], ref[k]), k
    assert np.array_equal(got["rho"].view(np.uint32), ref["rho"].view(np.uint32)), "rho bits"
    assert got["ahat"] == pytest.approx(ref["ahat"], rel=1e-6)


@pytest.mark.parametrize("B,V,width,depth", [(4, 64, 4, 4), (16, 128256, 4, 15), (16, 128256, 1, 16), (16, 128256, 16, 16),
                                             (16, 4099, 8, 8), (3, 3, 16, 3), (5, 2, 3, 5), (16, 9000, 2, 16), (8, 1, 4, 8)])
@pytest.mark.parametrize("sigma", [1.0, 5.0])
def test_matches_oracle(oracle, G, B, V, width, depth, sigma):
    marg = synth.marginals(800 + width, B, V, sigma)
    _same(oracle.tree_build_beam(marg, width, depth), G.run_tree_build_beam(marg, width, depth))


def test_ties_and_zeros(oracle, G):
    for marg in (np.full((4, 8), 0.125, dtype=np.float32),
                 np.array([[0.5, 0.5, 0, 0], [0.25, 0.25, 0.25, 0.25], [1, 0, 0, 0]], dtype=np.float32),
                 np.array([[0.5, 0.25, 0.25], [0.75, 0.25, 0.0]], dtype=np.float32)):
        for width in (1, 2, 3, 5, 16):
            d = marg.shape[0]
            _same(oracle.tree_build_beam(marg, width, d), G.run_tree_build_beam(marg, width, d))


def test_rejects_bad_arguments(G):
    import torch
    from paper_2605_29727_amd import binding as btv
    marg = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    i32 = lambda n: torch.zeros(n, dtype=torch.int32, device="cuda")
    f32 = lambda n: torch.zeros(n, dtype=torch.float32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_build_workspace(4, 64, 16))
    for width, depth in ((0, 2), (17, 2), (2, 0), (2, 5)):
        with pytest.raises(btv.BtvError):
            btv.btv_tree_build_beam(marg, width, depth, i32(64), i32(64), i32(64), f32(64), i32(1), f32(1), ws)


def test_topologies_through_the_same_kernels(oracle, G):
    """Best-first (N = 60), beam 4 x 15 and the greedy chain of 16 (Sec. 4.3) built on the GPU from one set of
    marginals, each verified by the same attention kernel against the oracle; best-first has the largest surrogate."""
    B, V, L, Hq, Hkv, D = 16, 128256, 512, 8, 2, 128
    marg = synth.marginals(31, B, V, 5.0)
    trees = {"best_first": G.run_tree_build(marg, 60), "beam": G.run_tree_build_beam(marg, 4, 15),
             "chain": G.run_tree_build_beam(marg, 1, 16)}
    assert trees["best_first"]["n"] == trees["beam"]["n"] == 60 and trees["chain"]["n"] == 16
    assert trees["best_first"]["ahat"] >= trees["beam"]["ahat"] >= trees["chain"]["ahat"] - 1e-6
    for name, t in trees.items():
        M = t["n"]
        qkv = synth.qkv(40, M, L, Hq, Hkv, D, "bf16", tag=name)
        O = G.run_verify_attn(qkv, t["parent"], L, "bf16")
        ref = oracle.tree_attn(qkv["Qf"], qkv["Kf"], qkv["Vf"], t["parent"], L)
        assert np.abs(O - ref).max() < 2e-2, name
