"""GPU parity of the fused LM head + greedy acceptance (App. E LM head, App. C "Acceptance") against the oracle.

The target token of a row is an integer decided by floating point: the kernel accumulates exact bf16 products in
fp32 on the matrix cores, the oracle in fp64.  A row whose two best logits are closer than AMBIG has no unique
answer at fp32 resolution: there the kernel's token must be one of the near-best ones; everywhere else it must be
the oracle's token, and the walk (which depends on the tokens only) must be identical.
"""
import numpy as np
import pytest

from paper_2605_29727_amd import synth

pytestmark = pytest.mark.gpu

@pytest.fixture(scope="module")
def gpu():
    import gpu_util
    return gpu_util


AMBIG = 1e-3      # logits are O(1) sums of h exact products; fp32 accumulation error is ~1e-5 here


def _check(oracle, xf, wf, parent, token, got):
    ref = oracle.lm_head_argmax(xf, wf)
    t, margin = ref["argmax"], ref["margin"]
    clear = margin > AMBIG
    assert np.array_equal(got["argmax"][clear], t[clear])
    for r in np.nonzero(~clear)[0]:          # near-ties: the kernel's token must be within AMBIG of the best logit
        z = wf.astype(np.float64) @ xf[r].astype(np.float64)
        assert z[got["argmax"][r]] >= z.max() - AMBIG
    # the walk depends on the tokens only: feed the kernel's own tokens to the oracle's walk as one-hot logits
    V = wf.shape[0]
    onehot = np.zeros((len(parent) + 1, V), dtype=np.float32)
    onehot[np.arange(len(parent) + 1), got["argmax"]] = 1.0
    walk = oracle.accept_greedy(onehot, parent, token)
    assert got["n_acc"] == walk["n_acc"] and got["path"].tolist() == walk["path"].tolist()
    assert got["bonus"] == walk["bonus"]
    return int(clear.sum())


@pytest.mark.parametrize("M,h,V", [(7, 128, 100), (1, 128, 1), (40, 256, 1000), (64, 512, 4100), (31, 1024, 129),
                                   (130, 384, 3000), (200, 128, 2049), (256, 256, 2500)])
def test_matches_oracle(oracle, gpu, M, h, V):
    for seed in range(2):
        parent = synth.tree_parents(seed, M, "random")
        token = synth.sibling_distinct_tokens(seed, parent, V) if V > M else np.zeros(M, dtype=np.int32)
        xs, xf, ws, wf = synth.lm_head(seed, M + 1, h, V, "bf16")
        if V > M:
            leaf = int(synth.integers(seed, "leaf", (1,), 0, M)[0])
            xs, xf = synth.round_to_dtype(synth.plant_hidden(xf, wf, parent, token, leaf), "bf16")
        got = gpu.run_accept_greedy_lm_head(xs, ws, parent, token)
        assert _check(oracle, xf, wf, parent, token, got) >= (M + 1) // 2


def test_planted_path_is_accepted(oracle, gpu):
    M, h, V = 64, 512, 5000
    parent = synth.tree_parents(3, M, "deep")
    token = synth.sibling_distinct_tokens(3, parent, V)
    _, xf, ws, wf = synth.lm_head(3, M + 1, h, V, "bf16")
    depth = np.zeros(M, dtype=np.int32)
    for i in range(M):
        depth[i] = 1 if parent[i] < 0 else depth[parent[i]] + 1
    leaf = int(depth.argmax())
    xs, xf = synth.round_to_dtype(synth.plant_hidden(xf, wf, parent, token, leaf), "bf16")
    got = gpu.run_accept_greedy_lm_head(xs, ws, parent, token)
    want = []
    i = leaf
    while i >= 0:
        want.append(i); i = int(parent[i])
    assert got["path"].tolist()[:len(want)] == want[::-1] and got["n_acc"] >= len(want)
    _check(oracle, xf, wf, parent, token, got)


def test_ties_go_to_the_lowest_token(oracle, gpu):
    """Duplicate weight rows give bit-identical logits on both sides: the lowest token id wins."""
    M, h, V = 5, 128, 700
    xs, xf, ws, wf = synth.lm_head(5, M + 1, h, V, "bf16")
    big = np.zeros(h, dtype=np.float32)
    big[:8] = 4.0
    bs, bf = synth.round_to_dtype(big.astype(np.float64), "bf16")
    for v in (650, 17, 300, 130):              # in different waves and workgroups
        ws[v], wf[v] = bs, bf
    xs[:, :8], xf[:, :8] = synth.round_to_dtype(np.full((M + 1, 8), 2.0), "bf16")
    parent = np.full(M, -1, dtype=np.int32)
    token = np.arange(M, dtype=np.int32)
    got = gpu.run_accept_greedy_lm_head(xs, ws, parent, token)
    assert got["argmax"].tolist() == [17] * (M + 1)
    assert oracle.lm_head_argmax(xf, wf)["argmax"].tolist() == [17] * (M + 1)


def test_full_vocabulary_8b_shape(oracle, gpu):
    """The benchmark's shape: 65 rows, h = 4096, V = 128256, every row against the oracle."""
    M, h, V = 64, 4096, 128256
    parent = synth.tree_parents(9, M, "random")
    token = synth.sibling_distinct_tokens(9, parent, V)
    _, xf, ws, wf = synth.lm_head(9, M + 1, h, V, "bf16")
    xs, xf = synth.round_to_dtype(synth.plant_hidden(xf, wf, parent, token, 40), "bf16")
    got = gpu.run_accept_greedy_lm_head(xs, ws, parent, token)
    assert _check(oracle, xf, wf, parent, token, got) >= 60


def test_rejects_bad_arguments(gpu):
    import torch
    from paper_2605_29727_amd import binding as btv
    x = torch.zeros((3, 100), dtype=torch.bfloat16, device="cuda")      # h not a multiple of 128
    W = torch.zeros((50, 100), dtype=torch.bfloat16, device="cuda")
    i32 = lambda n: torch.zeros(n, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_lm_head_workspace(2, 50))
    with pytest.raises(btv.BtvError):
        btv.btv_tree_accept_greedy_lm_head(x, W, i32(2), i32(2), i32(2), i32(1), i32(1), None, ws)
    x = torch.zeros((3, 128), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((50, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(btv.BtvError):
        btv.btv_tree_accept_greedy_lm_head(x, W, i32(2), i32(2), i32(2), i32(1), i32(1), None, ws[:64])   # workspace too small
