"""Parity of the HIP acceptance walks with the CPU oracle: argmax, path, n_acc and bonus are bit-exact."""
import numpy as np
import pytest

from paper_2605_29727_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _depths(parent):
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(len(parent)):
        d[i] = 1 if parent[i] < 0 else d[parent[i]] + 1
    return d


def _greedy_case(G, oracle, store, f32, bits, parent, token):
    ref = oracle.accept_greedy(f32, parent, token)
    got = G.run_accept_greedy(store, bits, parent, token)
    assert np.array_equal(got["argmax"], ref["argmax"])
    assert got["n_acc"] == ref["n_acc"] and np.array_equal(got["path"], ref["path"]) and got["bonus"] == ref["bonus"]
    return ref


def test_greedy_config1(G, oracle):
    w = synth.C1
    tree = oracle.tree_build(synth.marginals(w.seed, w.B, w.V, w.marg_sigma), w.N)
    store, f = synth.target_logits(w.seed, w.N + 1, w.V, w.logit_sigma, "fp32")
    _greedy_case(G, oracle, store, f, False, tree["parent"], tree["token"])
    for leaf in range(w.N):
        x = synth.plant_path(f, tree["parent"], tree["token"], leaf)
        r = _greedy_case(G, oracle, x, x, False, tree["parent"], tree["token"])
        assert r["n_acc"] >= tree["depth"][leaf]


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_greedy_config2_full_vocab_with_planted_paths(G, oracle, dtype):
    w = synth.C2
    tree = oracle.tree_build(synth.marginals(w.seed, w.B, w.V, w.marg_sigma), w.N)
    _, f = synth.target_logits(w.seed, w.N + 1, w.V, w.logit_sigma, "fp32")
    deep = int(np.argmax(tree["depth"]))
    for leaf in (-1, deep, 0, w.N // 2):
        x = synth.plant_path(f, tree["parent"], tree["token"], leaf)
        store, xf = synth.round_to_dtype(x.astype(np.float64), dtype)
        r = _greedy_case(G, oracle, store, xf, dtype == "bf16", tree["parent"], tree["token"])
        if leaf >= 0:
            assert r["n_acc"] >= tree["depth"][leaf]
    # bf16 logits tie often at 128k draws: the argmax must still be the lowest index
    store, xf = synth.round_to_dtype(np.round(f.astype(np.float64) * 4) / 4, dtype)
    _greedy_case(G, oracle, store, xf, dtype == "bf16", tree["parent"], tree["token"])


@pytest.mark.parametrize("kind", ["chain", "star", "binary", "random", "deep"])
@pytest.mark.parametrize("M,V", [(1, 1), (7, 13), (256, 1000), (100, 8193), (33, 128256)])
def test_greedy_tree_kinds_and_odd_vocabularies(G, oracle, kind, M, V):
    parent = synth.tree_parents(5, M, kind)
    fan = max(np.bincount(parent + 1).max(), 1)
    if fan > V:
        pytest.skip("fan-out exceeds the vocabulary")
    token = synth.sibling_distinct_tokens(5, parent, V)
    for dtype in ("bf16", "fp32"):
        _, f = synth.target_logits(6, M + 1, V, 1.0, "fp32", tag=f"{kind}{M}{V}")
        leaf = int(np.argmax(_depths(parent)))
        x = synth.plant_path(f, parent, token, leaf)
        store, xf = synth.round_to_dtype(x.astype(np.float64), dtype)
        _greedy_case(G, oracle, store, xf, dtype == "bf16", parent, token)


def test_greedy_all_equal_and_neg_inf_rows(G, oracle):
    M, V = 5, 300
    parent = synth.tree_parents(0, M, "chain")
    token = np.zeros(M, dtype=np.int32)
    x = np.zeros((M + 1, V), dtype=np.float32)
    r = _greedy_case(G, oracle, x, x, False, parent, token)     # every row ties everywhere: argmax 0 -> full chain
    assert r["n_acc"] == M and r["bonus"] == 0
    x[:] = -np.inf
    _greedy_case(G, oracle, x, x, False, parent, token)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_greedy_neg_inf_in_whole_units(G, oracle, dtype):
    """Rows that are -inf nearly everywhere, over a vocabulary of two whole scan units and a ragged one: a lane
    whose elements are all -inf has nothing "larger than the start value", which is the case the scan's cheap pass
    hands back to the exact one."""
    M, V = 4, 2 * 4096 + 777
    parent = synth.tree_parents(0, M, "chain")
    x = np.full((M + 1, V), -np.inf, dtype=np.float32)
    x[1, 5000] = -3.0                       # one finite value in the second unit
    x[2, V - 1] = 0.5                       # only the last element of the ragged unit
    x[3, :] = np.linspace(-4.0, 4.0, V, dtype=np.float32)[::-1]
    x[3, 4096] = 9.0
    x[4, 4095], x[4, 4096] = 2.0, 2.0       # a tie across two units
    token = np.array([0, 5000, V - 1, 4096], dtype=np.int32)
    store, xf = synth.round_to_dtype(x.astype(np.float64), dtype)
    r = _greedy_case(G, oracle, store, xf, dtype == "bf16", parent, token)
    assert r["n_acc"] == 4 and r["bonus"] == 4095


def test_greedy_signed_zeros_tie_and_workspace_reuse(G, oracle):
    """-0.0 and +0.0 are the same value: the lower index wins whichever sign it carries.  One workspace then serves
    calls of different sizes in a row: the slots that the workgroups leave their keys in are back at zero after each."""
    import torch
    from paper_2605_29727_amd import binding as btv
    M, V = 3, 9000
    parent = synth.tree_parents(0, M, "chain")
    x = np.full((M + 1, V), -1.0, dtype=np.float32)
    x[0, 5000], x[0, 17] = 0.0, -0.0
    x[1, 17], x[1, 8999] = 0.0, -0.0
    x[2, 8999], x[2, 4096] = -0.0, -0.0
    x[3, 1] = 0.0
    token = np.array([17, 17, 4096], dtype=np.int32)
    r = _greedy_case(G, oracle, x, x, False, parent, token)
    assert r["n_acc"] == 3 and r["bonus"] == 1

    V = 128256
    ws = btv.alloc_workspace(btv.btv_tree_accept_workspace(256, V, False))
    for M, kind, seed in ((64, "random", 1), (5, "chain", 2), (256, "deep", 3), (64, "random", 1)):
        parent = synth.tree_parents(seed, M, kind)
        token = synth.sibling_distinct_tokens(seed, parent, V)
        _, f = synth.target_logits(seed, M + 1, V, 1.0, "fp32", tag=f"reuse{M}")
        x = synth.plant_path(f, parent, token, int(np.argmax(_depths(parent))))
        store, xf = synth.round_to_dtype(x.astype(np.float64), "bf16")
        ref = oracle.accept_greedy(xf, parent, token)
        d = G.dev(store, True)
        par, tok = G.dev(parent.astype(np.int32)), G.dev(token.astype(np.int32))
        path = torch.full((M,), -7, dtype=torch.int32, device="cuda")
        n_acc = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        bonus = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        am = torch.full((M + 1,), -7, dtype=torch.int32, device="cuda")
        for _ in range(2):                                   # twice in a row on the same workspace
            btv.btv_tree_accept_greedy(d, par, tok, path, n_acc, bonus, am, ws)
        torch.cuda.synchronize()
        n = int(n_acc.item())
        assert n == ref["n_acc"] and bonus.item() == ref["bonus"], (M, kind)
        assert np.array_equal(path.cpu().numpy()[:n], ref["path"]) and np.array_equal(am.cpu().numpy(), ref["argmax"])
    assert torch.count_nonzero(ws).item() == 0               # the workspace is left as it was handed over


def test_greedy_collector_gives_up_within_its_limit(G, oracle):
    """The workgroup that collects the others' keys waits for them with a limit on the wall clock.  A negative
    limit makes it give up before its first look: the kernel ends normally, the workspace's flag reports it, and
    the outputs are those of all-zero argmax rows.  The same call with a real limit, on a workspace zero-filled
    again, then gives the oracle's result."""
    import torch
    from paper_2605_29727_amd import binding as btv
    M, V = 40, 20000
    parent = synth.tree_parents(5, M, "random")
    token = synth.sibling_distinct_tokens(5, parent, V)
    _, f = synth.target_logits(5, M + 1, V, 1.0, "fp32", tag="limit")
    x = synth.plant_path(f, parent, token, int(np.argmax(_depths(parent))))
    store, xf = synth.round_to_dtype(x.astype(np.float64), "bf16")
    ref = oracle.accept_greedy(xf, parent, token)
    d = G.dev(store, True)
    par, tok = G.dev(parent.astype(np.int32)), G.dev(token.astype(np.int32))
    path = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    n_acc = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    am = torch.full((M + 1,), -7, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_workspace(M, V, False))
    btv.btv_tree_accept_greedy_tuned(d, par, tok, path, n_acc, bonus, am, ws, -1)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == btv.BTV_EDATA
    assert torch.count_nonzero(am).item() == 0 and 0 <= n_acc.item() <= M
    ws.zero_()
    btv.btv_tree_accept_greedy_tuned(d, par, tok, path, n_acc, bonus, am, ws, 100_000_000)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == 0
    n = int(n_acc.item())
    assert n == ref["n_acc"] and bonus.item() == ref["bonus"]
    assert np.array_equal(path.cpu().numpy()[:n], ref["path"]) and np.array_equal(am.cpu().numpy(), ref["argmax"])
    assert torch.count_nonzero(ws).item() == 0


AMBIGUOUS, AMBIGUOUS_GAP = 1e-4, 1e-6


def _ambiguous(ref):
    return ref["margin"] < AMBIGUOUS or ref["bonus_gap"] < AMBIGUOUS_GAP


@pytest.mark.parametrize("logit_dtype", ["fp32", "bf16"])
def test_stochastic_parity(G, oracle, logit_dtype):
    """Seeds whose accept tests sit within AMBIGUOUS (relative) of the threshold, or whose bonus draw sits within
    AMBIGUOUS_GAP (absolute) of a CDF step, are skipped: there the outcome
    depends on the rounding of vocabulary-wide sums and either result is correct."""
    B, V, N = 8, 5000, 48
    checked = 0
    for seed in range(12):
        marg = synth.marginals(100 + seed, B, V, 2.0)
        tree = oracle.tree_build(marg, N)
        # target close to the draft so that acceptances and rejections both happen
        z = np.log(np.maximum(marg[np.minimum(np.concatenate([[0], tree["depth"]]), B - 1)].astype(np.float64), 1e-30))
        z += synth.normal(200 + seed, "noise", z.shape, 1.0)
        store, xf = synth.round_to_dtype(z, logit_dtype)
        u = synth.uniform(300 + seed, "u", (N + 1,)).astype(np.float32)
        ref = oracle.accept_stochastic(xf, marg, tree["parent"], tree["token"], tree["depth"], u)
        if _ambiguous(ref):
            continue
        got = G.run_accept_stochastic(store, logit_dtype == "bf16", marg, tree["parent"], tree["token"], u)
        assert got["n_acc"] == ref["n_acc"] and np.array_equal(got["path"], ref["path"]), seed
        assert got["bonus"] == ref["bonus"], seed
        checked += 1
    assert checked >= 8


def test_stochastic_extremes(G, oracle):
    B, V, N = 4, 640, 20
    marg = synth.marginals(7, B, V, 2.0)
    tree = oracle.tree_build(marg, N)
    store, xf = synth.target_logits(8, N + 1, V, 1.0, "fp32")
    for u in (np.zeros(N + 1, dtype=np.float32), np.full(N + 1, 0.999999, dtype=np.float32)):
        ref = oracle.accept_stochastic(xf, marg, tree["parent"], tree["token"], tree["depth"], u)
        got = G.run_accept_stochastic(store, False, marg, tree["parent"], tree["token"], u)
        assert got["n_acc"] == ref["n_acc"] and np.array_equal(got["path"], ref["path"]) and got["bonus"] == ref["bonus"]


def test_config5_stochastic_full_vocab(G, oracle):
    w = synth.C5
    marg = synth.marginals(w.seed, w.B, w.V, w.marg_sigma)
    tree = oracle.tree_build(marg, w.N)
    store, xf = synth.target_logits(w.seed, w.N + 1, w.V, w.logit_sigma, w.logit_dtype)
    done = 0
    for k in range(6):
        u = synth.uniform(w.seed, f"uniforms{k}", (w.N + 1,)).astype(np.float32)
        ref = oracle.accept_stochastic(xf, marg, tree["parent"], tree["token"], tree["depth"], u)
        if _ambiguous(ref):
            continue
        got = G.run_accept_stochastic(store, False, marg, tree["parent"], tree["token"], u)
        assert got["n_acc"] == ref["n_acc"] and np.array_equal(got["path"], ref["path"]) and got["bonus"] == ref["bonus"]
        done += 1
    assert done >= 3


@pytest.mark.parametrize("V,fan", [(300, 120), (5000, 200), (40000, 64), (2048 * 64 + 200, 48)])
def test_stochastic_wide_fans(G, oracle, V, fan):
    """Nodes with many children take the sorted-ratio path of the walk (prefix sums over the (e, q0) pairs in bins of
    q0/e): flat marginals give a wide fan under the root, a target close to the draft makes acceptances late in the
    fan likely, and vocabularies below and above the chunk limits are covered."""
    B = 3
    checked = 0
    for seed in range(8):
        marg = synth.marginals(700 + seed, B, V, 0.7)
        tree = oracle.tree_build(marg, fan)
        assert int((tree["parent"] == -1).sum()) >= min(fan, 40)
        z = np.log(np.maximum(marg[np.minimum(np.concatenate([[0], tree["depth"]]), B - 1)].astype(np.float64), 1e-30))
        z += synth.normal(800 + seed, "noise", z.shape, [0.3, 1.0, 2.0][seed % 3])
        store, xf = synth.round_to_dtype(z, "fp32")
        u = synth.uniform(900 + seed, "u", (fan + 1,)).astype(np.float32)
        if seed % 4 == 3:
            u[:] = 0.999999           # everything that can be rejected is: the whole fan is walked
        ref = oracle.accept_stochastic(xf, marg, tree["parent"], tree["token"], tree["depth"], u)
        if _ambiguous(ref):
            continue
        got = G.run_accept_stochastic(store, False, marg, tree["parent"], tree["token"], u)
        assert got["n_acc"] == ref["n_acc"] and np.array_equal(got["path"], ref["path"]), (V, fan, seed)
        assert got["bonus"] == ref["bonus"], (V, fan, seed)
        checked += 1
    assert checked >= 4


def test_stochastic_wide_fan_long_vocabulary(G, oracle):
    """A vocabulary of 300000: the sorted pairs' prefix sums take chunks of 256 pairs (a power of two, so that the
    chunk of a position is a shift) and the last chunk is ragged.  With probabilities this small most seeds fall
    under the ambiguity margins; those that do not must agree."""
    B, V, fan = 3, 300000, 40
    checked = 0
    for seed in range(8):
        marg = synth.marginals(700 + seed, B, V, 0.7)
        tree = oracle.tree_build(marg, fan)
        z = np.log(np.maximum(marg[np.minimum(np.concatenate([[0], tree["depth"]]), B - 1)].astype(np.float64), 1e-30))
        z += synth.normal(800 + seed, "noise", z.shape, [0.3, 1.0, 2.0][seed % 3])
        store, xf = synth.round_to_dtype(z, "fp32")
        u = synth.uniform(900 + seed, "u", (fan + 1,)).astype(np.float32)
        if seed % 4 == 3:
            u[:] = 0.999999
        ref = oracle.accept_stochastic(xf, marg, tree["parent"], tree["token"], tree["depth"], u)
        if _ambiguous(ref):
            continue
        got = G.run_accept_stochastic(store, False, marg, tree["parent"], tree["token"], u)
        assert got["n_acc"] == ref["n_acc"] and np.array_equal(got["path"], ref["path"]), seed
        assert got["bonus"] == ref["bonus"], seed
        checked += 1
    assert checked >= 2


def test_stochastic_token_outside_vocabulary_is_flagged_not_faulting():
    """A token id outside [0, V) is never used as an index: that child counts as rejected, the data flag is raised,
    and the walk goes on with the valid children."""
    import torch
    import gpu_util as G
    from paper_2605_29727_amd import binding as btv
    B, V, M = 4, 300, 6
    marg = synth.marginals(97, B, V, 2.0)
    parent = np.array([-1, -1, 0, 0, 1, 2], dtype=np.int32)
    token = np.array([10 ** 9, 7, 5, -3, 9, 11], dtype=np.int32)
    st, _ = synth.target_logits(97, M + 1, V, 1.0, "fp32")
    path = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    n_acc = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_workspace(M, V, True))
    btv.btv_tree_accept_stochastic(G.dev(st), G.dev(marg.astype(np.float32)), G.dev(parent), G.dev(token),
                                   G.dev(np.zeros(M + 1, dtype=np.float32)), path, n_acc, bonus, ws)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == btv.BTV_EDATA
    n = int(n_acc.item())
    assert 0 <= n <= M and 0 <= int(bonus.item()) < V
    assert 0 not in path.cpu().numpy()[:n].tolist()          # node 0 carries the invalid id: never accepted
