"""Batches of requests in one launch: tree_build_batch and tree_accept_greedy_batch must give, request by request,
exactly what the oracle gives for that request alone (bit-exact trees, tokens, paths)."""
import numpy as np
import pytest

from paper_2605_29727_amd import synth

pytestmark = pytest.mark.gpu


def _run_build(marg, n_nodes, q_offset, N_max):
    import torch
    from paper_2605_29727_amd import binding as btv
    batch, B, V = marg.shape
    total = int(q_offset[-1])
    m = torch.from_numpy(np.ascontiguousarray(marg, dtype=np.float32)).cuda()
    nn = torch.from_numpy(np.asarray(n_nodes, dtype=np.int32)).cuda()
    qo = torch.from_numpy(np.asarray(q_offset, dtype=np.int32)).cuda()
    parent = torch.full((max(total, 1),), -7, dtype=torch.int32, device="cuda")
    token, depth = torch.full_like(parent, -7), torch.full_like(parent, -7)
    rho = torch.full((max(total, 1),), -7.0, dtype=torch.float32, device="cuda")
    n_out = torch.full((batch,), -7, dtype=torch.int32, device="cuda")
    ahat = torch.zeros(batch, dtype=torch.float32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_build_batch_workspace(batch, B, V, N_max))
    btv.btv_tree_build_batch(m, nn, qo, N_max, parent, token, depth, rho, n_out, ahat, ws)
    torch.cuda.synchronize()
    return {"parent": parent.cpu().numpy(), "token": token.cpu().numpy(), "depth": depth.cpu().numpy(),
            "rho": rho.cpu().numpy(), "n_out": n_out.cpu().numpy(), "ahat": ahat.cpu().numpy(),
            "status": int(btv.btv_workspace_status(ws))}


@pytest.mark.parametrize("batch,B,V,N_max,slack", [(8, 16, 128256, 128, 0), (3, 4, 64, 16, 5), (16, 8, 5000, 64, 0),
                                                   (1, 16, 128256, 256, 0), (5, 6, 3, 40, 2)])
def test_tree_build_batch_matches_oracle(oracle, batch, B, V, N_max, slack):
    marg = np.stack([synth.marginals(900 + r, B, V, [1.0, 3.0, 5.0][r % 3]) for r in range(batch)])
    n_nodes = [int(x) for x in synth.integers(7, "nn", (batch,), 1, N_max)]
    n_nodes[0] = N_max
    q_offset = np.concatenate([[0], np.cumsum([n + slack for n in n_nodes])]).astype(np.int32)
    got = _run_build(marg, n_nodes, q_offset, N_max)
    assert got["status"] == 0
    for r in range(batch):
        ref = oracle.tree_build(marg[r], n_nodes[r])
        o, n = int(q_offset[r]), ref["n"]
        assert got["n_out"][r] == n
        for k in ("parent", "token", "depth"):
            assert np.array_equal(got[k][o:o + n], ref[k]), (r, k)
        assert np.array_equal(got["rho"][o:o + n].view(np.uint32), ref["rho"].view(np.uint32))
        assert got["ahat"][r] == pytest.approx(ref["ahat"], rel=1e-6)
        assert np.all(got["parent"][o + n:int(q_offset[r + 1])] == -7)        # nothing written past the request's nodes


def test_tree_build_batch_flags_bad_requests(oracle):
    marg = np.stack([synth.marginals(950 + r, 4, 100, 2.0) for r in range(3)])
    q_offset = np.array([0, 10, 20, 30], dtype=np.int32)
    got = _run_build(marg, [10, 11, 0], q_offset, 16)            # request 1 asks for more rows than it owns
    assert got["status"] != 0
    assert got["n_out"].tolist() == [10, 0, 0]
    ref = oracle.tree_build(marg[0], 10)
    assert np.array_equal(got["parent"][:10], ref["parent"])


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_accept_batch_matches_oracle(oracle, dtype):
    import torch
    import gpu_util as G
    from paper_2605_29727_amd import binding as btv
    V = 30000
    Ms = [40, 7, 128, 1, 64, 33]
    q_offset = np.concatenate([[0], np.cumsum(Ms)]).astype(np.int32)
    batch, total = len(Ms), int(q_offset[-1])
    parents, tokens, stores, refs = [], [], [], []
    for r, M in enumerate(Ms):
        par = synth.tree_parents(60 + r, M, ["random", "deep", "binary"][r % 3])
        tok = synth.sibling_distinct_tokens(60 + r, par, V)
        _, lf = synth.target_logits(60 + r, M + 1, V, 1.0, dtype)
        leaf = int(synth.integers(60 + r, "leaf", (1,), 0, M)[0]) if r % 2 == 0 else -1
        st, lf = synth.round_to_dtype(synth.plant_path(lf, par, tok, leaf).astype(np.float64), dtype)
        parents.append(par); tokens.append(tok); stores.append(st)
        refs.append(oracle.accept_greedy(lf, par, tok))
    logits = G.dev(np.concatenate(stores), dtype == "bf16")
    par = G.dev(np.concatenate(parents).astype(np.int32)); tok = G.dev(np.concatenate(tokens).astype(np.int32))
    qo = G.dev(q_offset)
    path = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    n_acc = torch.full((batch,), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((batch,), -7, dtype=torch.int32, device="cuda")
    am = torch.full((total + batch,), -7, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_batch_workspace(batch, total, V))
    btv.btv_tree_accept_greedy_batch(logits, par, tok, qo, max(Ms), path, n_acc, bonus, am, ws)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == 0
    path, n_acc, bonus, am = path.cpu().numpy(), n_acc.cpu().numpy(), bonus.cpu().numpy(), am.cpu().numpy()
    for r, M in enumerate(Ms):
        o, ref = int(q_offset[r]), refs[r]
        assert n_acc[r] == ref["n_acc"] and bonus[r] == ref["bonus"]
        assert path[o:o + ref["n_acc"]].tolist() == ref["path"].tolist()
        assert np.array_equal(am[o + r:o + r + M + 1], ref["argmax"])


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_accept_batch_neg_inf_in_whole_chunks(oracle, dtype):
    """Rows that are -inf nearly everywhere over two whole argmax chunks and a ragged one: a thread that saw
    nothing above -inf is the case that the chunk scan's cheap pass hands back to the exact one."""
    import torch
    import gpu_util as G
    from paper_2605_29727_amd import binding as btv
    M, V = 4, 2 * 8192 + 301
    parent = synth.tree_parents(0, M, "chain")
    x = np.full((M + 1, V), -np.inf, dtype=np.float32)
    x[1, 9000] = -3.0
    x[2, V - 1] = 0.5
    x[3, :] = np.linspace(-4.0, 4.0, V, dtype=np.float32)[::-1]
    x[3, 8192] = 9.0
    x[4, 8191], x[4, 8192] = 2.0, 2.0
    token = np.array([0, 9000, V - 1, 8192], dtype=np.int32)
    store, xf = synth.round_to_dtype(x.astype(np.float64), dtype)
    ref = oracle.accept_greedy(xf, parent, token)
    assert ref["n_acc"] == 4 and ref["bonus"] == 8191
    stores = np.concatenate([store, store])                  # two requests with the same tree and logits
    logits = G.dev(stores, dtype == "bf16")
    par = G.dev(np.concatenate([parent, parent]).astype(np.int32)); tok = G.dev(np.concatenate([token, token]))
    qo = G.dev(np.array([0, M, 2 * M], dtype=np.int32))
    path = torch.full((2 * M,), -7, dtype=torch.int32, device="cuda")
    n_acc = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    am = torch.full((2 * M + 2,), -7, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_batch_workspace(2, 2 * M, V))
    btv.btv_tree_accept_greedy_batch(logits, par, tok, qo, M, path, n_acc, bonus, am, ws)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == 0
    for r in range(2):
        assert n_acc[r].item() == 4 and bonus[r].item() == 8191
        assert path[r * M:r * M + 4].tolist() == ref["path"].tolist()
        assert np.array_equal(am[r * (M + 1):(r + 1) * (M + 1)].cpu().numpy(), ref["argmax"])


def test_stream_read_runs_and_checks_arguments():
    """The bandwidth-ceiling aid: any 16-byte multiple is read without touching anything else; bad arguments raise."""
    import torch
    from paper_2605_29727_amd import binding as btv
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    for nbytes in (16, 4096 + 16, (1 << 20) + 48, 64 << 20):
        buf = torch.ones(nbytes // 4, dtype=torch.int32, device="cuda")
        guard = torch.full((1024,), 7, dtype=torch.int32, device="cuda")
        btv.btv_stream_read(buf, sink)
        torch.cuda.synchronize()
        assert bool((guard == 7).all()) and bool((buf == 1).all())
    # xor of an even number of equal words per workgroup share is deterministic: 64 MiB of ones folds to zero
    sink.zero_()
    btv.btv_stream_read(torch.ones((64 << 20) // 4, dtype=torch.int32, device="cuda"), sink)
    torch.cuda.synchronize()
    assert int(sink.abs().sum().item()) == 0
    with pytest.raises(btv.BtvError):
        btv.btv_stream_read(torch.ones(5, dtype=torch.int32, device="cuda")[1:], sink)       # 16 bytes, misaligned
    with pytest.raises(btv.BtvError):
        btv.btv_stream_read(torch.ones(4, dtype=torch.int32, device="cuda"), sink[:8])       # sink too small


def test_mfma_peak_runs_and_checks_arguments():
    """The matrix-core ceiling aid: reports the operations it launches (8 waves x iters x 4 instructions of
    2*32*32*16 flops per workgroup), writes only its sink, and refuses bad arguments."""
    import torch
    from paper_2605_29727_amd import binding as btv
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    guard = torch.full((1024,), 7, dtype=torch.int32, device="cuda")
    for wgs, iters in ((1, 1), (3, 17), (512, 100)):
        assert btv.btv_mfma_peak(wgs, iters, sink) == wgs * 8 * iters * 4 * 2 * 32 * 32 * 16
    torch.cuda.synchronize()
    assert bool((guard == 7).all())
    # the accumulators hold sums of products of small non-negative numbers: every wave's folded word is a finite float
    sink.zero_()
    btv.btv_mfma_peak(1, 4, sink)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink[:8].view(torch.float32)).all()) and bool((sink[:8] != 0).all())
    for bad in ((0, 10), (10, 0), (70000, 1)):
        with pytest.raises(btv.BtvError):
            btv.btv_mfma_peak(bad[0], bad[1], sink)
    with pytest.raises(btv.BtvError):
        btv.btv_mfma_peak(1, 1, sink[:8])


def test_accept_batch_flags_request_reaching_past_the_arrays():
    """q_offset entries that would make a request read past the total_M rows are refused on the device: the request
    gets n_acc = 0 and the data flag is raised, the others are walked as usual."""
    import torch
    import gpu_util as G
    from paper_2605_29727_amd import binding as btv
    V, Ms = 500, [6, 5]
    total = sum(Ms)
    pars = [synth.tree_parents(70 + r, M, "random") for r, M in enumerate(Ms)]
    toks = [synth.sibling_distinct_tokens(70 + r, p, V) for r, p in enumerate(pars)]
    st, _ = synth.target_logits(70, total + 2, V, 1.0, "fp32")
    q_offset = np.array([0, 6, 6 + 9], dtype=np.int32)        # request 1 claims 9 nodes: 4 more than the arrays hold
    path = torch.full((total,), -7, dtype=torch.int32, device="cuda")
    n_acc = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_batch_workspace(2, total, V))
    btv.btv_tree_accept_greedy_batch(G.dev(st), G.dev(np.concatenate(pars).astype(np.int32)),
                                     G.dev(np.concatenate(toks).astype(np.int32)), G.dev(q_offset), 16, path, n_acc, bonus,
                                     None, ws)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == btv.BTV_EDATA
    assert int(n_acc[1].item()) == 0 and int(n_acc[0].item()) >= 0
