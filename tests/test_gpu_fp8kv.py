"""Parity of the FP8-KV tree-verify attention with the CPU oracle (needs an MI355X; all calls go through the C ABI).

The kernel converts the E4M3 codes exactly and then runs the bf16 arithmetic of the plain entry point, so the
tolerance is that path's: max-abs 2e-2 against the fp64 oracle over the numbers the codes stand for.
"""
import numpy as np
import pytest

from paper_2605_29727_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-2
D = 128


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _inputs(seed, M, L, Hq, Hkv, tag=""):
    q = synth.qkv(seed, M, L, Hq, Hkv, D, "bf16", tag=tag)
    kv = synth.kv_fp8(seed, L + M, Hkv, D, tag=tag)
    return q, kv


def _oracle(oracle, q, kv, parent, L, **kw):
    return oracle.tree_attn_fp8kv(q["Qf"], kv["K8"], kv["V8"], kv["k_scale"], kv["v_scale"], parent, L, **kw)


# (M, L, Hq, Hkv): both kernel shapes (G*M <= 128 and above, several row blocks), ragged tails, L = 0, L below a tile,
# a prefix/tree boundary inside a tile, a single node
SHAPES = [(16, 256, 32, 8), (1, 100, 4, 1), (5, 0, 8, 2), (33, 31, 8, 2), (64, 777, 32, 8), (100, 1000, 8, 2),
          (256, 300, 8, 2), (37, 513, 64, 8), (13, 64, 4, 4), (128, 96, 16, 2), (200, 40, 16, 1)]


@pytest.mark.parametrize("shape", SHAPES)
def test_elementwise_parity(G, oracle, shape):
    M, L, Hq, Hkv = shape
    for kind in ("random", "deep", "chain"):
        parent = synth.tree_parents(M + L, M, kind)
        q, kv = _inputs(71, M, L, Hq, Hkv, tag=f"{kind}{shape}")
        ref = _oracle(oracle, q, kv, parent, L)
        out = G.run_verify_attn_fp8kv(q["Q"], kv, parent, L)
        assert np.isfinite(out).all()
        assert np.abs(out - ref).max() <= TOL, (kind, shape, np.abs(out - ref).max())


@pytest.mark.parametrize("shape_id", [1, 2])
@pytest.mark.parametrize("dims", [(16, 700, 32, 8), (100, 1000, 8, 2), (37, 513, 64, 8), (256, 300, 8, 2)])
def test_every_kernel_shape_elementwise(G, oracle, shape_id, dims):
    """Both kernel shapes built for the FP8 cache on inputs the heuristic would give to the other one."""
    M, L, Hq, Hkv = dims
    parent = synth.tree_parents(M + L + shape_id, M, "deep")
    q, kv = _inputs(74, M, L, Hq, Hkv, tag=f"forced{dims}")
    ref = _oracle(oracle, q, kv, parent, L)
    out = G.run_verify_attn_fp8kv(q["Q"], kv, parent, L, nsplit=3, shape=shape_id)
    assert np.isfinite(out).all()
    assert np.abs(out - ref).max() <= TOL, (dims, shape_id, np.abs(out - ref).max())


@pytest.mark.parametrize("kind", ["chain", "star", "binary", "caterpillar", "random", "deep"])
def test_tree_kinds_with_split(G, oracle, kind):
    M, L, Hq, Hkv = 48, 1500, 16, 4
    parent = synth.tree_parents(3, M, kind)
    q, kv = _inputs(72, M, L, Hq, Hkv, tag=kind)
    ref = _oracle(oracle, q, kv, parent, L)
    outs = [G.run_verify_attn_fp8kv(q["Q"], kv, parent, L, nsplit=ns) for ns in (1, 2, 5, 25)]
    for o in outs:
        assert np.abs(o - ref).max() <= TOL
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() <= 2 ** -7


def test_scales_and_softmax_scale(G, oracle):
    M, L = 20, 150
    parent = synth.tree_parents(1, M, "random")
    q, kv = _inputs(73, M, L, 8, 2)
    for ks, vs, sc in ((kv["k_scale"], kv["v_scale"], 0.05), (0.0173, 2.9, 0.0), (1.0, 1.0, 0.001)):
        k2 = dict(kv, k_scale=ks, v_scale=vs)
        ref = _oracle(oracle, q, k2, parent, L, scale=sc if sc > 0 else None)
        out = G.run_verify_attn_fp8kv(q["Q"], k2, parent, L, scale=sc)
        # outputs scale with v_scale (codes up to 448 at v_scale 1): the bound is relative to that magnitude
        bound = TOL * max(1.0, np.abs(ref).max() / 4.0)
        assert np.abs(out - ref).max() <= bound, (ks, vs, sc)


def test_every_code_converts_exactly(G):
    """One node, no prefix: the node sees only itself, so O = V's own row.  With v_scale = 1 the output is the
    decoded code, exactly (every E4M3 number is a bf16 number).  Two KV heads x 128 channels hold all 256 codes."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    codes[[0x7F, 0xFF]] = [0x00, 0x80]                    # the two NaN codes are tested on their own below
    V8 = codes.reshape(1, 2, D)
    K8 = np.full((1, 2, D), 0x38, dtype=np.uint8)
    q = synth.qkv(74, 1, 0, 2, 2, D, "bf16")
    kv = {"K8": K8, "V8": V8, "k_scale": 1.0, "v_scale": 1.0}
    out = G.run_verify_attn_fp8kv(q["Q"], kv, np.array([-1], dtype=np.int32), 0)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy().reshape(2, D)
    assert np.array_equal(out[0], want)
    V8n = V8.copy()
    V8n[0, 1, 5] = 0x7F
    out = G.run_verify_attn_fp8kv(q["Q"], dict(kv, V8=V8n), np.array([-1], dtype=np.int32), 0)
    assert np.isnan(out[0, 1, 5]) and np.isfinite(out[0, 0]).all()


def test_matches_bf16_entry_point_on_the_same_numbers(G):
    """With both scales 1 the codes' values are bf16 numbers: the plain bf16 entry point on those numbers computes
    the same sums in another order."""
    import torch
    M, L, Hq, Hkv = 40, 700, 8, 2
    parent = synth.tree_parents(9, M, "random")
    q, kv = _inputs(75, M, L, Hq, Hkv)
    kv = dict(kv, k_scale=1.0, v_scale=1.0)
    o8 = G.run_verify_attn_fp8kv(q["Q"], kv, parent, L, scale=0.0009)
    t = dict(q)
    for nm in ("K", "V"):
        f = torch.from_numpy(kv[nm + "8"]).view(torch.float8_e4m3fn).to(torch.float32).numpy()
        t[nm] = synth.f32_to_bf16_bits(f)
        assert np.array_equal(synth.bf16_bits_to_f32(t[nm]), f)
    o16 = G.run_verify_attn(t, parent, L, "bf16", scale=0.0009)
    assert np.abs(o8 - o16).max() <= np.abs(o16).max() * 2 ** -6


def test_deterministic_and_mask_tight(G, oracle):
    M, L, Hq, Hkv = 40, 600, 8, 2
    parent = synth.tree_parents(11, M, "random")
    q, kv = _inputs(76, M, L, Hq, Hkv)
    a = G.run_verify_attn_fp8kv(q["Q"], kv, parent, L, nsplit=4)
    b = G.run_verify_attn_fp8kv(q["Q"], kv, parent, L, nsplit=4)
    assert np.array_equal(a, b)
    anc = oracle.ancestor_mask(parent)
    victim = 7
    kv2 = dict(kv)
    for nm in ("K8", "V8"):
        c = kv[nm].copy()
        c[L + victim] ^= np.uint8(0x14)
        c[L + victim][(c[L + victim] & 0x7F) == 0x7F] = 0x70          # keep clear of the NaN code
        kv2[nm] = c
    c = G.run_verify_attn_fp8kv(q["Q"], kv2, parent, L, nsplit=4)
    for i in range(M):
        sees = bool((anc[i, victim // 32] >> np.uint32(victim % 32)) & np.uint32(1))
        assert np.array_equal(c[i], a[i]) != sees, i


@pytest.mark.parametrize("which", ["c3_16", "c3_64", "c3_256", "c5"])
def test_full_size_configurations(G, oracle, which):
    w = synth.C5 if which == "c5" else synth.c3(int(which.split("_")[1]))
    N = w.N
    marg = synth.marginals(w.seed, w.B, w.V, w.marg_sigma)
    tree = oracle.tree_build(marg, N)
    q, kv = _inputs(w.seed, N, w.L, w.Hq, w.Hkv, tag=which)
    out = G.run_verify_attn_fp8kv(q["Q"], kv, tree["parent"], w.L)
    assert np.isfinite(out).all()
    ref = _oracle(oracle, q, kv, tree["parent"], w.L)                  # every (node, head) row
    assert np.abs(out - ref).max() <= TOL
    assert np.abs(out).max() <= 448.0 * kv["v_scale"] + 1e-2          # convex combinations of V rows


def _paged_case(G, oracle, Ls, Ns, Hq, Hkv, seed):
    import torch
    from paper_2605_29727_amd import binding as btv
    batch = len(Ls)
    bt, nb = synth.paged_layout(seed, [l + n for l, n in zip(Ls, Ns)])
    # unused pool slots hold the NaN code so that any stray read shows up
    Kp = np.full((nb, synth.PAGE, Hkv, D), 0x7F, dtype=np.uint8)
    Vp = np.full_like(Kp, 0x7F)
    qoff = np.zeros(batch + 1, dtype=np.int32)
    qoff[1:] = np.cumsum(Ns)
    Qall = np.zeros((int(qoff[-1]), Hq, D), dtype=np.uint16)
    parents = np.zeros(int(qoff[-1]), dtype=np.int32)
    reqs = []
    ks, vs = 0.0131, 0.0117                  # one pair of scales for the whole pool
    for r in range(batch):
        q, kv = _inputs(seed, Ns[r], Ls[r], Hq, Hkv, tag=f"req{r}")
        kinds = ["random", "deep", "binary", "chain", "star", "caterpillar"]
        parent = synth.tree_parents(seed + r, Ns[r], kinds[r % len(kinds)])
        synth.scatter_to_pages(kv["K8"], bt[r], Kp)
        synth.scatter_to_pages(kv["V8"], bt[r], Vp)
        Qall[qoff[r]:qoff[r + 1]] = q["Q"]
        parents[qoff[r]:qoff[r + 1]] = parent
        reqs.append((q, parent))
    Q, K, V = G.dev(Qall, True), G.dev(Kp), G.dev(Vp)
    O = torch.full_like(Q, float("nan"))
    M_max, L_max = max(Ns), max(Ls)
    ws = btv.alloc_workspace(btv.btv_tree_verify_attn_paged_fp8kv_workspace(batch, M_max, L_max, Hq, Hkv, D))
    btv.btv_tree_verify_attn_paged_fp8kv(Q, K, V, ks, vs, G.dev(bt), G.dev(qoff), G.dev(np.asarray(Ls, dtype=np.int32)),
                                         G.dev(parents), M_max, L_max, O, ws)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == 0
    out = G.host(O).astype(np.float64)
    assert np.isfinite(out).all()
    for r, (q, parent) in enumerate(reqs):
        o = out[qoff[r]:qoff[r + 1]]
        ref = oracle.tree_attn_fp8kv(q["Qf"], Kp, Vp, ks, vs, parent, Ls[r], block_table=bt[r], page=synth.PAGE)
        assert np.abs(o - ref).max() <= TOL, r


def test_paged_ragged(G, oracle):
    _paged_case(G, oracle, [100, 0, 333, 17, 1025], [9, 5, 33, 1, 64], 8, 2, seed=81)
    _paged_case(G, oracle, [5000, 300, 2500, 4097, 64, 9000], [40, 64, 7, 100, 130, 16], 8, 2, seed=83)


def test_config4_ragged_paged_full_size(G, oracle):
    Ls, Ns = synth.c4_request_shapes()
    _paged_case(G, oracle, Ls, Ns, 32, 8, seed=synth.C4.seed)


def test_unsupported_arguments_are_refused(G):
    import torch
    from paper_2605_29727_amd import binding as btv
    assert btv.btv_tree_verify_attn_fp8kv_workspace(8, 64, 4, 2, 64) == 0
    q = synth.qkv(77, 8, 64, 4, 2, D, "bf16")
    kv = synth.kv_fp8(77, 72, 2, D)
    Q, K8, V8 = G.dev(q["Q"], True), G.dev(kv["K8"]), G.dev(kv["V8"])
    par = G.dev(synth.tree_parents(0, 8, "chain"))
    O = torch.zeros_like(Q)
    ws = btv.alloc_workspace(btv.btv_tree_verify_attn_fp8kv_workspace(8, 64, 4, 2, D))
    for ks, vs in ((0.0, 1.0), (1.0, -1.0), (float("nan"), 1.0), (float("inf"), 1.0)):
        with pytest.raises(btv.BtvError):
            btv.btv_tree_verify_attn_fp8kv(Q, K8, V8, ks, vs, par, 64, O, ws)
    with pytest.raises(btv.BtvError):
        btv.btv_tree_verify_attn_fp8kv(Q, K8, V8, 1.0, 1.0, par, 64, O, ws[:64])
    assert (O == 0).all()


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes(G, oracle, seed):
    """Seeded random shapes inside the documented limits (ragged M and L, every GQA ratio up to 16, every tree kind),
    each compared element by element."""
    kinds = ["chain", "star", "binary", "caterpillar", "random", "deep"]
    r = lambda tag, lo, hi: int(synth.integers(3000 + seed, tag, (1,), lo, hi)[0])
    Hkv = (1, 2, 4, 8)[r("Hkv", 0, 3)]
    Gq = (1, 2, 4, 8, 16)[r("G", 0, 4)]
    M = r("M", 1, 256) if seed % 3 else r("M", 1, 40)
    L = (0, r("L", 1, 31), r("L", 32, 700), r("L", 701, 3000))[r("Lk", 0, 3)]
    kind = kinds[r("kind", 0, len(kinds) - 1)]
    if M * Gq * Hkv * (L + M) > 6_000_000:      # keep the oracle's share of the test short
        L = min(L, 600)
    parent = synth.tree_parents(seed, M, kind)
    q, kv = _inputs(4000 + seed, M, L, Hkv * Gq, Hkv, tag="fz")
    ref = _oracle(oracle, q, kv, parent, L)
    out = G.run_verify_attn_fp8kv(q["Q"], kv, parent, L)
    assert np.isfinite(out).all()
    assert np.abs(out - ref).max() <= TOL, (M, L, Hkv * Gq, Hkv, kind, np.abs(out - ref).max())
