"""Parity of the HIP tree-verify attention with the CPU oracle (needs an MI355X; all calls go through the C ABI).

Tolerances: max-abs 1e-5 for the fp32 path, 2e-2 for bf16 (outputs are O(1) convex combinations of N(0,1) values;
one bf16 rounding of the output alone is up to 2^-9 * |O| ~ 8e-3 at |O| = 4).
"""
import numpy as np
import pytest

from paper_2605_29727_amd import synth

pytestmark = pytest.mark.gpu

TOL_BF16, TOL_F32 = 2e-2, 1e-5
KINDS = ["chain", "star", "binary", "caterpillar", "random", "deep"]


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def test_config1_fp32_full_parity(G, oracle):
    w = synth.C1
    marg = synth.marginals(w.seed, w.B, w.V, w.marg_sigma)
    tree = oracle.tree_build(marg, w.N)
    t = synth.qkv(w.seed, w.N, w.L, w.Hq, w.Hkv, w.D, "fp32")
    ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], tree["parent"], w.L)
    out = G.run_verify_attn(t, tree["parent"], w.L, "fp32")
    assert np.abs(out - ref).max() <= TOL_F32


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("M,L,Hq,Hkv,D", [(16, 128, 1, 1, 64), (37, 300, 4, 2, 128), (5, 0, 2, 1, 64), (1, 77, 2, 2, 128)])
def test_fp32_shapes_and_trees(G, oracle, kind, M, L, Hq, Hkv, D):
    parent = synth.tree_parents(7, M, kind)
    t = synth.qkv(31, M, L, Hq, Hkv, D, "fp32", tag=kind)
    ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], parent, L)
    out = G.run_verify_attn(t, parent, L, "fp32")
    assert np.abs(out - ref).max() <= TOL_F32


# (M, L, Hq, Hkv, D): spans all three kernel configurations (G*M <= 64, <= 128, > 128 with several row blocks),
# ragged tails (M, L not multiples of 32 / 64), L = 0, L smaller than a tile, and a prefix/tree boundary inside a tile.
BF16_SHAPES = [
    (16, 256, 32, 8, 128), (1, 100, 4, 1, 128), (5, 0, 8, 2, 128), (33, 31, 8, 2, 128), (64, 777, 32, 8, 128),
    (100, 1000, 8, 2, 128), (256, 300, 8, 2, 128), (37, 513, 64, 8, 128), (16, 200, 8, 8, 64), (70, 129, 16, 4, 64),
    (13, 64, 4, 4, 128), (128, 96, 16, 2, 128),
]


@pytest.mark.parametrize("shape", BF16_SHAPES)
def test_bf16_elementwise_parity(G, oracle, shape):
    M, L, Hq, Hkv, D = shape
    for kind in ("random", "deep", "chain"):
        parent = synth.tree_parents(M + L, M, kind)
        t = synth.qkv(41, M, L, Hq, Hkv, D, "bf16", tag=f"{kind}{shape}")
        ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], parent, L)
        out = G.run_verify_attn(t, parent, L, "bf16")
        assert np.isfinite(out).all()
        assert np.abs(out - ref).max() <= TOL_BF16, (kind, shape, np.abs(out - ref).max())


@pytest.mark.parametrize("kind", KINDS)
def test_bf16_tree_kinds_with_split(G, oracle, kind):
    M, L, Hq, Hkv, D = 48, 1500, 16, 4, 128
    parent = synth.tree_parents(3, M, kind)
    t = synth.qkv(42, M, L, Hq, Hkv, D, "bf16", tag=kind)
    ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], parent, L)
    outs = [G.run_verify_attn(t, parent, L, "bf16", nsplit=ns) for ns in (1, 2, 5, 25)]
    for o in outs:
        assert np.abs(o - ref).max() <= TOL_BF16
    for o in outs[1:]:       # any split count gives the single-split result up to the final bf16 rounding
        assert np.abs(o - outs[0]).max() <= 2 ** -7


def test_bf16_scale_argument(G, oracle):
    M, L = 20, 150
    parent = synth.tree_parents(1, M, "random")
    t = synth.qkv(43, M, L, 8, 2, 128, "bf16")
    ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], parent, L, scale=0.05)
    out = G.run_verify_attn(t, parent, L, "bf16", scale=0.05)
    assert np.abs(out - ref).max() <= TOL_BF16


def test_bf16_deterministic_and_mask_tight(G, oracle):
    """Same input twice -> identical bits; changing K/V of a non-ancestor tree row leaves a node's output bit-identical."""
    M, L, Hq, Hkv, D = 40, 600, 8, 2, 128
    parent = synth.tree_parents(11, M, "random")
    t = synth.qkv(44, M, L, Hq, Hkv, D, "bf16")
    a = G.run_verify_attn(t, parent, L, "bf16", nsplit=4)
    b = G.run_verify_attn(t, parent, L, "bf16", nsplit=4)
    assert np.array_equal(a, b)
    anc = oracle.ancestor_mask(parent)
    victim = 7
    t2 = dict(t)
    for nm in ("K", "V"):
        bits = t[nm].copy()
        bits[L + victim] ^= np.uint16(0x0180)            # flip mantissa/exponent bits of that tree row
        t2[nm] = bits
        t2[nm + "f"] = synth.bf16_bits_to_f32(bits)
    c = G.run_verify_attn(t2, parent, L, "bf16", nsplit=4)
    for i in range(M):
        sees = bool((anc[i, victim // 32] >> np.uint32(victim % 32)) & np.uint32(1))
        assert np.array_equal(c[i], a[i]) != sees, i


def test_ancestor_mask_bit_exact(G, oracle):
    import torch
    from paper_2605_29727_amd import binding as btv
    for kind in KINDS:
        for M in (1, 31, 32, 33, 200, 256):
            parent = synth.tree_parents(M, M, kind)
            anc = torch.zeros((M, 8), dtype=torch.int32, device="cuda")
            ws = btv.alloc_workspace(256)
            btv.btv_tree_ancestor_mask(G.dev(parent), anc, ws)
            torch.cuda.synchronize()
            assert np.array_equal(anc.cpu().numpy().view(np.uint32), oracle.ancestor_mask(parent))


def test_invalid_parent_is_flagged_not_faulting(G):
    import torch
    from paper_2605_29727_amd import binding as btv
    M, L = 8, 64
    t = synth.qkv(45, M, L, 4, 2, 128, "bf16")
    parent = synth.tree_parents(0, M, "chain")
    parent[3] = 5                                             # parent >= own index: invalid
    Q, K, V = G.dev(t["Q"], True), G.dev(t["K"], True), G.dev(t["V"], True)
    O = torch.zeros_like(Q)
    ws = btv.alloc_workspace(btv.btv_tree_verify_attn_workspace(M, L, 4, 2, 128, btv.BTV_BF16))
    btv.btv_tree_verify_attn(Q, K, V, G.dev(parent), L, O, ws)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == btv.BTV_EDATA
    assert btv.btv_workspace_status(ws) == btv.BTV_OK        # the flag is cleared by the read
    assert torch.isfinite(O.float()).all()


def _full_size_check(G, oracle, w, N, seed_tag):
    """Every (node, head) row of the full-size configuration against the oracle (the oracle runs all rows of the
    largest configuration in well under a minute on the GPU machine's host cores)."""
    marg = synth.marginals(w.seed, w.B, w.V, w.marg_sigma)
    tree = oracle.tree_build(marg, N)
    t = synth.qkv(w.seed, N, w.L, w.Hq, w.Hkv, w.D, "bf16", tag=seed_tag)
    out = G.run_verify_attn(t, tree["parent"], w.L, "bf16")
    assert np.isfinite(out).all()
    ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], tree["parent"], w.L)
    assert out.shape == ref.shape
    assert np.abs(out - ref).max() <= TOL_BF16, np.abs(out - ref).max()
    return out


def test_config2_full_size(G, oracle):
    _full_size_check(G, oracle, synth.C2, synth.C2.N, "c2")


@pytest.mark.parametrize("N", synth.C3_SIZES)
@pytest.mark.parametrize("sharp", [True, False])
def test_config3_budget_sweep_full_size(G, oracle, N, sharp):
    _full_size_check(G, oracle, synth.c3(N, sharp), N, f"c3{N}{sharp}")


def test_config5_70b_shape_full_size(G, oracle):
    _full_size_check(G, oracle, synth.C5, synth.C5.N, "c5")


# Every kernel shape on inputs the heuristic would give to another one: (M, L, Hq, Hkv, D), ragged tails in M and L,
# prefix/tree boundary inside a tile, fewer rows than the workgroup holds, several row blocks, one and several splits.
FORCED_SHAPES = [(16, 700, 32, 8, 128), (100, 1000, 8, 2, 128), (37, 513, 64, 8, 128), (70, 129, 16, 4, 64),
                 (5, 0, 8, 2, 128), (256, 300, 8, 2, 128)]


@pytest.mark.parametrize("shape_id", [1, 2, 3])
@pytest.mark.parametrize("dims", FORCED_SHAPES)
def test_bf16_every_kernel_shape_elementwise(G, oracle, shape_id, dims):
    M, L, Hq, Hkv, D = dims
    for kind, ns in (("random", 0), ("deep", 3)):
        parent = synth.tree_parents(M + L + shape_id, M, kind)
        t = synth.qkv(46, M, L, Hq, Hkv, D, "bf16", tag=f"{kind}{dims}")
        ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], parent, L)
        out = G.run_verify_attn(t, parent, L, "bf16", nsplit=ns, shape=shape_id)
        assert np.isfinite(out).all()
        assert np.abs(out - ref).max() <= TOL_BF16, (kind, dims, shape_id, np.abs(out - ref).max())


@pytest.mark.parametrize("dims,kind", [((256, 16384, 32, 8, 128), "random"), ((131, 16397, 16, 2, 128), "deep"),
                                       ((250, 16415, 64, 8, 128), "chain")])
def test_bf16_long_prefix_many_rows_elementwise(G, oracle, dims, kind):
    """Sizes at which the heuristic itself picks the 256-row workgroup (at least 1024 packed rows per KV head over a
    prefix of at least 16384 keys): every element, with ragged tails in both dimensions and deep trees."""
    M, L, Hq, Hkv, D = dims
    parent = synth.tree_parents(M + L, M, kind)
    t = synth.qkv(47, M, L, Hq, Hkv, D, "bf16", tag=f"{kind}{dims}")
    ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], parent, L)
    out = G.run_verify_attn(t, parent, L, "bf16")
    assert np.isfinite(out).all()
    assert np.abs(out - ref).max() <= TOL_BF16, (dims, kind, np.abs(out - ref).max())


def _paged_case(G, oracle, Ls, Ns, Hq, Hkv, D, seed):
    import torch
    from paper_2605_29727_amd import binding as btv
    batch = len(Ls)
    bt, nb = synth.paged_layout(seed, [l + n for l, n in zip(Ls, Ns)])
    Kp = np.zeros((nb, synth.PAGE, Hkv, D), dtype=np.uint16)
    Vp = np.zeros_like(Kp)
    # unused pool slots hold NaN so that any stray read shows up
    Kp[:] = 0x7FC0
    Vp[:] = 0x7FC0
    qoff = np.zeros(batch + 1, dtype=np.int32)
    qoff[1:] = np.cumsum(Ns)
    Qall = np.zeros((int(qoff[-1]), Hq, D), dtype=np.uint16)
    parents = np.zeros(int(qoff[-1]), dtype=np.int32)
    reqs = []
    for r in range(batch):
        t = synth.qkv(seed, Ns[r], Ls[r], Hq, Hkv, D, "bf16", tag=f"req{r}")
        kinds = ["random", "deep", "binary", "chain", "star", "caterpillar"]
        parent = synth.tree_parents(seed + r, Ns[r], kinds[r % len(kinds)])
        synth.scatter_to_pages(t["K"], bt[r], Kp)
        synth.scatter_to_pages(t["V"], bt[r], Vp)
        Qall[qoff[r]:qoff[r + 1]] = t["Q"]
        parents[qoff[r]:qoff[r + 1]] = parent
        reqs.append((t, parent))
    Q, K, V = G.dev(Qall, True), G.dev(Kp, True), G.dev(Vp, True)
    O = torch.full_like(Q, float("nan"))
    M_max, L_max = max(Ns), max(Ls)
    ws = btv.alloc_workspace(btv.btv_tree_verify_attn_paged_workspace(batch, M_max, L_max, Hq, Hkv, D))
    btv.btv_tree_verify_attn_paged(Q, K, V, G.dev(bt), G.dev(qoff), G.dev(np.asarray(Ls, dtype=np.int32)),
                                   G.dev(parents), M_max, L_max, O, ws)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == 0
    out = G.host(O).astype(np.float64)
    assert np.isfinite(out).all()
    Kpf, Vpf = synth.bf16_bits_to_f32(Kp), synth.bf16_bits_to_f32(Vp)
    for r, (t, parent) in enumerate(reqs):
        o = out[qoff[r]:qoff[r + 1]]
        ref = oracle.tree_attn(t["Qf"], Kpf, Vpf, parent, Ls[r], block_table=bt[r], page=synth.PAGE)
        assert np.abs(o - ref).max() <= TOL_BF16, r


def test_paged_ragged_small(G, oracle):
    _paged_case(G, oracle, [100, 0, 333, 17, 1025], [9, 5, 33, 1, 64], 8, 2, 128, seed=61)
    _paged_case(G, oracle, [640, 64], [70, 130], 8, 2, 64, seed=62)


def test_config4_ragged_paged_full_size(G, oracle):
    Ls, Ns = synth.c4_request_shapes()
    _paged_case(G, oracle, Ls, Ns, 32, 8, 128, seed=synth.C4.seed)


def test_paged_ragged_several_splits(G, oracle):
    """Prefixes long enough for several key splits per request, of very different lengths: the split index is
    rotated per (request, head), short requests skip the splits they do not have, every element is compared."""
    _paged_case(G, oracle, [5000, 300, 2500, 4097, 64, 9000], [40, 64, 7, 100, 130, 16], 8, 2, 128, seed=63)
    _paged_case(G, oracle, [2100, 2047, 2049], [33, 32, 31], 4, 4, 64, seed=64)


@pytest.mark.parametrize("seed", range(24))
def test_bf16_random_shapes(G, oracle, seed):
    """Seeded random shapes inside the documented limits (ragged M and L, every GQA ratio up to 16, both head sizes,
    every tree kind), each compared element by element."""
    r = lambda tag, lo, hi: int(synth.integers(1000 + seed, tag, (1,), lo, hi)[0])
    D = (64, 128)[r("D", 0, 1)]
    Hkv = (1, 2, 4, 8)[r("Hkv", 0, 3)]
    Gq = (1, 2, 4, 8, 16)[r("G", 0, 4)]
    M = r("M", 1, 256) if seed % 3 else r("M", 1, 40)
    L = (0, r("L", 1, 31), r("L", 32, 700), r("L", 701, 3000))[r("Lk", 0, 3)]
    kind = KINDS[r("kind", 0, len(KINDS) - 1)]
    if M * Gq * Hkv * (L + M) > 6_000_000:      # keep the oracle's share of the test short
        L = min(L, 600)
    parent = synth.tree_parents(seed, M, kind)
    t = synth.qkv(2000 + seed, M, L, Hkv * Gq, Hkv, D, "bf16", tag="fz")
    ref = oracle.tree_attn(t["Qf"], t["Kf"], t["Vf"], parent, L)
    out = G.run_verify_attn(t, parent, L, "bf16")
    assert np.isfinite(out).all()
    assert np.abs(out - ref).max() <= TOL_BF16, (M, L, Hkv * Gq, Hkv, D, kind, np.abs(out - ref).max())
