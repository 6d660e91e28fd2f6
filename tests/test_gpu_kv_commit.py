"""Bit-exact parity of the HIP KV commit with the CPU oracle, contiguous and paged, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2605_29727_amd import binding as btv
from paper_2605_29727_amd import synth

pytestmark = pytest.mark.gpu


def _path(rng, M, n):
    return np.sort(rng.choice(M, size=n, replace=False)).astype(np.int32)


def _torch(a):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def _numpy(t, like):
    if like.dtype == np.uint16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


@pytest.mark.parametrize("layers,L,M,n,shape", [(1, 0, 4, 2, (2, 8)), (3, 37, 64, 9, (8, 128)), (2, 500, 256, 16, (1, 64)),
                                                (4, 100, 16, 16, (2, 16)), (2, 7, 5, 0, (2, 4)), (32, 8192, 64, 7, (8, 128)),
                                                (2, 300, 256, 200, (8, 128)), (1, 10, 256, 256, (8, 128))])
@pytest.mark.parametrize("dtype", [np.uint16, np.float32])
def test_contiguous(oracle, layers, L, M, n, shape, dtype):
    rng = np.random.default_rng(1000 * layers + L + M + n)
    Kh = rng.integers(0, 60000, size=(layers, L + M) + shape).astype(dtype)
    Vh = rng.integers(0, 60000, size=(layers, L + M) + shape).astype(dtype)
    path = _path(rng, M, n)
    Kd, Vd = _torch(Kh), _torch(Vh)
    pd = torch.full((M,), -3, dtype=torch.int32, device="cuda")
    pd[:n] = torch.from_numpy(path).cuda()
    nd = torch.tensor([n], dtype=torch.int32, device="cuda")
    new_len = torch.zeros(1, dtype=torch.int32, device="cuda")
    btv.btv_kv_commit(Kd, Vd, L, M, pd, nd, new_len)
    torch.cuda.synchronize()
    assert oracle.kv_commit(Kh, L, M, path) == L + n == int(new_len.item())
    oracle.kv_commit(Vh, L, M, path)
    assert np.array_equal(_numpy(Kd, Kh)[:, :L + n], Kh[:, :L + n])
    assert np.array_equal(_numpy(Vd, Vh)[:, :L + n], Vh[:, :L + n])


@pytest.mark.parametrize("layers,L,M,n", [(3, 37, 64, 9), (32, 8192, 64, 7), (2, 300, 256, 200)])
def test_contiguous_one_byte_elements(oracle, layers, L, M, n):
    """An FP8 cache: rows of Hkv * D single bytes."""
    rng = np.random.default_rng(77 + layers + L)
    Kh = rng.integers(0, 256, size=(layers, L + M, 8, 128)).astype(np.uint8)
    Vh = rng.integers(0, 256, size=(layers, L + M, 8, 128)).astype(np.uint8)
    path = _path(rng, M, n)
    Kd, Vd = _torch(Kh), _torch(Vh)
    pd = torch.full((M,), -3, dtype=torch.int32, device="cuda")
    pd[:n] = torch.from_numpy(path).cuda()
    nd = torch.tensor([n], dtype=torch.int32, device="cuda")
    btv.btv_kv_commit(Kd, Vd, L, M, pd, nd, None)
    torch.cuda.synchronize()
    assert oracle.kv_commit(Kh, L, M, path) == L + n
    oracle.kv_commit(Vh, L, M, path)
    assert np.array_equal(Kd.cpu().numpy()[:, :L + n], Kh[:, :L + n])
    assert np.array_equal(Vd.cpu().numpy()[:, :L + n], Vh[:, :L + n])


def test_paged_ragged_batch(oracle):
    """Eight requests with their own prefix lengths, trees and accepted paths over one pool (the ragged, paged
    configuration), four layers; blocks that belong to no request must stay as they were."""
    rng = np.random.default_rng(42)
    layers, batch, page, Hkv, D, M_max = 4, 8, synth.PAGE, 8, 128, 128
    Ls = rng.integers(1024, 4096, size=batch)
    Ms = rng.integers(32, M_max + 1, size=batch)
    nblk = [-(-(int(l) + int(m)) // page) for l, m in zip(Ls, Ms)]
    num_blocks = sum(nblk) + 17
    max_blocks = max(nblk)
    perm = rng.permutation(num_blocks)
    bt = np.zeros((batch, max_blocks), dtype=np.int32)
    o = 0
    for r in range(batch):
        bt[r, :nblk[r]] = perm[o:o + nblk[r]]; o += nblk[r]
    Kh = rng.integers(0, 60000, size=(layers, num_blocks, page, Hkv, D)).astype(np.uint16)
    Vh = rng.integers(0, 60000, size=(layers, num_blocks, page, Hkv, D)).astype(np.uint16)
    paths = np.full((batch, M_max), -5, dtype=np.int32)
    nacc = np.zeros(batch, dtype=np.int32)
    for r in range(batch):
        nacc[r] = rng.integers(0, 17)
        paths[r, :nacc[r]] = _path(rng, int(Ms[r]), int(nacc[r]))
    Kd, Vd = _torch(Kh), _torch(Vh)
    new_len = torch.zeros(batch, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(256)
    btv.btv_kv_commit_paged(Kd, Vd, torch.from_numpy(bt).cuda(), torch.from_numpy(Ls.astype(np.int32)).cuda(),
                            torch.from_numpy(paths).cuda(), torch.from_numpy(nacc).cuda(), new_len, ws)
    torch.cuda.synchronize()
    assert int(btv.btv_workspace_status(ws)) == 0
    for r in range(batch):
        oracle.kv_commit(Kh, int(Ls[r]), int(Ms[r]), paths[r, :nacc[r]], block_table=bt[r, :nblk[r]], page=page)
        oracle.kv_commit(Vh, int(Ls[r]), int(Ms[r]), paths[r, :nacc[r]], block_table=bt[r, :nblk[r]], page=page)
    assert np.array_equal(new_len.cpu().numpy(), (Ls + nacc).astype(np.int32))
    # dead rows (positions from L + n_acc on) are unspecified: compare the live positions and every block outside
    Kg, Vg = _numpy(Kd, Kh), _numpy(Vd, Vh)
    live = np.zeros((num_blocks, page), dtype=bool)
    owned = np.zeros(num_blocks, dtype=bool)
    for r in range(batch):
        pos = np.arange(int(Ls[r]) + int(nacc[r]))
        live[bt[r, pos // page], pos % page] = True
        owned[bt[r, :nblk[r]]] = True
    assert np.array_equal(Kg[:, live], Kh[:, live]) and np.array_equal(Vg[:, live], Vh[:, live])
    assert np.array_equal(Kg[:, ~owned], Kh[:, ~owned]) and np.array_equal(Vg[:, ~owned], Vh[:, ~owned])


def test_out_of_range_request_is_flagged_and_left_alone():
    layers, page, Hkv, D = 2, synth.PAGE, 2, 64
    K = torch.arange(layers * 8 * page * Hkv * D, dtype=torch.float32, device="cuda").reshape(layers, 8, page, Hkv, D)
    V = K.clone() + 1
    K0, V0 = K.clone(), V.clone()
    bt = torch.arange(8, dtype=torch.int32, device="cuda").reshape(1, 8)
    path = torch.zeros((1, 32), dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(256)
    btv.btv_kv_commit_paged(K, V, bt, torch.tensor([50], dtype=torch.int32, device="cuda"), path,
                            torch.tensor([40], dtype=torch.int32, device="cuda"), None, ws)     # n_acc > M_max
    torch.cuda.synchronize()
    assert int(btv.btv_workspace_status(ws)) != 0
    assert torch.equal(K, K0) and torch.equal(V, V0)


def test_host_checks():
    K = torch.zeros((1, 8, 2, 3), dtype=torch.bfloat16, device="cuda")           # 12-byte rows
    p = torch.zeros(4, dtype=torch.int32, device="cuda")
    n = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(btv.BtvError):
        btv.btv_kv_commit(K, K.clone(), 4, 4, p, n)
