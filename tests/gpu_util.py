"""Helpers for the -m gpu tests: numpy <-> device marshalling and one-call wrappers over the binding."""
import numpy as np
import torch

from paper_2605_29727_amd import binding as btv


def dev(a: np.ndarray, bf16_bits: bool = False) -> torch.Tensor:
    if bf16_bits:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


def run_verify_attn(t: dict, parent: np.ndarray, L: int, dtype: str, scale: float = 0.0, nsplit: int = 0, shape: int = 0,
                    check_status: bool = True):
    """t: dict from synth.qkv.  Returns O as float64 numpy [M,Hq,D].  With nsplit or shape the tuning entry point runs."""
    bits = dtype == "bf16"
    Q, K, V = dev(t["Q"], bits), dev(t["K"], bits), dev(t["V"], bits)
    par = dev(np.asarray(parent, dtype=np.int32))
    M, Hq, D = Q.shape
    O = torch.full_like(Q, float("nan"))
    if nsplit or shape:
        ws = btv.alloc_workspace(btv.btv_tree_verify_attn_tuned_workspace(M, L, Hq, K.shape[1], D, False, nsplit, shape))
        btv.btv_tree_verify_attn_tuned(Q, K, V, par, L, O, ws, scale, nsplit, shape)
    else:
        ws = btv.alloc_workspace(btv.btv_tree_verify_attn_workspace(M, L, Hq, K.shape[1], D, btv._dtype_code(Q)))
        btv.btv_tree_verify_attn(Q, K, V, par, L, O, ws, scale)
    torch.cuda.synchronize()
    if check_status:
        assert btv.btv_workspace_status(ws) == 0
    return host(O).astype(np.float64)


def run_verify_attn_fp8kv(Q_bits: np.ndarray, kv: dict, parent: np.ndarray, L: int, scale: float = 0.0, nsplit: int = 0,
                          shape: int = 0, check_status: bool = True):
    """Q_bits: bf16 bit patterns [M,Hq,D]; kv: dict from synth.kv_fp8 (K8, V8, k_scale, v_scale).  O as float64."""
    Q, K8, V8 = dev(Q_bits, True), dev(kv["K8"]), dev(kv["V8"])
    par = dev(np.asarray(parent, dtype=np.int32))
    M, Hq, D = Q.shape
    O = torch.full_like(Q, float("nan"))
    if nsplit or shape:
        ws = btv.alloc_workspace(btv.btv_tree_verify_attn_tuned_workspace(M, L, Hq, K8.shape[1], D, True, nsplit, shape))
        btv.btv_tree_verify_attn_tuned(Q, K8, V8, par, L, O, ws, scale, nsplit, shape, kv["k_scale"], kv["v_scale"])
    else:
        ws = btv.alloc_workspace(btv.btv_tree_verify_attn_fp8kv_workspace(M, L, Hq, K8.shape[1], D))
        btv.btv_tree_verify_attn_fp8kv(Q, K8, V8, kv["k_scale"], kv["v_scale"], par, L, O, ws, scale)
    torch.cuda.synchronize()
    if check_status:
        assert btv.btv_workspace_status(ws) == 0
    return host(O).astype(np.float64)


def run_tree_build(marg: np.ndarray, N: int, algo: int = 0) -> dict:
    """algo 0: btv_tree_build; 1 / 2: the tuned entry point with the one-wavefront / level-synchronous expansion."""
    m = dev(marg.astype(np.float32))
    B, V = marg.shape
    parent = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    token = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    depth = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    rho = torch.full((N,), -7.0, dtype=torch.float32, device="cuda")
    n_out = torch.zeros(1, dtype=torch.int32, device="cuda")
    ahat = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_build_workspace(B, V, N))
    if algo:
        btv.btv_tree_build_tuned(m, N, algo, parent, token, depth, rho, n_out, ahat, ws)
    else:
        btv.btv_tree_build(m, N, parent, token, depth, rho, n_out, ahat, ws)
    torch.cuda.synchronize()
    assert btv.btv_workspace_status(ws) == 0
    n = int(n_out.item())
    return {"n": n, "parent": parent.cpu().numpy()[:n], "token": token.cpu().numpy()[:n],
            "depth": depth.cpu().numpy()[:n], "rho": rho.cpu().numpy()[:n], "ahat": float(ahat.item()),
            "raw_parent": parent.cpu().numpy()}


def run_tree_build_adaptive(marg: np.ndarray, N_max: int, cost: np.ndarray, L_AR: float, algo: int = 0) -> dict:
    m = dev(marg.astype(np.float32))
    B, V = marg.shape
    c = torch.from_numpy(np.ascontiguousarray(cost, dtype=np.float64)).cuda()
    parent = torch.full((N_max,), -7, dtype=torch.int32, device="cuda")
    token = torch.full((N_max,), -7, dtype=torch.int32, device="cuda")
    depth = torch.full((N_max,), -7, dtype=torch.int32, device="cuda")
    rho = torch.full((N_max,), -7.0, dtype=torch.float32, device="cuda")
    n_out = torch.zeros(1, dtype=torch.int32, device="cuda")
    ahat = torch.zeros(1, dtype=torch.float32, device="cuda")
    s_best = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_build_workspace(B, V, N_max))
    if algo:
        btv.btv_tree_build_tuned(m, N_max, algo, parent, token, depth, rho, n_out, ahat, ws, cost=c, L_AR=L_AR, s_best=s_best)
    else:
        btv.btv_tree_build_adaptive(m, N_max, c, L_AR, parent, token, depth, rho, n_out, ahat, s_best, ws)
    torch.cuda.synchronize()
    n = int(n_out.item())
    status = int(btv.btv_workspace_status(ws))
    return {"n": n, "parent": parent.cpu().numpy()[:n], "token": token.cpu().numpy()[:n],
            "depth": depth.cpu().numpy()[:n], "rho": rho.cpu().numpy()[:n], "ahat": float(ahat.item()),
            "s_best": float(s_best.item()), "status": status, "raw_parent": parent.cpu().numpy()}


def run_accept_greedy(logits_store: np.ndarray, bf16_bits: bool, parent, token) -> dict:
    x = dev(logits_store, bf16_bits)
    M = len(parent)
    par, tok = dev(np.asarray(parent, dtype=np.int32)), dev(np.asarray(token, dtype=np.int32))
    path = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    n_acc = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    am = torch.full((M + 1,), -7, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_workspace(M, x.shape[1], False))
    btv.btv_tree_accept_greedy(x, par, tok, path, n_acc, bonus, am, ws)
    torch.cuda.synchronize()
    n = int(n_acc.item())
    return {"n_acc": n, "path": path.cpu().numpy()[:n], "bonus": int(bonus.item()), "argmax": am.cpu().numpy()}


def run_accept_stochastic(logits_store: np.ndarray, bf16_bits: bool, marg, parent, token, uniforms) -> dict:
    x = dev(logits_store, bf16_bits)
    M = len(parent)
    par, tok = dev(np.asarray(parent, dtype=np.int32)), dev(np.asarray(token, dtype=np.int32))
    m, u = dev(marg.astype(np.float32)), dev(np.asarray(uniforms, dtype=np.float32))
    path = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    n_acc = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_workspace(M, x.shape[1], True))
    btv.btv_tree_accept_stochastic(x, m, par, tok, u, path, n_acc, bonus, ws)
    torch.cuda.synchronize()
    n = int(n_acc.item())
    return {"n_acc": n, "path": path.cpu().numpy()[:n], "bonus": int(bonus.item())}


def run_accept_greedy_lm_head(hidden_bits: np.ndarray, W_bits, parent, token) -> dict:
    """W_bits: numpy uint16 [V, h] or a device bf16 tensor (so that a large matrix is uploaded once)."""
    x = dev(hidden_bits, True)
    W = W_bits if isinstance(W_bits, torch.Tensor) else dev(W_bits, True)
    M = len(parent)
    par, tok = dev(np.asarray(parent, dtype=np.int32)), dev(np.asarray(token, dtype=np.int32))
    path = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    n_acc = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    am = torch.full((M + 1,), -7, dtype=torch.int32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_accept_lm_head_workspace(M, W.shape[0]))
    btv.btv_tree_accept_greedy_lm_head(x, W, par, tok, path, n_acc, bonus, am, ws)
    torch.cuda.synchronize()
    n = int(n_acc.item())
    return {"n_acc": n, "path": path.cpu().numpy()[:n], "bonus": int(bonus.item()), "argmax": am.cpu().numpy()}


def run_tree_build_beam(marg: np.ndarray, width: int, depth_max: int) -> dict:
    m = dev(marg.astype(np.float32))
    B, V = marg.shape
    cap = width * depth_max
    parent = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
    token = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
    depth = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
    rho = torch.full((cap,), -7.0, dtype=torch.float32, device="cuda")
    n_out = torch.zeros(1, dtype=torch.int32, device="cuda")
    ahat = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = btv.alloc_workspace(btv.btv_tree_build_workspace(depth_max, V, width))
    btv.btv_tree_build_beam(m, width, depth_max, parent, token, depth, rho, n_out, ahat, ws)
    torch.cuda.synchronize()
    n = int(n_out.item())
    return {"n": n, "parent": parent.cpu().numpy()[:n], "token": token.cpu().numpy()[:n],
            "depth": depth.cpu().numpy()[:n], "rho": rho.cpu().numpy()[:n], "ahat": float(ahat.item()),
            "status": int(btv.btv_workspace_status(ws))}
