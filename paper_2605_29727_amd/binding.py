"""Thin ctypes binding over libbastion_tv.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/bastion_tv.h); tensors are
torch CUDA(ROCm) tensors used purely as device buffers, and the current torch stream is handed
to the library.  There is no fallback: if the shared library is missing or a call fails, a
BtvError is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbastion_tv.so")

BTV_F32, BTV_BF16 = 0, 1
BTV_MAX_NODES, BTV_MAX_DEPTH, BTV_PAGE, BTV_ANC_WORDS = 256, 16, 16, 8
BTV_OK, BTV_EINVAL, BTV_EWORKSPACE, BTV_EHIP, BTV_EDATA = 0, -1, -2, -3, -4

EXPORTS = [
    "btv_last_error", "btv_version", "btv_workspace_status", "btv_stream_read", "btv_mfma_peak", "btv_tree_build_workspace",
    "btv_tree_build",
    "btv_tree_build_adaptive", "btv_tree_build_beam", "btv_tree_build_batch_workspace", "btv_tree_build_batch",
    "btv_tree_accept_batch_workspace", "btv_tree_accept_greedy_batch", "btv_verify_cost", "btv_calib_fit_linear", "btv_calib_ema_update",
    "btv_verify_cost_curve", "btv_kv_commit", "btv_kv_commit_paged",
    "btv_tree_ancestor_mask", "btv_tree_verify_attn_workspace", "btv_tree_verify_attn",
    "btv_tree_verify_attn_paged_workspace", "btv_tree_verify_attn_paged", "btv_tree_verify_attn_fp8kv_workspace",
    "btv_tree_verify_attn_fp8kv", "btv_tree_verify_attn_paged_fp8kv_workspace", "btv_tree_verify_attn_paged_fp8kv",
    "btv_tree_accept_workspace",
    "btv_tree_accept_greedy", "btv_tree_accept_stochastic", "btv_tree_accept_lm_head_workspace",
    "btv_tree_accept_greedy_lm_head", "btv_tree_verify_attn_tuned_workspace", "btv_tree_verify_attn_tuned",
    "btv_tree_verify_attn_noalloc", "btv_tree_build_tuned", "btv_tree_accept_greedy_tuned",
]


class BtvError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libbastion_tv error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise BtvError(BTV_EHIP, f"{LIB_PATH} is not built; run __graft_entry__.build() "
                                     "(python -m paper_2605_29727_amd.build)")
        L = C.CDLL(LIB_PATH)
        L.btv_last_error.restype = C.c_char_p
        for n in ("btv_tree_build_workspace", "btv_tree_verify_attn_workspace",
                  "btv_tree_verify_attn_paged_workspace", "btv_tree_verify_attn_fp8kv_workspace",
                  "btv_tree_verify_attn_paged_fp8kv_workspace", "btv_tree_accept_workspace",
                  "btv_tree_accept_lm_head_workspace", "btv_tree_build_batch_workspace",
                  "btv_tree_accept_batch_workspace", "btv_tree_verify_attn_tuned_workspace"):
            getattr(L, n).restype = C.c_size_t
        for n in ("btv_version", "btv_workspace_status", "btv_tree_build", "btv_tree_build_beam", "btv_tree_ancestor_mask",
                  "btv_tree_verify_attn", "btv_tree_verify_attn_paged", "btv_tree_verify_attn_fp8kv",
                  "btv_tree_verify_attn_paged_fp8kv", "btv_tree_accept_greedy",
                  "btv_tree_accept_stochastic", "btv_tree_verify_attn_tuned", "btv_tree_verify_attn_noalloc",
                  "btv_tree_build_tuned", "btv_tree_accept_greedy_tuned"):
            getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int):
    if rc != BTV_OK:
        raise BtvError(rc, lib().btv_last_error().decode())


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t) -> int:
    if t.dtype == torch.float32:
        return BTV_F32
    if t.dtype == torch.bfloat16:
        return BTV_BF16
    raise BtvError(BTV_EINVAL, f"unsupported dtype {t.dtype}")


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """A zero-initialised device buffer of at least nbytes (torch allocations are 256-byte aligned)."""
    return torch.zeros(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def btv_version() -> int:
    return lib().btv_version()


def btv_workspace_status(ws) -> int:
    return lib().btv_workspace_status(_ptr(ws), _stream())


# ---------------------------------------------------------------------------------------------

def btv_tree_build_workspace(B: int, V: int, N: int) -> int:
    return int(lib().btv_tree_build_workspace(B, V, N))


def btv_tree_build(marginals, N: int, parent, token, depth, rho, n_out, ahat, ws) -> None:
    B, V = marginals.shape
    assert marginals.dtype == torch.float32
    _check(lib().btv_tree_build(_ptr(marginals), B, V, N, _ptr(parent), _ptr(token), _ptr(depth), _ptr(rho),
                                _ptr(n_out), _ptr(ahat), _ptr(ws), C.c_size_t(ws.numel() if ws is not None else 0),
                                _stream()))


def btv_tree_build_adaptive(marginals, N_max: int, cost, L_AR: float, parent, token, depth, rho, n_out, ahat, s_best, ws) -> None:
    B, V = marginals.shape
    assert marginals.dtype == torch.float32 and cost.dtype == torch.float64 and cost.numel() >= N_max
    _check(lib().btv_tree_build_adaptive(_ptr(marginals), B, V, N_max, _ptr(cost), C.c_double(L_AR), _ptr(parent),
                                         _ptr(token), _ptr(depth), _ptr(rho), _ptr(n_out), _ptr(ahat), _ptr(s_best),
                                         _ptr(ws), C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_build_tuned(marginals, N: int, algo: int, parent, token, depth, rho, n_out, ahat, ws, cost=None, L_AR: float = 0.0,
                         s_best=None) -> None:
    """btv_tree_build (cost None) or btv_tree_build_adaptive with the expansion chosen by the caller:
    algo 0 = the library's choice, 1 = one-wavefront best-first loop, 2 = level-synchronous."""
    B, V = marginals.shape
    assert marginals.dtype == torch.float32 and marginals.is_contiguous()
    assert cost is None or (cost.dtype == torch.float64 and cost.numel() >= N)
    _check(lib().btv_tree_build_tuned(_ptr(marginals), B, V, N, _ptr(cost), C.c_double(L_AR), int(algo), _ptr(parent),
                                      _ptr(token), _ptr(depth), _ptr(rho), _ptr(n_out), _ptr(ahat), _ptr(s_best),
                                      _ptr(ws), C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_stream_read(src, sink) -> None:
    """Measurement aid: one streaming read of `src` (any contiguous tensor) by all CUs."""
    _check(lib().btv_stream_read(_ptr(src), C.c_size_t(src.numel() * src.element_size()), _ptr(sink),
                                 C.c_size_t(sink.numel() * sink.element_size()), _stream()))


def btv_mfma_peak(workgroups: int, iters: int, sink) -> float:
    """Measurement aid: a register-resident bf16 matrix-core loop; returns the floating-point operations launched."""
    fl = C.c_double(0.0)
    _check(lib().btv_mfma_peak(workgroups, iters, _ptr(sink), C.c_size_t(sink.numel() * sink.element_size()), C.byref(fl),
                               _stream()))
    return fl.value


def btv_tree_build_batch_workspace(batch: int, B: int, V: int, N_max: int) -> int:
    return int(lib().btv_tree_build_batch_workspace(batch, B, V, N_max))


def btv_tree_build_batch(marginals, n_nodes, q_offset, N_max: int, parent, token, depth, rho, n_out, ahat, ws) -> None:
    batch, B, V = marginals.shape
    _check(lib().btv_tree_build_batch(_ptr(marginals), batch, B, V, _ptr(n_nodes), _ptr(q_offset), int(N_max), _ptr(parent),
                                      _ptr(token), _ptr(depth), _ptr(rho), _ptr(n_out), _ptr(ahat), _ptr(ws),
                                      C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_accept_batch_workspace(batch: int, total_M: int, V: int) -> int:
    return int(lib().btv_tree_accept_batch_workspace(batch, total_M, V))


def btv_tree_accept_greedy_batch(logits, parent, token, q_offset, M_max: int, path, n_acc, bonus, argmax_out, ws) -> None:
    rows, V = logits.shape
    batch = q_offset.numel() - 1
    _check(lib().btv_tree_accept_greedy_batch(_ptr(logits), _dtype_code(logits), _ptr(parent), _ptr(token), _ptr(q_offset),
                                              batch, rows - batch, int(M_max), V, _ptr(path), _ptr(n_acc), _ptr(bonus),
                                              _ptr(argmax_out), _ptr(ws), C.c_size_t(ws.numel() if ws is not None else 0),
                                              _stream()))


def btv_tree_build_beam(marginals, width: int, depth_max: int, parent, token, depth, rho, n_out, ahat, ws) -> None:
    B, V = marginals.shape
    _check(lib().btv_tree_build_beam(_ptr(marginals), B, V, int(width), int(depth_max), _ptr(parent), _ptr(token),
                                     _ptr(depth), _ptr(rho), _ptr(n_out), _ptr(ahat), _ptr(ws),
                                     C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_verify_cost(s, c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops, bandwidth, calib_scale=1.0,
                    calib_offset=0.0) -> dict:
    """Host-side cost model (no GPU work): FLOPs, bytes, roofline time and calibrated latency of a verifier pass."""
    out = (C.c_double * 4)()
    _check(lib().btv_verify_cost(*[C.c_double(float(x)) for x in (s, c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops,
                                                                  bandwidth, calib_scale, calib_offset)], out))
    return {"flops": out[0], "bytes": out[1], "roofline_s": out[2], "latency_s": out[3]}


def btv_calib_fit_linear(pred, obs) -> tuple:
    """Host-side static calibration: (calib_scale, calib_offset) of the least-squares line obs ~ scale * pred + offset."""
    n = len(pred)
    assert len(obs) == n
    p = (C.c_double * n)(*[float(x) for x in pred])
    o = (C.c_double * n)(*[float(x) for x in obs])
    a, b = C.c_double(), C.c_double()
    _check(lib().btv_calib_fit_linear(p, o, n, C.byref(a), C.byref(b)))
    return a.value, b.value


def btv_calib_ema_update(c: float, alpha: float, obs: float, pred: float) -> float:
    """Host-side online calibration: returns (1 - alpha) c + alpha obs / pred."""
    cc = C.c_double(float(c))
    _check(lib().btv_calib_ema_update(C.byref(cc), C.c_double(float(alpha)), C.c_double(float(obs)),
                                      C.c_double(float(pred))))
    return cc.value


def btv_verify_cost_curve(N_max, c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops, bandwidth, calib_scale=1.0,
                          calib_offset=0.0, c_ema=1.0, t_other=0.0) -> list:
    """Host-side cost curve C(N), N = 1..N_max, for btv_tree_build_adaptive (a list of floats)."""
    out = (C.c_double * max(int(N_max), 1))()
    _check(lib().btv_verify_cost_curve(int(N_max), *[C.c_double(float(x)) for x in (
        c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops, bandwidth, calib_scale, calib_offset, c_ema, t_other)], out))
    return [out[i] for i in range(int(N_max))]


def btv_tree_ancestor_mask(parent, anc, ws) -> None:
    _check(lib().btv_tree_ancestor_mask(_ptr(parent), parent.numel(), _ptr(anc), _ptr(ws),
                                        C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_verify_attn_workspace(M, L, Hq, Hkv, D, dtype_code) -> int:
    return int(lib().btv_tree_verify_attn_workspace(M, L, Hq, Hkv, D, dtype_code))


def btv_tree_verify_attn(Q, K, V, parent, L: int, O, ws, scale: float = 0.0) -> None:
    M, Hq, D = Q.shape
    Hkv = K.shape[1]
    assert K.shape[0] >= L + M and V.shape == K.shape and O.shape == Q.shape
    _check(lib().btv_tree_verify_attn(_ptr(Q), _ptr(K), _ptr(V), _ptr(parent), M, L, Hq, Hkv, D, _dtype_code(Q),
                                      C.c_float(scale), _ptr(O), _ptr(ws),
                                      C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_verify_attn_noalloc(Q, K, V, parent, L: int, O, status=None, scale: float = 0.0) -> None:
    """btv_tree_verify_attn without a workspace: the library's built-in scratch array is used."""
    M, Hq, D = Q.shape
    Hkv = K.shape[1]
    assert K.shape[0] >= L + M and V.shape == K.shape and O.shape == Q.shape
    _check(lib().btv_tree_verify_attn_noalloc(_ptr(Q), _ptr(K), _ptr(V), _ptr(parent), M, L, Hq, Hkv, D, _dtype_code(Q),
                                              C.c_float(scale), _ptr(O), _ptr(status), _stream()))


def btv_tree_verify_attn_tuned_workspace(M, L, Hq, Hkv, D, kv_fp8: bool, nsplit: int, shape: int) -> int:
    return int(lib().btv_tree_verify_attn_tuned_workspace(M, L, Hq, Hkv, D, 1 if kv_fp8 else 0, int(nsplit), int(shape)))


def btv_tree_verify_attn_tuned(Q, K, V, parent, L: int, O, ws, scale: float = 0.0, nsplit: int = 0, shape: int = 0,
                               k_scale: float = 1.0, v_scale: float = 1.0) -> None:
    """K, V bf16, or one-byte E4M3 codes (then k_scale, v_scale apply)."""
    M, Hq, D = Q.shape
    Hkv = K.shape[1]
    kv_fp8 = K.element_size() == 1
    assert K.shape[0] >= L + M and V.shape == K.shape and O.shape == Q.shape and Q.dtype == torch.bfloat16
    _check(lib().btv_tree_verify_attn_tuned(_ptr(Q), _ptr(K), _ptr(V), 1 if kv_fp8 else 0, C.c_float(k_scale),
                                            C.c_float(v_scale), _ptr(parent), M, L, Hq, Hkv, D, C.c_float(scale),
                                            int(nsplit), int(shape), _ptr(O), _ptr(ws),
                                            C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_verify_attn_paged_workspace(batch, M_max, L_max, Hq, Hkv, D) -> int:
    return int(lib().btv_tree_verify_attn_paged_workspace(batch, M_max, L_max, Hq, Hkv, D))


def btv_tree_verify_attn_paged(Q, Kpool, Vpool, block_table, q_offset, prefix_len, parent, M_max: int, L_max: int,
                               O, ws, scale: float = 0.0) -> None:
    total_M, Hq, D = Q.shape
    num_blocks, page, Hkv, _ = Kpool.shape
    assert page == BTV_PAGE and Q.dtype == torch.bfloat16
    batch, max_blocks = block_table.shape
    _check(lib().btv_tree_verify_attn_paged(_ptr(Q), _ptr(Kpool), _ptr(Vpool), num_blocks, _ptr(block_table),
                                            max_blocks, _ptr(q_offset), _ptr(prefix_len), _ptr(parent), batch,
                                            total_M, M_max, L_max, Hq, Hkv, D, C.c_float(scale), _ptr(O), _ptr(ws),
                                            C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_verify_attn_fp8kv_workspace(M, L, Hq, Hkv, D) -> int:
    return int(lib().btv_tree_verify_attn_fp8kv_workspace(M, L, Hq, Hkv, D))


def btv_tree_verify_attn_fp8kv(Q, K8, V8, k_scale: float, v_scale: float, parent, L: int, O, ws,
                               scale: float = 0.0) -> None:
    M, Hq, D = Q.shape
    Hkv = K8.shape[1]
    assert K8.shape[0] >= L + M and V8.shape == K8.shape and O.shape == Q.shape
    assert Q.dtype == torch.bfloat16 and K8.element_size() == 1 and V8.element_size() == 1
    _check(lib().btv_tree_verify_attn_fp8kv(_ptr(Q), _ptr(K8), _ptr(V8), C.c_float(k_scale), C.c_float(v_scale),
                                            _ptr(parent), M, L, Hq, Hkv, D, C.c_float(scale), _ptr(O), _ptr(ws),
                                            C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_verify_attn_paged_fp8kv_workspace(batch, M_max, L_max, Hq, Hkv, D) -> int:
    return int(lib().btv_tree_verify_attn_paged_fp8kv_workspace(batch, M_max, L_max, Hq, Hkv, D))


def btv_tree_verify_attn_paged_fp8kv(Q, K8pool, V8pool, k_scale: float, v_scale: float, block_table, q_offset,
                                     prefix_len, parent, M_max: int, L_max: int, O, ws, scale: float = 0.0) -> None:
    total_M, Hq, D = Q.shape
    num_blocks, page, Hkv, _ = K8pool.shape
    assert page == BTV_PAGE and Q.dtype == torch.bfloat16 and K8pool.element_size() == 1 and V8pool.element_size() == 1
    batch, max_blocks = block_table.shape
    _check(lib().btv_tree_verify_attn_paged_fp8kv(_ptr(Q), _ptr(K8pool), _ptr(V8pool), C.c_float(k_scale),
                                                  C.c_float(v_scale), num_blocks, _ptr(block_table), max_blocks,
                                                  _ptr(q_offset), _ptr(prefix_len), _ptr(parent), batch, total_M, M_max,
                                                  L_max, Hq, Hkv, D, C.c_float(scale), _ptr(O), _ptr(ws),
                                                  C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_accept_workspace(M: int, V: int, stochastic: bool) -> int:
    return int(lib().btv_tree_accept_workspace(M, V, 1 if stochastic else 0))


def btv_tree_accept_greedy_tuned(logits, parent, token, path, n_acc, bonus, argmax_out, ws, wait_ticks) -> None:
    rows, V = logits.shape
    _check(lib().btv_tree_accept_greedy_tuned(_ptr(logits), _dtype_code(logits), _ptr(parent), _ptr(token), rows - 1, V,
                                              _ptr(path), _ptr(n_acc), _ptr(bonus), _ptr(argmax_out), _ptr(ws),
                                              C.c_size_t(ws.numel() if ws is not None else 0), _stream(),
                                              C.c_longlong(int(wait_ticks))))


def btv_tree_accept_greedy(logits, parent, token, path, n_acc, bonus, argmax_out, ws) -> None:
    rows, V = logits.shape
    _check(lib().btv_tree_accept_greedy(_ptr(logits), _dtype_code(logits), _ptr(parent), _ptr(token), rows - 1, V,
                                        _ptr(path), _ptr(n_acc), _ptr(bonus), _ptr(argmax_out), _ptr(ws),
                                        C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_accept_lm_head_workspace(M: int, V: int) -> int:
    return int(lib().btv_tree_accept_lm_head_workspace(M, V))


def btv_tree_accept_greedy_lm_head(hidden, W, parent, token, path, n_acc, bonus, argmax_out, ws) -> None:
    rows, h = hidden.shape
    V = W.shape[0]
    assert W.shape[1] == h and _dtype_code(hidden) == BTV_BF16 and _dtype_code(W) == BTV_BF16
    _check(lib().btv_tree_accept_greedy_lm_head(_ptr(hidden), _ptr(W), h, _ptr(parent), _ptr(token), rows - 1, V,
                                                _ptr(path), _ptr(n_acc), _ptr(bonus), _ptr(argmax_out), _ptr(ws),
                                                C.c_size_t(ws.numel() if ws is not None else 0), _stream()))


def btv_tree_accept_stochastic(logits, marginals, parent, token, uniforms, path, n_acc, bonus, ws) -> None:
    rows, V = logits.shape
    B = marginals.shape[0]
    assert marginals.shape[1] == V and uniforms.numel() >= rows
    _check(lib().btv_tree_accept_stochastic(_ptr(logits), _dtype_code(logits), _ptr(marginals), B, _ptr(parent),
                                            _ptr(token), rows - 1, V, _ptr(uniforms), _ptr(path), _ptr(n_acc),
                                            _ptr(bonus), _ptr(ws), C.c_size_t(ws.numel() if ws is not None else 0),
                                            _stream()))


def btv_kv_commit(K, V, L: int, M: int, path, n_acc, new_len=None) -> None:
    """K, V [layers, rows >= L+M, ...] contiguous tensors of one dtype; reordered in place."""
    assert K.shape == V.shape and K.is_contiguous() and V.is_contiguous() and K.dim() >= 3
    layers = K.shape[0]
    row_bytes = K[0, 0].numel() * K.element_size()
    _check(lib().btv_kv_commit(_ptr(K), _ptr(V), layers, C.c_longlong(K.stride(0) * K.element_size()), L, M, row_bytes,
                               _ptr(path), _ptr(n_acc), _ptr(new_len), _stream()))


def btv_kv_commit_paged(Kpool, Vpool, block_table, prefix_len, path, n_acc, new_len=None, ws=None, q_offset=None,
                        M_max: int = 0) -> None:
    """Kpool, Vpool [layers, num_blocks, PAGE, ...]; block_table [batch, max_blocks]; path [batch, M_max], or with
    q_offset [batch + 1] the ragged [total_M] layout of the batch acceptance (then M_max must be given)."""
    assert Kpool.shape == Vpool.shape and Kpool.is_contiguous() and Vpool.is_contiguous() and Kpool.dim() >= 4
    layers, num_blocks = Kpool.shape[0], Kpool.shape[1]
    row_bytes = Kpool[0, 0, 0].numel() * Kpool.element_size()
    batch, max_blocks = block_table.shape
    if q_offset is None:
        total_M, M_max = 0, path.shape[1]
    else:
        total_M = path.numel()
        assert M_max >= 1
    _check(lib().btv_kv_commit_paged(_ptr(Kpool), _ptr(Vpool), layers, C.c_longlong(Kpool.stride(0) * Kpool.element_size()),
                                     num_blocks, _ptr(block_table), max_blocks, _ptr(prefix_len), _ptr(path), _ptr(q_offset),
                                     int(total_M), _ptr(n_acc), batch, int(M_max), row_bytes, _ptr(new_len), _ptr(ws),
                                     _stream()))
