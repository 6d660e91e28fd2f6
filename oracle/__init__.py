"""Python face of the CPU oracle (ctypes over oracle/bastion_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The HIP package never imports this module, and this module never
imports the HIP package.  Arrays in, arrays out; all arithmetic lives in the C file
(and in bruteforce.py for the exhaustive pins).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bastion_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over (node, head) pairs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.orc_tree_build.restype = C.c_int
        _lib.orc_tree_attn.restype = C.c_int
        _lib.orc_tree_attn_fp8kv.restype = C.c_int
        _lib.orc_fp8_e4m3_decode.restype = None
        _lib.orc_accept_greedy.restype = C.c_int
        _lib.orc_accept_stochastic.restype = C.c_int
        _lib.orc_num_threads.restype = C.c_int
        _lib.orc_ancestor_mask.restype = C.c_int
        _lib.orc_tree_build_adaptive.restype = C.c_int
        _lib.orc_tree_build_beam.restype = C.c_int
        _lib.orc_verify_cost.restype = None
        _lib.orc_kv_commit.restype = C.c_longlong
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def num_threads() -> int:
    return int(_load().orc_num_threads())


def rank_tokens(marg: np.ndarray) -> np.ndarray:
    marg = np.ascontiguousarray(marg, dtype=np.float32)
    B, V = marg.shape
    order = np.empty((B, V), dtype=np.int32)
    _load().orc_rank_tokens(_p(marg, C.c_float), B, V, _p(order, C.c_int32))
    return order


def tree_build(marg: np.ndarray, N: int) -> dict:
    """Best-first tree of N draft nodes from marginals [B, V] (Sec. 3.3, Prop. 3.3, Alg. 1 frontier rule)."""
    marg = np.ascontiguousarray(marg, dtype=np.float32)
    B, V = marg.shape
    parent = np.empty(max(N, 1), dtype=np.int32)
    token = np.empty_like(parent)
    depth = np.empty_like(parent)
    rank = np.empty_like(parent)
    rho = np.empty(max(N, 1), dtype=np.float32)
    ahat = C.c_double(0.0)
    n = _load().orc_tree_build(_p(marg, C.c_float), B, V, N, _p(parent, C.c_int32), _p(token, C.c_int32),
                               _p(depth, C.c_int32), _p(rho, C.c_float), _p(rank, C.c_int32), C.byref(ahat))
    if n < 0:
        raise ValueError("orc_tree_build: bad arguments")
    return {"n": n, "parent": parent[:n], "token": token[:n], "depth": depth[:n], "rank": rank[:n],
            "rho": rho[:n], "ahat": ahat.value}


def tree_build_beam(marg: np.ndarray, width: int, depth: int) -> dict:
    """Beam-search tree, width x depth below the root (Sec. 4.3's comparison topology; width 1 = greedy chain)."""
    marg = np.ascontiguousarray(marg, dtype=np.float32)
    B, V = marg.shape
    cap = max(width * depth, 1)
    parent = np.empty(cap, dtype=np.int32)
    token = np.empty_like(parent); dep = np.empty_like(parent); rank = np.empty_like(parent)
    rho = np.empty(cap, dtype=np.float32)
    ahat = C.c_double(0.0)
    n = _load().orc_tree_build_beam(_p(marg, C.c_float), B, V, int(width), int(depth), _p(parent, C.c_int32),
                                    _p(token, C.c_int32), _p(dep, C.c_int32), _p(rho, C.c_float), _p(rank, C.c_int32),
                                    C.byref(ahat))
    if n < 0:
        raise ValueError("orc_tree_build_beam: bad arguments")
    return {"n": n, "parent": parent[:n], "token": token[:n], "depth": dep[:n], "rank": rank[:n], "rho": rho[:n],
            "ahat": ahat.value}


def tree_build_adaptive(marg: np.ndarray, N_max: int, cost, L_AR: float) -> dict:
    """Algorithm 1 with its early stop: cost[N-1] = estimated cycle latency at budget N (Sec. 3.4, Eq. 6)."""
    marg = np.ascontiguousarray(marg, dtype=np.float32)
    cost = np.ascontiguousarray(cost, dtype=np.float64)
    assert len(cost) >= N_max
    B, V = marg.shape
    parent = np.empty(max(N_max, 1), dtype=np.int32)
    token = np.empty_like(parent); depth = np.empty_like(parent); rank = np.empty_like(parent)
    rho = np.empty(max(N_max, 1), dtype=np.float32)
    ahat, sbest, margin = C.c_double(0.0), C.c_double(0.0), C.c_double(0.0)
    n = _load().orc_tree_build_adaptive(_p(marg, C.c_float), B, V, N_max, _p(cost, C.c_double), C.c_double(L_AR),
                                        _p(parent, C.c_int32), _p(token, C.c_int32), _p(depth, C.c_int32),
                                        _p(rho, C.c_float), _p(rank, C.c_int32), C.byref(ahat), C.byref(sbest),
                                        C.byref(margin))
    if n < 0:
        raise ValueError("orc_tree_build_adaptive: bad arguments")
    return {"n": n, "parent": parent[:n], "token": token[:n], "depth": depth[:n], "rank": rank[:n], "rho": rho[:n],
            "ahat": ahat.value, "s_best": sbest.value, "margin": margin.value}


def verify_cost(s, c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops, bandwidth, calib_scale=1.0,
                calib_offset=0.0) -> dict:
    """App. E cost model: FLOPs, bytes, roofline time and calibrated latency of one verifier pass."""
    out = (C.c_double * 4)()
    _load().orc_verify_cost(*[C.c_double(float(x)) for x in (s, c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops,
                                                              bandwidth, calib_scale, calib_offset)], out)
    return {"flops": out[0], "bytes": out[1], "roofline_s": out[2], "latency_s": out[3]}


def calib_fit(pred, obs) -> tuple[float, float]:
    """Sec. 5.2 static calibration: least-squares line obs ~ scale * pred + offset."""
    pred = np.ascontiguousarray(pred, dtype=np.float64)
    obs = np.ascontiguousarray(obs, dtype=np.float64)
    assert pred.shape == obs.shape and pred.ndim == 1
    a, b = C.c_double(), C.c_double()
    rc = _load().orc_calib_fit(_p(pred, C.c_double), _p(obs, C.c_double), len(pred), C.byref(a), C.byref(b))
    if rc != 0:
        raise ValueError("calibration fit is undetermined")
    return a.value, b.value


def calib_ema(c: float, alpha: float, obs: float, pred: float) -> float:
    """Sec. 5.2 online calibration: c <- (1 - alpha) c + alpha obs / pred."""
    f = _load().orc_calib_ema
    f.restype = C.c_double
    return f(C.c_double(c), C.c_double(alpha), C.c_double(obs), C.c_double(pred))


def cost_curve(N_max, c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops, bandwidth, calib_scale=1.0, calib_offset=0.0,
               c_ema=1.0, t_other=0.0) -> np.ndarray:
    """C(N), N = 1..N_max, for the budget controller (Eq. 6): T_other + c_ema * calibrated T_verify(N + 1 tokens)."""
    out = np.zeros(N_max, dtype=np.float64)
    _load().orc_cost_curve(int(N_max), *[C.c_double(float(x)) for x in (c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops,
                                                                         bandwidth, calib_scale, calib_offset, c_ema,
                                                                         t_other)], _p(out, C.c_double))
    return out


def tree_attn(Qf, Kf, Vf, parent, L: int, scale: float | None = None, pairs=None, block_table=None, page: int = 16,
              nthreads: int = 0) -> np.ndarray:
    """Tree-masked attention by its definition (App. C), fp64.

    Qf [M,Hq,D], Kf/Vf [rows,Hkv,D] fp32 (exact stored values); rows = L+M when contiguous, or the flattened
    page pool when block_table (1-D, for this sequence) is given.  Returns [M,Hq,D] or [npairs,D] fp64.
    """
    Qf = np.ascontiguousarray(Qf, dtype=np.float32)
    Kf = np.ascontiguousarray(Kf, dtype=np.float32)
    Vf = np.ascontiguousarray(Vf, dtype=np.float32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    M, Hq, D = Qf.shape
    if Kf.ndim == 4:   # [num_blocks, page, Hkv, D]
        Kf = Kf.reshape(-1, Kf.shape[2], Kf.shape[3])
        Vf = Vf.reshape(-1, Vf.shape[2], Vf.shape[3])
    Hkv = Kf.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    if block_table is None:
        assert Kf.shape[0] >= L + M and Vf.shape[0] >= L + M
        bt = None
    else:
        block_table = np.ascontiguousarray(block_table, dtype=np.int32)
        assert len(block_table) * page >= L + M
        bt = _p(block_table, C.c_int32)
    if pairs is None:
        out = np.empty((M, Hq, D), dtype=np.float64)
        pp, npairs = None, 0
    else:
        pairs = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        out = np.empty((len(pairs), D), dtype=np.float64)
        pp, npairs = _p(pairs, C.c_int32), len(pairs)
    if nthreads <= 0:
        nthreads = num_threads()
    rc = _load().orc_tree_attn(_p(Qf, C.c_float), _p(Kf, C.c_float), _p(Vf, C.c_float), _p(parent, C.c_int32),
                               M, L, Hq, Hkv, D, C.c_double(scale), bt, page, pp, npairs, _p(out, C.c_double),
                               nthreads)
    if rc != 0:
        raise ValueError(f"orc_tree_attn: bad arguments ({rc})")
    return out


def fp8_e4m3_decode(codes) -> np.ndarray:
    """The numbers the 8-bit codes stand for (OCP E4M3: bias 7, subnormals, no infinities, one NaN per sign), fp32."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, dtype=np.float32)
    _load().orc_fp8_e4m3_decode(_p(codes, C.c_uint8), C.c_size_t(codes.size), _p(out, C.c_float))
    return out


def tree_attn_fp8kv(Qf, K8, V8, k_scale: float, v_scale: float, parent, L: int, scale: float | None = None, pairs=None,
                    block_table=None, page: int = 16, nthreads: int = 0) -> np.ndarray:
    """Tree-masked attention (App. C) over an FP8 KV cache: K8/V8 hold E4M3 codes (uint8, shaped like tree_attn's
    K/V) that stand for code * k_scale and code * v_scale.  Returns fp64 like tree_attn."""
    Qf = np.ascontiguousarray(Qf, dtype=np.float32)
    K8 = np.ascontiguousarray(K8, dtype=np.uint8)
    V8 = np.ascontiguousarray(V8, dtype=np.uint8)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    M, Hq, D = Qf.shape
    if K8.ndim == 4:
        K8 = K8.reshape(-1, K8.shape[2], K8.shape[3])
        V8 = V8.reshape(-1, V8.shape[2], V8.shape[3])
    assert K8.shape == V8.shape and K8.shape[2] == D
    Hkv = K8.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    if block_table is None:
        assert K8.shape[0] >= L + M
        bt = None
    else:
        block_table = np.ascontiguousarray(block_table, dtype=np.int32)
        assert len(block_table) * page >= L + M
        bt = _p(block_table, C.c_int32)
    if pairs is None:
        out = np.empty((M, Hq, D), dtype=np.float64)
        pp, npairs = None, 0
    else:
        pairs = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        out = np.empty((len(pairs), D), dtype=np.float64)
        pp, npairs = _p(pairs, C.c_int32), len(pairs)
    if nthreads <= 0:
        nthreads = num_threads()
    rc = _load().orc_tree_attn_fp8kv(_p(Qf, C.c_float), _p(K8, C.c_uint8), _p(V8, C.c_uint8), C.c_size_t(K8.size),
                                     C.c_double(k_scale), C.c_double(v_scale), _p(parent, C.c_int32), M, L, Hq, Hkv, D,
                                     C.c_double(scale), bt, page, pp, npairs, _p(out, C.c_double), nthreads)
    if rc != 0:
        raise ValueError(f"orc_tree_attn_fp8kv: bad arguments ({rc})")
    return out


def ancestor_mask(parent, words: int = 8) -> np.ndarray:
    """anc[i] bitset of node i and its ancestors (App. C verification mask), uint32 [M, words]."""
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    anc = np.empty((len(parent), words), dtype=np.uint32)
    rc = _load().orc_ancestor_mask(_p(parent, C.c_int32), len(parent), words, _p(anc, C.c_uint32))
    if rc != 0:
        raise ValueError(f"orc_ancestor_mask: bad arguments ({rc})")
    return anc


def row_argmax(logits_f32: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(logits_f32, dtype=np.float32)
    t = np.empty(x.shape[0], dtype=np.int32)
    _load().orc_row_argmax(_p(x, C.c_float), x.shape[0], x.shape[1], _p(t, C.c_int32))
    return t


def accept_greedy(logits_f32, parent, token) -> dict:
    """Greedy acceptance (App. C "Acceptance"): longest path matching the target's top-1 tokens."""
    x = np.ascontiguousarray(logits_f32, dtype=np.float32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    token = np.ascontiguousarray(token, dtype=np.int32)
    M = len(parent)
    assert x.shape[0] == M + 1
    path = np.empty(max(M, 1), dtype=np.int32)
    t = np.empty(M + 1, dtype=np.int32)
    bonus = C.c_int32(0)
    n = _load().orc_accept_greedy(_p(x, C.c_float), _p(parent, C.c_int32), _p(token, C.c_int32), M, x.shape[1],
                                  _p(path, C.c_int32), C.byref(bonus), _p(t, C.c_int32))
    return {"n_acc": n, "path": path[:n].copy(), "bonus": int(bonus.value), "argmax": t}


def lm_head_argmax(hidden_f32, W_f32, nthreads: int = 0) -> dict:
    """Target tokens from hidden states (App. E LM head + App. C top-1): argmax_v of hidden @ W^T in fp64."""
    x = np.ascontiguousarray(hidden_f32, dtype=np.float32)
    w = np.ascontiguousarray(W_f32, dtype=np.float32)
    R, h = x.shape
    V = w.shape[0]
    assert w.shape[1] == h
    t = np.empty(R, dtype=np.int32)
    margin = np.empty(R, dtype=np.float64)
    _load().orc_lm_head_argmax(_p(x, C.c_float), _p(w, C.c_float), R, h, V, _p(t, C.c_int32), _p(margin, C.c_double),
                               int(nthreads) if nthreads else num_threads())
    return {"argmax": t, "margin": margin}


def accept_stochastic(logits_f32, marg, parent, token, depth, uniforms) -> dict:
    """Token-level rejection walk at temperature 1 (the reading stated in the C file)."""
    x = np.ascontiguousarray(logits_f32, dtype=np.float32)
    marg = np.ascontiguousarray(marg, dtype=np.float32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    token = np.ascontiguousarray(token, dtype=np.int32)
    depth = np.ascontiguousarray(depth, dtype=np.int32)
    u = np.ascontiguousarray(uniforms, dtype=np.float32)
    M = len(parent)
    assert x.shape[0] == M + 1 and len(u) >= M + 1 and marg.shape[1] == x.shape[1]
    path = np.empty(max(M, 1), dtype=np.int32)
    bonus, used, margin, gap = C.c_int32(0), C.c_int32(0), C.c_double(0.0), C.c_double(0.0)
    n = _load().orc_accept_stochastic(_p(x, C.c_float), _p(marg, C.c_float), marg.shape[0], _p(parent, C.c_int32),
                                      _p(token, C.c_int32), _p(depth, C.c_int32), M, x.shape[1], _p(u, C.c_float),
                                      _p(path, C.c_int32), C.byref(bonus), C.byref(used), C.byref(margin),
                                      C.byref(gap))
    return {"n_acc": n, "path": path[:n].copy(), "bonus": int(bonus.value), "n_uniforms": int(used.value),
            "margin": float(margin.value), "bonus_gap": float(gap.value)}


def kv_commit(cache: np.ndarray, L: int, M: int, path, block_table=None, page: int = 16) -> int:
    """Reorder one cache (K or V) in place: position L+j takes the row of position L+path[j] (App. C "Acceptance").

    cache [layers, rows, ...] (contiguous) or [layers, num_blocks, page, ...] with a block table; any dtype.
    Returns the new sequence length L + len(path)."""
    assert cache.flags["C_CONTIGUOUS"]
    path = np.ascontiguousarray(path, dtype=np.int32)
    layers = cache.shape[0]
    layer_stride = cache.strides[0]
    row_bytes = int(np.prod(cache.shape[2:])) * cache.itemsize if block_table is None else \
        int(np.prod(cache.shape[3:])) * cache.itemsize
    bt = None
    if block_table is not None:
        block_table = np.ascontiguousarray(block_table, dtype=np.int32)
        bt = _p(block_table, C.c_int32)
    rc = _load().orc_kv_commit(cache.ctypes.data_as(C.POINTER(C.c_ubyte)), layers, C.c_longlong(layer_stride), L, M,
                               row_bytes, _p(path, C.c_int32), len(path), bt, page)
    if rc < 0:
        raise ValueError("orc_kv_commit: bad arguments")
    return int(rc)
