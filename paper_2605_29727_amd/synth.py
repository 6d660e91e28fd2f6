"""Seeded synthetic inputs for the tree-verify path (numpy; torch only for the library FP8 rounding).

This module produces DATA: random tensors, tree shapes, block tables and the
named workload configurations.  It holds none of the method's arithmetic (no
path scores, no attention, no acceptance rule) and is the only module that both
the CPU oracle's tests and the HIP path's tests draw from.

The generator is counter based (splitmix64 finaliser over seed/stream/counter)
so that every element is a pure function of (seed, tag, index): inputs are
bit-reproducible without depending on a library's RNG stream.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field

import numpy as np

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function, vectorised over uint64 (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
        z = z ^ (z >> _U64(31))
    return z


def _stream_base(seed: int, tag: str) -> np.uint64:
    h = zlib.crc32(tag.encode()) & 0xFFFFFFFF
    base = (int(seed) * 0x9E3779B97F4A7C15 + h * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & 0xFFFFFFFFFFFFFFFF
    return _mix(np.array([base], dtype=_U64))[0]


def raw_u64(seed: int, tag: str, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit words of stream (seed, tag), starting at counter `offset`."""
    base = _stream_base(seed, tag)
    with np.errstate(over="ignore"):
        ctr = (np.arange(offset, offset + n, dtype=_U64) + _U64(1)) * _GOLDEN + base
    return _mix(ctr)


def uniform(seed: int, tag: str, shape) -> np.ndarray:
    """float64 uniforms in [0, 1) with 53 random bits."""
    n = int(np.prod(shape))
    return ((raw_u64(seed, tag, n) >> _U64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)).reshape(shape)


def normal(seed: int, tag: str, shape, scale: float = 1.0) -> np.ndarray:
    """float64 N(0, scale^2) by Box-Muller on two counter-based uniforms per value."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float64)
    step = 1 << 22  # bound temporaries for the large KV tensors
    for s in range(0, n, step):
        m = min(step, n - s)
        w = raw_u64(seed, tag, 2 * m, offset=2 * s)
        u1 = ((w[0::2] >> _U64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)  # (0, 1]
        u2 = (w[1::2] >> _U64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        out[s:s + m] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    if scale != 1.0:
        out *= scale
    return out.reshape(shape)


def integers(seed: int, tag: str, shape, lo: int, hi: int) -> np.ndarray:
    """int64 uniform in [lo, hi] inclusive (modulo bias < 2^-40 for the ranges used here)."""
    n = int(np.prod(shape))
    span = _U64(hi - lo + 1)
    return ((raw_u64(seed, tag, n) % span).astype(np.int64) + lo).reshape(shape)


def permutation(seed: int, tag: str, n: int) -> np.ndarray:
    """Random permutation of range(n): argsort of n random words (stable)."""
    return np.argsort(raw_u64(seed, tag, n), kind="stable").astype(np.int64)


# ----------------------------------------------------------------------------------------------
# bf16 storage helpers (bit manipulation only)
# ----------------------------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x64: np.ndarray, dtype: str):
    """Returns (storage array, fp32 array holding exactly the stored values)."""
    x32 = x64.astype(np.float32)
    if dtype == "fp32":
        return x32, x32
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x32)
        return bits, bf16_bits_to_f32(bits)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------------------------
# tensors of the path
# ----------------------------------------------------------------------------------------------

def marginals(seed: int, B: int, V: int, sigma: float, tag: str = "marg") -> np.ndarray:
    """Draft marginals [B, V] fp32: each row is a softmax (computed in fp64) of sigma * N(0,1) logits."""
    z = normal(seed, tag, (B, V), sigma)
    z -= z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=1, keepdims=True)).astype(np.float32)


def marginals_drafter_like(seed: int, B: int, V: int, top1: float = 0.9, decay: float = 0.93, sigma: float = 3.0,
                           tag: str = "marg_dl") -> np.ndarray:
    """Draft marginals [B, V] fp32 shaped like a confident drafter whose confidence falls with the position: at
    position k one token holds top1 * decay^k, the rest is spread as softmax(sigma * N(0,1)) over the vocabulary."""
    base = marginals(seed, B, V, sigma, tag).astype(np.float64)
    hot = integers(seed, tag + "_hot", (B,), 0, V)
    out = np.empty((B, V), dtype=np.float64)
    for k in range(B):
        p = top1 * decay ** k
        row = base[k].copy()
        row[hot[k]] = 0.0
        row *= (1.0 - p) / row.sum()
        row[hot[k]] = p
        out[k] = row
    return out.astype(np.float32)


def qkv(seed: int, M: int, L: int, Hq: int, Hkv: int, D: int, dtype: str, tag: str = ""):
    """Q [M,Hq,D], K and V [L+M,Hkv,D], all N(0,1), rounded once to `dtype`.

    Returns dict with storage arrays (uint16 bits for bf16) under 'Q','K','V' and the
    exactly-equal fp32 values under 'Qf','Kf','Vf'.
    """
    out = {}
    for name, shape in (("Q", (M, Hq, D)), ("K", (L + M, Hkv, D)), ("V", (L + M, Hkv, D))):
        st, f = round_to_dtype(normal(seed, tag + name, shape), dtype)
        out[name], out[name + "f"] = st, f
    return out


def kv_fp8(seed: int, rows: int, Hkv: int, D: int, tag: str = ""):
    """K and V [rows,Hkv,D] ~ N(0,1) as an FP8 cache would hold them: one fp32 scale per tensor (largest magnitude
    / 448, the largest E4M3 number) and x / scale stored as 8-bit E4M3 codes (uint8).  The rounding is a library
    conversion (torch, round to nearest even).  Returns dict K8, V8 (uint8), k_scale, v_scale (python floats
    holding fp32 values).  Same streams as `qkv`, so the codes are the quantised form of that function's K and V."""
    import torch

    out = {}
    for name in ("K", "V"):
        x = normal(seed, tag + name, (rows, Hkv, D)).astype(np.float32)
        scale = np.float32(max(float(np.abs(x).max()), 1e-6) / 448.0)
        y = np.clip(x / scale, -448.0, 448.0).astype(np.float32)
        codes = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy().copy()
        out[name + "8"] = codes
        out[name.lower() + "_scale"] = float(scale)
    return out


def target_logits(seed: int, rows: int, V: int, sigma: float, dtype: str, tag: str = "logits"):
    st, f = round_to_dtype(normal(seed, tag, (rows, V), sigma), dtype)
    return st, f


def lm_head(seed: int, rows: int, h: int, V: int, dtype: str = "bf16", tag: str = "lmhead", base_rows: int = 8192):
    """Final hidden states [rows, h] ~ N(0,1) and LM-head weights [V, h] ~ N(0, 1/h), each rounded once to `dtype`.
    Returns (hidden storage, hidden fp32, W storage, W fp32).  Only the first `base_rows` vocabulary rows are drawn;
    block b of the rest repeats them rotated by 8 b positions along h (distinct rows of the same distribution), which
    keeps a 128k-token matrix affordable to generate."""
    hs, hf = round_to_dtype(normal(seed, tag + "_x", (rows, h)), dtype)
    nb = min(V, base_rows)
    bs, bf = round_to_dtype(normal(seed, tag + "_w", (nb, h), 1.0 / np.sqrt(h)), dtype)
    if V <= base_rows:
        return hs, hf, bs, bf
    ws = np.empty((V, h), dtype=bs.dtype)
    wf = np.empty((V, h), dtype=np.float32)
    for b, v0 in enumerate(range(0, V, base_rows)):
        v1 = min(v0 + base_rows, V)
        ws[v0:v1] = np.roll(bs[:v1 - v0], 8 * b, axis=1)
        wf[v0:v1] = np.roll(bf[:v1 - v0], 8 * b, axis=1)
    return hs, hf, ws, wf


def plant_hidden(hidden_f32: np.ndarray, W_f32: np.ndarray, parent: np.ndarray, token: np.ndarray, leaf: int,
                 boost: float = 12.0) -> np.ndarray:
    """Turn the hidden state at the parent's row of every node on the root-to-`leaf` path towards that node's
    LM-head row, so that the target's top-1 token there is the node's token (row 0 = root, row 1+i = node i)."""
    out = hidden_f32.astype(np.float64).copy()
    i = int(leaf)
    while i >= 0:
        w = W_f32[int(token[i])].astype(np.float64)
        out[int(parent[i]) + 1] += boost * w / max(float(np.sqrt((w * w).sum())), 1e-30) * np.sqrt(out.shape[1])
        i = int(parent[i])
    return out


# ----------------------------------------------------------------------------------------------
# tree shapes for property tests (parent[i] in {-1} u [0, i); -1 = child of the root)
# ----------------------------------------------------------------------------------------------

def tree_parents(seed: int, N: int, kind: str) -> np.ndarray:
    p = np.empty(N, dtype=np.int32)
    if kind == "chain":
        p[:] = np.arange(N) - 1
    elif kind == "star":
        p[:] = -1
    elif kind == "binary":          # heap-ordered binary tree under the root
        for i in range(N):
            p[i] = -1 if i < 2 else (i - 2) // 2
    elif kind == "caterpillar":     # a spine with one leaf hanging off every spine node
        for i in range(N):          # spine = even indices, leaf 2k+1 hangs off spine node 2k
            p[i] = max(i - 2, -1) if i % 2 == 0 else i - 1
    elif kind == "random":          # uniform random recursive tree
        r = raw_u64(seed, "tree_random", N)
        for i in range(N):
            p[i] = int(r[i] % _U64(i + 1)) - 1
    elif kind == "deep":            # mostly a chain with occasional branches
        r = raw_u64(seed, "tree_deep", N)
        for i in range(N):
            p[i] = i - 1 if (int(r[i] & _U64(7)) != 0 or i == 0) else int((r[i] >> _U64(8)) % _U64(i + 1)) - 1
    else:
        raise ValueError(kind)
    assert all(-1 <= int(p[i]) < i for i in range(N))
    return p


def sibling_distinct_tokens(seed: int, parent: np.ndarray, V: int) -> np.ndarray:
    """Token ids for a given tree such that siblings carry distinct tokens (needs V >= max fan-out)."""
    N = len(parent)
    tok = np.empty(N, dtype=np.int32)
    start = integers(seed, "tok_start", (N + 1,), 0, V - 1)
    nchild = {}
    for i in range(N):
        pa = int(parent[i])
        k = nchild.get(pa, 0)
        nchild[pa] = k + 1
        assert k < V
        tok[i] = (int(start[pa + 1]) + k * 7919) % V if V > 7919 else (int(start[pa + 1]) + k) % V
    return tok


def plant_path(logits_f32: np.ndarray, parent: np.ndarray, token: np.ndarray, leaf: int, boost: float = 20.0):
    """Raise the target logit of every token on the root-to-`leaf` path at its parent's row, so that a
    greedy verifier accepts exactly that path (row 0 = root, row 1+i = node i).  leaf = -1: plant nothing."""
    out = logits_f32.copy()
    i = int(leaf)
    while i >= 0:
        out[int(parent[i]) + 1, int(token[i])] += boost
        i = int(parent[i])
    return out


# ----------------------------------------------------------------------------------------------
# paged KV layout
# ----------------------------------------------------------------------------------------------

PAGE = 16


def paged_layout(seed: int, seq_lens, slack: float = 1.25):
    """Random block table for a batch of sequences with `PAGE`-token blocks.

    Returns (block_table [batch, max_blocks] int32 filled with -1 past each sequence's blocks, num_blocks).
    """
    need = [(int(s) + PAGE - 1) // PAGE for s in seq_lens]
    total = sum(need)
    num_blocks = max(1, int(np.ceil(total * slack)))
    perm = permutation(seed, "blocks", num_blocks)
    bt = np.full((len(need), max(need) if need else 1), -1, dtype=np.int32)
    o = 0
    for r, nb in enumerate(need):
        bt[r, :nb] = perm[o:o + nb]
        o += nb
    return bt, num_blocks


def scatter_to_pages(x: np.ndarray, table_row: np.ndarray, pool: np.ndarray):
    """Copy a contiguous [S, Hkv, D] tensor into pool [num_blocks, PAGE, Hkv, D] following one block-table row."""
    S = x.shape[0]
    for b in range((S + PAGE - 1) // PAGE):
        n = min(PAGE, S - b * PAGE)
        pool[int(table_row[b]), :n] = x[b * PAGE:b * PAGE + n]


# ----------------------------------------------------------------------------------------------
# named workloads (shapes, dtypes and distributions of the five benchmark configurations)
# ----------------------------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    Hq: int
    Hkv: int
    D: int
    L: int            # prefix length (per request for batch == 1)
    N: int            # draft-tree nodes
    B: int            # draft positions
    V: int            # vocabulary
    marg_sigma: float
    logit_sigma: float
    dtype: str        # attention dtype
    logit_dtype: str
    seed: int
    accept: str = "greedy"
    batch: int = 1
    extra: dict = field(default_factory=dict)


C1 = Workload("tiny_fp32", 1, 1, 64, 128, 16, 4, 64, 2.0, 1.0, "fp32", "fp32", 1)
C2 = Workload("llama3_8b_L2048_N64", 32, 8, 128, 2048, 64, 16, 128256, 3.0, 1.0, "bf16", "bf16", 2)


def c3(N: int, sharp: bool = True) -> Workload:
    return Workload(f"llama3_8b_L8192_N{N}_{'sharp' if sharp else 'flat'}", 32, 8, 128, 8192, N, 16, 128256,
                    5.0 if sharp else 1.0, 1.0, "bf16", "bf16", 3 if sharp else 4)


C3_SIZES = (16, 32, 64, 128, 256)
C4 = Workload("ragged8_paged", 32, 8, 128, 0, 0, 16, 128256, 3.0, 1.0, "bf16", "bf16", 5, batch=8,
              extra={"L_range": (1024, 16384), "N_range": (32, 128)})
C5 = Workload("llama_70b_L32768_N128", 64, 8, 128, 32768, 128, 16, 128256, 3.0, 3.0, "bf16", "fp32", 6,
              accept="stochastic")


def c4_request_shapes(seed: int = 5, batch: int = 8):
    Ls = integers(seed, "c4_L", (batch,), 1024, 16384)
    Ns = integers(seed, "c4_N", (batch,), 32, 128)
    return [int(x) for x in Ls], [int(x) for x in Ns]
