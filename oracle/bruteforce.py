"""Exhaustive definitions for tiny inputs (pure Python loops) that pin the C oracle.

TEST INFRASTRUCTURE ONLY.  Nothing here is fast and nothing here is used by the HIP path.
"""
from __future__ import annotations

import itertools

import numpy as np


def _ranked(marg: np.ndarray):
    """Per position: token ids sorted by (probability descending, id ascending)."""
    B, V = marg.shape
    return [sorted(range(V), key=lambda v, k=k: (-float(marg[k, v]), v)) for k in range(B)]


def all_prefixes(marg: np.ndarray):
    """Every prefix (x_1..x_d), 1 <= d <= B, of the full lattice with its path score (Eq. 1).

    rho is the left-to-right product in fp32 (one rounded multiply per edge, root = 1), the same
    arithmetic the tree builder is specified with.  Returns a list of (rho, depth, rank_path, tokens).
    """
    B, V = marg.shape
    order = _ranked(marg)
    out = []
    level = [(np.float32(1.0), (), ())]
    for k in range(B):
        nxt = []
        for rho, rp, toks in level:
            for r in range(V):
                tok = order[k][r]
                child = (np.float32(rho * np.float32(marg[k, tok])), rp + (r,), toks + (tok,))
                nxt.append(child)
        out.extend((float(c[0]), k + 1, c[1], c[2]) for c in nxt)
        level = nxt
    return out


def tree_build_bruteforce(marg: np.ndarray, N: int) -> dict:
    """Top-N prefixes of the full lattice under the order (rho desc, depth asc, rank path lexicographic).

    Prop. 3.3 (and step 2 of its proof): best-first expansion emits exactly these, in this order.
    """
    pref = all_prefixes(np.asarray(marg, dtype=np.float32))
    pref.sort(key=lambda p: (-p[0], p[1], p[2]))
    pref = pref[:N]
    index = {p[2]: i for i, p in enumerate(pref)}
    parent, token, depth, rho, rank = [], [], [], [], []
    for p in pref:
        rp = p[2]
        if len(rp) == 1:
            parent.append(-1)
        else:
            assert rp[:-1] in index, "top-N set is not prefix closed"
            parent.append(index[rp[:-1]])
        token.append(p[3][-1]); depth.append(p[1]); rho.append(p[0]); rank.append(rp[-1])
    return {"n": len(pref), "parent": np.array(parent, dtype=np.int32), "token": np.array(token, dtype=np.int32),
            "depth": np.array(depth, dtype=np.int32), "rho": np.array(rho, dtype=np.float32),
            "rank": np.array(rank, dtype=np.int32), "ahat": 1.0 + float(np.sum(np.array(rho, dtype=np.float64)))}


def best_surrogate_any_tree(marg: np.ndarray, N: int) -> float:
    """max over ALL prefix-closed size-N trees of sum rho (root's 1 not included): Prop. 3.3's optimum,
    by enumerating every size-N subset of the lattice and keeping the prefix-closed ones."""
    pref = all_prefixes(np.asarray(marg, dtype=np.float32))
    rho = {p[2]: p[0] for p in pref}
    keys = list(rho)
    best = -1.0
    for comb in itertools.combinations(keys, N):
        s = set(comb)
        if all(len(k) == 1 or k[:-1] in s for k in comb):
            best = max(best, sum(rho[k] for k in comb))
    return best


def accept_greedy_bruteforce(argmax_tok, parent, token) -> dict:
    """App. C "Acceptance", literally: score every root-to-node path against the target's top-1
    predictions and keep the longest one that matches everywhere."""
    M = len(parent)
    best_path = []
    for leaf in range(M):
        path = []
        i = leaf
        while i >= 0:
            path.append(i)
            i = int(parent[i])
        path.reverse()
        ok = all(int(token[c]) == int(argmax_tok[int(parent[c]) + 1]) for c in path)
        if ok and len(path) > len(best_path):
            best_path = path
    last = best_path[-1] if best_path else -1
    return {"n_acc": len(best_path), "path": np.array(best_path, dtype=np.int32), "bonus": int(argmax_tok[last + 1])}
