"""Seeded synthetic inputs shaped like the benchmark configurations.

This module only *makes inputs* (logits, candidate ids, token trees).  It holds
none of the verification arithmetic: both the HIP path and the CPU oracle are
fed from here and neither is imported here.

bfloat16 tensors are produced as ``uint16`` arrays of bit patterns (numpy has
no bfloat16); ``as_torch`` reinterprets them as ``torch.bfloat16``.
"""
from __future__ import annotations

import numpy as np

__all__ = ["to_bf16_bits", "bf16_bits_to_f32", "as_torch", "chain_inputs", "tree_inputs", "CONFIGS",
           "config_inputs"]


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round to nearest even (NaN kept quiet)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = x.view(np.uint32)
    bias = ((w >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((w + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r[nan] = np.uint16(0x7FC0)
    return r


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_torch(a: np.ndarray, device="cuda"):
    """numpy (float32 | uint16 bf16 bits | int32) -> torch tensor on ``device``."""
    import torch

    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def _finish(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return to_bf16_bits(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(dtype)


def _target_rows(rng, n: int, V: int, kind: str) -> np.ndarray:
    """n target-logit rows (float32) of one of the three recipes."""
    if kind == "gauss2":      # iid N(0, 2^2)
        return rng.standard_normal((n, V), dtype=np.float32) * np.float32(2.0)
    if kind == "peaked":      # N(0, 3^2) plus 20 random entries per row boosted by +8
        z = rng.standard_normal((n, V), dtype=np.float32) * np.float32(3.0)
        npk = min(20, V)
        for r in range(n):
            idx = rng.choice(V, size=npk, replace=False)
            z[r, idx] += np.float32(8.0)
        return z
    if kind == "zipf":        # -1.1 ln(rank) + N(0,1), random rank permutation per row
        z = rng.standard_normal((n, V), dtype=np.float32)
        base = (-1.1 * np.log(np.arange(1, V + 1, dtype=np.float64))).astype(np.float32)
        for r in range(n):
            z[r] += base[rng.permutation(V)]
        return z
    raise ValueError(kind)


def _sample_from_logits(rng, z: np.ndarray) -> np.ndarray:
    """one categorical draw per row of z (input recipe only: numpy Gumbel-max)."""
    g = rng.gumbel(size=z.shape).astype(np.float32)
    return np.argmax(z.astype(np.float32) + g, axis=-1).astype(np.int32)


def chain_inputs(B: int, K: int, V: int, dtype: str, kind: str, sigma, seed: int):
    """target [B,K+1,V], draft [B,K,V] = target[:, :K] + N(0, sigma_b^2), cand [B,K] ~ softmax(draft).

    ``sigma`` is a scalar, a length-B array, or a (lo, hi) tuple for sigma_b ~ U(lo, hi).
    Rounding to bf16 happens after both tensors are formed; candidates are drawn from the
    rounded draft logits.
    """
    rng = np.random.default_rng([seed, B, K, V])
    if isinstance(sigma, tuple):
        sig = rng.uniform(sigma[0], sigma[1], size=B)
    else:
        sig = np.broadcast_to(np.asarray(sigma, dtype=np.float64), (B,))
    target = np.empty((B, K + 1, V), dtype=np.uint16 if dtype == "bf16" else np.float32)
    draft = np.empty((B, K, V), dtype=target.dtype)
    cand = np.empty((B, K), dtype=np.int32)
    for b in range(B):
        t = _target_rows(rng, K + 1, V, kind)
        d = t[:K] + rng.standard_normal((K, V), dtype=np.float32) * np.float32(sig[b])
        target[b] = _finish(t, dtype)
        draft[b] = _finish(d, dtype)
        dz = bf16_bits_to_f32(draft[b]) if dtype == "bf16" else draft[b]
        cand[b] = _sample_from_logits(rng, dz)
    return dict(target=target, draft=draft, cand=cand, sigma=np.asarray(sig, dtype=np.float64))


def _log_softmax64(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.float64)
    m = z.max()
    return z - (m + np.log(np.exp(z - m).sum()))


def tree_inputs(B: int, N: int, V: int, dtype: str, sigma: float, seed: int, depth: int = 6,
                topk: int = 4, kind: str = "peaked"):
    """EAGLE-2-shaped token trees.

    Per tree: grow ``depth`` layers; each layer expands the ``topk`` contexts with the best
    cumulative draft log-probability, a context proposing its ``topk`` most probable tokens under
    a draft row = its target row + N(0, sigma^2).  All proposals are ranked by cumulative draft
    log-probability and the best N kept (a parent always outranks its children, so the kept set is
    closed under ancestors).  Nodes are renumbered breadth-first with siblings in descending
    probability, so parent[j] < j.  draft[j] = target row of node j's parent context plus
    independent N(0, sigma^2) noise; target row j+1 is a fresh row for the context after node j.
    """
    rng = np.random.default_rng([seed, B, N, V, 7])
    tdt = np.uint16 if dtype == "bf16" else np.float32
    target = np.empty((B, N + 1, V), dtype=tdt)
    draft = np.empty((B, N, V), dtype=tdt)
    parent = np.empty((B, N), dtype=np.int32)
    tokens = np.empty((B, N), dtype=np.int32)
    max_depth = 0
    for b in range(B):
        ctx_rows = {-1: _target_rows(rng, 1, V, kind)[0]}   # proposal id -> target row of its context
        props = []                                           # (parent proposal id, token, cum logp, depth)
        frontier = [(-1, 0.0, 0)]
        for _ in range(depth):
            new = []
            for pid, cum, dep in frontier:
                if pid not in ctx_rows:
                    ctx_rows[pid] = _target_rows(rng, 1, V, kind)[0]
                e = ctx_rows[pid] + rng.standard_normal(V, dtype=np.float32) * np.float32(sigma)
                lp = _log_softmax64(e)
                k = min(topk, V)
                top = np.argpartition(-lp, k - 1)[:k]
                top = top[np.argsort(-lp[top], kind="stable")]
                for tok in top:
                    props.append((pid, int(tok), cum + float(lp[tok]), dep + 1))
                    new.append((len(props) - 1, cum + float(lp[tok]), dep + 1))
            new.sort(key=lambda t: -t[1])
            frontier = new[:topk]
        order = sorted(range(len(props)), key=lambda i: -props[i][2])[:N]
        if len(order) < N:
            raise ValueError(f"tree recipe yields only {len(order)} proposals, need N={N}")
        kept = set(order)
        # breadth-first renumbering, siblings by descending cumulative probability
        children = {}
        for i in kept:
            children.setdefault(props[i][0], []).append(i)
        for lst in children.values():
            lst.sort(key=lambda i: -props[i][2])
        new_id, queue = {}, [-1]
        seq = []
        while queue:
            nxt = []
            for pid in queue:
                for i in children.get(pid, []):
                    new_id[i] = len(seq)
                    seq.append(i)
                    nxt.append(i)
            queue = nxt
        assert len(seq) == N
        trows = np.empty((N + 1, V), dtype=np.float32)
        drows = np.empty((N, V), dtype=np.float32)
        trows[0] = ctx_rows[-1]
        for j, i in enumerate(seq):
            pid, tok, _, dep = props[i]
            parent[b, j] = -1 if pid < 0 else new_id[pid]
            tokens[b, j] = tok
            max_depth = max(max_depth, dep)
            if i not in ctx_rows:
                ctx_rows[i] = _target_rows(rng, 1, V, kind)[0]
            trows[j + 1] = ctx_rows[i]
            drows[j] = ctx_rows[pid] + rng.standard_normal(V, dtype=np.float32) * np.float32(sigma)
        target[b] = _finish(trows, dtype)
        draft[b] = _finish(drows, dtype)
    return dict(target=target, draft=draft, parent=parent, node_tokens=tokens, max_depth=max_depth)


# The five benchmark configurations (C0..C4).  "T" lists the thresholds of the sweep.
CONFIGS = {
    "C0": dict(shape="chain", B=1, K=4, V=32000, dtype="f32", kind="gauss2", sigma=0.5,
               T=[0.0, 0.05, 0.2, 1e9]),
    "C1": dict(shape="chain", B=1, K=8, V=128256, dtype="bf16", kind="peaked", sigma=[0.25, 1.0, 4.0],
               T=[0.0, 0.005, 0.01, 0.05, 0.1, 0.3, 0.6, 0.7]),
    "C2": dict(shape="chain", B=64, K=8, V=128256, dtype="bf16", kind="peaked", sigma=(0.25, 4.0),
               T=[0.1]),
    "C3": dict(shape="chain", B=256, K=16, V=151936, dtype="f32", kind="zipf", sigma=1.0, T=[0.3]),
    "C4": dict(shape="tree", B=32, N=60, V=128256, dtype="bf16", kind="peaked", sigma=1.0, T=[0.15]),
    # the largest vocabulary among the paper's model pairs (its third family), C2's recipe otherwise
    "C5": dict(shape="chain", B=64, K=8, V=256000, dtype="bf16", kind="peaked", sigma=(0.25, 4.0), T=[0.1]),
}


def config_inputs(name: str, seed: int = 0, sigma=None, B=None):
    """Inputs of configuration ``name``; ``sigma`` picks one point of C1's sweep, ``B`` overrides
    the batch (used to bound host-side work in tests)."""
    c = CONFIGS[name]
    Bv = c["B"] if B is None else B
    if c["shape"] == "tree":
        return tree_inputs(Bv, c["N"], c["V"], c["dtype"], c["sigma"], seed, kind=c["kind"])
    s = c["sigma"] if sigma is None else sigma
    if isinstance(s, list):
        s = s[0]
    return chain_inputs(Bv, c["K"], c["V"], c["dtype"], c["kind"], s, seed)
