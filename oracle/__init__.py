"""TEST INFRASTRUCTURE -- float64 CPU oracle for the FSD verification step.

Thin ctypes/numpy access to ``fsd_oracle.c`` (the arithmetic lives there, each
function citing the passage of the paper it follows).  Only tests, the smoke
check and the bench's cpu_baseline leg import this package; the HIP library and
its Python binding never do, and this package imports nothing from them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fsd_oracle.c")
_LIB = os.path.join(_HERE, "libfsd_oracle.so")

F32, BF16 = 0, 1
DIV_KL, DIV_JS, DIV_TV = 0, 1, 2
SAMPLE, GREEDY = 0, 1
ST_NONFINITE, ST_BAD_PARENT, ST_TOO_DEEP, ST_BAD_TOKEN = 1, 2, 4, 8


def build(force: bool = False) -> str:
    """Compile fsd_oracle.c with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c = ctypes
        vp, i32, i64, u32, u64, dbl = c.c_void_p, c.c_int, c.c_long, c.c_uint32, c.c_uint64, c.c_double
        L.fsd_oracle_num_threads.restype = c.c_int
        L.fsd_oracle_set_num_threads.argtypes = [c.c_int]
        L.fsd_oracle_set_num_threads.restype = None
        L.fsd_oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.fsd_oracle_random_word.argtypes = [u64, u64, u32, u32, u32]
        L.fsd_oracle_random_word.restype = u32
        L.fsd_oracle_word_to_uniform.argtypes = [u32]
        L.fsd_oracle_word_to_uniform.restype = c.c_float
        L.fsd_oracle_flog32.argtypes = [c.c_float]
        L.fsd_oracle_flog32.restype = c.c_float
        L.fsd_oracle_gumbel.argtypes = [u32]
        L.fsd_oracle_gumbel.restype = c.c_float
        L.fsd_oracle_pair.argtypes = [vp, c.c_size_t, vp, c.c_size_t, i64, i32, vp, vp]
        L.fsd_oracle_pair.restype = c.c_int
        L.fsd_oracle_verify_chain.argtypes = [vp, vp, vp, i32, i32, i64, i32, i32, dbl, i32, u64, u64, i32,
                                              vp, vp, vp, vp, vp]
        L.fsd_oracle_verify_chain.restype = c.c_int
        L.fsd_oracle_verify_tree.argtypes = [vp, vp, vp, vp, i32, i32, i32, i64, i32, i32, dbl, i32,
                                             u64, u64, i32, vp, vp, vp, vp, vp, vp]
        L.fsd_oracle_verify_tree.restype = c.c_int
        L.sd_oracle_verify_chain.argtypes = [vp, vp, vp, i32, i32, i64, i32, i32, u64, u64, i32,
                                             vp, vp, vp, vp, vp, vp]
        L.sd_oracle_verify_chain.restype = c.c_int
        L.fsd_oracle_verify_tree_warped.argtypes = [vp, vp, vp, vp, i32, i32, i32, i64, i32, i32, dbl, i32,
                                                    u64, u64, i32, c.c_float, i32, dbl, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fsd_oracle_verify_tree_warped.restype = c.c_int
        L.sd_oracle_verify_tree.argtypes = [vp, vp, vp, vp, i32, i32, i32, i64, i32, i32, u64, u64, i32,
                                            vp, vp, vp, vp, vp, vp, vp]
        L.sd_oracle_verify_tree.restype = c.c_int
        L.rfsd_oracle_verify_chain.argtypes = [vp, vp, vp, i32, i32, i64, i32, i32, dbl, i32, u64, u64, i32,
                                               vp, vp, vp, vp, vp, vp, vp]
        L.rfsd_oracle_verify_chain.restype = c.c_int
        L.fsd_oracle_verify_chain_warped.argtypes = [vp, vp, vp, i32, i32, i64, i32, i32, dbl, i32, u64, u64, i32,
                                                     c.c_float, i32, dbl, vp, vp, vp, vp, vp, vp, vp]
        L.fsd_oracle_verify_chain_warped.restype = c.c_int
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().fsd_oracle_num_threads())


def set_num_threads(n: int) -> None:
    """threads of the loops over sequences (for timing the oracle on one core; results do not depend on it)"""
    lib().fsd_oracle_set_num_threads(int(n))


def _dt(a: np.ndarray) -> int:
    """float32 arrays are logits; uint16 arrays hold bfloat16 bit patterns."""
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"logits must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _c(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().fsd_oracle_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def random_word(seed: int, offset: int, stream: int, b: int, idx: int) -> int:
    return int(lib().fsd_oracle_random_word(seed, offset, stream, b, idx))


def word_to_uniform(w: int) -> float:
    return float(lib().fsd_oracle_word_to_uniform(w))


def flog32(x: float) -> float:
    return float(lib().fsd_oracle_flog32(x))


def gumbel(w: int) -> float:
    return float(lib().fsd_oracle_gumbel(w))


def pair_divergences(t_row: np.ndarray, d_row: np.ndarray):
    """(KL, JS, TV), (lse_t, lse_d), status for one (target row, draft row)."""
    t_row, d_row = _c(t_row), _c(d_row)
    assert t_row.ndim == 1 and t_row.shape == d_row.shape and t_row.dtype == d_row.dtype
    out = np.zeros(3)
    lse = np.zeros(2)
    st = lib().fsd_oracle_pair(_p(t_row), 0, _p(d_row), 0, t_row.shape[0], _dt(t_row), _p(out), _p(lse))
    return out, lse, int(st)


def verify_chain(target, draft, cand, T, div=DIV_JS, mode=SAMPLE, seed=0, offset=0, seq_offset=0):
    target, draft = _c(target), _c(draft)
    cand = _c(np.asarray(cand, dtype=np.int32))
    B, K1, V = target.shape
    K = K1 - 1
    assert draft.shape == (B, K, V) and cand.shape == (B, K) and draft.dtype == target.dtype
    out = dict(accept_len=np.zeros(B, np.int32), out_tokens=np.zeros((B, K + 1), np.int32),
               divs=np.zeros((B, K)), row_status=np.zeros(B, np.int32), gap=np.zeros(B, np.float32))
    lib().fsd_oracle_verify_chain(_p(target), _p(draft), _p(cand), B, K, V, _dt(target), div,
                                  float(np.float32(T)), mode, seed, offset, seq_offset,
                                  _p(out["accept_len"]), _p(out["out_tokens"]), _p(out["divs"]),
                                  _p(out["row_status"]),
                                  _p(out["gap"]))
    return out


def verify_tree(target, draft, node_tokens, parent, max_depth, T, div=DIV_JS, mode=SAMPLE, seed=0,
                offset=0, seq_offset=0):
    target, draft = _c(target), _c(draft)
    node_tokens = _c(np.asarray(node_tokens, dtype=np.int32))
    parent = _c(np.asarray(parent, dtype=np.int32))
    B, N1, V = target.shape
    N = N1 - 1
    assert draft.shape == (B, N, V) and node_tokens.shape == (B, N) and parent.shape == (B, N)
    out = dict(path_len=np.zeros(B, np.int32), path_nodes=np.zeros((B, max_depth), np.int32),
               out_tokens=np.zeros((B, max_depth + 1), np.int32), divs=np.zeros((B, N)),
               row_status=np.zeros(B, np.int32), gap=np.zeros(B, np.float32))
    lib().fsd_oracle_verify_tree(_p(target), _p(draft), _p(node_tokens), _p(parent), B, N, max_depth, V,
                                 _dt(target), div, float(np.float32(T)), mode, seed, offset, seq_offset,
                                 _p(out["path_len"]), _p(out["path_nodes"]), _p(out["out_tokens"]),
                                 _p(out["divs"]), _p(out["row_status"]), _p(out["gap"]))
    return out


def sd_verify_chain(target, draft, cand, mode=SAMPLE, seed=0, offset=0, seq_offset=0):
    target, draft = _c(target), _c(draft)
    cand = _c(np.asarray(cand, dtype=np.int32))
    B, K1, V = target.shape
    K = K1 - 1
    assert draft.shape == (B, K, V) and cand.shape == (B, K) and draft.dtype == target.dtype
    out = dict(accept_len=np.zeros(B, np.int32), out_tokens=np.zeros((B, K + 1), np.int32),
               log_ratio=np.zeros((B, K)), margin=np.zeros((B, K)), row_status=np.zeros(B, np.int32),
               gap=np.zeros(B))
    lib().sd_oracle_verify_chain(_p(target), _p(draft), _p(cand), B, K, V, _dt(target), mode, seed,
                                 offset, seq_offset, _p(out["accept_len"]), _p(out["out_tokens"]),
                                 _p(out["log_ratio"]), _p(out["margin"]), _p(out["row_status"]),
                                 _p(out["gap"]))
    return out


def verify_tree_warped(target, draft, node_tokens, parent, max_depth, T, div=DIV_JS, mode=SAMPLE, seed=0,
                       offset=0, seq_offset=0, temperature=1.0, top_k=0, top_p=1.0):
    """verify_tree with temperature / top-k / top-p applied where the token is drawn."""
    target, draft = _c(target), _c(draft)
    node_tokens = _c(np.asarray(node_tokens, dtype=np.int32))
    parent = _c(np.asarray(parent, dtype=np.int32))
    B, N1, V = target.shape
    N = N1 - 1
    assert draft.shape == (B, N, V) and node_tokens.shape == (B, N) and parent.shape == (B, N)
    assert temperature > 0 and top_k >= 0 and 0 < top_p <= 1
    inv_temp = float(np.float32(1.0 / float(temperature)))
    out = dict(path_len=np.zeros(B, np.int32), path_nodes=np.zeros((B, max_depth), np.int32),
               out_tokens=np.zeros((B, max_depth + 1), np.int32), divs=np.zeros((B, N)),
               row_status=np.zeros(B, np.int32), gap=np.zeros(B, np.float32),
               threshold=np.zeros(B, np.float32), slack=np.zeros(B))
    lib().fsd_oracle_verify_tree_warped(_p(target), _p(draft), _p(node_tokens), _p(parent), B, N, max_depth, V,
                                        _dt(target), div, float(np.float32(T)), mode, seed, offset, seq_offset,
                                        inv_temp, int(top_k), float(np.float32(top_p)), _p(out["path_len"]),
                                        _p(out["path_nodes"]), _p(out["out_tokens"]), _p(out["divs"]),
                                        _p(out["row_status"]), _p(out["gap"]), _p(out["threshold"]),
                                        _p(out["slack"]))
    return out


def sd_verify_tree(target, draft, node_tokens, parent, max_depth, mode=SAMPLE, seed=0, offset=0, seq_offset=0):
    """Strict SD over a token tree: children in index order, residual update after every rejection."""
    target, draft = _c(target), _c(draft)
    node_tokens = _c(np.asarray(node_tokens, dtype=np.int32))
    parent = _c(np.asarray(parent, dtype=np.int32))
    B, N1, V = target.shape
    N = N1 - 1
    assert draft.shape == (B, N, V) and node_tokens.shape == (B, N) and parent.shape == (B, N)
    assert draft.dtype == target.dtype
    out = dict(path_len=np.zeros(B, np.int32), path_nodes=np.zeros((B, max_depth), np.int32),
               out_tokens=np.zeros((B, max_depth + 1), np.int32), log_ratio=np.zeros((B, N)),
               margin=np.zeros((B, N)), row_status=np.zeros(B, np.int32), gap=np.zeros(B))
    lib().sd_oracle_verify_tree(_p(target), _p(draft), _p(node_tokens), _p(parent), B, N, max_depth, V,
                                _dt(target), mode, seed, offset, seq_offset, _p(out["path_len"]),
                                _p(out["path_nodes"]), _p(out["out_tokens"]), _p(out["log_ratio"]),
                                _p(out["margin"]), _p(out["row_status"]), _p(out["gap"]))
    return out


def rfsd_verify_chain(target, draft, cand, T, div, mode=SAMPLE, seed=0, offset=0, seq_offset=0):
    """Reducible FSD (Sec. 4.3): accept iff div <= T or the strict SD test accepts."""
    target, draft = _c(target), _c(draft)
    cand = _c(np.asarray(cand, dtype=np.int32))
    B, K1, V = target.shape
    K = K1 - 1
    assert draft.shape == (B, K, V) and cand.shape == (B, K) and draft.dtype == target.dtype
    out = dict(accept_len=np.zeros(B, np.int32), out_tokens=np.zeros((B, K + 1), np.int32),
               divs=np.zeros((B, K)), log_ratio=np.zeros((B, K)), margin=np.zeros((B, K)),
               row_status=np.zeros(B, np.int32), gap=np.zeros(B))
    lib().rfsd_oracle_verify_chain(_p(target), _p(draft), _p(cand), B, K, V, _dt(target), int(div),
                                   float(np.float32(T)), mode, seed, offset, seq_offset,
                                   _p(out["accept_len"]), _p(out["out_tokens"]), _p(out["divs"]),
                                   _p(out["log_ratio"]), _p(out["margin"]), _p(out["row_status"]),
                                   _p(out["gap"]))
    return out


def accepted_fraction(divs, T):
    """Share of all candidate positions the chain rule accepts at threshold T (Sec. 4 eq. 4 with the
    "<=" reading): per sequence, the positions before the first one whose divergence exceeds T."""
    divs = np.asarray(divs, dtype=np.float64)
    B, K = divs.shape
    acc = 0
    for b in range(B):
        for i in range(K):
            if not (divs[b, i] <= T):   # NaN rejects
                break
            acc += 1
    return acc / float(B * K)


def calibrate_threshold(divs, fraction):
    """Threshold tuning on a dev set (Sec. 6.2 "Selecting T", paragraph "Tuning T on small dev set"; App. A: the T that accepts
    about the same share of candidate tokens as strict SD): the smallest T, among the divergences that
    occur (and +inf), at which the chain rule accepts at least `fraction` of all candidate positions.
    Plain search over every candidate value; returns (T, accepted fraction at T).  0 < fraction <= 1."""
    assert 0.0 < fraction <= 1.0
    divs = np.asarray(divs, dtype=np.float64)
    values = np.unique(np.concatenate([divs[np.isfinite(divs)].ravel(), [np.inf]]))
    for T in values:            # ascending
        f = accepted_fraction(divs, T)
        if f >= fraction:
            return float(T), f
    return float("inf"), accepted_fraction(divs, np.inf)


def verify_chain_warped(target, draft, cand, T, div=DIV_JS, mode=SAMPLE, seed=0, offset=0, seq_offset=0,
                        temperature=1.0, top_k=0, top_p=1.0):
    """verify_chain with temperature / top-k / top-p applied where the token is drawn."""
    target, draft = _c(target), _c(draft)
    cand = _c(np.asarray(cand, dtype=np.int32))
    B, K1, V = target.shape
    K = K1 - 1
    assert draft.shape == (B, K, V) and cand.shape == (B, K) and draft.dtype == target.dtype
    assert temperature > 0 and top_k >= 0 and 0 < top_p <= 1
    inv_temp = float(np.float32(1.0 / float(temperature)))
    out = dict(accept_len=np.zeros(B, np.int32), out_tokens=np.zeros((B, K + 1), np.int32),
               divs=np.zeros((B, K)), row_status=np.zeros(B, np.int32), gap=np.zeros(B, np.float32),
               threshold=np.zeros(B, np.float32), slack=np.zeros(B))
    lib().fsd_oracle_verify_chain_warped(_p(target), _p(draft), _p(cand), B, K, V, _dt(target), div,
                                         float(np.float32(T)), mode, seed, offset, seq_offset, inv_temp,
                                         int(top_k), float(np.float32(top_p)), _p(out["accept_len"]),
                                         _p(out["out_tokens"]), _p(out["divs"]), _p(out["row_status"]),
                                         _p(out["gap"]), _p(out["threshold"]), _p(out["slack"]))
    return out
