"""ctypes binding of libfsd.so: argument marshalling only.

torch is used for device memory (outputs, workspace) and for the current stream handle; no
arithmetic of the method happens here.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

F32, BF16 = 0, 1
DIV_KL, DIV_JS, DIV_TV = 0, 1, 2
SAMPLE, GREEDY = 0, 1
ROW_NONFINITE, ROW_BAD_PARENT, ROW_TOO_DEEP, ROW_BAD_TOKEN, ROW_INTERNAL = 1, 2, 4, 8, 16

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfsd.so")
_lib = None


class FsdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = library().fsd_status_string(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


def library() -> ctypes.CDLL:
    """The loaded C ABI.  Raises if libfsd.so has not been built (python -m paper_2502_20704_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2502_20704_amd.build` "
                "(there is no CPU fallback)")
        # torch first: the library then binds to the HIP runtime torch has loaded.  Loaded before torch
        # it would bring in the system's copy, and a process with two HIP runtimes has its device
        # memory in one and this library's launches in the other.
        import torch  # noqa: F401

        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        vp, i32, u64, f32, sz = c.c_void_p, c.c_int, c.c_uint64, c.c_float, c.c_size_t
        L.fsd_max_vocab.argtypes = [i32]
        L.fsd_max_vocab.restype = c.c_int64
        L.fsd_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.fsd_workspace_bytes.restype = sz
        L.fsd_status_string.argtypes = [i32]
        L.fsd_status_string.restype = c.c_char_p
        L.fsd_verify_chain.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f32, i32, u64, u64,
                                       vp, vp, vp, vp, vp, sz, vp]
        L.fsd_verify_chain.restype = i32
        L.fsd_verify_chain_static.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f32, i32, u64, u64,
                                              vp, vp, vp, vp, vp]
        L.fsd_verify_chain_static.restype = i32
        L.fsd_verify_chain_warped.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f32, i32, u64, u64, f32, i32, f32,
                                              vp, vp, vp, vp, vp, sz, vp]
        L.fsd_verify_chain_warped.restype = i32
        L.fsd_verify_tree_warped.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, i32, u64, u64, f32, i32,
                                             f32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.fsd_verify_tree_warped.restype = i32
        L.fsd_verify_tree.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, i32, u64, u64,
                                      vp, vp, vp, vp, vp, vp, sz, vp]
        L.fsd_verify_tree.restype = i32
        L.sd_verify_chain.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, u64, u64,
                                      vp, vp, vp, vp, vp, sz, vp]
        L.sd_verify_chain.restype = i32
        L.sd_verify_tree.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, u64, u64,
                                     vp, vp, vp, vp, vp, vp, sz, vp]
        L.sd_verify_tree.restype = i32
        L.rfsd_verify_chain.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f32, i32, u64, u64,
                                        vp, vp, vp, vp, vp, vp, sz, vp]
        L.rfsd_verify_chain.restype = i32
        L.fsd_calibrate_workspace_bytes.argtypes = [i32, i32]
        L.fsd_calibrate_workspace_bytes.restype = sz
        L.fsd_calibrate_threshold.argtypes = [vp, i32, i32, f32, vp, vp, vp, sz, vp]
        L.fsd_calibrate_threshold.restype = i32
        L.fsd_profile_enable.argtypes = [i32]
        L.fsd_profile_enable.restype = i32
        L.fsd_profile_collect.argtypes = [vp, vp]
        L.fsd_profile_collect.restype = i32
        L.fsd_debug_set_shape.argtypes = [i32, i32]
        L.fsd_debug_set_shape.restype = i32
        L.fsd_debug_set_js_floor.argtypes = [f32]
        L.fsd_debug_set_js_floor.restype = f32
        L.fsd_debug_set_exact_js.argtypes = [i32]
        L.fsd_debug_set_exact_js.restype = i32
        L.fsd_debug_set_self_clear.argtypes = [i32]
        L.fsd_debug_set_self_clear.restype = i32
        L.fsd_debug_set_spin_limit.argtypes = [c.c_uint]
        L.fsd_debug_set_spin_limit.restype = c.c_uint
        _lib = L
    return _lib


_ws_bytes = {}


def fsd_workspace_bytes(B: int, rows_per_seq: int, V: int, dtype: int) -> int:
    key = (B, rows_per_seq, V, dtype)
    n = _ws_bytes.get(key)
    if n is None:   # the library's answer for a shape does not change: asked once
        n = _ws_bytes[key] = int(library().fsd_workspace_bytes(B, rows_per_seq, V, dtype))
    return n


def _dtype_code(t) -> int:
    import torch

    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"logits must be float32 or bfloat16, got {t.dtype}")


def _check(t, name, shape=None, dtype=None):
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtype}")


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _workspace(workspace, need, device):
    import torch

    if workspace is None:
        workspace = torch.empty(need + 256, dtype=torch.uint8, device=device)
    base = workspace.data_ptr()
    pad = (-base) % 256
    return workspace, ctypes.c_void_p(base + pad), workspace.numel() - pad


def _stream(stream):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def fsd_verify_chain(target, draft, cand, T, div=DIV_JS, mode=SAMPLE, seed=0, offset=0, *, out=None,
                     workspace=None, stream=None):
    """target [B,K+1,V], draft [B,K,V], cand int32 [B,K] on the GPU -> dict of device tensors
    accept_len [B], out_tokens [B,K+1], divergences [B,K], row_status [B]."""
    import torch

    B, K1, V = target.shape
    K = K1 - 1
    dt = _dtype_code(target)
    _check(target, "target")
    _check(draft, "draft", (B, K, V), target.dtype)
    _check(cand, "cand", (B, K), torch.int32)
    dev = target.device
    if out is None:
        out = dict(accept_len=torch.empty(B, dtype=torch.int32, device=dev),
                   out_tokens=torch.empty((B, K + 1), dtype=torch.int32, device=dev),
                   divergences=torch.empty((B, K), dtype=torch.float32, device=dev),
                   row_status=torch.empty(B, dtype=torch.int32, device=dev))
    need = fsd_workspace_bytes(B, K, V, dt)
    workspace, wptr, wbytes = _workspace(workspace, need, dev)
    st = library().fsd_verify_chain(_ptr(target), _ptr(draft), _ptr(cand), B, K, V, dt, div, float(T), mode,
                                    seed, offset, _ptr(out["accept_len"]), _ptr(out["out_tokens"]),
                                    _ptr(out.get("divergences")), _ptr(out.get("row_status")), wptr, wbytes,
                                    _stream(stream))
    if st != 0:
        raise FsdError(st, "fsd_verify_chain")
    out["_workspace"] = workspace
    return out


STATIC_SCRATCH_BYTES = 4 << 20


def fsd_verify_chain_static(target, draft, cand, T, div=DIV_JS, mode=SAMPLE, seed=0, offset=0, *, out, stream=None):
    """fsd_verify_chain on the library's own fixed scratch buffer: nothing is allocated, so the caller
    passes the output tensors (`out`: accept_len, out_tokens and optionally divergences, row_status)."""
    import torch

    B, K1, V = target.shape
    K = K1 - 1
    dt = _dtype_code(target)
    _check(target, "target")
    _check(draft, "draft", (B, K, V), target.dtype)
    _check(cand, "cand", (B, K), torch.int32)
    st = library().fsd_verify_chain_static(_ptr(target), _ptr(draft), _ptr(cand), B, K, V, dt, div, float(T), mode,
                                           seed, offset, _ptr(out["accept_len"]), _ptr(out["out_tokens"]),
                                           _ptr(out.get("divergences")), _ptr(out.get("row_status")), _stream(stream))
    if st != 0:
        raise FsdError(st, "fsd_verify_chain_static")
    return out


def fsd_verify_chain_warped(target, draft, cand, T, div=DIV_JS, mode=SAMPLE, seed=0, offset=0, *,
                            temperature=1.0, top_k=0, top_p=1.0, out=None, workspace=None, stream=None):
    """fsd_verify_chain with temperature / top-k / top-p applied where the token is drawn."""
    import torch

    B, K1, V = target.shape
    K = K1 - 1
    dt = _dtype_code(target)
    _check(target, "target")
    _check(draft, "draft", (B, K, V), target.dtype)
    _check(cand, "cand", (B, K), torch.int32)
    dev = target.device
    if out is None:
        out = dict(accept_len=torch.empty(B, dtype=torch.int32, device=dev),
                   out_tokens=torch.empty((B, K + 1), dtype=torch.int32, device=dev),
                   divergences=torch.empty((B, K), dtype=torch.float32, device=dev),
                   row_status=torch.empty(B, dtype=torch.int32, device=dev))
    need = fsd_workspace_bytes(B, K, V, dt)
    workspace, wptr, wbytes = _workspace(workspace, need, dev)
    st = library().fsd_verify_chain_warped(_ptr(target), _ptr(draft), _ptr(cand), B, K, V, dt, div, float(T), mode,
                                           seed, offset, float(temperature), int(top_k), float(top_p),
                                           _ptr(out["accept_len"]), _ptr(out["out_tokens"]),
                                           _ptr(out.get("divergences")), _ptr(out.get("row_status")), wptr, wbytes,
                                           _stream(stream))
    if st != 0:
        raise FsdError(st, "fsd_verify_chain_warped")
    out["_workspace"] = workspace
    return out


def fsd_verify_tree(target, draft, node_tokens, parent, max_depth, T, div=DIV_JS, mode=SAMPLE, seed=0,
                    offset=0, *, out=None, workspace=None, stream=None):
    """target [B,N+1,V], draft [B,N,V], node_tokens / parent int32 [B,N] -> dict of device tensors
    path_len [B], path_nodes [B,max_depth], out_tokens [B,max_depth+1], divergences [B,N], row_status [B]."""
    import torch

    B, N1, V = target.shape
    N = N1 - 1
    dt = _dtype_code(target)
    _check(target, "target")
    _check(draft, "draft", (B, N, V), target.dtype)
    _check(node_tokens, "node_tokens", (B, N), torch.int32)
    _check(parent, "parent", (B, N), torch.int32)
    dev = target.device
    if out is None:
        out = dict(path_len=torch.empty(B, dtype=torch.int32, device=dev),
                   path_nodes=torch.empty((B, max_depth), dtype=torch.int32, device=dev),
                   out_tokens=torch.empty((B, max_depth + 1), dtype=torch.int32, device=dev),
                   divergences=torch.empty((B, N), dtype=torch.float32, device=dev),
                   row_status=torch.empty(B, dtype=torch.int32, device=dev))
    need = fsd_workspace_bytes(B, N, V, dt)
    workspace, wptr, wbytes = _workspace(workspace, need, dev)
    st = library().fsd_verify_tree(_ptr(target), _ptr(draft), _ptr(node_tokens), _ptr(parent), B, N, max_depth,
                                   V, dt, div, float(T), mode, seed, offset, _ptr(out["path_len"]),
                                   _ptr(out["path_nodes"]), _ptr(out["out_tokens"]),
                                   _ptr(out.get("divergences")), _ptr(out.get("row_status")), wptr, wbytes,
                                   _stream(stream))
    if st != 0:
        raise FsdError(st, "fsd_verify_tree")
    out["_workspace"] = workspace
    return out


def fsd_verify_tree_warped(target, draft, node_tokens, parent, max_depth, T, div=DIV_JS, mode=SAMPLE, seed=0,
                           offset=0, *, temperature=1.0, top_k=0, top_p=1.0, out=None, workspace=None, stream=None):
    """fsd_verify_tree with temperature / top-k / top-p applied where the token is drawn."""
    import torch

    B, N1, V = target.shape
    N = N1 - 1
    dt = _dtype_code(target)
    _check(target, "target")
    _check(draft, "draft", (B, N, V), target.dtype)
    _check(node_tokens, "node_tokens", (B, N), torch.int32)
    _check(parent, "parent", (B, N), torch.int32)
    dev = target.device
    if out is None:
        out = dict(path_len=torch.empty(B, dtype=torch.int32, device=dev),
                   path_nodes=torch.empty((B, max_depth), dtype=torch.int32, device=dev),
                   out_tokens=torch.empty((B, max_depth + 1), dtype=torch.int32, device=dev),
                   divergences=torch.empty((B, N), dtype=torch.float32, device=dev),
                   row_status=torch.empty(B, dtype=torch.int32, device=dev))
    need = fsd_workspace_bytes(B, N, V, dt)
    workspace, wptr, wbytes = _workspace(workspace, need, dev)
    st = library().fsd_verify_tree_warped(_ptr(target), _ptr(draft), _ptr(node_tokens), _ptr(parent), B, N, max_depth,
                                          V, dt, div, float(T), mode, seed, offset, float(temperature), int(top_k),
                                          float(top_p), _ptr(out["path_len"]), _ptr(out["path_nodes"]),
                                          _ptr(out["out_tokens"]), _ptr(out.get("divergences")),
                                          _ptr(out.get("row_status")), wptr, wbytes, _stream(stream))
    if st != 0:
        raise FsdError(st, "fsd_verify_tree_warped")
    out["_workspace"] = workspace
    return out


def sd_verify_chain(target, draft, cand, mode=SAMPLE, seed=0, offset=0, *, out=None, workspace=None,
                    stream=None):
    """strict speculative decoding on the chain tensors -> accept_len, out_tokens, log_ratio, row_status."""
    import torch

    B, K1, V = target.shape
    K = K1 - 1
    dt = _dtype_code(target)
    _check(target, "target")
    _check(draft, "draft", (B, K, V), target.dtype)
    _check(cand, "cand", (B, K), torch.int32)
    dev = target.device
    if out is None:
        out = dict(accept_len=torch.empty(B, dtype=torch.int32, device=dev),
                   out_tokens=torch.empty((B, K + 1), dtype=torch.int32, device=dev),
                   log_ratio=torch.empty((B, K), dtype=torch.float32, device=dev),
                   row_status=torch.empty(B, dtype=torch.int32, device=dev))
    need = fsd_workspace_bytes(B, K, V, dt)
    workspace, wptr, wbytes = _workspace(workspace, need, dev)
    st = library().sd_verify_chain(_ptr(target), _ptr(draft), _ptr(cand), B, K, V, dt, mode, seed, offset,
                                   _ptr(out["accept_len"]), _ptr(out["out_tokens"]), _ptr(out.get("log_ratio")),
                                   _ptr(out.get("row_status")), wptr, wbytes, _stream(stream))
    if st != 0:
        raise FsdError(st, "sd_verify_chain")
    out["_workspace"] = workspace
    return out


def sd_verify_tree(target, draft, node_tokens, parent, max_depth, mode=SAMPLE, seed=0, offset=0, *, out=None,
                   workspace=None, stream=None):
    """strict speculative decoding over a token tree (tensors of fsd_verify_tree) -> path_len, path_nodes,
    out_tokens, log_ratio [B,N] (NaN for nodes never tried), row_status."""
    import torch

    B, N1, V = target.shape
    N = N1 - 1
    dt = _dtype_code(target)
    _check(target, "target")
    _check(draft, "draft", (B, N, V), target.dtype)
    _check(node_tokens, "node_tokens", (B, N), torch.int32)
    _check(parent, "parent", (B, N), torch.int32)
    dev = target.device
    if out is None:
        out = dict(path_len=torch.empty(B, dtype=torch.int32, device=dev),
                   path_nodes=torch.empty((B, max_depth), dtype=torch.int32, device=dev),
                   out_tokens=torch.empty((B, max_depth + 1), dtype=torch.int32, device=dev),
                   log_ratio=torch.empty((B, N), dtype=torch.float32, device=dev),
                   row_status=torch.empty(B, dtype=torch.int32, device=dev))
    need = fsd_workspace_bytes(B, N, V, dt)
    workspace, wptr, wbytes = _workspace(workspace, need, dev)
    st = library().sd_verify_tree(_ptr(target), _ptr(draft), _ptr(node_tokens), _ptr(parent), B, N, max_depth, V,
                                  dt, mode, seed, offset, _ptr(out["path_len"]), _ptr(out["path_nodes"]),
                                  _ptr(out["out_tokens"]), _ptr(out.get("log_ratio")), _ptr(out.get("row_status")),
                                  wptr, wbytes, _stream(stream))
    if st != 0:
        raise FsdError(st, "sd_verify_tree")
    out["_workspace"] = workspace
    return out


def rfsd_verify_chain(target, draft, cand, T, div=DIV_JS, mode=SAMPLE, seed=0, offset=0, *, out=None,
                      workspace=None, stream=None):
    """reducible FSD on the chain tensors -> accept_len, out_tokens, divergences, log_ratio, row_status."""
    import torch

    B, K1, V = target.shape
    K = K1 - 1
    dt = _dtype_code(target)
    _check(target, "target")
    _check(draft, "draft", (B, K, V), target.dtype)
    _check(cand, "cand", (B, K), torch.int32)
    dev = target.device
    if out is None:
        out = dict(accept_len=torch.empty(B, dtype=torch.int32, device=dev),
                   out_tokens=torch.empty((B, K + 1), dtype=torch.int32, device=dev),
                   divergences=torch.empty((B, K), dtype=torch.float32, device=dev),
                   log_ratio=torch.empty((B, K), dtype=torch.float32, device=dev),
                   row_status=torch.empty(B, dtype=torch.int32, device=dev))
    need = fsd_workspace_bytes(B, K, V, dt)
    workspace, wptr, wbytes = _workspace(workspace, need, dev)
    st = library().rfsd_verify_chain(_ptr(target), _ptr(draft), _ptr(cand), B, K, V, dt, int(div), float(T), mode,
                                     seed, offset, _ptr(out["accept_len"]), _ptr(out["out_tokens"]),
                                     _ptr(out.get("divergences")), _ptr(out.get("log_ratio")),
                                     _ptr(out.get("row_status")), wptr, wbytes, _stream(stream))
    if st != 0:
        raise FsdError(st, "rfsd_verify_chain")
    out["_workspace"] = workspace
    return out


def fsd_calibrate_threshold(divergences, target_fraction: float, *, stream=None):
    """(T, accepted fraction) as 1-element device tensors: the smallest occurring threshold at which
    the chain rule accepts at least `target_fraction` of the candidate positions of `divergences`."""
    import torch

    _check(divergences, "divergences", None, torch.float32)
    B, K = divergences.shape
    dev = divergences.device
    need = int(library().fsd_calibrate_workspace_bytes(B, K))
    if need == 0:
        raise FsdError(-2, "fsd_calibrate_workspace_bytes")
    ws = torch.empty(need + 256, dtype=torch.uint8, device=dev)
    off = (-ws.data_ptr()) % 256
    T = torch.empty(1, dtype=torch.float32, device=dev)
    frac = torch.empty(1, dtype=torch.float32, device=dev)
    st = library().fsd_calibrate_threshold(_ptr(divergences), B, K, float(target_fraction), _ptr(T), _ptr(frac),
                                           ctypes.c_void_p(ws.data_ptr() + off), need, _stream(stream))
    if st != 0:
        raise FsdError(st, "fsd_calibrate_threshold")
    T._workspace = ws   # keep the workspace alive until the stream has used it
    return T, frac


def profile_enable(on: bool) -> None:
    library().fsd_profile_enable(1 if on else 0)


def profile_collect():
    """(count, mean_ms, min_ms) of the vocabulary-reduction kernel since the last collect."""
    mean, mn = ctypes.c_float(0), ctypes.c_float(0)
    n = library().fsd_profile_collect(ctypes.byref(mean), ctypes.byref(mn))
    return int(n), float(mean.value), float(mn.value)


def debug_set_spin_limit(polls: int) -> int:
    return int(library().fsd_debug_set_spin_limit(polls))


def debug_warp_thresholds(out, B: int, rows: int, V: int, dtype_code: int):
    """the per-sequence cut fsd_verify_chain_warped left in its workspace (test hook), as a float32 tensor [B]"""
    import torch

    L = library()
    L.fsd_debug_warp_threshold_offset.argtypes = [ctypes.c_int] * 4
    L.fsd_debug_warp_threshold_offset.restype = ctypes.c_size_t
    off = L.fsd_debug_warp_threshold_offset(B, rows, V, dtype_code)
    ws = out["_workspace"]
    base = (-ws.data_ptr()) % 256          # the binding hands the library a 256-byte aligned start
    return ws[base + off: base + off + 4 * B].view(torch.float32).clone()


def debug_set_js_floor(floor_nats: float) -> float:
    """floor (nats) below which the bfloat16 JS reduction evaluates a pair again in the pointwise form"""
    return float(library().fsd_debug_set_js_floor(float(floor_nats)))


def debug_set_exact_js(on: bool) -> bool:
    """bfloat16 JS in the pointwise form only (test hook); returns the previous setting"""
    return bool(library().fsd_debug_set_exact_js(1 if on else 0))


def debug_set_self_clear(on: bool) -> bool:
    """Test hook: False makes every verify call launch the clearing kernel; returns the previous setting."""
    return bool(library().fsd_debug_set_self_clear(1 if on else 0))


def debug_set_shape(wavefronts: int, slots_per_thread: int) -> None:
    st = library().fsd_debug_set_shape(wavefronts, slots_per_thread)
    _ws_bytes.clear()   # the workspace a shape needs depends on the hook's setting
    if st != 0:
        raise FsdError(st, "fsd_debug_set_shape")
