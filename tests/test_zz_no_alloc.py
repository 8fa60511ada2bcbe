"""The entry point that allocates nothing (fsd_verify_chain_static: the workspace is a fixed buffer
inside the library) against fsd_verify_chain on the same inputs, through the C ABI: two calls in a
row, the second with a smaller input, so that what the first call left in the buffer is there when
the second starts."""
import ctypes

import numpy as np
import pytest

import paper_2502_20704_amd as fsd
from paper_2502_20704_amd import synth

pytestmark = pytest.mark.gpu


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _both(torch, L, inp, T, div, seed, offset):
    """(outputs of fsd_verify_chain, outputs of fsd_verify_chain_static) as numpy arrays, via the raw C ABI"""
    B, K1, V = inp["target"].shape
    K = K1 - 1
    dt = fsd.BF16 if inp["target"].dtype == np.uint16 else fsd.F32
    tgt, drf, cand = (synth.as_torch(inp[k]) for k in ("target", "draft", "cand"))
    res = []
    for static in (False, True):
        n = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        tok = torch.full((B, K + 1), -7, dtype=torch.int32, device="cuda")
        dv = torch.full((B, K), -7.0, dtype=torch.float32, device="cuda")
        rs = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        if static:
            st = L.fsd_verify_chain_static(_ptr(tgt), _ptr(drf), _ptr(cand), B, K, V, dt, div, T, fsd.SAMPLE, seed, offset,
                                           _ptr(n), _ptr(tok), _ptr(dv), _ptr(rs), stream)
        else:
            need = L.fsd_workspace_bytes(B, K, V, dt)
            assert 0 < need <= fsd.STATIC_SCRATCH_BYTES
            ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
            base = ws.data_ptr() + (-ws.data_ptr()) % 256
            st = L.fsd_verify_chain(_ptr(tgt), _ptr(drf), _ptr(cand), B, K, V, dt, div, T, fsd.SAMPLE, seed, offset,
                                    _ptr(n), _ptr(tok), _ptr(dv), _ptr(rs), ctypes.c_void_p(base), need, stream)
        assert st == 0, fsd.library().fsd_status_string(st)
        torch.cuda.synchronize()
        res.append(dict(accept_len=n.cpu().numpy(), out_tokens=tok.cpu().numpy(), divergences=dv.cpu().numpy(),
                        row_status=rs.cpu().numpy()))
    return res


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch

    assert torch.cuda.is_available()
    L = fsd.library()
    # first a call that uses a good part of the buffer, then a smaller one (fewer sequences, shorter
    # chains, smaller vocabulary, other dtype and divergence) that finds the first one's words there
    calls = [
        (synth.chain_inputs(24, 8, 128256, "bf16", "peaked", (0.25, 4.0), seed=71), 0.1, fsd.DIV_JS),
        (synth.chain_inputs(3, 5, 32000, "f32", "gauss2", 0.5, seed=72), 0.03, fsd.DIV_TV),
        (synth.chain_inputs(5, 3, 4097, "bf16", "zipf", 1.0, seed=73), 0.2, fsd.DIV_KL),
    ]
    for i, (inp, T, div) in enumerate(calls):
        print(f"static call {i}: shape {inp['target'].shape} div {div}", flush=True)
        ref, got = _both(torch, L, inp, T, div, seed=9, offset=i)
        assert (ref["row_status"] == 0).all()
        # same kernels, fixed summation order: the two entry points agree bit for bit
        assert (got["accept_len"] == ref["accept_len"]).all()
        assert (got["out_tokens"] == ref["out_tokens"]).all()
        assert (got["row_status"] == ref["row_status"]).all()
        assert (got["divergences"].view(np.uint32) == ref["divergences"].view(np.uint32)).all()
        assert (ref["accept_len"] >= 0).all() and (ref["out_tokens"] >= -1).all()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch

    L = fsd.library()
    B, K, V = 256, 16, 151936
    assert L.fsd_workspace_bytes(B, K, V, fsd.F32) > fsd.STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: the call is refused before anything is launched
    st = L.fsd_verify_chain_static(fake, fake, fake, B, K, V, fsd.F32, fsd.DIV_JS, 0.3, fsd.SAMPLE, 0, 0,
                                   fake, fake, None, None, None)
    assert st == -8
    assert b"static" in L.fsd_status_string(st)
    assert L.fsd_verify_chain_static(None, fake, fake, 2, 4, 1000, fsd.F32, fsd.DIV_JS, 0.3, fsd.SAMPLE, 0, 0,
                                     fake, fake, None, None, None) == -1
    torch.cuda.synchronize()
