"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import paper_2502_20704_amd as fsd
from paper_2502_20704_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    fsd.library()
    return torch


def run_chain(torch, inp, T, div, mode=fsd.SAMPLE, seed=0, offset=0):
    d = pu.to_dev(inp, ("target", "draft", "cand"))
    out = fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], T, div, mode, seed, offset)
    torch.cuda.synchronize()
    return pu.host(out, pu.CHAIN_KEYS)


def run_tree(torch, inp, T, div, max_depth, mode=fsd.SAMPLE, seed=0, offset=0):
    d = pu.to_dev(inp, ("target", "draft", "node_tokens", "parent"))
    out = fsd.fsd_verify_tree(d["target"], d["draft"], d["node_tokens"], d["parent"], max_depth, T, div, mode,
                              seed, offset)
    torch.cuda.synchronize()
    return pu.host(out, pu.TREE_KEYS)


# ------------------------------------------------------------------------------ small shapes

SMALL = [  # (B, K, V, dtype, kind, sigma): aligned and ragged V, one slot to several team members
    (3, 5, 8, "f32", "gauss2", 1.0),
    (2, 3, 100, "bf16", "gauss2", 0.5),
    (4, 7, 1000, "f32", "peaked", 1.0),
    (2, 4, 4097, "bf16", "peaked", 2.0),
    (3, 2, 4099, "f32", "zipf", 1.0),
    (5, 9, 32000, "bf16", "zipf", (0.25, 4.0)),
    (2, 6, 40004, "f32", "gauss2", 0.25),
    (1, 1, 1, "f32", "gauss2", 1.0),
    (1, 64, 2048, "bf16", "peaked", 1.0),
]


@pytest.mark.parametrize("B,K,V,dtype,kind,sigma", SMALL)
@pytest.mark.parametrize("div", [fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV])
def test_chain_small(torch_cuda, oracle, B, K, V, dtype, kind, sigma, div):
    inp = synth.chain_inputs(B, K, V, dtype, kind, sigma, seed=17)
    for T in (0.0, 0.03, 0.2, 1e9, -1.0):
        print(f"chain B={B} K={K} V={V} {dtype} div={div} T={T}", flush=True)
        g = run_chain(torch_cuda, inp, T, div, seed=5, offset=2)
        o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], T, div, seed=5, offset=2)
        pu.check_chain(g, o, T, pu.rel_tol(dtype), f"B={B} K={K} V={V} {dtype} div={div} T={T}")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_maximum_vocabulary(torch_cuda, oracle, dtype):
    """V = fsd_max_vocab: 256 wavefronts per row pair, merged in four rounds of 64; one more entry is refused."""
    vmax = int(fsd.library().fsd_max_vocab(fsd.BF16 if dtype == "bf16" else fsd.F32))
    assert vmax == 524288
    inp = synth.chain_inputs(1, 2, vmax, dtype, "zipf", 1.0, seed=61)
    for div in (fsd.DIV_JS, fsd.DIV_KL, fsd.DIV_TV):
        g = run_chain(torch_cuda, inp, 0.2, div, seed=2)
        o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.2, div, seed=2)
        pu.check_chain(g, o, 0.2, pu.rel_tol(dtype), f"max vocab {dtype} div={div}")
    assert fsd.fsd_workspace_bytes(1, 2, vmax + 1, fsd.BF16 if dtype == "bf16" else fsd.F32) == 0


def test_third_model_family_vocabulary(torch_cuda, oracle):
    """V = 256 000 (the largest vocabulary among the paper's model pairs), 125 wavefronts per pair."""
    inp = synth.chain_inputs(4, 4, 256000, "bf16", "peaked", (0.25, 4.0), seed=62)
    for div in (fsd.DIV_JS, fsd.DIV_KL, fsd.DIV_TV):
        g = run_chain(torch_cuda, inp, 0.1, div, seed=2)
        o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.1, div, seed=2)
        pu.check_chain(g, o, 0.1, 2e-3, f"V=256000 div={div}")


def test_many_short_sequences(torch_cuda, oracle):
    """far more row pairs than resident teams, smallest team size"""
    inp = synth.chain_inputs(700, 5, 1000, "bf16", "gauss2", (0.25, 2.0), seed=63)
    for div in (fsd.DIV_JS, fsd.DIV_KL):
        g = run_chain(torch_cuda, inp, 0.05, div, seed=2)
        o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.05, div, seed=2)
        pu.check_chain(g, o, 0.05, 2e-3, f"B=700 div={div}")


def test_chain_greedy_and_determinism(torch_cuda, oracle):
    inp = synth.chain_inputs(6, 5, 12345, "bf16", "peaked", 1.0, seed=3)
    g = run_chain(torch_cuda, inp, 0.05, fsd.DIV_JS, mode=fsd.GREEDY)
    o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.05, fsd.DIV_JS, mode=oracle.GREEDY)
    pu.check_chain(g, o, 0.05, 2e-3, "greedy")
    a = run_chain(torch_cuda, inp, 0.05, fsd.DIV_JS, seed=9)
    for _ in range(3):
        b = run_chain(torch_cuda, inp, 0.05, fsd.DIV_JS, seed=9)
        for k in pu.CHAIN_KEYS:
            assert np.array_equal(a[k].view(np.uint32) if a[k].dtype == np.float32 else a[k],
                                  b[k].view(np.uint32) if b[k].dtype == np.float32 else b[k]), k


def test_identical_rows_threshold_zero(torch_cuda, oracle):
    """identical logits and T = 0 accept every candidate, for all three divergences."""
    for dtype, V in (("f32", 32000), ("bf16", 128256), ("bf16", 999)):
        inp = synth.chain_inputs(2, 4, V, dtype, "peaked", 1.0, seed=1)
        inp["draft"] = inp["target"][:, :4].copy()
        for div in (fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV):
            g = run_chain(torch_cuda, inp, 0.0, div)
            assert (g["divergences"] == 0).all(), (dtype, V, div, g["divergences"])
            assert (g["accept_len"] == 4).all()
            o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.0, div)
            pu.check_chain(g, o, 0.0, pu.rel_tol(dtype), "identical")


def test_masked_entries_and_closed_form(torch_cuda, oracle):
    """-inf logits are legal; uniform vs half-uniform has JS = 3/4 ln(4/3), TV = 1/2, KL = +inf."""
    V = 128256
    t = np.zeros((1, 2, V), dtype=np.float32)
    d = np.zeros((1, 1, V), dtype=np.float32)
    d[0, 0, V // 2:] = -np.inf
    inp = dict(target=t, draft=d, cand=np.zeros((1, 1), dtype=np.int32))
    g = run_chain(torch_cuda, inp, 0.3, fsd.DIV_JS)
    assert g["divergences"][0, 0] == pytest.approx(0.75 * np.log(4 / 3), rel=1e-5)
    assert g["accept_len"][0] == 1
    g = run_chain(torch_cuda, inp, 0.3, fsd.DIV_TV)
    assert g["divergences"][0, 0] == pytest.approx(0.5, rel=1e-5) and g["accept_len"][0] == 0
    g = run_chain(torch_cuda, inp, 1e30, fsd.DIV_KL)
    assert np.isinf(g["divergences"][0, 0]) and g["accept_len"][0] == 0
    g = run_chain(torch_cuda, inp, float("inf"), fsd.DIV_KL)
    assert g["accept_len"][0] == 1
    # random masks on both sides, all divergences, both dtypes
    for dtype in ("f32", "bf16"):
        inp = synth.chain_inputs(3, 4, 5000, "f32", "gauss2", 1.0, seed=8)
        rng = np.random.default_rng(0)
        inp["target"][rng.random(inp["target"].shape) < 0.3] = -np.inf
        inp["draft"][rng.random(inp["draft"].shape) < 0.3] = -np.inf
        if dtype == "bf16":
            inp["target"], inp["draft"] = synth.to_bf16_bits(inp["target"]), synth.to_bf16_bits(inp["draft"])
        for div in (fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV):
            g = run_chain(torch_cuda, inp, 0.5, div)
            o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.5, div)
            pu.check_chain(g, o, 0.5, pu.rel_tol(dtype), f"masked {dtype} div={div}")


def test_wide_dynamic_range_across_the_team(torch_cuda, oracle):
    """slices of one row whose maxima lie hundreds of units apart: the wavefronts of a team then hold
    reference exponents more than 127 apart, sums relative to the lower ones overflow, and their
    entries must come out as weightless, not as NaN"""
    rng = np.random.default_rng(33)
    B, K, V = 3, 3, 70000
    base = np.where(np.arange(V) < V // 2, -180.0, 150.0).astype(np.float32)      # first half far below
    t = (base + rng.standard_normal((B, K + 1, V)).astype(np.float32) * 2).astype(np.float32)
    d = (base + rng.standard_normal((B, K, V)).astype(np.float32) * 2).astype(np.float32)
    d[1] = t[1, :K]                                                               # identical rows too
    t[2, :, : V // 2] = -np.inf                                                   # and a masked half
    cand = rng.integers(0, V, (B, K)).astype(np.int32)
    for dtype in ("f32", "bf16"):
        inp = dict(target=t, draft=d, cand=cand)
        if dtype == "bf16":
            inp = dict(target=synth.to_bf16_bits(t), draft=synth.to_bf16_bits(d), cand=cand)
        for div in (fsd.DIV_JS, fsd.DIV_KL, fsd.DIV_TV):
            g = run_chain(torch_cuda, inp, 0.3, div, seed=2)
            o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.3, div, seed=2)
            assert (g["row_status"] == 0).all() and np.isfinite(g["divergences"]).all()
            pu.check_chain(g, o, 0.3, pu.rel_tol(dtype), f"wide range {dtype} div={div}")
            assert (g["divergences"][1] == 0).all()


def test_mass_in_opposite_halves(torch_cuda, oracle):
    """target and draft put their mass on different halves of the vocabulary, `gap` units apart: in
    every slice one side's normalising factor vanishes (or nearly) while the other's does not.  JS goes
    to ln 2 and TV to 1.  KL is about `gap`: the bfloat16 path takes it in the log domain (one pass); the
    binary32 path forms p/q entry by entry, which saturates once q/p leaves binary32's range, and then
    has to fall back on the log-domain sums it carries along."""
    rng = np.random.default_rng(34)
    B, K, V = 2, 3, 70000
    for gap in (40.0, 330.0):
        base = np.where(np.arange(V) < V // 2, -gap / 2, gap / 2).astype(np.float32)
        t = (base + rng.standard_normal((B, K + 1, V)).astype(np.float32) * 2).astype(np.float32)
        d = (base[::-1] + rng.standard_normal((B, K, V)).astype(np.float32) * 2).astype(np.float32)
        cand = rng.integers(0, V, (B, K)).astype(np.int32)
        for dtype in ("f32", "bf16"):
            inp = dict(target=t, draft=d, cand=cand)
            if dtype == "bf16":
                inp = dict(target=synth.to_bf16_bits(t), draft=synth.to_bf16_bits(d), cand=cand)
            for div in (fsd.DIV_JS, fsd.DIV_TV, fsd.DIV_KL):
                g = run_chain(torch_cuda, inp, 0.3, div, seed=2)
                o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.3, div, seed=2)
                assert (g["row_status"] == 0).all()
                pu.check_chain(g, o, 0.3, pu.rel_tol(dtype), f"opposite halves gap={gap} {dtype} div={div}")


def test_exponentials_in_the_subnormal_range(torch_cuda, oracle):
    """logits spread evenly over 120 units: next to its largest entry every slice has entries whose
    exponential lies in binary32's subnormal range (87 to 103 below) or underflows altogether, on one
    side, on the other or on both.  Such entries carry no weight, and must not turn into inf or NaN."""
    rng = np.random.default_rng(35)
    B, K, V = 2, 3, 30000
    t = rng.uniform(-120.0, 0.0, (B, K + 1, V)).astype(np.float32)
    d = rng.uniform(-120.0, 0.0, (B, K, V)).astype(np.float32)
    d[1, 0] = t[1, 0]
    cand = rng.integers(0, V, (B, K)).astype(np.int32)
    for dtype in ("f32", "bf16"):
        inp = dict(target=t, draft=d, cand=cand)
        if dtype == "bf16":
            inp = dict(target=synth.to_bf16_bits(t), draft=synth.to_bf16_bits(d), cand=cand)
        for div in (fsd.DIV_JS, fsd.DIV_TV, fsd.DIV_KL):
            g = run_chain(torch_cuda, inp, 0.3, div, seed=3)
            o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.3, div, seed=3)
            assert (g["row_status"] == 0).all() and np.isfinite(g["divergences"]).all()
            assert g["divergences"][1, 0] == 0
            pu.check_chain(g, o, 0.3, pu.rel_tol(dtype), f"subnormal range {dtype} div={div}")


def test_accuracy_envelope_on_nearly_identical_rows(torch_cuda, oracle):
    """The kernels evaluate p and q in binary32, so a divergence carries an absolute error of about 1e-7
    times the mass involved, whatever its size: the relative bar (1e-5 binary32 logits, 2e-3 bfloat16)
    is met above 2e-2 resp. 1e-4, and below that the absolute error stays under 2.5e-7.  Rows that
    differ by noise of 0.001 ... 0.1 on flat and on peaked targets put divergences from 1e-9 to 1e-1."""
    rng = np.random.default_rng(11)
    B, K, V = 3, 3, 20000
    seen_small = 0
    for scale in (0.3, 3.0, 8.0):
        for noise in (0.001, 0.01, 0.1):
            t = (rng.standard_normal((B, K + 1, V)) * scale).astype(np.float32)
            d = (t[:, :K] + rng.standard_normal((B, K, V)) * noise).astype(np.float32)
            cand = rng.integers(0, V, (B, K)).astype(np.int32)
            for dtype in ("f32", "bf16"):
                inp = dict(target=t, draft=d, cand=cand)
                if dtype == "bf16":
                    inp = dict(target=synth.to_bf16_bits(t), draft=synth.to_bf16_bits(d), cand=cand)
                floor = 2e-2 if dtype == "f32" else 1e-4
                for div in (fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV):
                    g = run_chain(torch_cuda, inp, 0.3, div)["divergences"].astype(np.float64)
                    o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.3, div)["divs"]
                    err = np.abs(g - o)
                    what = f"scale={scale} noise={noise} {dtype} div={div}"
                    assert err.max() <= 2.5e-7, f"{what}: absolute error {err.max():.2e}"
                    big = o >= floor
                    assert (err[big] <= pu.rel_tol(dtype) * o[big]).all(), f"{what}: relative error above the floor"
                    assert (g >= 0).all()
                    seen_small += int((~big).sum())
    assert seen_small > 100          # the regime below the floors was exercised


def test_nonfinite_rows_are_flagged(torch_cuda, oracle):
    inp = synth.chain_inputs(4, 3, 3000, "f32", "gauss2", 1.0, seed=2)
    inp["target"][0, 1, 77] = np.nan
    inp["draft"][1, 0, 5] = np.inf
    inp["target"][2, 3, :] = -np.inf          # the bonus row of a sequence that accepts everything
    for div in (fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV):
        g = run_chain(torch_cuda, inp, 1e9, div)
        o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 1e9, div)
        assert list(o["row_status"]) == [1, 1, 1, 0]
        pu.check_chain(g, o, 1e9, 1e-5, f"nonfinite div={div}")
        assert (g["out_tokens"][:3] == -1).all() and (g["accept_len"][:3] == 0).all()


# ------------------------------------------------------------------- benchmark configurations

def test_config_c0(torch_cuda, oracle):
    inp = synth.config_inputs("C0", seed=0)
    for div in (fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV):
        for T in synth.CONFIGS["C0"]["T"]:
            g = run_chain(torch_cuda, inp, T, div, seed=1)
            o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], T, div, seed=1)
            r = pu.check_chain(g, o, T, 1e-5, f"C0 div={div} T={T}")
            print("C0", div, T, r, flush=True)


def test_config_c1_sweep(torch_cuda, oracle):
    for sigma in synth.CONFIGS["C1"]["sigma"]:
        inp = synth.config_inputs("C1", seed=0, sigma=sigma)
        for T in synth.CONFIGS["C1"]["T"]:
            g = run_chain(torch_cuda, inp, T, fsd.DIV_JS, seed=2)
            o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], T, fsd.DIV_JS, seed=2)
            r = pu.check_chain(g, o, T, 2e-3, f"C1 sigma={sigma} T={T}")
            print("C1", sigma, T, r, o["divs"][0, :3], flush=True)


def test_config_c2_full(torch_cuda, oracle):
    inp = synth.config_inputs("C2", seed=0)
    for div in (fsd.DIV_JS, fsd.DIV_KL, fsd.DIV_TV):
        g = run_chain(torch_cuda, inp, 0.1, div, seed=3, offset=11)
        o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.1, div, seed=3, offset=11)
        r = pu.check_chain(g, o, 0.1, 2e-3, f"C2 div={div}")
        print("C2", div, r, "accept_len histogram", np.bincount(o["accept_len"], minlength=9), flush=True)


def test_config_c2_strict_sd(torch_cuda, oracle):
    inp = synth.config_inputs("C2", seed=0)
    d = pu.to_dev(inp, ("target", "draft", "cand"))
    out = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], seed=4, offset=1)
    torch_cuda.cuda.synchronize()
    g = pu.host(out, pu.SD_KEYS)
    o = oracle.sd_verify_chain(inp["target"], inp["draft"], inp["cand"], seed=4, offset=1)
    check_sd(g, o, "C2 SD")


def check_sd(g, o, what):
    assert (g["row_status"] == o["row_status"]).all()
    fin = np.isfinite(o["log_ratio"])
    assert (np.isfinite(g["log_ratio"]) == fin).all()
    assert np.allclose(g["log_ratio"][fin], o["log_ratio"][fin], rtol=2e-5, atol=2e-5), what
    near = np.abs(o["margin"]) <= 1e-5
    n_near = n_tie = 0
    for b in range(o["accept_len"].shape[0]):
        ng, no = int(g["accept_len"][b]), int(o["accept_len"][b])
        if ng != no:
            assert near[b, min(ng, no)], f"{what}: accept_len[{b}] gpu {ng} oracle {no} margin {o['margin'][b]}"
            n_near += 1
            continue
        if not (g["out_tokens"][b] == o["out_tokens"][b]).all():
            # the residual score ln(p - q) is float32 on the GPU, float64 in the oracle: a
            # runner-up within 1e-4 of the winner may overtake it
            assert o["gap"][b] < 1e-4, f"{what}: tokens[{b}] gpu {g['out_tokens'][b]} oracle {o['out_tokens'][b]} gap {o['gap'][b]}"
            n_tie += 1
    print(what, "near-threshold rows", n_near, "near-tie rows", n_tie,
          "accept_len histogram", np.bincount(o["accept_len"]), flush=True)
    assert n_near + n_tie <= max(2, o["accept_len"].shape[0] // 20)


def test_strict_sd_small(torch_cuda, oracle):
    for (B, K, V, dtype, kind, sigma) in SMALL[:7]:
        inp = synth.chain_inputs(B, K, V, dtype, kind, sigma, seed=23)
        d = pu.to_dev(inp, ("target", "draft", "cand"))
        for mode in (fsd.SAMPLE, fsd.GREEDY):
            out = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], mode, seed=6, offset=3)
            torch_cuda.cuda.synchronize()
            g = pu.host(out, pu.SD_KEYS)
            o = oracle.sd_verify_chain(inp["target"], inp["draft"], inp["cand"], mode, seed=6, offset=3)
            check_sd(g, o, f"SD B={B} K={K} V={V} {dtype} mode={mode}")


def check_rfsd(g, o, T, tol, what, envelope=None):
    """reducible FSD: a position is decided by div <= T or by the SD margin; a sequence may differ
    from the oracle only where the deciding quantity sits on its threshold."""
    assert (g["row_status"] == o["row_status"]).all(), what
    pu.check_divs(g["divergences"], o["divs"], tol, what, envelope)
    fin = np.isfinite(o["log_ratio"])
    assert (np.isfinite(g["log_ratio"]) == fin).all()
    assert np.allclose(g["log_ratio"][fin], o["log_ratio"][fin], rtol=2e-5, atol=2e-5), what
    near = pu.near_threshold(o["divs"], T, envelope) | (np.abs(o["margin"]) <= 1e-5)
    n_near = n_tie = 0
    for b in range(o["accept_len"].shape[0]):
        ng, no = int(g["accept_len"][b]), int(o["accept_len"][b])
        if ng != no:
            assert near[b, min(ng, no)], f"{what}: accept_len[{b}] gpu {ng} oracle {no}"
            n_near += 1
            continue
        if not (g["out_tokens"][b] == o["out_tokens"][b]).all():
            assert o["gap"][b] < 1e-4, f"{what}: tokens[{b}] gpu {g['out_tokens'][b]} oracle {o['out_tokens'][b]} gap {o['gap'][b]}"
            n_tie += 1
    assert n_near + n_tie <= max(2, o["accept_len"].shape[0] // 20), what
    return dict(near=n_near, ties=n_tie)


def run_rfsd(torch_cuda, inp, T, div, mode=None, seed=0, offset=0):
    d = pu.to_dev(inp, ("target", "draft", "cand"))
    out = fsd.rfsd_verify_chain(d["target"], d["draft"], d["cand"], T, div, fsd.SAMPLE if mode is None else mode,
                                seed, offset)
    torch_cuda.cuda.synchronize()
    return pu.host(out, pu.RFSD_KEYS)


def test_rfsd_small(torch_cuda, oracle):
    for (B, K, V, dtype, kind, sigma) in SMALL[:7]:
        inp = synth.chain_inputs(B, K, V, dtype, kind, sigma, seed=31)
        tol = pu.rel_tol(dtype)
        for div in (fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV):
            base = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 1e9, div)
            T = float(np.float32(np.median(base["divs"])))
            for mode in (fsd.SAMPLE, fsd.GREEDY):
                g = run_rfsd(torch_cuda, inp, T, div, mode, seed=8, offset=2)
                o = oracle.rfsd_verify_chain(inp["target"], inp["draft"], inp["cand"], T, div, mode, seed=8, offset=2)
                check_rfsd(g, o, T, tol, f"rFSD B={B} K={K} V={V} {dtype} div={div} mode={mode}")


def test_rfsd_reduces_to_strict_sd_and_to_fsd(torch_cuda, oracle):
    """Sec. 4.3: with T = 0 the rule is strict SD's (bit-identical outputs); with a threshold nothing
    exceeds it is FSD's."""
    inp = synth.chain_inputs(16, 6, 32000, "bf16", "peaked", (0.25, 4.0), seed=33)
    d = pu.to_dev(inp, ("target", "draft", "cand"))
    sd = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], seed=12, offset=5)
    torch_cuda.cuda.synchronize()
    sd = pu.host(sd, pu.SD_KEYS)
    for div in (fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV):
        g = run_rfsd(torch_cuda, inp, 0.0, div, seed=12, offset=5)
        assert (g["accept_len"] == sd["accept_len"]).all() and (g["out_tokens"] == sd["out_tokens"]).all()
        f = run_chain(torch_cuda, inp, 1e9, div, seed=12, offset=5)
        g = run_rfsd(torch_cuda, inp, 1e9, div, seed=12, offset=5)
        assert (g["accept_len"] == 6).all() and (g["out_tokens"] == f["out_tokens"]).all()
        if div == fsd.DIV_JS:
            # (bfloat16 JS: FSD evaluates the entropy form, reducible FSD the pointwise one)
            assert np.allclose(g["divergences"], f["divergences"], rtol=0, atol=2e-6)
        else:
            assert np.array_equal(g["divergences"], f["divergences"])


def test_config_c2_rfsd(torch_cuda, oracle):
    inp = synth.config_inputs("C2", seed=0)
    for div in (fsd.DIV_JS, fsd.DIV_KL):
        g = run_rfsd(torch_cuda, inp, 0.1, div, seed=4, offset=1)
        o = oracle.rfsd_verify_chain(inp["target"], inp["draft"], inp["cand"], 0.1, div, seed=4, offset=1)
        r = check_rfsd(g, o, 0.1, 2e-3, f"C2 rFSD div={div}")
        sd = oracle.sd_verify_chain(inp["target"], inp["draft"], inp["cand"], seed=4, offset=1)
        print("C2 rFSD", div, r, "accept_len histogram", np.bincount(o["accept_len"], minlength=9),
              "strict SD", np.bincount(sd["accept_len"], minlength=9), flush=True)


def run_warped(torch_cuda, inp, T, div, mode, seed, offset, **kw):
    d = pu.to_dev(inp, ("target", "draft", "cand"))
    out = fsd.fsd_verify_chain_warped(d["target"], d["draft"], d["cand"], T, div, mode, seed, offset, **kw)
    torch_cuda.cuda.synchronize()
    g = pu.host(out, pu.CHAIN_KEYS)
    B, K1, V = d["target"].shape
    code = fsd.BF16 if inp["target"].dtype == np.uint16 else fsd.F32
    g["threshold"] = fsd.debug_warp_thresholds(out, B, K1 - 1, V, code).cpu().numpy()
    return g


def check_warped(g, o, T, tol, what, sampled=True, cut_active=True, envelope=None):
    """as check_chain; a token may differ where the nucleus mass sat on top_p (the kept set then
    differs by one value) or where two scores tie to 1e-6"""
    assert (g["row_status"] == o["row_status"]).all(), what
    pu.check_divs(g["divergences"], o["divs"], tol, what, envelope)
    assert (g["accept_len"] == o["accept_len"]).all() or pu.near_threshold(o["divs"], T, envelope).any(), what
    n_soft = 0
    for b in range(o["accept_len"].shape[0]):
        if g["accept_len"][b] != o["accept_len"][b]:
            n_soft += 1
            continue
        # the cut itself (the smallest kept scaled logit), not only the token it leads to: exact unless
        # the nucleus mass sits on top_p
        if sampled and o["row_status"][b] == 0 and o["slack"][b] >= 1e-5 and cut_active:
            assert g["threshold"][b] == o["threshold"][b], \
                f"{what}: cut[{b}] gpu {g['threshold'][b]} oracle {o['threshold'][b]} slack {o['slack'][b]}"
        if not (g["out_tokens"][b] == o["out_tokens"][b]).all():
            assert o["slack"][b] < 1e-5 or o["gap"][b] < 1e-6, \
                f"{what}: tokens[{b}] gpu {g['out_tokens'][b]} oracle {o['out_tokens'][b]} slack {o['slack'][b]} gap {o['gap'][b]}"
            n_soft += 1
    assert n_soft <= max(1, o["accept_len"].shape[0] // 20), what
    return n_soft


WARPS = [dict(temperature=0.7), dict(top_k=1), dict(top_k=40), dict(top_p=0.9), dict(top_p=0.3),
         dict(temperature=1.3, top_k=50, top_p=0.8), dict(temperature=0.5, top_k=100000, top_p=0.95)]


def test_warpers_small(torch_cuda, oracle):
    for (B, K, V, dtype, kind, sigma) in SMALL[:7]:
        inp = synth.chain_inputs(B, K, V, dtype, kind, sigma, seed=71)
        tol = pu.rel_tol(dtype)
        for kw in WARPS:
            g = run_warped(torch_cuda, inp, 0.1, fsd.DIV_JS, fsd.SAMPLE, 5, 2, **kw)
            o = oracle.verify_chain_warped(inp["target"], inp["draft"], inp["cand"], 0.1, fsd.DIV_JS, fsd.SAMPLE, 5, 2, **kw)
            active = 0 < kw.get("top_k", 0) < V or kw.get("top_p", 1.0) < 1.0   # otherwise no selection runs
            check_warped(g, o, 0.1, tol, f"warped B={B} K={K} V={V} {dtype} {kw}", cut_active=active)
    # warpers off: the plain call, bit for bit; greedy ignores them
    inp = synth.chain_inputs(5, 9, 32000, "bf16", "zipf", (0.25, 4.0), seed=72)
    a = run_chain(torch_cuda, inp, 0.1, fsd.DIV_JS, seed=5, offset=2)
    b = run_warped(torch_cuda, inp, 0.1, fsd.DIV_JS, fsd.SAMPLE, 5, 2)
    c = run_warped(torch_cuda, inp, 0.1, fsd.DIV_JS, fsd.GREEDY, 5, 2, temperature=0.6, top_k=7, top_p=0.5)
    gr = run_chain(torch_cuda, inp, 0.1, fsd.DIV_JS, mode=fsd.GREEDY, seed=5, offset=2)
    for k in pu.CHAIN_KEYS:
        assert np.array_equal(a[k], b[k]) and np.array_equal(c[k], gr[k]), k


def test_warpers_selection_edge_cases(torch_cuda, oracle):
    """the cut is exact on every path of the selection: the short way (per-thread maxima), its
    overflow into the general path (many equal entries), top-k beyond the short way's reach, a
    nucleus that fits the candidate list and one that does not"""
    rng = np.random.default_rng(81)
    B, K, V = 6, 2, 40000
    t = (rng.standard_normal((B, K + 1, V)) * 2).astype(np.float32)
    d = (t[:, :K] + rng.standard_normal((B, K, V)).astype(np.float32) * 0.5).astype(np.float32)
    t[0] = 1.25                                   # all equal: every entry ties with the k-th largest
    t[1, :, :30000] = -3.0                        # three quarters of the row tie far below the top
    t[2] = (rng.standard_normal((K + 1, V)) * 0.05).astype(np.float32)   # nearly flat: a huge nucleus
    t[3, :, 7] += 30.0                            # one dominant entry: the nucleus is that entry
    cand = rng.integers(0, V, (B, K)).astype(np.int32)
    for dtype in ("f32", "bf16"):
        inp = dict(target=t, draft=d, cand=cand)
        if dtype == "bf16":
            inp = dict(target=synth.to_bf16_bits(t), draft=synth.to_bf16_bits(d), cand=cand)
        for kw in (dict(top_k=5), dict(top_k=512), dict(top_k=513), dict(top_k=3000), dict(top_k=20000),
                   dict(top_p=0.5), dict(top_p=0.97), dict(top_k=300, top_p=0.9),
                   dict(temperature=2.5, top_k=1000, top_p=0.99)):
            print("selection edge cases", dtype, kw, flush=True)
            g = run_warped(torch_cuda, inp, 0.1, fsd.DIV_TV, fsd.SAMPLE, 9, 4, **kw)
            o = oracle.verify_chain_warped(inp["target"], inp["draft"], inp["cand"], 0.1, fsd.DIV_TV, fsd.SAMPLE, 9, 4, **kw)
            check_warped(g, o, 0.1, pu.rel_tol(dtype), f"selection edge cases {dtype} {kw}")


def test_tree_warpers(torch_cuda, oracle):
    """the tree call with warpers: the cut and the token against the oracle on random trees; off = the plain call"""
    rng = np.random.default_rng(91)
    for (N, V, dtype) in ((10, 1000, "f32"), (33, 9000, "bf16"), (200, 512, "bf16"), (1500, 64, "f32")):
        B = 4
        parent = np.stack([np.array([-1] + [int(rng.integers(-1, j)) for j in range(1, N)], dtype=np.int32)
                           for _ in range(B)])
        t = (rng.standard_normal((B, N + 1, V)) * 2).astype(np.float32)
        d = np.empty((B, N, V), dtype=np.float32)
        for b in range(B):
            for j in range(N):
                d[b, j] = t[b, parent[b, j] + 1] + rng.standard_normal(V) * rng.uniform(0.2, 1.2)
        toks = rng.integers(0, V, (B, N)).astype(np.int32)
        if dtype == "bf16":
            t, d = synth.to_bf16_bits(t), synth.to_bf16_bits(d)
        dv = pu.to_dev(dict(target=t, draft=d, node_tokens=toks, parent=parent), ("target", "draft", "node_tokens", "parent"))
        code = fsd.BF16 if dtype == "bf16" else fsd.F32
        for kw in (dict(), dict(temperature=0.7), dict(top_k=20), dict(top_p=0.8), dict(temperature=1.4, top_k=50, top_p=0.9)):
            out = fsd.fsd_verify_tree_warped(dv["target"], dv["draft"], dv["node_tokens"], dv["parent"], N, 0.12,
                                             fsd.DIV_JS, fsd.SAMPLE, 5, 2, **kw)
            torch_cuda.cuda.synchronize()
            g = pu.host(out, pu.TREE_KEYS)
            o = oracle.verify_tree_warped(t, d, toks, parent, N, 0.12, fsd.DIV_JS, fsd.SAMPLE, 5, 2, **kw)
            what = f"tree warped N={N} V={V} {dtype} {kw}"
            assert (g["row_status"] == o["row_status"]).all(), what
            thr = fsd.debug_warp_thresholds(out, B, N, V, code).cpu().numpy()
            active = 0 < kw.get("top_k", 0) < V or kw.get("top_p", 1.0) < 1.0
            near = pu.near_threshold(o["divs"], 0.12)
            for b in range(B):
                if not (g["path_nodes"][b] == o["path_nodes"][b]).all():
                    assert near[b].any(), what
                    continue
                if active and o["slack"][b] >= 1e-5:
                    assert thr[b] == o["threshold"][b], f"{what}: cut[{b}] gpu {thr[b]} oracle {o['threshold'][b]}"
                if not (g["out_tokens"][b] == o["out_tokens"][b]).all():
                    assert o["slack"][b] < 1e-5 or o["gap"][b] < 1e-6, f"{what}: tokens[{b}]"
            if not kw:
                plain = run_tree(torch_cuda, dict(target=t, draft=d, node_tokens=toks, parent=parent), 0.12, fsd.DIV_JS, N,
                                 seed=5, offset=2)
                for k in pu.TREE_KEYS:
                    assert np.array_equal(plain[k], g[k], equal_nan=True), k


def test_config_c2_warped(torch_cuda, oracle):
    inp = synth.config_inputs("C2", seed=0)
    for kw in (dict(temperature=0.8, top_k=50, top_p=0.9), dict(top_p=0.6)):
        g = run_warped(torch_cuda, inp, 0.1, fsd.DIV_JS, fsd.SAMPLE, 3, 11, **kw)
        o = oracle.verify_chain_warped(inp["target"], inp["draft"], inp["cand"], 0.1, fsd.DIV_JS, fsd.SAMPLE, 3, 11, **kw)
        n = check_warped(g, o, 0.1, 2e-3, f"C2 warped {kw}")
        kept = [(pu.synth.bf16_bits_to_f32(inp["target"][b, o["accept_len"][b]]) * np.float32(1 / kw.get("temperature", 1.0))
                 >= o["threshold"][b]).sum() for b in range(4)]
        print("C2 warped", kw, "soft rows", n, "kept entries of the first rows", kept, flush=True)


def test_threshold_calibration(torch_cuda, oracle):
    """fsd_calibrate_threshold against the oracle's plain search: bit-exact T, same accepted share."""
    torch = torch_cuda
    rng = np.random.default_rng(7)
    for (B, K) in ((1, 1), (3, 4), (64, 8), (257, 16), (3000, 5)):
        divs = rng.gamma(0.7, 0.2, size=(B, K)).astype(np.float32)
        divs[rng.random((B, K)) < 0.1] = 0.0
        divs[rng.random((B, K)) < 0.02] = np.nan
        if B * K > 100:
            divs[1, 2] = divs[0, 0]          # duplicates
        dev = torch.from_numpy(divs).cuda()
        fr = (1.0 / (B * K), 0.1, 0.5, 0.9, 1.0) if B * K <= 2000 else (0.37,)
        for frac in fr:
            T, got = fsd.fsd_calibrate_threshold(dev, frac)
            torch.cuda.synchronize()
            oT, ofrac = oracle.calibrate_threshold(divs, float(np.float32(frac)))
            assert float(T.item()) == oT, (B, K, frac, float(T.item()), oT)
            assert abs(float(got.item()) - ofrac) < 1e-6


def test_calibrated_threshold_matches_strict_sd_share(torch_cuda, oracle):
    """App. A's recipe on the GPU: divergences of a dev batch, strict SD's accepted share, the
    threshold that reaches it, and the FSD call at that threshold accepts exactly the promised share."""
    torch = torch_cuda
    inp = synth.chain_inputs(32, 8, 32000, "bf16", "peaked", (0.25, 4.0), seed=51)
    d = pu.to_dev(inp, ("target", "draft", "cand"))
    base = fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], 1e9, fsd.DIV_JS)
    sd = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], seed=3)
    share = float(sd["accept_len"].sum().item()) / (32 * 8)
    T, frac = fsd.fsd_calibrate_threshold(base["divergences"], share)
    torch.cuda.synchronize()
    out = fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], float(T.item()), fsd.DIV_JS)
    torch.cuda.synchronize()
    got = float(out["accept_len"].sum().item()) / (32 * 8)
    assert got >= share and abs(got - float(frac.item())) < 1e-6
    oT, ofrac = oracle.calibrate_threshold(base["divergences"].cpu().numpy(), float(np.float32(share)))
    assert float(T.item()) == oT and abs(ofrac - got) < 1e-9
    print("strict SD share", share, "-> T", float(T.item()), "FSD share", got, flush=True)


def test_config_c3_full(torch_cuda, oracle):
    """full-size C3 (B=256, K=16, V=151936, float32: teams of 76 wavefronts, merged in two rounds): every
    sequence against the oracle, all three divergences."""
    c = synth.CONFIGS["C3"]
    inp = synth.config_inputs("C3", seed=0)
    print("C3 inputs ready", flush=True)
    for div in (fsd.DIV_JS, fsd.DIV_KL, fsd.DIV_TV):
        g = run_chain(torch_cuda, inp, 0.3, div, seed=5)
        assert (g["row_status"] == 0).all()
        worst, n_near = 0.0, 0
        for b0 in range(0, c["B"], 32):   # the oracle in slices of 32 sequences (its working set stays small)
            sl = slice(b0, b0 + 32)
            o = oracle.verify_chain(inp["target"][sl], inp["draft"][sl], inp["cand"][sl], 0.3, div, seed=5, seq_offset=b0)
            r = pu.check_chain({k: v[sl] for k, v in g.items()}, o, 0.3, 1e-5, f"C3 div={div} b={b0}..{b0 + 31}")
            worst = max(worst, r["max_rel_err"])
            n_near += r["near_T_rows"]
        print("C3 div", div, "max rel err", worst, "near-T rows", n_near, "accept_len histogram",
              np.bincount(g["accept_len"], minlength=c["K"] + 1), flush=True)
        assert n_near <= 2


def test_config_c4_tree_full(torch_cuda, oracle):
    inp = synth.config_inputs("C4", seed=0)
    md = int(inp["max_depth"])
    print("C4 inputs ready, max depth", md, flush=True)
    g = run_tree(torch_cuda, inp, 0.15, fsd.DIV_JS, md, seed=6)
    o = oracle.verify_tree(inp["target"], inp["draft"], inp["node_tokens"], inp["parent"], md, 0.15, fsd.DIV_JS,
                           seed=6)
    r = pu.check_tree(g, o, 0.15, 2e-3, "C4")
    print("C4", r, "path_len histogram", np.bincount(o["path_len"]), flush=True)


# ----------------------------------------------------------------------------------- trees

def test_tree_small_random(torch_cuda, oracle):
    rng = np.random.default_rng(5)
    for trial, (N, V, dtype) in enumerate([(10, 8, "f32"), (33, 1000, "bf16"), (60, 4097, "f32"), (200, 512, "bf16"),
                                           (1, 64, "f32")]):
        B = 3
        parent = np.stack([np.array([-1] + [int(rng.integers(-1, j)) for j in range(1, N)], dtype=np.int32)
                           for _ in range(B)])
        t = (rng.standard_normal((B, N + 1, V)) * 2).astype(np.float32)
        d = np.empty((B, N, V), dtype=np.float32)
        for b in range(B):
            for j in range(N):
                d[b, j] = t[b, parent[b, j] + 1] + rng.standard_normal(V) * rng.uniform(0.2, 1.2)
        toks = rng.integers(0, V, (B, N)).astype(np.int32)
        if dtype == "bf16":
            t, d = synth.to_bf16_bits(t), synth.to_bf16_bits(d)
        inp = dict(target=t, draft=d, node_tokens=toks, parent=parent)
        for T in (0.0, 0.05, 0.12, 1e9):
            for div in (fsd.DIV_JS, fsd.DIV_TV):
                print(f"tree N={N} V={V} {dtype} T={T} div={div}", flush=True)
                g = run_tree(torch_cuda, inp, T, div, N, seed=trial)
                o = oracle.verify_tree(t, d, toks, parent, N, T, div, seed=trial)
                pu.check_tree(g, o, T, pu.rel_tol(dtype), f"tree N={N} V={V} T={T} div={div}")


def test_tree_runs_of_pairs_with_idle_teams(torch_cuda, oracle):
    """At the full vocabulary a team is 13 workgroups and about 39 teams are resident; a tree call hands
    each team a run of consecutive pairs.  111 pairs make runs of 3 that use up the pairs before the
    last teams get any; 126 pairs make runs of 4 that end in a run of 2 and leave more teams idle."""
    B, V = 3, 128256
    for N, seed in ((37, 21), (42, 22)):
        inp = synth.tree_inputs(B, N, V, "bf16", 1.0, seed=seed)
        md = int(inp["max_depth"])
        for div, T in ((fsd.DIV_JS, 0.15), (fsd.DIV_TV, 0.4)):
            print(f"tree runs N={N} div={div}", flush=True)
            g = run_tree(torch_cuda, inp, T, div, md, seed=seed)
            o = oracle.verify_tree(inp["target"], inp["draft"], inp["node_tokens"], inp["parent"], md, T, div, seed=seed)
            pu.check_tree(g, o, T, pu.rel_tol("bf16"), f"tree runs N={N} div={div}")


def test_chain_shaped_tree_equals_chain(torch_cuda):
    inp = synth.chain_inputs(4, 6, 9000, "bf16", "peaked", 1.0, seed=4)
    parent = np.broadcast_to(np.arange(-1, 5, dtype=np.int32), (4, 6)).copy()
    tinp = dict(target=inp["target"], draft=inp["draft"], node_tokens=inp["cand"], parent=parent)
    for T in (0.0, 0.1, 1e9):
        c = run_chain(torch_cuda, inp, T, fsd.DIV_JS, seed=8)
        t = run_tree(torch_cuda, tinp, T, fsd.DIV_JS, 6, seed=8)
        assert (c["accept_len"] == t["path_len"]).all()
        assert (c["out_tokens"] == t["out_tokens"]).all()
        assert np.array_equal(c["divergences"], t["divergences"])


def test_tree_bad_parent_and_depth(torch_cuda, oracle):
    inp = synth.chain_inputs(2, 4, 500, "f32", "gauss2", 1.0, seed=4)
    parent = np.array([[-1, 0, 2, 1], [-1, 0, 1, 2]], dtype=np.int32)
    tinp = dict(target=inp["target"], draft=inp["draft"], node_tokens=inp["cand"], parent=parent)
    g = run_tree(torch_cuda, tinp, 1e9, fsd.DIV_JS, 2)
    o = oracle.verify_tree(inp["target"], inp["draft"], inp["cand"], parent, 2, 1e9, fsd.DIV_JS)
    assert list(o["row_status"]) == [fsd.ROW_BAD_PARENT, fsd.ROW_TOO_DEEP]
    assert list(g["row_status"]) == list(o["row_status"])
    assert (g["path_len"] == 0).all() and (g["out_tokens"] == -1).all() and (g["path_nodes"] == -1).all()


def test_reduction_kernel_shapes_agree(torch_cuda, oracle):
    """the tuning hook: every shape of the reduction kernel gives the same decisions and tokens, and
    divergences that differ only by the rounding order of the partial sums"""
    try:
        for dtype, shapes in (("bf16", (2, 4, 5)), ("f32", (2, 4, 8))):
            inp = synth.chain_inputs(3, 4, 40000, dtype, "peaked", 1.0, seed=91)
            for div in (fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV):
                fsd.debug_set_shape(0, 0)
                ref = run_chain(torch_cuda, inp, 0.1, div, seed=9, offset=1)
                o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.1, div, seed=9, offset=1)
                pu.check_chain(ref, o, 0.1, pu.rel_tol(dtype), f"default shape {dtype} div={div}")
                for nv in shapes:
                    fsd.debug_set_shape(0, nv)
                    g = run_chain(torch_cuda, inp, 0.1, div, seed=9, offset=1)
                    what = f"{dtype} div={div} slots per lane {nv}"
                    assert (g["accept_len"] == ref["accept_len"]).all() and (g["out_tokens"] == ref["out_tokens"]).all(), what
                    # (the default bfloat16 JS kernel evaluates the entropy form, the hook's shapes the
                    # pointwise one: they agree to the former's absolute error)
                    atol = 2e-6 if (dtype == "bf16" and div == fsd.DIV_JS) else 1e-7
                    assert np.allclose(g["divergences"], ref["divergences"], rtol=2e-6, atol=atol), what
    finally:
        fsd.debug_set_shape(0, 0)


def _js_inputs():
    """(name, target, draft, cand) cases for the two evaluations of bfloat16 JS: rows from nearly equal to far
    apart, masked entries on one and on both sides, bit-identical rows, a vocabulary that is no multiple of the
    slot size, the headline vocabulary, and a team of more than 64 wavefronts"""
    cases = []
    for name, (B, K, V, kind, sigma, seed) in (("V=40000 sigma 0.02..3", (3, 6, 40000, "peaked", (0.02, 3.0), 5)),
                                               ("V=4097", (2, 4, 4097, "gauss2", (0.1, 2.0), 6)),
                                               ("V=128256", (2, 3, 128256, "peaked", (0.25, 4.0), 7)),
                                               ("V=524288", (1, 2, 524288, "peaked", (0.1, 1.0), 8))):
        inp = synth.chain_inputs(B, K, V, "bf16", kind, sigma, seed=seed)
        cases.append((name, inp["target"], inp["draft"], inp["cand"]))
    inp = synth.chain_inputs(3, 4, 40000, "bf16", "peaked", 1.0, seed=9)
    t, d = inp["target"].copy(), inp["draft"].copy()
    t[0, :, 100:5000] = 0xFF80
    d[0, :, 100:5000] = 0xFF80       # masked on both sides
    d[2, :, 7000:30000] = 0xFF80     # masked by the draft only
    d[1] = t[1, :4]                  # bit-identical rows
    cases.append(("masks and identical rows", t, d, inp["cand"]))
    return cases


JS_FLOOR = 1e-3   # the library's default floor of the entropy form (nats)


def test_js_bf16_both_evaluations(torch_cuda, oracle):
    """bfloat16 JS: the entropy form alone (floor 0), the pointwise second evaluation alone (floor +inf), the
    pointwise kernel, and the default mix, each against the oracle.  The entropy form is held to its absolute
    error, everything else to the relative bar."""
    try:
        for name, t, d, cand in _js_inputs():
            o = oracle.verify_chain(t, d, cand, 0.1, fsd.DIV_JS, seed=3, offset=2)
            inp = dict(target=t, draft=d, cand=cand)
            fin = np.isfinite(o["divs"])
            for what, floor, exact in (("entropy form", 0.0, False), ("second evaluation", float("inf"), False),
                                       ("pointwise kernel", None, True), ("default", None, False)):
                prev = fsd.debug_set_js_floor(floor) if floor is not None else None
                fsd.debug_set_exact_js(exact)
                print(f"{name}: {what}", flush=True)
                g = run_chain(torch_cuda, inp, 0.1, fsd.DIV_JS, seed=3, offset=2)
                if prev is not None:
                    fsd.debug_set_js_floor(prev)
                fsd.debug_set_exact_js(False)
                assert (g["row_status"] == o["row_status"]).all(), f"{name} {what}"
                assert (np.isfinite(g["divergences"]) == fin).all(), f"{name} {what}"
                err = np.abs(g["divergences"].astype(np.float64) - o["divs"])[fin]
                print(f"   max abs error {err.max():.3e}", flush=True)
                if what == "entropy form":
                    assert err.max() <= 1e-6, f"{name} {what}: {err.max()}"
                else:
                    env = pu.Envelope("bf16")
                    pu.check_chain(g, o, 0.1, pu.rel_tol("bf16"), f"{name} {what}", envelope=env)
                if what != "entropy form" and name == "masks and identical rows":
                    assert (g["divergences"][1] == 0.0).all(), f"{name} {what}: identical rows"
    finally:
        fsd.debug_set_exact_js(False)
        fsd.debug_set_js_floor(JS_FLOOR)


def test_js_bf16_second_evaluation_in_a_tree(torch_cuda, oracle):
    """the second evaluation where pairs share target rows: a tree whose drafts are close to their targets, so
    that most nodes fall below the floor, with the floor at its default and at +inf"""
    inp = synth.tree_inputs(3, 12, 40000, "bf16", 0.05, seed=21)
    md = int(inp["max_depth"])
    o = oracle.verify_tree(inp["target"], inp["draft"], inp["node_tokens"], inp["parent"], md, 0.001, fsd.DIV_JS, seed=4)
    assert (o["divs"] < 2e-3).mean() > 0.5
    try:
        for floor in (JS_FLOOR, 2e-3, float("inf")):
            fsd.debug_set_js_floor(floor)
            g = run_tree(torch_cuda, inp, 0.001, fsd.DIV_JS, md, seed=4)
            pu.check_tree(g, o, 0.001, pu.rel_tol("bf16"), f"tree, floor {floor}", envelope=pu.Envelope("bf16"))
    finally:
        fsd.debug_set_js_floor(JS_FLOOR)


def test_js_bf16_siblings_share_their_target_row(torch_cuda, oracle):
    """a tree's children follow each other and share their parent's target row, whose exponentials and sums the
    entropy-form kernel takes over from the previous pair: wide trees (many siblings), masked entries in target
    and draft rows, and a vocabulary whose last team member owns only a few slots"""
    for V, seed in ((40000, 31), (128256, 32), (4097, 33)):
        inp = synth.tree_inputs(2, 20, V, "bf16", 1.0, seed=seed, depth=3, topk=8)
        t, d = inp["target"].copy(), inp["draft"].copy()
        t[0, :, 10:V // 3] = 0xFF80          # masked in every target row of the first tree
        d[1, ::2, V // 2:] = 0xFF80          # masked in every other draft row of the second
        md = int(inp["max_depth"])
        case = dict(inp, target=t, draft=d)
        for T in (0.05, 0.3):
            o = oracle.verify_tree(t, d, inp["node_tokens"], inp["parent"], md, T, fsd.DIV_JS, seed=5)
            g = run_tree(torch_cuda, case, T, fsd.DIV_JS, md, seed=5)
            pu.check_tree(g, o, T, pu.rel_tol("bf16"), f"siblings V={V} T={T}", envelope=pu.Envelope("bf16"))


# ------------------------------------------------------------------ random shapes

def test_random_small_shapes(torch_cuda, oracle):
    """200 random draws of (B, K, V, dtype, input kind, noise, masks, divergence, T): the chain call, and in
    turn reducible FSD, strict SD and a random tree over the same rows, each against the oracle."""
    rng = np.random.default_rng(2024)
    env = {"f32": pu.Envelope("f32"), "bf16": pu.Envelope("bf16")}
    for it in range(200):
        B, K = int(rng.integers(1, 6)), int(rng.integers(1, 7))
        V = int(rng.choice([rng.integers(1, 40), rng.integers(40, 3000), rng.integers(3000, 70000),
                            8 * rng.integers(1, 3000)]))
        dtype = str(rng.choice(["f32", "bf16"]))
        kind = str(rng.choice(["gauss2", "peaked"]))
        sigma = float(rng.choice([0.1, 0.5, 1.0, 3.0]))
        seed = int(rng.integers(0, 10**6))
        inp = synth.chain_inputs(B, K, V, dtype, kind, sigma, seed=seed)
        if rng.random() < 0.25:   # entries the draft masks
            m = rng.random(inp["draft"].shape) < 0.1
            inp["draft"][m] = 0xFF80 if dtype == "bf16" else -np.inf
        div = int(rng.choice([fsd.DIV_KL, fsd.DIV_JS, fsd.DIV_TV]))
        T = float(rng.choice([0.0, 0.01, 0.05, 0.2, 0.5, 1e9]))
        what = f"it={it} B={B} K={K} V={V} {dtype} {kind} sigma={sigma} seed={seed} div={div} T={T}"
        print(what, flush=True)
        tol = pu.rel_tol(dtype)
        g = run_chain(torch_cuda, inp, T, div, seed=seed, offset=it)
        o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], T, div, seed=seed, offset=it)
        pu.check_chain(g, o, T, tol, what, env[dtype])
        if it % 3 == 0:
            g = run_rfsd(torch_cuda, inp, T, div, seed=seed, offset=it)
            o = oracle.rfsd_verify_chain(inp["target"], inp["draft"], inp["cand"], T, div, seed=seed, offset=it)
            check_rfsd(g, o, T, tol, "reducible " + what, env[dtype])
        elif it % 3 == 1:
            d = pu.to_dev(inp, ("target", "draft", "cand"))
            out = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], seed=seed, offset=it)
            torch_cuda.cuda.synchronize()
            o = oracle.sd_verify_chain(inp["target"], inp["draft"], inp["cand"], seed=seed, offset=it)
            check_sd(pu.host(out, pu.SD_KEYS), o, "strict SD " + what)
        elif K >= 2:
            parent = np.stack([np.array([-1] + [int(rng.integers(-1, j)) for j in range(1, K)], dtype=np.int32)
                               for _ in range(B)])
            tin = dict(target=inp["target"], draft=inp["draft"], node_tokens=inp["cand"], parent=parent)
            g = run_tree(torch_cuda, tin, T, div, K, seed=seed, offset=it)
            o = oracle.verify_tree(tin["target"], tin["draft"], tin["node_tokens"], parent, K, T, div, seed=seed,
                                   offset=it)
            pu.check_tree(g, o, T, tol, "tree " + what, env[dtype])
    for dtype, e in env.items():
        e.report(f"random small shapes, {dtype} logits")
        # the rows that only meet the absolute bound are the ones drawn with little noise: a minority
        assert e.below <= 0.35 * (e.met + e.below), dtype


# ------------------------------------------------------------------ strict SD over a token tree

def run_sd_tree(torch, inp, max_depth, mode=fsd.SAMPLE, seed=0, offset=0):
    d = pu.to_dev(inp, ("target", "draft", "node_tokens", "parent"))
    out = fsd.sd_verify_tree(d["target"], d["draft"], d["node_tokens"], d["parent"], max_depth, mode, seed, offset)
    torch.cuda.synchronize()
    return pu.host(out, pu.TREESD_KEYS)


def _ratio_condition(inp, o, b, j):
    """How strongly node j's log-ratio reacts to relative errors of the probabilities it is made of.
    The first child of a context: ln p(x) - ln q(x), one unit each.  A later child is tested against
    the residual chain r <- (r - q_m)+ / Z_m of the siblings rejected before it, and a difference
    r - q_m that is small against r and q_m multiplies the errors they carry.  The kernels take the
    rows' normalisers from binary32 exponentials (about 1e-7 relative), the oracle from float64."""
    def row(a, idx):
        z = a[b, idx]
        z = synth.bf16_bits_to_f32(z) if z.dtype == np.uint16 else z
        z = z.astype(np.float64)
        e = np.exp(z - z.max())
        return e / e.sum()
    par, tok = inp["parent"][b], inp["node_tokens"][b]
    x = int(tok[j])
    p = row(inp["target"], par[j] + 1)
    cond = 1.0
    for m in range(j):
        if par[m] != par[j] or np.isnan(o["log_ratio"][b, m]):
            continue
        # sibling m was tried before j and rejected (j would not have been tried otherwise)
        q = row(inp["draft"], m)
        if p[x] - q[x] <= 0:
            return np.inf
        cond = (p[x] * cond + q[x]) / (p[x] - q[x])
        r = np.maximum(p - q, 0.0)
        if r.sum() > 0:
            p = r / r.sum()
    return cond + 1.0


def check_sd_tree(g, o, what, inp=None):
    """Paths and tokens are exact unless a test sits on its threshold (|margin| <= 1e-5 in the oracle)
    or the residual draw has a runner-up within 1e-4; log-ratios of the nodes that were tried agree to
    5e-5 (plus 5e-5 of their size).  With the inputs at hand the condition number of a node's log-ratio
    is printed where the error comes near the bar (a later sibling's can be large): a diagnostic, no
    allowance is made for it."""
    assert (g["row_status"] == o["row_status"]).all(), what
    near = np.abs(np.nan_to_num(o["margin"], nan=1.0)) <= 1e-5
    n_near = n_tie = n_cond = 0
    for b in range(o["path_len"].shape[0]):
        same = int(g["path_len"][b]) == int(o["path_len"][b]) and (g["path_nodes"][b] == o["path_nodes"][b]).all()
        if not same:
            ok = bool(near[b].any())
            if not ok and inp is not None:
                # the first node on which the two sides decided differently
                for j in range(o["log_ratio"].shape[1]):
                    tg_, to_ = not np.isnan(g["log_ratio"][b, j]), not np.isnan(o["log_ratio"][b, j])
                    if tg_ and to_ and (j in g["path_nodes"][b]) != (j in o["path_nodes"][b]):
                        ok = abs(o["margin"][b, j]) <= 1e-5
                        print(f"{what}: tree {b} node {j} decided differently, margin {o['margin'][b, j]:.3e}, "
                              f"condition number {_ratio_condition(inp, o, b, j):.3g}", flush=True)
                        break
                    if tg_ != to_:
                        break
            assert ok, f"{what}: tree {b} path gpu {g['path_nodes'][b]} oracle {o['path_nodes'][b]}"
            n_near += 1
            continue
        tried = ~np.isnan(o["log_ratio"][b])
        assert (np.isnan(g["log_ratio"][b]) == ~tried).all(), f"{what}: tree {b} tried nodes differ"
        fin = np.isfinite(o["log_ratio"][b])
        assert (np.isfinite(g["log_ratio"][b]) == fin).all(), what
        for j in np.nonzero(fin)[0]:
            gv, ov = float(g["log_ratio"][b, j]), float(o["log_ratio"][b, j])
            tol = 5e-5 + 5e-5 * abs(ov)
            if abs(gv - ov) > 0.2 * tol and inp is not None:
                # diagnostic only: how ill-conditioned the node's log-ratio is (no allowance is made for it)
                kappa = _ratio_condition(inp, o, b, int(j))
                if kappa > 1e3:
                    n_cond += 1
                    print(f"{what}: tree {b} node {j} log_ratio error {abs(gv - ov):.2e} of {tol:.2e} allowed, "
                          f"condition number {kappa:.3g}", flush=True)
            assert abs(gv - ov) <= tol, f"{what}: tree {b} node {j} log_ratio gpu {gv} oracle {ov} (allowed {tol:.2e})"
        if not (g["out_tokens"][b] == o["out_tokens"][b]).all():
            assert o["gap"][b] < 1e-4, f"{what}: tree {b} tokens gpu {g['out_tokens'][b]} oracle {o['out_tokens'][b]} gap {o['gap'][b]}"
            n_tie += 1
    assert n_near + n_tie <= max(2, o["path_len"].shape[0] // 20), what
    return dict(near=n_near, ties=n_tie, ill_conditioned=n_cond)


def _random_tree_inputs(rng, B, N, V, dtype, star=False, noise=(0.2, 1.2)):
    if star:
        parent = np.full((B, N), -1, dtype=np.int32)
    else:
        parent = np.stack([np.array([-1] + [int(rng.integers(-1, j)) for j in range(1, N)], dtype=np.int32)
                           for _ in range(B)])
    t = (rng.standard_normal((B, N + 1, V)) * 2).astype(np.float32)
    d = np.empty((B, N, V), dtype=np.float32)
    toks = np.empty((B, N), dtype=np.int32)
    for b in range(B):
        for j in range(N):
            d[b, j] = t[b, parent[b, j] + 1] + rng.standard_normal(V) * rng.uniform(*noise)
            q = np.exp(d[b, j].astype(np.float64) - d[b, j].max())
            toks[b, j] = rng.choice(V, p=q / q.sum())          # proposals come from the draft rows
    if dtype == "bf16":
        t, d = synth.to_bf16_bits(t), synth.to_bf16_bits(d)
    return dict(target=t, draft=d, node_tokens=toks, parent=parent)


def test_sd_tree_small_random(torch_cuda, oracle):
    rng = np.random.default_rng(15)
    for trial, (N, V, dtype) in enumerate([(10, 8, "f32"), (33, 1000, "bf16"), (60, 4097, "f32"), (200, 512, "bf16"),
                                           (1, 64, "f32"), (24, 9000, "bf16")]):
        inp = _random_tree_inputs(rng, 6, N, V, dtype)
        for mode in (fsd.SAMPLE, fsd.GREEDY):
            print(f"sd tree N={N} V={V} {dtype} mode={mode}", flush=True)
            g = run_sd_tree(torch_cuda, inp, N, mode, seed=trial, offset=2)
            o = oracle.sd_verify_tree(inp["target"], inp["draft"], inp["node_tokens"], inp["parent"], N, mode,
                                      seed=trial, offset=2)
            r = check_sd_tree(g, o, f"sd tree N={N} V={V} {dtype} mode={mode}", inp)
            print("   ", r, "path_len", np.bincount(o["path_len"]), flush=True)


def test_sd_tree_star_many_rejections(torch_cuda, oracle):
    """all nodes are children of the root and the drafts are far from the target: long residual chains"""
    rng = np.random.default_rng(16)
    for (N, V, dtype) in ((12, 1000, "f32"), (9, 4097, "bf16"), (16, 50000, "bf16")):
        inp = _random_tree_inputs(rng, 8, N, V, dtype, star=True, noise=(1.5, 3.0))
        print(f"sd star N={N} V={V} {dtype}", flush=True)
        g = run_sd_tree(torch_cuda, inp, 1, seed=3, offset=1)
        o = oracle.sd_verify_tree(inp["target"], inp["draft"], inp["node_tokens"], inp["parent"], 1, seed=3, offset=1)
        r = check_sd_tree(g, o, f"sd star N={N} V={V} {dtype}", inp)
        tried = (~np.isnan(o["log_ratio"])).sum(axis=1)
        print("   ", r, "nodes tried per tree", tried, flush=True)
        assert tried.max() >= 4          # the case is exercised


def test_sd_tree_chain_shaped_equals_sd_chain(torch_cuda):
    inp = synth.chain_inputs(5, 6, 9000, "bf16", "peaked", 1.0, seed=4)
    parent = np.broadcast_to(np.arange(-1, 5, dtype=np.int32), (5, 6)).copy()
    tinp = dict(target=inp["target"], draft=inp["draft"], node_tokens=inp["cand"], parent=parent)
    d = pu.to_dev(inp, ("target", "draft", "cand"))
    for mode in (fsd.SAMPLE, fsd.GREEDY):
        out = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], mode, seed=8, offset=3)
        torch_cuda.cuda.synchronize()
        c = pu.host(out, pu.SD_KEYS)
        t = run_sd_tree(torch_cuda, tinp, 6, mode, seed=8, offset=3)
        assert (c["accept_len"] == t["path_len"]).all()
        assert (c["out_tokens"] == t["out_tokens"]).all()
        for b in range(5):
            n = min(int(c["accept_len"][b]) + 1, 6)
            assert np.array_equal(c["log_ratio"][b, :n], t["log_ratio"][b, :n])
            assert np.isnan(t["log_ratio"][b, n:]).all()


def test_sd_tree_bad_input(torch_cuda, oracle):
    inp = synth.chain_inputs(3, 4, 500, "f32", "gauss2", 1.0, seed=4)
    parent = np.array([[-1, 0, 2, 1], [-1, 0, 1, 2], [-1, -1, 0, 0]], dtype=np.int32)
    toks = inp["cand"].copy()
    toks[2, 3] = 500                                              # token id out of range
    tinp = dict(target=inp["target"], draft=inp["draft"], node_tokens=toks, parent=parent)
    g = run_sd_tree(torch_cuda, tinp, 2)
    o = oracle.sd_verify_tree(inp["target"], inp["draft"], toks, parent, 2)
    assert list(o["row_status"]) == [fsd.ROW_BAD_PARENT, fsd.ROW_TOO_DEEP, fsd.ROW_BAD_TOKEN]
    assert list(g["row_status"]) == list(o["row_status"])
    assert (g["path_len"] == 0).all() and (g["out_tokens"] == -1).all() and (g["path_nodes"] == -1).all()


def test_sd_tree_bounded_wait_expires_cleanly(torch_cuda, oracle):
    """the workgroups that share a tree's passes wait for each other with a poll budget: with a budget of
    zero the call ends, and every sequence is either right or flagged FSD_ROW_INTERNAL with empty outputs"""
    rng = np.random.default_rng(17)
    inp = _random_tree_inputs(rng, 4, 12, 50000, "bf16", star=True, noise=(1.5, 3.0))
    o = oracle.sd_verify_tree(inp["target"], inp["draft"], inp["node_tokens"], inp["parent"], 1, seed=3, offset=1)
    prev = fsd.debug_set_spin_limit(0)
    try:
        g = run_sd_tree(torch_cuda, inp, 1, seed=3, offset=1)
    finally:
        fsd.debug_set_spin_limit(prev)
    # (the normalisers come from the single-pass reduction, whose finisher flags the pair it could not
    # finish: a sequence is either flagged, with empty outputs, or right)
    bad = (g["row_status"] & fsd.ROW_INTERNAL) != 0
    assert ((g["row_status"] == 0) | bad).all()
    assert (g["path_len"][bad] == 0).all() and (g["out_tokens"][bad] == -1).all() and (g["path_nodes"][bad] == -1).all()
    if (~bad).any():
        check_sd_tree({k: v[~bad] for k, v in g.items()}, {k: v[~bad] for k, v in o.items()},
                      "zero poll budget, sequences that were not flagged")
    g = run_sd_tree(torch_cuda, inp, 1, seed=3, offset=1)
    check_sd_tree(g, o, "after restoring the poll budget")


def test_random_small_shapes_warped_and_tree_sd(torch_cuda, oracle):
    """150 random draws: the chain call with a random set of warpers, and strict SD over a random tree
    (or star), each against the oracle."""
    rng = np.random.default_rng(777)
    env = {"f32": pu.Envelope("f32"), "bf16": pu.Envelope("bf16")}
    for it in range(150):
        B, K = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        V = int(rng.choice([rng.integers(2, 40), rng.integers(40, 3000), rng.integers(3000, 140000),
                            8 * rng.integers(1, 16000)]))
        dtype = str(rng.choice(["f32", "bf16"]))
        kind = str(rng.choice(["gauss2", "peaked", "zipf"]))
        seed = int(rng.integers(0, 10**6))
        inp = synth.chain_inputs(B, K, V, dtype, kind, 1.0, seed=seed)
        kw = {}
        if rng.random() < 0.6:
            kw["temperature"] = float(rng.choice([0.3, 0.7, 1.0, 1.5]))
        if rng.random() < 0.6:
            kw["top_k"] = int(rng.choice([1, 2, 10, 50, 500, 5000, 200000]))
        if rng.random() < 0.6:
            kw["top_p"] = float(rng.choice([0.1, 0.5, 0.9, 0.99, 1.0]))
        what = f"it={it} B={B} K={K} V={V} {dtype} {kind} seed={seed} {kw}"
        print(what, flush=True)
        g = run_warped(torch_cuda, inp, 0.1, fsd.DIV_JS, fsd.SAMPLE, seed, it, **kw)
        o = oracle.verify_chain_warped(inp["target"], inp["draft"], inp["cand"], 0.1, fsd.DIV_JS, fsd.SAMPLE, seed, it,
                                       **kw)
        active = 0 < kw.get("top_k", 0) < V or kw.get("top_p", 1.0) < 1.0
        check_warped(g, o, 0.1, pu.rel_tol(dtype), what, cut_active=active, envelope=env[dtype])
        N = int(rng.integers(1, 30))
        Vt = int(rng.choice([rng.integers(2, 60), rng.integers(60, 5000), rng.integers(5000, 60000)]))
        tin = _random_tree_inputs(rng, B, N, Vt, dtype, star=bool(rng.random() < 0.3), noise=(0.3, 2.5))
        g = run_sd_tree(torch_cuda, tin, N, seed=seed, offset=it)
        o = oracle.sd_verify_tree(tin["target"], tin["draft"], tin["node_tokens"], tin["parent"], N, seed=seed,
                                  offset=it)
        check_sd_tree(g, o, f"sd tree it={it} N={N} V={Vt} {dtype}", tin)
    for dtype, e in env.items():
        e.report(f"random warped shapes, {dtype} logits")
        assert e.below <= 0.35 * (e.met + e.below), dtype


def test_config_c4_strict_sd_tree(torch_cuda, oracle):
    # the second set holds a later sibling whose token has nearly the same probability under the target
    # and under the sibling rejected before it: its log-ratio is ill-conditioned (condition number 5e3),
    # and still inside the plain bar since the walk forms its probabilities from float64 arguments
    for inputs_seed, seed, offset in ((0, 6, 2), (400, 400, 3)):
        inp = synth.config_inputs("C4", seed=inputs_seed)
        md = int(inp["max_depth"])
        g = run_sd_tree(torch_cuda, inp, md, seed=seed, offset=offset)
        o = oracle.sd_verify_tree(inp["target"], inp["draft"], inp["node_tokens"], inp["parent"], md, seed=seed,
                                  offset=offset)
        r = check_sd_tree(g, o, f"C4 strict SD inputs {inputs_seed}", inp)
        print("C4 strict SD", r, "path_len histogram", np.bincount(o["path_len"]),
              "nodes tried", (~np.isnan(o["log_ratio"])).sum(axis=1), flush=True)


# ------------------------------------------------------------------------------- robustness

def test_calls_can_be_captured_in_a_graph(torch_cuda):
    """a verify call is kernel launches only (its clearing is a kernel too), so it can be recorded into a
    HIP graph; every replay, with eager calls in between, gives the eager result"""
    torch = torch_cuda
    inp = synth.chain_inputs(6, 5, 32000, "bf16", "peaked", (0.25, 2.0), seed=12)
    d = pu.to_dev(inp, ("target", "draft", "cand"))
    other = pu.to_dev(synth.chain_inputs(6, 5, 32000, "bf16", "peaked", (0.25, 2.0), seed=13), ("target", "draft", "cand"))
    eager = fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], 0.1, fsd.DIV_JS, fsd.SAMPLE, 4, 9)
    eager_sd = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], fsd.SAMPLE, 4, 9)
    torch.cuda.synchronize()
    want = pu.host(eager, pu.CHAIN_KEYS)
    want_sd = pu.host(eager_sd, pu.SD_KEYS)
    # outputs and workspaces of the recorded calls exist before the capture: nothing allocates inside it
    out = {k: torch.empty_like(v) for k, v in eager.items() if k != "_workspace"}
    out_sd = {k: torch.empty_like(v) for k, v in eager_sd.items() if k != "_workspace"}
    ws = torch.empty_like(eager["_workspace"])
    ws_sd = torch.empty_like(eager_sd["_workspace"])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # one untimed pass on the capture stream first
        fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], 0.1, fsd.DIV_JS, fsd.SAMPLE, 4, 9, out=out, workspace=ws)
        fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], fsd.SAMPLE, 4, 9, out=out_sd, workspace=ws_sd)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], 0.1, fsd.DIV_JS, fsd.SAMPLE, 4, 9, out=out, workspace=ws)
        fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], fsd.SAMPLE, 4, 9, out=out_sd, workspace=ws_sd)
    for rep in range(3):
        for k in pu.CHAIN_KEYS:
            out[k].fill_(-7)
        for k in pu.SD_KEYS:
            out_sd[k].fill_(-7)
        # the program's own eager work between the replays, on other inputs
        fsd.fsd_verify_chain(other["target"], other["draft"], other["cand"], 0.2, fsd.DIV_TV, fsd.SAMPLE, rep, rep)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, got_sd = pu.host(out, pu.CHAIN_KEYS), pu.host(out_sd, pu.SD_KEYS)
        for k in pu.CHAIN_KEYS:
            assert np.array_equal(got[k], want[k], equal_nan=True), (rep, k)
        for k in pu.SD_KEYS:
            assert np.array_equal(got_sd[k], want_sd[k], equal_nan=True), (rep, k)



def test_bounded_wait_expires_cleanly(torch_cuda, oracle):
    """with a zero poll budget a workgroup may give up waiting for its team: the kernel still ends,
    and the call either is correct throughout or flags FSD_ROW_INTERNAL on every sequence."""
    inp = synth.chain_inputs(4, 4, 128256, "bf16", "peaked", 1.0, seed=6)
    o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.1, fsd.DIV_JS)
    prev = fsd.debug_set_spin_limit(0)
    try:
        g = run_chain(torch_cuda, inp, 0.1, fsd.DIV_JS)
    finally:
        fsd.debug_set_spin_limit(prev)
    if (g["row_status"] == 0).all():
        pu.check_chain(g, o, 0.1, 2e-3, "zero poll budget, nothing expired")
    else:
        assert ((g["row_status"] & fsd.ROW_INTERNAL) != 0).all()
        assert (g["accept_len"] == 0).all() and (g["out_tokens"] == -1).all()
    g = run_chain(torch_cuda, inp, 0.1, fsd.DIV_JS)
    pu.check_chain(g, o, 0.1, 2e-3, "after restoring the poll budget")


def test_calls_without_a_clearing_kernel_on_dirty_workspaces(torch_cuda, oracle):
    """The plain calls do not launch a kernel to clear their workspace: the reduction kernel's wavefronts
    clear their own exchange words and announce themselves with the call's number.  Whatever the
    workspace held must not matter: random bytes, all ones, the words another call on other inputs
    left behind (the realistic case: valid-looking words of the wrong call), and the same again with the
    clearing kernel switched back on.  JS (entropy form), TV (pointwise, two words per member), KL
    (single pass), binary32 logits, strict SD, and a shape with several team members per pair."""
    torch = torch_cuda
    cases = [(3, 5, 40004, "bf16", "peaked", 1.0), (2, 4, 128256, "bf16", "peaked", (0.25, 4.0)),
             (2, 3, 40004, "f32", "gauss2", 0.5), (5, 2, 4097, "bf16", "zipf", 1.0)]
    try:
        for on in (True, False):
            fsd.debug_set_self_clear(on)
            for ci, (B, K, V, dtype, kind, sigma) in enumerate(cases):
                inp = synth.chain_inputs(B, K, V, dtype, kind, sigma, seed=60 + ci)
                other = synth.chain_inputs(B, K, V, dtype, kind, sigma, seed=90 + ci)
                d = pu.to_dev(inp, ("target", "draft", "cand"))
                do = pu.to_dev(other, ("target", "draft", "cand"))
                dt = fsd.BF16 if dtype == "bf16" else fsd.F32
                need = fsd.fsd_workspace_bytes(B, K, V, dt)
                ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
                gen = torch.Generator(device="cuda")
                gen.manual_seed(5 + ci)
                for div in (fsd.DIV_JS, fsd.DIV_TV, fsd.DIV_KL):
                    o = oracle.verify_chain(inp["target"], inp["draft"], inp["cand"], 0.1, div, seed=8, offset=1)
                    for dirt in ("random", "ones", "other call", "same call"):
                        print(f"self_clear={on} case {ci} div {div} workspace: {dirt}", flush=True)
                        if dirt == "random":
                            ws.random_(0, 256, generator=gen)
                        elif dirt == "ones":
                            ws.fill_(255)
                        elif dirt == "other call":
                            fsd.fsd_verify_chain(do["target"], do["draft"], do["cand"], 0.3, div, fsd.SAMPLE, 1, 2, workspace=ws)
                        out = fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], 0.1, div, fsd.SAMPLE, 8, 1, workspace=ws)
                        torch.cuda.synchronize()
                        g = pu.host(out, pu.CHAIN_KEYS)
                        pu.check_chain(g, o, 0.1, pu.rel_tol(dtype), f"{dirt} workspace, case {ci}, div {div}, self_clear={on}",
                                       envelope=pu.Envelope(dtype))
                o = oracle.sd_verify_chain(inp["target"], inp["draft"], inp["cand"], fsd.SAMPLE, seed=6, offset=3)
                for dirt in ("random", "other call"):
                    print(f"self_clear={on} case {ci} strict SD workspace: {dirt}", flush=True)
                    if dirt == "random":
                        ws.random_(0, 256, generator=gen)
                    else:
                        fsd.sd_verify_chain(do["target"], do["draft"], do["cand"], fsd.SAMPLE, seed=2, offset=9, workspace=ws)
                    out = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], fsd.SAMPLE, seed=6, offset=3, workspace=ws)
                    torch.cuda.synchronize()
                    check_sd(pu.host(out, pu.SD_KEYS), o, f"SD {dirt} workspace, case {ci}, self_clear={on}")
            # a tree (runs of consecutive pairs per team, teams without pairs at the end)
            tinp = synth.tree_inputs(3, 14, 40004, "bf16", 1.0, seed=71, depth=4, topk=4)
            toth = synth.tree_inputs(3, 14, 40004, "bf16", 1.0, seed=72, depth=4, topk=4)
            md = int(tinp["max_depth"])
            td = pu.to_dev(tinp, ("target", "draft", "node_tokens", "parent"))
            to = pu.to_dev(toth, ("target", "draft", "node_tokens", "parent"))
            need = fsd.fsd_workspace_bytes(3, 14, 40004, fsd.BF16)
            ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
            for div in (fsd.DIV_JS, fsd.DIV_TV):
                o = oracle.verify_tree(tinp["target"], tinp["draft"], tinp["node_tokens"], tinp["parent"], md, 0.15, div, seed=4)
                for dirt in ("random", "ones", "other call"):
                    print(f"self_clear={on} tree div {div} workspace: {dirt}", flush=True)
                    if dirt == "random":
                        ws.random_(0, 256)
                    elif dirt == "ones":
                        ws.fill_(255)
                    else:
                        fsd.fsd_verify_tree(to["target"], to["draft"], to["node_tokens"], to["parent"], int(toth["max_depth"]),
                                            0.3, div, fsd.SAMPLE, 9, 0, workspace=ws)
                    out = fsd.fsd_verify_tree(td["target"], td["draft"], td["node_tokens"], td["parent"], md, 0.15, div,
                                              fsd.SAMPLE, 4, 0, workspace=ws)
                    torch.cuda.synchronize()
                    pu.check_tree(pu.host(out, pu.TREE_KEYS), o, 0.15, pu.rel_tol("bf16"),
                                  f"tree, {dirt} workspace, div {div}, self_clear={on}", envelope=pu.Envelope("bf16"))
            # a warped chain call (selection kernel between the reduction and the sampler) and strict SD over a
            # tree (walk kernel with shares of its own), each after another call of its kind on other inputs
            winp = synth.chain_inputs(3, 4, 40004, "bf16", "peaked", 1.0, seed=75)
            woth = synth.chain_inputs(3, 4, 40004, "bf16", "peaked", 1.0, seed=76)
            kw = dict(temperature=0.8, top_k=40, top_p=0.9)
            need = fsd.fsd_workspace_bytes(3, 4, 40004, fsd.BF16)
            ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
            wd, wo = pu.to_dev(winp, ("target", "draft", "cand")), pu.to_dev(woth, ("target", "draft", "cand"))
            o = oracle.verify_chain_warped(winp["target"], winp["draft"], winp["cand"], 0.1, fsd.DIV_JS, fsd.SAMPLE, 5, 2, **kw)
            for dirt in ("random", "other call"):
                print(f"self_clear={on} warped chain workspace: {dirt}", flush=True)
                if dirt == "random":
                    ws.random_(0, 256)
                else:
                    fsd.fsd_verify_chain_warped(wo["target"], wo["draft"], wo["cand"], 0.3, fsd.DIV_JS, fsd.SAMPLE, 1, 1, workspace=ws, **kw)
                out = fsd.fsd_verify_chain_warped(wd["target"], wd["draft"], wd["cand"], 0.1, fsd.DIV_JS, fsd.SAMPLE, 5, 2, workspace=ws, **kw)
                torch.cuda.synchronize()
                g = pu.host(out, pu.CHAIN_KEYS)
                g["threshold"] = fsd.debug_warp_thresholds(out, 3, 4, 40004, fsd.BF16).cpu().numpy()
                check_warped(g, o, 0.1, pu.rel_tol("bf16"), f"warped, {dirt} workspace, self_clear={on}")
            rng = np.random.default_rng(17)
            sinp = _random_tree_inputs(rng, 4, 12, 9000, "bf16")
            soth = _random_tree_inputs(rng, 4, 12, 9000, "bf16")
            need = fsd.fsd_workspace_bytes(4, 12, 9000, fsd.BF16)
            ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
            sd_, so_ = (pu.to_dev(x, ("target", "draft", "node_tokens", "parent")) for x in (sinp, soth))
            o = oracle.sd_verify_tree(sinp["target"], sinp["draft"], sinp["node_tokens"], sinp["parent"], 12, fsd.SAMPLE, seed=2, offset=2)
            for dirt in ("random", "other call"):
                print(f"self_clear={on} strict SD over a tree workspace: {dirt}", flush=True)
                if dirt == "random":
                    ws.random_(0, 256)
                else:
                    fsd.sd_verify_tree(so_["target"], so_["draft"], so_["node_tokens"], so_["parent"], 12, fsd.SAMPLE, 7, 7, workspace=ws)
                out = fsd.sd_verify_tree(sd_["target"], sd_["draft"], sd_["node_tokens"], sd_["parent"], 12, fsd.SAMPLE, 2, 2, workspace=ws)
                torch.cuda.synchronize()
                check_sd_tree(pu.host(out, pu.TREESD_KEYS), o, f"sd tree, {dirt} workspace, self_clear={on}", sinp)
    finally:
        fsd.debug_set_self_clear(True)


def test_many_calls_on_one_workspace_repeat_bit_for_bit(torch_cuda):
    """1200 calls of four shapes, three divergences and strict SD, mixed, on ONE workspace that starts
    full of random bytes: every call must give, bit for bit, what the first call of its kind gave.
    (The calls clear their own exchange words while other wavefronts already run: a word of an earlier
    call taken for one of this call's would show here as a result that differs once in a while.)"""
    torch = torch_cuda
    inputs = []
    for (B, K, V, dtype) in ((16, 8, 128256, "bf16"), (7, 5, 40004, "bf16"), (33, 3, 128256, "bf16"), (5, 6, 32000, "f32")):
        inp = synth.chain_inputs(B, K, V, dtype, "peaked", (0.25, 4.0), seed=7)
        d = pu.to_dev(inp, ("target", "draft", "cand"))
        d["code"] = fsd.BF16 if dtype == "bf16" else fsd.F32
        inputs.append(d)
    need = max(fsd.fsd_workspace_bytes(d["target"].shape[0], d["draft"].shape[1], d["target"].shape[2], d["code"]) for d in inputs)
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    ws.random_(0, 256)
    ref, bad = {}, []
    for i in range(1200):
        d = inputs[(i * 7 + i // 5) % len(inputs)]
        div = (fsd.DIV_JS, fsd.DIV_TV, fsd.DIV_KL)[(i // 3) % 3]
        if i % 4 == 3:
            out = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], fsd.SAMPLE, seed=3, offset=5, workspace=ws)
            keys, tag = ("accept_len", "out_tokens", "log_ratio", "row_status"), (id(d), "sd")
        else:
            out = fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], 0.1, div, fsd.SAMPLE, seed=3, offset=5, workspace=ws)
            keys, tag = ("accept_len", "out_tokens", "divergences", "row_status"), (id(d), div)
        got = {k: out[k].clone() for k in keys}
        if tag not in ref:
            torch.cuda.synchronize()
            assert int(got["row_status"].abs().max()) == 0
            ref[tag] = got
        else:
            for k in keys:
                a, b = got[k], ref[tag][k]
                if a.dtype.is_floating_point:
                    a, b = a.view(torch.int32 if a.element_size() == 4 else torch.int64), b.view(torch.int32 if b.element_size() == 4 else torch.int64)
                if not torch.equal(a, b):
                    bad.append((i, tag[1], k))
    torch.cuda.synchronize()
    assert not bad, bad[:10]
