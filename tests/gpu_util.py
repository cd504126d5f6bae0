"""Helpers for the GPU parity tests: the stated tolerance, and a record of how much of it was used."""
import json
import os

import numpy as np
import torch

from paper_2511_14617_amd.device_inputs import (  # noqa: F401  (re-exported for the tests)
    accept_device_inputs,
    attention_device_inputs,
    bf16_tensor,
)

ATOL, RTOL = 2e-3, 1e-2   # |gpu - ref| <= ATOL + RTOL*|ref|, the bar for bf16-in / fp32-accumulate attention

# every attention comparison of a test session: (what, worst err / plain bound, fraction outside the plain
# bound, normalised rms error); written to the file SEER_MARGIN_LOG names, if set, when the session ends
MARGINS = []


def attention_margin(got: np.ndarray, ref: np.ndarray) -> dict:
    """How much of the stated tolerance |gpu - ref| <= ATOL + RTOL*|ref| a result uses."""
    err = np.abs(got - ref)
    plain = ATOL + RTOL * np.abs(ref)
    if not err.size:
        return {"worst_over_plain": 0.0, "frac_outside_plain": 0.0, "nrms": 0.0, "max_err": 0.0, "max_ref": 0.0, "n": 0}
    return {"worst_over_plain": float((err / plain).max()), "frac_outside_plain": float((err > plain).mean()),
            "nrms": float(np.sqrt((err ** 2).mean()) / max(np.sqrt((ref ** 2).mean()), 1e-300)),
            "max_err": float(err.max()), "max_ref": float(np.abs(ref).max()), "n": int(err.size)}


def record_margin(what: str, m: dict) -> None:
    MARGINS.append(dict(m, what=what))
    print("[margin] %-48s worst err/plain bound %.3f, outside the plain bound %.2e of %d, nrms %.2e" % (
        what, m["worst_over_plain"], m["frac_outside_plain"], m["n"], m["nrms"]), flush=True)


def dump_margins() -> None:
    path = os.environ.get("SEER_MARGIN_LOG")
    if path and MARGINS:
        with open(path, "w") as f:
            json.dump(MARGINS, f, indent=1)


def assert_attention_close(gpu_bf16: torch.Tensor, ref: np.ndarray, what: str = "", hardened: bool = False,
                           ref_abs: np.ndarray = None):
    """The stated bar, elementwise: |gpu - ref| <= ATOL + RTOL*|ref|.  Returns the worst err / bound.
    See check_attention_values for `hardened` and `ref_abs`."""
    got = gpu_bf16.float().cpu().numpy().astype(np.float64)
    return check_attention_values(got, ref, what, hardened, ref_abs)


def check_attention_values(got: np.ndarray, ref: np.ndarray, what: str = "", hardened: bool = False,
                           ref_abs: np.ndarray = None):
    """|got - ref| <= ATOL + RTOL*|ref| elementwise on fp64 arrays (all outputs, or sampled rows).

    `ref_abs` (hardened inputs only) names a STATED DEVIATION from that bar, not a part of it: the kernels
    round the probabilities to bf16 before the P.V matrix product (relative error <= 2^-9 each), which can
    move the numerator by up to 2^-9 * sum_j p_j |v_j| = 2^-9 * ref_abs.  Where ref_abs is given, an element
    may exceed the plain bound by at most that term, at most 0.1 % of the elements may do so, and how far
    and how many is printed and recorded (see MARGINS) for every comparison.
    """
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), what + ": non-finite output"
    m = attention_margin(got, ref)
    record_margin(what, m)
    err = np.abs(got - ref)
    plain = ATOL + RTOL * np.abs(ref)
    bound = plain if ref_abs is None else plain + 2.0 ** -9 * ref_abs
    worst = float((err / bound).max()) if err.size else 0.0
    assert worst <= 1.0, "%s: max err/bound = %.3f (max |err| %.3e, max |ref| %.3e)" % (
        what, worst, m["max_err"], m["max_ref"])
    if ref_abs is not None and err.size:
        assert m["frac_outside_plain"] <= 1e-3, "%s: %.5f of the elements are outside the plain bound" % (
            what, m["frac_outside_plain"])
    if hardened and err.size:
        # on inputs whose outputs are O(1) the error must also be small relative to the signal
        assert m["nrms"] < 6e-3, "%s: normalised rms error %.3e" % (what, m["nrms"])
        assert m["max_err"] / m["max_ref"] < 1e-2, what + ": max error vs max signal"
        assert m["max_ref"] > 0.2, what + ": hardened inputs should give O(1) outputs"
    return worst
