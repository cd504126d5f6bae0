"""Helpers for the GPU parity tests: host arrays -> device tensors, the stated tolerance."""
import numpy as np
import torch

ATOL, RTOL = 2e-3, 1e-2   # |gpu - ref| <= ATOL + RTOL*|ref|, the bar for bf16-in / fp32-accumulate attention


def bf16_tensor(bits: np.ndarray, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def attention_device_inputs(inp, device="cuda"):
    d = dict(
        q=bf16_tensor(inp.q, device),
        k_pages=bf16_tensor(inp.k_pages, device),
        v_pages=None if inp.v_pages is None else bf16_tensor(inp.v_pages, device),
        block_table=torch.from_numpy(inp.block_table).to(device),
        ctx_len=torch.from_numpy(inp.ctx_len).to(device),
        tree_mask=None if inp.tree_mask is None else torch.from_numpy(inp.tree_mask.view(np.int64)).to(device),
    )
    return d


def accept_device_inputs(inp, device="cuda"):
    return dict(
        logits=torch.from_numpy(inp.logits).to(device),
        draft_tokens=torch.from_numpy(inp.draft_tokens).to(device),
        tree_parent=None if inp.tree_parent is None else torch.from_numpy(inp.tree_parent).to(device),
    )


def assert_attention_close(gpu_bf16: torch.Tensor, ref: np.ndarray, what: str = "", hardened: bool = False,
                           ref_abs: np.ndarray = None):
    """Elementwise |gpu - ref| <= ATOL + RTOL*|ref|.

    On hardened inputs (values O(1), peaked softmax) the probabilities that feed the P.V matrix
    product are rounded to bf16, each with relative error <= 2^-9, so the numerator can move by up to
    2^-9 * sum_j p_j |v_j|.  `ref_abs` is that sum (the oracle run on |V|); when given, it widens
    the bound by exactly this term, and the plain bound must still hold for 99.9 % of the elements.
    """
    got = gpu_bf16.float().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), what + ": non-finite output"
    err = np.abs(got - ref)
    plain = ATOL + RTOL * np.abs(ref)
    bound = plain if ref_abs is None else plain + 2.0 ** -9 * ref_abs
    worst = float((err / bound).max()) if err.size else 0.0
    assert worst <= 1.0, "%s: max err/bound = %.3f (max |err| %.3e, max |ref| %.3e)" % (
        what, worst, err.max(), np.abs(ref).max())
    if ref_abs is not None and err.size:
        frac = float((err <= plain).mean())
        assert frac >= 0.999, "%s: only %.5f of the elements are inside the plain bound" % (what, frac)
    if hardened and err.size:
        # on inputs whose outputs are O(1) the error must also be small relative to the signal
        nrms = float(np.sqrt((err ** 2).mean()) / np.sqrt((ref ** 2).mean()))
        assert nrms < 6e-3, "%s: normalised rms error %.3e" % (what, nrms)
        assert err.max() / np.abs(ref).max() < 1e-2, what + ": max error vs max signal"
        assert np.abs(ref).max() > 0.2, what + ": hardened inputs should give O(1) outputs"
    return worst
