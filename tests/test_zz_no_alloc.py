"""seer_accept_static -- the entry point for callers that cannot allocate -- against seer_accept, through
the C ABI: bit for bit the same four results, on two calls in a row, the second with a smaller input
(the shared scratch array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2511_14617_amd import workloads as W
from gpu_util import accept_device_inputs


def _both(cfg, seed, parent=None):
    from paper_2511_14617_amd import binding
    inp = W.make_accept_inputs(cfg, seed=seed, tree_parent=parent)
    e = accept_device_inputs(inp)
    want = binding.seer_accept(e["logits"], e["draft_tokens"], e["tree_parent"])
    B, T = cfg.B, cfg.T
    out = (torch.full((B,), -7, dtype=torch.int32, device="cuda"), torch.full((B, T), -7, dtype=torch.int32, device="cuda"),
           torch.full((B,), -7, dtype=torch.int32, device="cuda"), torch.full((B, T), -7, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = binding.seer_accept_static(e["logits"], e["draft_tokens"], e["tree_parent"], out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for g, w, name in zip(got, want, ("accepted_len", "accepted_path", "bonus_token", "target_argmax")):
        assert torch.equal(g, w), name
    assert np.array_equal(got[0].cpu().numpy(), inp.planted_len)


def test_static_entry_point_argument_errors_and_limit_before_any_hip_call():
    """No GPU needed: shape, pointer and size-limit errors come back before the library touches the device."""
    from paper_2511_14617_amd import binding as b
    lib = b.load_library()
    fake = 0x1000

    def run(B=4, T=5, V=1000, logits=fake, draft=fake, alen=fake, path=fake, tgt=fake):
        return lib.seer_accept_static(logits, draft, None, B, T, V, alen, path, None, tgt, None)

    assert run(T=0) == b.SEER_ESHAPE
    assert run(T=65) == b.SEER_ESHAPE
    assert run(V=0) == b.SEER_EINVAL
    assert run(B=-1) == b.SEER_EINVAL
    assert run(logits=None) == b.SEER_EINVAL
    assert run(tgt=None) == b.SEER_EINVAL
    assert run(logits=fake + 2) == b.SEER_EALIGN
    assert run(B=4096, T=64, V=16385) == b.SEER_ELIMIT            # 524 288 pairs
    assert run(B=b.SEER_ACCEPT_STATIC_MAX_PAIRS + 1, T=1, V=5) == b.SEER_ELIMIT
    assert "fixed-size" in b.seer_strerror(b.SEER_ELIMIT)


@pytest.mark.gpu
def test_static_scratch_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    from paper_2511_14617_amd import binding
    big = W.CONFIGS[5].scaled(B=24, V=152064)                 # tree, 792 rows x 10 chunks
    parent = W.multipath_parent(big.B, big.tree[0], big.tree[1], np.random.default_rng(5), 0.25)
    _both(big, 11, parent)
    small = W.CONFIGS[2].scaled(B=5, V=50001)                 # chain, fewer rows, fewer and ragged chunks
    _both(small, 12)
    _both(W.CONFIGS[1], 13)                                   # one chunk per row
    # beyond the fixed array: a clear error, nothing launched
    B, T, V = 4096, 64, 16385
    assert B * T * 2 > binding.SEER_ACCEPT_STATIC_MAX_PAIRS
    lib = binding.load_library()
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    rc = lib.seer_accept_static(one.data_ptr(), one.data_ptr(), None, B, T, V, one.data_ptr(), one.data_ptr(), None,
                                one.data_ptr(), None)
    assert rc == binding.SEER_ELIMIT
