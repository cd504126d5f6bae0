"""GPU parity for seer_accept: bit-exact against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_14617_amd import workloads as W
from gpu_util import accept_device_inputs

pytestmark = pytest.mark.gpu


def _check(inp, parent_np=None):
    from paper_2511_14617_amd import binding
    d = accept_device_inputs(inp)
    alen, path, bonus, tgt = binding.seer_accept(d["logits"], d["draft_tokens"], d["tree_parent"])
    torch.cuda.synchronize()
    ra, rp, rb, rt = oracle.verify_accept(inp.logits, inp.draft_tokens, inp.tree_parent)
    assert np.array_equal(tgt.cpu().numpy(), rt)
    assert np.array_equal(alen.cpu().numpy(), ra)
    assert np.array_equal(path.cpu().numpy(), rp)
    assert np.array_equal(bonus.cpu().numpy(), rb)
    return ra


def test_tiny_chain_config():
    inp = W.make_accept_inputs(W.CONFIGS[1])
    got = _check(inp)
    assert np.array_equal(got, inp.planted_len)


@pytest.mark.parametrize("V", [1, 7, 1000, 1001, 8192, 8193, 152064, 163840])
def test_chain_various_vocab_sizes(V):
    cfg = W.CONFIGS[2].scaled(B=6, V=V)
    inp = W.make_accept_inputs(cfg, seed=77 + V)
    got = _check(inp)
    if V > 16:
        assert np.array_equal(got, inp.planted_len)


def test_tree_with_duplicates_and_padding():
    cfg = W.CONFIGS[5].scaled(B=24, V=30011)
    rng = np.random.default_rng(4)
    parent = W.multipath_parent(cfg.B, 4, 8, rng, dedup_fraction=0.4)
    inp = W.make_accept_inputs(cfg, tree_parent=parent)
    got = _check(inp)
    assert np.array_equal(got, inp.planted_len)


def test_random_small_vocab_trees_unplanted():
    """Tiny vocabulary: many accidental matches, ties between paths, duplicate siblings."""
    rng = np.random.default_rng(8)
    B, T, V = 300, 13, 3
    cfg = W.CONFIGS[5].scaled(B=B, T=T, V=V, tree=(3, 4))
    parent = W.multipath_parent(B, 3, 4, rng, dedup_fraction=0.5)
    logits = rng.integers(-2, 3, size=(B, T, V)).astype(np.float32)   # ties inside rows too
    draft = rng.integers(0, V, size=(B, T)).astype(np.int32)
    inp = W.AcceptInputs(cfg, logits, draft, parent, np.zeros(B, np.int32), np.zeros((B, T), np.int32))
    got = _check(inp)
    assert got.max() >= 3


def test_argmax_edge_cases():
    from paper_2511_14617_amd import binding
    V = 20000
    rows = 12
    x = np.full((1, rows, V), -np.inf, dtype=np.float32)
    x[0, 1, 0] = 1.0
    x[0, 2, V - 1] = 1.0
    x[0, 3, [63, 64, 255, 256, 1023, 1024, 8191, 8192, 16383, 16384]] = 2.0   # equal maxima over lane/wave/chunk seams
    x[0, 4, [8192, 16384]] = 3.0
    x[0, 5, :] = -0.0
    x[0, 5, 9000] = 0.0
    x[0, 6, :] = np.linspace(-1, 1, V, dtype=np.float32)
    x[0, 7, :] = np.linspace(1, -1, V, dtype=np.float32)
    x[0, 8, 8191] = 5.0
    x[0, 9, 16384] = -1e30
    x[0, 10, :] = 7.0
    x[0, 11, 19999] = np.inf
    want = [0, 0, V - 1, 63, 8192, 0, V - 1, 0, 8191, 16384, 0, 19999]
    assert oracle.argmax(x)[0].tolist() == want
    draft = torch.zeros((1, rows), dtype=torch.int32, device="cuda")
    alen, path, bonus, tgt = binding.seer_accept(torch.from_numpy(x).cuda(), draft, None)
    assert tgt.cpu().numpy()[0].tolist() == want


def test_unaligned_logits_base_takes_the_scalar_path():
    from paper_2511_14617_amd import binding
    rng = np.random.default_rng(3)
    B, T, V = 3, 4, 4096
    buf = torch.zeros(B * T * V + 1, dtype=torch.float32, device="cuda")
    host = rng.standard_normal((B, T, V)).astype(np.float32)
    view = buf[1:].view(B, T, V)
    view.copy_(torch.from_numpy(host))
    assert view.data_ptr() % 16 != 0
    draft = torch.zeros((B, T), dtype=torch.int32, device="cuda")
    _, _, _, tgt = binding.seer_accept(view, draft, None)
    assert np.array_equal(tgt.cpu().numpy(), oracle.argmax(host))


def test_gamma_zero_and_empty_batch():
    from paper_2511_14617_amd import binding
    rng = np.random.default_rng(1)
    host = rng.standard_normal((5, 1, 777)).astype(np.float32)
    alen, path, bonus, tgt = binding.seer_accept(torch.from_numpy(host).cuda(),
                                                 torch.zeros((5, 1), dtype=torch.int32, device="cuda"), None)
    assert alen.cpu().tolist() == [0] * 5 and path.cpu().tolist() == [[0]] * 5
    assert np.array_equal(bonus.cpu().numpy(), np.argmax(host[:, 0], axis=-1))
    e = binding.seer_accept(torch.zeros((0, 3, 10), device="cuda"), torch.zeros((0, 3), dtype=torch.int32,
                                                                               device="cuda"), None)
    assert e[0].numel() == 0
