"""GPU parity, through the C ABI, for the calls around the verify step: acceptance under sampling
(bit-exact drawn tokens and acceptance against the CPU oracle's reproducible Gumbel-max draw) and the
commit of the accepted path (bit-exact pools, lengths and emitted tokens)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_14617_amd import workloads as W
from gpu_util import accept_device_inputs, attention_device_inputs

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ sampling
def _check_sampled(logits, draft, parent, tau, seed):
    from paper_2511_14617_amd import binding
    dev = "cuda"
    lg, dr = torch.from_numpy(logits).to(dev), torch.from_numpy(draft).to(dev)
    pa = None if parent is None else torch.from_numpy(parent).to(dev)
    alen, path, bonus, tok = binding.seer_accept_sampled(lg, dr, pa, tau, seed)
    torch.cuda.synchronize()
    drawn = oracle.argmax_sampled(logits, tau, seed)
    assert np.array_equal(tok.cpu().numpy(), drawn), "drawn tokens differ from the oracle's"
    ra, rp, rb = oracle.accept(drawn, draft, parent)
    assert np.array_equal(alen.cpu().numpy(), ra)
    assert np.array_equal(path.cpu().numpy(), rp)
    assert np.array_equal(bonus.cpu().numpy(), rb)
    return drawn, ra


@pytest.mark.parametrize("V,tau", [(1, 1.0), (7, 0.8), (1001, 1.0), (8192, 0.8), (8193, 1.0), (152064, 0.8),
                                   (163840, 1.0)])
def test_sampled_tokens_bit_exact(V, tau):
    cfg = W.CONFIGS[2].scaled(B=5, V=V)
    inp = W.make_accept_inputs(cfg, seed=300 + V)
    logits = inp.logits.copy()
    logits[..., : max(V // 50, 0)] = -np.inf                 # masked vocabulary entries are never drawn
    if V > 100:
        logits[0, 0, :] = -np.inf                            # a fully masked row resolves to token 0
    drawn, _ = _check_sampled(logits, inp.draft_tokens, None, tau, seed=0x1234567890ABCDEF + V)
    if V > 100:
        assert drawn[0, 0] == 0 and (drawn.reshape(-1)[1:] >= V // 50).all()


@pytest.mark.parametrize("case", ["peaked", "wide", "equal", "huge", "huge_tau", "nan_inf", "near_ties", "late_winner"])
def test_sampled_tokens_bit_exact_where_the_scan_skips_or_must_not(case):
    """The sampled scan skips the logarithms of elements whose upper bound lies below a value already met.  Shapes
    of logits that exercise it: a peaked row (nearly everything is skipped), a wide one (little is), equal logits
    (the noise alone decides; ties in the perturbed values resolve to the lowest index as in the oracle), magnitudes
    beyond the range in which the bound's roundings are covered (exact path), NaN and infinities, values within
    the bound's slack of one another, and a winner that sits at the very end of the row."""
    rng = np.random.default_rng(hash(case) % 1000)
    B, T, V = 3, 4, 40000
    tau = 0.8
    logits = rng.standard_normal((B, T, V)).astype(np.float32)
    if case == "peaked":
        logits *= 0.1
        logits[..., 777] = 30.0
    elif case == "wide":
        logits *= 12.0
    elif case == "equal":
        logits[:] = 1.25
    elif case == "huge":
        logits *= 3.0e5
        logits[1] = np.float32(2.0e5) + rng.standard_normal((T, V)).astype(np.float32) * 4.0
    elif case == "huge_tau":
        tau = 1.0e-5
    elif case == "nan_inf":
        logits[0, 0, 1::7] = np.nan                   # (not slot 0: a NaN there is the oracle's starting value)
        logits[0, 1, ::5] = -np.inf
        logits[0, 2, 123] = np.inf
        logits[1, 0, :] = np.nan
        logits[2, 3, 5:] = -np.inf
    elif case == "near_ties":
        logits[:] = (rng.integers(0, 3, size=(B, T, V)) * 0.02).astype(np.float32)
    elif case == "late_winner":
        logits *= 0.5
        logits[..., V - 1] = 25.0
    draft = rng.integers(0, V, size=(B, T)).astype(np.int32)
    for seed in (1, 0xFEDCBA9876543210):
        _check_sampled(logits, draft, None, tau, seed)


def test_sampled_acceptance_with_drafts_planted_on_the_draws():
    """Drafts that follow the drawn tokens down to a planted depth are accepted to exactly that depth,
    on a multi-path tree with a flat distribution (temperature matters: most draws are not the argmax)."""
    cfg = W.CONFIGS[5].scaled(B=40, V=5003)
    rng = np.random.default_rng(12)
    parent = W.multipath_parent(cfg.B, 4, 8, rng, dedup_fraction=0.3)
    logits = rng.normal(size=(cfg.B, cfg.T, cfg.V)).astype(np.float32)
    seed, tau = 99, 0.8
    drawn = oracle.argmax_sampled(logits, tau, seed)
    assert (drawn != logits.argmax(-1)).mean() > 0.9
    draft = rng.integers(0, cfg.V, size=(cfg.B, cfg.T)).astype(np.int32)
    planted = np.zeros(cfg.B, np.int32)
    for b in range(cfg.B):
        leaf = int(rng.integers(1, cfg.T))
        while parent[b, leaf] == -2:
            leaf = int(rng.integers(1, cfg.T))
        chain = []
        t = leaf
        while t > 0:
            chain.append(t)
            t = int(parent[b, t])
        chain = chain[::-1]
        keep = int(rng.integers(0, len(chain) + 1))
        for t in chain[:keep]:
            draft[b, t] = drawn[b, parent[b, t]]
        planted[b] = keep
    _, alen = _check_sampled(logits, draft, parent, tau, seed)
    assert (alen >= planted).all() and (alen == planted).mean() > 0.9    # (a random token can match by chance)


def test_sampled_draws_follow_the_softmax():
    """Frequencies of the GPU's draws over 60 000 rows against softmax(logits / tau)."""
    from paper_2511_14617_amd import binding
    logits = np.array([1.3, -0.2, 0.0, 2.1, -1.7, 0.4, 0.9, -0.5], np.float32)
    B, T, tau = 1000, 60, 0.8
    lg = torch.from_numpy(np.tile(logits, (B, T, 1))).cuda()
    draft = torch.zeros((B, T), dtype=torch.int32, device="cuda")
    _, _, _, tok = binding.seer_accept_sampled(lg, draft, None, tau, 4242)
    counts = np.bincount(tok.cpu().numpy().reshape(-1), minlength=logits.size)
    p = np.exp(logits.astype(np.float64) / tau)
    p /= p.sum()
    N = B * T
    assert ((counts - N * p) ** 2 / (N * p)).sum() < 29.9     # 99.99 % quantile, 7 degrees of freedom


# -------------------------------------------------------------------- commit
def _commit_case(cfg, seed, parent_kind):
    inp = W.make_attention_inputs(cfg, seed=cfg.seed + seed, values="peaked")
    acc = W.make_accept_inputs(cfg, seed=cfg.seed + seed, tree_parent=inp.tree_parent if parent_kind == "tree" else None)
    alen, path, bonus, _ = oracle.verify_accept(acc.logits, acc.draft_tokens, acc.tree_parent)
    return inp, acc, alen, path, bonus


def _run_commit(inp, acc, alen, path, bonus, with_tokens=True):
    from paper_2511_14617_amd import binding
    d = attention_device_inputs(inp)
    n = d["ctx_len"].clone()
    k, v = d["k_pages"].clone(), None if d["v_pages"] is None else d["v_pages"].clone()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kw = {}
    if with_tokens:
        kw = dict(draft_tokens=torch.from_numpy(acc.draft_tokens).cuda(), bonus_token=torch.from_numpy(bonus).cuda())
    res = binding.seer_kv_commit(k, v, d["block_table"], n, torch.from_numpy(alen).cuda(),
                                 torch.from_numpy(path).cuda(), status=status, **kw)
    torch.cuda.synchronize()
    return k, v, n, status, res


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


CASES = {
    "tree_T33": (W.CONFIGS[5].scaled(B=9, group_size=3, ctx=("uniform", 33, 900), shared_prefix=0), "tree"),
    "tree_T13_small_pages": (W.CONFIGS[5].scaled(B=7, group_size=7, T=13, tree=(3, 4), page_size=16, Hq=8, Hkv=4,
                                                ctx=("uniform", 13, 60), shared_prefix=0), "tree"),
    "chain_T9": (W.CONFIGS[2].scaled(B=6, group_size=3, ctx=("uniform", 9, 500), shared_prefix=0), "chain"),
    "mla_tree": (W.CONFIGS[4].scaled(B=5, Hq=8, T=9, tree=(2, 4), ctx=("uniform", 9, 700)), "tree"),
    "d256_page32": (W.CONFIGS[1].scaled(Hq=8, Hkv=2, Dqk=256, Dv=256, page_size=32, T=9, tree=(2, 4), B=4,
                                        ctx=("uniform", 9, 400)), "tree"),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_commit_bit_exact(name):
    cfg, kind = CASES[name]
    inp, acc, alen, path, bonus = _commit_case(cfg, 5, kind)
    rk, rv, rn = oracle.kv_commit(inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, alen, path)
    rem, rnem = oracle.emitted_tokens(acc.draft_tokens, alen, path, bonus)
    k, v, n, status, (em, nem) = _run_commit(inp, acc, alen, path, bonus)
    assert int(status.item()) == 0
    assert np.array_equal(_bits(k), rk)
    if rv is not None:
        assert np.array_equal(_bits(v), rv)
    assert np.array_equal(n.cpu().numpy(), rn)
    assert np.array_equal(em.cpu().numpy(), rem) and np.array_equal(nem.cpu().numpy(), rnem)
    if kind == "tree":
        assert not np.array_equal(rk, inp.k_pages)            # the case does move rows


def test_commit_then_decode_matches_the_verify_output_at_the_winner():
    """Attention kernel over the committed cache (T = 1, the winner's query) against the verify pass's
    output at the winner: both from the GPU path, tied together by the oracle's pinned identity."""
    from paper_2511_14617_amd import binding
    cfg, kind = CASES["tree_T33"]
    inp, acc, alen, path, bonus = _commit_case(cfg, 6, kind)
    d = attention_device_inputs(inp)
    out_tree = binding.seer_verify_attention(d["q"], d["k_pages"], d["v_pages"], d["block_table"], d["ctx_len"],
                                             d["tree_mask"], inp.scale).float().cpu().numpy()
    k, v, n, status, _ = _run_commit(inp, acc, alen, path, bonus, with_tokens=False)
    winner = path[np.arange(cfg.B), alen]
    q1 = d["q"][torch.arange(cfg.B), torch.from_numpy(winner).long().cuda()][:, None].contiguous()
    out_seq = binding.seer_verify_attention(q1, k, v, d["block_table"], n, None, inp.scale).float().cpu().numpy()
    ref = out_tree[np.arange(cfg.B), winner]
    assert np.abs(out_seq[:, 0] - ref).max() <= 2e-3 + 1e-2 * np.abs(ref).max()


def test_commit_reports_bad_requests_and_leaves_them():
    cfg, kind = CASES["tree_T13_small_pages"]
    inp, acc, alen, path, bonus = _commit_case(cfg, 7, kind)
    bad_path = path.copy()
    bad_len = alen.copy()
    bad_path[1, 0] = 2                    # does not start at the root
    bad_len[2] = cfg.T                    # longer than the draft
    bad_ctx = inp.ctx_len.copy()
    bad_ctx[3] = cfg.T - 1                # shorter than the verify slots
    # node ids far outside the T slots (garbage, huge, negative): reported, and never used as an index
    bad_len[4] = max(int(bad_len[4]), 2)
    bad_path[4, 1] = 0x3FFFFFF0
    bad_len[5] = max(int(bad_len[5]), 2)
    bad_path[5, 1], bad_path[5, 2] = 1, -0x40000000
    inp2 = inp.__class__(**{**inp.__dict__, "ctx_len": bad_ctx})
    rk, rv, rn = oracle.kv_commit(inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, alen, path)
    k, v, n, status, _ = _run_commit(inp2, acc, bad_len, bad_path, bonus, with_tokens=False)
    assert int(status.item()) == (1 | 4)
    got_n = n.cpu().numpy()
    for b in (1, 2, 3, 4, 5):
        assert got_n[b] == bad_ctx[b]
    ok = [b for b in range(cfg.B) if b not in (1, 2, 3, 4, 5)]
    assert np.array_equal(got_n[ok], rn[ok])
