"""Online acceptance statistics (Section 3.4.2: the per-position acceptance probabilities that Algorithm 1 reads are
collected online; Section 3.4.1: alpha = E(beta), expected tokens per step (1 - alpha^(gamma+1)) / (1 - alpha)).
Pins for the oracle -- hand-counted examples, identities that hold for any input, a second vectorised count,
planted acceptance probabilities, the expected-tokens law -- and the library's host function against it."""
import os

import numpy as np
import pytest

from oracle import stats_oracle as so

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _golden():
    blocks, cur = [], None
    for line in open(os.path.join(ROOT, "tests", "golden", "acceptance_stats_worked_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        kind, rest = line.split(None, 1)
        if kind == "T":
            cur = {"T": int(rest), "req": []}
            blocks.append(cur)
        elif kind == "req":
            a, path, par = [x.strip() for x in rest.split("|")]
            cur["req"].append((int(a), [int(x) for x in path.split()], None if par == "chain" else [int(x) for x in par.split()]))
        elif kind == "want":
            cur["want"] = [[int(x) for x in part.split()] for part in rest.split("|")]
    return blocks


@pytest.mark.parametrize("block", _golden())
def test_oracle_reproduces_the_hand_counted_examples(block):
    T = block["T"]
    counts = [[0] * T for _ in range(3)]
    for a, path, par in block["req"]:      # one request at a time: chains and trees mix in a block
        so.acceptance_counts([a], [path], None if par is None else [par], T, counts)
    assert counts == block["want"]


def _random_step(rng, B, T, top_k):
    """Random draft trees (level by level, top_k members per level at most, padded slots) and a random root path each."""
    parent = np.full((B, T), -2, dtype=np.int64)
    a = np.zeros(B, dtype=np.int64)
    path = np.full((B, T), -1, dtype=np.int64)
    for b in range(B):
        parent[b, 0] = 0
        level, t = [0], 1
        while t < T and level:
            nxt = []
            for _ in range(int(rng.integers(1, top_k + 1))):
                if t >= T:
                    break
                parent[b, t] = int(rng.choice(level))
                nxt.append(t)
                t += 1
            level = nxt if rng.random() < 0.85 else []
        # walk down from the root, stopping at random
        path[b, 0], v, n = 0, 0, 0
        while True:
            kids = [s for s in range(1, T) if parent[b, s] == v and s > v]
            if not kids or rng.random() < 0.3:
                break
            v = int(rng.choice(kids))
            n += 1
            path[b, n] = v
        a[b] = n
    return a, path, parent


def _vectorised_counts(a, path, parent, T):
    """The same three counts, said differently: depths by repeated gathering, membership tests on whole arrays."""
    B = len(a)
    depth = np.full((B, T), -1, dtype=np.int64)
    depth[:, 0] = 0
    par = parent.copy()
    par[:, 0] = -1
    for _ in range(T):
        ok = (par >= 0) & (par < np.arange(T)[None, :])
        pd = np.take_along_axis(depth, np.clip(par, 0, T - 1), axis=1)
        depth = np.where((np.arange(T)[None, :] > 0) & ok & (pd >= 0), pd + 1, depth)
    offered = np.array([(depth == k).any(axis=1).sum() for k in range(T)])
    accepted = np.array([(a >= k).sum() for k in range(T)])
    last = path[np.arange(B), a]
    has_child = ((par == last[:, None]) & (depth > 0)).any(axis=1)
    tried = accepted.copy()
    for b in range(B):
        if has_child[b]:
            tried[a[b] + 1] += 1
    return [offered.tolist(), tried.tolist(), accepted.tolist()]


@pytest.mark.parametrize("seed,T,top_k", [(1, 9, 1), (2, 17, 1), (3, 33, 4), (4, 13, 3), (5, 64, 2)])
def test_identities_and_a_second_count(seed, T, top_k):
    rng = np.random.default_rng(seed)
    a, path, parent = _random_step(rng, 300, T, top_k)
    c = so.acceptance_counts(a, path, parent, T)
    off, tri, acc = c
    assert sum(acc[1:]) == int(a.sum())                       # every accepted draft token is counted once
    assert off[0] == tri[0] == acc[0] == 300                   # the root: every step, always accepted
    for k in range(1, T):
        assert acc[k] <= tri[k] <= off[k]
        assert tri[k] <= acc[k - 1]                            # a position is tried only after the one before was accepted
    assert c == _vectorised_counts(a, path, parent, T)
    # two steps counted one after the other = both counted at once
    c2 = so.acceptance_counts(a[:100], path[:100], parent[:100], T)
    so.acceptance_counts(a[100:], path[100:], parent[100:], T, c2)
    assert c2 == c


def test_chain_without_parent_array_is_the_chain_with_one():
    rng = np.random.default_rng(7)
    T, B = 9, 200
    a = rng.integers(0, T, size=B)
    path = np.full((B, T), -1, dtype=np.int64)
    for b in range(B):
        path[b, : a[b] + 1] = np.arange(a[b] + 1)
    chain = np.tile(np.arange(-1, T - 1), (B, 1))
    chain[:, 0] = 0
    assert so.acceptance_counts(a, path, None, T) == so.acceptance_counts(a, path, chain, T)


def test_planted_probabilities_and_the_expected_tokens_law():
    """Chains of gamma draft tokens whose k-th token is accepted with probability q[k] once the ones before were:
    the conditional rates recover q, the default rates its running product, and with a constant q = alpha the
    tokens per step follow (1 - alpha^(gamma+1)) / (1 - alpha) (Section 3.4.1)."""
    rng = np.random.default_rng(11)
    gamma, B = 8, 60000
    T = gamma + 1
    q = np.array([0.9, 0.8, 0.85, 0.6, 0.7, 0.5, 0.9, 0.4])
    ok = rng.random((B, gamma)) < q[None, :]
    a = np.where(ok.all(axis=1), gamma, np.argmin(ok, axis=1))
    path = np.full((B, T), -1, dtype=np.int64)
    for b in range(B):
        path[b, : a[b] + 1] = np.arange(a[b] + 1)
    c = so.acceptance_counts(a, path, None, T)
    cond = np.array(so.beta_from_counts(c, T, conditional=True))
    cum = np.array(so.beta_from_counts(c, T))
    tried = np.array(c[so.TRIED][1:], dtype=np.float64)
    assert (np.abs(cond - q) < 5 * np.sqrt(q * (1 - q) / tried)).all()
    assert (np.abs(cum - np.cumprod(q)) < 5 * np.sqrt(0.25 / B)).all()
    assert (np.diff(cum) <= 0).all()
    assert abs(np.array(so.beta_from_counts(c, T, conditional=True, prior=0.5)) - cond).max() == 0   # prior unused here
    # constant alpha: tokens per step (accepted + bonus) against the closed form
    alpha = 0.7
    ok = rng.random((B, gamma)) < alpha
    a = np.where(ok.all(axis=1), gamma, np.argmin(ok, axis=1))
    for b in range(B):
        path[b] = -1
        path[b, : a[b] + 1] = np.arange(a[b] + 1)
    c = so.acceptance_counts(a, path, None, T)
    tokens = 1.0 + sum(so.beta_from_counts(c, T))            # 1 + sum_k P(k-th accepted)
    assert abs(tokens - (a.mean() + 1.0)) < 1e-12              # an identity of the counts
    assert abs(tokens - (1 - alpha ** (gamma + 1)) / (1 - alpha)) < 0.03


def test_prior_where_nothing_was_counted():
    c = so.acceptance_counts([1], [[0, 1, -1, -1]], [[0, 0, -2, -2]], 4)
    assert so.beta_from_counts(c, 4, prior=0.25) == [1.0, 0.25, 0.25]
    assert so.beta_from_counts(c, 4, conditional=True, prior=0.5) == [1.0, 0.5, 0.5]


# ---- the library's host function (no GPU needed) and its argument checks ---------------------------------------

def test_library_beta_matches_the_oracle():
    from paper_2511_14617_amd import binding
    rng = np.random.default_rng(21)
    for T, top_k in ((9, 1), (33, 4), (64, 2), (1, 1)):
        a, path, parent = _random_step(rng, 100, T, top_k)
        c = so.acceptance_counts(a, path, parent, T)
        for conditional in (False, True):
            for prior in (0.0, 0.3, 1.0):
                assert binding.seer_acceptance_beta(c, conditional, prior) == so.beta_from_counts(c, T, conditional, prior)


def test_host_side_argument_checks():
    import ctypes
    from paper_2511_14617_amd import binding
    lib = binding.load_library()
    counts = (ctypes.c_uint64 * 12)(*([4] * 12))
    beta = (ctypes.c_double * 3)()
    assert lib.seer_acceptance_beta(None, 4, 0, 0.0, beta) == binding.SEER_EINVAL
    assert lib.seer_acceptance_beta(counts, 4, 0, 0.0, None) == binding.SEER_EINVAL
    assert lib.seer_acceptance_beta(counts, 0, 0, 0.0, beta) == binding.SEER_ESHAPE
    assert lib.seer_acceptance_beta(counts, 65, 0, 0.0, beta) == binding.SEER_ESHAPE
    assert lib.seer_acceptance_beta(counts, 4, 0, 1.5, beta) == binding.SEER_EINVAL
    bad = (ctypes.c_uint64 * 12)(*([1] * 8 + [2] * 4))          # accepted > offered: not counts of the library
    assert lib.seer_acceptance_beta(bad, 4, 0, 0.0, beta) == binding.SEER_EINVAL
    assert lib.seer_acceptance_beta(counts, 4, 0, 0.0, beta) == binding.SEER_OK and list(beta) == [1.0, 1.0, 1.0]
    # the device call: shape, null and alignment errors are found before anything is launched
    fake = ctypes.c_void_p(1 << 20)
    assert lib.seer_acceptance_stats(fake, fake, None, -1, 4, fake, None) == binding.SEER_ESHAPE
    assert lib.seer_acceptance_stats(fake, fake, None, 1, 0, fake, None) == binding.SEER_ESHAPE
    assert lib.seer_acceptance_stats(fake, fake, None, 1, 65, fake, None) == binding.SEER_ESHAPE
    assert lib.seer_acceptance_stats(None, None, None, 0, 4, None, None) == binding.SEER_OK          # nothing to do
    assert lib.seer_acceptance_stats(None, fake, None, 1, 4, fake, None) == binding.SEER_EINVAL
    assert lib.seer_acceptance_stats(fake, fake, None, 1, 4, None, None) == binding.SEER_EINVAL
    assert lib.seer_acceptance_stats(fake, fake, None, 1, 4, ctypes.c_void_p((1 << 20) + 4), None) == binding.SEER_EALIGN


# ---- GPU parity: counts bit for bit ----------------------------------------------------------------------------

@pytest.mark.gpu
@pytest.mark.parametrize("seed,B,T,top_k", [(1, 1, 9, 1), (2, 300, 9, 1), (3, 128, 33, 4), (4, 77, 64, 3), (5, 1000, 17, 2), (6, 5, 1, 1)])
def test_gpu_counts_match_the_oracle(seed, B, T, top_k):
    import torch
    from paper_2511_14617_amd import binding
    rng = np.random.default_rng(seed)
    a, path, parent = _random_step(rng, B, T, top_k)
    # malformed requests (left out by both sides): a path through a padded slot, a length out of range, a wrong root
    if B >= 5:
        if T > 1:
            path[1, 1] = T - 1 if parent[1, T - 1] < 0 else path[1, 1]
            a[1] = max(a[1], 1)
        a[2] = T
        path[3, 0] = 1
        a[4] = -1
    want = so.acceptance_counts(a, path, parent, T)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).cuda()
    counts = torch.zeros((3, T), dtype=torch.int64, device="cuda")
    binding.seer_acceptance_stats(dev(a), dev(path), dev(parent), counts)
    assert counts.cpu().tolist() == want
    # a second step accumulates; a chain given without a parent array
    chain_a = rng.integers(0, T, size=B)
    chain_path = np.full((B, T), -1, dtype=np.int64)
    for b in range(B):
        chain_path[b, : chain_a[b] + 1] = np.arange(chain_a[b] + 1)
    so.acceptance_counts(chain_a, chain_path, None, T, want)
    binding.seer_acceptance_stats(dev(chain_a), dev(chain_path), None, counts)
    assert counts.cpu().tolist() == want
    assert binding.seer_acceptance_beta(want, False, 0.5) == so.beta_from_counts(want, T, False, 0.5)


@pytest.mark.gpu
def test_gpu_counts_after_accept_on_planted_trees():
    """draft trees with planted acceptance -> seer_accept -> seer_acceptance_stats, against the oracles of both."""
    import torch
    import oracle
    from paper_2511_14617_amd import binding, workloads as W
    from gpu_util import accept_device_inputs
    cfg = W.CONFIGS[5].scaled(B=24, V=1000)
    parent = W.multipath_parent(cfg.B, 4, 8, np.random.default_rng(4), dedup_fraction=0.4)
    acc = W.make_accept_inputs(cfg, tree_parent=parent)
    d = accept_device_inputs(acc)
    alen, apath, bonus, tgt = binding.seer_accept(d["logits"], d["draft_tokens"], d["tree_parent"])
    counts = torch.zeros((3, cfg.T), dtype=torch.int64, device="cuda")
    binding.seer_acceptance_stats(alen, apath, d["tree_parent"], counts)
    o_len, o_path, _, _ = oracle.verify_accept(acc.logits, acc.draft_tokens, acc.tree_parent)
    want = so.acceptance_counts(o_len, o_path, acc.tree_parent, cfg.T)
    assert counts.cpu().tolist() == want
    assert want[so.ACCEPTED][1] > 0
