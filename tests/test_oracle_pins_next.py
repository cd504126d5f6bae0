"""Pins for the second part of the CPU oracle: the commit of the accepted path (the step right
after verification) and verification under sampling (Section 4.1: temperatures 1.0 and 0.8).

Each test ties the oracle to something it did not compute itself: the published known-answer
vectors of the counter-based generator, libm's logarithm, the softmax distribution (a draw by
the Gumbel-max rule must be a sample of it), numpy's fancy indexing for the data movement, and
the attention oracle's already pinned tree semantics (reading the committed cache as an ordinary
sequence must give what the verify pass gave at the winning node)."""
import math

import numpy as np
import pytest

import oracle
from paper_2511_14617_amd import workloads as W


# ------------------------------------------------------------------ sampling
def test_philox_known_answers():
    """Known-answer vectors published with the generator's reference implementation (Random123:
    counter, key -> output, 10 rounds)."""
    kat = [
        ([0, 0, 0, 0], [0, 0], [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]),
        ([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2, [0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD]),
        ([0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], [0xA4093822, 0x299F31D0],
         [0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]),
    ]
    for ctr, key, want in kat:
        assert [int(x) for x in oracle.philox4x32_10(ctr, key)] == want


def test_deterministic_log2_against_libm():
    rng = np.random.default_rng(5)
    xs = np.concatenate([np.exp(rng.uniform(-60, 60, 4000)), 1.0 + rng.uniform(-1e-3, 1e-3, 500),
                         [2.0 ** -24, 1 - 2.0 ** -24, 1.0, 2.0, 0.5, 1.41421354, 1.41421366]]).astype(np.float32)
    for x in xs:
        got, want = oracle.log2_det(float(x)), math.log2(float(x))
        assert abs(got - want) <= 3e-7 + 1.5e-7 * abs(want), (float(x), got, want)


def test_gumbel_noise_moments():
    """Standard Gumbel: mean = Euler's constant, variance = pi^2 / 6."""
    g = np.array([oracle.gumbel(77, r, v) for r in range(60) for v in range(1000)])
    n = g.size
    assert abs(g.mean() - 0.5772156649) < 5 * math.sqrt(math.pi ** 2 / 6 / n)
    assert abs(g.var() - math.pi ** 2 / 6) < 0.05
    assert np.isfinite(g).all() and g.min() > -3.0 and g.max() < 17.0   # u in [2^-24, 1 - 2^-24]


def test_gumbel_of_words_is_the_noise_of_the_draws_and_has_the_closed_form():
    """The vectorised form takes the generator's word where `gumbel` takes (seed, row, v); both give the same
    deviate, and it is -ln(-ln u) of u = (word's upper 23 bits + 1/2) 2^-23 to the accuracy of the fixed logarithm."""
    seed, row = 0x1234567890ABCDEF, 17
    for v in (0, 1, 2, 3, 4, 1001, 151935):
        words = oracle.philox4x32_10([v >> 2, row, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.gumbel_of_words(words[v & 3: (v & 3) + 1])[0] == np.float32(oracle.gumbel(seed, row, v))
    rng = np.random.default_rng(5)
    w = rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32)
    u = ((w >> 9).astype(np.float64) + 0.5) * 2.0 ** -23
    want = -np.log(-np.log(u))
    assert np.max(np.abs(oracle.gumbel_of_words(w) - want)) < 2e-5


def test_every_word_stays_below_the_bound_by_leading_ones():
    """What lets the sampled scan skip the logarithms of most logits: with z leading one bits in the word's upper
    23 bits, 1 - u > 2^-(z+1) and so G < (z + 1) ln 2.  Checked for all 2^23 inputs of the fixed-polynomial
    arithmetic, with the slack the kernel's constant (ln 2 + 0.05) leaves for fp32 roundings: G + 0.04 <= bound."""
    hi = np.arange(1 << 23, dtype=np.uint32)
    g = oracle.gumbel_of_words(hi << np.uint32(9)).astype(np.float64)
    assert np.array_equal(g, oracle.gumbel_of_words((hi << np.uint32(9)) | np.uint32(0x1ff)))   # the low 9 bits play no part
    inv = (~hi) & np.uint32((1 << 23) - 1)
    # leading ones of a 23-bit field = 23 - bit length of its complement
    bitlen = np.zeros(hi.shape, dtype=np.int64)
    nz = inv > 0
    bitlen[nz] = np.floor(np.log2(inv[nz].astype(np.float64))).astype(np.int64) + 1
    z = 23 - bitlen
    assert z.min() == 0 and z.max() == 23 and np.count_nonzero(z == 23) == 1
    bound = z.astype(np.float64) * float(np.float32(0.693147182)) + float(np.float32(np.float32(0.693147182) + np.float32(0.05)))
    assert np.all(g + 0.04 <= bound)
    assert np.all(np.diff(g) >= 0)                       # and the noise grows with the word, as -ln(-ln u) does
    assert (bound - g)[z >= 8].max() < 0.75                      # no looser than a factor of two in 1 - u, plus the slack


@pytest.mark.parametrize("tau", [1.0, 0.8])
def test_draws_follow_softmax_of_logits_over_temperature(tau):
    """The token drawn at a verify position must be a sample of softmax(logits / tau): chi-square of
    120 000 independent rows (same logits, different row index -> different noise) against it."""
    logits = np.array([1.3, -0.2, 0.0, 2.1, -1.7, 0.4, 0.9], np.float32)
    N = 120000
    draws = oracle.argmax_sampled(np.tile(logits, (N, 1)), tau, seed=20251114)
    p = np.exp(logits.astype(np.float64) / tau)
    p /= p.sum()
    counts = np.bincount(draws, minlength=logits.size)
    chi2 = ((counts - N * p) ** 2 / (N * p)).sum()
    assert chi2 < 27.9          # 99.99 % quantile of chi-square with 6 degrees of freedom
    # and the wrong temperature is rejected by the same test (the test has teeth)
    q = np.exp(logits.astype(np.float64) / (tau * 1.15))
    q /= q.sum()
    assert ((counts - N * q) ** 2 / (N * q)).sum() > 100


def test_cold_sampling_is_greedy_and_seeds_matter():
    rng = np.random.default_rng(3)
    logits = rng.normal(size=(300, 257)).astype(np.float32)
    assert np.array_equal(oracle.argmax_sampled(logits, 1e-4, seed=1), oracle.argmax(logits))
    a, b = oracle.argmax_sampled(logits, 1.0, seed=1), oracle.argmax_sampled(logits, 1.0, seed=2)
    assert np.array_equal(a, oracle.argmax_sampled(logits, 1.0, seed=1))
    assert (a != b).mean() > 0.8
    # -inf entries are never drawn; a row of -inf gives index 0
    logits[:, ::2] = -np.inf
    assert (oracle.argmax_sampled(logits, 1.0, seed=3) % 2 == 1).all()
    assert oracle.argmax_sampled(np.full((2, 9), -np.inf, np.float32), 0.8, seed=3).tolist() == [0, 0]


def test_sampled_acceptance_is_the_greedy_rule_on_the_drawn_tokens():
    """Draft tokens planted along the DRAWN tokens are accepted to exactly the planted depth."""
    cfg = W.CONFIGS[2].scaled(B=40, T=9, V=300)
    rng = np.random.default_rng(8)
    logits = rng.normal(size=(cfg.B, cfg.T, cfg.V)).astype(np.float32)
    drawn = oracle.argmax_sampled(logits, 0.8, seed=11)
    planted = rng.integers(0, cfg.T, size=cfg.B)
    draft = rng.integers(0, cfg.V, size=(cfg.B, cfg.T)).astype(np.int32)
    for b in range(cfg.B):
        for i in range(1, planted[b] + 1):
            draft[b, i] = drawn[b, i - 1]
        if planted[b] + 1 < cfg.T:
            draft[b, planted[b] + 1] = (drawn[b, planted[b]] + 1) % cfg.V
    alen, path, bonus = oracle.accept(drawn, draft, None)
    assert np.array_equal(alen, planted)
    assert np.array_equal(bonus, drawn[np.arange(cfg.B), planted])


# -------------------------------------------------------------------- commit
def _tree_case(seed=0, shared_latent=False):
    if shared_latent:
        cfg = W.CONFIGS[4].scaled(B=5, Hq=4, T=9, V=64, ctx=("uniform", 9, 300), tree=(2, 4))
    else:
        cfg = W.CONFIGS[5].scaled(B=6, group_size=3, T=13, V=64, ctx=("uniform", 13, 300), tree=(3, 4),
                                  shared_prefix=0)
    inp = W.make_attention_inputs(cfg, seed=cfg.seed + seed, values="peaked")
    acc = W.make_accept_inputs(cfg, seed=cfg.seed + seed, tree_parent=inp.tree_parent)
    alen, path, bonus, tgt = oracle.verify_accept(acc.logits, acc.draft_tokens, inp.tree_parent)
    return cfg, inp, acc, alen, path, bonus


def _logical_rows(pool, block_table, b, positions, P):
    pos = np.asarray(positions, dtype=np.int64)
    return pool[block_table[b, pos // P], :, pos % P, :]          # [len, Hkv, D]


@pytest.mark.parametrize("shared_latent", [False, True])
def test_commit_moves_the_accepted_rows_and_nothing_else(shared_latent):
    cfg, inp, acc, alen, path, bonus = _tree_case(1, shared_latent)
    assert alen.max() >= 2 and (path[:, 1:].max(axis=1) > alen).any()    # some accepted path is not the first
    k2, v2, n2 = oracle.kv_commit(inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, alen, path)
    P, T = cfg.page_size, cfg.T
    touched_k = np.zeros(inp.k_pages.shape[:3], bool)
    for b in range(cfg.B):
        n0, a = int(inp.ctx_len[b]) - T, int(alen[b])
        assert n2[b] == n0 + 1 + a
        src = [n0 + int(path[b, i]) for i in range(1, a + 1)]
        dst = list(range(n0 + 1, n0 + 1 + a))
        for old, new in ((inp.k_pages, k2),) + (() if shared_latent else ((inp.v_pages, v2),)):
            assert np.array_equal(_logical_rows(new, inp.block_table, b, dst, P),
                                  _logical_rows(old, inp.block_table, b, src, P))
            # prefix and root untouched
            keep = np.arange(0, n0 + 1)
            assert np.array_equal(_logical_rows(new, inp.block_table, b, keep, P),
                                  _logical_rows(old, inp.block_table, b, keep, P))
        d = np.asarray(dst, dtype=np.int64)
        touched_k[inp.block_table[b, d // P], :, d % P] = True
    # every physical row that is not a destination is bit-identical
    assert np.array_equal(k2[~touched_k], inp.k_pages[~touched_k])
    if not shared_latent:
        assert np.array_equal(v2[~touched_k], inp.v_pages[~touched_k])
    else:
        assert v2 is None


def test_commit_of_a_chain_moves_nothing():
    cfg = W.CONFIGS[2].scaled(B=6, group_size=3, T=9, V=64, ctx=("uniform", 9, 200), shared_prefix=0)
    inp = W.make_attention_inputs(cfg)
    acc = W.make_accept_inputs(cfg)
    alen, path, bonus, _ = oracle.verify_accept(acc.logits, acc.draft_tokens, None)
    k2, v2, n2 = oracle.kv_commit(inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, alen, path)
    assert np.array_equal(k2, inp.k_pages) and np.array_equal(v2, inp.v_pages)
    assert np.array_equal(n2, inp.ctx_len - cfg.T + 1 + alen)


def test_committed_cache_read_as_a_sequence_gives_the_winners_verify_output():
    """Decode (T = 1) over the committed cache, with the winner's query, equals what the tree-masked
    verify pass produced at the winner: the commit realises 'prefix + accepted root path'."""
    cfg, inp, acc, alen, path, bonus = _tree_case(2)
    ref = oracle.verify_attention(inp.q, inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, inp.tree_mask,
                                  inp.scale, Dv=cfg.Dv)
    k2, v2, n2 = oracle.kv_commit(inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, alen, path)
    winner = path[np.arange(cfg.B), alen]
    q1 = inp.q[np.arange(cfg.B), winner][:, None]                    # [B, 1, Hq, D]
    out = oracle.verify_attention(q1, k2, v2, inp.block_table, n2, None, inp.scale, Dv=cfg.Dv)
    assert np.abs(out[:, 0] - ref[np.arange(cfg.B), winner]).max() < 1e-12


def test_emitted_tokens():
    cfg, inp, acc, alen, path, bonus = _tree_case(3)
    em, n = oracle.emitted_tokens(acc.draft_tokens, alen, path, bonus)
    for b in range(cfg.B):
        want = [int(acc.draft_tokens[b, path[b, i]]) for i in range(1, alen[b] + 1)] + [int(bonus[b])]
        assert n[b] == len(want) and em[b, : n[b]].tolist() == want and (em[b, n[b]:] == -1).all()
    # the emitted tokens are the planted targets along the planted path (what serial decoding would emit)
    tgt = acc.planted_target
    for b in range(cfg.B):
        nodes = [int(path[b, i]) for i in range(alen[b] + 1)]
        assert em[b, : n[b]].tolist() == [int(tgt[b, t]) for t in nodes]


def test_commit_argument_errors():
    cfg, inp, acc, alen, path, bonus = _tree_case(4)
    bad = path.copy()
    bad[0, 0] = 1
    with pytest.raises(ValueError):
        oracle.kv_commit(inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, alen, bad)
    with pytest.raises(ValueError):
        oracle.kv_commit(inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, alen + cfg.T, path)
