"""Pins for the CPU oracle: each test ties a part of it to something the oracle
did not compute itself -- a library routine on a special case (torch's fp64
scaled_dot_product_attention on a gathered dense sequence, numpy's argmax), a
closed form (constant V, constant K, the geometric expected-length law of
Section 3.4.1), an invariance, or brute-force enumeration on tiny trees."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2511_14617_amd import workloads as W

SMALL = W.CONFIGS[1]  # B=4, Hq=8, Hkv=2, D=128, P=16, T=5, ctx in [64, 512]


def _f64(bits):
    return W.bf16_bits_to_f32(bits).astype(np.float64)


def _dense_sequence(inp, b, positions):
    """K[Hkv, len, Dqk], V[Hkv, len, Dv] in fp64 for the given logical positions,
    gathered here with numpy indexing (not by the oracle)."""
    P = inp.cfg.page_size
    pos = np.asarray(positions)
    pages = inp.block_table[b, pos // P]
    slots = pos % P
    K = _f64(inp.k_pages[pages, :, slots, :])            # [len, Hkv, D]
    if inp.v_pages is None:
        V = K[..., : inp.cfg.Dv]
    else:
        V = _f64(inp.v_pages[pages, :, slots, :])
    return K.transpose(1, 0, 2), V.transpose(1, 0, 2)


def _sdpa_decode(inp, b, t, positions):
    """Textbook single-query attention over `positions` for query slot t, all
    heads, by torch's library routine in fp64."""
    cfg = inp.cfg
    K, V = _dense_sequence(inp, b, positions)
    G = cfg.G
    Kt = torch.from_numpy(np.repeat(K, G, axis=0))[None]      # [1, Hq, len, D]
    Vt = torch.from_numpy(np.repeat(V, G, axis=0))[None]
    qt = torch.from_numpy(_f64(inp.q[b, t]))[None, :, None, :]  # [1, Hq, 1, D]
    o = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=inp.scale)
    return o[0, :, 0, :].numpy()


def _run(inp, mask="own"):
    m = inp.tree_mask if isinstance(mask, str) else mask
    return oracle.verify_attention(inp.q, inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, m,
                                   inp.scale, Dv=inp.cfg.Dv)


# ---------------------------------------------------------------- attention
def test_T1_is_ordinary_decode():
    """gamma = 0 (speculation off, Algorithm 1's "disable speculation" branch) is plain decode."""
    cfg = SMALL.scaled(T=1)
    inp = W.make_attention_inputs(cfg, values="peaked")
    out = _run(inp)
    for b in range(cfg.B):
        ref = _sdpa_decode(inp, b, 0, np.arange(int(inp.ctx_len[b])))
        np.testing.assert_allclose(out[b, 0], ref, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("values", ["paper", "peaked"])
def test_chain_slot_equals_serial_decode(values):
    """Slot t of a chain must reproduce serial decoding at length n0 + t + 1 (losslessness)."""
    inp = W.make_attention_inputs(SMALL, values=values)
    out = _run(inp)
    T = SMALL.T
    for b in range(SMALL.B):
        n0 = int(inp.ctx_len[b]) - T
        for t in range(T):
            ref = _sdpa_decode(inp, b, t, np.arange(n0 + t + 1))
            np.testing.assert_allclose(out[b, t], ref, rtol=1e-11, atol=1e-12)


def test_tree_node_equals_decode_over_its_root_path():
    cfg = SMALL.scaled(T=1 + 3 * 3, tree=(3, 3), ctx=("uniform", 40, 200))
    inp = W.make_attention_inputs(cfg, values="peaked", dedup_fraction=0.5)
    assert (inp.tree_parent == -2).any(), "want at least one padded slot in this case"
    out = _run(inp)
    for b in range(cfg.B):
        n0 = int(inp.ctx_len[b]) - cfg.T
        for t in range(cfg.T):
            path = []
            s = t
            while s >= 0:
                path.append(s)
                s = int(inp.tree_parent[b, s]) if s > 0 else -1
            if inp.tree_parent[b, t] == -2:
                path = [t]              # padded slot: prefix + itself
            pos = np.concatenate([np.arange(n0), n0 + np.array(sorted(path))])
            ref = _sdpa_decode(inp, b, t, pos)
            np.testing.assert_allclose(out[b, t], ref, rtol=1e-11, atol=1e-12)


def test_block_table_shuffle_is_bit_identical():
    inp = W.make_attention_inputs(SMALL, values="peaked")
    out = _run(inp)
    rng = np.random.default_rng(7)
    perm = rng.permutation(inp.num_pages)              # old page -> new page
    k2 = np.empty_like(inp.k_pages)
    v2 = np.empty_like(inp.v_pages)
    k2[perm] = inp.k_pages
    v2[perm] = inp.v_pages
    bt2 = perm[inp.block_table].astype(np.int32)
    out2 = oracle.verify_attention(inp.q, k2, v2, bt2, inp.ctx_len, None, inp.scale)
    assert np.array_equal(out, out2)


def test_chain_mask_equals_no_mask():
    inp = W.make_attention_inputs(SMALL, values="peaked")
    chain = W.ancestor_masks(W.chain_parent(SMALL.B, SMALL.T))
    assert np.array_equal(_run(inp, None), _run(inp, chain))


def test_constant_V_gives_that_constant():
    inp = W.make_attention_inputs(SMALL, values="peaked")
    c = W.f32_to_bf16_bits(np.array([0.8125], dtype=np.float32))[0]
    inp.v_pages[...] = c
    np.testing.assert_allclose(_run(inp), 0.8125, rtol=1e-13)


def test_constant_K_gives_mean_of_visible_V():
    cfg = SMALL.scaled(T=1 + 2 * 3, tree=(2, 3), ctx=("uniform", 20, 90))
    inp = W.make_attention_inputs(cfg, values="peaked")
    inp.k_pages[...] = W.f32_to_bf16_bits(np.array([0.375], dtype=np.float32))[0]
    out = _run(inp)
    for b in range(cfg.B):
        n0 = int(inp.ctx_len[b]) - cfg.T
        for t in range(cfg.T):
            vis = [s for s in range(cfg.T) if (int(inp.tree_mask[b, t]) >> s) & 1]
            depth = len(vis) - 1
            assert len(vis) == bin(int(inp.tree_mask[b, t])).count("1")
            _, V = _dense_sequence(inp, b, np.concatenate([np.arange(n0), n0 + np.array(vis)]))
            assert V.shape[1] == n0 + depth + 1
            ref = np.repeat(V.mean(axis=1), cfg.G, axis=0)
            np.testing.assert_allclose(out[b, t], ref, rtol=1e-11, atol=1e-13)


def test_key_shift_invariance():
    """Adding one vector to every key shifts every score of a query by the same amount."""
    cfg = SMALL.scaled(ctx=("uniform", 30, 120))
    inp = W.make_attention_inputs(cfg, values="peaked")
    rng = np.random.default_rng(3)
    # keys on a 1/8 grid in [-2, 2] and an integer shift: both exactly representable in bf16
    kf = rng.integers(-16, 17, size=inp.k_pages.shape).astype(np.float32) / 8.0
    shift = rng.integers(-3, 4, size=cfg.Dqk).astype(np.float32)
    inp.k_pages = W.f32_to_bf16_bits(kf)
    base = _run(inp)
    inp.k_pages = W.f32_to_bf16_bits(kf + shift)
    assert np.array_equal(W.bf16_bits_to_f32(inp.k_pages), kf + shift)
    np.testing.assert_allclose(_run(inp), base, rtol=1e-9, atol=1e-12)


def test_gqa_equals_mha_on_replicated_kv():
    inp = W.make_attention_inputs(SMALL, values="peaked")
    out = _run(inp)
    G = SMALL.G
    k_rep = np.repeat(inp.k_pages, G, axis=1)
    v_rep = np.repeat(inp.v_pages, G, axis=1)
    out2 = oracle.verify_attention(inp.q, k_rep, v_rep, inp.block_table, inp.ctx_len, None, inp.scale)
    assert np.array_equal(out, out2)


def test_shared_latent_equals_explicit_value_pool():
    cfg = W.CONFIGS[4].scaled(B=2, Hq=4, T=3, ctx=("uniform", 70, 200))
    inp = W.make_attention_inputs(cfg, values="peaked")
    assert inp.v_pages is None
    out = _run(inp)
    v_explicit = np.ascontiguousarray(inp.k_pages[..., : cfg.Dv])
    out2 = oracle.verify_attention(inp.q, inp.k_pages, v_explicit, inp.block_table, inp.ctx_len, None,
                                   inp.scale)
    assert np.array_equal(out, out2)
    for b in range(cfg.B):
        ref = _sdpa_decode(inp, b, 0, np.arange(int(inp.ctx_len[b]) - cfg.T + 1))
        np.testing.assert_allclose(out[b, 0], ref, rtol=1e-11, atol=1e-12)


def test_needle_gets_the_weight_and_a_non_ancestor_gets_none():
    cfg = SMALL.scaled(B=2, T=1 + 2 * 2, tree=(2, 2), ctx=("uniform", 50, 100))
    inp = W.make_attention_inputs(cfg, values="paper")
    P = cfg.page_size
    b, t, h = 1, 2, 5           # slot 2 = second node of path 0; slots 3, 4 are the other path
    kvh = h // cfg.G
    n0 = int(inp.ctx_len[b]) - cfg.T
    qv = W.bf16_bits_to_f32(inp.q[b, t, h])
    needle = W.f32_to_bf16_bits(qv / np.linalg.norm(qv) * 300.0)

    def put(pos, vec_bits, vval):
        pg, sl = inp.block_table[b, pos // P], pos % P
        inp.k_pages[pg, kvh, sl] = vec_bits
        inp.v_pages[pg, kvh, sl] = W.f32_to_bf16_bits(np.full(cfg.Dv, vval, dtype=np.float32))

    put(n0 + 3, needle, 64.0)          # non-ancestor draft slot: must get zero weight
    out = _run(inp)
    assert abs(out[b, t, h]).max() < 1.0
    put(17, needle, -3.0)              # inside the prefix, across a page boundary from 15/16
    out = _run(inp)
    np.testing.assert_allclose(out[b, t, h], -3.0, atol=1e-6)
    assert abs(out[b, 3, h] + 3.0).max() > 1.0   # another query is not drawn to this needle alike


def test_rows_variant_matches_full():
    inp = W.make_attention_inputs(SMALL, values="peaked")
    full = _run(inp)
    rows = np.array([[0, 0, 0], [3, 4, 7], [2, 1, 3], [1, 2, 4]], dtype=np.int32)
    sub = oracle.verify_attention_rows(rows, inp.q, inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len,
                                       None, inp.scale)
    for i, (b, t, h) in enumerate(rows):
        assert np.array_equal(sub[i], full[b, t, h])


def test_argument_errors():
    inp = W.make_attention_inputs(SMALL)
    bad = inp.ctx_len.copy()
    bad[0] = SMALL.T - 1
    with pytest.raises(ValueError):
        oracle.verify_attention(inp.q, inp.k_pages, inp.v_pages, inp.block_table, bad, None, inp.scale)
    bt = inp.block_table.copy()
    bt[1, 0] = inp.num_pages
    with pytest.raises(ValueError):
        oracle.verify_attention(inp.q, inp.k_pages, inp.v_pages, bt, inp.ctx_len, None, inp.scale)


# ---------------------------------------------------------------- argmax
def test_argmax_against_numpy_with_many_ties():
    rng = np.random.default_rng(11)
    for V in (1, 2, 63, 64, 65, 1000, 4099):
        x = rng.integers(-5, 6, size=(37, V)).astype(np.float32)   # heavy ties
        assert np.array_equal(oracle.argmax(x), np.argmax(x, axis=-1).astype(np.int32))


def test_argmax_edge_cases():
    V = 1000
    x = np.full((6, V), -np.inf, dtype=np.float32)
    x[1, 0] = 1.0
    x[2, V - 1] = 1.0
    x[3, [255, 256, 511, 512]] = 2.0          # equal maxima: lowest index wins
    x[4, :] = -0.0
    x[4, 700] = 0.0                           # +0 does not beat the earlier -0
    x[5, :] = np.linspace(-1, 1, V, dtype=np.float32)
    assert oracle.argmax(x).tolist() == [0, 0, V - 1, 255, 0, V - 1]


# ---------------------------------------------------------------- acceptance
def _all_parent_arrays(T, allow_pad):
    choices = [[-1]] + [list(range(t)) + ([-2] if allow_pad else []) for t in range(1, T)]
    return [np.array(p, dtype=np.int32) for p in itertools.product(*choices)]


def _brute_force(parent, draft, target):
    """Enumerate every root->node path and test 'all its tokens match' directly.
    draft, target: [N, T] (all combinations at once); parent: [T]."""
    T = len(parent)
    N = draft.shape[0]
    best_len = np.zeros(N, dtype=np.int64)
    best_node = np.zeros(N, dtype=np.int64)
    for t in range(1, T):
        path = []
        s = t
        valid = True
        while s > 0:
            if parent[s] < 0:
                valid = False       # a padded slot, or one hanging below a padded slot
                break
            path.append(s)
            s = int(parent[s])
        if not valid:
            continue
        ok = np.ones(N, dtype=bool)
        for node in path:
            ok &= draft[:, node] == target[:, parent[node]]
        better = ok & (len(path) > best_len)          # strict: lowest index among equals
        best_len[better] = len(path)
        best_node[better] = t
    return best_len, best_node


@pytest.mark.parametrize("T,V,allow_pad", [(4, 3, True), (5, 3, False), (6, 2, False), (5, 2, True)])
def test_acceptance_against_exhaustive_enumeration(T, V, allow_pad):
    toks = np.array(list(itertools.product(range(V), repeat=T)), dtype=np.int32)       # [V^T, T]
    drafts = np.array(list(itertools.product(range(V), repeat=T - 1)), dtype=np.int32)
    drafts = np.concatenate([np.zeros((len(drafts), 1), np.int32), drafts], axis=1)
    draft = np.repeat(drafts, len(toks), axis=0)
    target = np.tile(toks, (len(drafts), 1))
    for parent in _all_parent_arrays(T, allow_pad):
        par = np.tile(parent, (len(draft), 1))
        alen, path, bonus = oracle.accept(target, draft, par)
        bl, bn = _brute_force(parent, draft, target)
        assert np.array_equal(alen, bl)
        last = path[np.arange(len(path)), alen]
        assert np.array_equal(last, bn)
        assert np.array_equal(bonus, target[np.arange(len(target)), bn])
        # the path is the winner's root path, padded with -1
        for i in range(0, len(path), 97):
            node, want = int(bn[i]), []
            while node >= 0:
                want.append(node)
                node = int(parent[node])
            want = want[::-1] + [-1] * (T - len(want))
            assert path[i].tolist() == want


def test_chain_parent_none_equals_explicit_chain():
    rng = np.random.default_rng(5)
    B, T = 200, 9
    target = rng.integers(0, 3, size=(B, T)).astype(np.int32)
    draft = rng.integers(0, 3, size=(B, T)).astype(np.int32)
    a = oracle.accept(target, draft, None)
    b = oracle.accept(target, draft, W.chain_parent(B, T))
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # a greedy scan written for chains only
    for i in range(B):
        n = 0
        while n + 1 < T and draft[i, n + 1] == target[i, n]:
            n += 1
        assert a[0][i] == n and a[2][i] == target[i, n]


def test_duplicate_siblings_take_the_deeper_continuation():
    # root -> 1 -> 2 and root -> 3 -> 4 -> 5, nodes 1 and 3 carry the same token
    parent = np.array([[-1, 0, 1, 0, 3, 4]], dtype=np.int32)
    target = np.array([[7, 8, 0, 8, 9, 4]], dtype=np.int32)
    draft = np.array([[0, 7, 5, 7, 8, 9]], dtype=np.int32)   # node 2 wrong; 3,4,5 all right
    alen, path, bonus = oracle.accept(target, draft, parent)
    assert alen.tolist() == [3] and path.tolist() == [[0, 3, 4, 5, -1, -1]] and bonus.tolist() == [4]


def test_gamma_zero_is_a_plain_greedy_step():
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((5, 1, 300)).astype(np.float32)
    alen, path, bonus, tgt = oracle.verify_accept(logits, np.zeros((5, 1), np.int32), None)
    assert alen.tolist() == [0] * 5 and path.tolist() == [[0]] * 5
    assert np.array_equal(bonus, np.argmax(logits[:, 0], axis=-1))


def test_planted_lengths_and_expected_tokens_law():
    """Planting accepted lengths from the i.i.d. per-position law must give back exactly those
    lengths, and their mean + 1 must follow (1 - alpha^(gamma+1)) / (1 - alpha) (Section 3.4.1)."""
    gamma, alpha, B = 8, 0.7, 6000
    cfg = W.CONFIGS[2].scaled(B=B, T=gamma + 1, V=97)
    rng = np.random.default_rng(123)
    acc = rng.random((B, gamma)) < alpha
    planted = np.where(acc.all(axis=1), gamma, np.argmin(acc, axis=1)).astype(np.int32)
    inp = W.make_accept_inputs(cfg, planted_len=planted)
    alen, path, bonus, tgt = oracle.verify_accept(inp.logits, inp.draft_tokens, None)
    assert np.array_equal(alen, planted)
    assert np.array_equal(tgt, inp.planted_target)
    assert np.array_equal(bonus, inp.planted_target[np.arange(B), planted])
    law = (1 - alpha ** (gamma + 1)) / (1 - alpha)
    emitted = alen.astype(np.float64) + 1.0
    assert abs(emitted.mean() - law) < 4.0 * emitted.std() / np.sqrt(B)


def test_planted_tree_acceptance():
    cfg = W.CONFIGS[5].scaled(B=64, V=211)
    rng = np.random.default_rng(9)
    parent = W.multipath_parent(cfg.B, 4, 8, rng, dedup_fraction=0.3)
    inp = W.make_accept_inputs(cfg, tree_parent=parent)
    alen, path, bonus, tgt = oracle.verify_accept(inp.logits, inp.draft_tokens, parent)
    assert np.array_equal(alen, inp.planted_len)
    assert np.array_equal(tgt, inp.planted_target)
    # at least one request has two accepted siblings with the same token (duplicate first tokens)
    dup = 0
    for b in range(cfg.B):
        kids = [t for t in range(1, cfg.T) if parent[b, t] == 0]
        toks = [int(inp.draft_tokens[b, t]) for t in kids]
        dup += len(set(toks)) < len(toks)
    assert dup >= 1
