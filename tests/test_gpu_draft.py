"""GPU parity, through the C ABI, of grouped n-gram drafting (seer_draft) against the CPU oracle: draft
tokens, parents, ancestor masks, node counts and match lengths, bit for bit.  The result is unique (integer
counts, a total order), so everything is compared."""
import os

import numpy as np
import pytest
import torch

from oracle import draft_oracle as D
from oracle import mba_oracle, stats_oracle
import oracle
from paper_2511_14617_amd import workloads as W

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _gpu_draft(d, *, status=None, max_group_tokens=None, workspace=None):
    from paper_2511_14617_amd import binding
    dev = "cuda"
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
    out = binding.seer_draft(t(d.tokens), t(d.seq_start), t(d.seq_len), t(d.group_first), t(d.req_group), t(d.pattern),
                             t(d.pattern_len), t(d.max_spec_tokens), gamma_max=d.gamma_max, top_k=d.top_k,
                             pattern_lookup_min=d.p_min, vocab=d.vocab,
                             max_group_tokens=max(d.max_group_tokens, 1) if max_group_tokens is None else max_group_tokens,
                             min_confidence=d.min_confidence, status=status, workspace=workspace)
    torch.cuda.synchronize()
    tok, par, msk, cnt, mlen = [x.cpu().numpy() for x in out]
    return tok, par, msk.view(np.uint64), cnt, mlen


def _oracle_draft(d):
    return D.batch_speculate(d.tokens, d.seq_start, d.seq_len, d.group_first, d.req_group, d.pattern, d.pattern_len,
                             d.max_spec_tokens, gamma_max=d.gamma_max, top_k=d.top_k, p_min=d.p_min, p_max=d.p_max,
                             min_confidence=d.min_confidence, vocab=d.vocab)


def _compare(d, what=""):
    got, want = _gpu_draft(d), _oracle_draft(d)
    for name, g, w in zip(("match_len", "node_count", "tree_parent", "draft_tokens", "tree_mask"),
                          (got[4], got[3], got[1], got[0], got[2]), (want[4], want[3], want[1], want[0], want[2])):
        bad = np.argwhere(g != w)
        assert bad.size == 0, "%s %s: first difference at %s: gpu %s, oracle %s" % (
            what, name, bad[0], g[tuple(bad[0])], w[tuple(bad[0])])
    return want


def _from_lists(seqs_per_group, req_group, patterns, *, gamma_max, top_k, p_min, p_max, vocab, min_confidence=0.0,
                max_spec=None, gap=3):
    """DraftInputs from explicit token lists (decoy tokens that repeat the sequence's tail fill the gaps)."""
    chunks, starts, lens, group_first, pos = [], [], [], [0], 0
    for seqs in seqs_per_group:
        for s in seqs:
            s = np.asarray(s, np.int32)
            starts.append(pos)
            lens.append(len(s))
            decoy = np.resize(s[-gap:], gap) if len(s) else np.zeros(gap, np.int32)
            chunks += [s, decoy.astype(np.int32)]
            pos += len(s) + gap
        group_first.append(len(starts))
    B = len(req_group)
    pattern = np.full((B, p_max), -1, np.int32)
    plen = np.zeros(B, np.int32)
    for b, p in enumerate(patterns):
        p = list(p)[-p_max:]
        plen[b] = len(p)
        if p:
            pattern[b, p_max - len(p):] = p
    return W.DraftInputs(tokens=np.concatenate(chunks + [np.zeros(4, np.int32)]).astype(np.int32),
                         seq_start=np.asarray(starts, np.int32), seq_len=np.asarray(lens, np.int32),
                         seq_capacity=np.asarray(lens, np.int32) + gap,
                         group_first=np.asarray(group_first, np.int32), req_group=np.asarray(req_group, np.int32),
                         req_seq=np.zeros(B, np.int32), pattern=pattern, pattern_len=plen,
                         max_spec_tokens=np.full(B, gamma_max, np.int32) if max_spec is None else np.asarray(max_spec, np.int32),
                         future=np.zeros((B, 1), np.int32), gamma_max=gamma_max, top_k=top_k, p_min=p_min, p_max=p_max,
                         min_confidence=min_confidence, vocab=vocab)


def test_hand_counted_examples_on_the_gpu():
    ints = lambda txt: [int(x) for x in txt.split()]
    n = 0
    for line in open(os.path.join(ROOT, "tests", "golden", "draft_worked_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        seqs, pat, args, mlen, tok, par, cnt = [f.strip() for f in line.split("|")]
        a = args.split()
        d = _from_lists([[ints(s) for s in seqs.split(";")]], [0], [ints(pat)], gamma_max=int(a[2]), top_k=int(a[3]),
                        p_min=int(a[0]), p_max=int(a[1]), vocab=int(a[5]), min_confidence=float(a[4]))
        got = _gpu_draft(d)
        assert got[4][0] == int(mlen) and got[0][0].tolist() == ints(tok)
        assert got[1][0].tolist() == ints(par) and got[3][0].tolist() == ints(cnt)
        n += 1
    assert n >= 7


@pytest.mark.parametrize("top_k,gamma_max,p_min,p_max,conf", [(1, 8, 2, 8, 0.0), (4, 8, 2, 8, 0.0), (2, 6, 1, 4, 0.05),
                                                                (7, 9, 1, 32, 0.0), (16, 3, 3, 5, 0.01), (3, 21, 0, 6, 0.3)])
def test_grouped_histories_reduced(top_k, gamma_max, p_min, p_max, conf):
    cfg = W.CONFIGS[2].scaled(B=24, ctx=("lognormal", 2500, 0.7, 530, 9000))
    d = W.make_draft_inputs(cfg, seed=500 + top_k, gamma_max=gamma_max, top_k=top_k, p_min=p_min, p_max=p_max,
                            min_confidence=conf)
    rng = np.random.default_rng(top_k)
    d.max_spec_tokens[:] = rng.integers(0, gamma_max + 1, size=cfg.B)
    d.max_spec_tokens[:4] = gamma_max
    d.pattern_len[5] = 0                                   # a request with no history yet
    d.pattern_len[6] = min(1, p_max)                       # shorter than p_min for most cases
    want = _compare(d, "reduced k=%d" % top_k)
    assert (want[4] > 0).sum() >= cfg.B // 2               # most requests find a match


@pytest.mark.parametrize("seed", range(6))
def test_tiny_vocabulary_many_places(seed):
    """A vocabulary of 2..4 tokens: every pattern occurs thousands of times (the hash table runs full-size,
    member lists are long) and almost every count ties with another."""
    rng = np.random.default_rng(900 + seed)
    vocab = int(rng.integers(2, 5))
    groups = [[rng.integers(0, vocab, size=int(rng.integers(0, 6000))).tolist() for _ in range(int(rng.integers(1, 6)))]
              for _ in range(3)]
    B = 9
    p_max = int(rng.integers(1, 4))
    pats = [rng.integers(0, vocab, size=int(rng.integers(1, 7))).tolist() for _ in range(B)]
    d = _from_lists(groups, rng.integers(0, 3, size=B), pats, gamma_max=int(rng.integers(2, 7)), top_k=int(rng.integers(1, 5)),
                    p_min=1, p_max=p_max, vocab=vocab, min_confidence=float(rng.choice([0.0, 0.1, 0.26])))
    want = _compare(d, "tiny vocabulary")
    assert want[3][:, 0].max() > 100


def test_more_distinct_continuations_than_table_slots():
    """The newest token is followed by 6000 different tokens: the hash table (4096 slots) overflows and the
    counting falls back to passes over token ranges.  A few continuations are repeated so that the top of
    the order is decided by counts, the rest by token ids."""
    rng = np.random.default_rng(31)
    vocab = 20000
    follow = rng.permutation(vocab - 1)[:6000] + 1
    follow = np.concatenate([follow, follow[:3], follow[:2], follow[10:11]])     # counts 3, 3, 2, 2 (one of them 11th)
    seq = np.stack([np.zeros(len(follow), np.int64), rng.permutation(follow)], axis=1).reshape(-1)
    seq2 = np.stack([np.zeros(500, np.int64), follow[:500][::-1], follow[1:501]], axis=1).reshape(-1)
    d = _from_lists([[seq.tolist(), seq2.tolist()]], [0, 0], [[5, 0], [0]], gamma_max=3, top_k=4, p_min=1, p_max=2,
                    vocab=vocab)
    want = _compare(d, "table overflow")
    assert want[3][0, 0] >= 6000 and want[3][0, 1] >= 3


def test_long_sequences_span_many_parts():
    cfg = W.CONFIGS[3].scaled(B=3, group_size=3, ctx=("uniform", 30000, 50000))
    d = W.make_draft_inputs(cfg, gamma_max=8, top_k=2, p_min=2, p_max=8)
    _compare(d, "long sequences")


def test_requests_with_unusable_inputs_get_a_root_only_draft_and_a_status_bit():
    from paper_2511_14617_amd import binding
    cfg = W.CONFIGS[1].scaled(B=8, group_size=4)
    d = W.make_draft_inputs(cfg, gamma_max=4, top_k=2, p_min=1, p_max=4)
    good = _oracle_draft(d)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = _gpu_draft(d, status=status)
    assert int(status.item()) == 0 and np.array_equal(got[0], good[0])
    d.req_group[2] = 7                                      # no such group
    d.seq_len[d.group_first[1]] = 1 << 21                   # group 1: a sequence running out of the pool
    status.zero_()
    got = _gpu_draft(d, status=status)
    assert int(status.item()) == 1
    for b in range(cfg.B):
        if b == 2 or d.req_group[b] == 1:
            assert got[4][b] == 0 and (got[1][b, 1:] == -2).all() and got[0][b, 0] == d.pattern[b, -1]
        else:
            assert np.array_equal(got[0][b], good[0][b]) and np.array_equal(got[1][b], good[1][b])
    # a group that holds more tokens than the workspace was sized for
    d = W.make_draft_inputs(cfg, gamma_max=4, top_k=2, p_min=1, p_max=4)
    sizes = [int(d.seq_len[d.group_first[g]:d.group_first[g + 1]].sum()) for g in range(2)]
    status.zero_()
    got = _gpu_draft(d, status=status, max_group_tokens=min(sizes))
    assert int(status.item()) == 2
    small = int(np.argmin(sizes))
    for b in range(cfg.B):
        if d.req_group[b] == small:
            assert np.array_equal(got[0][b], good[0][b])
        else:
            assert got[4][b] == 0 and (got[1][b, 1:] == -2).all()


def test_workspace_contents_do_not_matter():
    """Two calls on one workspace filled with ones, a smaller batch second: same results as fresh calls."""
    from paper_2511_14617_amd import binding
    cfg = W.CONFIGS[2].scaled(B=16, ctx=("lognormal", 2500, 0.7, 530, 9000))
    d1 = W.make_draft_inputs(cfg, seed=1, gamma_max=8, top_k=4)
    d2 = W.make_draft_inputs(cfg.scaled(B=8), seed=2, gamma_max=8, top_k=4)
    p = binding.SeerDraftParams(cfg.B, 2, 16, len(d1.tokens), max(d1.max_group_tokens, d2.max_group_tokens), 8, 4, 2, 8,
                                cfg.V, 0.0)
    ws = torch.full((binding.seer_draft_workspace(p),), 0xFF, dtype=torch.uint8, device="cuda")
    for d in (d1, d2):
        got = _gpu_draft(d, workspace=ws, max_group_tokens=max(d1.max_group_tokens, d2.max_group_tokens))
        want = _oracle_draft(d)
        assert all(np.array_equal(g, w) for g, w in zip(got, want))


@pytest.mark.parametrize("config_id,top_k,gamma_max", [(2, 1, 8), (3, 1, 16), (5, 4, 8)])
def test_full_size_configs(config_id, top_k, gamma_max):
    """The token histories that go with the verification workloads, at full size, every request compared."""
    cfg = W.CONFIGS[config_id]
    d = W.make_draft_inputs(cfg, gamma_max=gamma_max, top_k=top_k)
    assert d.T == cfg.T
    _compare(d, "config %d" % config_id)


def test_draft_feeds_verification():
    """seer_draft -> seer_accept on the device: logits that put the request's true next tokens on top accept
    exactly the drafted root path that agrees with them."""
    from paper_2511_14617_amd import binding
    cfg = W.CONFIGS[5].scaled(B=32, V=4099)
    d = W.make_draft_inputs(cfg, gamma_max=8, top_k=4, n_phrases=64, phrase_prob=0.6)
    dev = "cuda"
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
    tok, par, msk, cnt, mlen = binding.seer_draft(
        t(d.tokens), t(d.seq_start), t(d.seq_len), t(d.group_first), t(d.req_group), t(d.pattern), t(d.pattern_len),
        t(d.max_spec_tokens), gamma_max=8, top_k=4, pattern_lookup_min=d.p_min, vocab=cfg.V,
        max_group_tokens=d.max_group_tokens)
    h_tok, h_par = tok.cpu().numpy(), par.cpu().numpy()
    T = h_tok.shape[1]
    rng = np.random.default_rng(3)
    logits = rng.normal(size=(cfg.B, T, cfg.V)).astype(np.float32)
    expect = np.zeros(cfg.B, np.int32)
    for b in range(cfg.B):
        depth, ok = {0: 0}, {0: True}
        logits[b, 0, d.future[b, 0]] = 9.0
        for s in range(1, T):
            p = int(h_par[b, s])
            if p < 0:
                continue
            depth[s] = depth[p] + 1
            ok[s] = ok[p] and h_tok[b, s] == d.future[b, depth[s] - 1]
            if ok[s]:
                expect[b] = max(expect[b], depth[s])
                logits[b, s, d.future[b, depth[s]]] = 9.0     # a model that continues the true sequence
    alen, path, bonus, tgt = binding.seer_accept(torch.from_numpy(logits).to(dev), tok, par)
    torch.cuda.synchronize()
    assert np.array_equal(alen.cpu().numpy(), expect)
    ra, rp, rb = oracle.accept(logits.argmax(-1).astype(np.int32), h_tok, h_par)
    assert np.array_equal(alen.cpu().numpy(), ra) and np.array_equal(path.cpu().numpy(), rp)
    assert expect.mean() > 1.0
    assert np.array_equal(bonus.cpu().numpy(), d.future[np.arange(cfg.B), expect])


# ------------------------------------------------------------------ appending what a step emitted
def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to("cuda")


def test_history_append_parity_and_refusals():
    from paper_2511_14617_amd import binding
    cfg = W.CONFIGS[2].scaled(B=24, ctx=("lognormal", 1200, 0.7, 513, 4000))
    d = W.make_draft_inputs(cfg, seed=9, gamma_max=8, top_k=1, spare=5)
    rng = np.random.default_rng(4)
    T = 9
    emitted = rng.integers(0, cfg.V, size=(cfg.B, T)).astype(np.int32)
    n_emitted = rng.integers(0, T + 1, size=cfg.B).astype(np.int32)
    n_emitted[:3] = [0, T, 1]
    for b in (1, 6, 7, 8):                               # these sequences are one token short of room
        d.seq_capacity[d.req_seq[b]] = d.seq_len[d.req_seq[b]] + max(int(n_emitted[b]) - 1, 0)
    n_emitted[6] = max(n_emitted[6], 1)
    room = d.seq_capacity[d.req_seq] - d.seq_len[d.req_seq]
    assert (n_emitted > room).any() and (n_emitted <= room).any()      # some requests have no room: they append nothing
    want = D.history_append(d.tokens, d.seq_start, d.seq_len, d.seq_capacity, d.req_seq, emitted, n_emitted, d.p_max)
    tok, ln = _dev(d.tokens), _dev(d.seq_len)
    pat = torch.full((cfg.B, d.p_max), 77, dtype=torch.int32, device="cuda")
    plen = torch.zeros(cfg.B, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    binding.seer_history_append(tok, _dev(d.seq_start), ln, _dev(d.seq_capacity), _dev(d.req_seq), _dev(emitted),
                                _dev(n_emitted), pattern=pat, pattern_len=plen, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 2
    assert np.array_equal(tok.cpu().numpy(), want[0]) and np.array_equal(ln.cpu().numpy(), want[1])
    assert np.array_equal(pat.cpu().numpy(), want[2]) and np.array_equal(plen.cpu().numpy(), want[3])
    # a request that names no sequence is skipped and reported; the others are served
    req = d.req_seq.copy()
    req[5] = len(d.seq_start) + 3
    keep = np.ones(cfg.B, bool)
    keep[5] = False
    tok, ln = _dev(d.tokens), _dev(d.seq_len)
    status.zero_()
    binding.seer_history_append(tok, _dev(d.seq_start), ln, _dev(d.seq_capacity), _dev(req), _dev(emitted), _dev(n_emitted),
                                pattern=pat, pattern_len=plen, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 3
    skipped = int(d.req_seq[5])
    assert ln.cpu().numpy()[skipped] == d.seq_len[skipped]
    others = np.delete(np.arange(len(d.seq_len)), skipped)
    assert np.array_equal(ln.cpu().numpy()[others], want[1][others])


@pytest.mark.parametrize("top_k,gamma_max", [(1, 8), (4, 4)])
def test_decode_loop_emits_exactly_the_true_sequence(top_k, gamma_max):
    """draft -> accept -> append, six steps in a row on the device.  The stand-in for the model puts the
    request's true next token on top wherever a draft node's path agrees with the true sequence, so
    whatever is drafted, the tokens appended to the histories must be the true sequence, token for token
    (Section 3.1: speculative decoding changes the speed, not the output), and every step's drafts must
    be the oracle's for the histories as they are at that step."""
    from paper_2511_14617_amd import binding
    steps, V = 6, 3001
    cfg = W.CONFIGS[2].scaled(B=16, V=V, ctx=("lognormal", 1500, 0.6, 600, 5000))
    T = 1 + top_k * gamma_max
    d = W.make_draft_inputs(cfg, seed=21, gamma_max=gamma_max, top_k=top_k, horizon=steps * (gamma_max + 1) + 1,
                            spare=steps * (gamma_max + 1), n_phrases=96, phrase_prob=0.6)
    tokens, seq_len = _dev(d.tokens), _dev(d.seq_len)
    seq_start, seq_cap, group_first = _dev(d.seq_start), _dev(d.seq_capacity), _dev(d.group_first)
    req_group, req_seq, max_spec = _dev(d.req_group), _dev(d.req_seq), _dev(d.max_spec_tokens)
    pattern, pattern_len = _dev(d.pattern), _dev(d.pattern_len)
    h_tokens, h_len, h_pat, h_plen = d.tokens.copy(), d.seq_len.copy(), d.pattern.copy(), d.pattern_len.copy()
    done = np.zeros(cfg.B, np.int64)                    # tokens of the true continuation emitted so far
    rng = np.random.default_rng(8)
    total_accepted = 0
    max_group = int(d.max_group_tokens + cfg.group_size * steps * (gamma_max + 1))
    counts = torch.zeros((3, T), dtype=torch.int64, device="cuda")     # acceptance statistics over the six steps
    h_counts = None
    for step in range(steps):
        tok, par, msk, cnt, mlen = binding.seer_draft(tokens, seq_start, seq_len, group_first, req_group, pattern,
                                                       pattern_len, max_spec, gamma_max=gamma_max, top_k=top_k,
                                                       pattern_lookup_min=d.p_min, vocab=V, max_group_tokens=max_group)
        torch.cuda.synchronize()
        h_tok, h_par = tok.cpu().numpy(), par.cpu().numpy()
        want = D.batch_speculate(h_tokens, d.seq_start, h_len, d.group_first, d.req_group, h_pat, h_plen, d.max_spec_tokens,
                                 gamma_max=gamma_max, top_k=top_k, p_min=d.p_min, p_max=d.p_max, min_confidence=0.0, vocab=V)
        assert np.array_equal(h_tok, want[0]) and np.array_equal(h_par, want[1]), "step %d" % step
        logits = rng.normal(size=(cfg.B, T, V)).astype(np.float32)
        for b in range(cfg.B):
            truth = d.future[b, done[b]:]
            depth, ok = {0: 0}, {0: True}
            logits[b, 0, truth[0]] = 9.0
            for s_ in range(1, T):
                p_ = int(h_par[b, s_])
                if p_ < 0:
                    continue
                depth[s_] = depth[p_] + 1
                ok[s_] = ok[p_] and h_tok[b, s_] == truth[depth[s_] - 1]
                if ok[s_]:
                    logits[b, s_, truth[depth[s_]]] = 9.0
        alen, path, bonus, tgt = binding.seer_accept(torch.from_numpy(logits).to("cuda"), tok, par)
        torch.cuda.synchronize()
        a_, p_, bo = alen.cpu().numpy(), path.cpu().numpy(), bonus.cpu().numpy()
        binding.seer_acceptance_stats(alen, path, par, counts)
        h_counts = stats_oracle.acceptance_counts(a_, p_, h_par, T, h_counts)
        emitted = np.full((cfg.B, T), -1, np.int32)
        for b in range(cfg.B):
            for i in range(a_[b]):
                emitted[b, i] = h_tok[b, p_[b, i + 1]]
            emitted[b, a_[b]] = bo[b]
        n_emitted = (a_ + 1).astype(np.int32)
        total_accepted += int(a_.sum())
        binding.seer_history_append(tokens, seq_start, seq_len, seq_cap, req_seq, _dev(emitted), _dev(n_emitted),
                                    pattern=pattern, pattern_len=pattern_len)
        torch.cuda.synchronize()
        h_tokens, h_len, h_pat, h_plen = D.history_append(h_tokens, d.seq_start, h_len, d.seq_capacity, d.req_seq, emitted,
                                                          n_emitted, d.p_max)
        assert np.array_equal(tokens.cpu().numpy(), h_tokens) and np.array_equal(seq_len.cpu().numpy(), h_len)
        assert np.array_equal(pattern.cpu().numpy(), h_pat) and np.array_equal(pattern_len.cpu().numpy(), h_plen)
        for b in range(cfg.B):
            assert np.array_equal(emitted[b, :n_emitted[b]], d.future[b, done[b]:done[b] + n_emitted[b]])
        done += n_emitted
    for b in range(cfg.B):                                # the histories grew by exactly the true continuation
        q = int(d.req_seq[b])
        start, old = int(d.seq_start[q]), int(d.seq_len[q])
        assert h_len[q] == old + done[b]
        assert np.array_equal(h_tokens[start + old:start + h_len[q]], d.future[b, :done[b]])
    assert total_accepted > cfg.B                         # the drafts did shorten the loop
    # the statistics of the six steps, and the draft lengths the policy takes from them (Algorithm 1)
    assert counts.cpu().tolist() == h_counts
    assert sum(h_counts[2][1:]) == total_accepted
    beta = binding.seer_acceptance_beta(h_counts, prior=0.0)
    assert beta == stats_oracle.beta_from_counts(h_counts, T) and beta[0] > 0.0
    beta = (beta + [0.0] * (gamma_max + 1))[:gamma_max + 1]
    step_time = [1.0 + 0.05 * g for g in range(gamma_max + 1)]
    assert binding.seer_mba_draft_lengths(4, 12, beta, gamma_max, 2.0, step_time) == \
        mba_oracle.mba(4, 12, beta, gamma_max, 2.0, step_time)


@pytest.mark.parametrize("seed", range(64))
def test_random_shapes(seed):
    """Seeded random batches: groups of 1..5 sequences of 0..3000 tokens (some empty), vocabularies from 3 tokens
    to thousands, any pattern window, beam width, depth and threshold, requests spread over the groups in any
    order, patterns taken from a sequence's end, from its middle, or random."""
    rng = np.random.default_rng(5000 + seed)
    vocab = int(rng.choice([3, 7, 50, 1000, 40000]))
    n_groups = int(rng.integers(1, 5))
    groups = []
    for _ in range(n_groups):
        seqs = []
        for _ in range(int(rng.integers(1, 6))):
            n = int(rng.choice([0, 1, 2, int(rng.integers(3, 400)), int(rng.integers(400, 3000))]))
            base = rng.integers(0, vocab, size=max(n // 7, 1))
            seqs.append(np.resize(base, n).tolist() if rng.random() < 0.4 else rng.integers(0, vocab, size=n).tolist())
        groups.append(seqs)
    top_k = int(rng.integers(1, 9))
    gamma_max = int(rng.integers(1, min(63 // top_k, 12) + 1))
    p_max = int(rng.integers(1, 13))
    p_min = int(rng.integers(0, p_max + 1))
    B = int(rng.integers(1, 70))
    req_group = rng.integers(0, n_groups, size=B)
    pats = []
    for b in range(B):
        seqs = [s for s in groups[req_group[b]] if len(s) >= 2]
        kind = rng.random()
        if seqs and kind < 0.45:
            s = seqs[int(rng.integers(0, len(seqs)))]
            pats.append(s[-int(rng.integers(1, p_max + 3)):])
        elif seqs and kind < 0.9:
            s = seqs[int(rng.integers(0, len(seqs)))]
            e = int(rng.integers(1, len(s)))
            pats.append(s[max(0, e - int(rng.integers(1, p_max + 3))):e])
        else:
            pats.append(rng.integers(0, vocab, size=int(rng.integers(0, p_max + 2))).tolist())
    d = _from_lists(groups, req_group, pats, gamma_max=gamma_max, top_k=top_k, p_min=p_min, p_max=p_max, vocab=vocab,
                    min_confidence=float(rng.choice([0.0, 0.0, 0.05, 0.34, 1.0])),
                    max_spec=rng.integers(0, gamma_max + 1, size=B), gap=int(rng.integers(0, 9)))
    _compare(d, "random shapes %d" % seed)


def test_many_requests_per_group_in_any_order():
    """300 requests spread at random over 5 groups: a group's requests come in several windows of request ids."""
    rng = np.random.default_rng(77)
    vocab = 60
    groups = [[rng.integers(0, vocab, size=int(rng.integers(50, 1500))).tolist() for _ in range(int(rng.integers(1, 5)))]
              for _ in range(5)]
    B = 300
    req_group = rng.integers(0, 5, size=B)
    pats = []
    for b in range(B):
        s = groups[req_group[b]][0]
        e = int(rng.integers(2, len(s)))
        pats.append(s[max(0, e - 5):e])
    d = _from_lists(groups, req_group, pats, gamma_max=5, top_k=3, p_min=2, p_max=5, vocab=vocab)
    want = _compare(d, "many requests")
    assert (want[4] >= 2).mean() > 0.9


@pytest.mark.parametrize("top_k,gamma_max", [(1, 63), (2, 31), (16, 3), (3, 21)])
def test_widest_and_deepest_trees(top_k, gamma_max):
    """The extreme tree shapes (64 slots with a 63-token chain: the last bit of the mask word; 16 members per
    level) on periodic and on phrase-like histories, where chains really run that deep."""
    rng = np.random.default_rng(top_k * 100 + gamma_max)
    period = [int(x) for x in rng.permutation(50)[:7]]
    periodic = [period * 40, period * 25 + [99], (period[3:] + period[:3]) * 30]
    phrases = [rng.integers(0, 40, size=int(rng.integers(5, 30))).tolist() for _ in range(6)]
    mixed = []
    for _ in range(4):
        s = []
        while len(s) < 2500:
            s += phrases[int(rng.integers(0, len(phrases)))]
        mixed.append(s)
    pats = [period * 2, (period * 3)[:-2], mixed[0][-6:], mixed[1][100:108], [1, 2, 3]]
    d = _from_lists([periodic, mixed], [0, 0, 1, 1, 1], pats, gamma_max=gamma_max, top_k=top_k, p_min=2, p_max=8, vocab=128)
    want = _compare(d, "extreme trees %dx%d" % (top_k, gamma_max))
    depth_reached = max(int((want[1][b] >= 0).sum()) for b in range(5))
    assert depth_reached >= min(gamma_max, 20)
