"""Pins for the drafting oracle (grouped n-gram drafting: Section 2.3, pattern level; Section 3.4.2;
Appendix A.2, draft client).  The oracle works on lists of places; the checks here use other routes to the
same quantities: hand-counted examples, substring counting over an enumerated vocabulary, the regular
expression engine as string matcher, a closed form for periodic histories, and structural invariants."""
import itertools
import os
import re

import numpy as np
import pytest

from oracle import draft_oracle as D
from paper_2511_14617_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _ints(txt):
    return [int(x) for x in txt.split()]


def _golden():
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", "draft_worked_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        seqs, pat, args, mlen, tok, par, cnt = [f.strip() for f in line.split("|")]
        a = args.split()
        rows.append(dict(seqs=[_ints(s) for s in seqs.split(";")], pattern=_ints(pat), p_min=int(a[0]), p_max=int(a[1]),
                         gamma_max=int(a[2]), top_k=int(a[3]), min_confidence=float(a[4]), vocab=int(a[5]),
                         match_len=int(mlen), tokens=_ints(tok), parent=_ints(par), count=_ints(cnt)))
    return rows


def _draft(row, **over):
    kw = dict(max_spec_tokens=row["gamma_max"], gamma_max=row["gamma_max"], top_k=row["top_k"], p_min=row["p_min"],
              p_max=row["p_max"], min_confidence=row["min_confidence"], vocab=row["vocab"])
    kw.update(over)
    return D.draft_one(row["seqs"], row["pattern"], **kw)


@pytest.mark.parametrize("row", _golden())
def test_hand_counted_examples(row):
    r = _draft(row)
    assert r["match_len"] == row["match_len"]
    assert r["tokens"] == row["tokens"]
    assert r["parent"] == row["parent"]
    assert r["count"] == row["count"]


# ---------------------------------------------------------------- substring counting, tiny vocabulary --
def _count(seqs, w):
    """Occurrences of the token string w, counted window by window."""
    n = len(w)
    return sum(1 for s in seqs for j in range(len(s) - n + 1) if list(s[j:j + n]) == list(w))


def _draft_by_substring_counting(seqs, pattern, gamma, top_k, p_min, p_max, min_conf, vocab):
    """The definition read as statements about strings: every candidate token of the vocabulary is tried."""
    pat = list(pattern)[-p_max:]
    suffix = None
    for p in range(len(pat), max(p_min, 1) - 1, -1):
        s = pat[len(pat) - p:]
        if sum(_count(seqs, s + [x]) for x in range(-1, vocab + 3)) > 0:      # followed by any token at all
            suffix = s
            break
    T = 1 + top_k * gamma
    tokens, parent, count = [-1] * T, [-2] * T, [0] * T
    tokens[0], parent[0] = (pattern[-1] if len(pattern) else -1), -1
    if suffix is None:
        return 0, tokens, parent, count
    n_root = sum(_count(seqs, suffix + [x]) for x in range(-1, vocab + 3))
    count[0] = n_root
    level = [(0, [])]
    for d in range(1, gamma + 1):
        cands = []
        for rank, (_, path) in enumerate(level):
            for x in range(vocab):
                c = _count(seqs, suffix + path + [x])
                if c >= 1 and np.float32(c) >= np.float32(min_conf) * np.float32(n_root):
                    cands.append((-c, rank, x))
        cands.sort()
        nxt = []
        for j, (negc, rank, x) in enumerate(cands[:top_k]):
            slot = 1 + (d - 1) * top_k + j
            tokens[slot], parent[slot], count[slot] = x, level[rank][0], -negc
            nxt.append((slot, level[rank][1] + [x]))
        if not nxt:
            break
        level = nxt
    return len(suffix), tokens, parent, count


@pytest.mark.parametrize("seed", range(60))
def test_against_substring_counting_on_tiny_inputs(seed):
    rng = np.random.default_rng(1000 + seed)
    vocab = int(rng.integers(2, 5))
    n_seq = int(rng.integers(1, 4))
    # tokens up to vocab + 1: some lie outside the vocabulary
    seqs = [rng.integers(0, vocab + (seed % 3 == 0) * 2, size=int(rng.integers(0, 14))).tolist() for _ in range(n_seq)]
    p_max = int(rng.integers(1, 5))
    p_min = int(rng.integers(0, p_max + 1))
    pattern = rng.integers(0, vocab, size=int(rng.integers(0, p_max + 2))).tolist()
    gamma = int(rng.integers(1, 4))
    top_k = int(rng.integers(1, 4))
    min_conf = float(rng.choice([0.0, 0.0, 0.25, 0.5, 1.0]))
    r = D.draft_one(seqs, pattern, max_spec_tokens=gamma, gamma_max=gamma, top_k=top_k, p_min=p_min, p_max=p_max,
                    min_confidence=min_conf, vocab=vocab)
    mlen, tokens, parent, count = _draft_by_substring_counting(seqs, pattern, gamma, top_k, p_min, p_max, min_conf, vocab)
    assert (r["match_len"], r["tokens"], r["parent"], r["count"]) == (mlen, tokens, parent, count)


def test_exhaustive_two_token_vocabulary():
    """Every pair of histories up to length 4 over {0, 1}, every pattern up to length 2."""
    hist = [list(h) for n in range(0, 5) for h in itertools.product((0, 1), repeat=n)]
    pats = [list(p) for n in range(1, 3) for p in itertools.product((0, 1), repeat=n)]
    checked = 0
    for a in hist[::2]:
        for b in hist[::3]:
            for pat in pats:
                r = D.draft_one([a, b], pat, max_spec_tokens=2, gamma_max=2, top_k=2, p_min=1, p_max=2,
                                min_confidence=0.0, vocab=2)
                want = _draft_by_substring_counting([a, b], pat, 2, 2, 1, 2, 0.0, 2)
                assert (r["match_len"], r["tokens"], r["parent"], r["count"]) == want
                checked += 1
    assert checked > 500


# ---------------------------------------------------------------- the regex engine as string matcher --
def _regex_count(seqs, w):
    """Overlapping occurrences of w by the regular-expression engine over byte strings (tokens < 256)."""
    pat = re.compile(b"(?=" + re.escape(bytes(w)) + b")")
    return sum(len(pat.findall(bytes(s))) for s in seqs)


@pytest.mark.parametrize("seed", range(8))
def test_node_counts_equal_library_string_matching(seed):
    cfg = W.CONFIGS[1].scaled(V=200, B=8, group_size=4)
    d = W.make_draft_inputs(cfg, seed=77 + seed, gamma_max=4, top_k=3, p_min=1, p_max=4, n_phrases=24, phrase_prob=0.6)
    out = D.batch_speculate(d.tokens, d.seq_start, d.seq_len, d.group_first, d.req_group, d.pattern, d.pattern_len,
                            d.max_spec_tokens, gamma_max=4, top_k=3, p_min=1, p_max=4, min_confidence=0.0, vocab=200)
    tok, par, msk, cnt, mlen = out
    some = 0
    for b in range(cfg.B):
        g = int(d.req_group[b])
        seqs = [d.tokens[d.seq_start[q]:d.seq_start[q] + d.seq_len[q]].tolist()
                for q in range(d.group_first[g], d.group_first[g + 1])]
        p = int(mlen[b])
        if p == 0:
            continue
        suffix = d.pattern[b, d.p_max - p:].tolist()
        # the match is the LONGEST: one more pattern token in front occurs nowhere with a continuation
        if p < min(int(d.pattern_len[b]), d.p_max):
            longer = d.pattern[b, d.p_max - p - 1:].tolist()
            assert sum(_regex_count(seqs, longer + [x]) for x in range(200)) == 0
        assert cnt[b, 0] == sum(_regex_count(seqs, suffix + [x]) for x in range(200))
        for t in range(1, tok.shape[1]):
            if par[b, t] < 0:
                continue
            path, u = [], t
            while u > 0:
                path.append(int(tok[b, u]))
                u = int(par[b, u])
            assert cnt[b, t] == _regex_count(seqs, suffix + path[::-1])
            some += 1
    assert some > 10


# ---------------------------------------------------------------- closed form: periodic history --
@pytest.mark.parametrize("period,reps,gamma", [(4, 6, 8), (3, 5, 7), (5, 3, 9), (1, 9, 4)])
def test_periodic_history_closed_form(period, reps, gamma):
    """One sequence = a period of distinct tokens repeated `reps` times; the pattern is its last `period`
    tokens.  The chain must continue the period; a draft of depth d is backed by reps - 1 - floor((d - 1) /
    period) places (those whose continuation still fits before the end of the sequence)."""
    seq = list(range(10, 10 + period)) * reps
    r = D.draft_one([seq], seq[-period:], max_spec_tokens=gamma, gamma_max=gamma, top_k=1, p_min=1, p_max=period,
                    min_confidence=0.0, vocab=64)
    assert r["match_len"] == period and r["count"][0] == reps - 1
    for dpt in range(1, gamma + 1):
        backing = reps - 1 - (dpt - 1) // period
        if backing >= 1:
            assert r["tokens"][dpt] == seq[(dpt - 1) % period]
            assert r["count"][dpt] == backing and r["parent"][dpt] == dpt - 1
        else:
            assert r["tokens"][dpt] == -1 and r["parent"][dpt] == -2


# ---------------------------------------------------------------- structure of the returned tree --
@pytest.mark.parametrize("top_k,gamma_max", [(1, 8), (2, 6), (4, 8), (7, 9)])
def test_tree_invariants_on_grouped_histories(top_k, gamma_max):
    cfg = W.CONFIGS[2].scaled(B=16, ctx=("lognormal", 1500, 0.6, 600, 6000))
    d = W.make_draft_inputs(cfg, gamma_max=gamma_max, top_k=top_k, p_min=1, p_max=6, min_confidence=0.02)
    rng = np.random.default_rng(5)
    d.max_spec_tokens[:] = rng.integers(0, gamma_max + 1, size=cfg.B)
    tok, par, msk, cnt, mlen = D.batch_speculate(
        d.tokens, d.seq_start, d.seq_len, d.group_first, d.req_group, d.pattern, d.pattern_len, d.max_spec_tokens,
        gamma_max=gamma_max, top_k=top_k, p_min=1, p_max=6, min_confidence=0.02, vocab=d.vocab)
    T = 1 + top_k * gamma_max
    assert tok.shape == (cfg.B, T)
    for b in range(cfg.B):
        assert par[b, 0] == -1 and tok[b, 0] == d.pattern[b, -1]
        depth = {0: 0}
        for t in range(1, T):
            level = 1 + (t - 1) // top_k
            if par[b, t] == -2:
                assert tok[b, t] == -1 and cnt[b, t] == 0 and int(msk[b, t]) == 1 << t
                continue
            p = int(par[b, t])
            assert 0 <= p < t and par[b, p] != -2
            depth[t] = depth[p] + 1
            assert depth[t] == level <= d.max_spec_tokens[b]
            assert 1 <= cnt[b, t] <= cnt[b, p]                         # confidence never grows along a path
            assert np.float32(cnt[b, t]) >= np.float32(0.02) * np.float32(cnt[b, 0])
            assert int(msk[b, t]) == (1 << t) | int(msk[b, p])
            sib = [u for u in range(1, t) if par[b, u] == p]
            assert all(tok[b, u] != tok[b, t] for u in sib)           # children of one node are distinct tokens
            if (t - 1) % top_k:                                       # ranks inside a level are ordered
                prev = t - 1
                assert par[b, prev] != -2
                key = lambda u: (-int(cnt[b, u]), int(par[b, u]), int(tok[b, u]))
                assert key(prev) < key(t)
        for p in set(int(x) for x in par[b] if x >= 0):
            assert sum(int(cnt[b, u]) for u in range(1, T) if par[b, u] == p) <= cnt[b, p]


def test_width_one_is_the_greedy_chain_and_wider_beams_contain_it():
    cfg = W.CONFIGS[2].scaled(B=16, ctx=("lognormal", 1500, 0.6, 600, 6000))
    d = W.make_draft_inputs(cfg, gamma_max=6, top_k=1, p_min=2, p_max=6)
    kw = dict(gamma_max=6, p_min=2, p_max=6, min_confidence=0.0, vocab=d.vocab)
    args = (d.tokens, d.seq_start, d.seq_len, d.group_first, d.req_group, d.pattern, d.pattern_len, d.max_spec_tokens)
    t1, p1, _, c1, _ = D.batch_speculate(*args, top_k=1, **kw)
    t3, p3, _, c3, _ = D.batch_speculate(*args, top_k=3, **kw)
    for b in range(cfg.B):
        # rank 0 of every level of the wide beam is its best node; the chain's first token is that node
        assert t1[b, 1] == t3[b, 1] and c1[b, 1] == c3[b, 1]
        # the chain is a root path; all of it that the wide beam kept has the same counts
        node = 0
        for dpt in range(1, 7):
            if p1[b, dpt] == -2:
                break
            kids = [u for u in range(1, t3.shape[1]) if p3[b, u] == node and t3[b, u] == t1[b, dpt]]
            if not kids:
                break
            node = kids[0]
            assert c3[b, node] == c1[b, dpt]


def test_more_references_and_more_paths_accept_more():
    """The trend of the paper's Table 2 on the synthetic groups: drafts from the whole group's history are
    accepted further than drafts from the request's own history, and a wider beam never accepts less."""
    cfg = W.CONFIGS[2]

    def mean_accepted(d, tok, par):
        tot = 0
        for b in range(tok.shape[0]):
            ok, depth, best = {0: True}, {0: 0}, 0
            for t in range(1, tok.shape[1]):
                p = int(par[b, t])
                if p < 0:
                    continue
                depth[t] = depth[p] + 1
                ok[t] = ok[p] and tok[b, t] == d.future[b, depth[t] - 1]
                if ok[t]:
                    best = max(best, depth[t])
            tot += best + 1
        return tot / tok.shape[0]

    res = {}
    for name, kw in (("own", dict(own_only=True)), ("group", dict())):
        for k in (1, 4):
            d = W.make_draft_inputs(cfg, top_k=k, **kw)
            tok, par, _, _, _ = D.batch_speculate(d.tokens, d.seq_start, d.seq_len, d.group_first, d.req_group, d.pattern,
                                                  d.pattern_len, d.max_spec_tokens, gamma_max=d.gamma_max, top_k=k,
                                                  p_min=d.p_min, p_max=d.p_max, min_confidence=0.0, vocab=d.vocab)
            res[name, k] = mean_accepted(d, tok, par)
    assert res["group", 1] > res["own", 1] + 0.2
    assert res["group", 4] >= res["group", 1] and res["own", 4] >= res["own", 1]


# ---------------------------------------------------------------- appending what a step emitted --
def test_history_append_against_list_concatenation_and_composition():
    cfg = W.CONFIGS[1].scaled(V=500, B=8, group_size=4)
    d = W.make_draft_inputs(cfg, seed=3, gamma_max=4, top_k=1, p_max=6, spare=12)
    rng = np.random.default_rng(0)
    T = 5
    e1 = rng.integers(0, 500, size=(cfg.B, T)).astype(np.int32)
    e2 = rng.integers(0, 500, size=(cfg.B, T)).astype(np.int32)
    n1 = rng.integers(0, T + 1, size=cfg.B).astype(np.int32)
    n2 = rng.integers(0, T + 1, size=cfg.B).astype(np.int32)
    seqs = [d.tokens[s:s + n].tolist() for s, n in zip(d.seq_start, d.seq_len)]
    t1, l1, p1, pl1 = D.history_append(d.tokens, d.seq_start, d.seq_len, d.seq_capacity, d.req_seq, e1, n1, d.p_max)
    t2, l2, p2, pl2 = D.history_append(t1, d.seq_start, l1, d.seq_capacity, d.req_seq, e2, n2, d.p_max)
    touched = np.zeros(len(d.tokens), bool)
    for b in range(cfg.B):
        q = int(d.req_seq[b])
        grown = seqs[q] + e1[b, :n1[b]].tolist() + e2[b, :n2[b]].tolist()
        assert t2[d.seq_start[q]:d.seq_start[q] + l2[q]].tolist() == grown
        tail = grown[-d.p_max:]
        assert pl2[b] == len(tail) and p2[b, d.p_max - len(tail):].tolist() == tail and (p2[b, :d.p_max - len(tail)] == -1).all()
        touched[d.seq_start[q] + d.seq_len[q]:d.seq_start[q] + l2[q]] = True
    assert np.array_equal(t2[~touched], d.tokens[~touched])            # nothing else in the pool moved
    # two steps in one call (tokens joined) give the same histories
    both = np.full((cfg.B, 2 * T), -1, np.int32)
    for b in range(cfg.B):
        both[b, :n1[b] + n2[b]] = e1[b, :n1[b]].tolist() + e2[b, :n2[b]].tolist()
    t12, l12, p12, pl12 = D.history_append(d.tokens, d.seq_start, d.seq_len, d.seq_capacity, d.req_seq, both, n1 + n2, d.p_max)
    assert np.array_equal(t12, t2) and np.array_equal(l12, l2) and np.array_equal(p12, p2) and np.array_equal(pl12, pl2)
    # a sequence without room for all of a step's tokens takes none of them
    cap = d.seq_capacity.copy()
    q0 = int(d.req_seq[0])
    cap[q0] = d.seq_len[q0] + 2
    n = np.full(cfg.B, 3, np.int32)
    t3, l3, p3, pl3 = D.history_append(d.tokens, d.seq_start, d.seq_len, cap, d.req_seq, e1, n, d.p_max)
    assert l3[q0] == d.seq_len[q0] and p3[0, -1] == seqs[q0][-1] and l3[int(d.req_seq[1])] == d.seq_len[int(d.req_seq[1])] + 3


def test_decode_loop_with_the_oracles_emits_the_true_sequence():
    """Draft, verify against a stand-in model that knows the true continuation, append: whatever is drafted,
    what reaches the histories is the true sequence (Section 3.1: the output is that of plain decoding), and a
    step emits accepted + 1 tokens (Section 3.4.1)."""
    import oracle
    cfg = W.CONFIGS[2].scaled(B=8, V=997, ctx=("lognormal", 1200, 0.6, 600, 4000))
    gamma, top_k, steps = 4, 2, 5
    d = W.make_draft_inputs(cfg, seed=5, gamma_max=gamma, top_k=top_k, horizon=steps * (gamma + 1) + 1,
                            spare=steps * (gamma + 1), n_phrases=64, phrase_prob=0.6)
    tokens, lens, pat, plen = d.tokens, d.seq_len, d.pattern, d.pattern_len
    done = np.zeros(cfg.B, np.int64)
    T = 1 + top_k * gamma
    for _ in range(steps):
        tok, par, msk, cnt, mlen = D.batch_speculate(tokens, d.seq_start, lens, d.group_first, d.req_group, pat, plen,
                                                     d.max_spec_tokens, gamma_max=gamma, top_k=top_k, p_min=d.p_min,
                                                     p_max=d.p_max, min_confidence=0.0, vocab=cfg.V)
        target = np.zeros((cfg.B, T), np.int32)
        for b in range(cfg.B):
            truth = d.future[b, done[b]:]
            depth, ok = {0: 0}, {0: True}
            target[b, 0] = truth[0]
            for s in range(1, T):
                if par[b, s] < 0:
                    continue
                depth[s] = depth[int(par[b, s])] + 1
                ok[s] = ok[int(par[b, s])] and tok[b, s] == truth[depth[s] - 1]
                target[b, s] = truth[depth[s]] if ok[s] else (tok[b, s] + 1) % cfg.V
        alen, path, bonus = oracle.accept(target, tok, par)
        emitted, n_emitted = oracle.emitted_tokens(tok, alen, path, bonus)
        assert np.array_equal(n_emitted, alen + 1)
        for b in range(cfg.B):
            assert np.array_equal(emitted[b, :n_emitted[b]], d.future[b, done[b]:done[b] + n_emitted[b]])
        tokens, lens, pat, plen = D.history_append(tokens, d.seq_start, lens, d.seq_capacity, d.req_seq, emitted, n_emitted, d.p_max)
        done += n_emitted
    assert done.sum() > cfg.B * steps                      # some drafts were accepted
