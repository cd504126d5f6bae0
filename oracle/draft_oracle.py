"""Oracle for grouped n-gram drafting: the step right before verification.

TEST INFRASTRUCTURE ONLY: plain Python over lists and numpy arrays, one request at a time;
nothing in the product path imports it and it shares no code with the library.

What the paper fixes (Section 2.3, pattern level; Section 3.4.2; Appendix A.2, draft client):
a request's draft tokens come from the token sequences that ALL requests of its prompt group
have produced so far; every request of the group keeps a path of its own in the shared
structure (no n-gram runs from one request's tokens into another's); a lookup takes the
request's most recent tokens as the pattern (SpeculationArgs: pattern_lookup_min,
pattern_lookup_max), returns at most max_spec_tokens tokens per path, scores every candidate
path by the suffix statistics, drops low-probability candidates, and returns several paths by a
beam search of width top_k.  The paper leaves the scoring and the search to prior work and gives
no listing, so the definition below is this build's reading, written out as plain counting:

  count(w)     number of places (sequence, offset) of the group where the token string w occurs
  s            the longest suffix of the request's pattern, of length p with
               max(pattern_lookup_min, 1) <= p <= min(pattern_len, pattern_lookup_max), that
               occurs somewhere FOLLOWED BY at least one more token of the same sequence;
               no such suffix -> no draft (root only)
  node         a token string c_1 .. c_d (d >= 1) with count(s c_1 .. c_d) >= 1; its confidence
               is count(s c_1 .. c_d) / n_root, n_root = sum_x count(s x): the product of the
               conditional frequencies count(s c_1..c_i) / count(s c_1..c_{i-1}) along the path,
               with the root taken as the occurrences of s that have a continuation
  filter       a node is kept iff float32(count) >= float32(min_confidence) * float32(n_root)
               (one fp32 product, then the comparison: the decision is taken in fp32)
  beam         level 0 = {root}.  Level d = the first top_k, in the order (count descending,
               rank of the parent inside level d - 1 ascending, token ascending), of the kept
               one-token extensions of the members of level d - 1; d = 1 .. max_spec_tokens,
               stopping at the first empty level.  Tokens outside [0, vocab) are never proposed.
  output       T = 1 + top_k * gamma_max slots.  Slot 0 is the root (the request's newest token).
               The member of rank j of level d sits in slot 1 + (d - 1) * top_k + j, its parent
               is the slot of its parent (0 for level 1).  EVERY member of every level is a
               draft node (a level-d member whose extensions all lost at level d + 1 stays a
               leaf).  Unused slots: token -1, parent -2, count 0, mask = own bit only.
               mask[t] = own bit | mask[parent].

With top_k = 1 this is a single chain that follows the most frequent continuation, the
single-path form the paper takes from SuffixDecoding; its Table 2 ("Linear" against
"Multi-Path") is this call with top_k = 1, 2, 4.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np


def match_length(seq: Sequence[int], i: int, pattern: Sequence[int]) -> int:
    """Largest L <= len(pattern), L <= i + 1, with seq[i - L + 1 .. i] == the last L pattern tokens."""
    L = 0
    while L < len(pattern) and L <= i and seq[i - L] == pattern[len(pattern) - 1 - L]:
        L += 1
    return L


def find_occurrences(seqs: Sequence[Sequence[int]], pattern: Sequence[int], p_min: int) -> Tuple[int, List[Tuple[int, int]]]:
    """(p, places): p = length of the longest pattern suffix (>= max(p_min, 1)) that some sequence
    holds followed by at least one more token; places = (sequence, offset of the token that follows)
    for every such occurrence.  (0, []) if there is none."""
    best = 0
    places: List[Tuple[int, int]] = []
    if len(pattern) == 0:
        return 0, []
    for s, seq in enumerate(seqs):
        # i = last token of an occurrence; i + 1 must exist.  Only places that hold the newest pattern
        # token can match at all (a vectorised pre-selection, the match itself is counted token by token)
        for i in np.flatnonzero(np.asarray(seq[:-1]) == pattern[-1]).tolist():
            m = match_length(seq, i, pattern)
            if m > best:
                best, places = m, [(s, i + 1)]
            elif m == best and m > 0:
                places.append((s, i + 1))
    if best < max(p_min, 1):
        return 0, []
    return best, places


def draft_one(seqs: Sequence[Sequence[int]], pattern: Sequence[int], *, max_spec_tokens: int, gamma_max: int,
              top_k: int, p_min: int, p_max: int, min_confidence: float, vocab: int) -> Dict[str, object]:
    """Draft tree of one request.  `pattern` = its most recent tokens, newest last."""
    T = 1 + top_k * gamma_max
    tokens = [-1] * T
    parent = [-2] * T
    count = [0] * T
    mask = [1 << t for t in range(T)]
    parent[0] = -1
    tokens[0] = int(pattern[-1]) if len(pattern) else -1
    pat = list(pattern)[-p_max:] if p_max > 0 else []
    p, places = find_occurrences(seqs, pat, p_min)
    out = {"tokens": tokens, "parent": parent, "mask": mask, "count": count, "match_len": p}
    if p == 0:
        return out
    n_root = len(places)
    count[0] = n_root
    threshold = np.float32(min_confidence) * np.float32(n_root)
    level: List[Tuple[int, List[Tuple[int, int]]]] = [(0, places)]      # (slot, places of the next token)
    for d in range(1, min(max_spec_tokens, gamma_max) + 1):
        cands = []
        for rank, (_, plc) in enumerate(level):
            tally: Dict[int, int] = {}
            for s, off in plc:
                if off < len(seqs[s]) and 0 <= seqs[s][off] < vocab:
                    tally[int(seqs[s][off])] = tally.get(int(seqs[s][off]), 0) + 1
            for x, c in tally.items():
                if np.float32(c) >= threshold:
                    cands.append((-c, rank, x))
        cands.sort()
        nxt = []
        for j, (negc, rank, x) in enumerate(cands[:top_k]):
            slot = 1 + (d - 1) * top_k + j
            pslot, plc = level[rank]
            tokens[slot], parent[slot], count[slot] = x, pslot, -negc
            mask[slot] = (1 << slot) | mask[pslot]
            nxt.append((slot, [(s, off + 1) for s, off in plc if off < len(seqs[s]) and seqs[s][off] == x]))
        if not nxt:
            break
        level = nxt
    return out


def batch_speculate(tokens: np.ndarray, seq_start: np.ndarray, seq_len: np.ndarray, group_first: np.ndarray,
                    req_group: np.ndarray, pattern: np.ndarray, pattern_len: np.ndarray, max_spec_tokens: np.ndarray,
                    *, gamma_max: int, top_k: int, p_min: int, p_max: int, min_confidence: float, vocab: int):
    """All requests of a batch.  Layout as the library's call: `tokens` is one pool, sequence q holds
    tokens[seq_start[q] : seq_start[q] + seq_len[q]], group g owns sequences group_first[g] ..
    group_first[g + 1] - 1, `pattern` is [B, p_max] right-aligned (the newest token last, the first
    p_max - pattern_len[b] entries unused).  Returns draft_tokens, tree_parent [B, T] int32,
    tree_mask [B, T] uint64, node_count [B, T] int32, match_len [B] int32."""
    B = len(req_group)
    T = 1 + top_k * gamma_max
    d_tok = np.full((B, T), -1, np.int32)
    d_par = np.full((B, T), -2, np.int32)
    d_cnt = np.zeros((B, T), np.int32)
    d_msk = np.zeros((B, T), np.uint64)
    d_len = np.zeros(B, np.int32)
    per_group: Dict[int, List[np.ndarray]] = {}
    for b in range(B):
        g = int(req_group[b])
        if g not in per_group:
            per_group[g] = [np.asarray(tokens[int(seq_start[q]): int(seq_start[q]) + int(seq_len[q])])
                            for q in range(int(group_first[g]), int(group_first[g + 1]))]
        n = int(min(max(int(pattern_len[b]), 0), p_max))
        pat = pattern[b, p_max - n:].tolist() if n > 0 else []
        r = draft_one(per_group[g], pat, max_spec_tokens=int(max_spec_tokens[b]), gamma_max=gamma_max, top_k=top_k,
                      p_min=p_min, p_max=p_max, min_confidence=min_confidence, vocab=vocab)
        d_tok[b], d_par[b], d_cnt[b] = r["tokens"], r["parent"], r["count"]
        d_msk[b] = np.array(r["mask"], dtype=np.uint64)
        d_len[b] = r["match_len"]
    return d_tok, d_par, d_msk, d_cnt, d_len


def history_append(tokens: np.ndarray, seq_start: np.ndarray, seq_len: np.ndarray, seq_capacity: np.ndarray,
                   req_seq: np.ndarray, emitted_tokens: np.ndarray, n_emitted: np.ndarray, p_max: int):
    """What a step emitted goes behind the request's own sequence (Appendix A.2: updates are kept apart per
    request); the request's pattern becomes the newest p_max tokens of that sequence, right-aligned, -1 in
    front.  A request without room for its tokens appends nothing.  Returns new (tokens, seq_len, pattern,
    pattern_len)."""
    tokens, seq_len = tokens.copy(), seq_len.copy()
    B = len(req_seq)
    pattern = np.full((B, p_max), -1, np.int32)
    pattern_len = np.zeros(B, np.int32)
    for b in range(B):
        q, n = int(req_seq[b]), int(n_emitted[b])
        start, length = int(seq_start[q]), int(seq_len[q])
        if 0 <= n <= emitted_tokens.shape[1] and length + n <= int(seq_capacity[q]):
            tokens[start + length: start + length + n] = emitted_tokens[b, :n]
            length += n
            seq_len[q] = length
        tail = tokens[start + max(0, length - p_max): start + length]
        pattern_len[b] = len(tail)
        if len(tail):
            pattern[b, p_max - len(tail):] = tail
    return tokens, seq_len, pattern, pattern_len
