"""Seeded synthetic inputs for batched draft verification.

This module only *draws* inputs: context lengths, page tables, K/V/Q values,
draft chains and trees, logits.  It holds none of the method's arithmetic (no
attention, softmax, argmax or acceptance rule); both the CPU oracle's tests and
the HIP path's tests feed on the arrays it returns, so the two sides see
identical bits.  Everything is numpy on the host, seeded with PCG64.

Workload shapes follow the paper's evaluation setup (Table 3, the model
configurations and workload characteristics: group size 8 or 16, generation
lengths up to ~98k tokens; Section 3.4: batch sizes from a handful of
stragglers to several hundred, draft length gamma_max = 8, a 16-token baseline,
multi-path drafts with k = 4 in the long-tail stage).  The paper's own traces
and weights are not public, so the five named configurations below stand in for
them by shape only.

Conventions shared by every array produced here
-----------------------------------------------
* bf16 tensors are carried as ``uint16`` bit patterns (round-to-nearest-even
  from fp32) so that no library's bf16 type is needed on the host.
* ``ctx_len[b]`` counts the T verify positions: they are the last T logical
  positions of request b, slot s at logical position ``ctx_len[b] - T + s``.
* The KV pool is ``[num_pages, Hkv, page_size, D]``; a request's logical
  position j lives in page ``block_table[b, j // page_size]``, slot
  ``j % page_size``.
* Slot 0 of a draft is the last already-accepted token (tree root); slots
  1..T-1 are draft tokens.  ``tree_parent[b, 0] = -1``, ``0 <= parent[t] < t``,
  ``-2`` marks a padded (unused) slot.  ``tree_mask[b, t]`` has bit s set iff
  slot s is t itself or an ancestor of t.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 20251114

_CHUNK = 1 << 24  # values per generation chunk (fixed: part of the recipe)


# --------------------------------------------------------------------------
# format helpers (input preparation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(u16: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(seed_seq: np.random.SeedSequence, n: int, scale: float, threads: int = 8) -> np.ndarray:
    """n values ~ N(0,1)*scale as bf16 bits.  Chunked so that the stream does not
    depend on the thread count: chunk c always uses child seed c."""
    out = np.empty(n, dtype=np.uint16)
    nchunks = (n + _CHUNK - 1) // _CHUNK
    children = seed_seq.spawn(nchunks)

    def work(c: int) -> None:
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        g = np.random.Generator(np.random.PCG64(children[c]))
        x = g.standard_normal(hi - lo, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        out[lo:hi] = f32_to_bf16_bits(x)

    if nchunks <= 1 or threads <= 1:
        for c in range(nchunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(nchunks)))
    return out


def _normal_f32(seed_seq: np.random.SeedSequence, n: int, threads: int = 8) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    nchunks = (n + _CHUNK - 1) // _CHUNK
    children = seed_seq.spawn(nchunks)

    def work(c: int) -> None:
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        g = np.random.Generator(np.random.PCG64(children[c]))
        g.standard_normal(hi - lo, dtype=np.float32, out=out[lo:hi])

    if nchunks <= 1 or threads <= 1:
        for c in range(nchunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(nchunks)))
    return out


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class VerifyConfig:
    """One verification workload.  ``ctx`` is ("uniform", lo, hi) or
    ("lognormal", median, sigma, lo, hi); lengths include the T verify slots.
    ``tree`` is None (linear chain) or (n_paths, path_len)."""

    name: str
    config_id: int
    B: int
    group_size: int
    Hq: int
    Hkv: int
    Dqk: int
    Dv: int
    page_size: int
    T: int
    V: int
    ctx: Tuple
    shared_prefix: int = 0
    tree: Optional[Tuple[int, int]] = None
    shared_latent: bool = False

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.config_id

    @property
    def ctx_hi(self) -> int:
        return int(self.ctx[-1])

    @property
    def softmax_scale(self) -> float:
        return float(self.Dqk) ** -0.5

    def scaled(self, **kw) -> "VerifyConfig":
        """A copy with some fields replaced (reduced sizes for CPU-checkable cases)."""
        return dataclasses.replace(self, **kw)


CONFIGS = {
    1: VerifyConfig("tiny_chain", 1, B=4, group_size=4, Hq=8, Hkv=2, Dqk=128, Dv=128, page_size=16,
                    T=5, V=1024, ctx=("uniform", 64, 512)),
    2: VerifyConfig("grouped_rollout_8b", 2, B=64, group_size=8, Hq=32, Hkv=8, Dqk=128, Dv=128,
                    page_size=16, T=9, V=152064, ctx=("lognormal", 4096, 0.8, 512, 32768),
                    shared_prefix=512),
    3: VerifyConfig("long_tail", 3, B=8, group_size=8, Hq=32, Hkv=8, Dqk=128, Dv=128, page_size=16,
                    T=17, V=152064, ctx=("uniform", 65536, 131072)),
    4: VerifyConfig("mla_latent", 4, B=32, group_size=8, Hq=128, Hkv=1, Dqk=576, Dv=512, page_size=64,
                    T=5, V=163840, ctx=("uniform", 8192, 24576), shared_latent=True),
    5: VerifyConfig("multipath_tree", 5, B=128, group_size=8, Hq=32, Hkv=8, Dqk=128, Dv=128,
                    page_size=16, T=33, V=152064, ctx=("lognormal", 8192, 0.8, 1024, 32768),
                    shared_prefix=512, tree=(4, 8)),
}


def draw_ctx_len(cfg: VerifyConfig, rng: np.random.Generator) -> np.ndarray:
    kind = cfg.ctx[0]
    if kind == "uniform":
        _, lo, hi = cfg.ctx
        n = rng.integers(lo, hi + 1, size=cfg.B)
    elif kind == "lognormal":
        _, median, sigma, lo, hi = cfg.ctx
        n = np.rint(np.exp(np.log(median) + sigma * rng.standard_normal(cfg.B)))
        n = np.clip(n, lo, hi)
    elif kind == "fixed":
        n = np.asarray(cfg.ctx[1], dtype=np.int64)
        assert n.shape == (cfg.B,)
    else:
        raise ValueError(kind)
    n = np.maximum(n.astype(np.int64), cfg.T)
    return n.astype(np.int32)


# --------------------------------------------------------------------------
# draft trees
# --------------------------------------------------------------------------
def chain_parent(B: int, T: int) -> np.ndarray:
    p = np.tile(np.arange(-1, T - 1, dtype=np.int32), (B, 1))
    return p


def ancestor_masks(parent: np.ndarray) -> np.ndarray:
    """Bit s of mask[b, t] set iff s == t or s is an ancestor of t.  Padded slots
    (parent == -2) see only themselves."""
    B, T = parent.shape
    assert T <= 64
    mask = np.zeros((B, T), dtype=np.uint64)
    for t in range(T):
        own = np.uint64(1) << np.uint64(t)
        p = parent[:, t]
        has = p >= 0
        inherited = np.where(has, mask[np.arange(B), np.where(has, p, 0)], np.uint64(0))
        mask[:, t] = inherited | own
    return mask


def multipath_parent(B: int, n_paths: int, path_len: int, rng: np.random.Generator,
                     dedup_fraction: float = 0.0) -> np.ndarray:
    """Root + n_paths chains of path_len nodes.  With probability dedup_fraction a
    request's paths share a seeded common trunk (a deduplicated trie): it then has
    fewer nodes and the remaining slots are padded with parent = -2."""
    T = 1 + n_paths * path_len
    parent = np.full((B, T), -2, dtype=np.int32)
    parent[:, 0] = -1
    for b in range(B):
        if dedup_fraction > 0.0 and rng.random() < dedup_fraction and path_len >= 2:   # one-node paths have no trunk to share
            trunk = int(rng.integers(1, path_len))  # shared trunk length 1..path_len-1
            t = 1
            prev = 0
            for _ in range(trunk):
                parent[b, t] = prev
                prev = t
                t += 1
            trunk_end = prev
            for _p in range(n_paths):
                prev = trunk_end
                for _ in range(path_len - trunk):
                    parent[b, t] = prev
                    prev = t
                    t += 1
        else:
            t = 1
            for _p in range(n_paths):
                prev = 0
                for _ in range(path_len):
                    parent[b, t] = prev
                    prev = t
                    t += 1
    return parent


# --------------------------------------------------------------------------
# attention inputs
# --------------------------------------------------------------------------
@dataclass
class AttentionInputs:
    cfg: VerifyConfig
    q: np.ndarray            # [B,T,Hq,Dqk] uint16 (bf16 bits)
    k_pages: np.ndarray      # [num_pages,Hkv,P,Dqk] uint16
    v_pages: Optional[np.ndarray]  # [num_pages,Hkv,P,Dv] uint16, None when the latent is shared
    block_table: np.ndarray  # [B,max_pages_per_seq] int32
    ctx_len: np.ndarray      # [B] int32
    tree_parent: Optional[np.ndarray]  # [B,T] int32 or None (chain)
    tree_mask: Optional[np.ndarray]    # [B,T] uint64 or None (chain)
    scale: float
    num_pages: int
    max_pages_per_seq: int
    unique_kv_bytes: int     # bytes of K and V in pages that at least one request reads
    logical_kv_bytes: int    # the same counted once per request (shared pages counted again)


def make_attention_inputs(cfg: VerifyConfig, seed: Optional[int] = None, *, values: str = "paper",
                          dedup_fraction: float = 0.0, max_pages_per_seq: Optional[int] = None,
                          threads: int = 8) -> AttentionInputs:
    """Draw one batch of verify-attention inputs.

    values = "paper":  Q, K, V ~ N(0,1)/sqrt(D) (the stated benchmark distribution).
    values = "peaked": K, V ~ N(0,1), Q ~ N(0,1)*4/(scale*sqrt(Dqk)) so that scaled scores have
                       standard deviation about 4: the softmax concentrates on a few keys
                       and every output element is O(1), which gives the tolerance teeth.
    Slots past ctx_len in a request's last page, and pages no request owns, hold
    +-1e4 so that a read past the end is loud.  Unused block-table entries point
    at such unowned pages (in range on purpose: a stray read must stay in bounds).
    """
    seed = cfg.seed if seed is None else seed
    ss = np.random.SeedSequence([seed, 1])
    s_len, s_perm, s_k, s_v, s_q, s_tree = ss.spawn(6)
    rng = np.random.Generator(np.random.PCG64(s_len))
    P = cfg.page_size
    B, T = cfg.B, cfg.T

    ctx_len = draw_ctx_len(cfg, rng)
    n_pages_b = (ctx_len.astype(np.int64) + P - 1) // P

    # logical -> unique page ids; the first pages of a group are shared when they
    # lie wholly inside both the shared prompt prefix and the request's own prefix
    logical = []
    next_id = 0
    group_first = {}
    for b in range(B):
        g = b // cfg.group_size
        n0 = int(ctx_len[b]) - T
        n_shared = min(cfg.shared_prefix, max(n0, 0)) // P if cfg.shared_prefix else 0
        ids = np.empty(int(n_pages_b[b]), dtype=np.int64)
        if n_shared:
            have = group_first.get(g)
            if have is None or len(have) < n_shared:
                old = 0 if have is None else len(have)
                extra = np.arange(next_id, next_id + (n_shared - old), dtype=np.int64)
                next_id += n_shared - old
                have = extra if have is None else np.concatenate([have, extra])
                group_first[g] = have
            ids[:n_shared] = have[:n_shared]
        own = len(ids) - n_shared
        ids[n_shared:] = np.arange(next_id, next_id + own, dtype=np.int64)
        next_id += own
        logical.append(ids)
    n_unique = next_id
    n_decoy = max(2, (n_unique + 9) // 10)
    num_pages = n_unique + n_decoy
    prng = np.random.Generator(np.random.PCG64(s_perm))
    perm = prng.permutation(num_pages).astype(np.int32)  # unique id -> physical page
    decoys = perm[n_unique:]

    if max_pages_per_seq is None:
        max_pages_per_seq = max(int(n_pages_b.max()), (cfg.ctx_hi + P - 1) // P)
    assert max_pages_per_seq >= int(n_pages_b.max())
    block_table = decoys[prng.integers(0, n_decoy, size=(B, max_pages_per_seq))].astype(np.int32)
    for b in range(B):
        block_table[b, : len(logical[b])] = perm[logical[b]]

    if values == "paper":
        k_scale = float(cfg.Dqk) ** -0.5
        v_scale = float(cfg.Dqk) ** -0.5
        q_scale = float(cfg.Dqk) ** -0.5
    elif values == "peaked":
        k_scale = 1.0
        v_scale = 1.0
        q_scale = 4.0 / (cfg.softmax_scale * float(cfg.Dqk) ** 0.5)
    else:
        raise ValueError(values)

    k_pages = _normal_bf16(s_k, num_pages * cfg.Hkv * P * cfg.Dqk, k_scale, threads).reshape(
        num_pages, cfg.Hkv, P, cfg.Dqk)
    if cfg.shared_latent:
        v_pages = None
    else:
        v_pages = _normal_bf16(s_v, num_pages * cfg.Hkv * P * cfg.Dv, v_scale, threads).reshape(
            num_pages, cfg.Hkv, P, cfg.Dv)
    q = _normal_bf16(s_q, B * T * cfg.Hq * cfg.Dqk, q_scale, 1).reshape(B, T, cfg.Hq, cfg.Dqk)

    big = f32_to_bf16_bits(np.array([1.0e4, -1.0e4], dtype=np.float32))
    for pg in decoys:
        k_pages[pg].reshape(-1)[0::2] = big[0]
        k_pages[pg].reshape(-1)[1::2] = big[1]
        if v_pages is not None:
            v_pages[pg].reshape(-1)[0::2] = big[1]
            v_pages[pg].reshape(-1)[1::2] = big[0]
    for b in range(B):
        used = int(ctx_len[b]) % P
        if used:
            pg = block_table[b, int(n_pages_b[b]) - 1]
            k_pages[pg, :, used:, 0::2] = big[0]
            k_pages[pg, :, used:, 1::2] = big[1]
            if v_pages is not None:
                v_pages[pg, :, used:, 0::2] = big[1]
                v_pages[pg, :, used:, 1::2] = big[0]

    if cfg.tree is None:
        tree_parent = None
        tree_mask = None
    else:
        trng = np.random.Generator(np.random.PCG64(s_tree))
        tree_parent = multipath_parent(B, cfg.tree[0], cfg.tree[1], trng, dedup_fraction)
        assert tree_parent.shape[1] == T
        tree_mask = ancestor_masks(tree_parent)

    per_page = cfg.Hkv * P * (cfg.Dqk + (0 if cfg.shared_latent else cfg.Dv)) * 2
    return AttentionInputs(cfg=cfg, q=q, k_pages=k_pages, v_pages=v_pages, block_table=block_table,
                           ctx_len=ctx_len, tree_parent=tree_parent, tree_mask=tree_mask,
                           scale=cfg.softmax_scale, num_pages=num_pages,
                           max_pages_per_seq=max_pages_per_seq,
                           unique_kv_bytes=n_unique * per_page,
                           logical_kv_bytes=int(n_pages_b.sum()) * per_page)


# --------------------------------------------------------------------------
# acceptance inputs
# --------------------------------------------------------------------------
@dataclass
class AcceptInputs:
    cfg: VerifyConfig
    logits: np.ndarray               # [B,T,V] float32
    draft_tokens: np.ndarray         # [B,T] int32
    tree_parent: Optional[np.ndarray]  # [B,T] int32 or None (chain)
    planted_len: np.ndarray          # [B] int32: accepted draft tokens by construction
    planted_target: np.ndarray       # [B,T] int32: the token whose logit was raised, per slot


def make_accept_inputs(cfg: VerifyConfig, seed: Optional[int] = None, *,
                       tree_parent: Optional[np.ndarray] = None, planted_len: Optional[np.ndarray] = None,
                       duplicate_every: int = 8, threads: int = 8) -> AcceptInputs:
    """Logits ~ N(0,1) with one entry per (request, slot) raised to 7.5 + U[0,1) so that the
    target token of each slot is known by construction (no search is done here), and draft
    tokens that follow those targets down to a planted depth and then deviate.

    Chain: draft[i] = target[i-1] for 1 <= i <= a_b, draft[a_b+1] != target[a_b], rest random.
    Tree (tree_parent given): one path carries the planted depth; every other path copies the
    planted path's tokens down to a seeded depth (never deeper than the planted one) and then
    deviates.  Slots whose token history from the root is identical get identical logits
    rows, as a model would give them.  In every `duplicate_every`-th request at least one
    other path repeats the planted path's first token.
    """
    seed = cfg.seed if seed is None else seed
    ss = np.random.SeedSequence([seed, 2])
    s_logit, s_rest = ss.spawn(2)
    rng = np.random.Generator(np.random.PCG64(s_rest))
    B, T, V = cfg.B, cfg.T, cfg.V

    logits = _normal_f32(s_logit, B * T * V, threads).reshape(B, T, V)
    target = rng.integers(0, V, size=(B, T)).astype(np.int32)
    bump = (7.5 + rng.random(size=(B, T))).astype(np.float32)
    draft = rng.integers(0, V, size=(B, T)).astype(np.int32)

    def other_than(tok: int, *avoid: int) -> int:
        c = (tok + 1 + int(rng.integers(0, max(V - 1, 1)))) % V
        while c == tok or c in avoid:
            c = (c + 1) % V
        return int(c)

    if tree_parent is None:
        if planted_len is None:
            planted_len = rng.integers(0, T, size=B).astype(np.int32)
        planted_len = np.asarray(planted_len, dtype=np.int32)
        bi = np.arange(B)[:, None]
        ti = np.arange(T)[None, :]
        logits[bi, ti, target] = bump
        for b in range(B):
            a = int(planted_len[b])
            for i in range(1, a + 1):
                draft[b, i] = target[b, i - 1]
            if a + 1 < T and V > 1:
                draft[b, a + 1] = other_than(int(target[b, a]))
            # slots past a+1 stay random: they hang below a rejected node
        return AcceptInputs(cfg, logits, draft, None, planted_len, target)

    tree_parent = np.asarray(tree_parent, dtype=np.int32)
    assert tree_parent.shape == (B, T)
    out_len = np.zeros(B, dtype=np.int32)
    for b in range(B):
        par = tree_parent[b]
        children = {}
        for t in range(1, T):
            if par[t] >= 0:
                children.setdefault(int(par[t]), []).append(t)
        leaves = [t for t in range(T) if par[t] >= -1 and t not in children and (t == 0 or par[t] >= 0)]

        def root_path(t):
            p = []
            while t > 0:
                p.append(t)
                t = int(par[t])
            return p[::-1]

        paths = [root_path(l) for l in leaves if l != 0]
        if not paths:
            logits[b, np.arange(T), target[b]] = bump[b]
            continue
        star = int(rng.integers(0, len(paths)))
        pstar = paths[star]
        a = int(rng.integers(0, len(pstar) + 1)) if planted_len is None else min(int(planted_len[b]), len(pstar))
        out_len[b] = a
        # planted path
        prev = 0
        for i, node in enumerate(pstar):
            if i < a:
                draft[b, node] = target[b, prev]
            elif i == a and V > 1:
                draft[b, node] = other_than(int(target[b, prev]))
            prev = node
        # other paths copy the planted tokens down to a seeded depth, then deviate
        same_as = {0: 0}  # node -> representative node with the same token history
        for node in pstar:
            same_as[node] = node
        force_dup = duplicate_every > 0 and (b % duplicate_every == 0)
        for pi, path in enumerate(paths):
            if pi == star:
                continue
            lim = min(a, len(path))
            d = int(rng.integers(0, lim + 1))
            if force_dup and lim >= 1:
                d = max(d, 1)
                force_dup = False
            prev = 0
            for i, node in enumerate(path):
                if node in same_as:       # trunk shared with the planted path in a trie
                    prev = node
                    continue
                rep_prev = same_as.get(prev)
                if i < d and rep_prev is not None and i < len(pstar) and same_as.get(int(par[pstar[i]])) == rep_prev:
                    draft[b, node] = draft[b, pstar[i]]
                    same_as[node] = pstar[i]
                elif rep_prev is not None and V > 2:
                    sib = int(draft[b, pstar[i]]) if i < len(pstar) else -1
                    draft[b, node] = other_than(int(target[b, rep_prev]), sib)
                prev = node
        for node, rep in same_as.items():
            if node != rep:
                target[b, node] = target[b, rep]
                bump[b, node] = bump[b, rep]
                logits[b, node] = logits[b, rep]
        logits[b, np.arange(T), target[b]] = bump[b]
    return AcceptInputs(cfg, logits, draft, tree_parent, out_len, target)


# --------------------------------------------------------------------------
# grouped token histories for drafting
# --------------------------------------------------------------------------
@dataclass
class DraftInputs:
    """Token histories of prompt groups and the lookup patterns of the live requests."""

    tokens: np.ndarray            # [pool] int32: every sequence's tokens, gaps hold decoy tokens
    seq_start: np.ndarray         # [n_seq] int32
    seq_len: np.ndarray           # [n_seq] int32
    seq_capacity: np.ndarray      # [n_seq] int32: room of each sequence in the pool (its tokens + the gap behind it)
    group_first: np.ndarray       # [n_groups + 1] int32: group g owns sequences group_first[g] .. group_first[g+1]-1
    req_group: np.ndarray         # [B] int32
    req_seq: np.ndarray           # [B] int32: the sequence that is the request's own history
    pattern: np.ndarray           # [B, p_max] int32, right-aligned, newest token last
    pattern_len: np.ndarray       # [B] int32
    max_spec_tokens: np.ndarray   # [B] int32
    future: np.ndarray            # [B, horizon] int32: the tokens the request produces next (not in the pool)
    gamma_max: int
    top_k: int
    p_min: int
    p_max: int
    min_confidence: float
    vocab: int

    @property
    def T(self) -> int:
        return 1 + self.top_k * self.gamma_max

    @property
    def max_group_tokens(self) -> int:
        tot = [int(self.seq_len[self.group_first[g]:self.group_first[g + 1]].sum())
               for g in range(len(self.group_first) - 1)]
        return max(tot) if tot else 0


class _Zipf:
    """Ranks in [0, n) with probability proportional to 1 / (rank + 1)^a (inverse-CDF draws)."""

    def __init__(self, n: int, a: float = 1.1):
        self.n = n
        self.cdf = np.cumsum(1.0 / np.power(np.arange(1, n + 1, dtype=np.float64), a))

    def draw(self, rng: np.random.Generator, size: int) -> np.ndarray:
        u = rng.random(size) * self.cdf[-1]
        return np.minimum(np.searchsorted(self.cdf, u, side="right"), self.n - 1).astype(np.int64)


def make_draft_inputs(cfg: VerifyConfig, seed: Optional[int] = None, *, gamma_max: int = 8, top_k: int = 1,
                      p_min: int = 2, p_max: int = 8, min_confidence: float = 0.0, horizon: int = 16,
                      n_phrases: int = 1024, phrase_prob: float = 0.3, own_only: bool = False, spare: int = 0,
                      refs_per_group: Optional[int] = None, max_spec_tokens=None) -> DraftInputs:
    """Responses of a prompt group as the paper describes them (Section 2.3: responses to one prompt
    share recurring phrases; later requests find more of them in their group's history): every group
    draws a bank of `n_phrases` phrases (3..24 tokens, Zipf-distributed token ids under a seeded
    permutation of the vocabulary; half of them repeat the first tokens of an earlier phrase, so that
    a pattern can have several continuations); a response is a run of pieces, each with probability `phrase_prob`
    a phrase of the bank (Zipf-distributed choice), otherwise 1..8 free Zipf tokens.  Sequence lengths
    follow the configuration's context lengths (without the shared prompt and the verify slots).  The
    pool gives every sequence some spare room after its tokens, filled with decoy tokens that repeat
    the sequence's own tail (so a reader that runs past seq_len finds plausible matches and fails); `spare`
    more tokens of room are left behind every sequence (for tests that append).
    `refs_per_group` = number of sequences of each group that are in the pool (default: all
    group_size); `own_only` keeps just the request's own sequence (the no-reference baseline)."""
    seed = cfg.seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 3])))
    B, V, gs = cfg.B, cfg.V, cfg.group_size
    n_groups = (B + gs - 1) // gs
    ctx = draw_ctx_len(cfg, rng).astype(np.int64)
    resp_len = np.maximum(ctx - cfg.T - cfg.shared_prefix, 0)
    perm = rng.permutation(V)
    zip_v, zip_ph = _Zipf(V), _Zipf(max(1, n_phrases))
    seqs, futures = [], []
    for g in range(n_groups):
        ph_len = rng.integers(3, 25, size=zip_ph.n)
        bank = []
        for l in ph_len:                                  # half of the phrases start like an earlier one
            ph = perm[zip_v.draw(rng, int(l))]
            if bank and rng.random() < 0.5:
                src = bank[int(rng.integers(0, len(bank)))]
                n_same = int(rng.integers(1, min(len(src), len(ph))))
                ph[:n_same] = src[:n_same]
            bank.append(ph)
        for m in range(gs):
            b = g * gs + m
            want = int(resp_len[min(b, B - 1)]) + horizon
            n_pieces = want // 2 + 2                      # every piece has at least one token
            is_ph = rng.random(n_pieces) < phrase_prob
            ph_id = zip_ph.draw(rng, n_pieces)
            free_n = rng.integers(1, 9, size=n_pieces)
            free_tok = perm[zip_v.draw(rng, int(free_n.sum()))]
            free_at = np.concatenate([[0], np.cumsum(free_n)])
            parts, have, i = [], 0, 0
            while have < want:
                piece = bank[int(ph_id[i])] if is_ph[i] else free_tok[free_at[i]:free_at[i + 1]]
                parts.append(piece)
                have += len(piece)
                i += 1
            full = np.concatenate(parts)[:want].astype(np.int32)
            seqs.append(full[:want - horizon])
            futures.append(full[want - horizon:])
    # pool layout: the sequences of a group are neighbours; each is followed by 0..63 decoy tokens
    n_in_pool = gs if refs_per_group is None else max(1, min(gs, refs_per_group))
    starts, lens, caps, chunks, group_first, seq_of = [], [], [], [], [0], {}
    pos = int(rng.integers(0, 8))
    chunks.append(rng.integers(0, V, size=pos).astype(np.int32))
    for g in range(n_groups):
        for m in range(g * gs, g * gs + gs):
            live = m < B
            if own_only and not live:
                continue
            if not own_only and (m - g * gs) >= n_in_pool and not live:
                continue
            s_ = seqs[m]
            gap = spare + int(rng.integers(0, 64))
            decoy = np.resize(s_[-64:], gap) if len(s_) else rng.integers(0, V, size=gap)
            seq_of[m] = len(starts)
            starts.append(pos)
            lens.append(len(s_))
            caps.append(len(s_) + gap)
            chunks += [s_, np.asarray(decoy, np.int32)]
            pos += len(s_) + gap
            if own_only:
                group_first.append(len(starts))       # a group of its own: no references
        if not own_only:
            group_first.append(len(starts))
    req_group = np.arange(B, dtype=np.int32) if own_only else (np.arange(B) // gs).astype(np.int32)
    tokens = np.concatenate(chunks + [np.zeros(4, np.int32)]).astype(np.int32)
    pattern = np.full((B, p_max), -1, np.int32)
    pattern_len = np.zeros(B, np.int32)
    for b in range(B):
        s = seqs[b]
        n = min(len(s), p_max)
        pattern_len[b] = n
        if n:
            pattern[b, p_max - n:] = s[-n:]
    if max_spec_tokens is None:
        max_spec_tokens = np.full(B, gamma_max, np.int32)
    return DraftInputs(tokens=tokens, seq_start=np.asarray(starts, np.int32), seq_len=np.asarray(lens, np.int32),
                       seq_capacity=np.asarray(caps, np.int32), group_first=np.asarray(group_first, np.int32), req_group=req_group,
                       req_seq=np.asarray([seq_of[b] for b in range(B)], np.int32), pattern=pattern,
                       pattern_len=pattern_len, max_spec_tokens=np.asarray(max_spec_tokens, np.int32),
                       future=np.stack(futures[:B]) if B else np.zeros((0, horizon), np.int32),
                       gamma_max=gamma_max, top_k=top_k, p_min=p_min, p_max=p_max,
                       min_confidence=float(min_confidence), vocab=V)


def restrict_draft_inputs(d: DraftInputs, group_size: int, refs: int) -> DraftInputs:
    """The same pool seen by one live request per group (the group's first member) with `refs` of the other
    members' sequences as references (0 = its own history only): the setting of the paper's Table 2, whose rows
    are the number of grouped references."""
    n_groups = len(d.group_first) - 1
    keep_seq, group_first, live = [], [0], []
    for g in range(n_groups):
        q0, q1 = int(d.group_first[g]), int(d.group_first[g + 1])
        members = [b for b in range(len(d.req_group)) if d.req_group[b] == g]
        if not members:
            group_first.append(len(keep_seq))
            continue
        b0 = members[0]
        own = int(d.req_seq[b0])
        others = [q for q in range(q0, q1) if q != own][:refs]
        keep_seq += [own] + others
        group_first.append(len(keep_seq))
        live.append(b0)
    keep_seq = np.asarray(keep_seq, np.int64)
    live = np.asarray(live, np.int64)
    new_index = {int(q): i for i, q in enumerate(keep_seq)}
    return dataclasses.replace(
        d, seq_start=d.seq_start[keep_seq], seq_len=d.seq_len[keep_seq], seq_capacity=d.seq_capacity[keep_seq],
        group_first=np.asarray(group_first, np.int32), req_group=d.req_group[live],
        req_seq=np.asarray([new_index[int(d.req_seq[b])] for b in live], np.int32), pattern=d.pattern[live],
        pattern_len=d.pattern_len[live], max_spec_tokens=d.max_spec_tokens[live], future=d.future[live])
