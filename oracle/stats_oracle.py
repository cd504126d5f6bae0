"""Oracle for the online acceptance statistics that feed the draft-length policy (Section 3.4.2: Algorithm 1
takes "per-position acceptance probabilities beta[1], beta[2], ..." and is run on "online-collected acceptance
rates"; Section 3.4.1: alpha = E(beta)).

TEST INFRASTRUCTURE ONLY: plain Python loops over requests and nodes, the definition written out; nothing in the
product path imports it and it shares no code with the library's implementation.

The paper does not say how beta is collected.  Reading used here (and by the library), per verify step and request:
  * a draft is a tree of nodes under the root (slot 0, the token already accepted, depth 0); a chain is the tree in
    which slot t hangs under slot t - 1; a padded slot (parent -2, or any parent that is not an earlier node) is no node;
  * position k = depth k.  The step OFFERED position k if the tree has a node of depth k; it TRIED position k if
    the accepted path reached depth k - 1 and the node it reached there has a child (so a token of depth k was
    compared with the target's token); it ACCEPTED position k if accepted_len >= k;
  * beta[k] = accepted[k] / offered[k] (default: the share of the steps that drafted k or more tokens in which the
    k-th was accepted; non-increasing in k when all drafts are equally deep, beta[0] = 1), or, "conditional",
    accepted[k] / tried[k] (how often a token that was compared was accepted: the per-token rate of the
    geometric model behind the expected-tokens law);
  * a request whose accepted_len / accepted_path do not describe a root path of its tree is left out.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

OFFERED, TRIED, ACCEPTED = 0, 1, 2


def node_depths(parent: Optional[Sequence[int]], T: int) -> List[Optional[int]]:
    """Depth of every slot under the root, None for slots that are not nodes."""
    depth: List[Optional[int]] = [None] * T
    depth[0] = 0
    for t in range(1, T):
        p = t - 1 if parent is None else int(parent[t])
        if 0 <= p < t and depth[p] is not None:
            depth[t] = depth[p] + 1
    return depth


def parent_of(parent: Optional[Sequence[int]], t: int) -> int:
    return t - 1 if parent is None else int(parent[t])


def acceptance_counts(accepted_len, accepted_path, tree_parent, T: int, counts=None):
    """counts[3][T] (offered, tried, accepted by position), added to `counts` if given."""
    if counts is None:
        counts = [[0] * T for _ in range(3)]
    B = len(accepted_len)
    for b in range(B):
        parent = None if tree_parent is None else tree_parent[b]
        depth = node_depths(parent, T)
        a = int(accepted_len[b])
        path = [int(x) for x in accepted_path[b]]
        ok = 0 <= a <= T - 1 and path[0] == 0
        for i in range(1, a + 1):
            if not ok:
                break
            v = path[i]
            ok = 0 < v < T and depth[v] == i and parent_of(parent, v) == path[i - 1]
        if not ok:
            continue
        for k in range(1, T):
            if any(d == k for d in depth):
                counts[OFFERED][k] += 1
        for k in range(1, a + 1):
            counts[TRIED][k] += 1
            counts[ACCEPTED][k] += 1
        last = path[a]
        if a + 1 < T and any(depth[t] is not None and parent_of(parent, t) == last for t in range(1, T)):
            counts[TRIED][a + 1] += 1
        counts[OFFERED][0] += 1
        counts[TRIED][0] += 1
        counts[ACCEPTED][0] += 1
    return counts


def beta_from_counts(counts, T: int, conditional: bool = False, prior: float = 0.0) -> List[float]:
    """beta for positions 1 .. T - 1 (list index k - 1); `prior` where nothing was counted."""
    den = counts[TRIED] if conditional else counts[OFFERED]
    return [counts[ACCEPTED][k] / den[k] if den[k] > 0 else float(prior) for k in range(1, T)]
