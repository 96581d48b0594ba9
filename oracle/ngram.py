"""Oracle of the adaptive multi-level N-gram drafter, by definition.

TEST INFRASTRUCTURE ONLY.  The Memory of the paper's N-gram module
(Section 3.1, "Token Level N-gram Module": Initialize / Update / Query) is a
function of the committed token ids alone, so this oracle keeps no table: it
re-counts by scanning the committed sequence each time it is asked.

Readings where the paper is silent:
  * Query returns the most frequent follower of the context (the paper says
    the module predicts from frequency counts, Section 3.1 and Eq. 1).
  * Among equally frequent followers, the one whose latest occurrence after
    the context is most recent wins.
  * A level whose context is longer than the available history returns NULL.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple


def query(s: Sequence[int], ctx: Sequence[int], n: int) -> Optional[int]:
    """Level-n Query: the follower f maximising
    count_n(ctx, f) = #{ i in [n-1, len(s)) : s[i-n+1 .. i) == ctx and s[i] == f }.
    None (NULL) when every count is zero."""
    ctx = list(ctx)
    assert len(ctx) == n - 1
    count = {}
    latest = {}
    for i in range(n - 1, len(s)):
        if list(s[i - n + 1:i]) == ctx:
            f = s[i]
            count[f] = count.get(f, 0) + 1
            latest[f] = i
    if not count:
        return None
    return max(count, key=lambda f: (count[f], latest[f]))


def mln_query(s: Sequence[int], tail: Sequence[int], n_min: int, n_max: int) -> Tuple[Optional[int], int]:
    """Multi-Level N-gram query (Section 3.2, Algorithm 2): try n = n_max down
    to n_min on the last n-1 ids of ``tail``; the first level that answers
    wins.  Returns (token or None, level that hit or 0)."""
    for n in range(n_max, n_min - 1, -1):
        if len(tail) < n - 1:
            continue
        r = query(s, tail[len(tail) - (n - 1):], n)
        if r is not None:
            return r, n
    return None, 0


def propose(s: Sequence[int], max_k: int, n_min: int, n_max: int) -> Tuple[List[int], List[int]]:
    """Drafting loop of Algorithm 1: up to max_k iterative MLN queries, each on
    the committed ids followed by the tokens drafted so far.  Counts come from
    the committed ids only.  Drafting stops at the first NULL."""
    tail = list(s)
    drafts: List[int] = []
    levels: List[int] = []
    for _ in range(max_k):
        tok, lvl = mln_query(s, tail, n_min, n_max)
        if tok is None:
            break
        drafts.append(tok)
        levels.append(lvl)
        tail.append(tok)
    return drafts, levels


def followers_ranked(s: Sequence[int], ctx: Sequence[int], n: int) -> List[int]:
    """All followers of ``ctx`` at level n, most frequent first, the most recently seen first among
    equally frequent ones (the order Query's winner is the head of)."""
    ctx = list(ctx)
    assert len(ctx) == n - 1
    count = {}
    latest = {}
    for i in range(n - 1, len(s)):
        if list(s[i - n + 1:i]) == ctx:
            f = s[i]
            count[f] = count.get(f, 0) + 1
            latest[f] = i
    return sorted(count, key=lambda f: (count[f], latest[f]), reverse=True)


def propose_tree(s: Sequence[int], max_k: int, n_cand: int, max_drafts: int, n_min: int,
                 n_max: int) -> Tuple[List[int], List[int], List[int]]:
    """Drafts for multi-candidate verification (the paper names the idea as future work and gives no
    rule; this is the reading the library documents).  Candidate first tokens: levels n_max down to
    n_min, within a level the ranked followers of the context, distinct tokens, until n_cand are found.
    Each candidate is continued by the drafting loop of Algorithm 1 to at most max_k tokens; candidates
    are laid out one after the other, at most max_drafts drafts in all.  Returns (tokens, parents,
    levels); draft i is window row i + 1, parents are window rows (0 = the last accepted token)."""
    firsts: List[Tuple[int, int]] = []
    for n in range(n_max, n_min - 1, -1):
        if len(firsts) >= n_cand:
            break
        if len(s) < n - 1:
            continue
        for f in followers_ranked(s, s[len(s) - (n - 1):], n):
            if len(firsts) < n_cand and all(f != g for g, _ in firsts):
                firsts.append((f, n))
    tokens: List[int] = []
    parents: List[int] = []
    levels: List[int] = []
    if max_k <= 0:
        return tokens, parents, levels
    for first, lvl0 in firsts:
        tail = list(s)
        parent = 0
        for k in range(max_k):
            if len(tokens) >= max_drafts:
                break
            if k == 0:
                tok, lvl = first, lvl0
            else:
                tok, lvl = mln_query(s, tail, n_min, n_max)
                if tok is None:
                    break
            tokens.append(tok)
            parents.append(parent)
            levels.append(lvl)
            parent = len(tokens)
            tail.append(tok)
    return tokens, parents, levels
