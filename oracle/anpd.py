"""Oracle of the ANPD decode loop (paper, Algorithm 1) and of plain greedy decoding.

TEST INFRASTRUCTURE ONLY.  ``llm`` is any object with
  prefill(prompt) -> int          greedy token after the prompt; cache filled
  predict(window) -> list[int]    one greedy prediction per window row
  commit(n_rows)                  keep the first n_rows rows of the last window
(oracle/decoder.py's Decoder is one; tests also plug in scripted models).

Readings of Algorithm 1 (0-indexed here):
  * the sliding context of a draft query is the last N-1 ids of committed +
    drafted tokens (the printed slice is garbled);
  * a NULL query ends drafting for this step: the window is shorter;
  * after the accept loop the next token is predicts[a], a = number of
    accepted drafts, whether the loop broke or ran to the end;
  * the output is cut to exactly M tokens.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence

from . import ngram


def accept_length(drafts: Sequence[int], predicts: Sequence[int]) -> int:
    """Longest prefix of the drafts that the LLM reproduces: draft j (0-based)
    is accepted while it equals the prediction made after window row j."""
    a = 0
    while a < len(drafts) and drafts[a] == predicts[a]:
        a += 1
    return a


def greedy_generate(llm, prompt: Sequence[int], M: int) -> List[int]:
    """Plain autoregressive greedy decoding: the definition ANPD must reproduce."""
    c = llm.prefill(prompt)
    out: List[int] = []
    while len(out) < M:
        out.append(c)
        p = llm.predict([c])
        llm.commit(1)
        c = p[0]
    return out


def anpd_generate(llm, prompt: Sequence[int], K: int, M: int, n_min: int = 2, n_max: int = 5,
                  drafter: Optional[Callable[[List[int], int], List[int]]] = None) -> Dict[str, object]:
    """Algorithm 1.  ``drafter(committed_ids, K)`` replaces the N-gram module
    when given (used to script perfect / adversarial drafts)."""
    s = list(prompt)
    out: List[int] = []
    c = llm.prefill(prompt)
    steps = []
    while len(out) < M:
        s.append(c)
        out.append(c)
        if drafter is not None:
            drafts = list(drafter(s, K))[:K]
        else:
            drafts, _ = ngram.propose(s, K, n_min, n_max)
        window = [c] + drafts
        p = llm.predict(window)
        a = accept_length(drafts, p)
        s.extend(drafts[:a])
        out.extend(drafts[:a])
        llm.commit(1 + a)
        steps.append({"window": window, "predicts": list(p), "accepted": a, "next": p[a]})
        c = p[a]
    proposed = sum(len(st["window"]) - 1 for st in steps)
    accepted = sum(st["accepted"] for st in steps)
    return {"tokens": out[:M], "steps": steps, "n_steps": len(steps),
            "proposed": proposed, "accepted": accepted}


def tree_path(parent: Sequence[int], r: int) -> List[int]:
    """Window rows from the root to row r."""
    path = [r]
    while parent[path[-1]] >= 0:
        path.append(parent[path[-1]])
    return path[::-1]


def tree_predict(llm, window: Sequence[int], parent: Sequence[int]) -> List[int]:
    """Multi-candidate verification by its definition: every row of the draft tree gets the
    prediction it would get at the end of the linear window made of its own root-to-row path.
    Nothing is committed."""
    preds = []
    for r in range(len(window)):
        p = llm.predict([window[i] for i in tree_path(parent, r)])
        preds.append(p[-1])
    return preds


def tree_accept(window: Sequence[int], parent: Sequence[int], predicts: Sequence[int]):
    """Algorithm 1's accept rule along every path: row r > 0 is accepted iff its parent is and
    window[r] equals the prediction at the parent.  The deepest accepted row wins, the lowest index
    among equally deep ones.  Returns (depth a, winning row, path root .. winner)."""
    depth = [0] * len(window)
    ok = [False] * len(window)
    ok[0] = True
    best = 0
    for r in range(1, len(window)):
        depth[r] = depth[parent[r]] + 1
        ok[r] = ok[parent[r]] and window[r] == predicts[parent[r]]
        if ok[r] and depth[r] > depth[best]:
            best = r
    return depth[best], best, tree_path(parent, best)


def anpd_generate_multi(llm, prompt: Sequence[int], K: int, n_cand: int, M: int, max_drafts: int = 31,
                        n_min: int = 2, n_max: int = 5) -> Dict[str, object]:
    """Algorithm 1 with several candidate drafts per step (oracle/ngram.propose_tree), verified
    together (tree_predict), the longest accepted candidate kept."""
    s = list(prompt)
    out: List[int] = []
    c = llm.prefill(prompt)
    steps = []
    while len(out) < M:
        s.append(c)
        out.append(c)
        toks, pars, _ = ngram.propose_tree(s, K, n_cand, max_drafts, n_min, n_max)
        window, parent = [c] + toks, [-1] + pars
        p = tree_predict(llm, window, parent)
        a, best, path = tree_accept(window, parent, p)
        kept = [window[r] for r in path[1:]]
        llm.predict([window[r] for r in path])   # leave the winning path's rows in the cache
        llm.commit(1 + a)
        s.extend(kept)
        out.extend(kept)
        steps.append({"window": window, "parent": parent, "predicts": list(p), "accepted": a, "path": path, "next": p[best]})
        c = p[best]
    return {"tokens": out[:M], "steps": steps, "n_steps": len(steps),
            "proposed": sum(len(st["window"]) - 1 for st in steps), "accepted": sum(st["accepted"] for st in steps)}


def hit_ratio(accepted: int, proposed: int) -> float:
    """Draft hit ratio alpha (Section 4.4): accepted drafts / proposed drafts."""
    return accepted / proposed if proposed else 0.0


def speedup_bound(alpha: float, K: float) -> float:
    """Theoretical speed-up the paper derives from the hit ratio: alpha * K + 1."""
    return alpha * K + 1.0
