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


def hit_ratio(accepted: int, proposed: int) -> float:
    """Draft hit ratio alpha (Section 4.4): accepted drafts / proposed drafts."""
    return accepted / proposed if proposed else 0.0


def speedup_bound(alpha: float, K: float) -> float:
    """Theoretical speed-up the paper derives from the hit ratio: alpha * K + 1."""
    return alpha * K + 1.0
