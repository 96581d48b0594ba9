"""Ablations of the drafting module on synthetic streams (paper, Section 4.3: draft size K at N = 2,
the N x K grid, multi-level against single-level N-gram; Section 5: several candidates per step), host only.

A seeded copy-heavy stream stands for a model whose output re-uses spans of its context: the first
`prompt` tokens initialise the table, the rest is what the LLM would decode greedily.  Algorithm 1
runs on the library's N-gram table (``anpd_ngram_*``) against that continuation, with verification
answered from the stream itself, so the accepted counts are exactly those a lossless verifier
gives.  Reported per setting: draft hit ratio alpha, mean draft length, tokens per step (the speed-up
when a window costs what one row costs, the premise of Section 3.1) and, given measured step times
per window size (``bench.py --sweep`` output), the speed-up those times allow.

    python -m paper_2404_08698_amd.ablation [--workload llama7b] [--step-times sweep.jsonl] [--length L]
"""
from __future__ import annotations

import argparse
import json
import sys
from typing import Dict, List, Optional, Sequence

from . import binding as B
from . import synth


def run_stream(stream: Sequence[int], prompt_len: int, n_min: int, n_max: int, K: int, vocab: int,
               max_tokens: Optional[int] = None) -> Dict[str, float]:
    """Algorithm 1 over stream[prompt_len:], the table seeded with stream[:prompt_len]."""
    table = B.NgramTable(n_min, n_max, vocab)
    table.update(list(stream[:prompt_len]))
    end = len(stream) if max_tokens is None else min(len(stream), prompt_len + max_tokens)
    pos = prompt_len                       # stream[pos] is the token the LLM has just produced (window row 0)
    steps = proposed = accepted = 0
    windows: Dict[int, int] = {}           # rows per window -> count
    while pos < end:
        table.update([stream[pos]])
        drafts, _ = table.propose(K)
        a = 0
        while a < len(drafts) and pos + 1 + a < end and drafts[a] == stream[pos + 1 + a]:
            a += 1
        if a:
            table.update(list(stream[pos + 1:pos + 1 + a]))
        steps += 1
        proposed += len(drafts)
        accepted += a
        windows[1 + len(drafts)] = windows.get(1 + len(drafts), 0) + 1
        pos += 1 + a
    table.close()
    tokens = pos - prompt_len
    return {"steps": steps, "tokens": tokens, "proposed": proposed, "accepted": accepted,
            "alpha": accepted / proposed if proposed else 0.0,
            "mean_draft": proposed / steps if steps else 0.0,
            "tokens_per_step": tokens / steps if steps else 0.0,
            "windows": windows}


def accept_pattern(stream: Sequence[int], prompt_len: int, n_min: int, n_max: int, K: int, vocab: int, n_steps: int,
                   adaptive: bool = False, k_adaptive: Optional[int] = None) -> List[tuple]:
    """(drafts proposed, drafts accepted) of the first n_steps steps of Algorithm 1 over stream[prompt_len:]:
    what the table really proposes on that stream and what a lossless verifier keeps.  ``adaptive`` cuts a
    step's drafts to adaptive_draft_length() with at most ``k_adaptive`` (default K) drafts."""
    table = B.NgramTable(n_min, n_max, vocab)
    table.update(list(stream[:prompt_len]))
    pos, out = prompt_len, []
    while len(out) < n_steps and pos < len(stream):
        table.update([stream[pos]])
        drafts, levels = table.propose(K)
        if adaptive:
            drafts = drafts[:B.adaptive_draft_length(levels, K if k_adaptive is None else k_adaptive)]
        a = 0
        while a < len(drafts) and pos + 1 + a < len(stream) and drafts[a] == stream[pos + 1 + a]:
            a += 1
        if a:
            table.update(list(stream[pos + 1:pos + 1 + a]))
        out.append((len(drafts), a))
        pos += 1 + a
    table.close()
    return out


def run_stream_multi(stream: Sequence[int], prompt_len: int, n_min: int, n_max: int, K: int, n_cand: int, vocab: int,
                     max_drafts: int = 31, max_tokens: Optional[int] = None) -> Dict[str, float]:
    """run_stream with up to n_cand candidate drafts per step (anpd_ngram_propose_tree), verified together:
    the deepest candidate prefix that follows the stream is kept."""
    table = B.NgramTable(n_min, n_max, vocab)
    table.update(list(stream[:prompt_len]))
    end = len(stream) if max_tokens is None else min(len(stream), prompt_len + max_tokens)
    pos = prompt_len
    steps = proposed = accepted = 0
    windows: Dict[int, int] = {}
    while pos < end:
        table.update([stream[pos]])
        toks, pars, _ = table.propose_tree(K, n_cand, max_drafts)
        depth, ok, best = [0], [True], 0
        for i, (tok, par) in enumerate(zip(toks, pars)):
            d = depth[par] + 1
            depth.append(d)
            ok.append(ok[par] and pos + d < end and tok == stream[pos + d])
            if ok[-1] and d > depth[best]:
                best = i + 1
        a = depth[best]
        if a:
            table.update(list(stream[pos + 1:pos + 1 + a]))
        steps += 1
        proposed += len(toks)
        accepted += a
        windows[1 + len(toks)] = windows.get(1 + len(toks), 0) + 1
        pos += 1 + a
    table.close()
    tokens = pos - prompt_len
    return {"steps": steps, "tokens": tokens, "proposed": proposed, "accepted": accepted,
            "mean_rows": 1 + proposed / steps if steps else 0.0,
            "tokens_per_step": tokens / steps if steps else 0.0, "windows": windows}


def speedup_with_times(res: Dict[str, float], ms_by_rows: Dict[int, float]) -> float:
    """Greedy time / ANPD time for the run `res`, with the measured time of a step of each window size."""
    def t(rows: int) -> float:
        keys = sorted(ms_by_rows)
        for k in keys:
            if rows <= k:
                return ms_by_rows[k]
        return ms_by_rows[keys[-1]]
    anpd = sum(n * t(rows) for rows, n in res["windows"].items())
    return res["tokens"] * t(1) / anpd if anpd else 0.0


def load_step_times(path: str, L: int, pages: str = "identity") -> Dict[int, float]:
    for line in open(path):
        line = line.strip()
        if not line.startswith("{"):
            continue
        rec = json.loads(line)
        if rec.get("L") == L and rec.get("pages") == pages and "ms_per_step_by_rows" in rec:
            return {int(k): float(v) for k, v in rec["ms_per_step_by_rows"].items()}
    raise SystemExit("no record for L=%d pages=%s in %s" % (L, pages, path))


def main(argv: Optional[List[str]] = None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="llama7b", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--generate", type=int, default=2048, help="tokens decoded after the prompt")
    ap.add_argument("--step-times", help="JSON lines written by `bench.py --sweep`")
    ap.add_argument("--length", type=int, default=512, help="cache length of the step-time record to use")
    args = ap.parse_args(argv)
    wl = synth.WORKLOADS[args.workload]
    vocab, P = wl["shape"].vocab, wl["prompt"]
    stream = synth.markov_stream(vocab, P + args.generate, wl["p_copy"], wl["span"][0], wl["span"][1], wl["seed"])
    times = load_step_times(args.step_times, args.length) if args.step_times else None

    def row(label: str, n_min: int, n_max: int, K: int) -> None:
        r = run_stream(stream, P, n_min, n_max, K, vocab)
        extra = "  speed-up at measured step times %.2f" % speedup_with_times(r, times) if times else ""
        print("%-22s K=%-2d alpha %.3f  mean draft %.2f  tokens/step %.2f  bound alpha*K+1 %.2f%s" % (
            label, K, r["alpha"], r["mean_draft"], r["tokens_per_step"], r["alpha"] * r["mean_draft"] + 1, extra))

    print("stream: %s recipe (p_copy %.2f, spans %d-%d), prompt %d, %d tokens decoded" % (
        args.workload, wl["p_copy"], wl["span"][0], wl["span"][1], P, args.generate))
    print("-- draft size K at N = 2 (Section 4.3, first ablation)")
    for K in (1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 16):
        row("N=2", 2, 2, K)
    print("-- multi-level N-gram, levels 2..N (Section 3.2), K in {6, 7, 8}")
    for N in (2, 3, 4, 5, 6, 7, 8):
        for K in (6, 7, 8):
            row("MLN 2..%d" % N, 2, N, K)
    print("-- single level N only (no fallback to shorter contexts), K = 7")
    for N in (2, 3, 4, 5, 6, 7, 8):
        row("single N=%d" % N, N, N, 7)
    print("-- candidates per step, verified together (Section 5, future work 2), levels 2..5")
    for K, budget in ((3, 7), (5, 15), (7, 31)):
        for n_cand in (1, 2, 3, 4):
            r = run_stream_multi(stream, P, 2, 5, K, n_cand, vocab, budget)
            extra = "  speed-up at measured step times %.2f" % speedup_with_times(r, times) if times else ""
            print("K=%d, %d candidate(s), at most %2d drafts: mean rows %.2f  tokens/step %.2f%s" % (
                K, n_cand, budget, r["mean_rows"], r["tokens_per_step"], extra))
    return 0


if __name__ == "__main__":
    sys.exit(main())
