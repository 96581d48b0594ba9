"""Pins of the ANPD loop oracle: the paper's invariants (lossless, 1..K+1
tokens per step, K = 0 is plain decoding) on scripted and on real oracle LLMs,
and the printed case-study bound."""
import os

import pytest

from oracle import anpd, decoder as od
from paper_2404_08698_amd import synth


class ScriptedLLM:
    """A deterministic 'LLM' whose next token is a fixed function of the whole
    prefix; lets the loop be checked without any floating point."""

    def __init__(self, fn):
        self.fn, self.ctx, self.window, self.calls = fn, [], [], 0

    def prefill(self, prompt):
        self.ctx = list(prompt)
        return self.fn(self.ctx)

    def predict(self, window):
        self.calls += 1
        self.window = list(window)
        return [self.fn(self.ctx + self.window[: r + 1]) for r in range(len(window))]

    def commit(self, n_rows):
        assert 1 <= n_rows <= len(self.window)
        self.ctx += self.window[:n_rows]
        self.window = []


def periodic(ctx):          # highly predictable: repeats with period 5
    return (len(ctx) * 3) % 5 + 10


def hashed(ctx):            # unpredictable from n-grams
    return synth.splitmix64(sum((i + 1) * t for i, t in enumerate(ctx[-6:]))) % 50


def mixed(ctx):             # copies the token 7 back most of the time
    return ctx[-7] if len(ctx) >= 7 and len(ctx) % 4 else hashed(ctx)


@pytest.mark.parametrize("fn", [periodic, hashed, mixed])
@pytest.mark.parametrize("K", [0, 1, 3, 7])
@pytest.mark.parametrize("N", [2, 3, 5])
def test_lossless_on_scripted_llms(fn, K, N):
    prompt = [10, 13, 11, 14, 12, 10, 13, 11, 14, 12, 10, 13]
    M = 40
    ref = anpd.greedy_generate(ScriptedLLM(fn), prompt, M)
    llm = ScriptedLLM(fn)
    res = anpd.anpd_generate(llm, prompt, K, M, 2, N)
    assert res["tokens"] == ref
    assert llm.calls == res["n_steps"] <= M
    for st in res["steps"]:
        k = len(st["window"]) - 1
        assert 0 <= st["accepted"] <= k <= K        # 1 <= tokens per step <= K+1
    if K == 0:
        assert res["n_steps"] == M and res["proposed"] == 0
    if fn is periodic and K >= 3 and N >= 3:
        assert res["n_steps"] < M / 2               # drafts do get accepted


def test_perfect_and_adversarial_drafters():
    prompt = [1, 2, 3, 4]
    M, K = 30, 4
    ref = anpd.greedy_generate(ScriptedLLM(hashed), prompt, M + K + 1)

    def perfect(s, k):
        n = len(s) - len(prompt)
        return ref[n:n + k]

    res = anpd.anpd_generate(ScriptedLLM(hashed), prompt, K, M, drafter=perfect)
    assert res["tokens"] == ref[:M]
    assert all(st["accepted"] == K for st in res["steps"])
    assert all(st["next"] == ref[(i + 1) * (K + 1)] for i, st in enumerate(res["steps"]))
    assert res["n_steps"] == -(-M // (K + 1))

    def wrong(s, k):
        n = len(s) - len(prompt)
        return [(t + 1) % 50 for t in ref[n:n + k]]

    res = anpd.anpd_generate(ScriptedLLM(hashed), prompt, K, M, drafter=wrong)
    assert res["tokens"] == ref[:M]
    assert res["accepted"] == 0 and res["n_steps"] == M

    def half(s, k):        # right for two tokens, then wrong
        n = len(s) - len(prompt)
        d = ref[n:n + k]
        return d[:2] + [(t + 1) % 50 for t in d[2:]]

    res = anpd.anpd_generate(ScriptedLLM(hashed), prompt, K, M, drafter=half)
    assert res["tokens"] == ref[:M]
    assert all(st["accepted"] == 2 for st in res["steps"])


def test_accept_length():
    assert anpd.accept_length([], [9]) == 0
    assert anpd.accept_length([4, 5, 6], [4, 5, 6, 7]) == 3
    assert anpd.accept_length([4, 5, 6], [4, 9, 6, 7]) == 1
    assert anpd.accept_length([4, 5, 6], [0, 5, 6, 7]) == 0


def test_case_study_bound_printed_by_the_paper():
    path = os.path.join(os.path.dirname(__file__), "golden", "case_study_speedup_bound.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    alpha, K, printed, measured = (float(x) for x in rows[0])
    bound = anpd.speedup_bound(alpha, K)
    assert abs(bound - 2.4413) < 1e-4
    assert round(bound, 2) == printed
    assert measured < bound
    assert anpd.hit_ratio(7, 34) == pytest.approx(0.20588, abs=1e-4)
    assert anpd.hit_ratio(0, 0) == 0.0


@pytest.mark.parametrize("N,K", [(2, 4), (3, 4), (5, 8), (3, 0)])
def test_lossless_on_the_tiny_decoder(N, K, tiny_weights):
    """The tiny configuration: prompt 128, generate 64."""
    shape = synth.TINY
    prompt = synth.workload_prompt("tiny")
    M = 64
    ref = anpd.greedy_generate(od.Decoder(shape, tiny_weights, 128 + M + 16), prompt, M)
    res = anpd.anpd_generate(od.Decoder(shape, tiny_weights, 128 + M + 16), prompt, K, M, 2, N)
    assert res["tokens"] == ref
    tokens_per_step = M / res["n_steps"]
    if K:
        alpha = anpd.hit_ratio(res["accepted"], res["proposed"])
        kbar = res["proposed"] / res["n_steps"]
        # identity tokens/step = 1 + alpha * mean draft length (up to the final cut to M)
        total = res["n_steps"] + res["accepted"]
        assert total >= M and total - M <= K
        assert abs(total / res["n_steps"] - anpd.speedup_bound(alpha, kbar)) < 1e-12
    else:
        assert tokens_per_step == 1.0
