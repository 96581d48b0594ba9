"""The host-only ablation driver against the oracle's Algorithm 1 (paper, Algorithm 1, Section 4.3)."""
from oracle import anpd as oanpd
from paper_2404_08698_amd import ablation, synth


class StreamModel:
    """A scripted LLM whose greedy output is a fixed stream (oracle/anpd.py's llm interface)."""

    def __init__(self, stream, prompt_len):
        self.s, self.pos = stream, prompt_len          # cache holds s[:pos]

    def prefill(self, prompt):
        assert list(prompt) == list(self.s[:self.pos])
        return self.s[self.pos]

    def predict(self, window):
        return [self.s[self.pos + 1 + r] if self.pos + 1 + r < len(self.s) else -1 for r in range(len(window))]

    def commit(self, n_rows):
        self.pos += n_rows


def test_driver_counts_match_the_oracle_loop():
    vocab, P, G = 64, 48, 160
    stream = synth.markov_stream(vocab, P + G + 40, 0.5, 3, 9, 123)
    for n_min, n_max, K in ((2, 2, 4), (2, 5, 7), (3, 3, 5), (2, 4, 1)):
        ref = oanpd.anpd_generate(StreamModel(stream, P), stream[:P], K, G, n_min, n_max)
        got = ablation.run_stream(stream[:P + G + 40], P, n_min, n_max, K, vocab, max_tokens=None)
        # same drafts and acceptances step by step: compare over the steps the oracle took
        n = ref["n_steps"]
        again = ablation.run_stream(stream, P, n_min, n_max, K, vocab, max_tokens=sum(1 + s["accepted"] for s in ref["steps"]))
        assert again["steps"] == n
        assert again["proposed"] == ref["proposed"] and again["accepted"] == ref["accepted"]
        assert got["alpha"] >= 0.0


def test_periodic_stream_is_drafted_perfectly_and_step_times_are_applied():
    period = [5, 9, 2, 7, 11, 3]
    stream = period * 40
    r = ablation.run_stream(stream, 24, 2, 3, 5, 16)
    assert r["alpha"] > 0.98 and r["tokens_per_step"] > 5.5
    flat = {1: 3.0, 8: 3.0}
    assert abs(ablation.speedup_with_times(r, flat) - r["tokens_per_step"]) < 1e-9
    slow = {1: 3.0, 8: 6.0}
    assert ablation.speedup_with_times(r, slow) < r["tokens_per_step"]


def test_multi_candidate_driver_counts_match_the_oracle_loop():
    vocab, P, G = 64, 48, 120
    stream = synth.markov_stream(vocab, P + G + 40, 0.5, 3, 9, 321)
    for n_min, n_max, K, n_cand, budget in ((2, 4, 4, 3, 31), (2, 2, 3, 2, 5), (2, 5, 6, 1, 31)):
        ref = oanpd.anpd_generate_multi(StreamModel(stream, P), stream[:P], K, n_cand, G, budget, n_min, n_max)
        got = ablation.run_stream_multi(stream, P, n_min, n_max, K, n_cand, vocab, budget,
                                        max_tokens=sum(1 + s["accepted"] for s in ref["steps"]))
        assert got["steps"] == ref["n_steps"]
        assert got["proposed"] == ref["proposed"] and got["accepted"] == ref["accepted"]
        if n_cand == 1:
            one = ablation.run_stream(stream, P, n_min, n_max, K, vocab, max_tokens=got["tokens"])
            assert (one["steps"], one["accepted"]) == (got["steps"], got["accepted"])


def test_accept_pattern_follows_the_stream_and_the_adaptive_cut():
    # (drafts, accepted) per step: what the table proposes on the stream and what a lossless verifier keeps;
    # the adaptive form cuts a step's drafts to 2^(level - 2) of the level that answered, and to k_adaptive
    period = [5, 9, 2, 7, 11, 3, 8]
    stream = period * 40
    plain = ablation.accept_pattern(stream, 28, 2, 6, 16, 16, 12)
    assert all(d == 16 and a == 16 for d, a in plain)                # a periodic stream is drafted perfectly
    adaptive = ablation.accept_pattern(stream, 28, 2, 6, 16, 16, 12, adaptive=True)
    assert all(d == 16 and a == 16 for d, a in adaptive)             # level 6 answers: 2^4 drafts
    capped = ablation.accept_pattern(stream, 28, 2, 6, 16, 16, 12, adaptive=True, k_adaptive=15)
    assert all(d == 15 and a == 15 for d, a in capped)
    low = ablation.accept_pattern(stream, 28, 2, 3, 16, 16, 12, adaptive=True, k_adaptive=15)
    assert all(d == 2 and a == 2 for d, a in low)                    # level 3 answers: 2 drafts
    vocab = 64
    noisy = synth.markov_stream(vocab, 400, 0.5, 3, 9, 77)
    for d, a in ablation.accept_pattern(noisy, 48, 2, 5, 7, vocab, 60):
        assert 0 <= a <= d <= 7
