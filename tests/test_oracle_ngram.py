"""Pins of the N-gram / MLN oracle: hand-worked cases, the textbook bigram
reduction via a library counter, and structural invariants."""
import collections
import itertools

from oracle import ngram


def test_hand_worked_bigram_counts():
    #    index: 0  1  2  3  4  5  6
    s = [1, 2, 1, 3, 1, 2, 1]
    # followers of 1: 2 (i=1), 3 (i=3), 2 (i=5) -> 2 wins with count 2
    assert ngram.query(s, [1], 2) == 2
    # followers of 2: 1, 1
    assert ngram.query(s, [2], 2) == 1
    # 3 is followed once by 1; 7 never occurs
    assert ngram.query(s, [3], 2) == 1
    assert ngram.query(s, [7], 2) is None
    # trigram (2,1)->3 once; (1,2)->1 twice; the final (2,1) has no follower yet
    assert ngram.query(s, [2, 1], 3) == 3
    assert ngram.query(s, [1, 2], 3) == 1
    assert ngram.query(s, [3, 3], 3) is None


def test_tie_goes_to_most_recent_follower():
    # followers of 5: 8 (i=1), 9 (i=3): one each; 9 is the later one
    assert ngram.query([5, 8, 5, 9, 4], [5], 2) == 9
    assert ngram.query([5, 9, 5, 8, 4], [5], 2) == 8
    # count beats recency
    assert ngram.query([5, 8, 5, 8, 5, 9], [5], 2) == 8


def test_mln_prefers_longest_level_then_falls_back():
    #    0  1  2  3  4  5  6  7
    s = [1, 2, 3, 9, 2, 3, 7, 4, 3]
    # tail ends (2,3)?  use explicit tails
    # level 3 on (2,3): followers 9 (i=3), 7 (i=6) -> tie -> 7 (later)
    assert ngram.mln_query(s, [2, 3], 2, 3) == (7, 3)
    # level 4 on (1,2,3): follower 9
    assert ngram.mln_query(s, [1, 2, 3], 2, 4) == (9, 4)
    # (5,3): no trigram hit, falls back to bigram on 3: followers 9, 7 -> 7
    assert ngram.mln_query(s, [5, 3], 2, 3) == (7, 2)
    # nothing known about 6 at any level
    assert ngram.mln_query(s, [2, 6], 2, 3) == (None, 0)
    # context shorter than a level's n-1: that level is skipped
    assert ngram.mln_query(s, [3], 2, 5) == (7, 2)


def test_bigram_level_is_most_frequent_follower_library_counter():
    # exhaustive over all sequences of a 3-letter alphabet up to length 7
    for T in range(1, 8):
        for s in itertools.product(range(3), repeat=T):
            pairs = collections.Counter(zip(s[:-1], s[1:]))
            for c in range(3):
                got = ngram.query(s, [c], 2)
                foll = {f: n for (a, f), n in pairs.items() if a == c}
                if not foll:
                    assert got is None
                else:
                    top = max(foll.values())
                    assert foll[got] == top
                    tied = [f for f, n in foll.items() if n == top]
                    # recency rule among the tied ones
                    last = {f: max(i for i in range(1, T) if s[i - 1] == c and s[i] == f) for f in tied}
                    assert got == max(tied, key=lambda f: last[f])


def test_propose_follows_a_periodic_sequence_and_stops_on_null():
    s = [4, 5, 6, 4, 5, 6, 4]
    drafts, levels = ngram.propose(s, 5, 2, 3)
    assert drafts == [5, 6, 4, 5, 6]
    assert levels == [3, 3, 3, 3, 3]
    # last token never seen before: every level is NULL, no draft at all
    assert ngram.propose([4, 5, 6, 9], 5, 2, 3) == ([], [])
    # drafting uses drafted tokens as context but never counts them:
    # after 1 -> 2 the chain stops because 2 has no known follower
    assert ngram.propose([1, 2, 7, 1], 4, 2, 2) == ([2, 7, 1, 2], [2, 2, 2, 2])
    assert ngram.propose([3, 1, 2], 4, 2, 2) == ([], [])
    assert ngram.propose([1, 2, 1], 4, 2, 2)[0] == [2, 1, 2, 1]
    assert ngram.propose([1, 2, 3, 1], 4, 2, 2)[0] == [2, 3, 1, 2]
    assert ngram.propose([1, 2, 1], 0, 2, 2) == ([], [])


def test_counts_span_the_prompt_generation_boundary():
    prompt, generated = [1, 2], [3, 1, 2]
    s = prompt + generated
    # the pair (2 -> 3) straddles the boundary and must be counted
    assert ngram.query(s, [2], 2) == 3
    assert ngram.query(s, [1, 2], 3) == 3


def _independent_level(s, ctx, n):
    """Level-n answer from a library counter over the n-tuples of s (no scan of windows by index as the oracle
    does): count every tuple zip(s, s[1:], ..., s[n-1:]), keep those whose first n-1 items are ctx, take the
    most frequent last item, the one whose last such tuple starts latest among equals."""
    tuples = list(zip(*[s[j:] for j in range(n)]))
    counts = collections.Counter(tuples)
    foll = {t[-1]: c for t, c in counts.items() if t[:-1] == tuple(ctx)}
    if not foll:
        return None
    top = max(foll.values())
    tied = [f for f, c in foll.items() if c == top]
    last_start = {f: max(i for i, t in enumerate(tuples) if t == tuple(ctx) + (f,)) for f in tied}
    return max(tied, key=lambda f: last_start[f])


def test_higher_levels_and_mln_against_tuple_counter_exhaustively():
    # Section 3.1 (Query at level n) and Section 3.2 / Algorithm 2 (longest level first): every sequence over
    # a 3-letter alphabet up to length 8, every context of length 2 and 3, and the multi-level answer on every
    # tail of length 3, against a formulation that shares nothing with the oracle's scan
    alphabet = range(3)
    contexts = {n: list(itertools.product(alphabet, repeat=n - 1)) for n in (2, 3, 4)}
    for T in range(1, 9):
        for s in itertools.product(alphabet, repeat=T):
            want = {}
            for n in (2, 3, 4):
                for ctx in contexts[n]:
                    want[ctx] = _independent_level(s, ctx, n)
                    if n > 2:
                        assert ngram.query(s, list(ctx), n) == want[ctx], (s, ctx, n)
            for tail in contexts[4]:
                exp = (None, 0)
                for n in (4, 3, 2):
                    r = want[tail[len(tail) - (n - 1):]]
                    if r is not None:
                        exp = (r, n)
                        break
                assert ngram.mln_query(s, list(tail), 2, 4) == exp, (s, tail)
            # a tail shorter than a level's context skips that level
            for tail in contexts[2]:
                r = want[tail]
                assert ngram.mln_query(s, list(tail), 2, 4) == ((r, 2) if r is not None else (None, 0))
