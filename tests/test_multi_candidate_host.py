"""Multi-candidate drafting and acceptance without a GPU: the oracle's tree rules pinned by hand-worked
cases and by the paper's invariants, and the library's drafting checked against the oracle bit for bit."""
import itertools

import pytest

from oracle import anpd, ngram as ong
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth
from test_oracle_anpd import ScriptedLLM, hashed, mixed, periodic


def test_ranked_followers_by_hand():
    #    index: 0  1  2  3  4  5  6  7  8
    s = [5, 8, 5, 9, 5, 8, 5, 7, 5]
    # followers of 5: 8 twice (i=1, 5), 9 once (i=3), 7 once (i=7): 8, then 7 (later than 9), then 9
    assert ong.followers_ranked(s, [5], 2) == [8, 7, 9]
    assert ong.followers_ranked(s, [8, 5], 3) == [7, 9]
    assert ong.followers_ranked(s, [4], 2) == []
    # the head of the ranking is Query's answer
    for ctx, n in (([5], 2), ([8, 5], 3), ([9, 5], 3)):
        assert ong.followers_ranked(s, ctx, n)[0] == ong.query(s, ctx, n)


def test_tree_drafts_by_hand():
    s = [5, 8, 5, 9, 5, 8, 5, 7, 5]
    # one candidate: the ordinary chain
    assert ong.propose_tree(s, 3, 1, 31, 2, 3)[:2] == (ong.propose(s, 3, 2, 3)[0], [0, 1, 2])
    # level 3 on (7, 5) knows nothing; level 2 on (5): candidates 8, 7, 9.
    toks, pars, lvls = ong.propose_tree(s, 2, 3, 31, 2, 3)
    # chain of 8: (5, 8) -> 5 at level 3; chain of 7: (5, 7) -> 5; chain of 9: (5, 9) -> 5
    assert toks == [8, 5, 7, 5, 9, 5]
    assert pars == [0, 1, 0, 3, 0, 5]
    assert lvls == [2, 3, 2, 3, 2, 3]
    # the row budget cuts later candidates short
    assert ong.propose_tree(s, 2, 3, 3, 2, 3)[:2] == ([8, 5, 7], [0, 1, 0])
    assert ong.propose_tree(s, 0, 3, 31, 2, 3) == ([], [], [])
    # a higher level contributes its followers first, lower levels fill up with distinct tokens
    s2 = [1, 2, 3, 1, 2, 4, 9, 2, 3, 1, 2]
    # level 3 on (1, 2): followers 3 (i=2), 4 (i=5): one each, 4 later -> [4, 3]; level 2 on (2): 3 twice, 4 once
    toks, pars, lvls = ong.propose_tree(s2, 1, 3, 31, 2, 3)
    assert toks == [4, 3] and pars == [0, 0] and lvls == [3, 3]


def test_tree_accept_by_hand():
    #        row:  0   1   2   3   4   5
    window = [10, 11, 12, 21, 22, 23]
    parent = [-1, 0, 1, 0, 3, 4]
    # chain A = 11 12, chain B = 21 22 23.  The model continues 10 with 21, 21 with 22, 22 with 99.
    preds = [21, 0, 0, 22, 99, 0]
    assert anpd.tree_accept(window, parent, preds) == (2, 4, [0, 3, 4])
    # nothing matches: the root alone
    assert anpd.tree_accept(window, parent, [7, 7, 7, 7, 7, 7]) == (0, 0, [0])
    # equal depth on two candidates is impossible here (siblings hold distinct tokens); a child whose
    # parent was rejected is rejected even if its own token matches
    assert anpd.tree_accept(window, parent, [11, 5, 0, 22, 23, 0]) == (1, 1, [0, 1])
    # a chain reduces to the linear accept rule
    w, p = [3, 4, 5, 6], [-1, 0, 1, 2]
    for preds in ([4, 5, 6, 1], [4, 5, 0, 1], [0, 5, 6, 1]):
        assert anpd.tree_accept(w, p, preds)[0] == anpd.accept_length(w[1:], preds)


@pytest.mark.parametrize("fn", [periodic, hashed, mixed])
@pytest.mark.parametrize("n_cand", [1, 2, 4])
def test_multi_candidate_loop_is_lossless_on_scripted_llms(fn, n_cand):
    prompt = [10, 13, 11, 14, 12, 10, 13, 11, 14, 12, 10, 13]
    M = 40
    ref = anpd.greedy_generate(ScriptedLLM(fn), prompt, M)
    res = anpd.anpd_generate_multi(ScriptedLLM(fn), prompt, 4, n_cand, M, 31, 2, 3)
    assert res["tokens"] == ref
    for st in res["steps"]:
        assert 0 <= st["accepted"] <= 4 and len(st["window"]) <= 32
    if n_cand == 1:
        one = anpd.anpd_generate(ScriptedLLM(fn), prompt, 4, M, 2, 3)
        assert [st["window"] for st in res["steps"]] == [st["window"] for st in one["steps"]]
        assert [st["accepted"] for st in res["steps"]] == [st["accepted"] for st in one["steps"]]


def test_more_candidates_never_accept_less_from_the_same_state():
    """From one and the same committed context the first candidate is the single-candidate draft, so the
    best of several candidates is at least as long."""
    fn = mixed
    s = [10, 13, 11, 14, 12, 10, 13, 11, 14, 12, 10, 13]
    for _ in range(30):
        s.append(fn(s))
        c = s[-1]
        base = None
        for n_cand in (1, 2, 4):
            toks, pars, _ = ong.propose_tree(s, 4, n_cand, 31, 2, 4)
            llm = ScriptedLLM(fn)
            llm.ctx = s[:-1]
            a = anpd.tree_accept([c] + toks, [-1] + pars, anpd.tree_predict(llm, [c] + toks, [-1] + pars))[0]
            base = a if base is None else base
            assert a >= base


def _check(s, n_min, n_max, K, n_cand, budget):
    t = B.NgramTable(n_min, n_max, max(s) + 1)
    t.update(s)
    assert t.propose_tree(K, n_cand, budget) == ong.propose_tree(s, K, n_cand, budget, n_min, n_max)
    return t


def test_library_tree_drafts_match_the_oracle_exhaustively_on_tiny_alphabets():
    for T in range(1, 8):
        for s in itertools.product(range(3), repeat=T):
            _check(list(s), 2, 4, 3, 3, 31)
            _check(list(s), 2, 3, 2, 2, 3)


@pytest.mark.parametrize("n_min,n_max", [(2, 2), (2, 5), (3, 6)])
def test_library_tree_drafts_match_the_oracle_on_copy_heavy_streams(n_min, n_max):
    for seed in range(3):
        s = synth.markov_stream(40, 260, 0.4, 4, 16, seed)
        t = B.NgramTable(n_min, n_max, 40)
        for i, tok in enumerate(s):
            t.update([tok])
            if i % 9 == 0 or i > 245:
                for n_cand, K, budget in ((1, 5, 31), (3, 5, 31), (4, 8, 20), (2, 3, 4)):
                    assert t.propose_tree(K, n_cand, budget) == ong.propose_tree(s[:i + 1], K, n_cand, budget, n_min, n_max)
                toks, pars, lv = t.propose_tree(5, 1, 31)
                assert (toks, lv) == t.propose(5) and pars == list(range(len(toks)))


def test_tree_draft_argument_errors():
    t = B.NgramTable(2, 3, 10)
    t.update([1, 2, 1])
    assert t.propose_tree(0, 2, 31) == ([], [], [])
    assert t.propose_tree(3, 2, 0) == ([], [], [])
    with pytest.raises(B.AnpdError) as e:
        t.propose_tree(3, 0, 31)
    assert e.value.code == B.E_INVAL
