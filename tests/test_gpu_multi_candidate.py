"""Multi-candidate verification (anpd_verify_tree) against the oracle: every row of a draft tree must get
the logits of the linear window made of its own root-to-row path; acceptance, the cache it leaves and the
decode loop built on it."""
import numpy as np
import pytest
import torch

from oracle import anpd as oanpd
from oracle import decoder as od
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth
from helpers import TOL, gpu_logits, make_pair, top2_gap

pytestmark = pytest.mark.gpu


def _oracle_tree_logits(dec, window, parent):
    """Row r: last row of the oracle's forward over the path root .. r (nothing committed)."""
    return np.stack([dec.forward([window[i] for i in oanpd.tree_path(parent, r)])[-1] for r in range(len(window))])


def _tree_logits(model, kv, window, parent):
    buf = torch.empty(len(window), model.vocab, dtype=torch.float32, device="cuda")
    a, nxt, path, preds = B.verify_tree(model, kv, window, parent, want_predicts=True, out_logits=buf)
    return a, nxt, path, preds, buf.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("rows", [11, 8])   # 8 rows: the one-kernel step in its draft-tree form (bf16 shapes)
@pytest.mark.parametrize("shape_name,tol", [("TINY", "f32"), ("TINY_BF16", "bf16"), ("MID_BF16", "bf16")])
def test_tree_rows_match_their_linear_windows(shape_name, tol, rows):
    shape = getattr(synth, shape_name)
    L = 45   # not a multiple of the page size
    dec, model, kv = make_pair(shape, 31, 160)
    prompt = synth.markov_stream(shape.vocab, L, 0.3, 4, 12, 9)
    dec.prefill(prompt)
    B.prefill(model, kv, prompt)
    # the oracle's own greedy continuation of some root token
    root = 7
    g, ctx = [], [root]
    for _ in range(4):
        g.append(od.argmax(dec.forward(ctx)[-1]))
        ctx.append(g[-1])
    wrong = lambda t: (t + 1) % shape.vocab
    #   row:      0     1      2            3            4          5     6     7      8          9         10
    window = [root, g[0], wrong(g[1]), wrong(g[0]), wrong(g[0]), g[0], g[1], g[2], wrong(g[3]), wrong(g[2]), 5]
    parent = [-1,   0,    1,           0,           3,           0,    5,    6,    7,           6,           9]
    # candidates: (g0, x)  (x, x)  (g0, g1, g2, x)  and a side branch below row 6
    if rows == 8:
        #   row:      0     1      2            3           4     5     6     7
        window = [root, g[0], wrong(g[1]), wrong(g[0]), g[0], g[1], g[2], wrong(g[3])]
        parent = [-1,   0,    1,           0,           0,    4,    5,    6]
    ref = _oracle_tree_logits(dec, window, parent)
    a, nxt, path, preds, got = _tree_logits(model, kv, window, parent)
    err = float(np.max(np.abs(got - ref)))
    assert err < TOL[tol], err
    clear = all(top2_gap(ref[r]) > TOL[tol] for r in range(len(window)))
    ref_preds = [od.argmax(ref[r]) for r in range(len(window))]
    a_ref, best_ref, path_ref = oanpd.tree_accept(window, parent, ref_preds)
    # two rows hold the same first token: the deeper candidate wins
    assert a_ref == 3 and path_ref == ([0, 5, 6, 7] if rows == 11 else [0, 4, 5, 6])
    if tol == "f32":
        assert clear
    if clear:
        assert preds == ref_preds and (a, nxt, path) == (a_ref, ref_preds[best_ref], path_ref)
    assert kv.length == L + 1 + a
    # the cache now holds the winning path at consecutive positions: compare with the oracle's after it
    # commits the same path, then run a linear step on top
    dec.forward([window[r] for r in path])
    dec.set_length(L + 1 + a)
    for layer in range(shape.n_layers):
        k_gpu, v_gpu = kv.read(layer, L, 1 + a)
        k_ref, v_ref = dec.kv_read(layer, L, 1 + a)
        assert float(np.max(np.abs(k_gpu.cpu().numpy() - k_ref))) < (2e-2 if tol == "bf16" else 1e-5)
        assert float(np.max(np.abs(v_gpu.cpu().numpy() - v_ref))) < (2e-2 if tol == "bf16" else 1e-5)
    nxt_window = [nxt] + synth.random_tokens(shape.vocab, 4, 77)
    want = dec.forward(nxt_window)
    _, _, _, have = gpu_logits(model, kv, nxt_window)
    assert float(np.max(np.abs(have - want))) < TOL[tol]


def test_a_chain_is_bit_identical_to_the_linear_step():
    shape = synth.MID_BF16
    w = synth.make_weights(shape, 32, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=200)
    kv_a, kv_b = B.KVCache(model, 200), B.KVCache(model, 200)
    prompt = synth.markov_stream(shape.vocab, 70, 0.3, 4, 12, 10)
    c = B.prefill(model, kv_a, prompt)
    B.prefill(model, kv_b, prompt)
    for n in (1, 6, 8, 13, 29):
        window = [c] + synth.random_tokens(shape.vocab, n - 1, 50 + n)
        kv_a.truncate(70)
        kv_b.truncate(70)
        a1, n1, p1, lin = gpu_logits(model, kv_a, window)
        a2, n2, path, p2, tree = _tree_logits(model, kv_b, window, list(range(-1, n - 1)))
        assert (a1, n1, p1) == (a2, n2, p2) and path == list(range(a2 + 1))
        assert np.array_equal(lin, tree)
        assert kv_a.length == kv_b.length
        for layer in range(shape.n_layers):
            ka, va = kv_a.read(layer, 70, 1 + a1)
            kb, vb = kv_b.read(layer, 70, 1 + a2)
            assert torch.equal(ka, kb) and torch.equal(va, vb)


@pytest.mark.parametrize("n_cand", [2, 4])
def test_multi_candidate_generation_reproduces_greedy_decoding(n_cand):
    shape = synth.MID_BF16
    w = synth.make_weights(shape, 33, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=400)
    kv = B.KVCache(model, 400)
    prompt = synth.markov_stream(shape.vocab, 180, 0.4, 4, 16, 6)
    greedy = B.greedy_generate(model, kv, prompt, 64)
    kv.truncate(0)
    table = B.NgramTable(2, 5, shape.vocab)
    one = B.anpd_generate(model, kv, table, prompt, 5, 64)
    kv.truncate(0)
    res = B.anpd_generate_multi(model, kv, B.NgramTable(2, 5, shape.vocab), prompt, 5, n_cand, 64)
    assert one["tokens"] == greedy
    # a tree row sums the same terms as the plain step in another order: equal except where two logits tie to rounding
    same = sum(1 for x, y in zip(res["tokens"], greedy) if x == y)
    assert res["tokens"] == greedy, same
    assert res["n_steps"] <= one["n_steps"]


def test_tree_argument_errors_leave_the_cache_alone():
    shape = synth.TINY_BF16
    w = synth.make_weights(shape, 34, device="cuda")
    model = B.Model(shape, w, max_window=8, max_positions=64)
    kv = B.KVCache(model, 64)
    B.prefill(model, kv, synth.markov_stream(shape.vocab, 20, 0.3, 4, 12, 8))
    for window, parent, code in (([1, 2, 3], [-1, 0, 2], B.E_INVAL), ([1, 2, 3], [0, 0, 1], B.E_INVAL),
                                 ([1, 2, 3], [-1, -1, 0], B.E_INVAL), ([1, shape.vocab], [-1, 0], B.E_RANGE),
                                 (list(range(9)), [-1] + list(range(8)), B.E_CAPACITY)):
        with pytest.raises(B.AnpdError) as e:
            B.verify_tree(model, kv, window, parent)
        assert e.value.code == code and kv.length == 20
