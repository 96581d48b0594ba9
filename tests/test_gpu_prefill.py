"""Prompt processing in one pass (anpd_prefill) against the fp64 oracle: the last row's logits and
first generated token, the cache it leaves behind, and the verification steps that follow."""
import numpy as np
import pytest
import torch

from oracle import decoder as od
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth
from helpers import TOL, gpu_logits, make_pair, top2_gap

pytestmark = pytest.mark.gpu


def _prompt(shape, n, seed):
    return synth.markov_stream(shape.vocab, n, 0.3, 4, 12, seed)


def _check_cache(shape, dec, kv, pos0, n):
    """K and V of positions pos0 .. pos0 + n - 1, every layer: bf16 values that agree with the
    oracle's except where a rounding decision fell the other way (one unit in the last place)."""
    for layer in range(shape.n_layers):
        k_gpu, v_gpu = kv.read(layer, pos0, n)
        k_ref, v_ref = dec.kv_read(layer, pos0, n)
        for got, ref in ((k_gpu.cpu().numpy().astype(np.float64), k_ref), (v_gpu.cpu().numpy().astype(np.float64), v_ref)):
            excess = float(np.max(np.abs(got - ref) - 2.0 ** -7 * np.abs(ref)))
            assert excess < 5e-4, (layer, excess)   # small-magnitude elements: absolute error of the fp32 arithmetic
            assert np.mean(got == ref) > 0.85, (layer, float(np.mean(got == ref)))   # most roundings fall the same way


@pytest.mark.parametrize("shape_name,P", [("TINY_BF16", 77), ("TINY_BF16", 16), ("MID_BF16", 1), ("MID_BF16", 200),
                                          ("MID_BF16", 333)])
def test_prefill_matches_the_oracle(shape_name, P):
    shape = getattr(synth, shape_name)
    dec, model, kv = make_pair(shape, 21, P + 40)
    prompt = _prompt(shape, P, 3)
    ref = dec.forward(prompt)
    dec.set_length(P)
    buf = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    nxt = B.prefill(model, kv, prompt, out_logits=buf)
    assert kv.length == P
    got = buf.cpu().numpy().astype(np.float64)
    assert float(np.max(np.abs(got - ref[-1]))) < TOL["bf16"]
    if top2_gap(ref[-1]) > TOL["bf16"]:
        assert nxt == od.argmax(ref[-1])
    assert nxt == int(np.argmax(got))
    _check_cache(shape, dec, kv, 0, P)
    # verification steps on top of that cache
    for M in (6, 1, 17):
        window = synth.random_tokens(shape.vocab, M, 40 + M)
        want = dec.forward(window)
        kv.truncate(P)
        _, _, _, have = gpu_logits(model, kv, window)
        assert float(np.max(np.abs(have - want))) < TOL["bf16"], M


def test_prompt_fed_in_pieces_is_bit_identical_and_lengths_need_no_alignment():
    """37 + 50 + 1 + 112 rows against 200 at once: a row's arithmetic does not depend on how the
    prompt was cut, nor on where in its cache page the piece starts."""
    shape = synth.MID_BF16
    dec, model, kv = make_pair(shape, 22, 260)
    kv2 = B.KVCache(model, 260)
    prompt = _prompt(shape, 200, 4)
    one = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    pieces = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    n1 = B.prefill(model, kv, prompt, out_logits=one)
    lo = 0
    for n in (37, 50, 1, 112):
        n2 = B.prefill(model, kv2, prompt[lo:lo + n], out_logits=pieces)
        lo += n
        assert kv2.length == lo
    assert n1 == n2 and torch.equal(one, pieces)
    for layer in range(shape.n_layers):
        ka, va = kv.read(layer, 0, 200)
        kb, vb = kv2.read(layer, 0, 200)
        assert torch.equal(ka, kb) and torch.equal(va, vb)
    # and the second piece alone against the oracle (rows 37 .. 86 start in the middle of a page)
    ref = dec.forward(prompt[:87])
    kv2.truncate(37)
    n3 = B.prefill(model, kv2, prompt[37:87], out_logits=pieces)
    assert float(np.max(np.abs(pieces.cpu().numpy().astype(np.float64) - ref[-1]))) < TOL["bf16"]
    if top2_gap(ref[-1]) > TOL["bf16"]:
        assert n3 == od.argmax(ref[-1])


def test_one_pass_and_windowed_prompt_agree_to_rounding():
    shape = synth.MID_BF16
    w = synth.make_weights(shape, 23, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=300)
    kv_a, kv_b = B.KVCache(model, 300), B.KVCache(model, 300)
    prompt = _prompt(shape, 150, 5)
    la = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    B.prefill(model, kv_a, prompt, out_logits=la)
    B.prefill_windows(model, kv_b, prompt[:-1])
    lb = torch.empty(1, shape.vocab, dtype=torch.float32, device="cuda")
    B.verify(model, kv_b, prompt[-1:], B.APPEND, out_logits=lb)
    assert kv_a.length == kv_b.length == 150
    assert float((la - lb[0]).abs().max()) < 5e-3
    for layer in range(shape.n_layers):
        ka, va = kv_a.read(layer, 0, 150)
        kb, vb = kv_b.read(layer, 0, 150)
        assert float(((ka - kb).abs() - 2.0 ** -7 * kb.abs()).max()) < 5e-4
        assert float((ka == kb).float().mean()) > 0.85 and float((va == vb).float().mean()) > 0.85


def test_scrambled_pages_and_generation_after_a_one_pass_prompt():
    """Pages handed out in a scrambled order; ANPD after the one-pass prompt still reproduces
    plain greedy decoding token for token, and both follow the oracle while its top-2 gap is clear."""
    shape = synth.MID_BF16
    dec, model, kv = make_pair(shape, 24, 400)
    n = kv.num_pages
    kv.set_page_order([(7 * i + 3) % n for i in range(n)])
    prompt = synth.markov_stream(shape.vocab, 180, 0.4, 4, 16, 6)
    greedy = B.greedy_generate(model, kv, prompt, 48)
    kv.truncate(0)
    table = B.NgramTable(2, 5, shape.vocab)
    res = B.anpd_generate(model, kv, table, prompt, 5, 48)
    assert res["tokens"] == greedy
    assert res["n_steps"] < 48
    # oracle greedy, teacher-forced with the GPU's tokens
    c = dec.prefill(prompt)
    for t in greedy[:12]:
        logits = dec.forward([c])
        if top2_gap(logits[0]) <= TOL["bf16"]:
            break
        assert c == t
        dec.set_length(dec.length + 1)
        c = od.argmax(logits[0])


def test_dot_product_models_take_the_windowed_route():
    shape = synth.TINY
    dec, model, kv = make_pair(shape, 25, 200, max_window=8)
    kv2 = B.KVCache(model, 200)
    prompt = _prompt(shape, 61, 7)
    assert B.prefill_workspace_bytes(model, 61) == 0
    la = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    na = B.prefill(model, kv, prompt, out_logits=la)
    nb = B.prefill_windows(model, kv2, prompt)
    assert na == nb and kv.length == kv2.length == 61
    ref = dec.forward(prompt)
    assert float(np.max(np.abs(la.cpu().numpy().astype(np.float64) - ref[-1]))) < TOL["f32"]
    assert na == od.argmax(ref[-1])


def test_prefill_rejects_bad_input_and_leaves_the_cache_alone():
    shape = synth.TINY_BF16
    w = synth.make_weights(shape, 26, device="cuda")
    model = B.Model(shape, w, max_window=8, max_positions=64)
    kv = B.KVCache(model, 64)
    B.prefill(model, kv, _prompt(shape, 20, 8))
    for bad, code in (([1, 2, shape.vocab], B.E_RANGE), ([-1], B.E_RANGE), (list(range(45)), B.E_CAPACITY), ([], B.E_INVAL)):
        with pytest.raises(B.AnpdError) as e:
            B.prefill(model, kv, bad)
        assert e.value.code == code
        assert kv.length == 20
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    import ctypes as C
    out = C.c_int32(0)
    rc = B.lib().anpd_prefill(model._h, kv._h, (C.c_int32 * 3)(1, 2, 3), 3, C.byref(out), 0, small.data_ptr(), 256, 0)
    assert rc == B.E_CAPACITY and kv.length == 20
