"""Grouped key / value heads (n_kv_heads < n_heads, the arrangement of the ChatGLM model the paper also
evaluates) through every device path, against the oracle: windows of all classes, the one-pass prompt,
draft trees, cache import / export, and the decode loops."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoder as od
from oracle import anpd as oanpd
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth
from helpers import TOL, gpu_logits, make_pair, seed_kv_both, top2_gap

pytestmark = pytest.mark.gpu

SHAPES = [("TINY_MQA", "f32"), ("TINY_MQA_BF16", "bf16"), ("MID_GQA", "bf16")]


@pytest.mark.parametrize("shape_name,tol", SHAPES)
def test_windows_of_every_class_match_the_oracle(shape_name, tol):
    shape = getattr(synth, shape_name)
    L = 150
    dec, model, kv = make_pair(shape, 41, 260)
    seed_kv_both(shape, dec, kv, L, 42)
    k, v = kv.read(0, 0, L)
    assert k.shape == (L, shape.kv_dim) and v.shape == (L, shape.kv_dim)
    k_ref, v_ref = dec.kv_read(0, 0, L)
    assert np.array_equal(k.cpu().numpy().astype(np.float64), k_ref) and np.array_equal(v.cpu().numpy().astype(np.float64), v_ref)
    full = None
    for M in (29, 1, 6, 8, 13):
        kv.truncate(L)
        window = synth.random_tokens(shape.vocab, 29, 43)[:M]
        ref = dec.forward(window)
        a, nxt, preds, got = gpu_logits(model, kv, window)
        assert float(np.max(np.abs(got - ref))) < TOL[tol], M
        for r in range(M):
            if top2_gap(ref[r]) > TOL[tol]:
                assert preds[r] == od.argmax(ref[r])
        if full is None:
            full = got
        else:
            assert np.array_equal(got, full[:M])   # a row does not depend on the window it came in
    # what the step wrote
    kv.truncate(L)
    window = synth.random_tokens(shape.vocab, 5, 44)
    dec.forward(window)
    B.verify(model, kv, window, B.APPEND)
    for layer in range(shape.n_layers):
        k, v = kv.read(layer, L, 5)
        k_ref, v_ref = dec.kv_read(layer, L, 5)
        lim = 2e-2 if tol == "bf16" else 1e-5
        assert float(np.max(np.abs(k.cpu().numpy() - k_ref))) < lim and float(np.max(np.abs(v.cpu().numpy() - v_ref))) < lim


@pytest.mark.parametrize("shape_name", ["TINY_MQA_BF16", "MID_GQA"])
def test_one_kernel_step_equals_one_launch_per_operation(shape_name):
    shape = getattr(synth, shape_name)
    w = synth.make_weights(shape, 45, device="cuda")
    model = B.Model(shape, w, max_window=8, max_positions=300)
    model_l = B.Model(shape, w, max_window=8, max_positions=300, gemm_path=B.GEMM_MFMA_LAUNCHES)
    kv, kv_l = B.KVCache(model, 300), B.KVCache(model_l, 300)
    prompt = synth.markov_stream(shape.vocab, 140, 0.3, 4, 12, 12)
    assert B.prefill(model, kv, prompt) == B.prefill(model_l, kv_l, prompt)
    for M in (1, 5, 8):
        window = synth.random_tokens(shape.vocab, M, 60 + M)
        a1, n1, p1, l1 = gpu_logits(model, kv, window)
        a2, n2, p2, l2 = gpu_logits(model_l, kv_l, window)
        assert (a1, n1, p1) == (a2, n2, p2) and np.array_equal(l1, l2)


@pytest.mark.parametrize("shape_name,tol", SHAPES)
def test_prompt_tree_and_decode_loops(shape_name, tol):
    shape = getattr(synth, shape_name)
    dec, model, kv = make_pair(shape, 46, 400)
    prompt = synth.markov_stream(shape.vocab, 120, 0.4, 4, 16, 13)
    ref = dec.forward(prompt)
    dec.set_length(len(prompt))
    buf = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    c = B.prefill(model, kv, prompt, out_logits=buf)
    assert float(np.max(np.abs(buf.cpu().numpy().astype(np.float64) - ref[-1]))) < TOL[tol]
    for layer in range(shape.n_layers):
        k, v = kv.read(layer, 0, len(prompt))
        k_ref, v_ref = dec.kv_read(layer, 0, len(prompt))
        lim = 2e-2 if tol == "bf16" else 1e-5
        assert float(np.max(np.abs(k.cpu().numpy() - k_ref))) < lim and float(np.max(np.abs(v.cpu().numpy() - v_ref))) < lim
    # a draft tree of 8 rows and one of 12
    for parent in ([-1, 0, 1, 0, 3, 4, 0, 6], [-1, 0, 1, 2, 3, 0, 5, 6, 0, 8, 9, 10]):
        window = [c] + synth.random_tokens(shape.vocab, len(parent) - 1, 70 + len(parent))
        want = np.stack([dec.forward([window[i] for i in oanpd.tree_path(parent, r)])[-1] for r in range(len(window))])
        kv.truncate(len(prompt))
        out = torch.empty(len(window), shape.vocab, dtype=torch.float32, device="cuda")
        B.verify_tree(model, kv, window, parent, out_logits=out)
        assert float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - want))) < TOL[tol]
    # losslessness on the device
    kv.truncate(0)
    greedy = B.greedy_generate(model, kv, prompt, 40)
    kv.truncate(0)
    res = B.anpd_generate(model, kv, B.NgramTable(2, 4, shape.vocab), prompt, 5, 40)
    assert res["tokens"] == greedy
    kv.truncate(0)
    multi = B.anpd_generate_multi(model, kv, B.NgramTable(2, 4, shape.vocab), prompt, 3, 2, 40)
    assert multi["tokens"] == greedy


def test_bad_group_count_is_rejected():
    shape = dataclasses.replace(synth.TINY_BF16, n_kv_heads=3)
    w = synth.make_weights(dataclasses.replace(shape, n_kv_heads=1), 47, device="cuda")
    with pytest.raises(B.AnpdError) as e:
        B.Model(shape, w, max_window=8, max_positions=64)
    assert e.value.code == B.E_INVAL
