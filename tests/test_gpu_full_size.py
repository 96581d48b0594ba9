"""Parity at the benchmark's own sizes and launch configuration, and at the other
workloads' distinguishing shapes (13B widths, long paged context)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import anpd as oanpd
from oracle import decoder as od
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth
from helpers import TOL, top2_gap

pytestmark = pytest.mark.gpu


def _seed_both(shape, dec, kvs, n_tokens, seed):
    for layer in range(shape.n_layers):
        k, v = synth.kv_fill(shape, seed, layer, n_tokens, device="cuda")
        kf, vf = k.float().contiguous(), v.float().contiguous()
        dec.kv_load(layer, 0, kf.cpu().numpy(), vf.cpu().numpy())
        for kv in kvs:
            kv.write(layer, 0, kf, vf)
    dec.set_length(n_tokens)
    for kv in kvs:
        kv.truncate(n_tokens)


def _check_cache_rows(shape, dec, kv, pos0, n, layers):
    """K and V of positions pos0 .. pos0 + n - 1 in the given layers: bf16 values that agree with the
    oracle's except where a rounding decision fell the other way (one unit in the last place, 2^-7
    relative), plus the absolute error that 32 or 40 layers of bf16-weight arithmetic leave on elements
    of small magnitude."""
    for layer in layers:
        k_gpu, v_gpu = kv.read(layer, pos0, n)
        k_ref, v_ref = dec.kv_read(layer, pos0, n)
        for got, want in ((k_gpu.cpu().numpy().astype(np.float64), k_ref), (v_gpu.cpu().numpy().astype(np.float64), v_ref)):
            assert got.shape == want.shape
            excess = float(np.max(np.abs(got - want) - 2.0 ** -7 * np.abs(want)))
            assert excess < 5e-3, (layer, excess)
            assert np.mean(got == want) > 0.7, (layer, float(np.mean(got == want)))   # most roundings fall the same way


def _step_logits(model, kv, window):
    buf = torch.empty(len(window), model.vocab, dtype=torch.float32, device="cuda")
    a, nxt, preds = B.verify(model, kv, window, B.VERIFY, want_predicts=True, out_logits=buf)
    return a, nxt, preds, buf


def test_llama7b_step_in_the_bench_configuration():
    """One verification step of the 7B shape, window 6, 512 cached tokens: the persistent kernel
    (what bench.py times) against the fp64 oracle on all 6 x 32000 logits, and against the
    one-launch-per-operation path bit for bit."""
    shape = synth.LLAMA_7B
    L, K = 512, 5
    w = synth.make_weights(shape, 2, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=L + 64)
    model_l = B.Model(shape, w, max_window=32, max_positions=L + 64, gemm_path=B.GEMM_MFMA_LAUNCHES)
    kv, kv_l = B.KVCache(model, L + 64), B.KVCache(model_l, L + 64)
    w_host = {k_: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k_, v in w.items()}
    dec = od.Decoder(shape, w_host, L + 64)
    _seed_both(shape, dec, [kv, kv_l], L, seed=7)
    window = synth.random_tokens(shape.vocab, K + 1, 5)

    ref = dec.forward(window)
    a, nxt, preds, got = _step_logits(model, kv, window)
    a2, nxt2, preds2, got2 = _step_logits(model_l, kv_l, window)
    assert torch.equal(got, got2) and (a, nxt, preds) == (a2, nxt2, preds2)
    g = got.cpu().numpy().astype(np.float64)
    err = float(np.max(np.abs(g - ref)))
    print("7B step: max |logit error| = %.2e, logit std %.3f" % (err, float(np.std(ref))))
    assert err < TOL["bf16"]
    assert np.std(ref) > 0.3
    ref_preds = [od.argmax(ref[r]) for r in range(K + 1)]
    for r in range(K + 1):
        if top2_gap(ref[r]) > TOL["bf16"]:
            assert preds[r] == ref_preds[r]
    a_ref = oanpd.accept_length(window[1:], ref_preds)
    if all(top2_gap(ref[r]) > TOL["bf16"] for r in range(a_ref + 1)):
        assert (a, nxt) == (a_ref, ref_preds[a_ref])
    assert kv.length == L + 1 + a

    # row 0 of the window == the plain greedy step at the same position, bit for bit
    kv.truncate(L)
    _, _, _, one = _step_logits(model, kv, window[:1])
    assert torch.equal(one[0], got[0])
    # the K and V rows the step wrote match the oracle's cache (bf16 storage, rounding ties aside)
    dec.set_length(L + 1)
    _check_cache_rows(shape, dec, kv, L, 1, (0, shape.n_layers // 2, shape.n_layers - 1))

    # windows of 9 and 16 rows (one kernel, two operand fragments) and of 17 (separate launches, four):
    # against the oracle, row for row the bits of the widest window, and 9 / 16 rows also against the
    # one-launch-per-operation path
    wide = synth.random_tokens(shape.vocab, 17, 21)
    dec.set_length(L)
    ref = dec.forward(wide)
    full = None
    for M in (17, 16, 9):
        kv.truncate(L)
        _, _, preds, got = _step_logits(model, kv, wide[:M])
        err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref[:M])))
        print("7B step, %d rows: max |logit error| = %.2e" % (M, err))
        assert err < TOL["bf16"], (M, err)
        for r in range(M):
            if top2_gap(ref[r]) > TOL["bf16"]:
                assert preds[r] == od.argmax(ref[r])
        if full is None:
            full = got
        else:
            assert torch.equal(got, full[:M]), M
            kv_l.truncate(L)
            _, _, preds_l, got_l = _step_logits(model_l, kv_l, wide[:M])
            assert torch.equal(got, got_l) and preds == preds_l, M


def test_llama13b_step_at_full_depth():
    """All 40 layers of the 13B shape (d_model 5120, 40 heads, FFN 13824), 300 cached positions: the
    workload's window of 9 rows (separate launches, two operand fragments) and windows of 8 rows and 1 row
    (the one-kernel step with work items of 10 k-steps) against the oracle; rows agree bit for bit across
    the window sizes, and the one-kernel step with the one-launch-per-operation path."""
    shape = synth.LLAMA_13B
    L = 300
    w = synth.make_weights(shape, 4, device="cuda")
    model = B.Model(shape, w, max_window=16, max_positions=L + 32)
    model_l = B.Model(shape, w, max_window=16, max_positions=L + 32, gemm_path=B.GEMM_MFMA_LAUNCHES)
    kv, kv_l = B.KVCache(model, L + 32), B.KVCache(model_l, L + 32)
    w_host = {k_: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k_, v in w.items()}
    dec = od.Decoder(shape, w_host, L + 32)
    _seed_both(shape, dec, [kv, kv_l], L, seed=8)
    window = synth.random_tokens(shape.vocab, 9, 11)
    ref = dec.forward(window)
    full = None
    for M in (9, 8, 1):
        kv.truncate(L)
        kv_l.truncate(L)
        a, nxt, preds, got = _step_logits(model, kv, window[:M])
        a2, nxt2, preds2, got2 = _step_logits(model_l, kv_l, window[:M])
        assert torch.equal(got, got2) and (a, nxt, preds) == (a2, nxt2, preds2), M
        err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref[:M])))
        print("13B step, %d rows: max |logit error| = %.2e, logit std %.3f" % (M, err, float(np.std(ref))))
        assert err < TOL["bf16"], (M, err)
        for r in range(M):
            if top2_gap(ref[r]) > TOL["bf16"]:
                assert preds[r] == od.argmax(ref[r])
        if full is None:
            full = got
        else:
            assert torch.equal(got, full[:M]), M
    dec.set_length(L + 1)
    _check_cache_rows(shape, dec, kv, L, 1, (0, shape.n_layers - 1))


def test_llama7b_long_context_in_permuted_pages():
    """The long-context workload's own shape: 7B, 3584 cached positions in 16-token pages handed out in a
    scrambled order, windows of 17 rows (its k + 1; separate launches), 16 and 9 (one kernel, two operand
    fragments), 8 and 1 (one kernel).  Every size against the oracle; rows agree bit for bit across sizes."""
    shape = synth.LLAMA_7B
    L = 3584
    w = synth.make_weights(shape, 2, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=L + 64)
    kv = B.KVCache(model, L + 64)
    n = kv.num_pages
    kv.set_page_order([(37 * i + 11) % n for i in range(n)])
    w_host = {k_: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k_, v in w.items()}
    dec = od.Decoder(shape, w_host, L + 64)
    _seed_both(shape, dec, [kv], L, seed=9)
    window = synth.random_tokens(shape.vocab, 17, 13)
    ref = dec.forward(window)
    full = None
    for M in (17, 16, 9, 8, 1):
        kv.truncate(L)
        _, _, preds, got = _step_logits(model, kv, window[:M])
        err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref[:M])))
        print("7B step over %d positions, %d rows: max |logit error| = %.2e" % (L, M, err))
        assert err < TOL["bf16"], (M, err)
        for r in range(M):
            if top2_gap(ref[r]) > TOL["bf16"]:
                assert preds[r] == od.argmax(ref[r])
        if full is None:
            full = got
        else:
            assert torch.equal(got, full[:M]), M
    dec.set_length(L + 1)
    _check_cache_rows(shape, dec, kv, L, 1, (0, shape.n_layers - 1))


def test_13b_widths_two_layers():
    """d_model 5120, 40 heads, FFN 13824: the register-resident GEMM form with 20 k-steps per wave
    and the streaming form at K = 13824, windows of 9 (the 13B workload's k + 1) and fewer rows."""
    shape = dataclasses.replace(synth.LLAMA_13B, n_layers=2)
    L = 300
    w = synth.make_weights(shape, 4, device="cuda")
    model = B.Model(shape, w, max_window=16, max_positions=L + 32)
    kv = B.KVCache(model, L + 32)
    w_host = {k_: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k_, v in w.items()}
    dec = od.Decoder(shape, w_host, L + 32)
    _seed_both(shape, dec, [kv], L, seed=8)
    full = None
    for M in (9, 1, 6):
        kv.truncate(L)
        window = synth.random_tokens(shape.vocab, 9, 11)[:M]
        ref = dec.forward(window)
        _, _, preds, got = _step_logits(model, kv, window)
        err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref)))
        assert err < TOL["bf16"], (M, err)
        for r in range(M):
            if top2_gap(ref[r]) > TOL["bf16"]:
                assert preds[r] == od.argmax(ref[r])
        if full is None:
            full = got
        else:
            assert torch.equal(got, full[:M])


def test_long_paged_context_and_adaptive_draft_length():
    """3584 cached tokens in 16-token pages handed out in a scrambled order; windows up to 17 rows."""
    shape = synth.MID_BF16
    L = 3584
    w = synth.make_weights(shape, 5)
    wc = {k_: ([t.cuda() for t in v] if isinstance(v, list) else v.cuda()) for k_, v in w.items()}
    model = B.Model(shape, wc, max_window=32, max_positions=L + 600)
    kv = B.KVCache(model, L + 600)
    n = kv.num_pages
    kv.set_page_order([(37 * i + 11) % n for i in range(n)])
    dec = od.Decoder(shape, w, L + 600)
    _seed_both(shape, dec, [kv], L, seed=9)
    full = None
    for M in (17, 1, 9, 6):
        kv.truncate(L)
        window = synth.random_tokens(shape.vocab, 17, 13)[:M]
        ref = dec.forward(window)
        _, _, _, got = _step_logits(model, kv, window)
        assert float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref))) < TOL["bf16"]
        if full is None:
            full = got
        else:
            assert torch.equal(got, full[:M])
    # adaptive draft length from the level that answered the first draft: k = 2^(level - 2), 1..16
    kv.truncate(0)
    prompt = synth.markov_stream(shape.vocab, 400, 0.2, 4, 16, 5)
    ref_tokens = B.greedy_generate(model, kv, prompt, 96)
    kv.truncate(0)
    table = B.NgramTable(2, 6, shape.vocab)
    res = B.anpd_generate(model, kv, table, prompt, 16, 96, adaptive=True)
    assert res["tokens"] == ref_tokens
    assert res["n_steps"] <= 96


def test_llama7b_prompt_in_one_pass():
    """anpd_prefill at the 7B shape.  (a) 48 rows appended behind 500 seeded positions (the piece
    starts in the middle of a cache page): last-row logits and the K / V rows of the last layer
    against the oracle.  (b) The benchmark's 512-token prompt in the launch configuration bench.py
    times: the oracle cannot follow at that size, so the check is agreement with the same prompt
    appended through the verification step in 32-row windows, a path the oracle covers above."""
    shape = synth.LLAMA_7B
    L, P = 500, 48
    w = synth.make_weights(shape, 2, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=640)
    kv, kv_w = B.KVCache(model, 640), B.KVCache(model, 640)
    w_host = {k_: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k_, v in w.items()}
    dec = od.Decoder(shape, w_host, 640)
    _seed_both(shape, dec, [kv], L, seed=7)
    tokens = synth.random_tokens(shape.vocab, P, 17)
    ref = dec.forward(tokens)
    buf = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    nxt = B.prefill(model, kv, tokens, out_logits=buf)
    assert kv.length == L + P
    err = float(np.max(np.abs(buf.cpu().numpy().astype(np.float64) - ref[-1])))
    print("7B prompt piece: max |logit error| of the last row = %.2e" % err)
    assert err < TOL["bf16"]
    if top2_gap(ref[-1]) > TOL["bf16"]:
        assert nxt == od.argmax(ref[-1])
    dec.set_length(L + P)
    k_gpu, v_gpu = kv.read(shape.n_layers - 1, L, P)
    k_ref, v_ref = dec.kv_read(shape.n_layers - 1, L, P)
    for got, want in ((k_gpu.cpu().numpy().astype(np.float64), k_ref), (v_gpu.cpu().numpy().astype(np.float64), v_ref)):
        assert float(np.max(np.abs(got - want) - 2.0 ** -7 * np.abs(want))) < 5e-3
        assert np.mean(got == want) > 0.7
    del dec

    prompt = synth.workload_prompt("llama7b")
    kv.truncate(0)
    one = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    n_one = B.prefill(model, kv, prompt, out_logits=one)
    B.prefill_windows(model, kv_w, prompt[:-1])
    win = torch.empty(1, shape.vocab, dtype=torch.float32, device="cuda")
    _, n_win = B.verify(model, kv_w, prompt[-1:], B.APPEND, out_logits=win)
    assert kv.length == kv_w.length == len(prompt)
    diff = float((one - win[0]).abs().max())
    print("7B prompt of %d rows: one pass vs windows, max |logit difference| = %.2e" % (len(prompt), diff))
    assert diff < TOL["bf16"]
    srt = torch.sort(win[0], descending=True).values
    if float(srt[0] - srt[1]) > TOL["bf16"]:
        assert n_one == n_win
    for layer in (0, shape.n_layers - 1):
        ka, va = kv.read(layer, 0, len(prompt))
        kb, vb = kv_w.read(layer, 0, len(prompt))
        # two bf16 roundings of values that carry the rounding noise of up to 32 layers
        assert float((ka - kb).abs().max()) < 0.05 and float((va - vb).abs().max()) < 0.05
        assert float((ka - kb).abs().mean()) < 2e-3 and float((va - vb).abs().mean()) < 2e-3


def test_glm6b_shape_step_with_grouped_heads():
    """The second model shape at full size (28 layers, 32 query heads over 2 key / value heads, FFN 13696,
    vocabulary 65024): one verification step of 6 rows over 512 seeded positions, the persistent kernel
    against the oracle and against the one-launch-per-operation path bit for bit."""
    shape = synth.GLM_6B
    L, K = 512, 5
    w = synth.make_weights(shape, 6, device="cuda")
    model = B.Model(shape, w, max_window=8, max_positions=L + 64)
    model_l = B.Model(shape, w, max_window=8, max_positions=L + 64, gemm_path=B.GEMM_MFMA_LAUNCHES)
    kv, kv_l = B.KVCache(model, L + 64), B.KVCache(model_l, L + 64)
    w_host = {k_: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k_, v in w.items()}
    dec = od.Decoder(shape, w_host, L + 64)
    _seed_both(shape, dec, [kv, kv_l], L, seed=10)
    window = synth.random_tokens(shape.vocab, K + 1, 6)
    ref = dec.forward(window)
    a, nxt, preds, got = _step_logits(model, kv, window)
    a2, nxt2, preds2, got2 = _step_logits(model_l, kv_l, window)
    assert torch.equal(got, got2) and (a, nxt, preds) == (a2, nxt2, preds2)
    err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref)))
    print("GLM-6B shape step: max |logit error| = %.2e" % err)
    assert err < TOL["bf16"]
    for r in range(K + 1):
        if top2_gap(ref[r]) > TOL["bf16"]:
            assert preds[r] == od.argmax(ref[r])
    k_gpu, _ = kv.read(shape.n_layers - 1, L, 1)
    assert k_gpu.shape == (1, shape.kv_dim)
    dec.set_length(L + 1)
    _check_cache_rows(shape, dec, kv, L, 1, (0, shape.n_layers - 1))


def test_phases_of_one_two_and_three_items_per_block():
    """d_model 2048, FFN 6144, vocabulary 8192 on 256 compute units: QKV 384 tiles of one item (blocks with one
    and with two), O 128 tiles (half the blocks have none), gate/up three items per block, down one tile of
    three items with the operand streamed, LM head two: the ends of the persistent kernel's weight ring.
    Against the oracle, and against the one-launch-per-operation path bit for bit."""
    shape = synth.RING_BF16
    L = 200
    w = synth.make_weights(shape, 9, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=L + 64)
    model_l = B.Model(shape, w, max_window=32, max_positions=L + 64, gemm_path=B.GEMM_MFMA_LAUNCHES)
    kv, kv_l = B.KVCache(model, L + 64), B.KVCache(model_l, L + 64)
    w_host = {k_: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k_, v in w.items()}
    dec = od.Decoder(shape, w_host, L + 64)
    _seed_both(shape, dec, [kv, kv_l], L, seed=10)
    for M in (8, 1, 5):
        kv.truncate(L)
        kv_l.truncate(L)
        window = synth.random_tokens(shape.vocab, 8, 12)[:M]
        ref = dec.forward(window)
        a, nxt, preds, got = _step_logits(model, kv, window)
        a2, nxt2, preds2, got2 = _step_logits(model_l, kv_l, window)
        assert torch.equal(got, got2) and (a, nxt, preds) == (a2, nxt2, preds2), M
        err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref)))
        assert err < TOL["bf16"], (M, err)
        for r in range(M):
            if top2_gap(ref[r]) > TOL["bf16"]:
                assert preds[r] == od.argmax(ref[r])


def test_two_fragment_windows_repeat_their_bits_after_other_steps():
    """Windows of 9 to 15 rows run the one-kernel step with two operand fragments of which the second is partly
    filled.  Their bits must not depend on what ran before: every repetition, after a 17-row step (separate
    launches) or a 16-row step (the same kernel) on the same model, equals the one-launch-per-operation path.
    (A step that read its LDS copy of the operand before the copy had arrived got one tile in some ten
    thousand wrong: a few repetitions of 32 layers x 4 phases x 256 tiles find that.)"""
    shape = synth.LLAMA_7B
    L = 512
    w = synth.make_weights(shape, 2, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=L + 64)
    model_l = B.Model(shape, w, max_window=32, max_positions=L + 64, gemm_path=B.GEMM_MFMA_LAUNCHES)
    kv, kv_l = B.KVCache(model, L + 64), B.KVCache(model_l, L + 64)
    for layer in range(shape.n_layers):
        k, v = synth.kv_fill(shape, 7, layer, L, device="cuda")
        kf, vf = k.float().contiguous(), v.float().contiguous()
        kv.write(layer, 0, kf, vf)
        kv_l.write(layer, 0, kf, vf)
    wide = synth.random_tokens(shape.vocab, 17, 21)

    def run(m, k_, M):
        k_.truncate(L)
        buf = torch.empty(M, m.vocab, dtype=torch.float32, device="cuda")
        B.verify(m, k_, wide[:M], B.APPEND, out_logits=buf)
        return buf

    for M in (9, 12, 15):
        want = run(model_l, kv_l, M)
        for it in range(24):
            run(model, kv, 17 if it % 2 == 0 else 16)
            got = run(model, kv, M)
            assert torch.equal(got, want), (M, it)
