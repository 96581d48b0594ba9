"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Integer results are compared exactly; logits to
the stated max-abs tolerance (1e-4 fp32, 2e-2 bf16)."""
import numpy as np
import pytest
import torch

from oracle import anpd as oanpd
from oracle import decoder as od
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth
from helpers import TOL, gpu_logits, make_pair, seed_kv_both, to_cuda, top2_gap

pytestmark = pytest.mark.gpu

PATHS = [("f32", B.GEMM_DOT), ("bf16", B.GEMM_DOT), ("bf16", B.GEMM_MFMA), ("mid", B.GEMM_MFMA), ("mid", B.GEMM_DOT)]
LINEAR_PATHS = PATHS[:3] + [("bf16", B.GEMM_MFMA_STREAM)]


def _shape(dt):
    return {"f32": synth.TINY, "bf16": synth.TINY_BF16, "mid": synth.MID_BF16}[dt]


# ------------------------------------------------------------------ GEMM

@pytest.mark.parametrize("dt,path", LINEAR_PATHS)
@pytest.mark.parametrize("M,N,K", [(1, 64, 256), (6, 688, 256), (5, 256, 688), (8, 1024, 512),
                                   (9, 48, 1000), (16, 256, 4096), (17, 32, 40), (32, 128, 1032)])
def test_linear_against_oracle(dt, path, M, N, K):
    X = synth.approx_normal(11, M * 7 + K, M * K, 1.0).reshape(M, K)
    W = synth.approx_normal(12, N + K, N * K, 0.02).reshape(N, K)
    W = W.to(torch.bfloat16) if dt == "bf16" else W
    ref = od.linear(X.double().numpy(), od.to_numpy_weight(W))
    Y = B.linear(X.cuda(), W.cuda(), path).cpu().double().numpy()
    assert Y.shape == ref.shape
    assert np.max(np.abs(Y - ref)) < 1e-4
    assert np.std(ref) > 0.05


@pytest.mark.parametrize("dt,path", LINEAR_PATHS)
@pytest.mark.parametrize("K,N", [(688, 256), (4096, 512), (5120, 64), (11008, 32)])
def test_linear_rows_do_not_depend_on_window_size(dt, path, K, N):
    X = synth.approx_normal(13, 1, 32 * K, 1.0).reshape(32, K).cuda()
    W = synth.approx_normal(14, 2, N * K, 0.02).reshape(N, K)
    W = (W.to(torch.bfloat16) if dt == "bf16" else W).cuda()
    full = B.linear(X, W, path)
    for M in (1, 2, 6, 8, 9, 16, 17, 31):
        part = B.linear(X[:M].contiguous(), W, path)
        assert torch.equal(part, full[:M]), M


def test_both_mfma_forms_are_bit_identical():
    for K, N in [(256, 64), (4096, 4096 + 16), (5120, 48), (11008, 32)]:
        X = synth.approx_normal(15, K, 8 * K, 1.0).reshape(8, K).cuda()
        W = synth.approx_normal(16, K, N * K, 0.02).reshape(N, K).to(torch.bfloat16).cuda()
        Wp = B.pack_weights(W)
        for M in (1, 5, 8):
            a = B.linear(X[:M].contiguous(), W, B.GEMM_MFMA, packed=Wp)
            b = B.linear(X[:M].contiguous(), W, B.GEMM_MFMA_STREAM, packed=Wp)
            assert torch.equal(a, b), (K, N, M)


# -------------------------------------------------------------- whole step

@pytest.mark.parametrize("dt,path", PATHS)
def test_teacher_forced_logits_and_predictions(dt, path):
    shape = _shape(dt)
    dec, model, kv = make_pair(shape, 1, 256, gemm_path=path)
    toks = synth.markov_stream(shape.vocab, 200, 0.3, 4, 12, 7)
    pos, worst = 0, 0.0
    for n in (32, 17, 1, 6, 9, 16, 2, 32, 5, 31, 8, 3):   # ragged windows crossing pages and splits
        win = toks[pos:pos + n]
        ref = dec.forward(win)
        dec.set_length(pos + n)
        a, nxt, preds, got = gpu_logits(model, kv, win, B.APPEND)
        assert a == n - 1 and kv.length == pos + n
        err = np.max(np.abs(got - ref))
        worst = max(worst, err)
        assert err < TOL[dt], (n, err)
        for r in range(n):
            if top2_gap(ref[r]) > TOL[dt]:
                assert preds[r] == od.argmax(ref[r])
        assert nxt == preds[-1]
        pos += n
    assert np.std(ref) > 0.05
    print("max |logit error|", dt, path, worst)


@pytest.mark.parametrize("dt,path", PATHS)
@pytest.mark.parametrize("L", [0, 63, 200])
def test_seeded_cache_windows(dt, path, L):
    """Kernel-sweep style: random seeded K/V contents, windows of 1..17 rows."""
    shape = _shape(dt)
    dec, model, kv = make_pair(shape, 2, 256, gemm_path=path)
    for M in (1, 2, 4, 8, 16, 17):
        seed_kv_both(shape, dec, kv, L, seed=3)
        win = synth.random_tokens(shape.vocab, M, 40 + M)
        ref = dec.forward(win)
        preds_ref = [od.argmax(ref[r]) for r in range(M)]
        a_ref = oanpd.accept_length(win[1:], preds_ref)
        a, nxt, preds, got = gpu_logits(model, kv, win, B.VERIFY)
        assert np.max(np.abs(got - ref)) < TOL[dt]
        safe = all(top2_gap(ref[r]) > TOL[dt] for r in range(a_ref + 1))
        if safe:
            assert (a, nxt) == (a_ref, preds_ref[a_ref])
        assert kv.length == L + 1 + a


@pytest.mark.parametrize("dt,path", PATHS)
def test_accept_rule_perfect_partial_and_wrong_drafts(dt, path):
    shape = _shape(dt)
    w = synth.make_weights(shape, 1)
    prompt = synth.workload_prompt("tiny")
    _, model, kv = make_pair(shape, 1, 256, gemm_path=path, weights=w)
    g = B.greedy_generate(model, kv, prompt, 24)
    for n_right, k in [(5, 5), (2, 5), (0, 5), (0, 0), (7, 7), (3, 16)]:
        kv.truncate(0)
        c = B.prefill(model, kv, prompt)
        assert c == g[0]
        drafts = g[1:1 + n_right] + [(t + 1) % shape.vocab for t in g[1 + n_right:1 + k]]
        a, nxt, preds = B.verify(model, kv, [c] + drafts, B.VERIFY, want_predicts=True)
        assert a == n_right and nxt == g[1 + n_right]
        assert preds[:n_right + 1] == g[1:2 + n_right]
        assert kv.length == len(prompt) + 1 + n_right


@pytest.mark.parametrize("dt,path", PATHS)
@pytest.mark.parametrize("N,K", [(3, 4), (5, 7), (2, 16), (4, 0)])
def test_anpd_is_lossless_on_the_gpu(dt, path, N, K):
    """GPU ANPD == GPU greedy token for token, with no tolerance."""
    shape = _shape(dt)
    w = synth.make_weights(shape, 1)
    prompt = synth.workload_prompt("tiny")
    _, model, kv = make_pair(shape, 1, 256, gemm_path=path, weights=w)
    ref = B.greedy_generate(model, kv, prompt, 64)
    kv.truncate(0)
    table = B.NgramTable(2, N, shape.vocab)
    res = B.anpd_generate(model, kv, table, prompt, K, 64)
    assert res["tokens"] == ref
    assert res["n_steps"] + res["accepted"] >= 64
    if K == 0:
        assert res["n_steps"] == 64
    if K >= 4 and dt != "mid":
        assert res["accepted"] > 0       # the tiny model loops, drafts do hit


def test_generation_matches_oracle_until_a_near_tie():
    shape = synth.TINY
    w = synth.make_weights(shape, 1)
    prompt = synth.workload_prompt("tiny")
    dec, model, kv = make_pair(shape, 1, 256, weights=w)
    table = B.NgramTable(2, 3, shape.vocab)
    got = B.anpd_generate(model, kv, table, prompt, 4, 64)
    ref = oanpd.anpd_generate(dec, prompt, 4, 64, 2, 3)
    # a free-running comparison is valid up to the first row whose top-2 gap is below tolerance
    dec2 = od.Decoder(shape, w, 256)
    dec2.prefill(prompt)
    n_safe = 0
    for t in ref["tokens"]:
        logits = dec2.forward([t])
        dec2.set_length(dec2.length + 1)
        if top2_gap(logits[0]) <= TOL["f32"]:
            break
        n_safe += 1
    assert n_safe >= 8
    assert got["tokens"][:n_safe + 1] == ref["tokens"][:n_safe + 1]
    if n_safe == 64:
        assert (got["n_steps"], got["proposed"], got["accepted"]) == (ref["n_steps"], ref["proposed"], ref["accepted"])


# ------------------------------------------------------------- invariants

@pytest.mark.parametrize("dt,path", PATHS)
def test_rows_are_causal_and_independent_of_window_size(dt, path):
    shape = _shape(dt)
    _, model, kv = make_pair(shape, 1, 256, gemm_path=path)
    toks = synth.markov_stream(shape.vocab, 120, 0.3, 4, 12, 9)
    B.prefill(model, kv, toks[:70])
    L = kv.length
    win = toks[70:87]                      # 17 rows
    _, _, _, full = gpu_logits(model, kv, win, B.VERIFY)
    kv.truncate(L)
    other = win[:5] + [(t + 3) % shape.vocab for t in win[5:]]
    _, _, _, changed = gpu_logits(model, kv, other, B.VERIFY)
    assert np.array_equal(full[:5], changed[:5])
    assert not np.array_equal(full[5:], changed[5:])
    # row r of the window == a one-row step at the same position, bit for bit
    kv.truncate(L)
    for r in range(17):
        _, _, _, one = gpu_logits(model, kv, [win[r]], B.APPEND)
        assert np.array_equal(one[0], full[r]), r
    # and windows of every class reproduce the same rows
    for M in (2, 8, 9, 16):
        kv.truncate(L)
        _, _, _, part = gpu_logits(model, kv, win[:M], B.VERIFY)
        assert np.array_equal(part, full[:M]), M


@pytest.mark.parametrize("dt,path", PATHS)
def test_same_step_twice_is_bit_identical(dt, path):
    shape = _shape(dt)
    _, model, kv = make_pair(shape, 1, 256, gemm_path=path)
    toks = synth.markov_stream(shape.vocab, 100, 0.3, 4, 12, 10)
    B.prefill(model, kv, toks[:80])
    _, _, _, a = gpu_logits(model, kv, toks[80:90], B.VERIFY)
    kv.truncate(80)
    _, _, _, b = gpu_logits(model, kv, toks[80:90], B.VERIFY)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("dt", ["f32", "mid"])
def test_a_callers_stream_gives_the_same_bits(dt):
    """Every entry point takes the caller's stream: prompt, steps of every window class, a draft tree and a
    batch on a stream of the caller's own (default priority) against the same calls on the default stream."""
    shape = _shape(dt)
    w = to_cuda(synth.make_weights(shape, 3))
    toks = synth.markov_stream(shape.vocab, 140, 0.3, 4, 12, 11)
    side = torch.cuda.Stream()
    runs = []
    for stream in (None, side):
        model = B.Model(shape, w, max_window=32, max_positions=256, stream=stream)
        kv, kv2 = B.KVCache(model, 256), B.KVCache(model, 256)
        out = [B.prefill(model, kv, toks[:90], stream=stream), B.prefill(model, kv2, toks[:41], stream=stream)]
        for M in (1, 6, 8, 13, 29):
            buf = torch.empty(M, shape.vocab, dtype=torch.float32, device="cuda")
            out.append(B.verify(model, kv, toks[90:90 + M], B.VERIFY, want_predicts=True, out_logits=buf, stream=stream))
            torch.cuda.synchronize()
            out.append(buf.cpu())
        out.append(B.verify_tree(model, kv, toks[100:107], [-1, 0, 1, 0, 3, 0, 5], stream=stream))
        if shape.dtype == "bf16":
            out.append(B.verify_batch(model, [kv, kv2], [toks[110:113], toks[120:122]], stream=stream))
        out.append((kv.length, kv2.length))
        k, v = kv.read(shape.n_layers - 1, 0, kv.length, stream=stream)
        torch.cuda.synchronize()
        out += [k.cpu(), v.cpu()]
        runs.append(out)
    for a, b in zip(*runs):
        assert torch.equal(a, b) if isinstance(a, torch.Tensor) else a == b


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_rollback_leaves_the_cache_of_plain_decoding(dt):
    shape = _shape(dt)
    w = synth.make_weights(shape, 1)
    prompt = synth.workload_prompt("tiny")[:50]
    _, model, kv = make_pair(shape, 1, 128, weights=w)
    _, model2, kv2 = make_pair(shape, 1, 128, weights=w)
    g = B.greedy_generate(model2, kv2, prompt, 12)           # plain decoding: cache holds prompt + g[:12]
    c = B.prefill(model, kv, prompt)
    # step 1: 2 right drafts then garbage -> rollback of 3 rows
    a, nxt = B.verify(model, kv, [c, g[1], g[2], 5, 6, 7], B.VERIFY)
    assert (a, nxt) == (2, g[3])
    # step 2: all wrong -> rollback of everything but row 0; straddles a page boundary (50+3 .. 50+9)
    a, nxt = B.verify(model, kv, [g[3], 1, 2, 3, 4, 5], B.VERIFY)
    assert (a, nxt) == (0, g[4])
    # step 3: all right
    a, nxt = B.verify(model, kv, [g[4]] + g[5:9], B.VERIFY)
    assert (a, nxt) == (4, g[9])
    n = kv.length
    assert n == 50 + 9
    for layer in range(shape.n_layers):
        k1, v1 = kv.read(layer, 0, n)
        k2, v2 = kv2.read(layer, 0, n)
        assert torch.equal(k1, k2) and torch.equal(v1, v2)


@pytest.mark.parametrize("dt,path", [("f32", B.GEMM_DOT), ("bf16", B.GEMM_MFMA)])
def test_page_order_does_not_change_results(dt, path):
    shape = _shape(dt)
    w = synth.make_weights(shape, 1)
    toks = synth.markov_stream(shape.vocab, 90, 0.3, 4, 12, 11)
    _, model, kv = make_pair(shape, 1, 128, gemm_path=path, weights=w)
    _, model2, kv2 = make_pair(shape, 1, 128, gemm_path=path, weights=w)
    n = kv2.num_pages
    perm = [(5 * i + 3) % n for i in range(n)]
    assert sorted(perm) == list(range(n))
    kv2.set_page_order(perm)
    B.prefill(model, kv, toks[:75]); B.prefill(model2, kv2, toks[:75])
    _, _, _, a = gpu_logits(model, kv, toks[75:88], B.VERIFY)
    _, _, _, b = gpu_logits(model2, kv2, toks[75:88], B.VERIFY)
    assert np.array_equal(a, b)
    # the data really sits in different physical pages
    assert not torch.equal(kv.pool[: 1 << 16], kv2.pool[: 1 << 16])


def test_kv_write_read_roundtrip_and_storage_rounding():
    shape = synth.TINY_BF16
    _, model, kv = make_pair(shape, 1, 64)
    k, v = synth.kv_fill(shape, 5, 1, 40)
    kv.write(1, 3, k.float().cuda(), v.float().cuda())
    k2, v2 = kv.read(1, 3, 40)
    assert torch.equal(k2.cpu(), k.float()) and torch.equal(v2.cpu(), v.float())
    # values that are not bf16-representable are rounded to nearest even
    x = torch.full((1, shape.d_model), 1.0 + 2.0 ** -8).cuda()
    kv.write(0, 0, x, x * 3)
    k3, _ = kv.read(0, 0, 1)
    assert float(k3[0, 0]) == 1.0


# ---------------------------------------------------------------- errors

def test_error_paths_leave_state_unchanged():
    shape = synth.TINY
    _, model, kv = make_pair(shape, 1, 40, max_window=8)
    B.prefill(model, kv, list(range(30)))
    for bad, code in [([1, shape.vocab], B.E_RANGE), ([-1], B.E_RANGE), (list(range(9)), B.E_CAPACITY),
                      ([], B.E_INVAL)]:
        with pytest.raises(B.AnpdError) as e:
            B.verify(model, kv, bad)
        assert e.value.code == code and kv.length == 30
    B.verify(model, kv, list(range(8)), B.APPEND)
    with pytest.raises(B.AnpdError) as e:            # 38 + 3 > 40
        B.verify(model, kv, [1, 2, 3])
    assert e.value.code == B.E_CAPACITY and kv.length == 38
    with pytest.raises(B.AnpdError):
        kv.truncate(41)
    with pytest.raises(B.AnpdError):
        B.verify(model, kv, [1], mode=7)
    with pytest.raises(B.AnpdError):
        B.KVCache(model, 41)                         # beyond max_positions
    # still healthy afterwards
    a, nxt = B.verify(model, kv, [1, 2])
    assert 0 <= a <= 1 and kv.length == 39 + a
