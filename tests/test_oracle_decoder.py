"""Pins of the CPU oracle decoder against things other than itself:
library routines (torch fp64 matmul / softmax / silu), closed forms,
invariants, and an independent full-sequence (cache-free) expression of the
LLaMA layer written with torch tensor algebra only in this file.
"""
import dataclasses
import math

import numpy as np
import pytest
import torch

from oracle import decoder as od
from paper_2404_08698_amd import synth


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- pieces

def test_linear_is_x_times_w_transposed_library_matmul():
    r = _rng(0)
    X = r.standard_normal((5, 37))
    W = r.standard_normal((11, 37)).astype(np.float32)
    Y = od.linear(X, W)
    ref = torch.from_numpy(X) @ torch.from_numpy(W).double().T
    assert np.allclose(Y, ref.numpy(), rtol=0, atol=1e-12)
    # a transposed operand would not even have this shape; check asymmetry too
    assert Y.shape == (5, 11)


def test_linear_bf16_bits_are_widened_exactly():
    r = _rng(1)
    Wt = torch.from_numpy(r.standard_normal((7, 16)).astype(np.float32)).to(torch.bfloat16)
    X = r.standard_normal((3, 16))
    Y = od.linear(X, od.to_numpy_weight(Wt))
    ref = torch.from_numpy(X) @ Wt.double().T
    assert np.allclose(Y, ref.numpy(), rtol=0, atol=1e-12)


def test_round_bf16_matches_torch_and_known_values():
    assert od.round_bf16(1.0) == 1.0
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: ties go to even (1.0)
    assert od.round_bf16(1.0 + 2.0 ** -8) == 1.0
    assert od.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    xs = _rng(2).standard_normal(2000) * 3.0
    ref = torch.from_numpy(xs).float().to(torch.bfloat16).double().numpy()
    got = np.array([od.round_bf16(x) for x in xs])
    assert np.array_equal(got, ref)


def test_rmsnorm_closed_forms():
    d, eps = 64, 1e-5
    g = np.full(d, 2.0, dtype=np.float32)
    x = np.full(d, 3.0)
    out = od.rmsnorm(x, g, eps)
    assert np.allclose(out, 3.0 * 2.0 / math.sqrt(9.0 + eps), atol=1e-14)
    # scale invariance up to eps; gain is applied per element
    r = _rng(3)
    x = r.standard_normal(d)
    g = (1 + 0.1 * r.standard_normal(d)).astype(np.float32)
    a = od.rmsnorm(x, g, 0.0)
    b = od.rmsnorm(7.5 * x, g, 0.0)
    assert np.allclose(a, b, atol=1e-13)
    assert np.allclose(a, x / np.sqrt(np.mean(x * x)) * g.astype(np.float64), atol=1e-13)
    # unit gain: output has unit mean square
    one = np.ones(d, dtype=np.float32)
    assert abs(np.mean(od.rmsnorm(x, one, 0.0) ** 2) - 1.0) < 1e-13


def test_rope_properties():
    H, dh, base = 2, 8, 10000.0
    r = _rng(4)
    q = r.standard_normal(H * dh)
    k = r.standard_normal(H * dh)
    # position 0 is the identity
    assert np.array_equal(od.rope(q, H, dh, 0, base), q)
    # a rotation: per-head norms are kept
    q5 = od.rope(q, H, dh, 5, base)
    assert np.allclose(np.linalg.norm(q5.reshape(H, dh), axis=1), np.linalg.norm(q.reshape(H, dh), axis=1))
    # relative-position property: <rope(q,p+s), rope(k,p'+s)> = <rope(q,p), rope(k,p')> per head
    for s in (1, 17):
        a = (od.rope(q, H, dh, 9, base).reshape(H, dh) * od.rope(k, H, dh, 4, base).reshape(H, dh)).sum(1)
        b = (od.rope(q, H, dh, 9 + s, base).reshape(H, dh) * od.rope(k, H, dh, 4 + s, base).reshape(H, dh)).sum(1)
        assert np.allclose(a, b, atol=1e-12)
    # closed form: unit vector on lane i of head 0 goes to (cos, sin) on lanes (i, i+dh/2)
    for i in range(dh // 2):
        e = np.zeros(H * dh)
        e[i] = 1.0
        out = od.rope(e, H, dh, 3, base)
        ang = 3.0 * base ** (-2.0 * i / dh)
        want = np.zeros(H * dh)
        want[i], want[i + dh // 2] = math.cos(ang), math.sin(ang)
        assert np.allclose(out, want, atol=1e-15)
    # lane 0 turns by exactly pos radians (theta_0 = 1): after pos = 2 the pair (1, 0) -> (cos 2, sin 2)
    e = np.zeros(H * dh)
    e[dh] = 1.0  # head 1, lane 0
    out = od.rope(e, H, dh, 2, base)
    assert abs(out[dh] - math.cos(2.0)) < 1e-15 and abs(out[dh + dh // 2] - math.sin(2.0)) < 1e-15


def test_attention_special_cases_and_library_softmax():
    H, dh, n = 3, 4, 9
    d = H * dh
    r = _rng(5)
    q = r.standard_normal(d)
    V = r.standard_normal((n, d))
    # identical keys -> uniform weights -> mean of V
    K = np.tile(r.standard_normal(d), (n, 1))
    assert np.allclose(od.attention(q, K, V, H, dh), V.mean(0), atol=1e-13)
    # a single key -> its V exactly
    assert np.allclose(od.attention(q, K[:1], V[:1], H, dh), V[0], atol=1e-15)
    # general case against torch.softmax
    K = r.standard_normal((n, d))
    qt, Kt, Vt = (torch.from_numpy(a) for a in (q, K, V))
    s = torch.einsum("hd,nhd->hn", qt.view(H, dh), Kt.view(n, H, dh)) / math.sqrt(dh)
    ref = torch.einsum("hn,nhd->hd", torch.softmax(s, dim=-1), Vt.view(n, H, dh)).reshape(d)
    assert np.allclose(od.attention(q, K, V, H, dh), ref.numpy(), atol=1e-13)
    # large scores do not overflow (max-subtracted softmax)
    big = od.attention(q * 1e3, K, V, H, dh)
    assert np.all(np.isfinite(big))


def test_swiglu_against_library_silu():
    r = _rng(6)
    g = r.standard_normal(100) * 4
    u = r.standard_normal(100)
    ref = torch.nn.functional.silu(torch.from_numpy(g)) * torch.from_numpy(u)
    assert np.allclose(od.swiglu(g, u), ref.numpy(), atol=1e-14)
    assert od.swiglu(np.zeros(1), np.ones(1))[0] == 0.0
    # silu is not symmetric in its arguments: swapping gate and up changes the result
    assert not np.allclose(od.swiglu(g, u), od.swiglu(u, g))


def test_argmax_lowest_index_on_ties_in_float32():
    assert od.argmax(np.array([0.0, 3.0, 3.0, 1.0])) == 1
    assert od.argmax(np.array([5.0])) == 0
    # two doubles that round to the same float32 tie -> lowest index
    assert od.argmax(np.array([1.0, 1.0 + 1e-12, 0.5])) == 0
    assert od.argmax(np.array([-2.0, -1.0, -3.0])) == 1


# ------------------------------------------------- whole forward, independent

def _torch_full_sequence_logits(shape, w, tokens, kv_bf16):
    """All positions at once, no cache, explicit causal mask, rotation written
    with complex numbers: an independent statement of the same layer."""
    f64 = torch.float64
    T = len(tokens)
    H, dh, d = shape.n_heads, shape.head_dim, shape.d_model
    Hkv = shape.kv_heads
    W = lambda t: t.to(f64)

    def norm(x, g):
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + shape.rms_eps) * W(g)

    pos = torch.arange(T, dtype=f64)
    theta = shape.rope_base ** (-torch.arange(0, dh // 2, dtype=f64) * 2.0 / dh)
    rot = torch.polar(torch.ones(T, dh // 2, dtype=f64), pos[:, None] * theta[None, :])  # [T][dh/2]

    def rope(t):  # t: [T][heads][dh]
        z = torch.complex(t[..., : dh // 2], t[..., dh // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    def store(t):
        return t.float().to(torch.bfloat16).to(f64) if kv_bf16 else t

    x = W(w["embed"])[torch.tensor(tokens)]
    mask = torch.full((T, T), float("-inf"), dtype=f64).triu(1)
    for l in range(shape.n_layers):
        h = norm(x, w["attn_norm"][l])
        q = rope((h @ W(w["wq"][l]).T).view(T, H, dh))
        # key/value head j serves the query heads j * (H / Hkv) .. (j + 1) * (H / Hkv) - 1
        k = store(rope((h @ W(w["wk"][l]).T).view(T, Hkv, dh))).repeat_interleave(H // Hkv, dim=1)
        v = store((h @ W(w["wv"][l]).T).view(T, Hkv, dh)).repeat_interleave(H // Hkv, dim=1)
        s = torch.einsum("thd,shd->hts", q, k) / math.sqrt(dh) + mask
        o = torch.einsum("hts,shd->thd", torch.softmax(s, -1), v).reshape(T, d)
        x = x + o @ W(w["wo"][l]).T
        h = norm(x, w["ffn_norm"][l])
        a = torch.nn.functional.silu(h @ W(w["w_gate"][l]).T) * (h @ W(w["w_up"][l]).T)
        x = x + a @ W(w["w_down"][l]).T
    return (norm(x, w["final_norm"]) @ W(w["lm_head"]).T).numpy()


@pytest.mark.parametrize("which", ["f32", "bf16"])
def test_incremental_windowed_forward_equals_full_sequence(which, tiny_weights, tiny_bf16_weights):
    shape = synth.TINY if which == "f32" else synth.TINY_BF16
    w = tiny_weights if which == "f32" else tiny_bf16_weights
    tokens = synth.markov_stream(shape.vocab, 40, 0.3, 4, 12, 3)
    ref = _torch_full_sequence_logits(shape, w, tokens, kv_bf16=(which == "bf16"))
    dec = od.Decoder(shape, w, max_tokens=64)
    # ragged windows: 13 + 1 + 7 + 19 tokens
    got = []
    for n in (13, 1, 7, 19):
        lo = dec.length
        got.append(dec.forward(tokens[lo:lo + n]))
        dec.set_length(lo + n)
    got = np.concatenate(got, 0)
    # bf16 KV rounding can flip on last-bit differences between the two
    # formulations; fp64 elsewhere
    tol = 1e-9 if which == "f32" else 2e-3
    assert np.max(np.abs(got - ref)) < tol
    assert np.std(ref) > 0.05  # the comparison is not vacuous


def test_grouped_attention_is_attention_over_repeated_key_value_heads():
    rng = np.random.default_rng(5)
    H, Hkv, dh, n = 6, 2, 8, 11
    q = rng.standard_normal(H * dh)
    K = rng.standard_normal((n, Hkv * dh))
    V = rng.standard_normal((n, Hkv * dh))
    rep = lambda a: np.repeat(a.reshape(n, Hkv, dh), H // Hkv, axis=1).reshape(n, H * dh)
    assert np.array_equal(od.attention_grouped(q, K, V, H, Hkv, dh), od.attention(q, rep(K), rep(V), H, dh))
    assert np.array_equal(od.attention_grouped(q, rep(K), rep(V), H, H, dh), od.attention(q, rep(K), rep(V), H, dh))
    # one shared key/value head, one key: every query head returns that value row
    out = od.attention_grouped(q, K[:1, :dh], V[:1, :dh], H, 1, dh)
    assert np.allclose(out.reshape(H, dh), V[0, :dh])


@pytest.mark.parametrize("shape", [synth.TINY_MQA, synth.TINY_MQA_BF16, dataclasses.replace(synth.TINY, n_kv_heads=2)])
def test_grouped_heads_forward(shape):
    """Grouped key/value heads: the windowed forward against the cache-free full-sequence statement, and
    against the same model written with one key/value head per query head (weights repeated per group)."""
    w = synth.make_weights(shape, 11)
    tokens = synth.markov_stream(shape.vocab, 30, 0.3, 4, 12, 4)
    ref = _torch_full_sequence_logits(shape, w, tokens, kv_bf16=(shape.dtype == "bf16"))
    dec = od.Decoder(shape, w, max_tokens=40)
    got = []
    for n in (9, 1, 20):
        lo = dec.length
        got.append(dec.forward(tokens[lo:lo + n]))
        dec.set_length(lo + n)
    got = np.concatenate(got, 0)
    assert np.max(np.abs(got - ref)) < (1e-9 if shape.dtype == "f32" else 2e-3)
    assert np.std(ref) > 0.05
    k0, _ = dec.kv_read(0, 0, 30)
    assert k0.shape == (30, shape.kv_dim)
    # the equivalent model without sharing
    g, dh = shape.n_heads // shape.kv_heads, shape.head_dim
    full = dataclasses.replace(shape, n_kv_heads=0)
    rep = lambda t: t.view(shape.kv_heads, dh, -1).repeat_interleave(g, dim=0).reshape(shape.d_model, -1).contiguous()
    w2 = dict(w)
    w2["wk"] = [rep(t) for t in w["wk"]]
    w2["wv"] = [rep(t) for t in w["wv"]]
    dec2 = od.Decoder(full, w2, max_tokens=40)
    assert np.array_equal(dec2.forward(tokens), od.Decoder(shape, w, max_tokens=40).forward(tokens))


def test_rollback_then_recompute_equals_fresh_cache(tiny_weights):
    shape = synth.TINY
    toks = synth.markov_stream(shape.vocab, 24, 0.3, 4, 12, 5)
    a = od.Decoder(shape, tiny_weights, 64)
    a.forward(toks[:10]); a.set_length(10)
    a.forward([5, 6, 7, 8])          # a window that is then rejected after its first row
    a.set_length(11)                 # keep row 0 only
    la = a.forward(toks[11:16])
    b = od.Decoder(shape, tiny_weights, 64)
    b.forward(toks[:10] + [5]); b.set_length(11)
    lb = b.forward(toks[11:16])
    assert np.array_equal(la, lb)
    ka, va = a.kv_read(1, 0, 11)
    kb, vb = b.kv_read(1, 0, 11)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)


def test_window_rows_are_causal(tiny_weights):
    shape = synth.TINY
    dec = od.Decoder(shape, tiny_weights, 64)
    dec.forward([1, 2, 3, 4, 5, 6]); dec.set_length(6)
    w1 = dec.forward([10, 11, 12, 13])
    w2 = dec.forward([10, 11, 99, 98])
    assert np.array_equal(w1[:2], w2[:2])
    assert not np.allclose(w1[2:], w2[2:])
    # row r of a window equals the single-row step at the same position
    dec.forward([10]); dec.set_length(7)
    single = dec.forward([11])
    assert np.allclose(single[0], w1[1], atol=1e-12)


def test_forward_rejects_bad_input(tiny_weights):
    dec = od.Decoder(synth.TINY, tiny_weights, 8)
    with pytest.raises(ValueError):
        dec.forward([1024])
    with pytest.raises(ValueError):
        dec.forward(list(range(9)))
