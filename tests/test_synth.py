"""Seeded input generators: reproducibility and the stated structure."""
import torch

from paper_2404_08698_amd import synth


def test_splitmix_tensor_matches_python_ints():
    xs = [0, 1, 2, 12345, (1 << 63) - 1, (1 << 63) + 5, (1 << 64) - 1]
    t = torch.tensor([x - (1 << 64) if x >= (1 << 63) else x for x in xs], dtype=torch.int64)
    got = synth.splitmix64_t(t).tolist()
    want = [synth.splitmix64(x) for x in xs]
    assert [g & ((1 << 64) - 1) for g in got] == want


def test_approx_normal_moments_and_determinism():
    a = synth.approx_normal(7, 3, 200000, 0.02)
    b = synth.approx_normal(7, 3, 200000, 0.02, chunk=4096)
    assert torch.equal(a, b)
    assert abs(a.mean().item()) < 3e-4
    assert abs(a.std().item() - 0.02) < 3e-4
    c = synth.approx_normal(7, 4, 1000, 0.02)
    assert not torch.equal(a[:1000], c)


def test_weight_shapes_and_param_count():
    w = synth.make_weights(synth.TINY, 1)
    assert w["embed"].shape == (1024, 256) and w["embed"].dtype == torch.float32
    assert len(w["wq"]) == 2 and w["w_down"][0].shape == (256, 688)
    assert synth.TINY.n_params_streamed == 1843200
    assert synth.LLAMA_7B.n_params_streamed == 6607077376
    assert synth.LLAMA_13B.n_params_streamed == 12851609600
    assert synth.LLAMA_7B.kv_bytes_per_token == 524288
    assert abs(w["attn_norm"][0].mean().item() - 1.0) < 0.01


def test_markov_stream_is_seeded_and_copy_heavy():
    a = synth.markov_stream(1024, 128, 0.30, 4, 12, 1)
    assert a == synth.markov_stream(1024, 128, 0.30, 4, 12, 1)
    assert a != synth.markov_stream(1024, 128, 0.30, 4, 12, 2)
    assert len(a) == 128 and all(0 <= t < 1024 for t in a)
    # repeated 4-grams exist (copied spans), none would at p_copy = 0 with V = 32000
    b = synth.markov_stream(32000, 512, 0.40, 4, 16, 2)
    grams = [tuple(b[i:i + 4]) for i in range(len(b) - 3)]
    assert len(set(grams)) < len(grams) - 20
    c = synth.markov_stream(32000, 512, 0.0, 4, 16, 2)
    grams_c = [tuple(c[i:i + 4]) for i in range(len(c) - 3)]
    assert len(set(grams_c)) >= len(grams_c) - 8
