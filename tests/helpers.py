"""Shared plumbing of the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

from oracle import decoder as od
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth

TOL = {"f32": 1e-4, "bf16": 2e-2, "mid": 2e-2}   # max-abs on logits, stated by the build target


def to_cuda(weights):
    out = {}
    for k, v in weights.items():
        out[k] = [t.cuda() for t in v] if isinstance(v, list) else v.cuda()
    return out


def make_pair(shape, seed, max_tokens, max_window=32, gemm_path=B.GEMM_AUTO, weights=None):
    """(oracle decoder, GPU model, GPU cache) on the same weight bits."""
    w = weights if weights is not None else synth.make_weights(shape, seed)
    dec = od.Decoder(shape, w, max_tokens)
    model = B.Model(shape, to_cuda(w), max_window=max_window, max_positions=max_tokens, gemm_path=gemm_path)
    kv = B.KVCache(model, max_tokens)
    return dec, model, kv


def gpu_logits(model, kv, window, mode=B.VERIFY):
    buf = torch.empty(len(window), model.vocab, dtype=torch.float32, device="cuda")
    a, nxt, preds = B.verify(model, kv, window, mode, want_predicts=True, out_logits=buf)
    return a, nxt, preds, buf.cpu().numpy().astype(np.float64)


def top2_gap(row):
    part = np.partition(row, -2)
    return part[-1] - part[-2]


def seed_kv_both(shape, dec, kv, n_tokens, seed):
    """Fill both caches with the same seeded contents (kernel-sweep style)."""
    for layer in range(shape.n_layers):
        k, v = synth.kv_fill(shape, seed, layer, n_tokens)
        dec.kv_load(layer, 0, k.float().numpy(), v.float().numpy())
        kv.write(layer, 0, k.float().cuda().contiguous(), v.float().cuda().contiguous())
    dec.set_length(n_tokens)
    kv.truncate(n_tokens)
