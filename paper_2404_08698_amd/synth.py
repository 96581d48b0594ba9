"""Seeded synthetic inputs: weights, token streams and KV-cache contents.

This module holds no arithmetic of the decoding method.  It only produces
reproducible inputs that both the HIP path and the CPU oracle consume, so the
two sides see the same bits.  Everything is derived from a 64-bit counter hash
(the published splitmix64 finaliser) evaluated with integer operations only,
so the values are identical on the CPU and on the GPU.

The paper evaluates on summarisation and code prompts whose relevant structure
is a long prompt followed by output that re-uses spans of it (Section 4.4,
case study).  ``markov_stream`` stands in for those: an order-2 Markov chain
over the vocabulary with a stated probability of copying an earlier span.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List

import torch

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def splitmix64(x: int) -> int:
    """One splitmix64 output for counter ``x`` (Python integers)."""
    z = (x + _GAMMA) & _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _s64(c: int) -> int:
    """Two's-complement view of an unsigned 64-bit constant."""
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def splitmix64_t(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 on an int64 tensor (wrap-around arithmetic, any device)."""
    z = x + _s64(_GAMMA)
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


# Sum of eight independent uniform 16-bit integers, centred: an Irwin-Hall
# variate with variance 8 * (2**32 - 1) / 12.  It needs no transcendental
# function, so host and device produce the same float32 bit pattern.
_IH_STD = (8.0 * ((1 << 32) - 1) / 12.0) ** 0.5


def approx_normal(seed: int, stream: int, numel: int, std: float,
                  device: torch.device | str = "cpu", mean: float = 0.0,
                  chunk: int = 1 << 25) -> torch.Tensor:
    """``numel`` float32 values, approximately N(mean, std**2).

    Element ``i`` depends only on (seed, stream, i).
    """
    key = splitmix64((seed * 0x100000001B3 + stream) & _M64)
    out = torch.empty(numel, dtype=torch.float32, device=device)
    scale = torch.tensor(std / _IH_STD, dtype=torch.float32, device=device)
    for lo in range(0, numel, chunk):
        hi = min(numel, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device)
        acc = torch.zeros(hi - lo, dtype=torch.int64, device=device)
        for half in range(2):
            h = splitmix64_t(idx * 2 + half + _s64(key))
            for f in range(4):
                acc += _lsr(h, 16 * f) & 0xFFFF
        acc -= 4 * 0xFFFF
        vals = acc.to(torch.float32) * scale
        if mean != 0.0:
            vals = vals + torch.tensor(mean, dtype=torch.float32, device=device)
        out[lo:hi] = vals
    return out


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """LLaMA-shaped decoder dimensions (names follow the usual notation)."""
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # storage type of weights and KV: "f32" | "bf16"
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    n_kv_heads: int = 0          # key/value heads shared by groups of query heads; 0 = one per query head

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads or self.n_heads

    @property
    def kv_dim(self) -> int:
        """Width of a cached K (or V) row."""
        return self.kv_heads * self.head_dim

    @property
    def n_params_streamed(self) -> int:
        """Weights read once per forward (embedding rows excluded)."""
        d, f = self.d_model, self.d_ffn
        return self.n_layers * (2 * d * d + 2 * d * self.kv_dim + 3 * d * f) + self.vocab * d

    @property
    def kv_bytes_per_token(self) -> int:
        el = 2 if self.dtype == "bf16" else 4
        return self.n_layers * 2 * self.kv_dim * el


TINY = ModelShape(2, 256, 4, 64, 688, 1024, "f32")
TINY_BF16 = dataclasses.replace(TINY, dtype="bf16")
# head_dim 128 like the LLaMA shapes, small enough for the oracle: used by parity tests
MID_BF16 = ModelShape(3, 512, 4, 128, 1408, 2048, "bf16")
LLAMA_7B = ModelShape(32, 4096, 32, 128, 11008, 32000, "bf16")
LLAMA_13B = ModelShape(40, 5120, 40, 128, 13824, 32000, "bf16")
# Grouped key/value heads and a vocabulary twice LLaMA's: the dimensions of the ChatGLM3-6B model
# the paper also evaluates (28 layers, 32 query heads over 2 key/value heads, FFN 13696).
GLM_6B = ModelShape(28, 4096, 32, 128, 13696, 65024, "bf16", n_kv_heads=2)
MID_GQA = ModelShape(3, 512, 4, 128, 1408, 2048, "bf16", n_kv_heads=2)
# d_model 2048 with FFN 6144 and vocabulary 8192: in the one-kernel step on 256 compute units its phases have
# one, two and three work items per block (a test shape for the ends of the weight pipeline)
RING_BF16 = ModelShape(2, 2048, 16, 128, 6144, 8192, "bf16")
TINY_MQA = ModelShape(2, 256, 4, 64, 688, 1024, "f32", n_kv_heads=1)
TINY_MQA_BF16 = dataclasses.replace(TINY_MQA, dtype="bf16")

_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def weight_shapes(s: ModelShape) -> Dict[str, tuple]:
    d, f, v, kvd = s.d_model, s.d_ffn, s.vocab, s.kv_dim
    return {
        "embed": (v, d), "final_norm": (d,), "lm_head": (v, d),
        "attn_norm": (d,), "wq": (d, d), "wk": (kvd, d), "wv": (kvd, d), "wo": (d, d),
        "ffn_norm": (d,), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }


def make_weights(s: ModelShape, seed: int, device="cpu", std: float = 0.02) -> Dict[str, object]:
    """All tensors of the decoder, [out][in] row-major, in the storage dtype.

    Matrices and the embedding are ~N(0, std); norm gains are 1 + ~N(0, std)
    so that a mis-indexed gain is visible to a parity test.  Per-layer
    entries are lists of length ``n_layers``.
    """
    tdtype = torch.bfloat16 if s.dtype == "bf16" else torch.float32
    shapes = weight_shapes(s)

    def gen(name: str, stream: int) -> torch.Tensor:
        shp = shapes[name]
        n = 1
        for x in shp:
            n *= x
        mean = 1.0 if name.endswith("norm") else 0.0
        return approx_normal(seed, stream, n, std, device, mean).to(tdtype).reshape(shp).contiguous()

    w: Dict[str, object] = {
        "embed": gen("embed", 1), "final_norm": gen("final_norm", 2), "lm_head": gen("lm_head", 3),
    }
    for j, name in enumerate(_PER_LAYER):
        w[name] = [gen(name, 1000 + 16 * layer + j) for layer in range(s.n_layers)]
    return w


def markov_stream(vocab: int, length: int, p_copy: float, span_lo: int, span_hi: int,
                  seed: int) -> List[int]:
    """Copy-heavy order-2 Markov token stream.

    State (a, b) has four candidate successors hash(a, b, i) mod vocab with
    probabilities 0.55/0.25/0.12/0.08.  At each position t >= span_hi, with
    probability ``p_copy`` a span of U[span_lo, span_hi] earlier tokens is
    copied instead.
    """
    ctr = [splitmix64(seed ^ 0xA5A5A5A55A5A5A5A)]

    def rnd() -> int:
        ctr[0] = (ctr[0] + 1) & _M64
        return splitmix64(ctr[0])

    def unit() -> float:
        return (rnd() >> 11) / float(1 << 53)

    out: List[int] = [rnd() % vocab, rnd() % vocab]
    cum = (0.55, 0.80, 0.92, 1.0)
    while len(out) < length:
        t = len(out)
        if t >= span_hi and unit() < p_copy:
            ell = span_lo + rnd() % (span_hi - span_lo + 1)
            start = rnd() % (t - ell + 1)
            out.extend(out[start:start + ell])
        else:
            a, b = out[-2], out[-1]
            u = unit()
            i = next(j for j, c in enumerate(cum) if u < c)
            out.append(splitmix64((a * 0x1F123BB5 + b) * 4 + i + (seed << 40) & _M64) % vocab)
    return out[:length]


def kv_fill(s: ModelShape, seed: int, layer: int, n_tokens: int, device="cpu"):
    """Seeded K and V contents for ``n_tokens`` cached positions of one layer.

    Returns two [n_tokens][kv_dim] tensors in the storage dtype, ~N(0, 1).
    """
    tdtype = torch.bfloat16 if s.dtype == "bf16" else torch.float32
    n = n_tokens * s.kv_dim
    k = approx_normal(seed, 50000 + 2 * layer, n, 1.0, device).to(tdtype).reshape(n_tokens, s.kv_dim)
    v = approx_normal(seed, 50001 + 2 * layer, n, 1.0, device).to(tdtype).reshape(n_tokens, s.kv_dim)
    return k, v


def random_tokens(vocab: int, n: int, seed: int) -> List[int]:
    return [splitmix64((seed << 20) + i) % vocab for i in range(n)]


# The workloads named by the benchmark configuration (prompt recipe per config).
WORKLOADS = {
    "tiny": dict(shape=TINY, prompt=128, p_copy=0.30, span=(4, 12), gen=64, n_min=2, n_max=3, k=4, seed=1),
    "llama7b": dict(shape=LLAMA_7B, prompt=512, p_copy=0.40, span=(4, 16), gen=256, n_min=2, n_max=5, k=5, seed=2),
    "llama13b": dict(shape=LLAMA_13B, prompt=1024, p_copy=0.50, span=(8, 32), gen=256, n_min=2, n_max=7, k=8, seed=4),
    "long7b": dict(shape=LLAMA_7B, prompt=3584, p_copy=0.20, span=(4, 16), gen=512, n_min=2, n_max=6, k=16, seed=5),
    "glm6b": dict(shape=GLM_6B, prompt=512, p_copy=0.40, span=(4, 16), gen=256, n_min=2, n_max=5, k=5, seed=6),
}


def workload_prompt(name: str) -> List[int]:
    w = WORKLOADS[name]
    return markov_stream(w["shape"].vocab, w["prompt"], w["p_copy"], w["span"][0], w["span"][1], w["seed"])
