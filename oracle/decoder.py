"""ctypes front end of the C oracle decoder (oracle/decoder.c).

TEST INFRASTRUCTURE ONLY: see the package docstring.  The functions mirror
the C file one to one; each cites the passage it follows there.
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Sequence

import numpy as np

from . import build as _build

ORC_F32, ORC_BF16 = 0, 1

_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class _Cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_double), ("rope_base", C.c_double),
                ("w_dtype", C.c_int32), ("kv_bf16", C.c_int32), ("n_kv_heads", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in _PER_LAYER]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        dp = C.POINTER(C.c_double)
        L.orc_round_bf16.restype = C.c_double
        L.orc_round_bf16.argtypes = [C.c_double]
        L.orc_rmsnorm.restype = None
        L.orc_rmsnorm.argtypes = [dp, C.c_void_p, C.c_int, C.c_int, C.c_double, dp]
        L.orc_linear.restype = None
        L.orc_linear.argtypes = [dp, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int, dp]
        L.orc_rope.restype = None
        L.orc_rope.argtypes = [dp, C.c_int, C.c_int, C.c_int, C.c_double]
        L.orc_attention.restype = None
        L.orc_attention.argtypes = [dp, dp, dp, C.c_int, C.c_int, C.c_int, dp]
        L.orc_attention_grouped.restype = None
        L.orc_attention_grouped.argtypes = [dp, dp, dp, C.c_int, C.c_int, C.c_int, C.c_int, dp]
        L.orc_swiglu.restype = None
        L.orc_swiglu.argtypes = [dp, dp, C.c_int, dp]
        L.orc_argmax.restype = C.c_int32
        L.orc_argmax.argtypes = [dp, C.c_int]
        L.orc_model_create.restype = C.c_void_p
        L.orc_model_create.argtypes = [C.POINTER(_Cfg), C.POINTER(_Weights)]
        L.orc_model_destroy.restype = None
        L.orc_model_destroy.argtypes = [C.c_void_p]
        L.orc_kv_create.restype = C.c_void_p
        L.orc_kv_create.argtypes = [C.c_void_p, C.c_int32]
        L.orc_kv_destroy.restype = None
        L.orc_kv_destroy.argtypes = [C.c_void_p]
        L.orc_kv_len.restype = C.c_int32
        L.orc_kv_len.argtypes = [C.c_void_p]
        L.orc_kv_set_len.restype = C.c_int32
        L.orc_kv_set_len.argtypes = [C.c_void_p, C.c_int32]
        fp = C.POINTER(C.c_float)
        L.orc_kv_load.restype = C.c_int32
        L.orc_kv_load.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, fp, fp]
        L.orc_kv_read.restype = C.c_int32
        L.orc_kv_read.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, dp, dp]
        L.orc_forward.restype = C.c_int32
        L.orc_forward.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_int32, dp]
        L.orc_num_threads.restype = C.c_int32
        L.orc_num_threads.argtypes = []
        _lib = L
    return _lib


def _dp(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _wptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"] and a.dtype in (np.float32, np.uint16)
    return a.ctypes.data, (ORC_BF16 if a.dtype == np.uint16 else ORC_F32)


def to_numpy_weight(t) -> np.ndarray:
    """torch float32 / bfloat16 CPU tensor -> float32 / uint16 (bf16 bits) array."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.to(torch.float32).numpy()


def num_threads() -> int:
    return int(lib().orc_num_threads())


def round_bf16(x: float) -> float:
    return float(lib().orc_round_bf16(float(x)))


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty_like(x)
    p, dt = _wptr(np.ascontiguousarray(g))
    lib().orc_rmsnorm(_dp(x), p, dt, x.shape[-1], eps, _dp(out))
    return out


def linear(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X @ W.T with W [N][K] stored as float32 or bf16 bits (uint16)."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    M, K = X.shape
    N = W.shape[0]
    assert W.shape[1] == K
    Y = np.empty((M, N), dtype=np.float64)
    p, dt = _wptr(W)
    lib().orc_linear(_dp(X), M, K, p, dt, N, _dp(Y))
    return Y


def rope(v: np.ndarray, n_heads: int, head_dim: int, pos: int, base: float) -> np.ndarray:
    out = np.ascontiguousarray(v, dtype=np.float64).copy()
    lib().orc_rope(_dp(out), n_heads, head_dim, pos, base)
    return out


def attention(q: np.ndarray, Kc: np.ndarray, Vc: np.ndarray, n_heads: int, head_dim: int) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.float64)
    Kc = np.ascontiguousarray(Kc, dtype=np.float64)
    Vc = np.ascontiguousarray(Vc, dtype=np.float64)
    out = np.empty_like(q)
    lib().orc_attention(_dp(q), _dp(Kc), _dp(Vc), Kc.shape[0], n_heads, head_dim, _dp(out))
    return out


def attention_grouped(q: np.ndarray, Kc: np.ndarray, Vc: np.ndarray, n_heads: int, n_kv_heads: int,
                      head_dim: int) -> np.ndarray:
    """Kc, Vc: [n_keys][n_kv_heads * head_dim]; query head h reads key/value head h // (n_heads // n_kv_heads)."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    Kc = np.ascontiguousarray(Kc, dtype=np.float64)
    Vc = np.ascontiguousarray(Vc, dtype=np.float64)
    out = np.empty_like(q)
    lib().orc_attention_grouped(_dp(q), _dp(Kc), _dp(Vc), Kc.shape[0], n_heads, n_kv_heads, head_dim, _dp(out))
    return out


def swiglu(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    gate = np.ascontiguousarray(gate, dtype=np.float64)
    up = np.ascontiguousarray(up, dtype=np.float64)
    out = np.empty_like(gate)
    lib().orc_swiglu(_dp(gate), _dp(up), gate.size, _dp(out))
    return out


def argmax(logits: np.ndarray) -> int:
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    return int(lib().orc_argmax(_dp(logits), logits.size))


class Decoder:
    """The oracle LLM: weights + one sequence's KV cache.

    ``shape`` needs the attributes n_layers, d_model, n_heads, head_dim, d_ffn,
    vocab, rms_eps, rope_base, dtype ("f32" | "bf16").  ``weights`` maps the
    tensor names to float32 / uint16 numpy arrays (or torch CPU tensors);
    per-layer names map to lists.
    """

    def __init__(self, shape, weights: Dict[str, object], max_tokens: int):
        self.shape = shape
        self.vocab = shape.vocab
        self._keep: List[np.ndarray] = []

        def conv(t):
            a = t if isinstance(t, np.ndarray) else to_numpy_weight(t)
            a = np.ascontiguousarray(a)
            self._keep.append(a)
            return a

        want = ORC_BF16 if shape.dtype == "bf16" else ORC_F32
        ws = _Weights()
        for name in ("embed", "final_norm", "lm_head"):
            p, dt = _wptr(conv(weights[name]))
            assert dt == want, name
            setattr(ws, name, p)
        self._arrays = []
        for name in _PER_LAYER:
            arr = (C.c_void_p * shape.n_layers)()
            for l in range(shape.n_layers):
                p, dt = _wptr(conv(weights[name][l]))
                assert dt == want, name
                arr[l] = p
            self._arrays.append(arr)
            setattr(ws, name, C.cast(arr, C.POINTER(C.c_void_p)))
        cfg = _Cfg(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn,
                   shape.vocab, shape.rms_eps, shape.rope_base, want, 1 if want == ORC_BF16 else 0,
                   int(getattr(shape, "n_kv_heads", 0) or 0))
        self.kv_dim = (cfg.n_kv_heads or shape.n_heads) * shape.head_dim
        self._ws, self._cfg = ws, cfg
        self._model = lib().orc_model_create(C.byref(cfg), C.byref(ws))
        self._kv = lib().orc_kv_create(self._model, max_tokens)
        if not self._kv:
            raise MemoryError("oracle KV cache")
        self.max_tokens = max_tokens

    def close(self):
        if self._kv:
            lib().orc_kv_destroy(self._kv)
            self._kv = None
        if self._model:
            lib().orc_model_destroy(self._model)
            self._model = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def length(self) -> int:
        return int(lib().orc_kv_len(self._kv))

    def set_length(self, n: int) -> None:
        if lib().orc_kv_set_len(self._kv, n) != 0:
            raise ValueError("bad KV length %d" % n)

    def kv_load(self, layer: int, pos0: int, k: np.ndarray, v: np.ndarray) -> None:
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        fp = C.POINTER(C.c_float)
        if lib().orc_kv_load(self._kv, layer, pos0, k.shape[0], k.ctypes.data_as(fp),
                             v.ctypes.data_as(fp)) != 0:
            raise ValueError("kv_load out of range")

    def kv_read(self, layer: int, pos0: int, n: int):
        d = self.kv_dim
        k = np.empty((n, d), dtype=np.float64)
        v = np.empty((n, d), dtype=np.float64)
        if lib().orc_kv_read(self._kv, layer, pos0, n, _dp(k), _dp(v)) != 0:
            raise ValueError("kv_read out of range")
        return k, v

    def forward(self, tokens: Sequence[int]) -> np.ndarray:
        """Logits [n][vocab] for a window at positions length..length+n-1.

        The cache length is left unchanged; call ``set_length`` to commit.
        """
        n = len(tokens)
        toks = (C.c_int32 * n)(*[int(t) for t in tokens])
        logits = np.empty((n, self.vocab), dtype=np.float64)
        if lib().orc_forward(self._model, self._kv, toks, n, _dp(logits)) != 0:
            raise ValueError("oracle forward rejected its input")
        return logits

    # -- the three calls the ANPD loop needs (oracle/anpd.py) --
    def prefill(self, prompt: Sequence[int], chunk: int = 64) -> int:
        """LLM(prompt): fills the cache, returns the greedy token after the prompt."""
        nxt = -1
        for lo in range(0, len(prompt), chunk):
            part = prompt[lo:lo + chunk]
            logits = self.forward(part)
            self.set_length(self.length + len(part))
            nxt = argmax(logits[-1])
        return nxt

    def predict(self, window: Sequence[int]) -> List[int]:
        """LLM(drafts): one greedy prediction per window row; nothing committed."""
        logits = self.forward(window)
        self.last_logits = logits
        return [argmax(logits[r]) for r in range(len(window))]

    def commit(self, n_rows: int) -> None:
        """Keep the first n_rows window rows in the cache, drop the rest."""
        self.set_length(self.length + n_rows)
