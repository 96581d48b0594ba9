"""Thin ctypes binding of libanpd.so: argument marshalling only.

Every step of the verification path runs inside the library's HIP kernels.
PyTorch appears here only as the allocator of device memory and the owner of
the stream.  There is no CPU fallback: if the library is missing, importing
``lib()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libanpd.so")

OK, E_INVAL, E_RANGE, E_CAPACITY, E_NOMEM, E_HIP, E_UNIMPLEMENTED = 0, -1, -2, -3, -4, -5, -6
F32, BF16 = 0, 1
VERIFY, APPEND = 0, 1
GEMM_AUTO, GEMM_DOT, GEMM_MFMA, GEMM_MFMA_STREAM, GEMM_MFMA_LAUNCHES = 0, 1, 2, 3, 4
MAX_WINDOW = 32

_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")

# every symbol include/anpd.h declares
EXPORTS = (
    "anpd_last_error",
    "anpd_ngram_create", "anpd_ngram_destroy", "anpd_ngram_reset", "anpd_ngram_update",
    "anpd_ngram_length", "anpd_ngram_query", "anpd_ngram_propose", "anpd_ngram_propose_tree",
    "anpd_model_workspace_bytes", "anpd_model_create", "anpd_model_destroy",
    "anpd_kv_pool_bytes", "anpd_kv_create", "anpd_kv_destroy", "anpd_kv_length", "anpd_kv_truncate",
    "anpd_kv_set_page_order", "anpd_kv_num_pages", "anpd_kv_write", "anpd_kv_read",
    "anpd_verify", "anpd_verify_tree", "anpd_verify_batch", "anpd_prefill_workspace_bytes", "anpd_prefill", "anpd_linear_workspace_bytes", "anpd_linear",
    "anpd_model_profile", "anpd_model_profile_read", "anpd_packed_bytes", "anpd_pack_weights",
    "anpd_model_trace", "anpd_model_set_barrier_spin_limit", "anpd_linear_static",
)
PROF_CATEGORIES = ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head", "attn", "other", "step")


class AnpdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("anpd error %d: %s" % (code, msg))
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32),
                ("page_tokens", C.c_int32), ("max_window", C.c_int32), ("max_positions", C.c_int32),
                ("gemm_path", C.c_int32), ("n_kv_heads", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in _PER_LAYER]


_lib = None


def lib():
    """Load libanpd.so (built by ``build.build()``); fail loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libanpd.so is not built: run `python -m paper_2404_08698_amd.build` "
                          "(there is no fallback path)")
    # PyTorch ships its own copy of the HIP runtime.  Load it first, so that this library binds to the
    # runtime the device memory comes from: with the order reversed the process ends up with two runtimes,
    # and the second one finds no device.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(LIB_PATH)
    i32p, vp = C.POINTER(C.c_int32), C.c_void_p
    L.anpd_last_error.restype = C.c_char_p
    L.anpd_last_error.argtypes = []
    L.anpd_ngram_create.restype = C.c_int32
    L.anpd_ngram_create.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(vp)]
    L.anpd_ngram_destroy.restype = None
    L.anpd_ngram_destroy.argtypes = [vp]
    L.anpd_ngram_reset.restype = C.c_int32
    L.anpd_ngram_reset.argtypes = [vp]
    L.anpd_ngram_update.restype = C.c_int32
    L.anpd_ngram_update.argtypes = [vp, i32p, C.c_int64]
    L.anpd_ngram_length.restype = C.c_int64
    L.anpd_ngram_length.argtypes = [vp]
    L.anpd_ngram_query.restype = C.c_int32
    L.anpd_ngram_query.argtypes = [vp, i32p, C.c_int32, i32p, i32p]
    L.anpd_ngram_propose.restype = C.c_int32
    L.anpd_ngram_propose.argtypes = [vp, C.c_int32, i32p, i32p]
    L.anpd_ngram_propose_tree.restype = C.c_int32
    L.anpd_ngram_propose_tree.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, i32p, i32p, i32p]
    L.anpd_model_workspace_bytes.restype = C.c_size_t
    L.anpd_model_workspace_bytes.argtypes = [C.POINTER(ModelCfg)]
    L.anpd_model_create.restype = C.c_int32
    L.anpd_model_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(Weights), vp, C.c_size_t, vp, C.POINTER(vp)]
    L.anpd_model_destroy.restype = None
    L.anpd_model_destroy.argtypes = [vp]
    L.anpd_kv_pool_bytes.restype = C.c_size_t
    L.anpd_kv_pool_bytes.argtypes = [vp, C.c_int32]
    L.anpd_kv_create.restype = C.c_int32
    L.anpd_kv_create.argtypes = [vp, vp, C.c_size_t, C.c_int32, C.POINTER(vp)]
    L.anpd_kv_destroy.restype = None
    L.anpd_kv_destroy.argtypes = [vp]
    L.anpd_kv_length.restype = C.c_int32
    L.anpd_kv_length.argtypes = [vp]
    L.anpd_kv_truncate.restype = C.c_int32
    L.anpd_kv_truncate.argtypes = [vp, C.c_int32, vp]
    L.anpd_kv_set_page_order.restype = C.c_int32
    L.anpd_kv_set_page_order.argtypes = [vp, i32p, C.c_int32]
    L.anpd_kv_num_pages.restype = C.c_int32
    L.anpd_kv_num_pages.argtypes = [vp]
    L.anpd_kv_write.restype = C.c_int32
    L.anpd_kv_write.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, vp, vp, vp]
    L.anpd_kv_read.restype = C.c_int32
    L.anpd_kv_read.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, vp, vp, vp]
    L.anpd_verify.restype = C.c_int32
    L.anpd_verify.argtypes = [vp, vp, i32p, C.c_int32, C.c_int32, i32p, i32p, i32p, vp, vp]
    L.anpd_verify_tree.restype = C.c_int32
    L.anpd_verify_tree.argtypes = [vp, vp, i32p, i32p, C.c_int32, i32p, i32p, i32p, i32p, vp, vp]
    L.anpd_verify_batch.restype = C.c_int32
    L.anpd_verify_batch.argtypes = [vp, C.POINTER(vp), C.c_int32, C.POINTER(i32p), i32p, C.c_int32, i32p, i32p, vp, vp]
    L.anpd_prefill_workspace_bytes.restype = C.c_size_t
    L.anpd_prefill_workspace_bytes.argtypes = [vp, C.c_int32]
    L.anpd_prefill.restype = C.c_int32
    L.anpd_prefill.argtypes = [vp, vp, i32p, C.c_int32, i32p, vp, vp, C.c_size_t, vp]
    L.anpd_linear_workspace_bytes.restype = C.c_size_t
    L.anpd_linear_workspace_bytes.argtypes = [C.c_int32, C.c_int32]
    L.anpd_linear.restype = C.c_int32
    L.anpd_linear.argtypes = [vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, C.c_size_t, vp]
    L.anpd_linear_static.restype = C.c_int32
    L.anpd_linear_static.argtypes = [vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, vp]
    L.anpd_packed_bytes.restype = C.c_size_t
    L.anpd_packed_bytes.argtypes = [C.c_int32, C.c_int32]
    L.anpd_pack_weights.restype = C.c_int32
    L.anpd_pack_weights.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_size_t, vp]
    L.anpd_model_trace.restype = C.c_int32
    L.anpd_model_trace.argtypes = [vp, vp, C.c_size_t]
    L.anpd_model_set_barrier_spin_limit.restype = C.c_int32
    L.anpd_model_set_barrier_spin_limit.argtypes = [vp, C.c_int32]
    L.anpd_model_profile.restype = C.c_int32
    L.anpd_model_profile.argtypes = [vp, C.c_int32]
    L.anpd_model_profile_read.restype = C.c_int32
    L.anpd_model_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    _lib = L
    return L


def _alive() -> bool:
    """False once the interpreter is shutting down (module globals are being cleared)."""
    import sys
    return _lib is not None and lib is not None and not sys.is_finalizing()


def _check(rc: int) -> int:
    if rc < 0:
        raise AnpdError(rc, lib().anpd_last_error().decode("utf-8", "replace"))
    return rc


def _ints(seq: Sequence[int]):
    return (C.c_int32 * max(1, len(seq)))(*[int(t) for t in seq])


# --------------------------------------------------------------- host table

class NgramTable:
    """anpd_ngram_*: the adaptive multi-level N-gram drafter (host)."""

    def __init__(self, n_min: int, n_max: int, vocab: int):
        h = C.c_void_p()
        _check(lib().anpd_ngram_create(n_min, n_max, vocab, C.byref(h)))
        self._h = h

    def close(self):
        try:
            if getattr(self, "_h", None) and _alive():
                lib().anpd_ngram_destroy(self._h)
        except TypeError:   # interpreter shutdown: this module's globals are already gone
            pass
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self) -> None:
        _check(lib().anpd_ngram_reset(self._h))

    def update(self, tokens: Sequence[int]) -> int:
        return _check(lib().anpd_ngram_update(self._h, _ints(tokens), len(tokens)))

    def __len__(self) -> int:
        return int(lib().anpd_ngram_length(self._h))

    def query(self, tail: Sequence[int]) -> Tuple[Optional[int], int]:
        tok, lvl = C.c_int32(-1), C.c_int32(0)
        hit = _check(lib().anpd_ngram_query(self._h, _ints(tail), len(tail), C.byref(tok), C.byref(lvl)))
        return (tok.value, lvl.value) if hit else (None, 0)

    def propose(self, max_k: int) -> Tuple[List[int], List[int]]:
        toks, lvls = (C.c_int32 * max(1, max_k))(), (C.c_int32 * max(1, max_k))()
        n = _check(lib().anpd_ngram_propose(self._h, max_k, toks, lvls))
        return list(toks[:n]), list(lvls[:n])


# ------------------------------------------------------------- device side

def _propose_tree(self, max_k: int, n_cand: int, max_drafts: int):
    """anpd_ngram_propose_tree: (tokens, parents, levels) of the drafts; draft i is window row i + 1."""
    n = max(1, max_drafts)
    toks, pars, lvls = (C.c_int32 * n)(), (C.c_int32 * n)(), (C.c_int32 * n)()
    k = _check(lib().anpd_ngram_propose_tree(self._h, max_k, n_cand, max_drafts, toks, pars, lvls))
    return list(toks[:k]), list(pars[:k]), list(lvls[:k])


NgramTable.propose_tree = _propose_tree


def _stream_ptr(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


class Model:
    """anpd_model_*: borrows torch CUDA weight tensors, owns a workspace tensor."""

    def __init__(self, shape, weights: Dict[str, object], max_window: int = 8, max_positions: int = 1024,
                 page_tokens: int = 16, gemm_path: int = GEMM_AUTO, stream=None):
        import torch
        self.shape = shape
        self.vocab = shape.vocab
        self.weights = weights  # keep the tensors alive
        want = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        cfg = ModelCfg(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                       shape.rms_eps, shape.rope_base, BF16 if shape.dtype == "bf16" else F32, page_tokens,
                       max_window, max_positions, gemm_path, int(getattr(shape, "n_kv_heads", 0) or 0))
        self.cfg = cfg

        def ptr(t):
            if not (t.is_cuda and t.is_contiguous() and t.dtype == want):
                raise ValueError("weights must be contiguous CUDA tensors of the model dtype")
            return t.data_ptr()

        ws = Weights()
        for name in ("embed", "final_norm", "lm_head"):
            setattr(ws, name, ptr(weights[name]))
        self._arrays = []
        for name in _PER_LAYER:
            arr = (C.c_void_p * shape.n_layers)(*[ptr(t) for t in weights[name]])
            self._arrays.append(arr)
            setattr(ws, name, C.cast(arr, C.POINTER(C.c_void_p)))
        nbytes = lib().anpd_model_workspace_bytes(C.byref(cfg))
        if nbytes == 0:
            _check(E_INVAL)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=weights["embed"].device)
        h = C.c_void_p()
        _check(lib().anpd_model_create(C.byref(cfg), C.byref(ws), self.workspace.data_ptr(), nbytes,
                                       _stream_ptr(stream), C.byref(h)))
        self._h = h
        self.device = weights["embed"].device
        self.max_window = max_window

    def close(self):
        try:
            if getattr(self, "_h", None) and _alive():
                lib().anpd_model_destroy(self._h)
        except TypeError:   # interpreter shutdown: this module's globals are already gone
            pass
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def trace(self, enable: bool):
        """Barrier timestamps of the one-kernel step: returns an int64 CUDA tensor [grid][1024] (or None)."""
        import torch
        if not enable:
            _check(lib().anpd_model_trace(self._h, None, 0))
            self._trace = None
            return None
        grid = _check(lib().anpd_model_trace(self._h, None, 0))
        if grid == 0:
            return None
        self._trace = torch.zeros(grid, 1024, dtype=torch.int64, device=self.device)
        _check(lib().anpd_model_trace(self._h, self._trace.data_ptr(), self._trace.numel() * 8))
        return self._trace

    def set_barrier_spin_limit(self, spins: int) -> None:
        """Test hook: polls before a grid-barrier wait of the one-kernel step gives up (0 = default)."""
        _check(lib().anpd_model_set_barrier_spin_limit(self._h, spins))

    def profile(self, enable: bool) -> None:
        _check(lib().anpd_model_profile(self._h, 1 if enable else 0))

    def profile_read(self) -> Dict[str, object]:
        n = len(PROF_CATEGORIES)
        ms, cnt, steps = (C.c_double * n)(), (C.c_int64 * n)(), C.c_int64(0)
        _check(lib().anpd_model_profile_read(self._h, ms, cnt, C.byref(steps)))
        return {"steps": steps.value, "ms": dict(zip(PROF_CATEGORIES, list(ms))),
                "intervals": dict(zip(PROF_CATEGORIES, list(cnt)))}

class KVCache:
    """anpd_kv_*: one sequence's paged KV cache in a torch-allocated pool."""

    def __init__(self, model: Model, max_tokens: int):
        import torch
        self.model = model
        nbytes = lib().anpd_kv_pool_bytes(model._h, max_tokens)
        if nbytes == 0:
            _check(E_INVAL)
        self.pool = torch.empty(nbytes, dtype=torch.uint8, device=model.device)
        h = C.c_void_p()
        _check(lib().anpd_kv_create(model._h, self.pool.data_ptr(), nbytes, max_tokens, C.byref(h)))
        self._h = h
        self.max_tokens = max_tokens

    def close(self):
        try:
            if getattr(self, "_h", None) and _alive():
                lib().anpd_kv_destroy(self._h)
        except TypeError:   # interpreter shutdown: this module's globals are already gone
            pass
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def length(self) -> int:
        return _check(lib().anpd_kv_length(self._h))

    @property
    def num_pages(self) -> int:
        return _check(lib().anpd_kv_num_pages(self._h))

    def truncate(self, new_len: int, stream=None) -> None:
        _check(lib().anpd_kv_truncate(self._h, new_len, _stream_ptr(stream)))

    def set_page_order(self, perm: Sequence[int]) -> None:
        _check(lib().anpd_kv_set_page_order(self._h, _ints(perm), len(perm)))

    def write(self, layer: int, pos0: int, k, v, stream=None) -> None:
        """k, v: CUDA float32 [n][n_kv_heads * head_dim]."""
        import torch
        assert k.is_cuda and k.dtype == torch.float32 and k.is_contiguous() and v.is_contiguous()
        _check(lib().anpd_kv_write(self._h, layer, pos0, k.shape[0], k.data_ptr(), v.data_ptr(), _stream_ptr(stream)))

    def read(self, layer: int, pos0: int, n: int, stream=None):
        import torch
        d = (getattr(self.model.shape, "n_kv_heads", 0) or self.model.shape.n_heads) * self.model.shape.head_dim
        k = torch.empty(n, d, dtype=torch.float32, device=self.model.device)
        v = torch.empty(n, d, dtype=torch.float32, device=self.model.device)
        _check(lib().anpd_kv_read(self._h, layer, pos0, n, k.data_ptr(), v.data_ptr(), _stream_ptr(stream)))
        return k, v


def verify(model: Model, kv: KVCache, window: Sequence[int], mode: int = VERIFY, want_predicts: bool = False,
           out_logits=None, stream=None):
    """anpd_verify.  Returns (accepted, next) or (accepted, next, predicts)."""
    n = len(window)
    acc, nxt = C.c_int32(0), C.c_int32(0)
    preds = (C.c_int32 * max(1, n))() if want_predicts else None
    lp = 0
    if out_logits is not None:
        import torch
        assert out_logits.is_cuda and out_logits.dtype == torch.float32 and out_logits.is_contiguous()
        assert out_logits.numel() >= n * model.vocab
        lp = out_logits.data_ptr()
    _check(lib().anpd_verify(model._h, kv._h, _ints(window), n, mode, C.byref(acc), C.byref(nxt), preds, lp,
                             _stream_ptr(stream)))
    if want_predicts:
        return acc.value, nxt.value, list(preds[:n])
    return acc.value, nxt.value


def verify_tree(model: Model, kv: KVCache, window: Sequence[int], parent: Sequence[int], want_predicts: bool = False,
                out_logits=None, stream=None):
    """anpd_verify_tree.  Returns (accepted depth, next token, path rows) or with the per-row predictions appended."""
    n = len(window)
    assert len(parent) == n
    acc, nxt = C.c_int32(0), C.c_int32(0)
    path = (C.c_int32 * (n + 1))()
    preds = (C.c_int32 * max(1, n))() if want_predicts else None
    lp = 0
    if out_logits is not None:
        import torch
        assert out_logits.is_cuda and out_logits.dtype == torch.float32 and out_logits.is_contiguous()
        assert out_logits.numel() >= n * model.vocab
        lp = out_logits.data_ptr()
    _check(lib().anpd_verify_tree(model._h, kv._h, _ints(window), _ints(parent), n, C.byref(acc), C.byref(nxt), path, preds, lp,
                                  _stream_ptr(stream)))
    if want_predicts:
        return acc.value, nxt.value, list(path[:acc.value + 1]), list(preds[:n])
    return acc.value, nxt.value, list(path[:acc.value + 1])


def verify_batch(model: Model, kvs: Sequence[KVCache], windows: Sequence[Sequence[int]], mode: int = VERIFY,
                 out_logits=None, stream=None):
    """anpd_verify_batch: one step for several sequences.  Returns [(accepted, next)] per sequence."""
    n = len(kvs)
    assert len(windows) == n
    handles = (C.c_void_p * max(1, n))(*[kv._h for kv in kvs])
    rows = [_ints(w) for w in windows]
    wins = (C.POINTER(C.c_int32) * max(1, n))(*[C.cast(r, C.POINTER(C.c_int32)) for r in rows])
    counts = _ints([len(w) for w in windows])
    acc, nxt = (C.c_int32 * max(1, n))(), (C.c_int32 * max(1, n))()
    lp = 0
    if out_logits is not None:
        import torch
        assert out_logits.is_cuda and out_logits.dtype == torch.float32 and out_logits.is_contiguous()
        assert out_logits.numel() >= sum(len(w) for w in windows) * model.vocab
        lp = out_logits.data_ptr()
    _check(lib().anpd_verify_batch(model._h, handles, n, wins, counts, mode, acc, nxt, lp, _stream_ptr(stream)))
    return [(acc[i], nxt[i]) for i in range(n)]


def pack_weights(W, stream=None):
    """anpd_pack_weights: bf16 CUDA [N][K] -> fragment-order buffer (uint8 tensor)."""
    import torch
    N, K = W.shape
    assert W.is_cuda and W.dtype == torch.bfloat16 and W.is_contiguous()
    nb = lib().anpd_packed_bytes(N, K)
    if nb == 0:
        _check(E_INVAL)
    out = torch.empty(nb, dtype=torch.uint8, device=W.device)
    _check(lib().anpd_pack_weights(W.data_ptr(), N, K, out.data_ptr(), nb, _stream_ptr(stream)))
    return out


def linear(X, W, path: int, stream=None, packed=None, Y=None, workspace=None):
    """anpd_linear: Y = X @ W.T.  X: CUDA float32 [M][K]; W: CUDA [N][K] float32 or bfloat16.
    For the MFMA paths the weights are repacked first unless ``packed`` (from pack_weights) is given."""
    import torch
    M, K = X.shape
    N = W.shape[0]
    assert X.is_cuda and X.dtype == torch.float32 and X.is_contiguous() and W.is_contiguous() and W.shape[1] == K
    dtype = BF16 if W.dtype == torch.bfloat16 else F32
    if Y is None:
        Y = torch.empty(M, N, dtype=torch.float32, device=X.device)
    nb = lib().anpd_linear_workspace_bytes(M, K)
    ws = workspace if workspace is not None else torch.empty(max(nb, 256), dtype=torch.uint8, device=X.device)
    wptr = W.data_ptr()
    if path in (GEMM_MFMA, GEMM_MFMA_STREAM):
        if dtype != BF16:
            _check(lib().anpd_linear(X.data_ptr(), wptr, Y.data_ptr(), M, N, K, dtype, path, ws.data_ptr(), nb,
                                     _stream_ptr(stream)))
        if packed is None:
            packed = pack_weights(W, stream)
        wptr = packed.data_ptr()
    _check(lib().anpd_linear(X.data_ptr(), wptr, Y.data_ptr(), M, N, K, dtype, path, ws.data_ptr(), nb,
                             _stream_ptr(stream)))
    return Y


def linear_static(X, packed, N: int, Y, stream=None):
    """anpd_linear_static: Y = X @ W.T on the matrix cores with the library's built-in scratch; allocates
    nothing (the caller passes the output).  ``packed``: W as written by pack_weights."""
    M, K = X.shape
    _check(lib().anpd_linear_static(X.data_ptr(), packed.data_ptr(), Y.data_ptr(), M, N, K, _stream_ptr(stream)))
    return Y


# ------------------------------------------------------------ decode loops

def prefill_workspace_bytes(model: Model, n_tokens: int) -> int:
    """anpd_prefill_workspace_bytes (0 for models that process the prompt in windows)."""
    return int(lib().anpd_prefill_workspace_bytes(model._h, n_tokens))


def prefill(model: Model, kv: KVCache, prompt: Sequence[int], stream=None, out_logits=None, workspace=None) -> int:
    """anpd_prefill: LLM(prompt) of Algorithm 1, all rows in one pass; returns the greedy token
    after the prompt.  ``out_logits``: CUDA float32 [vocab] for the last row's logits.
    ``workspace``: a CUDA uint8 tensor to reuse (allocated here if absent)."""
    import torch
    n = len(prompt)
    nb = prefill_workspace_bytes(model, n) if n >= 1 else 0
    ws = workspace
    if ws is None or ws.numel() < nb:
        ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    lp = 0
    if out_logits is not None:
        assert out_logits.is_cuda and out_logits.dtype == torch.float32 and out_logits.is_contiguous()
        assert out_logits.numel() >= model.vocab
        lp = out_logits.data_ptr()
    nxt = C.c_int32(0)
    _check(lib().anpd_prefill(model._h, kv._h, _ints(prompt), n, C.byref(nxt), lp, ws.data_ptr(), ws.numel(),
                              _stream_ptr(stream)))
    return nxt.value


def prefill_windows(model: Model, kv: KVCache, prompt: Sequence[int], stream=None) -> int:
    """The prompt appended through the verification step in windows of max_window rows (what
    anpd_prefill replaces on the matrix-core path); returns the greedy token after it."""
    nxt = -1
    for lo in range(0, len(prompt), model.max_window):
        _, nxt = verify(model, kv, prompt[lo:lo + model.max_window], APPEND, stream=stream)
    return nxt


def greedy_generate(model: Model, kv: KVCache, prompt: Sequence[int], n_tokens: int, stream=None) -> List[int]:
    """Plain autoregressive decoding: windows of one row."""
    c = prefill(model, kv, prompt, stream)
    out: List[int] = []
    while len(out) < n_tokens:
        out.append(c)
        _, c = verify(model, kv, [c], VERIFY, stream=stream)
    return out


def adaptive_draft_length(levels: Sequence[int], k_max: int) -> int:
    """Draft length chosen from the level that answered the first draft: 2^(level - 2), capped
    (level 2 -> 1 draft, 3 -> 2, 4 -> 4, 5 -> 8, 6 -> 16); no answer -> no drafts."""
    if not levels:
        return 0
    return max(1, min(k_max, 1 << (levels[0] - 2)))


def anpd_generate_multi(model: Model, kv: KVCache, table: NgramTable, prompt: Sequence[int], K: int, n_cand: int,
                        n_tokens: int, stream=None) -> Dict[str, object]:
    """Algorithm 1 with multi-candidate verification: every step drafts up to n_cand candidate
    continuations (NgramTable.propose_tree), scores them in one forward (verify_tree) and keeps the
    longest accepted one."""
    table.reset()
    table.update(prompt)
    c = prefill(model, kv, prompt, stream)
    out: List[int] = []
    steps = proposed = accepted = rows = 0
    while len(out) < n_tokens:
        table.update([c])
        out.append(c)
        toks, pars, _ = table.propose_tree(K, n_cand, model.max_window - 1)
        a, nxt, path = verify_tree(model, kv, [c] + toks, [-1] + pars, stream=stream)
        kept = [toks[r - 1] for r in path[1:]]
        if kept:
            table.update(kept)
            out.extend(kept)
        steps += 1
        proposed += len(toks)
        rows += 1 + len(toks)
        accepted += a
        c = nxt
    return {"tokens": out[:n_tokens], "n_steps": steps, "proposed": proposed, "accepted": accepted, "rows": rows}


def anpd_generate(model: Model, kv: KVCache, table: NgramTable, prompt: Sequence[int], K: int, n_tokens: int,
                  stream=None, drafter=None, adaptive: bool = False) -> Dict[str, object]:
    """Algorithm 1: commit, draft K tokens from the table, verify, accept the
    matching prefix, continue from the LLM's own token.  ``adaptive`` cuts the
    drafts of a step to adaptive_draft_length()."""
    table.reset()
    table.update(prompt)
    c = prefill(model, kv, prompt, stream)
    out: List[int] = []
    steps = proposed = accepted = 0
    while len(out) < n_tokens:
        table.update([c])
        out.append(c)
        if drafter is not None:
            drafts = drafter(len(out), K)
        else:
            drafts, levels = table.propose(K)
            if adaptive:
                drafts = drafts[:adaptive_draft_length(levels, K)]
        a, nxt = verify(model, kv, [c] + drafts, VERIFY, stream=stream)
        if a:
            table.update(drafts[:a])
            out.extend(drafts[:a])
        steps += 1
        proposed += len(drafts)
        accepted += a
        c = nxt
    return {"tokens": out[:n_tokens], "n_steps": steps, "proposed": proposed, "accepted": accepted}
