"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its N-gram table agrees bit for bit with the scanning
oracle.  No compute call touches a GPU here."""
import ctypes
import itertools
import os
import re

import pytest

from oracle import ngram as ong
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "anpd.h")).read()
    declared = set(re.findall(r"\b(anpd_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


def _check_stream(s, n_min, n_max, K=6):
    t = B.NgramTable(n_min, n_max, max(s) + 1)
    # feed in ragged pieces: update(a) + update(b) == update(a || b)
    cut = len(s) // 3
    t.update(s[:cut]); t.update(s[cut:cut + 1]); t.update(s[cut + 1:])
    assert len(t) == len(s)
    assert t.propose(K) == ong.propose(s, K, n_min, n_max)
    return t


def test_table_matches_oracle_exhaustively_on_tiny_alphabets():
    for T in range(1, 8):
        for s in itertools.product(range(3), repeat=T):
            s = list(s)
            t = _check_stream(s, 2, 4, K=4)
            for tail in ([0], [1, 2], [2, 2, 1], [0, 1, 0, 2]):
                assert t.query(tail) == ong.mln_query(s, tail, 2, 4)


@pytest.mark.parametrize("n_min,n_max", [(2, 2), (2, 5), (3, 3), (4, 7)])
def test_table_matches_oracle_on_copy_heavy_streams(n_min, n_max):
    for seed in range(4):
        s = synth.markov_stream(50, 300, 0.4, 4, 16, seed)
        t = B.NgramTable(n_min, n_max, 50)
        # incremental: the proposal after every prefix agrees with a fresh scan
        for i, tok in enumerate(s):
            t.update([tok])
            if i % 7 == 0 or i > 280:
                assert t.propose(5) == ong.propose(s[:i + 1], 5, n_min, n_max)


def test_reset_and_errors():
    t = B.NgramTable(2, 3, 10)
    t.update([1, 2, 1])
    assert t.propose(3)[0] == [2, 1, 2]
    t.reset()
    assert len(t) == 0 and t.propose(3) == ([], [])
    with pytest.raises(B.AnpdError) as e:
        t.update([1, 10])
    assert e.value.code == B.E_RANGE and len(t) == 0      # nothing appended
    with pytest.raises(B.AnpdError):
        t.update([-1])
    for bad in [(1, 3, 10), (3, 2, 10), (2, 17, 10), (2, 3, 0)]:
        with pytest.raises(B.AnpdError) as e:
            B.NgramTable(*bad)
        assert e.value.code == B.E_INVAL
    assert t.query([]) == (None, 0)
    assert t.propose(0) == ([], [])


def test_device_side_argument_errors_need_no_gpu():
    L = B.lib()
    cfg = B.ModelCfg(2, 256, 4, 64, 688, 1024, 1e-5, 10000.0, B.F32, 16, 8, 256, B.GEMM_AUTO)
    assert L.anpd_model_workspace_bytes(ctypes.byref(cfg)) > 0
    bad = B.ModelCfg(2, 256, 4, 60, 688, 1024, 1e-5, 10000.0, B.F32, 16, 8, 256, B.GEMM_AUTO)
    assert L.anpd_model_workspace_bytes(ctypes.byref(bad)) == 0
    assert b"head_dim" in L.anpd_last_error()
    bad = B.ModelCfg(2, 256, 4, 64, 688, 1024, 1e-5, 10000.0, B.F32, 16, 33, 256, B.GEMM_AUTO)
    assert L.anpd_model_workspace_bytes(ctypes.byref(bad)) == 0
    bad = B.ModelCfg(2, 256, 4, 64, 688, 1024, 1e-5, 10000.0, B.F32, 16, 8, 256, B.GEMM_MFMA)
    assert L.anpd_model_workspace_bytes(ctypes.byref(bad)) == 0
    h = ctypes.c_void_p()
    assert L.anpd_model_create(ctypes.byref(cfg), None, None, 0, None, ctypes.byref(h)) == B.E_INVAL
    assert L.anpd_kv_length(None) == B.E_INVAL
    a = ctypes.c_int32()
    assert L.anpd_verify(None, None, None, 1, 0, ctypes.byref(a), ctypes.byref(a), None, None, None) == B.E_INVAL
    assert L.anpd_linear(None, None, None, 1, 16, 8, 0, 1, None, 0, None) == B.E_INVAL
    assert L.anpd_linear_workspace_bytes(0, 64) == 0
    assert L.anpd_verify_tree(None, None, None, None, 1, ctypes.byref(a), ctypes.byref(a), None, None, None, None) == B.E_INVAL
    assert L.anpd_verify_batch(None, None, 1, None, None, 0, ctypes.byref(a), ctypes.byref(a), None, None) == B.E_INVAL
    assert L.anpd_prefill(None, None, None, 1, ctypes.byref(a), None, None, 0, None) == B.E_INVAL
    assert L.anpd_prefill_workspace_bytes(None, 5) == 0
    grouped = B.ModelCfg(2, 256, 4, 64, 688, 1024, 1e-5, 10000.0, B.BF16, 16, 8, 256, B.GEMM_AUTO, 2)
    plain = B.ModelCfg(2, 256, 4, 64, 688, 1024, 1e-5, 10000.0, B.BF16, 16, 8, 256, B.GEMM_AUTO, 0)
    assert 0 < L.anpd_model_workspace_bytes(ctypes.byref(grouped)) < L.anpd_model_workspace_bytes(ctypes.byref(plain))
    bad = B.ModelCfg(2, 256, 4, 64, 688, 1024, 1e-5, 10000.0, B.BF16, 16, 8, 256, B.GEMM_AUTO, 3)
    assert L.anpd_model_workspace_bytes(ctypes.byref(bad)) == 0 and b"n_kv_heads" in L.anpd_last_error()
