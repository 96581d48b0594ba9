"""The one-kernel step's own facilities: barrier trace, barrier time-out and recovery."""
import numpy as np
import pytest
import torch

from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth
from helpers import to_cuda

pytestmark = pytest.mark.gpu


def _tiny_model(max_tokens=256):
    shape = synth.TINY_BF16
    w = synth.make_weights(shape, 5)
    model = B.Model(shape, to_cuda(w), max_window=8, max_positions=max_tokens, gemm_path=B.GEMM_MFMA)
    kv = B.KVCache(model, max_tokens)
    return shape, model, kv


def test_barrier_trace_has_one_ordered_stamp_pair_per_barrier():
    shape, model, kv = _tiny_model()
    prompt = synth.workload_prompt("tiny")[:40]
    c = B.prefill(model, kv, prompt)
    tr = model.trace(True)
    assert tr is not None and tr.shape[1] == 1024          # this model runs the step as one kernel
    B.verify(model, kv, [c] + synth.random_tokens(shape.vocab, 4, 9))
    torch.cuda.synchronize()
    t = tr.cpu().numpy()
    n_events = 1 + 2 * (1 + 5 * shape.n_layers + 1)         # start, then arrive / release per barrier
    used = t[:, :n_events]
    assert (used > 0).all()
    assert (np.diff(used, axis=1) >= 0).all()               # every block's stamps are in program order
    assert (t[:, n_events:] == 0).all()
    # a barrier releases nobody before its last arrival: release k of any block >= every arrival k
    # (10 ns clock: allow one tick)
    # (the barrier that ends a QKV phase is arrived at but not waited for: attention tasks wait for
    # their own head's tiles instead, so those stamp pairs are exempt)
    for k in range(1 + 5 * shape.n_layers + 1):
        if k >= 1 and (k - 1) % 5 == 0 and k < 1 + 5 * shape.n_layers:
            continue
        arrive, release = used[:, 1 + 2 * k], used[:, 2 + 2 * k]
        assert release.min() >= arrive.max() - 1
    assert model.trace(False) is None


def test_barrier_timeout_is_reported_and_the_next_step_is_correct():
    shape, model, kv = _tiny_model()
    prompt = synth.workload_prompt("tiny")[:48]
    c = B.prefill(model, kv, prompt)
    L0 = kv.length
    window = [c] + synth.random_tokens(shape.vocab, 5, 21)
    buf = torch.empty(len(window), shape.vocab, dtype=torch.float32, device="cuda")
    want = B.verify(model, kv, window, B.VERIFY, want_predicts=True, out_logits=buf)
    want_logits = buf.clone()
    kv.truncate(L0)

    model.set_barrier_spin_limit(1)                         # every wait gives up at once
    with pytest.raises(B.AnpdError):
        B.verify(model, kv, window)
    assert kv.length == L0                                  # the host's view did not advance
    model.set_barrier_spin_limit(0)
    kv.truncate(L0)                                         # cache contents past L0 are undefined after the error
    got = B.verify(model, kv, window, B.VERIFY, want_predicts=True, out_logits=buf)
    assert got == want
    assert torch.equal(buf, want_logits)
    with pytest.raises(B.AnpdError):
        model.set_barrier_spin_limit(-1)
