"""Several sequences verified in one step (anpd_verify_batch): every sequence must get, bit for bit, what
anpd_verify gives it alone (and hence what the oracle checks there), whatever shares the step with it."""
import numpy as np
import pytest
import torch

from oracle import decoder as od
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth
from helpers import TOL, gpu_logits, to_cuda

pytestmark = pytest.mark.gpu


def _setup(shape, lengths, seed, max_window=32):
    w = synth.make_weights(shape, seed)
    model = B.Model(shape, to_cuda(w), max_window=max_window, max_positions=400)
    prompts = [synth.markov_stream(shape.vocab, n, 0.3, 4, 12, 100 + i) for i, n in enumerate(lengths)]
    alone, joint = [], []
    for p in prompts:
        for group in (alone, joint):
            kv = B.KVCache(model, 400)
            B.prefill(model, kv, p)
            group.append(kv)
    return w, model, prompts, alone, joint


@pytest.mark.parametrize("shape_name", ["MID_BF16", "MID_GQA", "TINY_BF16"])
def test_each_sequence_gets_what_it_gets_alone(shape_name):
    shape = getattr(synth, shape_name)
    lengths = [37, 150, 290, 16]
    w, model, prompts, alone, joint = _setup(shape, lengths, 51)
    for round_, rows in enumerate(([5, 1, 9, 3], [1, 1, 1, 1], [8, 8, 8, 8], [2, 17, 1, 4], [2, 1, 3, 2], [1, 4, 1, 1])):
        windows = [synth.random_tokens(shape.vocab, n, 200 + 10 * round_ + i) for i, n in enumerate(rows)]
        for kv_a, kv_j, n in zip(alone, joint, lengths):
            kv_a.truncate(n)
            kv_j.truncate(n)
        singles = [gpu_logits(model, kv, win) for kv, win in zip(alone, windows)]
        buf = torch.empty(sum(rows), shape.vocab, dtype=torch.float32, device="cuda")
        got = B.verify_batch(model, joint, windows, out_logits=buf)
        logits = buf.cpu().numpy().astype(np.float64)
        r = 0
        for i, (a, nxt, preds, lg) in enumerate(singles):
            assert got[i] == (a, nxt), (round_, i)
            assert np.array_equal(logits[r:r + rows[i]], lg), (round_, i)
            r += rows[i]
            assert joint[i].length == alone[i].length == lengths[i] + 1 + a
            for layer in range(shape.n_layers):
                ka, va = alone[i].read(layer, lengths[i], 1 + a)    # the rows the step kept
                kj, vj = joint[i].read(layer, lengths[i], 1 + a)
                assert torch.equal(ka, kj) and torch.equal(va, vj)
    # and one of them against the oracle, through the batch
    dec = od.Decoder(shape, w, 400)
    dec.prefill(prompts[1])
    for kv_j, n in zip(joint, lengths):
        kv_j.truncate(n)
    windows = [synth.random_tokens(shape.vocab, n, 300 + i) for i, n in enumerate([3, 6, 2, 1])]
    buf = torch.empty(12, shape.vocab, dtype=torch.float32, device="cuda")
    B.verify_batch(model, joint, windows, B.APPEND, out_logits=buf)
    ref = dec.forward(windows[1])
    assert float(np.max(np.abs(buf[3:9].cpu().numpy().astype(np.float64) - ref))) < TOL["bf16"]
    assert [kv.length for kv in joint] == [n + m for n, m in zip(lengths, [3, 6, 2, 1])]


def test_thirty_two_sequences_decoding_one_token_each():
    shape = synth.MID_BF16
    w = synth.make_weights(shape, 52, device="cuda")
    model = B.Model(shape, w, max_window=32, max_positions=128)
    kvs_a, kvs_j, cur = [], [], []
    for i in range(32):
        p = synth.markov_stream(shape.vocab, 20 + 3 * i, 0.3, 4, 12, 400 + i)
        ka, kj = B.KVCache(model, 128), B.KVCache(model, 128)
        cur.append(B.prefill(model, ka, p))
        B.prefill(model, kj, p)
        kvs_a.append(ka)
        kvs_j.append(kj)
    alone, joint = [list(cur)], [list(cur)]
    for _ in range(4):
        alone.append([B.verify(model, kv, [t])[1] for kv, t in zip(kvs_a, alone[-1])])
        joint.append([nxt for _, nxt in B.verify_batch(model, kvs_j, [[t] for t in joint[-1]])])
    assert alone == joint
    assert [kv.length for kv in kvs_a] == [kv.length for kv in kvs_j]


def test_eight_rows_or_fewer_run_in_the_persistent_kernel_with_the_same_bits():
    """Batches of at most 8 rows take the one-kernel form of the step; a model built for separate launches
    takes the fused launches.  Same results, bit for bit, over several decoding steps with lengths that
    cross a page and an attention split."""
    shape = synth.MID_BF16
    w = synth.make_weights(shape, 55, device="cuda")
    one = B.Model(shape, w, max_window=8, max_positions=400)
    many = B.Model(shape, w, max_window=8, max_positions=400, gemm_path=B.GEMM_MFMA_LAUNCHES)
    lengths = [125, 15, 260, 1, 127, 64, 31, 200]
    state = []
    for model in (one, many):
        kvs, cur = [], []
        for i, n in enumerate(lengths):
            kv = B.KVCache(model, 400)
            cur.append(B.prefill(model, kv, synth.markov_stream(shape.vocab, n, 0.3, 4, 12, 500 + i)))
            kvs.append(kv)
        state.append((model, kvs, cur))
    assert state[0][2] == state[1][2]
    bufs = [torch.empty(8, shape.vocab, dtype=torch.float32, device="cuda") for _ in range(2)]
    for step in range(5):
        outs = []
        for (model, kvs, cur), buf in zip(state, bufs):
            res = B.verify_batch(model, kvs, [[t] for t in cur], out_logits=buf)
            outs.append(res)
            cur[:] = [nxt for _, nxt in res]
        assert outs[0] == outs[1], step
        assert torch.equal(bufs[0], bufs[1]), step
    assert [kv.length for kv in state[0][1]] == [kv.length for kv in state[1][1]] == [n + 5 for n in lengths]
    # ragged windows with drafts: 3 sequences, 8 rows in all, verification mode
    for (model, kvs, cur), buf in zip(state, bufs):
        wins = [[cur[0], 5, 6], [cur[1]], [cur[2], 7, 8, 9]]
        res = B.verify_batch(model, kvs[:3], wins, out_logits=buf)
        state[state.index((model, kvs, cur))] = (model, kvs, res)
    assert state[0][2] == state[1][2] and torch.equal(bufs[0], bufs[1])
    for layer in range(shape.n_layers):
        for a, b, n in zip(state[0][1], state[1][1], lengths):
            ka, va = a.read(layer, 0, a.length)
            kb, vb = b.read(layer, 0, b.length)
            assert a.length == b.length and torch.equal(ka, kb) and torch.equal(va, vb)


def test_batch_argument_errors():
    shape = synth.TINY_BF16
    w = synth.make_weights(shape, 53, device="cuda")
    model = B.Model(shape, w, max_window=8, max_positions=64)
    kv1, kv2 = B.KVCache(model, 64), B.KVCache(model, 64)
    B.prefill(model, kv1, [1, 2, 3])
    B.prefill(model, kv2, [4, 5])
    for kvs, wins, code in (([kv1, kv1], [[1], [2]], B.E_INVAL), ([kv1, kv2], [[1] * 5, [2] * 4], B.E_CAPACITY),
                            ([kv1, kv2], [[1], [shape.vocab]], B.E_RANGE), ([kv1, kv2], [[1], []], B.E_INVAL)):
        with pytest.raises(B.AnpdError) as e:
            B.verify_batch(model, kvs, wins)
        assert e.value.code == code and (kv1.length, kv2.length) == (3, 2)
    f32 = synth.TINY
    model32 = B.Model(f32, synth.make_weights(f32, 54, device="cuda"), max_window=8, max_positions=64)
    kv3 = B.KVCache(model32, 64)
    with pytest.raises(B.AnpdError) as e:
        B.verify_batch(model32, [kv3], [[1]])
    assert e.value.code == B.E_UNIMPLEMENTED
