"""The benchmark's algorithmic byte and flop counts against explicit enumerations on small shapes: every weight
tensor of the blob that a decode step streams, every (query, key) pair a causal prefill touches."""
import dataclasses

import numpy as np

import bench
from paper_2603_20661_amd import synth

SHAPE = synth.ModelShape("acct", 3, 128, 4, 2, 32, 224, 96, 1e-5, 1e4, synth.WDTYPE_BF16, seed=1)


def test_decode_step_bytes_are_the_streamed_tensors_plus_the_context():
    ctx = np.array([5, 17, 64, 33])
    B = len(ctx)
    entries, _ = synth.blob_layout(SHAPE)
    weights = sum(rows * cols * 2 for name, _, rows, cols, dt in entries if dt == synth.WDTYPE_BF16 and name != "embed")
    kv_token = SHAPE.n_layers * 2 * SHAPE.n_kv_heads * (SHAPE.head_dim * 2 + 4)      # 16-bit codes and one fp32 scale per vector
    want = weights + B * SHAPE.d_model * 2 + int(ctx.sum()) * kv_token + B * kv_token + B * SHAPE.vocab * 4
    assert bench.decode_step_bytes(SHAPE, ctx, B) == want


def test_quantised_formats_count_their_own_bytes():
    ctx = np.array([40, 9])
    entries, _ = synth.blob_layout(SHAPE)
    n_weights = sum(rows * cols for name, _, rows, cols, dt in entries if dt == synth.WDTYPE_BF16 and name != "embed")
    base = bench.decode_step_bytes(SHAPE, ctx, 2)
    for dt, per_weight in ((synth.WDTYPE_FP8WO, 1.0), (synth.WDTYPE_INT4WO_128, 0.5 + 2 / 128), (synth.WDTYPE_INT4WO_32, 0.5 + 2 / 32)):
        got = bench.decode_step_bytes(dataclasses.replace(SHAPE, weight_dtype=dt), ctx, 2)
        assert got == base - n_weights * 2 + n_weights * per_weight


def test_prefill_flops_enumerated():
    """Chunks with cached prefixes, counted token by token and pair by pair.  The method runs a bulk pass over all new
    tokens (every layer's QKV projection; attention, O and FFN of all layers but the last) and then the final position
    of every sequence once more through all layers and the output head."""
    s = SHAPE
    d, F, V, L, hd, Hq = s.d_model, s.ffn_dim, s.vocab, s.n_layers, s.head_dim, s.n_q_heads
    QD, KD = Hq * hd, s.n_kv_heads * hd
    q_lens, seq_lens = [7, 1, 20], [7, 12, 31]
    qkv = 2 * (QD + 2 * KD) * d                 # flops of the QKV projection of one token
    rest = 2 * (d * QD + 3 * F * d)             # O, gate, up and down projections of one token
    pair = 2 * 2 * Hq * hd                      # one (query, key) pair: score and value products of every head
    total = 0
    for q, n in zip(q_lens, seq_lens):
        prefix = n - q
        for i in range(q):                      # bulk pass: new token i sits at position prefix + i
            total += qkv * L + rest * (L - 1)
            total += pair * (prefix + i + 1) * (L - 1)
        total += (qkv + rest) * L + pair * n * L + 2 * V * d      # single-token pass of the final position
    assert bench.prefill_call_flops(s, q_lens, seq_lens) == total
    assert bench.prefill_flops(s, [5, 9]) == bench.prefill_call_flops(s, [5, 9], [5, 9])
