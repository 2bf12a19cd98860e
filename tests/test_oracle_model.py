"""Pins for the oracle's whole forward pass: library-routine composition in fp64, structural
invariants (paged == contiguous, chunked == unchunked == token-by-token, GQA == MHA with repeated
heads, causality, batch independence) and closed-form special cases (zeroed projections)."""
import dataclasses

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as O
from paper_2603_20661_amd import synth

SMALL = synth.ModelShape("small", 3, 64, 4, 2, 16, 96, 50, 1e-5, 1e4, synth.WDTYPE_F32, seed=11)
SMALL_BF16 = dataclasses.replace(SMALL, weight_dtype=synth.WDTYPE_BF16, seed=12)
SMALL_QKN = dataclasses.replace(SMALL, qk_norm=1, seed=13)       # query and key heads normalised before the rotation


def library_forward(shape, blob, tokens):
    """Logits at every position of ONE sequence, composed of PyTorch CPU library routines in fp64:
    embedding, rms_norm, linear, scaled_dot_product_attention(is_causal, enable_gqa), silu.
    The rotary embedding is written as complex multiplication."""
    t = lambda name: torch.from_numpy(synth.blob_tensor(shape, blob, name)).double()
    S, hd, Hq, Hkv = len(tokens), shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    x = F.embedding(torch.as_tensor(tokens, dtype=torch.long), t("embed"))
    ang = torch.arange(S, dtype=torch.float64)[:, None] * shape.rope_theta ** (-torch.arange(hd // 2, dtype=torch.float64) * 2 / hd)
    rot = torch.polar(torch.ones_like(ang), ang)                     # e^{i p theta_i}

    def rope(v):                                                     # v [S, H, hd]
        z = torch.complex(v[..., : hd // 2], v[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    for l in range(shape.n_layers):
        u = F.rms_norm(x, (shape.d_model,), t(f"l{l}.attn_norm"), eps=shape.rms_eps)
        qkv = F.linear(u, t(f"l{l}.wqkv"))
        q, k, v = qkv.split([Hq * hd, Hkv * hd, Hkv * hd], -1)
        q, k, v = q.view(S, Hq, hd), k.view(S, Hkv, hd), v.view(S, Hkv, hd)
        if shape.qk_norm:
            q = F.rms_norm(q, (hd,), t(f"l{l}.q_norm"), eps=shape.rms_eps)
            k = F.rms_norm(k, (hd,), t(f"l{l}.k_norm"), eps=shape.rms_eps)
        q, k = rope(q), rope(k)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           is_causal=True, enable_gqa=True)[0].transpose(0, 1).reshape(S, Hq * hd)
        x = x + F.linear(o, t(f"l{l}.wo"))
        u = F.rms_norm(x, (shape.d_model,), t(f"l{l}.ffn_norm"), eps=shape.rms_eps)
        g, up = F.linear(u, t(f"l{l}.wgu")).split([shape.ffn_dim, shape.ffn_dim], -1)
        x = x + F.linear(F.silu(g) * up, t(f"l{l}.wd"))
    return F.linear(F.rms_norm(x, (shape.d_model,), t("final_norm"), eps=shape.rms_eps), t("lm_head")).numpy()


def run_prefill(shape, blob, lens, toks, permute=True, paged=True, seed=3, num_blocks=64, mbs=8):
    m = O.OracleModel(shape, blob, max_seqs=len(lens), max_ctx=mbs * 16, num_blocks=num_blocks)
    m.set_kv_mode(paged)
    bt = synth.block_tables(seed, [mbs * 16 // 2] * len(lens), num_blocks, mbs, permute=permute)
    out = m.forward(toks, lens, lens, seq_ids=np.arange(len(lens)), block_table=bt, trace=True)
    return m, bt, out


@pytest.mark.parametrize("shape", [SMALL, SMALL_BF16, SMALL_QKN])
def test_forward_matches_library_composition(shape):
    blob = synth.make_blob(shape, std=0.2, gain_std=0.1)            # large weights: attention is far from uniform
    lens = np.array([23, 1, 40], np.int32)
    toks = synth.tokens(7, int(lens.sum()), shape.vocab)
    _, _, (logits, nxt, _) = run_prefill(shape, blob, lens, toks)
    at = 0
    for b, n in enumerate(lens):
        ref = library_forward(shape, blob, toks[at:at + n])[-1]
        at += n
        np.testing.assert_allclose(logits[b], ref, rtol=1e-5, atol=2e-5)
        assert nxt[b] == int(np.argmax(ref))


def test_tiny_config_first_token_matches_library_composition():
    wl = synth.workload("tiny")
    blob = synth.make_blob(wl.shape)
    m = O.OracleModel(wl.shape, blob, max_seqs=4, max_ctx=160, num_blocks=40)
    bt = synth.block_tables(0, [160] * 4, 40, 10)
    logits, nxt, _ = m.forward(wl.prompt_tokens, wl.prompt_lens, wl.prompt_lens, seq_ids=np.arange(4), block_table=bt)
    for b in range(4):
        ref = library_forward(wl.shape, blob, wl.prompt_tokens[b * 128:(b + 1) * 128])[-1]
        assert np.abs(logits[b] - ref).max() <= 1e-4
        assert nxt[b] == int(np.argmax(ref))


def test_head_normalisation_forgets_the_length_of_queries_and_keys():
    """With normalised heads, multiplying all weights of one query head and one key head by a constant changes nothing
    (up to the epsilon under the root, 1e-5 against mean squares of order 10); without, the same change moves the logits.
    The value heads are not normalised: scaling one of them does move the logits."""
    lens = np.array([19, 7], np.int32)
    toks = synth.tokens(21, int(lens.sum()), SMALL_QKN.vocab)
    hd, Hq, Hkv = SMALL_QKN.head_dim, SMALL_QKN.n_q_heads, SMALL_QKN.n_kv_heads

    def logits_with(shape, q_factor, k_factor, v_factor):
        blob = synth.make_blob(shape, std=0.2, gain_std=0.1)
        ent = {e[0]: e for e in synth.blob_layout(shape)[0]}
        for l in range(shape.n_layers):
            _, off, rows, cols, _ = ent[f"l{l}.wqkv"]
            w = blob[off:off + 4 * rows * cols].view(np.float32).reshape(rows, cols)
            w[1 * hd:2 * hd] *= q_factor                              # query head 1
            w[(Hq + 1) * hd:(Hq + 2) * hd] *= k_factor                # key head 1
            w[(Hq + Hkv) * hd:(Hq + Hkv + 1) * hd] *= v_factor        # value head 0
        return run_prefill(shape, blob, lens, toks)[2][0]

    base = logits_with(SMALL_QKN, 1.0, 1.0, 1.0)
    np.testing.assert_allclose(logits_with(SMALL_QKN, 4.0, 0.25, 1.0), base, rtol=0, atol=2e-4)
    assert np.abs(logits_with(SMALL_QKN, 1.0, 1.0, 4.0) - base).max() > 1e-2
    plain = dataclasses.replace(SMALL_QKN, qk_norm=0)
    assert np.abs(logits_with(plain, 4.0, 1.0, 1.0) - logits_with(plain, 1.0, 1.0, 1.0)).max() > 1e-2


def test_paged_equals_contiguous_and_block_permutation_is_invisible():
    blob = synth.make_blob(SMALL, std=0.2, gain_std=0.1)
    lens = np.array([33, 16, 5], np.int32)
    toks = synth.tokens(8, int(lens.sum()), SMALL.vocab)
    base = run_prefill(SMALL, blob, lens, toks, permute=False, paged=False)[2]
    for permute, paged, seed in ((False, True, 3), (True, True, 3), (True, True, 4), (True, False, 5)):
        other = run_prefill(SMALL, blob, lens, toks, permute=permute, paged=paged, seed=seed)[2]
        assert np.array_equal(base[0], other[0]) and np.array_equal(base[2], other[2])


def test_paged_pool_holds_rows_exactly_where_the_slot_map_says():
    blob = synth.make_blob(SMALL, std=0.2)
    lens = np.array([33, 16], np.int32)
    toks = synth.tokens(8, int(lens.sum()), SMALL.vocab)
    m, bt, _ = run_prefill(SMALL, blob, lens, toks, permute=True)
    pool = m.kv_paged()                                   # [blocks, L, 2, 16, Hkv*hd]
    flat = pool.transpose(1, 2, 0, 3, 4).reshape(SMALL.n_layers, 2, -1, pool.shape[-1])     # [L, 2, slot, row]
    used = np.zeros(flat.shape[2], bool)
    for b, n in enumerate(lens):
        for p in range(n):
            s = O.slot(bt[b], p)
            used[s] = True
            assert np.abs(flat[:, :, s]).sum() > 0
    assert np.abs(flat[:, :, ~used]).sum() == 0           # nothing written anywhere else


@pytest.mark.parametrize("chunk", [1, 5, 16, 37])
def test_chunked_prefill_and_decode_equal_one_prefill(chunk):
    blob = synth.make_blob(SMALL, std=0.2, gain_std=0.1)
    lens = np.array([45, 18], np.int32)
    toks = synth.tokens(9, int(lens.sum()), SMALL.vocab)
    _, _, (ref_logits, _, ref_trace) = run_prefill(SMALL, blob, lens, toks)
    m = O.OracleModel(SMALL, blob, max_seqs=2, max_ctx=128, num_blocks=64)
    bt = synth.block_tables(21, [64, 64], 64, 8)
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
    done = np.zeros(2, np.int64)
    rows = [[], []]
    last_logits = [None, None]
    while (done < lens).any():
        q = np.minimum(chunk, lens - done).astype(np.int32)
        act = np.nonzero(q > 0)[0]
        packed = np.concatenate([toks[starts[b] + done[b]: starts[b] + done[b] + q[b]] for b in act])
        lg, _, tr = m.forward(packed, q[act], (done + q)[act], seq_ids=act, block_table=bt[act], trace=True)
        at = 0
        for i, b in enumerate(act):
            rows[b].append(tr[-1, at:at + q[b]])
            at += q[b]
            last_logits[b] = lg[i]
        done += q
    for b in range(2):
        got = np.concatenate(rows[b])
        assert np.array_equal(got, ref_trace[-1, starts[b]:starts[b] + lens[b]])
        assert np.array_equal(last_logits[b], ref_logits[b])


def test_gqa_equals_mha_with_repeated_kv_heads():
    blob = synth.make_blob(SMALL, std=0.2, gain_std=0.1)
    mha = dataclasses.replace(SMALL, n_kv_heads=SMALL.n_q_heads)
    entries_g, _ = synth.blob_layout(SMALL)
    entries_m, total_m = synth.blob_layout(mha)
    blob_m = np.zeros(total_m, np.uint8)
    G, hd, Hq, Hkv = 2, SMALL.head_dim, SMALL.n_q_heads, SMALL.n_kv_heads
    for (name, off, r, c, dt), (_, off_m, r_m, c_m, _) in zip(entries_g, entries_m):
        src = blob[off:off + r * c * 4].view(np.float32).reshape(r, c)
        if name.endswith("wqkv"):
            q, k, v = src[:Hq * hd], src[Hq * hd:(Hq + Hkv) * hd], src[(Hq + Hkv) * hd:]
            rep = lambda a: np.repeat(a.reshape(Hkv, hd, c), G, axis=0).reshape(Hq * hd, c)   # head h uses KV head h // G
            src = np.concatenate([q, rep(k), rep(v)])
        blob_m[off_m:off_m + src.size * 4] = src.reshape(-1).view(np.uint8)
    lens = np.array([29, 7], np.int32)
    toks = synth.tokens(10, int(lens.sum()), SMALL.vocab)
    a = run_prefill(SMALL, blob, lens, toks)[2]
    b = run_prefill(mha, blob_m, lens, toks)[2]
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[2], b[2])


def test_causality_and_batch_independence():
    blob = synth.make_blob(SMALL, std=0.2, gain_std=0.1)
    lens = np.array([30, 12], np.int32)
    toks = synth.tokens(11, int(lens.sum()), SMALL.vocab)
    _, _, (lg, _, tr) = run_prefill(SMALL, blob, lens, toks)
    t2 = toks.copy()
    t2[20:30] = (t2[20:30] + 1) % SMALL.vocab            # change the tail of sequence 0
    _, _, (lg2, _, tr2) = run_prefill(SMALL, blob, lens, t2)
    assert np.array_equal(tr[:, :20], tr2[:, :20])         # earlier positions cannot see later tokens
    assert not np.array_equal(tr[-1, 20:30], tr2[-1, 20:30])
    assert np.array_equal(tr[:, 30:], tr2[:, 30:]) and np.array_equal(lg[1], lg2[1])   # the other sequence is untouched
    _, _, (lg3, _, tr3) = run_prefill(SMALL, blob, lens[1:], toks[30:])                 # alone in the batch
    assert np.array_equal(lg3[0], lg[1]) and np.array_equal(tr3[-1], tr[-1, 30:])


def _zero(shape, blob, suffixes):
    blob = blob.copy()
    for name, off, r, c, dt in synth.blob_layout(shape)[0]:
        if any(name.endswith(s) for s in suffixes):
            blob[off:off + r * c * 4] = 0
    return blob


def test_zeroed_projections_reduce_to_closed_forms():
    blob = synth.make_blob(SMALL, std=0.2, gain_std=0.1)
    lens = np.array([9], np.int32)
    toks = synth.tokens(12, 9, SMALL.vocab)
    # Wo = Wd = 0: the residual stream is the embedding, logits = rmsnorm(E[token]) W_lm^T
    z = _zero(SMALL, blob, (".wo", ".wd"))
    lg, _, tr = run_prefill(SMALL, z, lens, toks)[2]
    E = synth.blob_tensor(SMALL, z, "embed").astype(np.float64)
    g = synth.blob_tensor(SMALL, z, "final_norm").astype(np.float64)
    W = synth.blob_tensor(SMALL, z, "lm_head").astype(np.float64)
    e = E[toks[-1]]
    ref = (e / np.sqrt((e ** 2).mean() + 1e-5) * g) @ W.T
    np.testing.assert_allclose(lg[0], ref, rtol=1e-5, atol=1e-6)
    assert np.array_equal(tr[-1], E[toks].astype(np.float32))
    # Wd = 0 only: the feed-forward block is the identity on the residual, so the stream after layer l
    # equals the stream of a model whose FFN was never there; check against Wgu = 0 (also inert)
    a = run_prefill(SMALL, _zero(SMALL, blob, (".wd",)), lens, toks)[2]
    b = run_prefill(SMALL, _zero(SMALL, blob, (".wd", ".wgu")), lens, toks)[2]
    assert np.array_equal(a[0], b[0])
    assert not np.array_equal(a[0], run_prefill(SMALL, blob, lens, toks)[2][0])


def test_greedy_decode_of_tiny_config_is_self_consistent():
    """prefill + 16 greedy steps token by token == one prefill over prompt + generated tokens"""
    wl = synth.workload("tiny")
    blob = synth.make_blob(wl.shape)
    B, S, N = wl.batch, 128, wl.decode_steps
    m = O.OracleModel(wl.shape, blob, max_seqs=B, max_ctx=S + N + 1, num_blocks=B * 10)
    bt = synth.block_tables(0, [S + N + 1] * B, B * 10, 10)
    lens = wl.prompt_lens.copy()
    _, nxt, _ = m.forward(wl.prompt_tokens, lens, lens, seq_ids=np.arange(B), block_table=bt)
    gen = [nxt.copy()]
    all_logits = []
    for _ in range(N):
        lens = lens + 1
        lg, nxt, _ = m.forward(gen[-1], np.ones(B, np.int32), lens, seq_ids=np.arange(B), block_table=bt)
        all_logits.append(lg)
        gen.append(nxt.copy())
    gen = np.stack(gen, 1)                                 # [B, N+1]
    m2 = O.OracleModel(wl.shape, blob, max_seqs=B, max_ctx=S + N + 1, num_blocks=B * 10)
    full = np.concatenate([np.concatenate([wl.prompt_tokens[b * S:(b + 1) * S], gen[b, :N]]) for b in range(B)])
    lg2, nxt2, _ = m2.forward(full, np.full(B, S + N, np.int32), np.full(B, S + N, np.int32), seq_ids=np.arange(B),
                              block_table=synth.block_tables(1, [S + N + 1] * B, B * 10, 10))
    assert np.array_equal(lg2, all_logits[-1]) and np.array_equal(nxt2, gen[:, N])


def test_bad_arguments_are_rejected():
    blob = synth.make_blob(SMALL)
    m = O.OracleModel(SMALL, blob, max_seqs=1, max_ctx=32, num_blocks=4)
    bt = np.array([[0, 1, -1, -1]], np.int32)
    ok = lambda **k: m.forward(k.get("t", [1, 2]), k.get("q", [2]), k.get("s", [2]), seq_ids=k.get("i", [0]), block_table=k.get("bt", bt))
    ok()
    for bad in (dict(s=[1]), dict(i=[1]), dict(s=[40], q=[2]), dict(t=[1, 50]), dict(s=[33], q=[2], t=[1, 2]),
                dict(bt=np.array([[7, 1, -1, -1]], np.int32)), dict(s=[20], bt=np.array([[0, -1, -1, -1]], np.int32))):
        with pytest.raises(ValueError):
            ok(**bad)
