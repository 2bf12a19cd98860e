"""The fp8 weight-only oracle (oracle/quant.py) against the E4M3 format definition, and the blob decoder against a
direct decode of single tensors."""
import dataclasses
import math

import numpy as np
import pytest

from oracle import quant as Q
from paper_2603_20661_amd import synth

T8 = synth.ModelShape("t8", 2, 64, 4, 2, 16, 96, 48, 1e-5, 1e4, synth.WDTYPE_FP8WO, seed=51)


def test_e4m3_values_are_the_format_s():
    t = Q.TABLE
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and math.copysign(1.0, t[0x80]) == -1.0
    assert t[0x38] == 1.0 and t[0x40] == 2.0 and t[0x3C] == 1.5 and t[0xB8] == -1.0
    assert t[0x7E] == 448.0 and t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9 and t[0x08] == 2.0 ** -6
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(np.delete(t, [0x7F, 0xFF])).all()
    pos = t[:0x7F]
    assert (np.diff(pos) > 0).all()                                 # codes order the magnitudes
    assert np.array_equal(t[0x80:0xFF], -pos)
    # within a binade the 8 values are equally spaced, and each binade doubles the spacing
    for e in range(1, 15):
        step = np.diff(pos[8 * e: 8 * e + 8])
        assert (step == 2.0 ** (e - 7 - 3)).all()


def test_generator_codes_are_the_nearest_values_ties_to_even():
    """The blob's codes come from the generator's encoder (an input recipe); here it is held to the format: nearest
    representable value, ties to the even code, saturation at 448."""
    lib = synth._load()
    xs = np.concatenate([synth.normal_f32(9, 1, 20000, std=60.0), np.array([0.0, -0.0, 1e-9, 2.0 ** -10, 3 * 2.0 ** -10, 447.9, 448.0,
                         463.9, 464.0, 1e6, -1e6, 1.0625, 1.1875, 17.0, 19.0, 2.0 ** -6 - 2.0 ** -11], np.float32)]).astype(np.float32)
    codes = np.empty(xs.size, np.uint8)
    lib.wwwsynth_encode_e4m3(xs.ctypes.data, xs.size, 1.0, codes.ctypes.data)
    pos = Q.TABLE[:0x7F].astype(np.float64)
    for x, c in zip(xs.astype(np.float64), codes):
        a = min(abs(x), 448.0)
        err = np.abs(pos - a)
        best = np.flatnonzero(err == err.min())
        want = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]
        assert (c & 0x7F) == want and bool(c & 0x80) == bool(np.signbit(x)), (x, c, want)
    assert codes[20000 + 2] == 0x00 and codes[20000 + 3] == 0x00 and codes[20000 + 4] == 0x02   # 2^-10 ties to even 0, 3*2^-10 to 2
    assert codes[20000 + 8] == 0x7E and codes[20000 + 9] == 0x7E and codes[20000 + 10] == 0xFE  # saturation, never NaN


def test_blob_decoder_matches_tensor_by_tensor_decode():
    blob = synth.make_blob(T8, gain_std=0.1)
    entries, total = synth.blob_layout(T8)
    assert total == blob.size
    shape32, blob32 = Q.dequantize_blob(T8, blob)
    assert shape32.weight_dtype == synth.WDTYPE_F32 and blob32.size == synth.blob_layout(shape32)[1]
    by_name = {e[0]: e for e in entries}
    for name in ("l0.wqkv", "l1.wd", "lm_head", "l1.wgu"):
        _, off, rows, cols, dt = by_name[name]
        assert dt == synth.WDTYPE_FP8WO
        codes = blob[off:off + rows * cols].reshape(rows, cols)
        scale = blob[by_name[name + ".scale"][1]:][:4].view(np.float32)[0]
        want = np.array([[np.float32(Q.e4m3_value(int(c))) * scale for c in row] for row in codes[:5]], np.float32)
        got = synth.blob_tensor(shape32, blob32, name)
        assert np.array_equal(got[:5], want)
        assert np.abs(got).max() == pytest.approx(448.0 * scale, rel=1e-6)      # the largest weight sits on the top code
        assert 0.015 < got.std() < 0.025                                         # still ~N(0, 0.02)
    assert np.array_equal(synth.blob_tensor(shape32, blob32, "l1.ffn_norm"),
                          blob[by_name["l1.ffn_norm"][1]:][:4 * T8.d_model].view(np.float32))
    emb = synth.blob_tensor(shape32, blob32, "embed")
    assert np.array_equal(emb, synth.bf16_bits_to_f32(blob[:2 * T8.vocab * T8.d_model].view(np.uint16)).reshape(T8.vocab, T8.d_model))


@pytest.mark.parametrize("wd", [synth.WDTYPE_FP8WO, synth.WDTYPE_INT4WO_32])
def test_blob_decoder_carries_the_head_normalisation_gains(wd):
    """a weight-only quantised model with normalised query / key heads: the two gain vectors that follow wqkv arrive
    unchanged at their place in the decoded blob, and so does everything behind them"""
    shape = synth.ModelShape("t8qkn", 2, 64, 4, 2, 32, 96, 48, 1e-5, 1e4, wd, seed=53, qk_norm=1)
    blob = synth.make_blob(shape, gain_std=0.1)
    by_name = {e[0]: e for e in synth.blob_layout(shape)[0]}
    shape32, blob32 = Q.dequantize_blob(shape, blob)
    assert shape32.qk_norm == 1 and blob32.size == synth.blob_layout(shape32)[1]
    for name, n in (("l0.q_norm", shape.head_dim), ("l1.k_norm", shape.head_dim), ("l1.ffn_norm", shape.d_model), ("final_norm", shape.d_model)):
        src = blob[by_name[name][1]:][:4 * n].view(np.float32)
        assert np.array_equal(synth.blob_tensor(shape32, blob32, name), src) and src.std() > 0.05
    plain32 = Q.dequantize_blob(dataclasses.replace(shape, qk_norm=0), synth.make_blob(dataclasses.replace(shape, qk_norm=0), gain_std=0.1))[1]
    assert blob32.size == plain32.size + 2 * shape.n_layers * 256          # two 256-byte slots per layer more than the plain model


T4 = {g: synth.ModelShape(f"t4g{g}", 2, 128, 4, 2, 32, 256, 48, 1e-5, 1e4, dt, seed=52)
      for g, dt in ((128, synth.WDTYPE_INT4WO_128), (32, synth.WDTYPE_INT4WO_32))}


@pytest.mark.parametrize("group", [128, 32])
def test_int4_blob_decoder_against_the_definition_and_the_recipe(group):
    """Decoded weights are (code - 8) * scale element by element (checked through an independent unpacking), every group's
    largest weight lands on code 1 or 15, and the rounding error of a weight is at most half a step of its group."""
    sh = T4[group]
    blob = synth.make_blob(sh)
    entries, total = synth.blob_layout(sh)
    assert total == blob.size
    shape32, blob32 = Q.dequantize_blob(sh, blob)
    by_name = {e[0]: (t, e) for t, e in enumerate(entries)}
    for name in ("l0.wqkv", "l1.wd", "lm_head"):
        t, (_, off, rows, cols, dt) = by_name[name]
        _, (_, soff, srows, ng, sdt) = by_name[name + ".scale"]
        assert (srows, ng, sdt) == (rows, cols // group, synth.WDTYPE_BF16)
        got = synth.blob_tensor(shape32, blob32, name)
        scales = synth.bf16_bits_to_f32(blob[soff:soff + rows * ng * 2].view(np.uint16)).reshape(rows, ng)
        for r, k in ((0, 0), (0, 1), (3, group - 1), (rows - 1, cols - 1), (5, group % cols), (7, cols // 2 + 3)):
            byte = int(blob[off + (r * cols + k) // 2])
            code = (byte >> 4) if k % 2 else (byte & 0xF)
            assert got[r, k] == np.float32((code - 8) * float(scales[r, k // group]))
        w = synth.normal_f32(sh.seed, t, rows * cols, std=0.02).reshape(rows, cols)     # what the codes were made from
        step = np.repeat(scales, group, axis=1)
        assert (np.abs(got - w) <= 0.5 * step * (1 + 1e-6)).all()
        amax_code = np.abs(got / step).reshape(rows, ng, group).max(axis=2)
        assert (amax_code == 7).all()


def test_quantised_model_runs_through_the_model_oracle_and_stays_close_to_the_unquantised_one():
    """Sanity of the whole chain: the decoded blob is a valid fp32 model whose logits differ from those of the fp32
    weights it was rounded from by a few per cent of their spread (E4M3 keeps 3 mantissa bits)."""
    from oracle import oracle as O
    blob8 = synth.make_blob(T8)
    shape32, blob32 = Q.dequantize_blob(T8, blob8)
    ref_shape = dataclasses.replace(T8, weight_dtype=synth.WDTYPE_F32)
    # the unquantised weights: same seed and streams (the fp8 layout numbers its tensors differently, so draw by name)
    entries8 = {e[0]: t for t, e in enumerate(synth.blob_layout(T8)[0])}
    ref_entries, ref_total = synth.blob_layout(ref_shape)
    ref = np.zeros(ref_total, np.uint8)
    for name, off, rows, cols, dt in ref_entries:
        n = rows * cols
        view = ref[off:off + 4 * n].view(np.float32)
        if name.endswith("norm"):
            view[:] = 1.0
        elif name == "embed":
            view[:] = synth.blob_tensor(shape32, blob32, "embed").reshape(-1)
        else:
            synth.normal_f32(T8.seed, entries8[name], n, std=0.02, out=view)
    toks = synth.tokens(3, 24, T8.vocab)
    outs = []
    for sh, bl in ((shape32, blob32), (ref_shape, ref)):
        m = O.OracleModel(sh, bl, max_seqs=1, max_ctx=32)
        lg, _, _ = m.forward(toks, [24], [24], seq_ids=[0])
        outs.append(lg[0])
        m.close()
    rel = np.abs(outs[0] - outs[1]).max() / outs[1].std()
    assert 0.0 < rel < 0.5, rel
