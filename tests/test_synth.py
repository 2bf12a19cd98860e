"""The seeded input generator: determinism, published known answers of its mixing function,
distribution moments, bf16 rounding against a library conversion, workload recipes."""
import os

import numpy as np
import pytest
import torch

from paper_2603_20661_amd import synth

M64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15


def py_mix(z):
    z = (z + GOLDEN) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def test_mix_is_splitmix64():
    # SplitMix64 seeded with 0 produces these first outputs (Steele, Lea, Flood 2014; the values are
    # the ones every published implementation lists).  Output n is mix(n * GOLDEN) in our notation.
    expect = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    got = [synth.mix((n * GOLDEN) & M64) for n in range(3)]
    assert got == expect
    assert [py_mix((n * GOLDEN) & M64) for n in range(3)] == expect


def test_words_follow_stream_definition():
    for seed, stream in [(0, 0), (1, 7), (2, 1_000_001)]:
        key = py_mix(seed ^ py_mix(stream))
        expect = [py_mix((key + c * GOLDEN) & M64) for c in range(16)]
        assert synth.words(seed, stream, 16).tolist() == expect


def test_golden_vectors():
    path = os.path.join(os.path.dirname(__file__), "golden", "synth_vectors.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    for seed, stream, *vals in rows:
        got = synth.normal_bf16(int(seed), int(stream), len(vals), std=0.02)
        assert [f"{v:04x}" for v in got] == vals


def test_normal_moments_and_box_muller():
    n = 1_000_000
    x = synth.normal_f32(3, 5, n, std=0.02).astype(np.float64)
    assert abs(x.mean()) < 3 * 0.02 / np.sqrt(n)
    assert abs(x.std() - 0.02) < 3 * 0.02 / np.sqrt(2 * n)
    assert abs(((x / 0.02) ** 4).mean() - 3.0) < 0.05           # Gaussian kurtosis
    # element 2p and 2p+1 are the cos and sin branch of one Box-Muller pair built from word p
    w = synth.words(3, 5, 4)
    u1 = ((w >> np.uint64(32)).astype(np.float64) + 0.5) / 2.0 ** 32
    u2 = ((w & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) / 2.0 ** 32
    r = np.sqrt(-2 * np.log(u1))
    expect = np.stack([r * np.cos(2 * np.pi * u2), r * np.sin(2 * np.pi * u2)], 1).reshape(-1) * 0.02
    np.testing.assert_allclose(x[:8], expect.astype(np.float32), rtol=1e-6)


def test_bf16_rounding_matches_library_conversion():
    f = synth.normal_f32(9, 9, 100_000, std=0.02)
    b = synth.normal_bf16(9, 9, 100_000, std=0.02)
    lib = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b, lib)
    assert np.array_equal(synth.bf16_bits_to_f32(b), torch.from_numpy(f).to(torch.bfloat16).float().numpy())


def test_uniform_ints_and_permutation():
    t = synth.tokens(0, 200_000, 1024)
    assert t.min() == 0 and t.max() == 1023
    counts = np.bincount(t, minlength=1024)
    assert abs(counts.mean() - 200_000 / 1024) < 1e-9 and counts.std() < 3 * np.sqrt(200_000 / 1024)
    p = synth.permutation(4, 4, 1000)
    assert sorted(p.tolist()) == list(range(1000)) and not np.array_equal(p, np.arange(1000))


def test_param_counts_and_blob_layout():
    assert synth.TINY.n_params() == 1_975_552
    assert synth.M1B.n_params() == 1_104_218_112
    assert synth.M8B.n_params() == 8_030_261_248
    entries, total = synth.blob_layout(synth.TINY)
    assert sum(r * c for _, _, r, c, _ in entries) == synth.TINY.n_params()
    offs = [e[1] for e in entries]
    assert all(o % 256 == 0 for o in offs) and offs == sorted(offs) and total % 256 == 0
    blob = synth.make_blob(synth.TINY, gain_std=0.1)
    assert blob.size == total
    w = synth.blob_tensor(synth.TINY, blob, "l1.wgu")
    assert w.shape == (2 * 688, 256) and abs(w.std() - 0.02) < 1e-3
    g = synth.blob_tensor(synth.TINY, blob, "final_norm")
    assert g.shape == (256,) and abs(g.mean() - 1) < 0.05 and g.std() > 0.05


def test_workload_recipes():
    w = synth.workload("tiny")
    assert w.batch == 4 and (w.prompt_lens == 128).all() and w.decode_steps == 16 and w.prompt_tokens.max() < 1024
    w = synth.workload("1b")
    assert w.batch == 32 and w.prompt_lens.min() >= 512 and w.prompt_lens.max() <= 2048 and w.decode_steps == 128
    w = synth.workload("8b")
    assert w.batch == 64 and w.prompt_lens.min() >= 16 and w.prompt_lens.max() <= 4096 and w.decode_steps == 256
    assert 900 < np.median(w.prompt_lens) < 1200
    a, b = synth.workload("duel_1b"), synth.workload("duel_8b")
    assert np.array_equal(a.prompt_tokens, b.prompt_tokens) and a.prompt_tokens.max() < 32000
    z = synth.lengths_zipf(2, 128, 1.2, 256, 16384)
    assert z.min() >= 256 and z.max() <= 16384


def test_block_tables():
    caps = [1, 16, 17, 100, 0]
    for permute in (False, True):
        t = synth.block_tables(5, caps, 64, 8, permute=permute)
        need = [1, 1, 2, 7, 0]
        used = []
        for b, nb in enumerate(need):
            assert (t[b, :nb] >= 0).all() and (t[b, nb:] == -1).all()
            used += t[b, :nb].tolist()
        assert len(set(used)) == len(used) and max(used) < 64
    assert np.array_equal(synth.block_tables(5, caps, 64, 8, permute=False)[3, :7], np.arange(4, 11))
    with pytest.raises(AssertionError):
        synth.block_tables(5, [16 * 65], 64, 100)
