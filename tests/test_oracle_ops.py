"""Pins for the oracle's elementary operations: closed forms, invariants, library routines.

Each check is something other than the oracle's own formula retyped: an invariant of the
mathematics, a closed form for a special input, or a PyTorch/NumPy library routine in fp64.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as O
from paper_2603_20661_amd import synth

rng = np.random.default_rng(0)


# ------------------------------------------------------------------ softmax
def test_softmax_rows_sum_to_one_and_shift_invariance():
    for n in (1, 2, 17, 1000):
        s = rng.normal(size=n).astype(np.float32) * 3
        p = O.softmax(s)
        assert abs(p.astype(np.float64).sum() - 1) <= 1e-6 and (p >= 0).all()
        p2 = O.softmax(s + np.float32(8.0))       # exact shift in fp32 for these magnitudes is not guaranteed,
        np.testing.assert_allclose(p2, p, rtol=2e-6, atol=1e-9)   # so compare to rounding
    assert np.array_equal(O.softmax(np.full(64, 3.25, np.float32)), np.full(64, 1 / 64, np.float32))
    big = O.softmax(np.array([1000.0, 0.0, -1000.0], np.float32))     # no overflow
    assert big.tolist() == [1.0, 0.0, 0.0]


def test_softmax_vs_library():
    s = rng.normal(size=333).astype(np.float32) * 4
    ref = torch.softmax(torch.from_numpy(s).double(), 0).numpy()
    np.testing.assert_allclose(O.softmax(s), ref, rtol=1e-6, atol=1e-12)


# ------------------------------------------------------------------ attention of one query
def test_attention_single_key_returns_its_value_exactly():
    for hd in (16, 64, 128):
        q, k, v = (rng.normal(size=hd).astype(np.float32) for _ in range(3))
        assert np.array_equal(O.attend(q, k[None], v[None]), v)


def test_attention_equal_scores_give_mean_of_values():
    hd, n = 64, 40
    q = np.zeros(hd, np.float32)
    K = rng.normal(size=(n, hd)).astype(np.float32)
    V = rng.normal(size=(n, hd)).astype(np.float32)
    np.testing.assert_allclose(O.attend(q, K, V), V.astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)


def test_attention_vs_library_sdpa():
    for hd, n in ((64, 1), (64, 37), (128, 300)):
        q = rng.normal(size=hd).astype(np.float32)
        K = rng.normal(size=(n, hd)).astype(np.float32)
        V = rng.normal(size=(n, hd)).astype(np.float32)
        ref = F.scaled_dot_product_attention(torch.from_numpy(q).double()[None, None, None],
                                             torch.from_numpy(K).double()[None, None],
                                             torch.from_numpy(V).double()[None, None])[0, 0, 0].numpy()
        np.testing.assert_allclose(O.attend(q, K, V), ref, rtol=2e-6, atol=1e-7)


def test_attention_key_value_pairing_and_scale():
    # two keys: the output must be the convex combination with weight sigmoid((q.k0 - q.k1)/sqrt(hd))
    hd = 16
    q = rng.normal(size=hd).astype(np.float32)
    K = rng.normal(size=(2, hd)).astype(np.float32)
    V = rng.normal(size=(2, hd)).astype(np.float32)
    d = (q.astype(np.float64) @ (K[0] - K[1]).astype(np.float64)) / 4.0
    w0 = 1 / (1 + np.exp(-d))
    np.testing.assert_allclose(O.attend(q, K, V), w0 * V[0] + (1 - w0) * V[1], rtol=2e-6, atol=1e-7)


# ------------------------------------------------------------------ rotary embedding
@pytest.mark.parametrize("hd,theta", [(64, 1e4), (128, 5e5)])
def test_rope_invariants(hd, theta):
    x = rng.normal(size=hd).astype(np.float32)
    assert np.array_equal(O.rope(x, 0, theta), x)
    for p in (1, 17, 4095, 16383):
        y = O.rope(x, p, theta)
        assert abs(np.linalg.norm(y.astype(np.float64)) / np.linalg.norm(x.astype(np.float64)) - 1) < 1e-6
        # pairs are (i, i + hd/2): each pair's own norm is preserved
        half = hd // 2
        np.testing.assert_allclose(np.hypot(y[:half], y[half:]), np.hypot(x[:half], x[half:]), rtol=1e-5)
        # theta_0 = 1: pair 0 turns by exactly p radians
        c, s = np.cos(float(p)), np.sin(float(p))
        np.testing.assert_allclose([y[0], y[half]], [x[0] * c - x[half] * s, x[half] * c + x[0] * s], rtol=1e-5, atol=1e-6)


def test_rope_is_complex_multiplication():
    hd, theta, p = 128, 5e5, 777
    x = rng.normal(size=hd).astype(np.float32)
    half = hd // 2
    z = x[:half].astype(np.float64) + 1j * x[half:].astype(np.float64)
    w = z * np.exp(1j * p * theta ** (-np.arange(half) * 2.0 / hd))
    y = O.rope(x, p, theta)
    np.testing.assert_allclose(y[:half], w.real, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(y[half:], w.imag, rtol=1e-5, atol=1e-6)


def test_rope_scores_depend_on_relative_position_only():
    hd, theta = 64, 1e4
    q, k = rng.normal(size=hd).astype(np.float32), rng.normal(size=hd).astype(np.float32)
    base = O.rope(q, 40, theta).astype(np.float64) @ O.rope(k, 33, theta).astype(np.float64)
    for c in (1, 100, 3000):
        s = O.rope(q, 40 + c, theta).astype(np.float64) @ O.rope(k, 33 + c, theta).astype(np.float64)
        assert abs(s - base) < 1e-5 * max(1, abs(base)) + 2e-5
    other = O.rope(q, 41, theta).astype(np.float64) @ O.rope(k, 33, theta).astype(np.float64)
    assert abs(other - base) > 1e-3       # and they do depend on it


# ------------------------------------------------------------------ RMSNorm, SiLU
def test_rmsnorm_closed_forms_and_library():
    d = 256
    ones = np.ones(d, np.float32)
    np.testing.assert_allclose(O.rmsnorm(ones, ones, 0.0), ones, rtol=1e-7)
    np.testing.assert_allclose(O.rmsnorm(3 * ones, ones, 1e-5), np.full(d, 3 / np.sqrt(9 + 1e-5)), rtol=1e-6)
    x = rng.normal(size=d).astype(np.float32)
    y = O.rmsnorm(x, ones, 0.0)
    assert abs(np.sqrt((y.astype(np.float64) ** 2).mean()) - 1) < 1e-6           # unit RMS
    np.testing.assert_allclose(O.rmsnorm(7.5 * x, ones, 0.0), y, rtol=1e-6)       # scale invariance
    g = rng.normal(size=d).astype(np.float32)
    ref = F.rms_norm(torch.from_numpy(x).double(), (d,), torch.from_numpy(g).double(), eps=1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), ref, rtol=1e-6, atol=1e-8)


def test_silu_mul():
    z = np.array([0.0, 30.0, -30.0, 1.0], np.float32)
    a = O.silu_mul(z, np.ones(4, np.float32))
    assert a[0] == 0.0 and abs(a[1] - 30.0) < 1e-5 and abs(a[2]) < 1e-10
    assert abs(a[3] - 1 / (1 + np.exp(-1.0))) < 1e-7
    g, u = rng.normal(size=1000).astype(np.float32), rng.normal(size=1000).astype(np.float32)
    ref = (F.silu(torch.from_numpy(g).double()) * torch.from_numpy(u).double()).numpy()
    np.testing.assert_allclose(O.silu_mul(g, u), ref, rtol=1e-6, atol=1e-9)


# ------------------------------------------------------------------ projections, argmax, slots
def test_matmul_vs_library_and_orientation():
    T, N, K = 5, 7, 33
    x = rng.normal(size=(T, K)).astype(np.float32)
    w = rng.normal(size=(N, K)).astype(np.float32)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    np.testing.assert_allclose(O.matmul(x, w, 0), ref, rtol=1e-6, atol=1e-6)
    # identity weights return the input, one-hot rows pick columns: catches a transposed operand
    assert np.array_equal(O.matmul(x, np.eye(K, dtype=np.float32), 0), x)
    pick = np.zeros((2, K), np.float32); pick[0, 3] = 1; pick[1, 30] = 1
    assert np.array_equal(O.matmul(x, pick, 0), x[:, [3, 30]])
    wb = synth.normal_bf16(1, 1, N * K, std=0.02).reshape(N, K)
    refb = F.linear(torch.from_numpy(x).double(), torch.from_numpy(wb.view(np.int16)).view(torch.bfloat16).double()).numpy()
    np.testing.assert_allclose(O.matmul(x, wb, 1), refb, rtol=1e-6, atol=1e-8)


def test_argmax_lowest_index_wins_ties():
    assert O.argmax(np.array([1, 5, 5, 2], np.float32)) == 1
    assert O.argmax(np.array([-1, -1], np.float32)) == 0
    x = rng.normal(size=5000).astype(np.float32)
    assert O.argmax(x) == int(np.argmax(x))


def test_slot_mapping_brute_force():
    # lay tokens into a pool by walking the table block by block; slot() must find each of them
    table = np.array([5, 0, 9, 2, -1, -1], np.int32)
    n = 16 * 3 + 7
    pool = np.full(10 * 16, -1, np.int64)
    pos = 0
    for blk in table:
        for s in range(16):
            if pos < n:
                pool[blk * 16 + s] = pos
                pos += 1
    for p in range(n):
        assert pool[O.slot(table, p)] == p
    # 64-bit: a block id whose byte offset overflows 32 bits still maps exactly
    big = np.array([2_000_000_000 // 16 * 9], np.int32)
    assert O.slot(big, 3) == int(big[0]) * 16 + 3
