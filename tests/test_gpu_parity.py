"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Bars: block-table / slot indexing bit-exact; max |dlogit| <= 3e-2 against the oracle; teacher-forced
greedy agreement >= 99 %.  KV pools start filled with NaN patterns, so any read of a slot the
library did not write shows up as a non-finite logit."""
import dataclasses

import numpy as np
import pytest

from paper_2603_20661_amd import synth
from helpers import GpuSession, compare, gpu_job, oracle_job

pytestmark = pytest.mark.gpu

TOL = 3e-2
AGREE = 0.99

MID128 = synth.ModelShape("mid128", 3, 512, 8, 2, 128, 1392, 2048, 1e-5, 5e5, synth.WDTYPE_BF16, seed=21)
MID64 = synth.ModelShape("mid64", 2, 256, 8, 4, 64, 704, 1024, 1e-5, 1e4, synth.WDTYPE_BF16, seed=22)
MIDF32 = dataclasses.replace(MID64, name="midf32", weight_dtype=synth.WDTYPE_F32, seed=23)


MIN_ROWS = 256   # logit rows per case: enough for the 99 % agreement bar to be a statement about a rate
WIDE_ROWS = 1024  # ... and for the full-width cases, whose logit errors (3e-3 .. 7e-3 over vocabularies of 32 000 and more) flip
                  # an exact near-tie of the oracle's two best logits in 0.2 - 0.3 % of the rows


def run_job(shape, lens, steps, seed, chunk=None, permute=True, gain_std=0.1, std=0.02, num_blocks=None, blob=None, max_batch=None,
            min_rows=MIN_ROWS):
    """`steps` is the least number of decode steps; more are taken until the case has `min_rows` logit rows."""
    lens = np.asarray(lens, np.int32)
    Bn = len(lens)
    steps = max(steps, -(-min_rows // Bn) - 1)
    cap = lens + steps + 1
    mbs = int((cap.max() + 15) // 16)
    need = int(((cap + 15) // 16).sum())
    num_blocks = num_blocks or need + 7
    blob = synth.make_blob(shape, std=std, gain_std=gain_std) if blob is None else blob
    toks = synth.tokens(seed, int(lens.sum()), shape.vocab)
    table = synth.block_tables(seed, cap, num_blocks, mbs, permute=permute)
    o_logits, o_tok = oracle_job(shape, blob, lens, toks, steps, table, num_blocks, chunk=chunk)
    sess = GpuSession(shape, blob, max_batch or Bn, mbs * 16, max(int(lens.sum()), 1), num_blocks)
    try:
        g_logits, g_tok = gpu_job(sess, lens, toks, steps, table, o_tok, chunk=chunk)
    finally:
        sess.close()
    return o_logits, o_tok, g_logits, g_tok


def check(res, what):
    """max |dlogit| <= 3e-2 and teacher-forced greedy agreement >= 99 %, both strict, on every case (each has at least
    MIN_ROWS logit rows); the tie-aware figure is printed for information only."""
    err, agree, tie = compare(*res)
    n = res[1].size
    print(f"{what}: max|dlogit|={err:.3e} agreement={agree:.4f} tie-aware={tie:.4f} samples={n}", flush=True)
    assert n >= MIN_ROWS, f"{what}: only {n} logit rows"
    assert err <= TOL, f"{what}: max |dlogit| {err}"
    assert agree >= AGREE, f"{what}: greedy agreement {agree}"


def test_slot_indexing_bit_exact():
    import torch
    from oracle import oracle as O
    from paper_2603_20661_amd import binding as B
    dev = torch.device("cuda:0")
    for seed, nblk in ((1, 64), (2, 200_000)):
        row = synth.permutation(seed, 77, nblk)[:50].astype(np.int32)
        if nblk > 1000:
            row[3] = 2_000_000_000 // 16                     # slot index beyond 32 bits
        pos = synth.uniform_i32(seed, 78, 300, 50 * 16)
        got = B.www_debug_slots(torch.from_numpy(row).to(dev), torch.from_numpy(pos).to(dev)).cpu().numpy()
        ref = np.array([O.slot(row, p) for p in pos], np.int64)
        assert np.array_equal(got, ref)


def test_decode_path_alone_token_by_token():
    """feeding a prompt one token at a time through www_decode_step == the oracle's prefill of the same tokens"""
    from oracle import oracle as O
    shape = MID64
    blob = synth.make_blob(shape, gain_std=0.1)
    Bn, n = 3, 37
    toks = synth.tokens(5, Bn * n, shape.vocab).reshape(Bn, n)
    table = synth.block_tables(5, [n] * Bn, 16, 3)
    sess = GpuSession(shape, blob, Bn, 48, 16, 16)
    m = O.OracleModel(shape, blob, num_blocks=16)
    try:
        worst, agree = 0.0, []
        for i in range(n):
            lens = np.full(Bn, i + 1, np.int32)
            g_lg, g_nx = sess.decode(toks[:, i], lens, table)
            o_lg, o_nx, _ = m.forward(toks[:, i], np.ones(Bn, np.int32), lens, block_table=table)
            assert np.isfinite(g_lg).all(), f"step {i}"
            worst = max(worst, float(np.abs(g_lg - o_lg).max()))
            agree.append(g_nx == o_nx)
        print(f"decode-only: max|dlogit|={worst:.3e} agreement={np.mean(agree):.4f}", flush=True)
        assert worst <= TOL and np.mean(agree) >= AGREE
    finally:
        sess.close()


def test_tiny_config_prefill_and_decode():
    wl = synth.workload("tiny")
    res = run_job(wl.shape, wl.prompt_lens, wl.decode_steps, seed=0, gain_std=0.0)
    check(res, "tiny")


@pytest.mark.parametrize("shape,lens,steps", [
    (MID64, [70, 1, 16, 300, 33], 6),
    (MID128, [129, 17, 64, 5, 260, 31, 2], 5),
    (MIDF32, [40, 90], 4),
])
def test_ragged_prefill_then_decode(shape, lens, steps):
    check(run_job(shape, lens, steps, seed=31), f"{shape.name} ragged")


@pytest.mark.parametrize("batch", [17, 33, 70])
def test_batch_sizes_cross_token_group_boundaries(batch):
    lens = 3 + synth.uniform_i32(batch, 9, batch, 40)
    check(run_job(MID64, lens, 3, seed=40 + batch), f"batch {batch}")


@pytest.mark.parametrize("batch", [20, 40])
def test_fp32_weights_at_two_and_four_token_groups(batch):
    """weights given in fp32 are carried as hi + lo planes (three MFMA passes); here with 2 and with 4 token groups per
    workgroup, the instantiations with the most live registers"""
    lens = 2 + synth.uniform_i32(batch, 9, batch, 30)
    check(run_job(MIDF32, lens, 3, seed=60 + batch), f"fp32 weights, batch {batch}")


def test_chunked_prefill_matches_oracle():
    check(run_job(MID128, [200, 75, 33], 3, seed=50, chunk=48), "chunked prefill (48)")


def test_long_context_many_splits():
    check(run_job(MID128, [1100, 520], 2, seed=60), "long context")


@pytest.mark.parametrize("hd", [64, 128])
@pytest.mark.parametrize("group", [1, 2, 4, 8])
def test_every_head_dim_and_group_size(hd, group):
    """each (head_dim, query heads per kv head) pair is its own instantiation of the attention kernels: run every one over
    contexts of one key pair, several pairs, and several splits plus the merge"""
    n_kv = 2 if group <= 4 else 1
    shape = synth.ModelShape(f"hd{hd}g{group}", 1, 256, n_kv * group, n_kv, hd, 352, 512, 1e-5, 1e4, synth.WDTYPE_BF16,
                             seed=100 + hd + group)
    check(run_job(shape, [1045, 3, 31, 530, 64], 3, seed=80 + group), shape.name)


def test_block_permutation_is_invisible_bitwise():
    """GPU vs GPU: identity and permuted block tables give bit-identical logits"""
    shape = MID128
    blob = synth.make_blob(shape, gain_std=0.1)
    a = run_job(shape, [150, 40, 9], 3, seed=70, permute=False, blob=blob, num_blocks=40)
    b = run_job(shape, [150, 40, 9], 3, seed=70, permute=True, blob=blob, num_blocks=40)
    assert np.array_equal(a[2], b[2])


# ------------------------------------------------------------------ full-width shapes (the launch configurations bench.py times)
WIDE8B = dataclasses.replace(synth.M8B, name="wide8b", n_layers=2, seed=31)
WIDE1B = dataclasses.replace(synth.M1B, name="wide1b", n_layers=2, seed=32)


@pytest.mark.parametrize("shape,batch", [(WIDE8B, 64), (WIDE1B, 32), (WIDE1B, 64)])
def test_full_width_layers_at_bench_batch(shape, batch):
    """every matrix has its full 8B / 1B size (same tiles, split-K factors and token groups as the benchmark);
    only the layer count is cut so the oracle finishes in about a minute.  The 1B-wide model at batch 64 is the case in
    which the gate/up GEMM runs with eight wavefronts per workgroup AND split over k (its 128 row tiles do not fill the
    device)."""
    lens = 1 + synth.uniform_i32(batch, 11, batch, 40)
    lens[0], lens[1] = 1, 16
    check(run_job(shape, lens, 3, seed=80 + batch, gain_std=0.05, min_rows=WIDE_ROWS), f"{shape.name} B={batch}")


# ------------------------------------------------------------------ models with normalised query / key heads
MID64_QKN = dataclasses.replace(MID64, name="mid64qkn", qk_norm=1, seed=41)
MID128_QKN = dataclasses.replace(MID128, name="mid128qkn", qk_norm=1, seed=42)
MIDF32_QKN = dataclasses.replace(MIDF32, name="midf32qkn", qk_norm=1, seed=43)
# one query head and one kv head of 64: 192 rows of wqkv, so the last 128-row tile of the decode GEMM and the only
# 256-row tile of the prefill GEMM end in the middle (the missing heads' sums must not leak into real ones)
ODD64_QKN = synth.ModelShape("odd64qkn", 2, 256, 1, 1, 64, 352, 512, 1e-5, 1e4, synth.WDTYPE_BF16, seed=44, qk_norm=1)
WIDE8B_QKN = dataclasses.replace(WIDE8B, name="wide8bqkn", qk_norm=1, seed=45)
WIDE1B_QKN = dataclasses.replace(WIDE1B, name="wide1bqkn", qk_norm=1, seed=46)


@pytest.mark.parametrize("shape,lens,steps,chunk", [
    (MID64_QKN, [70, 1, 16, 300, 33], 5, None),
    (MID128_QKN, [129, 17, 64, 5, 260, 31, 2], 4, 48),
    (MIDF32_QKN, [40, 90], 4, None),
    (ODD64_QKN, [50, 3, 270], 4, None),
    (dataclasses.replace(MID128_QKN, name="mid128qknfp8", weight_dtype=synth.WDTYPE_FP8WO), [129, 17, 64, 5], 4, None),
    (synth.ModelShape("q32hd64qkn", 2, 256, 8, 4, 64, 736, 1024, 1e-5, 1e4, synth.WDTYPE_INT4WO_32, seed=47, qk_norm=1), [129, 17, 64, 5], 4, None),
])
def test_models_with_normalised_query_and_key_heads(shape, lens, steps, chunk):
    """per-head RMS normalisation of q and k in front of the rotation, in the QKV epilogues of both GEMMs (gains drawn
    around 1 with spread 0.1, so a gain applied to the wrong row of a rotary pair shows)"""
    check(run_job(shape, lens, steps, seed=90, chunk=chunk), f"{shape.name}")


def test_normalised_heads_across_token_group_boundaries():
    lens = 3 + synth.uniform_i32(33, 9, 33, 40)
    check(run_job(MID64_QKN, lens, 3, seed=91), "mid64qkn batch 33")


@pytest.mark.parametrize("shape,batch", [(WIDE8B_QKN, 64), (WIDE1B_QKN, 32)])
def test_normalised_heads_full_width_layers(shape, batch):
    """the 8B- and 1B-wide matrices with the benchmark's tiles and split-K factors (the head sums cross the four
    wavefronts of the workgroup that finishes a split row tile)"""
    lens = 1 + synth.uniform_i32(batch, 11, batch, 40)
    lens[0], lens[1] = 1, 16
    check(run_job(shape, lens, 3, seed=92, gain_std=0.05, min_rows=WIDE_ROWS), f"{shape.name} B={batch}")


_DIGEST_JOB = r"""
import hashlib, sys
import numpy as np
sys.path.insert(0, {tests!r})
from paper_2603_20661_amd import synth
from helpers import GpuSession
from test_gpu_parity import WIDE1B
n_seq, plen, steps = 32, 768, 96
lens = np.full(n_seq, plen, np.int32)
toks = synth.tokens(12345, n_seq * plen, 32000)
blob = synth.make_blob(WIDE1B, gain_std=0.05)
cap = lens + steps + 1
mbs = int((cap.max() + 15) // 16)
nb = int(((cap + 15) // 16).sum()) + 11
table = synth.block_tables(8, cap, nb, mbs, permute=True)
sess = GpuSession(WIDE1B, blob, n_seq, mbs * 16, n_seq * plen, nb)
lg, nxt = sess.prefill(toks, lens, lens, table)
h = hashlib.sha256(lg.tobytes())
cur = lens.copy()
for _ in range(steps):
    cur = cur + 1
    lg, nxt = sess.decode(nxt, cur, table)
    h.update(lg.tobytes())
sess.close()
print("DIGEST", h.hexdigest())
"""


def test_fresh_processes_agree_bit_for_bit():
    """The same job (1B-wide layers, 32 x 768 prompt tokens, 96 greedy steps: every decode GEMM hands partial tiles from
    workgroup to workgroup) run by three separate, freshly started processes gives the same logits in every bit.  A
    hand-over that does not wait for its stores showed here and nowhere else: about once in twenty fresh processes."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = _DIGEST_JOB.format(tests=os.path.join(root, "tests"))
    digests = []
    for _ in range(3):
        out = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
        assert out.returncode == 0, out.stderr[-2000:]
        digests.append([line for line in out.stdout.splitlines() if line.startswith("DIGEST")][-1])
    assert len(set(digests)) == 1, digests


def test_results_do_not_depend_on_what_device_memory_held_before():
    """GPU vs GPU: the same job over memory that was filled with zeros, with ones (fp16 1.0 / fp32 0.0078) and with NaN
    patterns before the library got it (workspace, KV pool and blob buffer are carved out of the poisoned block) gives
    bit-identical logits: nothing reads a byte that the library or the caller has not written."""
    import torch
    shape = MID128
    blob = synth.make_blob(shape, gain_std=0.1)
    lens = np.array([150, 40, 9, 257], np.int32)
    steps = 3
    cap = lens + steps + 1
    mbs = int((cap.max() + 15) // 16)
    nb = int(((cap + 15) // 16).sum()) + 5
    toks = synth.tokens(71, int(lens.sum()), shape.vocab)
    table = synth.block_tables(71, cap, nb, mbs, permute=True)
    runs = []
    for pattern in (0, 0x3C00, 0x7FC0):
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        junk = torch.empty(1 << 29, dtype=torch.int16, device="cuda:0")     # 1 GiB, far more than the session needs
        junk.fill_(pattern)
        torch.cuda.synchronize()
        del junk                                                           # stays in the allocator's cache: the session reuses it
        sess = GpuSession(shape, blob, len(lens), mbs * 16, int(lens.sum()), nb, kv_poison=False)
        try:
            lg, nx = sess.prefill(toks, lens, lens, table)
            out, cur = [lg], lens.copy()
            for _ in range(steps):
                cur = cur + 1
                lg, nx = sess.decode(nx, cur, table)
                out.append(lg)
            runs.append(np.stack(out))
        finally:
            sess.close()
    assert np.isfinite(runs[0]).all()
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[0].view(np.uint32), runs[2].view(np.uint32))


# ------------------------------------------------------------------ the largest sizes a configuration may name
def test_widest_model_the_configuration_allows():
    """d_model 8192, the documented maximum: every one of the 64 entries per token of the decode path's sum-of-squares
    table and of the 32 of the prefill path's is in use, and the QKV matrix has 80 row tiles of 128"""
    shape = synth.ModelShape("max8192", 2, 8192, 64, 8, 128, 2048, 1024, 1e-5, 5e5, synth.WDTYPE_BF16, seed=51)
    lens = 1 + synth.uniform_i32(51, 11, 40, 30)
    lens[0], lens[1] = 300, 1
    check(run_job(shape, lens, 2, seed=93, gain_std=0.05, min_rows=WIDE_ROWS), "d_model 8192")


def test_largest_batch_the_configuration_allows():
    """1024 sequences in one prefill call and in every decode step (16 groups of 64 tokens per decode GEMM)"""
    lens = 1 + synth.uniform_i32(52, 11, 1024, 20)
    check(run_job(MID64, lens, 2, seed=94, min_rows=WIDE_ROWS), "batch 1024")


@pytest.mark.parametrize("shape", [WIDE1B, WIDE1B_QKN])
def test_batches_so_large_that_no_decode_gemm_splits_k(shape):
    """576 sequences on the 1B-wide layers: nine groups of 64 tokens times the row tiles of every matrix exceed the
    number of compute units, so the QKV, O and down GEMMs run without split-K and finish in their own epilogues (no
    hand-over), and the gate/up GEMM runs its eight-wavefront form once per token group"""
    lens = 1 + synth.uniform_i32(53, 11, 576, 6)
    check(run_job(shape, lens, 2, seed=95, gain_std=0.05, min_rows=WIDE_ROWS), f"{shape.name} batch 576")


# ------------------------------------------------------------------ fp8 weight-only models
MID128_FP8 = dataclasses.replace(MID128, name="mid128fp8", weight_dtype=synth.WDTYPE_FP8WO, seed=24)
MID64_FP8 = dataclasses.replace(MID64, name="mid64fp8", weight_dtype=synth.WDTYPE_FP8WO, seed=25)
WIDE8B_FP8 = dataclasses.replace(WIDE8B, name="wide8bfp8", weight_dtype=synth.WDTYPE_FP8WO, seed=33)
WIDE1B_FP8 = dataclasses.replace(WIDE1B, name="wide1bfp8", weight_dtype=synth.WDTYPE_FP8WO, seed=34)


@pytest.mark.parametrize("shape,lens,steps,chunk", [
    (MID64_FP8, [1, 17, 150, 40, 9], 6, None),            # token group of 16, ragged prompts
    (MID128_FP8, [200, 31, 64, 5, 90, 33, 16, 1] * 3, 5, None),   # 24 sequences: two token groups
    (MID128_FP8, [130, 47, 300], 4, 37),                   # chunked prefill
])
def test_fp8_weight_only_models(shape, lens, steps, chunk):
    """Weights stored as E4M3 codes with one scale per matrix: the decode path widens the codes in registers, the
    prefill path reads an fp16 copy; the oracle runs the decoded fp32 model.  Same bars as everywhere."""
    check(run_job(shape, lens, steps, seed=120 + len(lens), chunk=chunk, gain_std=0.1), f"{shape.name} lens={len(lens)} chunk={chunk}")


# int4 groups need ffn widths that are multiples of the group size
Q128_HD128 = synth.ModelShape("q128hd128", 3, 512, 8, 2, 128, 1408, 2048, 1e-5, 5e5, synth.WDTYPE_INT4WO_128, seed=26)
Q32_HD64 = synth.ModelShape("q32hd64", 2, 256, 8, 4, 64, 736, 1024, 1e-5, 1e4, synth.WDTYPE_INT4WO_32, seed=28)
WIDE8B_Q128 = dataclasses.replace(WIDE8B, name="wide8bq128", weight_dtype=synth.WDTYPE_INT4WO_128, seed=35)
WIDE1B_Q32 = dataclasses.replace(WIDE1B, name="wide1bq32", weight_dtype=synth.WDTYPE_INT4WO_32, seed=36)


@pytest.mark.parametrize("shape,lens,steps,chunk", [
    (Q32_HD64, [1, 17, 150, 40, 9], 6, None),
    (Q128_HD128, [200, 31, 64, 5, 90, 33, 16, 1] * 3, 5, None),
    (Q128_HD128, [130, 47, 300], 4, 37),
])
def test_int4_weight_only_models(shape, lens, steps, chunk):
    """Weights stored as 4-bit codes with a bf16 scale per group of 128 / 32: the decode path widens and scales the codes
    in registers, the prefill path reads an fp16 copy; the oracle runs the decoded fp32 model."""
    check(run_job(shape, lens, steps, seed=160 + len(lens), chunk=chunk, gain_std=0.1), f"{shape.name} lens={len(lens)} chunk={chunk}")


@pytest.mark.parametrize("shape,batch", [(WIDE8B_Q128, 64), (WIDE1B_Q32, 32), (WIDE8B_Q128, 70)])
def test_int4_weight_only_full_width_layers(shape, batch):
    lens = 1 + synth.uniform_i32(batch, 14, batch, 40)
    lens[0], lens[1] = 1, 16
    check(run_job(shape, lens, 3, seed=180 + batch, gain_std=0.05, min_rows=WIDE_ROWS), f"{shape.name} B={batch}")


@pytest.mark.parametrize("shape,batch", [(WIDE8B_FP8, 64), (WIDE1B_FP8, 32), (WIDE8B_FP8, 70), (WIDE1B_FP8, 64)])
def test_fp8_weight_only_full_width_layers(shape, batch):
    lens = 1 + synth.uniform_i32(batch, 13, batch, 40)
    lens[0], lens[1] = 1, 16
    check(run_job(shape, lens, 3, seed=140 + batch, gain_std=0.05, min_rows=WIDE_ROWS), f"{shape.name} B={batch}")


@pytest.mark.parametrize("fence,batch", [("0", 32), ("1", 32), ("0", 64)])
def test_repeated_calls_are_bitwise_identical(fence, batch, monkeypatch):
    """GPU vs GPU: the same decode step and the same prefill, issued again and again on one model, give the same bits.
    Split-K partial tiles travel between workgroups on different XCDs inside one kernel; a hand-over without a
    device-scope release showed up here as a few differing logits in a few per cent of the calls.  Both hand-over modes
    are run: the default (all splits of a row tile behind one L2, confirmed by a placement probe at load, no fence) and
    the fallback with the fence (WWW_HANDOVER_FENCE=1, read when a model is loaded)."""
    monkeypatch.setenv("WWW_HANDOVER_FENCE", fence)
    shape = WIDE1B
    lens = (1 + synth.uniform_i32(batch, 11, batch, 40)).astype(np.int32)
    cap = lens + 4
    mbs = int((cap.max() + 15) // 16)
    nb = int(((cap + 15) // 16).sum()) + 7
    blob = synth.make_blob(shape, gain_std=0.05)
    toks = synth.tokens(113, int(lens.sum()), shape.vocab)
    table = synth.block_tables(113, cap, nb, mbs, permute=True)
    sess = GpuSession(shape, blob, batch, mbs * 16, int(lens.sum()), nb)
    try:
        first, nxt = sess.prefill(toks, lens, lens, table)
        for rep in range(10):
            again, _ = sess.prefill(toks, lens, lens, table)
            assert np.array_equal(first.view(np.uint32), again.view(np.uint32)), f"prefill call {rep + 2} differs from the first"
        ref, _ = sess.decode(nxt, lens + 1, table)
        for rep in range(60):
            again, _ = sess.decode(nxt, lens + 1, table)
            assert np.array_equal(ref.view(np.uint32), again.view(np.uint32)), f"decode call {rep + 2} differs from the first"
    finally:
        sess.close()


def test_graph_replays_equal_eager_launches_bitwise(monkeypatch):
    """GPU vs GPU: a decode step replayed from its captured HIP graph gives the bits of the same step launched kernel by
    kernel (WWW_NO_GRAPH=1, read when a model is loaded), on every replay, with other work of the program (prefill calls,
    eager steps of the second model, synchronisations) between the replays and with the sequence lengths advancing in
    place in device memory."""
    shape = MID128
    lens = np.array([70, 5, 33, 129, 16, 250], np.int32)
    steps = 12
    cap = lens + steps + 1
    mbs = int((cap.max() + 15) // 16)
    nb = int(((cap + 15) // 16).sum()) + 5
    blob = synth.make_blob(shape, gain_std=0.1)
    toks = synth.tokens(131, int(lens.sum()), shape.vocab)
    table = synth.block_tables(131, cap, nb, mbs, permute=True)
    monkeypatch.setenv("WWW_NO_GRAPH", "1")
    eager = GpuSession(shape, blob, len(lens), mbs * 16, int(lens.sum()), nb)
    monkeypatch.delenv("WWW_NO_GRAPH")
    graph = GpuSession(shape, blob, len(lens), mbs * 16, int(lens.sum()), nb)
    try:
        import torch
        from paper_2603_20661_amd import binding as B
        outs = {}
        for name, sess in (("eager", eager), ("graph", graph)):
            lg, nxt = sess.prefill(toks, lens, lens, table)
            # fixed device arrays, updated in place, so that the graph session replays ONE captured step
            tok_dev, seq_dev, tab_dev = sess.dev_i32(nxt), sess.dev_i32(lens), sess.dev_i32(table)
            logits = torch.empty((len(lens), shape.vocab), dtype=torch.float32, device=sess.dev)
            rows = []
            for s in range(steps):
                with torch.cuda.stream(sess.stream):
                    seq_dev.add_(1)
                    B.www_decode_step(sess.model, tok_dev, seq_dev, tab_dev, logits, tok_dev, stream=sess.stream)
                sess.stream.synchronize()
                rows.append(logits.cpu().numpy().copy())
                if s % 3 == 1:                       # unrelated work between the replays
                    other = eager if sess is graph else graph
                    other.prefill(toks[:int(lens[0])], lens[:1], lens[:1], table[:1])
                    torch.cuda.synchronize()
            outs[name] = np.stack(rows)
            # the throw-away prefill calls above rewrote sequence 0's prompt positions with the same values: harmless
        assert np.isfinite(outs["graph"]).all()
        for s in range(steps):
            assert np.array_equal(outs["graph"][s].view(np.uint32), outs["eager"][s].view(np.uint32)), f"replay {s + 1} differs from the eager step"
    finally:
        eager.close()
        graph.close()


def test_block_boundaries_and_single_token_sequences():
    shape = MID128
    for lens in ([1], [15, 16, 17], [31, 32, 33, 1]):
        check(run_job(shape, lens, 18, seed=90 + len(lens), max_batch=8), f"lens {lens}")


def test_capacity_and_argument_errors_on_device():
    import torch
    from paper_2603_20661_amd import binding as B
    shape = MID64
    blob = synth.make_blob(shape)
    sess = GpuSession(shape, blob, max_batch=2, max_ctx=64, max_prefill_tokens=32, num_blocks=8)
    try:
        dev = sess.dev
        i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=dev)
        table = i32([[0, 1, 2, 3], [4, 5, 6, 7]])
        three = i32([[0, 1, 2, 3]] * 3)
        with pytest.raises(B.WwwError) as e:                                   # batch 3 > max_batch 2
            B.www_decode_step(sess.model, i32([1, 2, 3]), i32([1, 1, 1]), three, stream=sess.stream)
        assert e.value.code == B.E_CAPACITY
        with pytest.raises(B.WwwError) as e:                                   # 40 new tokens > max_prefill_tokens 32
            B.www_prefill(sess.model, i32([1] * 40), i32([20, 20]), i32([20, 20]), table, stream=sess.stream)
        assert e.value.code == B.E_CAPACITY
        with pytest.raises(B.WwwError) as e:                                   # fewer tokens than sequences
            B.www_prefill(sess.model, i32([1]), i32([1, 1]), i32([1, 1]), table, stream=sess.stream)
        assert e.value.code == B.E_INVALID_ARG
        # an empty batch is a no-op, and the model still works afterwards
        B.www_decode_step(sess.model, i32([]), i32([]), table[:0], stream=sess.stream)
        lg, nx = sess.decode([5, 6], [1, 1], table.cpu().numpy())
        assert np.isfinite(lg).all()
    finally:
        sess.close()


@pytest.mark.parametrize("name", ["8b", "1b", "8b-qknorm", "1b-qknorm"])
def test_bench_configuration_sampled_against_oracle(name):
    """The 8B- and 1B-shaped workloads exactly as bench.py launches them (8B: batch 64, 80 231 prompt tokens in one
    prefill call; 1B: batch 32, about 40 000 prompt tokens; then decode steps), at full depth.  Properties at full size:
    logits finite although the pool starts as NaN, bit-identical under a different physical block placement.  Sampled
    parity: the shortest sequence is recomputed alone by the oracle (prefill + 2 decode steps) and compared with its rows
    of the batched GPU run.  The "-qknorm" names are the same jobs on models with normalised query and key heads."""
    from oracle import oracle as O
    wl = synth.workload(name)
    shape, lens, toks = wl.shape, wl.prompt_lens.astype(np.int32), wl.prompt_tokens
    steps = 2
    Bn = wl.batch
    cap = lens + steps + 1
    mbs = int((cap.max() + 15) // 16)
    nblocks = int(((cap + 15) // 16).sum()) + 64
    blob = synth.make_blob(shape)
    b0 = int(np.argmin(lens))
    start = int(np.cumsum(lens)[b0] - lens[b0])
    # oracle on the sampled sequence
    m = O.OracleModel(shape, blob, num_blocks=(int(cap[b0]) + 15) // 16)
    tab1 = np.arange((int(cap[b0]) + 15) // 16, dtype=np.int32)[None]
    o_lg, o_nx, _ = m.forward(toks[start:start + lens[b0]], lens[b0:b0 + 1], lens[b0:b0 + 1], block_table=tab1)
    o_logits, o_next = [o_lg[0]], [int(o_nx[0])]
    for s in range(steps):
        ol, on, _ = m.forward([o_next[s]], [1], [int(lens[b0]) + s + 1], block_table=tab1)
        o_logits.append(ol[0])
        o_next.append(int(on[0]))
    m.close()
    # GPU, two placements of the same job; decode is teacher-forced for the sampled sequence, free-running for the rest
    results = []
    for placement in (0, 1):
        table = synth.block_tables(100 + placement, cap, nblocks, mbs, permute=True)
        sess = GpuSession(shape, blob, Bn, mbs * 16, int(lens.sum()), nblocks)
        try:
            lg, nx = sess.prefill(toks, lens, lens, table)
            out = [lg]
            cur = lens.copy()
            for s in range(steps):
                feed = nx.copy()
                feed[b0] = o_next[s]
                cur = cur + 1
                lg, nx = sess.decode(feed, cur, table)
                out.append(lg)
            results.append(np.stack(out))
        finally:
            sess.close()
    a, b = results
    assert np.isfinite(a).all()
    assert np.array_equal(a, b), "logits depend on the physical block placement"
    got = a[:, b0]
    ref = np.stack(o_logits)
    err = float(np.abs(got - ref).max())
    agree = float((got.argmax(-1) == ref.argmax(-1)).mean())
    print(f"{name} bench configuration, sequence {b0} (len {lens[b0]}): max|dlogit|={err:.3e} agreement={agree:.3f}", flush=True)
    assert err <= TOL and agree == 1.0


def test_values_close_to_the_fp16_limit():
    """Operands are IEEE fp16 and are clamped to +-65504 on conversion.  Here the value rows of every layer's QKV matrix are
    scaled by 2^14 (exact in bf16 and in fp16), so that the cached values (standard deviation 7 400, the largest of the
    117 000 about 30 000), the probabilities-times-values products and the attention output that feeds the O projection
    come close to that limit (checked on the packed operand the attention kernel wrote: within a factor of eight), and
    nothing is clamped: the result still matches the oracle, which has no such limit.  (RMSNorm makes the rest of the network indifferent to the scale of the residual stream.)"""
    import torch
    from paper_2603_20661_amd import binding as B
    shape = MID128
    blob = synth.make_blob(shape, gain_std=0.1).copy()
    entries, _ = synth.blob_layout(shape)
    qd, kd = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    for name, off, rows, cols, dt in entries:
        if name.endswith(".wqkv"):
            w = blob[off:off + rows * cols * 2].view(np.uint16).reshape(rows, cols)
            v = w[qd + kd:]
            v[(v & 0x7F80) != 0] += np.uint16(14 << 7)          # bf16: exponent + 14
    lens = np.array([150, 40, 1, 257], np.int32)
    res = run_job(shape, lens, 3, seed=72, blob=blob)
    check(res, "values near the fp16 limit")
    # the operand of the O projection as the attention kernels left it after one more decode step of a fresh session
    cap = lens + 2
    mbs = int((cap.max() + 15) // 16)
    nb = int(((cap + 15) // 16).sum()) + 3
    toks = synth.tokens(72, int(lens.sum()), shape.vocab)
    table = synth.block_tables(72, cap, nb, mbs, permute=True)
    sess = GpuSession(shape, blob, len(lens), mbs * 16, int(lens.sum()), nb)
    try:
        _, nx = sess.prefill(toks, lens, lens, table)
        sess.decode(nx, lens + 1, table)
        raw = B.www_debug_read(sess.model, 2, 16 * qd, stream=sess.stream).numpy()       # one token group: hi and lo planes
        halves = raw.view(np.float16).astype(np.float32)
        assert np.isfinite(halves).all()
        top = float(np.abs(halves).max())
        print(f"largest fp16 operand of the O projection: {top:.0f}", flush=True)
        assert 65504 / 8 < top < 65504
    finally:
        sess.close()
