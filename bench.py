#!/usr/bin/env python3
"""Benchmark of the MI355X inference hot path on one GPU.

One "step" is one pass of the whole path over one synthetic batch: a ragged prefill of all prompts
(one www_prefill call) followed by the workload's greedy decode steps (www_decode_step, replayed from
a HIP graph, tokens fed back on the device).  Prints ONE JSON line:

  value / metric      decode tokens per second over the timed steps (inputs resident in HBM)
  prefill_tokens_per_s prompt tokens per second of the prefill calls in the same steps
  roofline            dominant decode kernel: algorithmic HBM bytes per launch / its mean duration
                      (HIP events around every kernel of extra, untimed, eagerly launched steps)
  roofline_decode_step / roofline_prefill   whole-phase figures from the timed region
  cpu_baseline        the CPU oracle timed on a bounded sample of the same decode workload

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 8b|1b|tiny]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
CALIB_COPY_BYTES = 1 << 28  # size of the counter-calibration copy

# HBM traffic of the dominant decode kernel class (decode_attn_kernel + decode_attn_merge_kernel), from two
# `rocprofv3 --pmc` runs of this file (FETCH_SIZE, then WRITE_SIZE; profiles/decode_attention_8b_traffic.md).
# Counter units per launch, averaged over the 256 launches of those runs; scale = bytes per unit / 1024, from what the
# same counter read for the calibration copy above (131 087.7 units of FETCH_SIZE for 262 144 KiB read, 262 144.0 units
# of WRITE_SIZE for 262 144 KiB written); algorithmic bytes of those same launches for rescaling to another context.
# Valid only for the kernel sources it was taken with: reported as null when their hash differs.
TRAFFIC = {
    "workload": "8b", "kernel": "decode_attention",
    "fetch_units": 163128.2 + 1674.1, "write_units": 3112.9 + 1024.0,
    "fetch_scale": 262144.0 / 131087.7, "write_scale": 1.0,
    "algorithmic_bytes_of_measured_launches": 80383 * 4096,
    "sources": ("paper_2603_20661_amd/csrc/decode.hip", "paper_2603_20661_amd/csrc/common.h"),
    "sha256": "939c8bdcfbb2560336996ea8f70ec4bd146804aba225cc1811b9c390dd7182b3",
}


def measured_traffic(workload, kernel, algorithmic_bytes_per_launch):
    """HBM bytes per launch of `kernel` from the stored counter readings, rescaled linearly to this launch's algorithmic
    bytes (attention traffic is proportional to the context); None if there is no reading for this workload / kernel or the
    kernel sources have changed since it was taken."""
    import hashlib
    if workload != TRAFFIC["workload"] or kernel != TRAFFIC["kernel"]:
        return None
    h = hashlib.sha256()
    for f in TRAFFIC["sources"]:
        with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), f), "rb") as fh:
            h.update(fh.read())
    if h.hexdigest() != TRAFFIC["sha256"]:
        return None
    measured = (TRAFFIC["fetch_units"] * TRAFFIC["fetch_scale"] + TRAFFIC["write_units"] * TRAFFIC["write_scale"]) * 1024.0
    return int(round(measured * algorithmic_bytes_per_launch / TRAFFIC["algorithmic_bytes_of_measured_launches"]))
MFMA_PEAK_TFLOPS = 2500.0  # dense fp16 / bf16


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def decode_bytes_per_class(shape, ctx_lens, batch):
    """Algorithmic HBM bytes of ONE launch of each decode kernel class (weights streamed once, K and V of
    the real context once per kv head, outputs written once; activations are not counted)."""
    d, F, V, L = shape.d_model, shape.ffn_dim, shape.vocab, shape.n_layers
    QD, KD = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    kv_tok_layer = 2 * KD * 2
    return {
        "embed": batch * d * 2,
        "qkv_gemm": (QD + 2 * KD) * d * 2 + batch * kv_tok_layer,     # weights + this token's K/V write
        "decode_attention": float(np.sum(ctx_lens)) * kv_tok_layer,
        "o_gemm": d * QD * 2,
        "gate_up_gemm": 2 * F * d * 2,
        "down_gemm": d * F * 2,
        "lm_head_gemm": V * d * 2 + batch * V * 4,
        "argmax": batch * V * 4,
    }, {"embed": 1, "qkv_gemm": L, "decode_attention": L, "o_gemm": L, "gate_up_gemm": L, "down_gemm": L,
        "lm_head_gemm": 1, "argmax": 1}


def decode_step_bytes(shape, ctx_lens, batch):
    per, mult = decode_bytes_per_class(shape, ctx_lens, batch)
    return sum(per[k] * mult[k] for k in per if k != "argmax")


def prefill_flops(shape, lens):
    """Flops of the prefill as this method performs it: all layers' QKV projections and attention for every
    prompt token, O / gate-up / down projections for all layers but the last (the last layer's output is only
    needed at the final position), plus one full single-token pass and the output head per sequence."""
    d, F, V, L = shape.d_model, shape.ffn_dim, shape.vocab, shape.n_layers
    hd, Hq = shape.head_dim, shape.n_q_heads
    QD, KD = Hq * hd, shape.n_kv_heads * hd
    T, B = float(np.sum(lens)), len(lens)
    qkv = 2 * (QD + 2 * KD) * d
    rest = 2 * (d * QD + 3 * F * d)
    attn_layers = L - 1
    S = np.asarray(lens, np.float64)
    attn = 2 * Hq * hd * float(np.sum(S * S + S)) * attn_layers
    bulk = T * (qkv * L + rest * (L - 1)) + attn
    last = B * ((qkv + rest) * L + 2 * V * d) + 2 * 2 * Hq * hd * float(np.sum(S)) * L
    return bulk + last


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="8b", choices=["tiny", "1b", "8b"])
    ap.add_argument("--decode-steps", type=int, default=None, help="override the workload's decode steps (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (sequences are independent, nothing is sharded); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_20661_amd import binding as B
    from paper_2603_20661_amd import synth

    wl = synth.workload(args.workload)
    shape = wl.shape
    nsteps = wl.decode_steps if args.decode_steps is None else args.decode_steps
    lens = wl.prompt_lens.astype(np.int32)
    Bn, T = wl.batch, int(lens.sum())
    cap = lens + nsteps + 1
    mbs = int((cap.max() + 15) // 16)
    num_blocks = int(((cap + 15) // 16).sum()) + 64
    table = synth.block_tables(shape.seed, cap, num_blocks, mbs, permute=True)

    t0 = time.time()
    blob = synth.make_blob(shape)
    log(f"{wl.name}: weights {blob.size / 2**30:.2f} GiB generated in {time.time() - t0:.1f} s; batch {Bn}, prompt tokens {T}, "
        f"{nsteps} decode steps, {num_blocks} KV blocks")

    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()
    cfg = B.make_config(shape, Bn, mbs, T, num_blocks)
    with torch.cuda.stream(stream):
        blob_dev = torch.from_numpy(blob).to(dev)
        model = B.Model(cfg, blob_dev, stream=stream)
        stream.synchronize()
        del blob_dev
        torch.cuda.empty_cache()
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(dev)
        tok_dev, qlen_dev, table_dev = i32(wl.prompt_tokens), i32(lens), i32(table)
        lens0_dev = i32(lens)
        seq_dev = torch.empty_like(lens0_dev)
        cur_tok = torch.empty(Bn, dtype=torch.int32, device=dev)
        logits = torch.empty((Bn, shape.vocab), dtype=torch.float32, device=dev)
        ev = lambda: torch.cuda.Event(enable_timing=True)
        # a plain device copy of known size, outside the timed region: under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE`
        # its counter reading calibrates the counters of the library's kernels (bytes per counter unit)
        calib_src = torch.empty(CALIB_COPY_BYTES, dtype=torch.uint8, device=dev)
        calib_dst = torch.empty_like(calib_src)
        calib_src.fill_(1)
        calib_dst.copy_(calib_src)
        stream.synchronize()
        del calib_src, calib_dst

        def one_pass(timed):
            e0, e1, e2 = ev(), ev(), ev()
            seq_dev.copy_(lens0_dev)
            e0.record(stream)
            B.www_prefill(model, tok_dev, qlen_dev, seq_dev, table_dev, logits=None, next_tokens=cur_tok, stream=stream)
            e1.record(stream)
            for _ in range(nsteps):
                seq_dev.add_(1)                 # lengths advance on the device; block tables already cover them
                B.www_decode_step(model, cur_tok, seq_dev, table_dev, logits=logits, next_tokens=cur_tok, stream=stream)
            e2.record(stream)
            return e0, e1, e2

        for _ in range(args.warmup):
            one_pass(False)
        stream.synchronize()
        torch.cuda.synchronize()
        wall0 = time.time()
        evs = [one_pass(True) for _ in range(args.steps)]
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.time() - wall0
        pre_ms = sum(a.elapsed_time(b) for a, b, _ in evs)
        dec_ms = sum(b.elapsed_time(c) for _, b, c in evs)
        final_tokens = cur_tok.cpu().numpy()

        # per-kernel timing on extra eager steps at the workload's mid-decode context lengths
        kernels = {}
        mid_ctx = lens + nsteps // 2 + 1
        seq_dev.copy_(i32(mid_ctx))
        B.www_debug_profile(model, True)
        nprof = 3
        for _ in range(nprof):
            B.www_decode_step(model, cur_tok, seq_dev, table_dev, logits=logits, next_tokens=cur_tok, stream=stream)
        prof = B.www_debug_profile_read(model, stream=stream)
        B.www_debug_profile(model, False)
        per_bytes, _ = decode_bytes_per_class(shape, mid_ctx, Bn)
        for k, (ms, n) in prof.items():
            if n:
                avg = ms / n
                gbs = per_bytes[k] / (avg * 1e-3) / 1e9
                kernels[k] = {"launches_per_step": n // nprof, "avg_ms": round(avg, 5), "GBps": round(gbs, 1),
                              "ms_per_step": round(ms / nprof, 4)}
    assert np.isfinite(logits.cpu().numpy()).all(), "non-finite logits"

    dec_tok_s = Bn * nsteps * args.steps / (dec_ms * 1e-3) if nsteps else 0.0
    pre_tok_s = T * args.steps / (pre_ms * 1e-3)
    # average algorithmic bytes of a decode step over the run (context grows by one token per step)
    step_bytes = float(np.mean([decode_step_bytes(shape, lens + s + 1, Bn) for s in range(max(nsteps, 1))]))
    step_ms = dec_ms / (args.steps * max(nsteps, 1))
    step_gbs = step_bytes / (step_ms * 1e-3) / 1e9
    pf = prefill_flops(shape, lens)
    pre_tflops = pf * args.steps / (pre_ms * 1e-3) / 1e12

    dom = max((k for k in kernels if k != "argmax"), key=lambda k: kernels[k]["ms_per_step"]) if kernels else None
    roofline = None
    if dom:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(kernels[dom]["GBps"] / HBM_PEAK_GBS, 4),
                    "traffic": measured_traffic(args.workload, dom, per_bytes[dom]),
                    "algorithmic_bytes_per_launch": int(per_bytes[dom]), "avg_launch_ms": kernels[dom]["avg_ms"]}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(shape, blob, lens, nsteps)

    out = {
        "metric": "decode_tokens_per_s", "value": round(dec_tok_s, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round((pre_ms + dec_ms) / args.steps, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{wl.name}-shaped decoder, batch {Bn}, prompts {int(lens.min())}..{int(lens.max())} tokens "
                               f"(sum {T}), {nsteps} greedy decode steps, KV block 16, random-init weights seed {shape.seed}"},
        "prefill_tokens_per_s": round(pre_tok_s, 1),
        "decode_ms_per_token_step": round(step_ms, 4),
        "prefill_ms": round(pre_ms / args.steps, 3),
        "roofline": roofline,
        "roofline_decode_step": {"bound": "hbm", "achieved": round(step_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": round(step_gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes_per_step": int(step_bytes)},
        "roofline_prefill": {"bound": "mfma", "achieved": round(pre_tflops, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": round(pre_tflops / MFMA_PEAK_TFLOPS, 4), "algorithmic_flops": pf},
        "decode_kernels": kernels,
        "cpu_baseline": cpu,
        "wall_s_timed_region": round(wall, 3),
        "checksum_last_tokens": int(final_tokens.astype(np.int64).sum()),
    }
    print(json.dumps(out), flush=True)
    model.close()


def cpu_baseline(shape, blob, lens, nsteps):
    """The CPU oracle, untuned, on a bounded sample: ONE decode step of the first `n` sequences at their first
    decode-step context lengths.  Its KV cache is pre-filled with seeded N(0,1) values instead of running the
    prompt through the CPU (same work per step, different values)."""
    from oracle import oracle as O
    from paper_2603_20661_amd import synth
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
    per_tok_flops = 2.0 * (shape.n_params() - shape.vocab * shape.d_model)
    n = int(max(1, min(len(lens), 25.0 * 3e9 * threads / per_tok_flops)))   # ~25 s at ~3 GFLOP/s per thread
    ctx = lens[:n] + 1
    mbs = int((ctx.max() + 15) // 16)
    nb = int(((ctx + 15) // 16).sum())
    table = synth.block_tables(7, ctx, nb, mbs, permute=True)
    m = O.OracleModel(shape, blob, num_blocks=nb)
    pool = m.kv_paged().reshape(-1)
    tile = synth.normal_f32(99, 1, min(pool.size, 1 << 24))
    for at in range(0, pool.size, tile.size):
        k = min(tile.size, pool.size - at)
        pool[at:at + k] = tile[:k]
    toks = synth.tokens(99, n, shape.vocab)
    t0 = time.time()
    m.forward(toks, np.ones(n, np.int32), ctx, block_table=table)
    dt = time.time() - t0
    m.close()
    return {"value": round(n / dt, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"1 decode step of the first {n} sequences (context {int(ctx.min())}..{int(ctx.max())}), KV pre-filled with "
                      f"seeded N(0,1) values, {dt:.1f} s"}


if __name__ == "__main__":
    main()
