#!/usr/bin/env python3
"""Benchmark of the MI355X inference hot path on one GPU.

One "step" is one pass of the whole path over one synthetic batch: a ragged prefill of all prompts
(one www_prefill call) followed by the workload's greedy decode steps (www_decode_step, replayed from
a HIP graph, tokens fed back on the device).  Prints ONE JSON line:

  value / metric      decode tokens per second over the timed steps (inputs resident in HBM)
  prefill_tokens_per_s prompt tokens per second of the prefill calls in the same steps
  roofline            dominant decode kernel: algorithmic HBM bytes per launch / its mean duration
                      (HIP events around every kernel of extra, untimed, eagerly launched steps)
                      (event_pair_floor_ms: what an event pair around a near-empty kernel reads in a busy stream, for
                      information; whole_step_frac repeats roofline_decode_step.frac, the figure the target is about)
  roofline_decode_step / roofline_prefill   whole-phase figures from the timed region
  measured_copy_bandwidth   read + written bytes per second of a plain 1 GiB device copy on the same stream: the achievable
                      figure beside the published peak (roofline_decode_step.frac_of_measured_copy relates the step to it)
  cpu_baseline        the CPU oracle timed on a bounded sample of the same decode workload

Two composite workloads print the same kind of line with their own phases:
  --workload duel    one duel-and-judge round (Sec. 4.2): 32 prompts of 768 tokens answered with 256 greedy tokens by a
                     1B-shaped and an 8B-shaped model resident together, then the 8B-shaped judge's prefill over
                     prompt + answer A + answer B and the votes read off its logits; the five phases are timed
                     separately, `value` is the round's time; the duels are then settled in the credit ledger
  --workload mixed   128 sequences with Zipf(1.2) lengths in [256, 16384] on the 8B-shaped model: 512-token prefill chunks
                     (8192-token budget per call) interleaved with decode steps over the sequences whose prompt is
                     complete, block tables scattered over a KV pool of 90 % of the memory left beside the weights;
                     `value` is the schedule's wall time, the two call classes are reported beside it

  --workload 8b-fp8wo / 1b-fp8wo   the 8B / 1B jobs with the matrices stored as FP8 E4M3 codes (weight-only; arithmetic
                     and activations unchanged); rooflines count one byte per streamed weight
  --workload 8b-int4wo128 / 8b-int4wo32 / 1b-...   the same with 4-bit codes and a bf16 scale per group of 128 / 32
  --workload 8b-qknorm / 1b-qknorm   the same jobs on a model whose query and key heads are RMS-normalised before the rotation

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 8b|1b|tiny|duel|mixed|8b-fp8wo|8b-int4wo128|...]
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

# HBM traffic of the decode kernel classes, from two `rocprofv3 --pmc` runs of this file (FETCH_SIZE, then WRITE_SIZE;
# profiles/decode_kernels_8b_traffic.md).  Counter units per launch, averaged over the 256 launches per class of those runs
# (8 for the output head); scale = KiB per unit, from what the same counter read for the calibration copy above (131 087.1
# units of FETCH_SIZE for 262 144 KiB read, 262 144.0 units of WRITE_SIZE for 262 144 KiB written).  The attention
# reading is rescaled linearly to the reported launch's context (its traffic is proportional to it); the GEMMs' bytes do
# not depend on the step.  Valid only for the kernels it was taken with: the hash covers the text of decode.hip and
# common.h; every reading is reported as null when that text has changed.
TRAFFIC = {
    "workload": "8b",
    "fetch_scale": 262144.0 / 131087.1, "write_scale": 1.0,
    "classes": {   # class: (FETCH_SIZE units, WRITE_SIZE units, algorithmic bytes of the measured launches or None = this run's)
        "decode_attention": (165304.6 + 1669.0, 3107.2 + 1024.0, 80383 * 4160),
        "qkv_gemm": (32960.2, 9513.0, None),
        "o_gemm": (25222.0, 10313.0, None),
        "gate_up_gemm": (118939.6, 3584.0, None),
        "down_gemm": (76424.4, 10313.0, None),
        "lm_head_gemm": (529392.8, 32068.2, None),
    },
    "sources": ("paper_2603_20661_amd/csrc/decode.hip", "paper_2603_20661_amd/csrc/common.h"),
    "sha256": "342b09e6dd9f9cefa0e384a9223eea53e53d2bd049cfa55c14bb3eb7a7807254",
}


def kernel_text_hash():
    """sha256 over the source text of the measured kernels"""
    import hashlib
    h = hashlib.sha256()
    for f in TRAFFIC["sources"]:
        with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def measured_traffic(workload, kernel, algorithmic_bytes_per_launch):
    """HBM bytes per launch of a decode kernel class from the stored counter readings (the attention class rescaled
    linearly to this launch's algorithmic bytes); None if there is no reading for this workload / class or the kernel
    sources have changed since it was taken."""
    if workload != TRAFFIC["workload"] or kernel not in TRAFFIC["classes"]:
        return None
    try:
        if kernel_text_hash() != TRAFFIC["sha256"]:
            return None
    except OSError:
        return None
    fetch, write, alg_measured = TRAFFIC["classes"][kernel]
    measured = (fetch * TRAFFIC["fetch_scale"] + write * TRAFFIC["write_scale"]) * 1024.0
    if alg_measured:
        measured *= algorithmic_bytes_per_launch / alg_measured
    return int(round(measured))


MFMA_PEAK_TFLOPS = 2500.0  # dense fp16 / bf16


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def decode_bytes_per_class(shape, ctx_lens, batch):
    """Algorithmic HBM bytes of ONE launch of each decode kernel class (weights streamed once, K and V of
    the real context once per kv head, outputs written once; activations are not counted)."""
    d, F, V, L = shape.d_model, shape.ffn_dim, shape.vocab, shape.n_layers
    QD, KD = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    kv_tok_layer = 2 * shape.n_kv_heads * (shape.head_dim * 2 + 4)   # 16-bit codes plus one fp32 scale per (kv head, K|V)
    # bytes per streamed weight: 16-bit, FP8 codes, or 4-bit codes plus a bf16 scale per group of 128 / 32
    wb = {0: 2, 1: 2, 2: 1, 3: 0.5 + 2 / 128, 4: 0.5 + 2 / 32}[shape.weight_dtype]
    return {
        "embed": batch * d * 2,
        "qkv_gemm": (QD + 2 * KD) * d * wb + batch * kv_tok_layer,     # weights + this token's K/V write
        "decode_attention": float(np.sum(ctx_lens)) * kv_tok_layer,
        "o_gemm": d * QD * wb,
        "gate_up_gemm": 2 * F * d * wb,
        "down_gemm": d * F * wb,
        "lm_head_gemm": V * d * wb + batch * V * 4,
        "argmax": batch * V * 4,
    }, {"embed": 1, "qkv_gemm": L, "decode_attention": L, "o_gemm": L, "gate_up_gemm": L, "down_gemm": L,
        "lm_head_gemm": 1, "argmax": 1}


def decode_step_bytes(shape, ctx_lens, batch):
    per, mult = decode_bytes_per_class(shape, ctx_lens, batch)
    return float(sum(per[k] * mult[k] for k in per if k != "argmax"))


def prefill_call_flops(shape, q_lens, seq_lens):
    """Flops of one www_prefill call as this method performs it, over chunks of q new tokens whose sequences then hold seq
    tokens (cached prefix P = seq - q): all layers' QKV projections and attention (prefix plus the chunk's own causal
    triangle) for every new token, O / gate-up / down projections for all layers but the last (the last layer's output
    is only needed at a chunk's final position), plus one full single-token pass and the output head per sequence."""
    d, F, V, L = shape.d_model, shape.ffn_dim, shape.vocab, shape.n_layers
    hd, Hq = shape.head_dim, shape.n_q_heads
    QD, KD = Hq * hd, shape.n_kv_heads * hd
    q = np.asarray(q_lens, np.float64)
    P = np.asarray(seq_lens, np.float64) - q
    T, B = float(q.sum()), len(q)
    qkv = 2 * (QD + 2 * KD) * d
    rest = 2 * (d * QD + 3 * F * d)
    attn = 2 * Hq * hd * float(np.sum(q * (2 * P + q + 1))) * (L - 1)
    bulk = T * (qkv * L + rest * (L - 1)) + attn
    last = B * ((qkv + rest) * L + 2 * V * d) + 2 * 2 * Hq * hd * float(np.sum(P + q)) * L
    return bulk + last


def prefill_flops(shape, lens):
    """Flops of a prefill of whole prompts (no cached prefix)."""
    return prefill_call_flops(shape, lens, lens)


def _common_fields(args, workload_text):
    return {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
            "data": "synthetic", "config": {"workload": workload_text}}


def bench_duel(args):
    """One duel-and-judge round (Sec. 4.2): two executors answer the same prompts, the judge reads both answers."""
    import torch
    from paper_2603_20661_amd import binding as B
    from paper_2603_20661_amd import synth

    n_seq, plen = 32, 768
    nsteps = 256 if args.decode_steps is None else args.decode_steps
    jlen = plen + 2 * nsteps
    lens = np.full(n_seq, plen, np.int32)
    prompts = synth.tokens(12345, n_seq * plen, 32000).reshape(n_seq, plen)     # ids valid for both vocabularies
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    execs = {}
    with torch.cuda.stream(stream):
        for name, shape in (("1b", synth.M1B), ("8b", synth.M8B)):
            t0 = time.time()
            blob = synth.make_blob(shape)
            log(f"duel: {name} weights {blob.size / 2**30:.2f} GiB generated in {time.time() - t0:.1f} s")
            cap = [plen + nsteps + 1] * n_seq + ([jlen] * n_seq if name == "8b" else [])   # the 8B model is also the judge
            cap = np.asarray(cap, np.int64)
            mbs = int((cap.max() + 15) // 16)
            nb = int(((cap + 15) // 16).sum()) + 64
            table = synth.block_tables(shape.seed, cap, nb, mbs, permute=True)
            cfg = B.make_config(shape, n_seq, mbs, n_seq * max(plen, jlen if name == "8b" else 0), nb)
            blob_dev = torch.from_numpy(blob).to(dev)
            model = B.Model(cfg, blob_dev, stream=stream)
            stream.synchronize()
            del blob_dev, blob
            torch.cuda.empty_cache()
            execs[name] = {"shape": shape, "model": model, "table": i32(table[:n_seq]), "judge_table": i32(table[n_seq:]),
                           "answers": torch.zeros((nsteps, n_seq), dtype=torch.int32, device=dev),
                           "cur": torch.empty(n_seq, dtype=torch.int32, device=dev),
                           "logits": torch.empty((n_seq, shape.vocab), dtype=torch.float32, device=dev)}
        prompts_dev, lens_dev, seq_dev = i32(prompts), i32(lens), i32(lens)
        jl_dev = i32(np.full(n_seq, jlen))
        judge_logits = execs["8b"]["logits"]
        judge_next = torch.empty(n_seq, dtype=torch.int32, device=dev)
        votes_dev = torch.empty(n_seq, dtype=torch.int32, device=dev)
        vote_tokens = (32, 33)   # the two designated ids whose last-position logits decide a vote (any two distinct ids)

        def one_round():
            marks = [ev()]
            marks[0].record(stream)
            for name in ("1b", "8b"):
                x = execs[name]
                seq_dev.copy_(lens_dev)
                B.www_prefill(x["model"], prompts_dev.view(-1), lens_dev, seq_dev, x["table"], logits=None, next_tokens=x["cur"], stream=stream)
                marks.append(ev()); marks[-1].record(stream)
                for s in range(nsteps):
                    x["answers"][s].copy_(x["cur"])         # the answer leaves the loop token by token
                    seq_dev.add_(1)
                    B.www_decode_step(x["model"], x["cur"], seq_dev, x["table"], logits=x["logits"], next_tokens=x["cur"], stream=stream)
                marks.append(ev()); marks[-1].record(stream)
            judge_in = torch.cat([prompts_dev, execs["1b"]["answers"].t(), execs["8b"]["answers"].t()], dim=1).contiguous()
            B.www_prefill(execs["8b"]["model"], judge_in.view(-1), jl_dev, jl_dev, execs["8b"]["judge_table"], logits=judge_logits,
                          next_tokens=judge_next, stream=stream)
            B.www_judge_verdict(judge_logits, vote_tokens[0], vote_tokens[1], votes_dev, None, stream=stream)
            marks.append(ev()); marks[-1].record(stream)
            return marks

        for _ in range(args.warmup):
            one_round()
        stream.synchronize()
        torch.cuda.synchronize()
        wall0 = time.time()
        rounds = [one_round() for _ in range(args.steps)]
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.time() - wall0
        ms = np.array([[a.elapsed_time(b) for a, b in zip(m[:-1], m[1:])] for m in rounds]).mean(axis=0)
        assert torch.isfinite(judge_logits).all(), "non-finite judge logits"
        checksum = int(judge_next.cpu().numpy().astype(np.int64).sum())
        votes = votes_dev.cpu().numpy()
    # settle the round's 32 duels in the credit ledger (host side, outside the timed region): node 0 ran the 1B executor,
    # node 1 the 8B executor, node 2 the judge
    ledger = B.Ledger([100.0, 100.0, 100.0], base_reward=1.0, duel_reward=0.5, duel_penalty=0.5, judge_reward=0.1)
    for r in range(n_seq):
        ledger.serve(r, 0)
        ledger.serve(r, 1)
        ledger.duel(r, 0, 1, [2], [int(votes[r])])
    settled = {"votes_for_second_executor": int(votes.sum()), "ledger_operations": len(ledger.ops()), "stakes_after": ledger.stakes()}
    ledger.close()

    phases = {}
    for k, name in enumerate(("1b", "8b")):
        shape = execs[name]["shape"]
        pre, dec = float(ms[2 * k]), float(ms[2 * k + 1])
        pf = prefill_flops(shape, lens)
        step_bytes = float(np.mean([decode_step_bytes(shape, lens + s + 1, n_seq) for s in range(max(nsteps, 1))]))
        gbs = step_bytes * nsteps / (dec * 1e-3) / 1e9 if nsteps else 0.0
        phases[f"executor_{name}_prefill"] = {"ms": round(pre, 3), "tokens_per_s": round(n_seq * plen / (pre * 1e-3), 1),
                                              "TFLOPs": round(pf / (pre * 1e-3) / 1e12, 1), "frac_mfma_peak": round(pf / (pre * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4)}
        phases[f"executor_{name}_decode"] = {"ms": round(dec, 3), "ms_per_step": round(dec / max(nsteps, 1), 4),
                                             "tokens_per_s": round(n_seq * nsteps / (dec * 1e-3), 1), "GBps": round(gbs, 1),
                                             "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes_per_step": int(step_bytes)}
    jf = prefill_flops(synth.M8B, np.full(n_seq, jlen))
    jms = float(ms[4])
    phases["judge_prefill"] = {"ms": round(jms, 3), "tokens_per_s": round(n_seq * jlen / (jms * 1e-3), 1),
                               "TFLOPs": round(jf / (jms * 1e-3) / 1e12, 1), "frac_mfma_peak": round(jf / (jms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4)}
    out = {"metric": "duel_round_seconds", "value": round(float(ms.sum()) * 1e-3, 4), "unit": "s", "higher_is_better": False,
           "ms_per_step": round(float(ms.sum()), 3)}
    out.update(_common_fields(args, f"duel-and-judge round: {n_seq} prompts of {plen} tokens, {nsteps} greedy tokens each by a 1B-shaped "
                                    f"(seed 1) and an 8B-shaped (seed 2) model resident together, judge prefill by the 8B-shaped "
                                    f"model over {jlen} tokens per sequence; KV block 16, random-init weights"))
    out.update({"phases": phases, "settlement": settled, "wall_s_timed_region": round(wall, 3), "checksum_judge_tokens": checksum})
    print(json.dumps(out), flush=True)
    for x in execs.values():
        x["model"].close()


def mixed_schedule(lens, n_seq, chunk, budget, dec_steps):
    """The interleaved schedule of the long-context mixed batch, as a list of calls: ("prefill", ids, q, seq_after) with
    chunks of up to `chunk` tokens dealt round-robin to the sequences still prefilling within `budget` tokens per call, each
    followed by ("decode", ids, seq_after) over the sequences whose prompt is complete, until every one has `dec_steps`."""
    done = np.zeros(n_seq, np.int64)
    ndec = np.zeros(n_seq, np.int64)
    rr, calls = 0, []
    while (ndec < dec_steps).any():
        pending = [b for b in list(range(rr, n_seq)) + list(range(rr)) if done[b] < lens[b]]
        pick, left = [], budget
        for b in pending:
            q = int(min(chunk, lens[b] - done[b]))
            if q > left:
                break
            pick.append((b, q))
            left -= q
        if pick:
            rr = (pick[-1][0] + 1) % n_seq
            ids = np.array([b for b, _ in pick])
            q = np.array([q for _, q in pick], np.int64)
            calls.append(("prefill", ids, q, done[ids] + q, done[ids].copy()))
            done[ids] += q
        ids = np.nonzero((done == lens) & (ndec < dec_steps))[0]
        if len(ids):
            calls.append(("decode", ids, None, lens[ids] + ndec[ids] + 1, None))
            ndec[ids] += 1
    return calls


def time_scheduler(B, lens, n_seq, chunk, budget, dec_steps, mbs, n_calls):
    """Host cost of the library's continuous-batching scheduler on the same request set (all requests queued at the start,
    the whole pool usable): it plans the very schedule that is timed above, one plan + commit per iteration."""
    need = int(((lens + dec_steps + 15) // 16).sum())
    s = B.Scheduler(n_seq, mbs, budget, chunk, need, 1.0)
    for b in range(n_seq):
        s.submit(b, int(lens[b]), dec_steps + 1)
    t0 = time.perf_counter()
    iterations = planned_calls = 0
    while True:
        pre, dec = s.plan()
        planned_calls += (1 if pre else 0) + (1 if dec else 0)
        s.commit()
        iterations += 1
        if s.stats()["active"] == 0:
            break
    dt = time.perf_counter() - t0
    s.close()
    return {"iterations": iterations, "calls_planned": planned_calls, "equals_timed_schedule": planned_calls == n_calls,
            "host_us_per_iteration": round(dt / iterations * 1e6, 1), "what": "www_sched_plan + www_sched_commit + www_get_stats through the binding"}


def bench_mixed(args):
    """Long-context mixed batch: chunked prefill interleaved with decode steps on the 8B-shaped model."""
    import torch
    from paper_2603_20661_amd import binding as B
    from paper_2603_20661_amd import synth

    shape = synth.M8B
    n_seq, chunk, budget = 128, 512, 8192
    dec_steps = 64 if args.decode_steps is None else args.decode_steps
    lens = synth.lengths_zipf(2, n_seq, 1.2, 256, 16384).astype(np.int64)
    cap = lens + dec_steps + 1
    mbs = int((cap.max() + 15) // 16)
    calls = mixed_schedule(lens, n_seq, chunk, budget, dec_steps)
    prompts = [synth.tokens(1000 + b, int(lens[b]), shape.vocab) for b in range(n_seq)]

    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(dev)
    i64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int64)).to(dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    t0 = time.time()
    blob = synth.make_blob(shape)
    log(f"mixed: weights {blob.size / 2**30:.2f} GiB generated in {time.time() - t0:.1f} s; {len(calls)} calls, "
        f"{int(lens.sum())} prompt tokens, longest {int(lens.max())}")
    with torch.cuda.stream(stream):
        blob_dev = torch.from_numpy(blob).to(dev)
        # KV pool: 90 % of the memory that is free once the weights (the blob and its packed copy) are resident
        probe = B.make_config(shape, n_seq, mbs, budget, 1)
        _, _, ws_bytes = B.www_query_sizes(probe)
        free_bytes, _ = torch.cuda.mem_get_info()
        block_bytes = shape.n_layers * 2 * shape.n_kv_heads * 16 * (shape.head_dim * 2 + 4)
        nb = int(0.90 * (free_bytes - ws_bytes)) // block_bytes
        table = synth.block_tables(2, cap, nb, mbs, permute=True)
        cfg = B.make_config(shape, n_seq, mbs, budget, nb)
        model = B.Model(cfg, blob_dev, stream=stream)
        stream.synchronize()
        del blob_dev, blob
        table_dev = i32(table)
        # per-call arguments, resident before the timed region; decode calls go through fixed staging buffers so that a
        # step of a given batch size finds its captured graph again
        prepared = []
        for kind, ids, q, seq_after, done_before in calls:
            c = {"kind": kind, "n": len(ids), "ids": i64(ids), "seq": i32(seq_after)}
            if kind == "prefill":
                c["tokens"] = i32(np.concatenate([prompts[b][d0: d0 + qq] for b, qq, d0 in zip(ids, q, done_before)]))
                c["q"] = i32(q)
                c["table"] = table_dev[c["ids"]].contiguous()
                fin = np.nonzero(seq_after == lens[ids])[0]
                c["fin_rows"], c["fin_ids"] = i64(fin), i64(ids[fin])
                c["flops"] = prefill_call_flops(shape, q, seq_after)
                c["ntok"] = int(q.sum())
            else:
                c["bytes"] = decode_step_bytes(shape, seq_after, len(ids))
            prepared.append(c)
        last_tok = torch.zeros(n_seq, dtype=torch.int32, device=dev)
        pre_next = torch.empty(n_seq, dtype=torch.int32, device=dev)
        dec_tok = torch.empty(n_seq, dtype=torch.int32, device=dev)
        dec_seq = torch.empty(n_seq, dtype=torch.int32, device=dev)
        dec_table = torch.empty((n_seq, mbs), dtype=torch.int32, device=dev)
        logits = torch.empty((n_seq, shape.vocab), dtype=torch.float32, device=dev)

        def one_pass():
            marks = []
            for c in prepared:
                n = c["n"]
                e0, e1 = ev(), ev()
                if c["kind"] == "prefill":
                    e0.record(stream)
                    B.www_prefill(model, c["tokens"], c["q"], c["seq"], c["table"], logits=None, next_tokens=pre_next[:n], stream=stream)
                    e1.record(stream)
                    if c["fin_ids"].numel():
                        last_tok.index_copy_(0, c["fin_ids"], pre_next[:n].index_select(0, c["fin_rows"]))
                else:
                    torch.index_select(last_tok, 0, c["ids"], out=dec_tok[:n])
                    torch.index_select(table_dev, 0, c["ids"], out=dec_table[:n])
                    dec_seq[:n].copy_(c["seq"])
                    e0.record(stream)
                    B.www_decode_step(model, dec_tok[:n], dec_seq[:n], dec_table[:n], logits=logits[:n], next_tokens=dec_tok[:n], stream=stream)
                    e1.record(stream)
                    last_tok.index_copy_(0, c["ids"], dec_tok[:n])
                marks.append((e0, e1))
            return marks

        for _ in range(args.warmup):
            one_pass()
        stream.synchronize()
        torch.cuda.synchronize()
        walls, per_call = [], np.zeros(len(prepared))
        for _ in range(args.steps):
            t0 = time.time()
            marks = one_pass()
            stream.synchronize()
            torch.cuda.synchronize()
            walls.append(time.time() - t0)
            per_call += np.array([a.elapsed_time(b) for a, b in marks])
        per_call /= args.steps
        assert torch.isfinite(logits).all(), "non-finite logits"
        checksum = int(last_tok.cpu().numpy().astype(np.int64).sum())

    pre = [(c, t) for c, t in zip(prepared, per_call) if c["kind"] == "prefill"]
    dec = [(c, t) for c, t in zip(prepared, per_call) if c["kind"] == "decode"]
    pre_ms, dec_ms = sum(t for _, t in pre), sum(t for _, t in dec)
    pre_tf = sum(c["flops"] for c, _ in pre) / (pre_ms * 1e-3) / 1e12
    dec_gbs = sum(c["bytes"] for c, _ in dec) / (dec_ms * 1e-3) / 1e9
    full = [(c, t) for c, t in dec if c["n"] == n_seq]
    classes = {
        "prefill_chunks": {"calls": len(pre), "ms": round(pre_ms, 2), "tokens_per_s": round(sum(c["ntok"] for c, _ in pre) / (pre_ms * 1e-3), 1),
                           "TFLOPs": round(pre_tf, 1), "frac_mfma_peak": round(pre_tf / MFMA_PEAK_TFLOPS, 4)},
        "decode_steps": {"calls": len(dec), "ms": round(dec_ms, 2), "tokens_per_s": round(sum(c["n"] for c, _ in dec) / (dec_ms * 1e-3), 1),
                         "GBps": round(dec_gbs, 1), "frac_hbm_peak": round(dec_gbs / HBM_PEAK_GBS, 4)},
    }
    if full:
        fb, ft = sum(c["bytes"] for c, _ in full), sum(t for _, t in full)
        classes["decode_steps_all_128_active"] = {"calls": len(full), "ms_per_step": round(ft / len(full), 3),
                                                  "algorithmic_bytes_per_step": int(fb / len(full)),
                                                  "GBps": round(fb / (ft * 1e-3) / 1e9, 1), "frac_hbm_peak": round(fb / (ft * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    wall = float(np.mean(walls))
    out = {"metric": "schedule_wall_seconds", "value": round(wall, 4), "unit": "s", "higher_is_better": False, "ms_per_step": round(wall * 1e3, 3)}
    out.update(_common_fields(args, f"long-context mixed batch on the 8b-shaped decoder: {n_seq} sequences, Zipf(1.2) lengths "
                                    f"{int(lens.min())}..{int(lens.max())} (sum {int(lens.sum())}), {chunk}-token prefill chunks within {budget} "
                                    f"tokens per call interleaved with decode steps, {dec_steps} greedy tokens per sequence, KV pool "
                                    f"{nb} blocks = {nb * block_bytes / 2**30:.0f} GiB with permuted block tables"))
    out.update({"call_classes": classes, "kv_pool_GiB": round(nb * block_bytes / 2**30, 1), "checksum_last_tokens": checksum,
                "scheduler": time_scheduler(B, lens, n_seq, chunk, budget, dec_steps, mbs, len(calls))})
    print(json.dumps(out), flush=True)
    model.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="8b", choices=["tiny", "1b", "8b", "duel", "mixed", "1b-fp8wo", "8b-fp8wo", "1b-int4wo128", "8b-int4wo128",
                                                          "1b-int4wo32", "8b-int4wo32", "1b-qknorm", "8b-qknorm"])
    ap.add_argument("--decode-steps", type=int, default=None, help="override the workload's decode steps (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (sequences are independent, nothing is sharded); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.workload == "duel":
        return bench_duel(args)
    if args.workload == "mixed":
        return bench_mixed(args)

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
                              "ms_per_step": round(ms / nprof, 4), "frac": round(gbs / HBM_PEAK_GBS, 4),
                              "algorithmic_bytes": int(per_bytes[k]), "traffic": measured_traffic(args.workload, k, per_bytes[k])}
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

    copy_peak = measured_copy_bandwidth(dev, stream)
    mfma_rate = measured_mfma_rate(dev, stream)
    if roofline:
        # what an event pair around a near-empty kernel reads in the middle of a busy stream: the part of avg_launch_ms that
        # is dispatch and event handling rather than the kernel (a kernel trace's durations are shorter by about this much)
        roofline["event_pair_floor_ms"] = event_pair_floor(dev, stream)
        # the whole decode step beside its dominant kernel: the figure the 70 % target is about
        roofline["whole_step_frac"] = round(step_gbs / HBM_PEAK_GBS, 4)

    cpu = None
    if not args.no_cpu_baseline and shape.weight_dtype < 2:   # (the weight-only quantised workloads are not the bench line)
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
                                 "frac": round(step_gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes_per_step": int(step_bytes),
                                 "frac_of_measured_copy": round(step_gbs / copy_peak["GBps"], 4)},
        "measured_copy_bandwidth": copy_peak,
        "roofline_prefill": {"bound": "mfma", "achieved": round(pre_tflops, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": round(pre_tflops / MFMA_PEAK_TFLOPS, 4), "algorithmic_flops": pf,
                             "frac_of_measured_mfma_loop": round(pre_tflops / mfma_rate["TFLOPs"], 4)},
        "measured_mfma_loop": mfma_rate,
        "decode_kernels": kernels,
        "cpu_baseline": cpu,
        "wall_s_timed_region": round(wall, 3),
        "checksum_last_tokens": int(final_tokens.astype(np.int64).sum()),
    }
    print(json.dumps(out), flush=True)
    model.close()


def measured_copy_bandwidth(dev, stream):
    """What a plain device-to-device copy reaches on this GPU (read plus written bytes over the time between two events):
    the achievable figure beside the published 8 TB/s that the roofline fractions are quoted against."""
    import torch
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    src.fill_(3)
    times = []
    with torch.cuda.stream(stream):
        for it in range(7):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            dst.copy_(src)
            e1.record(stream)
            stream.synchronize()
            if it >= 2:
                times.append(e0.elapsed_time(e1))
    del src, dst
    torch.cuda.empty_cache()
    ms = float(np.median(times))
    return {"GBps": round(2 * nbytes / ms * 1e-6, 1), "what": "device-to-device copy of 1 GiB, read + written bytes, median of 5 after 2 warm-up"}


def measured_mfma_rate(dev, stream):
    """What a loop of nothing but fp16 MFMAs on register operands sustains on this GPU (www_debug_mfma_loop: two workgroups
    of four wavefronts per compute unit, pseudo-random operands): the achievable figure beside the published dense peak
    that the prefill fraction is quoted against."""
    import torch
    from paper_2603_20661_amd import binding as B
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    wgs, iters = 8 * cus, 12000
    sink = torch.empty(wgs * 4, dtype=torch.float32, device=dev)
    times, flops = [], 0.0
    with torch.cuda.stream(stream):
        for it in range(7):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            flops = B.www_debug_mfma_loop(wgs, iters, sink, stream=stream)
            e1.record(stream)
            stream.synchronize()
            if it >= 2:
                times.append(e0.elapsed_time(e1))
    ms = float(np.median(times))
    return {"TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1), "ms": round(ms, 3),
            "what": f"{wgs} workgroups x 4 wavefronts x {iters} rounds of 8 independent 32x32x16 fp16 MFMAs on register operands, median of 5 after 2 warm-up"}


def event_pair_floor(dev, stream):
    import torch
    busy = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
    tiny = torch.zeros(64, dtype=torch.int32, device=dev)
    with torch.cuda.stream(stream):
        busy.fill_(1)   # keeps the queue ahead of the device while the pairs are enqueued
        busy.fill_(2)
        evs = []
        for _ in range(64):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            tiny.add_(1)
            e1.record(stream)
            evs.append((e0, e1))
        stream.synchronize()
    del busy
    return round(float(np.median([a.elapsed_time(b) for a, b in evs])), 5)


def cpu_model_name():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(shape, blob, lens, nsteps):
    """The CPU oracle, untuned, on a bounded sample: one to four decode steps (about 12 s of CPU work) of the first `n`
    sequences from their first decode-step context lengths on.  Its KV cache is pre-filled with seeded N(0,1) values
    instead of running the prompt through the CPU (same work per step, different values)."""
    from oracle import oracle as O
    from paper_2603_20661_amd import synth
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
    per_tok_flops = 2.0 * (shape.n_params() - shape.vocab * shape.d_model)
    n = int(max(1, min(len(lens), 25.0 * 3e9 * threads / per_tok_flops)))   # ~25 s at ~3 GFLOP/s per thread
    ctx = lens[:n] + 1
    cap = ctx + 3                                   # room for up to 4 steps
    mbs = int((cap.max() + 15) // 16)
    nb = int(((cap + 15) // 16).sum())
    table = synth.block_tables(7, cap, nb, mbs, permute=True)
    m = O.OracleModel(shape, blob, num_blocks=nb)
    pool = m.kv_paged().reshape(-1)
    tile = synth.normal_f32(99, 1, min(pool.size, 1 << 24))
    for at in range(0, pool.size, tile.size):
        k = min(tile.size, pool.size - at)
        pool[at:at + k] = tile[:k]
    toks = synth.tokens(99, n, shape.vocab)
    # decode steps over the same sequences until about 12 s of CPU work are spent (at most 4 steps; the tables leave room)
    t0 = time.time()
    steps_done = 0
    while steps_done < 4 and (steps_done == 0 or time.time() - t0 < 12.0):
        m.forward(toks, np.ones(n, np.int32), ctx + steps_done, block_table=table)
        steps_done += 1
    dt = time.time() - t0
    m.close()
    return {"value": round(n * steps_done / dt, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle", "cpu": cpu_model_name(),
            "sample": f"{steps_done} decode step(s) of the first {n} sequences (context {int(ctx.min())}..{int(ctx.max()) + steps_done - 1}), KV "
                      f"pre-filled with seeded N(0,1) values, {dt:.1f} s"}


if __name__ == "__main__":
    main()
