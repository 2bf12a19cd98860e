#!/usr/bin/env python3
"""Writes the stored oracle results of the full-depth parity cases (tests/full_depth_cases.py has the recipes and the
file format).  Calls only the CPU oracle and the seeded input generators; nothing of the GPU library is imported.

    python tests/golden/make_full_depth.py 1b | 8b | 8b-long | duel | mixed

Run times on 8 host cores: 1b about 10 minutes, 8b 25, mixed 10, duel 35, 8b-long (one 4096-token prompt) 75.
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))                    # tests/
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))   # repository root

import full_depth_cases as C                 # noqa: E402
from helpers import oracle_greedy            # noqa: E402  (prefill + greedy steps through the oracle, nothing else)
from paper_2603_20661_amd import synth       # noqa: E402


def log(msg):
    print(f"[golden {time.strftime('%H:%M:%S')}] {msg}", flush=True)


def greedy(shape, blob, prompts, steps, chunk=None):
    return oracle_greedy(shape, blob, prompts, steps, chunk=chunk, log=log)


def main():
    case = sys.argv[1]
    out = {}
    if case in C.BENCH_FILES:
        name, which = C.BENCH_FILES[case]
        wl, sample = C.bench_case(name)
        ids = [sample[k] for k in which]
        starts = np.concatenate([[0], np.cumsum(wl.prompt_lens)[:-1]])
        prompts = [wl.prompt_tokens[starts[b]: starts[b] + wl.prompt_lens[b]] for b in ids]
        cols = C.sample_columns(wl.shape.vocab, 1)
        blob = synth.make_blob(wl.shape)
        log(f"{case}: sequences {ids} of lengths {[len(p) for p in prompts]}, {wl.decode_steps} steps")
        logits = greedy(wl.shape, blob, prompts, wl.decode_steps)
        out["cols"], out["seq_ids"] = cols, np.array(ids, np.int32)
        for b, lg in zip(ids, logits):
            C.pack_rows(f"seq{b}", lg, cols, out)
    elif case == "duel":
        d = C.DUEL
        prompt = C.duel_prompts()[d["sample"]]
        answers = {}
        for name, shape in (("A", synth.M1B), ("B", synth.M8B)):
            cols = C.sample_columns(shape.vocab, 2)
            blob = synth.make_blob(shape)
            log(f"duel executor {name} ({shape.name})")
            lg = greedy(shape, blob, [prompt], d["steps"])[0]
            out[f"cols{name}"] = cols
            C.pack_rows(f"exec{name}", lg, cols, out)
            answers[name] = out[f"exec{name}.tokens"][:d["steps"]]       # the first `steps` greedy tokens are the answer
        judge_in = np.concatenate([prompt, answers["A"], answers["B"]]).astype(np.int32)
        log(f"judge pass over {len(judge_in)} tokens")
        lg = greedy(synth.M8B, blob, [judge_in], 0)[0]                   # blob: still the 8B-shaped model's
        out["cols"] = out["colsB"]
        C.pack_rows("judge", lg, out["cols"], out)
        out["judge_in"] = judge_in
    elif case == "mixed":
        lens, prompts, ids = C.mixed_case()
        shape = synth.M8B
        cols = C.sample_columns(shape.vocab, 3)
        blob = synth.make_blob(shape)
        log(f"mixed batch: sequences {ids} of {[int(lens[b]) for b in ids]} tokens in chunks of {C.MIXED['chunk']}")
        logits = greedy(shape, blob, [prompts[b] for b in ids], C.MIXED["dec_steps"], chunk=C.MIXED["chunk"])
        out["cols"], out["seq_ids"] = cols, np.array(ids, np.int32)
        for b, lg in zip(ids, logits):
            C.pack_rows(f"seq{b}", lg, cols, out)
    else:
        raise SystemExit(f"unknown case {case}")
    np.savez(C.golden_path(case), **out)
    log(f"wrote {C.golden_path(case)}")


if __name__ == "__main__":
    main()
