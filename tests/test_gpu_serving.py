"""GPU: a serving loop driven by the library's scheduler (requests arrive over time, wait in the queue, are admitted
under the pool's target share, prefilled in chunks and decoded together) against the CPU oracle.  Sequences are
independent, so every third request is first run alone by the oracle (prefill and greedy decoding on its own tokens);
in the serving loop those requests are fed the oracle's tokens, the others the GPU's own: logits of every generated
token within 3e-2, greedy agreement >= 99 %; the scheduler's own plans are compared with its oracle as the loop runs."""
import numpy as np
import pytest

from oracle import sched as OS
from paper_2603_20661_amd import synth
from helpers import GpuSession, oracle_greedy

pytestmark = pytest.mark.gpu

SHAPE = synth.ModelShape("serve128", 2, 512, 8, 2, 128, 1392, 2048, 1e-5, 5e5, synth.WDTYPE_BF16, seed=27)


def test_scheduler_driven_serving_matches_oracle_per_request():
    import torch
    from paper_2603_20661_amd import binding as B
    n_req = 40
    cfg = dict(max_batch=8, max_blocks_per_seq=24, token_budget=160, chunk_tokens=64, num_kv_blocks=110, target_utilisation=0.7)
    plen = 1 + synth.uniform_i32(3, 1, n_req, 300)
    new = 1 + synth.uniform_i32(3, 2, n_req, 60)
    new[5], plen[6] = 1, 1                                   # a request that needs no decode step; a one-token prompt
    prompts = {r: synth.tokens(500 + r, int(plen[r]), SHAPE.vocab) for r in range(n_req)}
    blob = synth.make_blob(SHAPE, gain_std=0.05)
    # the oracle goes first, on its own: logits [new[r], V] of every third request; their argmax are the tokens fed below
    sampled = list(range(0, n_req, 3))
    ref_logits = {r: oracle_greedy(SHAPE, blob, [prompts[r]], int(new[r]) - 1)[0] for r in sampled}
    forced = {r: ref_logits[r].argmax(-1).astype(np.int32) for r in sampled}

    def emitted(r, token):            # the token request r consumes next: the oracle's for a sampled request
        i = len(out_tokens[r])
        out_tokens[r].append(int(token))
        last[r] = int(forced[r][i]) if r in forced else int(token)

    sess = GpuSession(SHAPE, blob, cfg["max_batch"], cfg["max_blocks_per_seq"] * 16, cfg["token_budget"], cfg["num_kv_blocks"])
    sched, ref = B.Scheduler(**cfg), OS.Scheduler(**cfg)
    out_tokens = {r: [] for r in range(n_req)}
    out_logits = {r: [] for r in range(n_req)}
    last = {}
    max_queued = 0
    try:
        at = 0
        for it in range(10000):
            for r in range(at, min(at + 2, n_req)):            # two arrivals per iteration
                sched.submit(r, int(plen[r]), int(new[r])); ref.submit(r, int(plen[r]), int(new[r]))
            at = min(at + 2, n_req)
            pre, dec = sched.plan()
            assert (pre, dec) == ref.plan()
            if pre:
                rows = np.array([sched.table_row(e[0]) for e in pre], np.int32)
                packed = np.concatenate([prompts[e[4]][e[3]: e[3] + e[1]] for e in pre])
                lg, nxt = sess.prefill(packed, [e[1] for e in pre], [e[2] for e in pre], rows)
                for k, (slot, q, seq_len, off, r) in enumerate(pre):
                    if seq_len == plen[r]:                     # the prompt is complete: this is the request's first token
                        out_logits[r].append(lg[k]); emitted(r, nxt[k])
            if dec:
                rows = np.array([sched.table_row(e[0]) for e in dec], np.int32)
                lg, nxt = sess.decode([last[e[2]] for e in dec], [e[1] for e in dec], rows)
                for k, (slot, seq_len, r) in enumerate(dec):
                    assert seq_len == plen[r] + len(out_tokens[r])
                    out_logits[r].append(lg[k]); emitted(r, nxt[k])
            done = sched.commit()
            assert done == ref.commit() and sched.stats() == ref.stats()
            for r in done:
                assert len(out_tokens[r]) == new[r]
            st = sched.stats()
            assert st["kv_utilisation"] <= 0.7
            max_queued = max(max_queued, st["queued"])
            if at == n_req and st["active"] == 0 and st["queued"] == 0:
                break
        assert st["finished"] == n_req and st["tokens_generated"] == int(new.sum()) and st["prompt_tokens_done"] == int(plen.sum())
        assert max_queued > 0, "the pool was meant to be tight enough for requests to queue"
        print(f"serving loop: {it + 1} iterations, {int(plen.sum())} prompt tokens, {int(new.sum())} generated, up to {max_queued} queued", flush=True)
    finally:
        sched.close()
        sess.close()
    worst, hits, total = 0.0, 0, 0
    for r in sampled:
        got = np.stack(out_logits[r])
        assert np.isfinite(got).all() and got.shape == ref_logits[r].shape
        worst = max(worst, float(np.abs(got - ref_logits[r]).max()))
        hits += int((forced[r] == np.array(out_tokens[r])).sum())
        total += len(out_tokens[r])
    print(f"serving loop: max|dlogit|={worst:.3e} agreement={hits / total:.4f} samples={total}", flush=True)
    assert total >= 100 and worst <= 3e-2 and hits / total >= 0.99
