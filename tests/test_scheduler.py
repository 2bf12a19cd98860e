"""The serving loop's scheduler without a GPU.  The oracle (oracle/sched.py) is checked against properties that hold
for any workload (no block owned twice, the target share of the pool and the token budget respected, first come first
served, every request gets exactly its tokens) and against an independent formulation of the same policy (the fixed
schedule of the long-context mixed batch in bench.py, written as one loop over arrays); then the library's scheduler
is compared with the oracle plan by plan."""
import numpy as np
import pytest

import bench
from oracle import sched as O
from paper_2603_20661_amd import synth

B = pytest.importorskip("paper_2603_20661_amd.binding", reason="libwww.so is not built")


def workload(seed, n, max_prompt, max_new):
    plen = 1 + synth.uniform_i32(seed, 1, n, max_prompt)
    new = 1 + synth.uniform_i32(seed, 2, n, max_new)
    return [(1000 + r, int(plen[r]), int(new[r])) for r in range(n)]


def drive(s, requests, arrivals_per_iteration, check=None, limit=100000):
    """Feeds the requests a few per iteration and runs the loop dry.  Returns the list of (prefill, decode, finished)."""
    log, at = [], 0
    while True:
        for r in requests[at:at + arrivals_per_iteration]:
            s.submit(*r)
        at += arrivals_per_iteration
        pre, dec = s.plan()
        if check:
            check(s, pre, dec)
        done = s.commit()
        log.append((pre, dec, done))
        st = s.stats()
        if at >= len(requests) and st["active"] == 0 and st["queued"] == 0:
            return log
        assert len(log) < limit, "the loop does not drain"


def test_properties_under_a_tight_pool():
    cfg = dict(max_batch=6, max_blocks_per_seq=24, token_budget=96, chunk_tokens=40, num_kv_blocks=90, target_utilisation=0.7)
    reqs = workload(5, 60, 300, 80)
    s = O.Scheduler(**cfg)
    admitted, seen_blocks = [], set()

    def check(s, pre, dec):
        owned = [b for q in s.slots if q for b in q["blocks"]]
        assert len(owned) == len(set(owned)) == s.reserved <= int(0.7 * 90)          # no block twice, target share kept
        assert not set(owned) & set(s.free) and len(owned) + len(s.free) == 90
        seen_blocks.update(owned)
        assert sum(e[1] for e in pre) <= 96 and all(1 <= e[1] <= 40 for e in pre)      # budget and chunk size
        assert len({e[0] for e in pre}) == len(pre) and len({e[0] for e in dec}) == len(dec)
        for q in s.slots:
            if q and q["request"] not in admitted:
                admitted.append(q["request"])
        for i, q_len, seq_len, off, req in pre:
            q = s.slots[i]
            assert q["request"] == req and off == q["prefilled"] and seq_len == off + q_len <= q["plen"]
        for i, seq_len, req in dec:
            q = s.slots[i]
            assert q["request"] == req and seq_len <= q["plen"] + q["max_new"] - 1 <= 16 * len(q["blocks"])

    log = drive(s, reqs, 3, check)
    assert admitted == [r[0] for r in reqs]                                             # first come first served
    assert sorted(r for _, _, done in log for r in done) == sorted(r[0] for r in reqs)
    st = s.stats()
    assert st["prompt_tokens_done"] == sum(r[1] for r in reqs) and st["tokens_generated"] == sum(r[2] for r in reqs)
    assert st["kv_blocks_reserved"] == 0 and len(s.free) == 90
    # per request: chunks cover the prompt in order, then decode lengths count up one by one to prompt + max_new - 1
    for req, plen, new in reqs:
        offs = [(off, q) for pre, _, _ in log for _, q, _, off, r in pre if r == req]
        assert [o for o, _ in offs] == list(np.cumsum([0] + [q for _, q in offs[:-1]])) and sum(q for _, q in offs) == plen
        lens = [l for _, dec, _ in log for _, l, r in dec if r == req]
        assert lens == list(range(plen + 1, plen + new))
    assert len(seen_blocks) <= 63                                                       # recycled blocks are reused first


def test_equals_the_fixed_schedule_of_the_mixed_batch():
    n_seq, chunk, budget, dec_steps = 128, 512, 8192, 64
    lens = synth.lengths_zipf(2, n_seq, 1.2, 256, 16384).astype(np.int64)
    calls = bench.mixed_schedule(lens, n_seq, chunk, budget, dec_steps)
    mbs = int((lens.max() + dec_steps + 15) // 16)
    s = O.Scheduler(n_seq, mbs, budget, chunk, num_kv_blocks=int(((lens + dec_steps + 15) // 16).sum()), target_utilisation=1.0)
    for b in range(n_seq):
        s.submit(b, int(lens[b]), dec_steps + 1)
    mine = []
    while True:
        pre, dec = s.plan()
        if pre:
            mine.append(("prefill", [e[0] for e in pre], [e[1] for e in pre], [e[2] for e in pre], [e[3] for e in pre]))
        if dec:
            mine.append(("decode", [e[0] for e in dec], None, [e[1] for e in dec], None))
        s.commit()
        if s.stats()["active"] == 0:
            break
    ref = [(k, list(map(int, ids)), None if q is None else list(map(int, q)), list(map(int, after)),
            None if before is None else list(map(int, before))) for k, ids, q, after, before in calls]
    assert mine == ref


def test_benchmark_drives_the_library_scheduler_over_the_timed_schedule():
    """bench.py's host-cost figure comes from the library's scheduler planning exactly the calls that were timed"""
    n_seq, chunk, budget, dec_steps = 24, 64, 512, 5
    lens = synth.lengths_zipf(3, n_seq, 1.2, 20, 900).astype(np.int64)
    calls = bench.mixed_schedule(lens, n_seq, chunk, budget, dec_steps)
    mbs = int((lens.max() + dec_steps + 1 + 15) // 16)
    r = bench.time_scheduler(B, lens, n_seq, chunk, budget, dec_steps, mbs, len(calls))
    assert r["equals_timed_schedule"] and r["calls_planned"] == len(calls) and r["iterations"] >= dec_steps
    assert r["host_us_per_iteration"] > 0


@pytest.mark.parametrize("seed,arrivals", [(11, 1), (12, 4), (13, 50)])
def test_library_scheduler_equals_oracle_plan_by_plan(seed, arrivals):
    cfg = dict(max_batch=7, max_blocks_per_seq=30, token_budget=128, chunk_tokens=48, num_kv_blocks=120, target_utilisation=0.7)
    reqs = workload(seed, 80, 400, 70)
    o, g = O.Scheduler(**cfg), B.Scheduler(**cfg)
    try:
        at = 0
        for it in range(100000):
            for r in reqs[at:at + arrivals]:
                o.submit(*r); g.submit(*r)
            at += arrivals
            assert g.plan() == o.plan()
            for i in range(cfg["max_batch"]):
                assert g.table_row(i) == o.table_row(i)
            assert g.commit() == o.commit()
            assert g.stats() == o.stats()
            if at >= len(reqs) and o.stats()["active"] == 0 and o.stats()["queued"] == 0:
                break
        assert o.stats()["finished"] == len(reqs) and o.stats()["iterations"] == it + 1
    finally:
        g.close()


def test_library_rejects_what_it_cannot_serve():
    g = B.Scheduler(max_batch=2, max_blocks_per_seq=4, token_budget=32, chunk_tokens=16, num_kv_blocks=10, target_utilisation=0.5)
    try:
        for args, code in (((1, 0, 5), B.E_INVALID_ARG), ((1, 5, 0), B.E_INVALID_ARG), ((1, 60, 6), B.E_CAPACITY), ((1, 64, 18), B.E_CAPACITY)):
            with pytest.raises(B.WwwError) as e:
                g.submit(*args)
            assert e.value.code == code
        with pytest.raises(B.WwwError):
            g.commit()                                     # nothing planned
        g.submit(7, 60, 5)                                 # 4 blocks of the 5 the target share allows
        g.submit(8, 20, 4)                                 # needs 2: has to wait although a slot is free
        pre, dec = g.plan()
        assert [e[4] for e in pre] == [7] and g.stats()["queued"] == 1 and g.stats()["kv_utilisation"] == 0.4
        with pytest.raises(B.WwwError):
            g.plan()                                       # the previous plan is not committed
        g.commit()
        with pytest.raises(B.WwwError):
            B.Scheduler(2, 4, 32, 16, 10, target_utilisation=1.5)
        with pytest.raises(B.WwwError) as e:               # a full chunk that can never fit an iteration's budget
            B.Scheduler(2, 4, token_budget=16, chunk_tokens=32, num_kv_blocks=10)
        assert e.value.code == B.E_BAD_CONFIG
    finally:
        g.close()


def test_a_chunk_as_large_as_the_budget_still_makes_progress():
    """chunk_tokens == token_budget is the tightest configuration that is accepted: one full chunk per iteration, every
    request finishes"""
    g = B.Scheduler(max_batch=3, max_blocks_per_seq=8, token_budget=32, chunk_tokens=32, num_kv_blocks=24, target_utilisation=1.0)
    try:
        for r, plen in enumerate((100, 32, 7)):
            g.submit(r, plen, 3)
        for it in range(200):
            pre, dec = g.plan()
            assert pre or dec, f"iteration {it}: nothing planned although requests are active"
            assert sum(e[1] for e in pre) <= 32
            g.commit()
            if g.stats()["active"] == 0 and g.stats()["queued"] == 0:
                break
        assert g.stats()["finished"] == 3
    finally:
        g.close()
