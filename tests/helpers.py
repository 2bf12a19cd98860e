"""Shared harness of the GPU parity tests: runs one synthetic job through the CPU oracle and through
the HIP library (teacher-forced with the oracle's greedy tokens) and returns both sets of logits."""
from __future__ import annotations

import numpy as np

from paper_2603_20661_amd import synth


def oracle_view(shape, blob):
    """What the model oracle is given: the blob itself, or, for a weight-only quantised model, its decoded fp32 form."""
    if shape.weight_dtype in (synth.WDTYPE_FP8WO, synth.WDTYPE_INT4WO_128, synth.WDTYPE_INT4WO_32):
        from oracle import quant
        return quant.dequantize_blob(shape, blob)
    return shape, blob


def gpu_modules():
    import torch
    from paper_2603_20661_amd import binding
    return torch, binding


class GpuSession:
    """One model instance on the GPU plus its block tables."""

    def __init__(self, shape, blob, max_batch, max_ctx, max_prefill_tokens, num_blocks, kv_poison=True):
        torch, B = gpu_modules()
        self.torch, self.B = torch, B
        self.dev = torch.device("cuda:0")
        self.shape = shape
        self.mbs = (max_ctx + 15) // 16
        self.cfg = B.make_config(shape, max_batch, self.mbs, max_prefill_tokens, num_blocks)
        self.stream = torch.cuda.Stream()
        blob_dev = torch.from_numpy(blob).to(self.dev)
        with torch.cuda.stream(self.stream):
            # 0x7FC0 is a bf16 quiet NaN: any read of a slot that was never written poisons the logits
            self.model = B.Model(self.cfg, blob_dev, stream=self.stream, kv_fill=0x7FC0 if kv_poison else 0)
        self.stream.synchronize()
        del blob_dev

    def dev_i32(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(self.dev)

    def prefill(self, tokens, q_lens, seq_lens, table):
        torch, B = self.torch, self.B
        Bn = len(q_lens)
        logits = torch.empty((Bn, self.shape.vocab), dtype=torch.float32, device=self.dev)
        nxt = torch.empty(Bn, dtype=torch.int32, device=self.dev)
        with torch.cuda.stream(self.stream):
            B.www_prefill(self.model, self.dev_i32(tokens), self.dev_i32(q_lens), self.dev_i32(seq_lens), self.dev_i32(table),
                          logits, nxt, stream=self.stream)
        self.stream.synchronize()
        return logits.cpu().numpy(), nxt.cpu().numpy()

    def decode(self, last_tokens, seq_lens, table):
        torch, B = self.torch, self.B
        Bn = len(last_tokens)
        logits = torch.empty((Bn, self.shape.vocab), dtype=torch.float32, device=self.dev)
        nxt = torch.empty(Bn, dtype=torch.int32, device=self.dev)
        with torch.cuda.stream(self.stream):
            B.www_decode_step(self.model, self.dev_i32(last_tokens), self.dev_i32(seq_lens), self.dev_i32(table), logits, nxt,
                              stream=self.stream)
        self.stream.synchronize()
        return logits.cpu().numpy(), nxt.cpu().numpy()

    def close(self):
        self.model.close()


def oracle_replay(shape, blob, prompt, generated):
    """One sequence alone through the oracle: prefill of `prompt`, then one decode step per entry of `generated`
    (teacher-forced).  Returns logits [1 + len(generated), V]: after the prompt and after each appended token."""
    from oracle import oracle as O
    n = len(prompt) + len(generated)
    shape, blob = oracle_view(shape, blob)
    m = O.OracleModel(shape, blob, max_seqs=1, max_ctx=n + 1)
    out = []
    lg, _, _ = m.forward(prompt, [len(prompt)], [len(prompt)], seq_ids=[0])
    out.append(lg[0])
    for i, t in enumerate(generated):
        lg, _, _ = m.forward([t], [1], [len(prompt) + i + 1], seq_ids=[0])
        out.append(lg[0])
    m.close()
    return np.stack(out)


def oracle_greedy(shape, blob, prompts, steps, chunk=None, log=None):
    """The oracle on its own: each prompt alone through its prefill (optionally in chunks of `chunk` tokens), then `steps`
    greedy decode steps of all sequences together, each fed its own previous token.  Returns one array per prompt,
    logits [steps + 1, V]: row 0 after the prompt, row s after s generated tokens; the greedy tokens are their argmax
    (lowest index on ties, as the oracle's own argmax)."""
    import time
    from oracle import oracle as O
    n = len(prompts)
    shape, blob = oracle_view(shape, blob)
    m = O.OracleModel(shape, blob, max_seqs=n, max_ctx=max(len(p) for p in prompts) + steps + 1)
    rows = [[] for _ in range(n)]
    last = np.zeros(n, np.int32)
    for i, p in enumerate(prompts):
        t0 = time.time()
        width = len(p) if chunk is None else chunk
        for a in range(0, len(p), width):
            q = min(width, len(p) - a)
            lg, nx, _ = m.forward(p[a:a + q], [q], [a + q], seq_ids=[i])
        rows[i].append(lg[0])
        last[i] = nx[0]
        if log:
            log(f"prefill of sequence {i} ({len(p)} tokens): {time.time() - t0:.0f} s")
    cur = np.array([len(p) for p in prompts], np.int32)
    t0 = time.time()
    for s in range(steps):
        cur = cur + 1
        lg, nx, _ = m.forward(last, np.ones(n, np.int32), cur, seq_ids=np.arange(n, dtype=np.int32))
        for i in range(n):
            rows[i].append(lg[i])
        last = nx.astype(np.int32)
        if log and s % 32 == 31:
            log(f"decode step {s + 1} of {steps}: {time.time() - t0:.0f} s")
    m.close()
    return [np.stack(r) for r in rows]


def oracle_job(shape, blob, lens, toks, steps, table, num_blocks, chunk=None):
    """Oracle: prefill (optionally in chunks) then `steps` greedy decode steps.
    Returns logits [steps+1, B, V] and the greedy tokens [steps+1, B]."""
    from oracle import oracle as O
    Bn = len(lens)
    shape, blob = oracle_view(shape, blob)
    m = O.OracleModel(shape, blob, max_seqs=0, max_ctx=0, num_blocks=num_blocks)
    lens = np.asarray(lens, np.int32)
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
    if chunk is None:
        lg, nxt, _ = m.forward(toks, lens, lens, block_table=table)
    else:
        done = np.zeros(Bn, np.int64)
        lg = np.zeros((Bn, shape.vocab), np.float32)
        nxt = np.zeros(Bn, np.int32)
        while (done < lens).any():
            q = np.minimum(chunk, lens - done).astype(np.int32)
            act = np.nonzero(q > 0)[0]
            packed = np.concatenate([toks[starts[b] + done[b]: starts[b] + done[b] + q[b]] for b in act])
            l2, n2, _ = m.forward(packed, q[act], (done + q)[act], block_table=table[act])
            fin = (done + q)[act] == lens[act]
            lg[act[fin]] = l2[fin]
            nxt[act[fin]] = n2[fin]
            done += q
    all_logits, all_tok = [lg], [nxt.copy()]
    cur = lens.copy()
    for _ in range(steps):
        cur = cur + 1
        lg, nxt, _ = m.forward(all_tok[-1], np.ones(Bn, np.int32), cur, block_table=table)
        all_logits.append(lg)
        all_tok.append(nxt.copy())
    m.close()
    return np.stack(all_logits), np.stack(all_tok)


def gpu_job(sess: GpuSession, lens, toks, steps, table, forced_tokens, chunk=None):
    """HIP library on the same job, fed the oracle's tokens. Returns logits [steps+1, B, V], tokens [steps+1, B]."""
    lens = np.asarray(lens, np.int32)
    Bn = len(lens)
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
    if chunk is None:
        lg, nxt = sess.prefill(toks, lens, lens, table)
    else:
        done = np.zeros(Bn, np.int64)
        lg = np.zeros((Bn, sess.shape.vocab), np.float32)
        nxt = np.zeros(Bn, np.int32)
        while (done < lens).any():
            q = np.minimum(chunk, lens - done).astype(np.int32)
            act = np.nonzero(q > 0)[0]
            packed = np.concatenate([toks[starts[b] + done[b]: starts[b] + done[b] + q[b]] for b in act])
            l2, n2 = sess.prefill(packed, q[act], (done + q)[act], table[act])
            fin = (done + q)[act] == lens[act]
            lg[act[fin]] = l2[fin]
            nxt[act[fin]] = n2[fin]
            done += q
    all_logits, all_tok = [lg], [nxt.copy()]
    cur = lens.copy()
    for s in range(steps):
        cur = cur + 1
        lg, nxt = sess.decode(forced_tokens[s], cur, table)
        all_logits.append(lg)
        all_tok.append(nxt.copy())
    return np.stack(all_logits), np.stack(all_tok)


def compare(o_logits, o_tok, g_logits, g_tok):
    """-> (max |dlogit|, strict greedy agreement, tie-aware agreement)"""
    assert np.isfinite(g_logits).all(), "non-finite logits from the GPU path"
    err = float(np.abs(o_logits - g_logits).max())
    agree = float((o_tok == g_tok).mean())
    top2 = np.sort(o_logits, axis=-1)[..., -2:]
    gap = top2[..., 1] - top2[..., 0]
    tie = float(((o_tok == g_tok) | (gap < 2 * err)).mean())
    return err, agree, tie
