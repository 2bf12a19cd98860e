"""Why the KV cache and the matrix-core operands are IEEE fp16 and not bf16 (both are 16 bits wide and run at the same
matrix-core rate): measured with the oracle alone.  The 16-layer 1B-shaped model prefills four prompts of 256 tokens; from there three
copies of the cache are decoded side by side, one exact (fp32, the oracle's own), one rounded to bf16 after every call
and one rounded to fp16 after every call - nothing else differs.  With bf16 storage the logits alone leave the 3e-2
tolerance that the GPU path as a whole has to hold; with fp16 storage they stay an order of magnitude inside it.
The rounding itself is the library conversion of PyTorch (round to nearest even), not code of the oracle or of the GPU
path."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2603_20661_amd import synth

TOL = 3e-2


def rounded(a: np.ndarray, dtype) -> np.ndarray:
    return torch.from_numpy(a).to(dtype).float().numpy()


def test_bf16_kv_storage_alone_breaks_the_tolerance_and_fp16_does_not():
    shape = synth.M1B
    blob = synth.make_blob(shape)
    n_seq, plen, steps = 4, 256, 6
    toks = synth.tokens(5, n_seq * plen, shape.vocab)
    cap = plen + steps
    mbs = (cap + 15) // 16
    nb = n_seq * mbs
    table = synth.block_tables(5, [cap] * n_seq, nb, mbs)
    lens = np.full(n_seq, plen, np.int32)
    exact = O.OracleModel(shape, blob, num_blocks=nb)
    variants = {"bf16": (O.OracleModel(shape, blob, num_blocks=nb), torch.bfloat16), "fp16": (O.OracleModel(shape, blob, num_blocks=nb), torch.float16)}
    try:
        _, nxt, _ = exact.forward(toks, lens, lens, block_table=table)
        for m, dt in variants.values():              # the same prefill, its cache rounded to the storage format
            m.kv_paged()[:] = rounded(exact.kv_paged().copy(), dt)
        worst = {k: 0.0 for k in variants}
        for s in range(steps):
            lens = lens + 1
            ref, nxt_new, _ = exact.forward(nxt, np.ones(n_seq, np.int32), lens, block_table=table)
            for k, (m, dt) in variants.items():
                got, _, _ = m.forward(nxt, np.ones(n_seq, np.int32), lens, block_table=table)
                m.kv_paged()[:] = rounded(m.kv_paged().copy(), dt)
                worst[k] = max(worst[k], float(np.abs(got - ref).max()))
            nxt = nxt_new
        print(f"KV storage alone, 1B shape, {n_seq} x {plen} tokens + {steps} steps: max|dlogit| bf16 {worst['bf16']:.3e}, fp16 {worst['fp16']:.3e}")
        assert worst["bf16"] > TOL, worst
        assert worst["fp16"] < TOL / 4, worst
        assert worst["bf16"] > 6 * worst["fp16"], worst       # three more significant bits: a factor of eight, give or take
    finally:
        exact.close()
        for m, _ in variants.values():
            m.close()
