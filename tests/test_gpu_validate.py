"""GPU: the opt-in validation mode (WWW_VALIDATE=1 at load).  Calls whose device-resident arguments break the contract
(token id, block id, lengths, a block named twice) come back with WWW_E_INVALID_ARG and nothing of the model runs on
them: the output buffers keep their sentinel values.  The checks themselves run in a small kernel of the library; the
bad values are only ever compared, never used as addresses.  Valid calls give the bits of a model without the mode."""
import numpy as np
import pytest

from paper_2603_20661_amd import synth
from helpers import GpuSession

pytestmark = pytest.mark.gpu

SHAPE = synth.ModelShape("val64", 2, 256, 8, 4, 64, 704, 1024, 1e-5, 1e4, synth.WDTYPE_BF16, seed=61)


def test_bad_device_arguments_are_rejected_before_any_model_kernel(monkeypatch):
    import torch
    from paper_2603_20661_amd import binding as B
    blob = synth.make_blob(SHAPE, gain_std=0.1)
    nb, mbs = 12, 4
    monkeypatch.setenv("WWW_VALIDATE", "1")
    checked = GpuSession(SHAPE, blob, max_batch=3, max_ctx=mbs * 16, max_prefill_tokens=64, num_blocks=nb)
    monkeypatch.delenv("WWW_VALIDATE")
    plain = GpuSession(SHAPE, blob, max_batch=3, max_ctx=mbs * 16, max_prefill_tokens=64, num_blocks=nb)
    try:
        dev = checked.dev
        i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=dev)
        table = [[0, 1, 2, 3], [4, 5, 6, 7], [8, 9, 10, 11]]
        good = dict(tokens=list(range(30)), q=[10, 5, 15], seq=[10, 5, 15], table=table)

        def prefill(sess, a, expect=None):
            logits = torch.full((3, SHAPE.vocab), -77.0, dtype=torch.float32, device=dev)
            nxt = torch.full((3,), -7, dtype=torch.int32, device=dev)
            with torch.cuda.stream(sess.stream):
                if expect is None:
                    B.www_prefill(sess.model, i32(a["tokens"]), i32(a["q"]), i32(a["seq"]), i32(a["table"]), logits, nxt, stream=sess.stream)
                else:
                    with pytest.raises(B.WwwError) as e:
                        B.www_prefill(sess.model, i32(a["tokens"]), i32(a["q"]), i32(a["seq"]), i32(a["table"]), logits, nxt, stream=sess.stream)
                    assert e.value.code == B.E_INVALID_ARG and expect in str(e.value), str(e.value)
            sess.stream.synchronize()
            return logits.cpu().numpy(), nxt.cpu().numpy()

        def decode(sess, toks, seq, tab, expect=None):
            logits = torch.full((3, SHAPE.vocab), -77.0, dtype=torch.float32, device=dev)
            nxt = torch.full((3,), -7, dtype=torch.int32, device=dev)
            with torch.cuda.stream(sess.stream):
                if expect is None:
                    B.www_decode_step(sess.model, i32(toks), i32(seq), i32(tab), logits, nxt, stream=sess.stream)
                else:
                    with pytest.raises(B.WwwError) as e:
                        B.www_decode_step(sess.model, i32(toks), i32(seq), i32(tab), logits, nxt, stream=sess.stream)
                    assert e.value.code == B.E_INVALID_ARG and expect in str(e.value), str(e.value)
            sess.stream.synchronize()
            return logits.cpu().numpy(), nxt.cpu().numpy()

        def untouched(out):
            return (out[0] == -77.0).all() and (out[1] == -7).all()

        bad_cases = [
            (dict(good, tokens=good["tokens"][:29] + [SHAPE.vocab]), "token id"),
            (dict(good, tokens=[-1] + good["tokens"][1:]), "token id"),
            (dict(good, table=[[0, 1, 2, 3], [4, 5, 6, 7], [nb, 9, 10, 11]]), "block id outside"),
            (dict(good, table=[[0, 1, 2, 3], [-1, 5, 6, 7], [8, 9, 10, 11]]), "block id outside"),
            (dict(good, table=[[0, 1, 2, 3], [0, 5, 6, 7], [8, 9, 10, 11]]), "used twice"),
            (dict(good, q=[10, 5, 15], seq=[10, 4, 15]), "lengths"),                 # q_len > seq_len
            (dict(good, seq=[10, 5, mbs * 16 + 1]), "lengths"),                      # longer than a table row
            (dict(good, q=[10, 0, 20], seq=[10, 5, 20]), "lengths"),                 # an empty chunk
            (dict(good, q=[10, 5, 14], seq=[10, 5, 15]), "add up"),                  # 29 new tokens announced as 30
        ]
        for args, expect in bad_cases:
            assert untouched(prefill(checked, args, expect)), expect
        # entries beyond a sequence's length are not looked at
        ok = dict(good, table=[[0, -5, 2, 3], [4, 99999, 6, 7], [8, 9, 10, 11]])     # seq 0 uses 1 block, seq 1 one, seq 2 one
        a = prefill(checked, ok)
        b = prefill(plain, good)
        assert np.isfinite(a[0]).all() and np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
        nxt = a[1]
        assert untouched(decode(checked, [int(nxt[0]), SHAPE.vocab + 5, int(nxt[2])], [11, 6, 16], table, "token id"))
        assert untouched(decode(checked, nxt, [11, 6, 16], [[0, 1, 2, 3], [4, 5, 6, 7], [2_000_000, 9, 10, 11]], "block id outside"))
        assert untouched(decode(checked, nxt, [11, 0, 16], table, "lengths"))
        assert untouched(decode(checked, nxt, [11, 6, mbs * 16 + 1], table, "lengths"))
        c = decode(checked, nxt, [11, 6, 16], table)
        d = decode(plain, nxt, [11, 6, 16], table)
        assert np.isfinite(c[0]).all() and np.array_equal(c[0], d[0]) and np.array_equal(c[1], d[1])
        B.www_check(checked.model, stream=checked.stream)
    finally:
        checked.close()
        plain.close()


def test_a_row_of_nan_logits_yields_a_token_inside_the_vocabulary():
    """the greedy token of a row without any ordered value is 0, never an index that a later step would use as an address.
    The NaN comes from the model: the embedding row of token 3 is NaN, so the residual stream of a position holding token
    3, its RMSNorm factor and with it every logit of that row are NaN."""
    blob = synth.make_blob(SHAPE, gain_std=0.1).copy()
    entries, _ = synth.blob_layout(SHAPE)
    off = [e for e in entries if e[0] == "embed"][0][1]
    blob[off + 3 * SHAPE.d_model * 2: off + 4 * SHAPE.d_model * 2].view(np.uint16)[:] = 0x7FC0      # bf16 quiet NaN
    sess = GpuSession(SHAPE, blob, max_batch=2, max_ctx=32, max_prefill_tokens=16, num_blocks=4)
    try:
        table = np.array([[0, 1], [2, 3]], np.int32)
        lg, nx = sess.prefill([5, 6, 3, 3], [3, 1], [3, 1], table)
        assert np.isnan(lg).all() and (nx == 0).all(), (nx, np.isnan(lg).mean())
        lg, nx = sess.decode([3, 3], [4, 2], table)
        assert np.isnan(lg).all() and (nx == 0).all(), (nx, np.isnan(lg).mean())
    finally:
        sess.close()
