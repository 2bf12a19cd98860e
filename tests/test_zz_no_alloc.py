"""GPU: the sampling entry point that allocates nothing (its scratch buffer is an array built into the library) against
the entry point it is a variant of, called through the C ABI: same tokens bit for bit, on two calls in a row, the second
with a smaller input (the array keeps the first call's contents), and a size beyond the array's is refused."""
import ctypes

import numpy as np
import pytest

from paper_2603_20661_amd import synth

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_equals_the_caller_buffer_one():
    import torch
    from paper_2603_20661_amd import binding as B
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    vp = ctypes.c_void_p
    for call, (batch, vocab, std, temperature, top_p) in enumerate(((64, 128256, 6.0, 0.8, 0.9), (5, 32000, 3.0, 1.2, 0.6))):
        lg = synth.normal_f32(301 + call, vocab, batch * vocab, std=std).reshape(batch, vocab)
        u = synth.uniform01(302 + call, vocab, batch).astype(np.float32)
        lg_dev, u_dev = torch.from_numpy(lg).to(dev), torch.from_numpy(u).to(dev)
        scratch = torch.empty((batch, vocab), dtype=torch.float32, device=dev)
        want = torch.full((batch,), -1, dtype=torch.int32, device=dev)
        got = torch.full((batch,), -2, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        # raw C ABI: pointers and sizes
        rc = B.lib.www_sample_top_p(vp(lg_dev.data_ptr()), batch, vocab, temperature, top_p, vp(u_dev.data_ptr()),
                                    vp(scratch.data_ptr()), vp(want.data_ptr()), vp(stream))
        assert rc == 0, B.lib.www_last_error()
        rc = B.lib.www_sample_top_p_static(vp(lg_dev.data_ptr()), batch, vocab, temperature, top_p, vp(u_dev.data_ptr()),
                                           vp(got.data_ptr()), vp(stream))
        assert rc == 0, B.lib.www_last_error()
        torch.cuda.synchronize()
        w, g = want.cpu().numpy(), got.cpu().numpy()
        assert (w >= 0).all() and (w < vocab).all()
        assert np.array_equal(w, g), f"call {call}: {int((w != g).sum())} of {batch} tokens differ"
        print(f"call {call}: batch {batch} vocab {vocab}: {batch} tokens equal", flush=True)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2603_20661_amd import binding as B
    dev = torch.device("cuda:0")
    vocab = 128256
    batch = B.SAMPLE_STATIC_MAX_FLOATS // vocab + 1
    lg = torch.zeros((batch, vocab), dtype=torch.float32, device=dev)
    u = torch.zeros(batch, dtype=torch.float32, device=dev)
    tok = torch.full((batch,), -7, dtype=torch.int32, device=dev)
    with pytest.raises(B.WwwError) as e:
        B.www_sample_top_p_static(lg, 1.0, 0.9, u, tok)
    assert e.value.code == B.E_CAPACITY
    with pytest.raises(B.WwwError) as e:
        B.www_sample_top_p_static(lg[:2], 0.0, 0.9, u[:2], tok[:2])
    assert e.value.code == B.E_INVALID_ARG
    torch.cuda.synchronize()
    assert (tok.cpu().numpy() == -7).all()          # nothing ran
