"""GPU: the verdict kernel (votes of a judge pass read off last-position logits) against the oracle, bit for bit, on
seeded synthetic logits of the 8B vocabulary with planted ties."""
import numpy as np
import pytest

from oracle import duel as O
from paper_2603_20661_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("batch,vocab,ta,tb", [(32, 128256, 32, 33), (300, 32000, 31999, 0), (1, 1024, 5, 700)])
def test_verdicts_match_oracle_bitwise(batch, vocab, ta, tb):
    import torch
    from paper_2603_20661_amd import binding as B
    lg = synth.normal_f32(71, batch, batch * vocab, std=3.0).reshape(batch, vocab)
    lg[::7, tb] = lg[::7, ta]                                  # planted ties go to answer A
    if batch > 2:
        lg[1, ta], lg[1, tb] = -0.0, 0.0
    ref_v, ref_m = O.verdicts(lg, ta, tb)
    dev = torch.device("cuda:0")
    v = torch.full((batch,), -1, dtype=torch.int32, device=dev)
    m = torch.zeros(batch, dtype=torch.float32, device=dev)
    B.www_judge_verdict(torch.from_numpy(lg).to(dev), ta, tb, v, m)
    torch.cuda.synchronize()
    assert np.array_equal(v.cpu().numpy(), ref_v)
    assert np.array_equal(m.cpu().numpy().view(np.uint32), ref_m.view(np.uint32))
    assert 0 < ref_v.sum() < batch or batch == 1
    v2 = torch.full((batch,), -1, dtype=torch.int32, device=dev)
    B.www_judge_verdict(torch.from_numpy(lg).to(dev), ta, tb, v2, None)      # margins are optional
    torch.cuda.synchronize()
    assert np.array_equal(v2.cpu().numpy(), ref_v)
    with pytest.raises(B.WwwError) as e:
        B.www_judge_verdict(torch.from_numpy(lg).to(dev), ta, ta, v, m)
    assert e.value.code == B.E_INVALID_ARG
