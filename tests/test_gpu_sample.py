"""GPU: the nucleus sampling kernel against its oracle.  Several tokens can be correct where an fp32 sum lands within
rounding of a decision point, so what is checked is: the token is a member of the oracle's nucleus (up to 1e-4 relative on
the threshold), the draw u falls into the token's interval of the running mass (up to 1e-4 of the nucleus mass), and in
at least 95 % of the rows the token is exactly the oracle's; and a second call gives the same tokens bit for bit."""
import numpy as np
import pytest

from oracle import sample as S
from paper_2603_20661_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("vocab,std,temperature,top_p", [
    (128256, 3.0, 1.0, 0.95),      # flat: the nucleus holds most of the vocabulary
    (128256, 12.0, 0.7, 0.95),     # peaked: a handful of members
    (32000, 6.0, 1.3, 0.5),
    (1024, 2.0, 1.0, 1.0),         # plain softmax sampling
    (5000, 5.0, 0.05, 0.9),        # nearly greedy
])
def test_sampled_tokens_are_valid_and_mostly_the_oracle_s(vocab, std, temperature, top_p):
    import torch
    from paper_2603_20661_amd import binding as B
    batch = 48
    lg = synth.normal_f32(81, vocab, batch * vocab, std=std).reshape(batch, vocab)
    lg[3, 100:140] = lg[3].max()                                  # a block of exact ties at the top
    u = synth.uniform01(82, vocab, batch).astype(np.float32)
    u[0], u[1] = 0.0, np.float32(1.0 - 2.0 ** -24)
    dev = torch.device("cuda:0")
    lg_dev, u_dev = torch.from_numpy(lg).to(dev), torch.from_numpy(u).to(dev)
    scratch = torch.empty((batch, vocab), dtype=torch.float32, device=dev)
    tok = torch.full((batch,), -1, dtype=torch.int32, device=dev)
    B.www_sample_top_p(lg_dev, temperature, top_p, u_dev, scratch, tok)
    torch.cuda.synchronize()
    got = tok.cpu().numpy()
    tok2 = torch.full((batch,), -1, dtype=torch.int32, device=dev)
    B.www_sample_top_p(lg_dev, temperature, top_p, u_dev, scratch, tok2)
    torch.cuda.synchronize()
    assert np.array_equal(tok2.cpu().numpy(), got)
    exact = 0
    for b in range(batch):
        want, e, mask, run, target = S.sample(lg[b], temperature, top_p, float(u[b]))
        t = int(got[b])
        assert 0 <= t < vocab
        tau = e[mask].min()
        assert e[t] >= tau * (1 - 1e-4), f"row {b}: token {t} is outside the nucleus"
        eps = 1e-4 * run[-1]
        before = run[t] - (e[t] if mask[t] else 0.0)
        assert before - eps <= target <= run[t] + eps, f"row {b}: draw {u[b]} is not in the interval of token {t}"
        exact += int(t == want)
    print(f"vocab {vocab} std {std} T {temperature} top_p {top_p}: {exact}/{batch} rows equal the oracle's token", flush=True)
    assert exact >= 0.95 * batch


def test_arguments():
    import torch
    from paper_2603_20661_amd import binding as B
    dev = torch.device("cuda:0")
    lg = torch.zeros((2, 64), dtype=torch.float32, device=dev)
    u = torch.zeros(2, dtype=torch.float32, device=dev)
    tok = torch.zeros(2, dtype=torch.int32, device=dev)
    for T, p in ((0.0, 0.9), (-1.0, 0.9), (1.0, 0.0), (1.0, 1.5)):
        with pytest.raises(B.WwwError) as e:
            B.www_sample_top_p(lg, T, p, u, torch.empty_like(lg), tok)
        assert e.value.code == B.E_INVALID_ARG
    B.www_sample_top_p(lg, 1.0, 1.0, u, torch.empty_like(lg), tok)    # all logits equal, u = 0: the first token
    torch.cuda.synchronize()
    assert tok.cpu().tolist() == [0, 0]
