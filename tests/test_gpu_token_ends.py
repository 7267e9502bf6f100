"""Ends of the token loop on the GPU (embedding row, final norm + task head, softmax and token choice)
against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import tpi_oracle as O
from paper_2410_00531_amd import binding as B
from tpi_testlib import FP32_TOL, rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("vocab,h", [(53, 40), (1000, 1024), (4099, 2052), (32000, 4096), (515, 8192)])
def test_embedding_and_task_head_match_oracle(vocab, h):
    rng = np.random.default_rng(vocab + h)
    w_emb = (rng.standard_normal((vocab, h)) * 0.02).astype(np.float32)
    w_head = (rng.standard_normal((vocab, h)) * 0.02).astype(np.float32)
    g = (1 + 0.02 * rng.standard_normal(h)).astype(np.float32)
    x = rng.standard_normal(h).astype(np.float32)
    we, wh, gt, xt = (torch.from_numpy(a).cuda() for a in (w_emb, w_head, g, x))
    out = torch.full((h,), float("nan"), device="cuda")
    for token in (0, vocab - 1, vocab // 3):
        B.tpi_embed_token(we, token, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint32), O.embed_token(w_emb, token).view(np.uint32))
    logits = torch.full((vocab,), float("nan"), device="cuda")
    B.tpi_lm_head(gt, wh, xt, logits)
    torch.cuda.synchronize()
    ref = O.lm_head(g, w_head, x)
    e = rel_err(logits.cpu().numpy(), ref)
    assert e <= FP32_TOL, f"logits rel err {e:.3e}"


@pytest.mark.parametrize("vocab", [1, 7, 1024, 1025, 32000, 128256])
def test_softmax_and_token_choice(vocab):
    rng = np.random.default_rng(vocab)
    z = (rng.standard_normal(vocab) * 3).astype(np.float32)
    if vocab > 4:
        z[vocab // 2] = z[vocab // 2 + 1] = z.max() + 1.0       # two equal largest logits: the lower index wins
    zt = torch.from_numpy(z).cuda()
    probs = torch.full((vocab,), float("nan"), device="cuda")
    tok = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    B.tpi_next_token(zt, -1.0, tok, probs=probs)
    torch.cuda.synchronize()
    p64 = O.softmax(z)
    assert rel_err(probs.cpu().numpy(), p64) <= FP32_TOL
    # the decision is taken on the same fp32 logits on both sides: exactly one index is right
    assert int(tok.item()) == O.greedy_token(z)
    cdf = np.cumsum(p64)
    eps = 1e-5      # fp32 cumulative sums of up to 128256 terms against the fp64 ones
    for u in (0.0, 0.1, 0.5, 0.9, 0.999999):
        B.tpi_next_token(zt, u, tok)
        torch.cuda.synchronize()
        k = int(tok.item())
        assert 0 <= k < vocab
        # valid inverse-CDF answer up to rounding: cdf[k-1] <= u < cdf[k]
        assert (cdf[k] > u - eps or k == vocab - 1) and (k == 0 or cdf[k - 1] <= u + eps), (u, k, cdf[max(k - 1, 0)], cdf[k])
        ko = O.sample_token(z, u)
        assert abs(cdf[k] - cdf[ko]) <= 2 * eps + p64[k] + p64[ko]


def test_sampling_frequencies_follow_the_distribution():
    vocab = 37
    rng = np.random.default_rng(5)
    z = rng.standard_normal(vocab).astype(np.float32)
    zt = torch.from_numpy(z).cuda()
    tok = torch.empty(1, dtype=torch.int32, device="cuda")
    n = 4000
    counts = np.zeros(vocab)
    for i in range(n):
        B.tpi_next_token(zt, (i + 0.5) / n, tok)
        counts[int(tok.item())] += 1
    np.testing.assert_allclose(counts / n, O.softmax(z), atol=2.0 / n)


@pytest.mark.parametrize("vocab", [1, 5, 1024, 4097])
def test_greedy_choice_when_no_logit_is_finite(vocab):
    # every logit -inf: nothing compares greater, so the first index is the answer on both sides and the
    # token stays inside [0, vocab)
    z = np.full(vocab, -np.inf, dtype=np.float32)
    tok = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    B.tpi_next_token(torch.from_numpy(z).cuda(), -1.0, tok)
    torch.cuda.synchronize()
    assert int(tok.item()) == O.greedy_token(z) == 0
    # one finite logit among them is found wherever it lies
    for at in sorted({0, vocab // 2, vocab - 1}):
        z2 = z.copy(); z2[at] = -3.0e38
        B.tpi_next_token(torch.from_numpy(z2).cuda(), -1.0, tok)
        torch.cuda.synchronize()
        assert int(tok.item()) == O.greedy_token(z2) == at
