"""Pins of the ReMoE loss oracle (Eq. 2-12): closed forms, library routines in fp64, identities."""
import math

import pytest
import torch

import oracle

LAGS = (1, 2, 4, 8, 16)


def _dists(seed, S, T, N, temp=1.5):
    g = torch.Generator().manual_seed(seed)
    return torch.softmax(torch.randn(S, T, N, generator=g) * temp, -1).float().contiguous()


def _topk(p, K):
    return torch.topk(p, K, dim=-1).indices.to(torch.int32).contiguous()


def test_identical_and_constant_distributions():
    S, T, N, K = 2, 40, 16, 4
    row = _dists(1, S, 1, N)
    p = row.expand(S, T, N).contiguous()                  # the same distribution at every step
    idx = _topk(p, K)
    out = oracle.remoe_losses(p, p, idx, LAGS, 8)
    m = torch.gather(row[:, 0].double(), -1, idx[:, 0].long()).sum(-1) / K
    assert torch.allclose(out[:, 0], m, rtol=1e-14)                      # rho = mass of the top-K set / K
    assert torch.allclose(out[:, 1], -torch.log(m + 1e-8), rtol=1e-14)
    assert out[:, 2].abs().max() == 0 and out[:, 3].abs().max() == 0 and out[:, 4].abs().max() == 0
    h = torch.special.entr(row[:, 0].double()).sum(-1)
    assert torch.allclose(out[:, 5], h, rtol=1e-12)                      # the window mean is the distribution itself


def test_uniform_distribution_closed_forms():
    S, T, N, K = 1, 33, 8, 2
    p = torch.full((S, T, N), 1.0 / N, dtype=torch.float32)
    idx = torch.zeros(S, T, K, dtype=torch.int32); idx[..., 1] = 1
    out = oracle.remoe_losses(p, p, idx, LAGS, 4)[0]
    assert abs(float(out[0]) - 1.0 / N) < 1e-15 and abs(float(out[1]) + math.log(1.0 / N + 1e-8)) < 1e-14
    assert abs(float(out[5]) - math.log(N)) < 1e-14 and float(out[3]) == 0.0


@pytest.mark.parametrize("S,T,N,K,W", [(2, 50, 16, 4, 8), (1, 37, 64, 6, 16), (3, 20, 5, 2, 3)])
def test_against_torch_library_routines(S, T, N, K, W):
    p, q = _dists(S + T, S, T, N), _dists(S + T + 1, S, T, N)
    idx = _topk(p, K)
    out = oracle.remoe_losses(p, q, idx, LAGS, W)
    pd, qd = p.double(), q.double()
    kl = lambda a, b: torch.nn.functional.kl_div(b.log(), a, reduction="none").sum(-1)     # KL(a || b)
    sym = lambda a, b: 0.5 * (kl(a, b) + kl(b, a))
    for s in range(S):
        trust = kl(pd[s], qd[s]).mean()
        smooth = sym(pd[s, 1:], pd[s, :-1]).sum() / (T - 1)
        lag = sum(sym(pd[s, d:], pd[s, :-d]).sum() for d in LAGS if d < T) / len(LAGS) / (T - 1)
        m = torch.gather(pd[s, 1:], -1, idx[s, :-1].long()).sum(-1) / K
        n = T // W
        bar = pd[s, :n * W].reshape(n, W, N).mean(1)
        ws = torch.special.entr(bar).sum(-1).mean()
        want = torch.stack([m.mean(), -torch.log(m.mean() + 1e-8), trust, smooth, lag, ws])
        assert torch.allclose(out[s], want, rtol=1e-11, atol=1e-14), (out[s], want)


def test_lag_with_single_unit_lag_is_smoothness_and_missing_partners_are_left_out():
    p = _dists(5, 2, 30, 12)
    idx = _topk(p, 3)
    a = oracle.remoe_losses(p, p, idx, (1,), 4)
    assert torch.allclose(a[:, 4], a[:, 3], rtol=1e-15)
    # lags longer than the sequence have no partner anywhere: they only count in the 1/|D| normalisation
    b = oracle.remoe_losses(p, p, idx, (1, 64), 4)
    assert torch.allclose(b[:, 4], a[:, 3] / 2, rtol=1e-15)


def test_short_sequences_and_windows():
    p = _dists(6, 1, 1, 8)
    out = oracle.remoe_losses(p, p, _topk(p, 2), LAGS, 4)[0]
    assert float(out[0]) == 0.0 and abs(float(out[1]) + math.log(1e-8)) < 1e-12
    assert float(out[3]) == 0.0 and float(out[4]) == 0.0 and float(out[5]) == 0.0     # no pair, no full window
