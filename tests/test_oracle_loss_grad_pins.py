"""Pins of the oracle's loss gradient (Eq. 2-12 differentiated through the softmax) and gate gradient.

The gradient in the oracle is written out by hand term by term.  Here the same losses are written
once more as differentiable tensor expressions and differentiated by torch.autograd in fp64; the
oracle's forward function is also differenced numerically.  A wrong sign, a missing partner in the
symmetric terms, a wrong normaliser or a dropped softmax projection fails at least one of these.
"""
import math

import pytest
import torch

import oracle

LAGS = [1, 2, 4]


def _inputs(seed, S, T, N, K, scale=1.5):
    g = torch.Generator().manual_seed(seed)
    z = scale * torch.randn(S, T, N, dtype=torch.float64, generator=g)
    zr = z + 0.3 * torch.randn(S, T, N, dtype=torch.float64, generator=g)
    P = torch.softmax(z, -1)
    idx = torch.topk(P, K, -1).indices.int()
    return z, torch.softmax(zr, -1).float(), idx


def _symkl(p, q):
    return 0.5 * ((p * (p / q).log()).sum(-1) + (q * (q / p).log()).sum(-1))


def _losses_autograd(P, Pref, idx, lags, window):
    """[S, 5] differentiable: Reuse, Trust, Smooth, Lag, WS from P [S, T, N] fp64."""
    S, T, N = P.shape
    K = idx.shape[2]
    zero = P.sum() * 0.0
    if T > 1:
        m = torch.gather(P[:, 1:], 2, idx[:, :-1].long()).sum(-1) / K          # m_t, t >= 2; E_{t-1} constant
        reuse = -(m.mean(1) + 1e-8).log()
        smooth = _symkl(P[:, 1:], P[:, :-1]).mean(1)
        lag = torch.zeros(S, dtype=P.dtype)
        for d in lags:
            if d < T:
                lag = lag + _symkl(P[:, d:], P[:, :-d]).sum(1)
        lag = lag / ((T - 1) * len(lags)) if lags else lag * 0
    else:
        reuse = -(torch.zeros(S, dtype=P.dtype) + 1e-8).log() + zero
        smooth = torch.zeros(S, dtype=P.dtype) + zero
        lag = torch.zeros(S, dtype=P.dtype) + zero
    trust = (P * (P / Pref).log()).sum(-1).mean(1)
    n = T // window
    if n > 0:
        bar = P[:, : n * window].reshape(S, n, window, N).mean(2)
        ws = torch.special.entr(bar).sum(-1).mean(1)
    else:
        ws = torch.zeros(S, dtype=P.dtype) + zero
    return torch.stack([reuse, trust, smooth, lag, ws], 1)


def _autograd_grad(z, Pref, idx, lags, window, coef):
    z = z.clone().requires_grad_(True)
    P = torch.softmax(z, -1)
    P32 = P.detach().float().double()
    Pv = P32 + (P - P.detach())                  # the fp32-rounded values the oracle sees, exact Jacobian
    L = (_losses_autograd(Pv, Pref.double(), idx, lags, window) * torch.tensor(coef, dtype=torch.float64)).sum()
    L.backward()
    return z.grad, P32.float()


@pytest.mark.parametrize("coef", [[1, 0, 0, 0, 0], [0, 1, 0, 0, 0], [0, 0, 1, 0, 0], [0, 0, 0, 1, 0], [0, 0, 0, 0, 1],
                                  [0.7, 0.1, 1.3, 0.4, 2.0]])
@pytest.mark.parametrize("S,T,N,K,window", [(2, 13, 8, 2, 4), (1, 40, 60, 4, 7), (3, 5, 16, 4, 5), (1, 9, 128, 8, 1)])
def test_grad_matches_autograd(coef, S, T, N, K, window):
    z, Pref, idx = _inputs(10 + T, S, T, N, K)
    want, P32 = _autograd_grad(z, Pref, idx, LAGS, window, coef)
    got = oracle.remoe_loss_grad(P32, Pref, idx, LAGS, window, coef)
    scale = want.abs().max().item() + 1e-30
    assert (got - want).abs().max().item() <= 2e-6 * scale, ((got - want).abs().max().item(), scale)


def test_forward_of_the_autograd_expression_is_the_oracle_forward():
    """The differentiable expression used above is the same function as oracle.remoe_losses."""
    z, Pref, idx = _inputs(3, 2, 24, 16, 4)
    P32 = torch.softmax(z, -1).float()
    a = _losses_autograd(P32.double(), Pref.double(), idx, LAGS, 6)
    b = oracle.remoe_losses(P32, Pref, idx, LAGS, 6)[:, 1:]
    assert torch.allclose(a, b, rtol=1e-12, atol=1e-14)


def test_grad_matches_central_differences_of_the_oracle_forward():
    S, T, N, K, W = 1, 11, 8, 2, 3
    coef = [0.5, 1.0, 0.8, 0.6, 1.5]
    z, Pref, idx = _inputs(21, S, T, N, K, scale=1.0)
    P32 = torch.softmax(z, -1).float()
    got = oracle.remoe_loss_grad(P32, Pref, idx, LAGS, W, coef)
    c = torch.tensor(coef, dtype=torch.float64)

    def total(zz):
        return float((oracle.remoe_losses(torch.softmax(zz, -1).float(), Pref, idx, LAGS, W)[0, 1:] * c).sum())

    h = 2e-3
    for (t, k) in [(0, 0), (1, 3), (4, 7), (5, int(idx[0, 4, 0])), (10, 2), (9, int(idx[0, 8, 1]))]:
        zp, zm = z.clone(), z.clone()
        zp[0, t, k] += h
        zm[0, t, k] -= h
        fd = (total(zp) - total(zm)) / (2 * h)
        assert abs(fd - float(got[0, t, k])) < 3e-4, (t, k, fd, float(got[0, t, k]))


def test_single_step_sequence_has_only_the_trust_term_in_closed_form():
    """T = 1: no reuse, smoothness or lag partner exists; with W = 2 no window is complete.  Then
    dL/dz = c_trust * P (log(P / Pref) - KL(P || Pref)) (softmax gradient of a KL divergence)."""
    z, Pref, idx = _inputs(5, 2, 1, 16, 4)
    P32 = torch.softmax(z, -1).float()
    got = oracle.remoe_loss_grad(P32, Pref, idx, LAGS, 2, [3.0, 0.25, 5.0, 7.0, 11.0])
    P, Q = P32.double(), Pref.double()
    lr = (P / Q).log()
    want = 0.25 * P * (lr - (P * lr).sum(-1, keepdim=True))
    # (the fp32 probabilities sum to 1 only within rounding: the constant +1 of the KL derivative leaves 1e-8)
    assert torch.allclose(got, want, rtol=1e-6, atol=1e-9)


def test_identical_steps_have_no_smoothness_or_lag_gradient_and_rows_sum_to_zero():
    S, T, N, K = 1, 12, 16, 4
    P = torch.softmax(torch.randn(1, 1, N, dtype=torch.float64, generator=torch.Generator().manual_seed(1)), -1)
    P32 = P.float().expand(S, T, N).contiguous()
    idx = torch.topk(P32, K, -1).indices.int()
    g = oracle.remoe_loss_grad(P32, P32, idx, LAGS, 4, [0, 0, 1, 1, 0])
    assert g.abs().max().item() == 0.0
    g = oracle.remoe_loss_grad(P32, P32, idx, LAGS, 4, [1, 1, 1, 1, 1])
    assert g.sum(-1).abs().max().item() < 1e-6 * g.abs().max().item()       # P32 sums to 1 within fp32 rounding
    # every step reuses the same set: rho = sum of the K largest, reuse gradient pushes mass into the set
    in_set = torch.zeros(N, dtype=torch.bool)
    in_set[idx[0, 0].long()] = True
    gr = oracle.remoe_loss_grad(P32, P32, idx, LAGS, 4, [1, 0, 0, 0, 0])[0, 1:]
    assert (gr[:, in_set] < 0).all() and (gr[:, ~in_set] > 0).all() and gr[0].abs().max() > 0
    assert oracle.remoe_loss_grad(P32, P32, idx, LAGS, 4, [1, 0, 0, 0, 0])[0, 0].abs().max().item() == 0.0


def test_gate_grad_is_a_matrix_product():
    g = torch.Generator().manual_seed(8)
    T, N, H = 37, 12, 20
    dz = torch.randn(T, N, generator=g)
    x = torch.randn(T, H, generator=g).bfloat16()
    want = dz.double().T @ x.double()
    got = oracle.gate_grad(dz, x)
    assert torch.allclose(got, want, rtol=1e-13, atol=1e-13)
    pick = torch.tensor([[0, 0], [11, 19], [5, 7]], dtype=torch.int32)
    assert torch.allclose(oracle.gate_grad(dz, x, pick), want[pick[:, 0].long(), pick[:, 1].long()], rtol=1e-13, atol=1e-13)
    # one token: the outer product
    assert torch.allclose(oracle.gate_grad(dz[:1], x[:1]), torch.outer(dz[0].double(), x[0].double()), rtol=1e-14, atol=0)
