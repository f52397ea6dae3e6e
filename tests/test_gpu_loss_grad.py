"""GPU parity of remoe_loss_backward (Eq. 2-12 differentiated through the softmax) and remoe_gate_grad
(dz^T x) against the fp64 oracle."""
import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LAGS = [1, 2, 4, 8, 16]


def _say(msg):
    print(msg, flush=True)


def _inputs(seed, S, T, N, K, rho=0.8):
    g = torch.Generator().manual_seed(seed)
    z = torch.empty(S, T, N)
    z[:, 0] = torch.randn(S, N, generator=g)
    for t in range(1, T):                                   # AR(1) logits: adjacent steps are correlated
        z[:, t] = rho * z[:, t - 1] + (1 - rho * rho) ** 0.5 * torch.randn(S, N, generator=g)
    P = torch.softmax(2.0 * z, -1)
    Q = torch.softmax(2.0 * z + 0.2 * torch.randn(S, T, N, generator=g), -1)
    idx = torch.topk(P, K, -1).indices.int()
    return P.contiguous(), Q.contiguous(), idx.contiguous()


def _backward(P, Q, idx, lags, window, coef):
    S, T, N = P.shape
    p, q, i = P.to(DEV), Q.to(DEV), idx.to(DEV)
    vals = torch.zeros(S, 6, dtype=torch.float64, device=DEV)
    ws = torch.empty(remoe.remoe_loss_workspace_bytes(S), dtype=torch.uint8, device=DEV)
    remoe.remoe_loss_forward(p, q, i, list(lags), window, vals, ws)
    dz = torch.full((S, T, N), float("nan"), dtype=torch.float32, device=DEV)
    ws2 = torch.empty(remoe.remoe_loss_backward_workspace_bytes(S, T, N, window), dtype=torch.uint8, device=DEV)
    remoe.remoe_loss_backward(p, q, i, list(lags), window, coef, vals, dz, ws2)
    torch.cuda.synchronize()
    return dz


def _check_grad(P, Q, idx, lags, window, coef):
    got = _backward(P, Q, idx, lags, window, coef).cpu().double()
    want = oracle.remoe_loss_grad(P, Q, idx, lags, window, coef)
    scale = want.abs().max().item() + 1e-300
    err = (got - want).abs().max().item()
    # fp64 arithmetic on both sides, one rounding to fp32 on the device side
    assert err <= 1.5e-7 * scale, (err, scale)
    return err / scale


@pytest.mark.parametrize("S,T,N,K,window,lags", [
    (2, 37, 16, 2, 5, [1, 2, 4]),            # ragged last window, small N
    (3, 300, 60, 4, 16, LAGS),               # several chunks of steps, N not a multiple of 32
    (1, 1, 64, 6, 1, LAGS),                  # a single step: only the trust and window terms exist
    (2, 9, 128, 8, 4, [1, 16]),              # a lag longer than the sequence
    (1, 70, 128, 8, 100, []),                # no lag term, no complete window
])
@pytest.mark.parametrize("coef", [[1.0, 1.0, 1.0, 1.0, 1.0], [0.3, 0.0, 2.0, 0.5, 0.0]])
def test_loss_backward_matches_oracle(S, T, N, K, window, lags, coef):
    _say(f"loss backward S={S} T={T} N={N} K={K} W={window} lags={lags} coef={coef}")
    P, Q, idx = _inputs(40 + T, S, T, N, K)
    rel = _check_grad(P, Q, idx, lags, window, coef)
    _say(f"  worst error / largest gradient {rel:.2e}")


def test_loss_backward_full_size():
    """The prefill workload's shape: 16 sequences of 4096 steps, 128 experts, K = 8."""
    S, T, N, K = 16, 4096, 128, 8
    _say(f"loss backward full size S={S} T={T} N={N} K={K}")
    P, Q, idx = _inputs(7, S, T, N, K)
    rel = _check_grad(P, Q, idx, LAGS, 64, [1.0, 0.1, 0.5, 0.5, 0.2])
    _say(f"  worst error / largest gradient {rel:.2e}")


def _gate_grad(dz, x):
    T, N = dz.shape
    H = x.shape[1]
    dw = torch.full((N, H), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(remoe.remoe_gate_grad_workspace_bytes(T, N, H), dtype=torch.uint8, device=DEV)
    remoe.remoe_gate_grad(dz, x, dw, ws)
    torch.cuda.synchronize()
    return dw


@pytest.mark.parametrize("T,N,H,dt", [
    (100, 16, 256, torch.float32),
    (333, 60, 512, torch.bfloat16),          # N not a multiple of 32, odd token count
    (1, 128, 128, torch.bfloat16),           # one token: an outer product
    (4099, 128, 2048, torch.bfloat16),       # many chunks, ragged
    (257, 8, 64, torch.float32),
])
def test_gate_grad_matches_oracle(T, N, H, dt):
    _say(f"gate grad T={T} N={N} H={H} {dt}")
    g = torch.Generator().manual_seed(T + N)
    dz = (torch.randn(T, N, generator=g) * 1e-3).contiguous()
    x = torch.randn(T, H, generator=g).to(dt).contiguous()
    got = _gate_grad(dz.to(DEV), x.to(DEV)).cpu().double()
    want = oracle.gate_grad(dz, x)
    bound = dz.double().abs().T @ x.double().abs()           # sum of |terms| per entry
    err = ((got - want).abs() / (bound + 1e-300)).max().item()
    # fp32 products are exact in fp32 MFMA inputs' precision; accumulation error grows with the chunk length
    assert err <= 2e-6, err
    _say(f"  worst error / sum of |terms| {err:.2e}")


def test_gate_grad_full_size_sampled_and_repeatable():
    T, N, H = 65536, 128, 2048
    _say(f"gate grad full size T={T} N={N} H={H} bf16")
    g = torch.Generator(device=DEV).manual_seed(11)
    dz = (torch.randn(T, N, generator=g, device=DEV) * 1e-3).contiguous()
    x = torch.randn(T, H, generator=g, device=DEV).bfloat16().contiguous()
    a = _gate_grad(dz, x)
    b = _gate_grad(dz, x)
    assert torch.equal(a.view(torch.int32), b.view(torch.int32)), "the fixed summation order must repeat bit for bit"
    pick = torch.stack([torch.randint(0, N, (96,), generator=torch.Generator().manual_seed(1)),
                        torch.randint(0, H, (96,), generator=torch.Generator().manual_seed(2))], 1).int()
    pick[0] = torch.tensor([0, 0])
    pick[1] = torch.tensor([N - 1, H - 1])
    dzc, xc = dz.cpu(), x.cpu()
    want = oracle.gate_grad(dzc, xc, pick)
    got = a.cpu().double()[pick[:, 0].long(), pick[:, 1].long()]
    bound = (dzc.double()[:, pick[:, 0].long()].abs() * xc.double()[:, pick[:, 1].long()].abs()).sum(0)
    err = ((got - want).abs() / bound).max().item()
    assert err <= 2e-6, err
    _say(f"  worst error / sum of |terms| over 96 sampled entries {err:.2e}")


def test_backward_and_gate_grad_reject_bad_arguments():
    P, Q, idx = _inputs(1, 1, 8, 16, 2)
    p, q, i = P.to(DEV), Q.to(DEV), idx.to(DEV)
    vals = torch.zeros(1, 6, dtype=torch.float64, device=DEV)
    dz = torch.zeros(1, 8, 16, device=DEV)
    ws = torch.empty(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(remoe.RemoeError, match="lag"):
        remoe.remoe_loss_backward(p, q, i, [0], 4, [1, 1, 1, 1, 1], vals, dz, ws)
    with pytest.raises(remoe.RemoeError, match="window"):
        remoe.remoe_loss_backward(p, q, i, [1], 0, [1, 1, 1, 1, 1], vals, dz, ws)
    with pytest.raises(remoe.RemoeError, match="coef"):
        remoe.remoe_loss_backward(p, q, i, [1], 4, [1, float("nan"), 1, 1, 1], vals, dz, ws)
    with pytest.raises(remoe.RemoeError, match="workspace"):
        remoe.remoe_loss_backward(p, q, i, [1], 1, [1, 1, 1, 1, 1], vals, dz, ws[:8])
    x = torch.zeros(8, 96, device=DEV)
    dw = torch.zeros(16, 96, device=DEV)
    with pytest.raises(remoe.RemoeError, match="hidden"):
        remoe.remoe_gate_grad(dz[0], x, dw, torch.empty(1 << 20, dtype=torch.uint8, device=DEV))
    x = torch.zeros(8, 128, device=DEV)
    with pytest.raises(remoe.RemoeError, match="workspace"):
        remoe.remoe_gate_grad(dz[0], x, torch.zeros(16, 128, device=DEV), ws[:16])
