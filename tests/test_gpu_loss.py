"""GPU parity of remoe_loss_forward (Eq. 2-12) against the fp64 oracle.

Both sides work in fp64 from the same fp32 probabilities; they differ only in the order of the
additions (the kernel adds per lane, per wavefront, per chunk), so the bound is 1e-11 relative.
"""
import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe
import workload as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LAGS = (1, 2, 4, 8, 16)


def _dists(seed, S, T, N, temp=1.5, rho=0.8):
    """Softmax of AR(1) logits: neighbouring steps resemble each other, as routing distributions do."""
    g = torch.Generator().manual_seed(seed)
    z = torch.randn(S, T, N, generator=g)
    for t in range(1, T):
        z[:, t] = rho * z[:, t - 1] + (1 - rho * rho) ** 0.5 * z[:, t]
    return torch.softmax(z * temp, -1).float().contiguous()


def _run(p, q, idx, lags, window):
    S = p.shape[0]
    out = torch.full((S, 6), float("nan"), dtype=torch.float64, device=DEV)
    ws = torch.empty(remoe.remoe_loss_workspace_bytes(S), dtype=torch.uint8, device=DEV)
    remoe.remoe_loss_forward(p.to(DEV), q.to(DEV), idx.to(DEV), list(lags), window, out, ws)
    torch.cuda.synchronize()
    return out.cpu()


@pytest.mark.parametrize("S,T,N,K,lags,W", [
    (2, 50, 16, 4, LAGS, 8),
    (3, 300, 64, 6, LAGS, 32),           # DeepSeek-V2-Lite-shaped router
    (2, 1000, 128, 8, LAGS, 64),         # Qwen3-shaped router: both halves of the expert range, ragged chunks
    (2, 37, 60, 4, (1, 3), 5),           # Qwen1.5-shaped, other lags, windows that do not divide T
    (1, 20, 5, 2, (), 3),                # no lag set
    (2, 1, 8, 2, LAGS, 4),               # a single step
    (1, 2, 8, 2, (2, 16), 1),            # no unit lag: the smoothness term has its own pass
])
def test_losses_match_oracle(S, T, N, K, lags, W):
    print(f"loss S={S} T={T} N={N} K={K} lags={lags} W={W}", flush=True)
    p, q = _dists(S * T + N, S, T, N), _dists(S * T + N + 1, S, T, N, temp=1.2)
    idx = torch.topk(p, K, dim=-1).indices.to(torch.int32).contiguous()
    got = _run(p, q, idx, lags, W)
    ref = oracle.remoe_losses(p, q, idx, lags, W)
    assert torch.allclose(got, ref, rtol=1e-11, atol=1e-13), (got, ref)


def test_losses_of_router_outputs_full_length():
    """Two routers (a gate matrix and a perturbed copy) on a full-length Qwen3-shaped sequence through moe_route,
    then the losses: the chain a fine-tuning step would run, against the oracle on the same probabilities."""
    cfg = wl.get_config("qwen3_prefill")
    S, T, H, N, K = 2, cfg.seq_len, cfg.hidden, cfg.n_experts, cfg.top_k
    x = wl.ar1_hidden_states(cfg.seed, S, T, H, 0.8, torch.bfloat16, DEV).reshape(S * T, H).contiguous()
    w0 = wl.gaussian(cfg.seed, "w_router", (N, H), cfg.weight_std, 0, 0, torch.float32, DEV)
    w1 = (w0 + 0.1 * wl.gaussian(cfg.seed + 1, "w_router", (N, H), cfg.weight_std, 0, 0, torch.float32, DEV)).contiguous()
    desc = remoe.LayerDesc.from_config(cfg)
    idx = torch.empty(S * T, K, dtype=torch.int32, device=DEV)
    gw = torch.empty(S * T, K, dtype=torch.float32, device=DEV)
    p = torch.empty(S * T, N, dtype=torch.float32, device=DEV)
    q = torch.empty(S * T, N, dtype=torch.float32, device=DEV)
    remoe.moe_route(desc, x, w0, idx, gw, None, q)
    remoe.moe_route(desc, x, w1, idx, gw, None, p)
    out = torch.empty(S, 6, dtype=torch.float64, device=DEV)
    ws = torch.empty(remoe.remoe_loss_workspace_bytes(S), dtype=torch.uint8, device=DEV)
    remoe.remoe_loss_forward(p.view(S, T, N), q.view(S, T, N), idx.view(S, T, K), list(LAGS), 64, out, ws)
    torch.cuda.synchronize()
    ref = oracle.remoe_losses(p.view(S, T, N).cpu(), q.view(S, T, N).cpu(), idx.view(S, T, K).cpu(), LAGS, 64)
    assert torch.allclose(out.cpu(), ref, rtol=1e-11, atol=1e-13)
    assert (ref[:, 2] > 0).all() and (ref[:, 0] > 1.0 / N).all()   # the routers differ; the previous set keeps above-average mass


def test_loss_rejects_bad_arguments():
    p = torch.zeros(1, 4, 8, dtype=torch.float32, device=DEV)
    idx = torch.zeros(1, 4, 2, dtype=torch.int32, device=DEV)
    out = torch.zeros(1, 6, dtype=torch.float64, device=DEV)
    ws = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(remoe.RemoeError, match="lag"):
        remoe.remoe_loss_forward(p, p, idx, [0], 4, out, ws)
    with pytest.raises(remoe.RemoeError, match="window"):
        remoe.remoe_loss_forward(p, p, idx, [1], 0, out, ws)
    with pytest.raises(remoe.RemoeError, match="workspace"):
        remoe.remoe_loss_forward(p, p, idx, [1], 4, out, ws[:8])
