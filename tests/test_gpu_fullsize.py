"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

One layer of each batched configuration runs at its real token count.  The oracle cannot redo
65,536 tokens of a 2048-wide layer in test time, so routing and layer outputs are compared on an
evenly spaced sample of tokens it evaluates one by one, properties that hold for every token are
checked on all of them, and the trace statistics (pure integer functions of the expert ids) are
compared bit for bit on the complete traces.
"""
import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe
import workload as wl
from helpers import check_output, compare_routing, to_oracle_weights

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def _forward(cfg, layer, rho):
    desc = remoe.LayerDesc.from_config(cfg)
    T, H, K = cfg.n_tokens, cfg.hidden, cfg.top_k
    w = wl.layer_weights(cfg, layer, DEV)
    x = wl.hidden_states(cfg, rho, device=DEV).reshape(T, H).contiguous()
    ws = torch.empty(remoe.remoe_workspace_bytes(desc, T), dtype=torch.uint8, device=DEV)
    y = torch.full((T, H), float("nan"), dtype=desc.torch_dtype, device=DEV)
    idx = torch.full((T, K), -1, dtype=torch.int32, device=DEV)
    gw = torch.full((T, K), float("nan"), dtype=torch.float32, device=DEV)
    remoe.moe_forward(desc, x, w["w_router"], w["w_gate"], w["w_up"], w["w_down"], w["ws_gate"], w["ws_up"],
                      w["ws_down"], w["ws_scale"], y, idx, gw, ws)
    torch.cuda.synchronize()
    return desc, w, x, y, idx, gw


def _check_layer(cfg, layer, rho, n_route, n_out):
    _say(f"full size {cfg.name} layer {layer} rho {rho}: {cfg.n_tokens} tokens")
    desc, w, x, y, idx, gw = _forward(cfg, layer, rho)
    T, K, N = cfg.n_tokens, cfg.top_k, cfg.n_experts
    # ---- properties of every token
    assert torch.isfinite(y.float()).all()
    assert (idx >= 0).all() and (idx < N).all()
    srt = torch.sort(idx, 1).values
    assert (srt[:, 1:] != srt[:, :-1]).all(), "a token selected an expert twice"
    assert (gw[:, :-1] >= gw[:, 1:]).all(), "gate weights are not in descending order"
    sums = gw.sum(1)
    if cfg.renorm:
        assert torch.allclose(sums, torch.ones_like(sums), atol=1e-5)
    else:
        assert (sums < 1.0 + 1e-6).all() and (gw > 0).all()
    counts = torch.bincount(idx.flatten().long(), minlength=N)
    assert int(counts.sum()) == T * K
    # ---- routing on a sample the oracle recomputes
    wc = to_oracle_weights(w)
    r_tok = torch.arange(n_route, dtype=torch.int64) * (T // n_route) + (T // n_route) // 2
    orc = oracle.route(x[r_tok.to(DEV)].cpu(), wc["w_router"], K, cfg.renorm, want_probs=True)
    ties, exp_w = compare_routing(idx[r_tok.to(DEV)], gw[r_tok.to(DEV)], orc, cfg.renorm)
    # ---- layer output on a smaller sample (the GPU's expert choice, the oracle's gate weights)
    o_tok = r_tok[:: max(1, n_route // n_out)][:n_out]
    sel = torch.searchsorted(r_tok, o_tok)
    xs = x[o_tok.to(DEV)].cpu()
    y_ref = oracle.experts_sparse(xs, idx[o_tok.to(DEV)].cpu(), exp_w[sel], wc)
    err = check_output(y[o_tok.to(DEV)], y_ref, cfg.dtype)
    _say(f"  {n_route} routed / {len(o_tok)} evaluated sample tokens: rel L2 {err:.3e}, tie tokens {len(ties)}")
    # ---- trace statistics on the complete trace of this layer
    tr = idx.view(cfg.n_seq, cfg.seq_len, K)
    S, Ts = cfg.n_seq, cfg.seq_len
    ov = torch.empty(S, Ts, dtype=torch.uint8, device=DEV)
    osum = torch.empty(S, dtype=torch.int64, device=DEV)
    miss = torch.empty(S, Ts, dtype=torch.uint8, device=DEV)
    tot = torch.empty(S, dtype=torch.int64, device=DEV)
    nb = torch.empty(S, dtype=torch.int64, device=DEV)
    remoe.trace_reuse(tr, N, ov, osum)
    remoe.lru_simulate(tr, N, cfg.capacities[0], cfg.expert_bytes, 0, None, miss, tot, nb)
    torch.cuda.synchronize()
    trc = tr.cpu()
    rov, rsum = oracle.trace_reuse(trc, N)
    rmiss, rtot, rnb = oracle.lru_list(trc, N, cfg.capacities[0], cfg.expert_bytes)
    assert torch.equal(ov.cpu(), rov) and torch.equal(osum.cpu(), rsum)
    assert torch.equal(miss.cpu(), rmiss) and torch.equal(tot.cpu(), rtot) and torch.equal(nb.cpu(), rnb)
    # Prop. 3.1 on real traces: with C >= K every step fetches at most K - overlap experts
    assert (miss[:, 1:].cpu() <= K - ov[:, 1:].cpu()).all()
    return float(rsum.sum()) / (K * (Ts - 1) * S)


def test_dsv2lite_full_layer():
    cfg = wl.get_config("dsv2lite")
    assert cfg.expert_bytes == 17_301_504
    _check_layer(cfg, 0, 0.8, n_route=2048, n_out=48)


def test_qwen15moe_full_layer_both_correlations():
    cfg = wl.get_config("qwen15moe")
    eor0 = _check_layer(cfg, 1, 0.0, n_route=2048, n_out=32)
    eor8 = _check_layer(cfg, 1, 0.8, n_route=2048, n_out=32)
    # independent steps overlap by K/N on average; correlated hidden states by much more
    assert abs(eor0 - cfg.top_k / cfg.n_experts) < 0.01
    assert eor8 > 3 * eor0


def test_qwen3_prefill_full_layers():
    cfg = wl.get_config("qwen3_prefill")
    assert cfg.expert_bytes == 9_437_184
    _check_layer(cfg, 0, 0.8, n_route=4096, n_out=64)
    _check_layer(cfg, 47, 0.8, n_route=2048, n_out=32)


def test_qwen3_decode_full_stack():
    """All 48 layers resident (54 GiB), launches of 128 steps as bench.py times them.  Every layer-step's
    statistics are compared bit for bit on the complete traces; routing and layer outputs on the
    layers the oracle is given (it evaluates their tokens one by one)."""
    cfg = wl.get_config("qwen3_decode")
    L, H, K, N = cfg.n_layers, cfg.hidden, cfg.top_k, cfg.n_experts
    T = 256                                      # two launches of 128 steps
    caps = list(cfg.capacities)
    _say(f"full size {cfg.name}: {L} layers x {T} steps")
    desc = remoe.LayerDesc.from_config(cfg)
    x = wl.hidden_states(cfg, cfg.rhos[-1], device=DEV).reshape(cfg.seq_len, H)[:T].contiguous()
    weights = [wl.layer_weights(cfg, l, device=DEV) for l in range(L)]
    table = torch.tensor([[w["w_router"].data_ptr(), w["w_gate"].data_ptr(), w["w_up"].data_ptr(),
                           w["w_down"].data_ptr()] for w in weights], dtype=torch.int64, device=DEV)
    y = torch.full((T, L, H), float("nan"), dtype=torch.bfloat16, device=DEV)
    idx = torch.full((L, T, K), -1, dtype=torch.int32, device=DEV)
    gw = torch.full((L, T, K), float("nan"), dtype=torch.float32, device=DEV)
    state = torch.zeros(L, N, dtype=torch.int32, device=DEV)
    ov = torch.full((L, T), 255, dtype=torch.uint8, device=DEV)
    miss = torch.full((len(caps), L, T), 255, dtype=torch.uint8, device=DEV)
    sum_ov = torch.zeros(L, dtype=torch.int64, device=DEV)
    tot = torch.zeros(len(caps), L, dtype=torch.int64, device=DEV)
    nbytes = torch.zeros(len(caps), L, dtype=torch.int64, device=DEV)
    ws = torch.zeros(remoe.remoe_decode_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    for pos in range(0, T, 128):
        remoe.moe_decode(desc, table, x, pos, 128, y, idx, gw, caps, cfg.expert_bytes, state, ov, miss, sum_ov, tot,
                         nbytes, ws, 0, remoe.REMOE_DECODE_PIPELINED)
    torch.cuda.synchronize()
    assert int(ws[128:132].view(torch.int32)[0]) == 0, "a wait inside the kernel timed out"
    # ---- properties of every layer-step
    assert torch.isfinite(y.float()).all()
    assert (idx >= 0).all() and (idx < N).all()
    srt = torch.sort(idx, 2).values
    assert (srt[..., 1:] != srt[..., :-1]).all(), "a step selected an expert twice"
    assert torch.allclose(gw.sum(2), torch.ones(L, T, device=DEV), atol=1e-5)
    # ---- statistics, complete traces
    tr = idx.cpu()
    rov, rsum = oracle.trace_reuse(tr, N)
    assert torch.equal(ov.cpu(), rov) and torch.equal(sum_ov.cpu(), rsum)
    for c, cap in enumerate(caps):
        rmiss, rtot, rb = oracle.lru_list(tr, N, cap, cfg.expert_bytes)
        assert torch.equal(miss[c].cpu(), rmiss), f"LRU misses differ at capacity {cap}"
        assert torch.equal(tot[c].cpu(), rtot) and torch.equal(nbytes[c].cpu(), rb)
    # ---- routing and outputs of sampled layers (first, one of a group with uneven position, last)
    xc = x.cpu()
    steps = torch.tensor([0, 1, 63, 127, 128, 200, 255])
    worst = 0.0
    for l in (0, 13, 47):
        wc = to_oracle_weights(weights[l])
        orc = oracle.route(xc, wc["w_router"], K, cfg.renorm, want_probs=True)
        _, exp_w = compare_routing(idx[l], gw[l], orc, cfg.renorm)
        y_ref = oracle.experts_sparse(xc[steps], idx[l].cpu()[steps], exp_w[steps], wc)
        worst = max(worst, check_output(y[steps.to(DEV), l], y_ref, cfg.dtype))
    _say(f"  3 layers x {T} steps routed, {len(steps)} steps each evaluated: worst rel L2 {worst:.3e}")
