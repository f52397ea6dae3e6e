"""Edge cases through the C ABI on the GPU: empty inputs leave the outputs untouched (or give the
empty sum), single elements work, and a single token or step gives what the oracle gives."""
import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe
import workload as wl
from helpers import check_output, compare_routing, to_oracle_weights

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def _layer(seed, H, N, I, dt):
    g = lambda name, shape, d: wl.gaussian(seed, name, shape, 0.05, 0, 0, d, DEV)
    return {"w_router": g("w_router", (N, H), torch.float32), "w_gate": g("w_gate", (N, I, H), dt),
            "w_up": g("w_up", (N, I, H), dt), "w_down": g("w_down", (N, H, I), dt),
            "ws_gate": None, "ws_up": None, "ws_down": None, "ws_scale": None}


def test_no_tokens_is_a_no_op():
    _say("empty batch: moe_route, moe_forward")
    H, N, I, K = 256, 16, 128, 2
    desc = remoe.LayerDesc(H, N, I, K, 0, 0, 0, 0)
    w = _layer(1, H, N, I, torch.float32)
    x = torch.zeros(0, H, device=DEV)
    idx = torch.full((4, K), -7, dtype=torch.int32, device=DEV)
    gw = torch.full((4, K), -7.0, device=DEV)
    y = torch.full((4, H), -7.0, device=DEV)
    ws = torch.empty(max(remoe.remoe_workspace_bytes(desc, 0), 256), dtype=torch.uint8, device=DEV)
    remoe.moe_route(desc, x, w["w_router"], idx, gw, None, None)
    remoe.moe_forward(desc, x, w["w_router"], w["w_gate"], w["w_up"], w["w_down"], None, None, None, None, y, idx, gw, ws)
    torch.cuda.synchronize()
    assert (idx == -7).all() and (gw == -7).all() and (y == -7).all()


def test_single_token_matches_oracle():
    _say("one token, fp32 and bf16")
    for dt, name in ((torch.float32, "f32"), (torch.bfloat16, "bf16")):
        H, N, I, K = 256, 16, 128, 4
        desc = remoe.LayerDesc(H, N, I, K, 1, 0, 0, 0 if dt == torch.float32 else 1)
        w = _layer(2, H, N, I, dt)
        x = wl.gaussian(2, "x", (1, H), 1.0, 0, 0, dt, DEV)
        idx = torch.empty(1, K, dtype=torch.int32, device=DEV)
        gw = torch.empty(1, K, device=DEV)
        y = torch.empty(1, H, dtype=dt, device=DEV)
        ws = torch.empty(remoe.remoe_workspace_bytes(desc, 1), dtype=torch.uint8, device=DEV)
        remoe.moe_forward(desc, x, w["w_router"], w["w_gate"], w["w_up"], w["w_down"], None, None, None, None, y, idx, gw, ws)
        torch.cuda.synchronize()
        wc = to_oracle_weights(w)
        orc = oracle.route(x.cpu(), wc["w_router"], K, True, want_probs=True)
        _, exp_w = compare_routing(idx, gw, orc, True)
        y_ref = oracle.experts_sparse(x.cpu(), idx.cpu(), exp_w, wc)
        check_output(y, y_ref, name)


def test_empty_traces_and_single_steps():
    _say("empty and one-step traces: trace_reuse, lru_simulate, cache_simulate, routing_balance")
    N, K = 16, 2
    # no traces at all
    e = torch.zeros(0, 5, K, dtype=torch.int32, device=DEV)
    z8 = torch.zeros(0, 5, dtype=torch.uint8, device=DEV)
    z64 = torch.zeros(0, dtype=torch.int64, device=DEV)
    remoe.trace_reuse(e, N, z8, z64)
    remoe.lru_simulate(e, N, 4, 10, 0, None, z8, z64, z64)
    # traces without steps: totals are the empty sum
    e = torch.zeros(3, 0, K, dtype=torch.int32, device=DEV)
    z8 = torch.zeros(3, 0, dtype=torch.uint8, device=DEV)
    s = torch.full((3,), -1, dtype=torch.int64, device=DEV)
    t = torch.full((3,), -1, dtype=torch.int64, device=DEV)
    b = torch.full((3,), -1, dtype=torch.int64, device=DEV)
    remoe.trace_reuse(e, N, z8, s)
    remoe.lru_simulate(e, N, 4, 10, 0, None, z8, t, b)
    torch.cuda.synchronize()
    assert (s == 0).all() and (t == 0).all() and (b == 0).all()
    # one step: no previous step to overlap with, every distinct expert is a miss
    one = torch.tensor([[[3, 9]], [[5, 5]]], dtype=torch.int32, device=DEV)
    ov = torch.full((2, 1), 255, dtype=torch.uint8, device=DEV)
    sm = torch.full((2,), -1, dtype=torch.int64, device=DEV)
    ms = torch.full((2, 1), 255, dtype=torch.uint8, device=DEV)
    tt = torch.full((2,), -1, dtype=torch.int64, device=DEV)
    bb = torch.full((2,), -1, dtype=torch.int64, device=DEV)
    remoe.trace_reuse(one, N, ov, sm)
    remoe.lru_simulate(one, N, 4, 10, 0, None, ms, tt, bb)
    torch.cuda.synchronize()
    rov, rsum = oracle.trace_reuse(one.cpu(), N)
    rmiss, rtot, rb = oracle.lru_list(one.cpu(), N, 4, 10)
    assert torch.equal(ov.cpu(), rov) and torch.equal(sm.cpu(), rsum)
    assert torch.equal(ms.cpu(), rmiss) and torch.equal(tt.cpu(), rtot) and torch.equal(bb.cpu(), rb)
    assert ms.cpu().flatten().tolist() == [2, 1]
    for pol in (remoe.REMOE_CACHE_LRU, remoe.REMOE_CACHE_FIFO, remoe.REMOE_CACHE_LFU, remoe.REMOE_CACHE_BELADY):
        m2 = torch.full((2, 1), 255, dtype=torch.uint8, device=DEV)
        u2 = torch.full((2, 1), 255, dtype=torch.uint8, device=DEV)
        h2 = torch.full((2, 1), 255, dtype=torch.uint8, device=DEV)
        a = torch.full((2,), -1, dtype=torch.int64, device=DEV)
        c = torch.full((2,), -1, dtype=torch.int64, device=DEV)
        d = torch.full((2,), -1, dtype=torch.int64, device=DEV)
        nb = remoe.remoe_cache_workspace_bytes(2, 1, K, pol)
        wsp = torch.empty(max(nb, 16), dtype=torch.uint8, device=DEV) if nb else None
        remoe.cache_simulate(one, N, 4, pol, 10, m2, u2, h2, a, c, d, wsp)
        torch.cuda.synchronize()
        assert m2.cpu().flatten().tolist() == [2, 1] and a.cpu().tolist() == [2, 1] and d.cpu().tolist() == [20, 10]


def test_gate_grad_of_no_tokens_is_zero_and_loss_of_no_sequences_is_a_no_op():
    _say("empty sums: remoe_gate_grad with T = 0, remoe_loss_forward / backward with S = 0")
    N, H = 16, 128
    dz = torch.zeros(0, N, device=DEV)
    x = torch.zeros(0, H, device=DEV)
    dw = torch.full((N, H), 5.0, device=DEV)
    ws = torch.empty(max(remoe.remoe_gate_grad_workspace_bytes(0, N, H), 256), dtype=torch.uint8, device=DEV)
    remoe.remoe_gate_grad(dz, x, dw, ws)
    torch.cuda.synchronize()
    assert (dw == 0).all()
    p = torch.zeros(0, 4, N, device=DEV)
    i = torch.zeros(0, 4, 2, dtype=torch.int32, device=DEV)
    out = torch.full((1, 6), 3.0, dtype=torch.float64, device=DEV)
    wsl = torch.empty(256, dtype=torch.uint8, device=DEV)
    remoe.remoe_loss_forward(p, p, i, [1], 2, out, wsl)
    remoe.remoe_loss_backward(p, p, i, [1], 2, [1, 1, 1, 1, 1], out, p, wsl)
    torch.cuda.synchronize()
    assert (out == 3.0).all()


def test_decode_of_no_steps_is_a_no_op():
    _say("moe_decode with n_steps = 0")
    H, N, I, K, L = 512, 16, 64, 4, 2
    desc = remoe.LayerDesc(H, N, I, K, 1, 0, 0, 1)
    ws = torch.zeros(remoe.remoe_decode_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    w = [_layer(3 + l, H, N, I, torch.bfloat16) for l in range(L)]
    table = torch.tensor([[v["w_router"].data_ptr(), v["w_gate"].data_ptr(), v["w_up"].data_ptr(), v["w_down"].data_ptr()]
                          for v in w], dtype=torch.int64, device=DEV)
    x = torch.zeros(4, H, dtype=torch.bfloat16, device=DEV)
    y = torch.full((4, L, H), 9.0, dtype=torch.bfloat16, device=DEV)
    idx = torch.full((L, 4, K), -3, dtype=torch.int32, device=DEV)
    gw = torch.full((L, 4, K), -3.0, device=DEV)
    st = torch.zeros(L, N, dtype=torch.int32, device=DEV)
    ov = torch.full((L, 4), 77, dtype=torch.uint8, device=DEV)
    ms = torch.full((1, L, 4), 77, dtype=torch.uint8, device=DEV)
    z = torch.zeros(L, dtype=torch.int64, device=DEV)
    z1 = torch.zeros(1, L, dtype=torch.int64, device=DEV)
    for order in (remoe.REMOE_DECODE_CHAINED, remoe.REMOE_DECODE_PIPELINED):
        remoe.moe_decode(desc, table, x, 2, 0, y, idx, gw, [4], 1, st, ov, ms, z, z1, z1.clone(), ws, 0, order)
        torch.cuda.synchronize()
        assert (y == 9.0).all() and (idx == -3).all() and (ov == 77).all() and (ms == 77).all() and (z == 0).all()
