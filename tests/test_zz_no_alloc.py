"""moe_decode_static (no workspace, scratch in a static device array) against moe_decode.

Two calls in a row on the same GPU, the second with a smaller input (fewer layers, a narrower
layer and fewer steps), in both layer orders: expert ids, gate weights, overlaps, misses, totals,
bytes and the LRU state must equal moe_decode's bit for bit; layer outputs are produced by the same
kernels with the same arithmetic, so they are compared bit for bit as well, and against the oracle
to the bf16 bound.
"""
import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe
import workload as wl
from helpers import check_output, compare_routing

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _layers(seed, L, H, N, I, std):
    out = []
    for l in range(L):
        g = lambda name, shape, dt: wl.gaussian(seed, name, shape, std, l, 0, dt, DEV)
        out.append({"w_router": g("w_router", (N, H), torch.float32),
                    "w_gate": g("w_gate", (N, I, H), torch.bfloat16),
                    "w_up": g("w_up", (N, I, H), torch.bfloat16),
                    "w_down": g("w_down", (N, H, I), torch.bfloat16)})
    return out


def _buffers(L, T, H, N, K, n_caps):
    return {
        "y": torch.full((T, L, H), float("nan"), dtype=torch.bfloat16, device=DEV),
        "idx": torch.full((L, T, K), -1, dtype=torch.int32, device=DEV),
        "w": torch.full((L, T, K), float("nan"), dtype=torch.float32, device=DEV),
        "state": torch.zeros(L, N, dtype=torch.int32, device=DEV),
        "ov": torch.full((L, T), 255, dtype=torch.uint8, device=DEV),
        "miss": torch.full((n_caps, L, T), 255, dtype=torch.uint8, device=DEV),
        "sum_ov": torch.zeros(L, dtype=torch.int64, device=DEV),
        "tot": torch.zeros(n_caps, L, dtype=torch.int64, device=DEV),
        "bytes": torch.zeros(n_caps, L, dtype=torch.int64, device=DEV),
    }


def _case(seed, L, T, H, N, I, K, caps, pieces, order):
    print(f"no-alloc decode: order={order} L={L} T={T} H={H} N={N} I={I} K={K} caps={caps} pieces={pieces}", flush=True)
    layers = _layers(seed, L, H, N, I, 0.05)
    x = wl.ar1_hidden_states(seed, 1, T, H, 0.9, torch.bfloat16, DEV)[0].contiguous()
    desc = remoe.LayerDesc(H, N, I, K, 1, 0, 0, 1)
    eb = 3 * H * I * 2
    table = torch.tensor([[w["w_router"].data_ptr(), w["w_gate"].data_ptr(), w["w_up"].data_ptr(),
                           w["w_down"].data_ptr()] for w in layers], dtype=torch.int64, device=DEV)
    ref, got = _buffers(L, T, H, N, K, len(caps)), _buffers(L, T, H, N, K, len(caps))
    ws = torch.zeros(remoe.remoe_decode_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    abort = torch.full((1,), 77, dtype=torch.int32, device=DEV)
    assert remoe.remoe_decode_workspace_bytes(desc) <= remoe.remoe_decode_static_bytes()
    pos = 0
    for n in pieces:
        remoe.moe_decode(desc, table, x, pos, n, ref["y"], ref["idx"], ref["w"], caps, eb, ref["state"], ref["ov"],
                         ref["miss"], ref["sum_ov"], ref["tot"], ref["bytes"], ws, 0, order)
        torch.cuda.synchronize()
        remoe.moe_decode_static(desc, table, x, pos, n, got["y"], got["idx"], got["w"], caps, eb, got["state"],
                                got["ov"], got["miss"], got["sum_ov"], got["tot"], got["bytes"], abort, 0, order)
        torch.cuda.synchronize()
        assert int(abort[0]) == 0, "a wait inside the kernel timed out"
        pos += n
    assert int(ws[128:132].view(torch.int32)[0]) == 0
    for k in ("idx", "ov", "miss", "sum_ov", "tot", "bytes", "state"):
        assert torch.equal(ref[k], got[k]), k
    assert torch.equal(ref["w"].view(torch.int32), got["w"].view(torch.int32))
    assert torch.equal(ref["y"].view(torch.int16), got["y"].view(torch.int16))
    # and against the oracle, as for moe_decode itself
    xc = x.cpu()
    for l in range(L):
        wc = {k: v.cpu() for k, v in layers[l].items()}
        orc = oracle.route(xc, wc["w_router"], K, True, want_probs=True)
        _, exp_w = compare_routing(got["idx"][l], got["w"][l], orc, True)
        y_ref = oracle.experts_sparse(xc, got["idx"][l].cpu(), exp_w, wc)
        check_output(got["y"][:, l], y_ref, "bf16")
    tr = got["idx"].cpu()
    rov, rsum = oracle.trace_reuse(tr, N)
    assert torch.equal(got["ov"].cpu(), rov) and torch.equal(got["sum_ov"].cpu(), rsum)
    for c, cap in enumerate(caps):
        rmiss, rtot, rbytes = oracle.lru_list(tr, N, cap, eb)
        assert torch.equal(got["miss"][c].cpu(), rmiss) and torch.equal(got["tot"][c].cpu(), rtot)
        assert torch.equal(got["bytes"][c].cpu(), rbytes)


@pytest.mark.parametrize("order", [remoe.REMOE_DECODE_CHAINED, remoe.REMOE_DECODE_PIPELINED], ids=["chained", "pipelined"])
def test_static_decode_matches_workspace_decode_twice(order):
    # first call: the Qwen3-30B-A3B layer shape, fed in two pieces; second call: a smaller stack
    _case(301, 4, 20, 2048, 128, 768, 8, [16, 32, 64], [12, 8], order)
    _case(302, 2, 9, 512, 16, 64, 4, [4], [9], order)


def test_static_decode_rejects_what_it_cannot_hold():
    z = torch.zeros(64, dtype=torch.int64, device=DEV)
    x = torch.zeros(4, 512, dtype=torch.bfloat16, device=DEV)
    t = torch.zeros(1, 4, dtype=torch.int64, device=DEV)
    desc = remoe.LayerDesc(512, 16, 64, 4, 1, 0, 0, 1)
    with pytest.raises(remoe.RemoeError, match="out_abort"):
        remoe.moe_decode_static(desc, t, x, 0, 4, x, z, z, [4], 1, z, z, z, z, z, z, None)
    assert remoe.remoe_decode_static_bytes() == 2_625_792
