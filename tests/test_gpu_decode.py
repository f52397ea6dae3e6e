"""GPU parity of the M = 1 decode kernel (moe_decode) against the CPU oracle.

Every layer-step is checked: expert ids (tie window aside) and gate weights against the oracle's
router, layer outputs against the oracle's expert evaluation, and the online overlap / LRU-miss
statistics bit for bit against the oracle's trace functions run on the same expert ids.
"""
import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe
import workload as wl
from helpers import check_output, compare_routing

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def _layers(seed, L, H, N, I, std):
    out = []
    for l in range(L):
        g = lambda name, shape, dt: wl.gaussian(seed, name, shape, std, l, 0, dt, DEV)
        out.append({"w_router": g("w_router", (N, H), torch.float32),
                    "w_gate": g("w_gate", (N, I, H), torch.bfloat16),
                    "w_up": g("w_up", (N, I, H), torch.bfloat16),
                    "w_down": g("w_down", (N, H, I), torch.bfloat16)})
    return out


def _run_decode(desc, layers, x, caps, expert_bytes, pieces, spin_limit_us=0, order=remoe.REMOE_DECODE_PIPELINED):
    L, T = len(layers), x.shape[0]
    K, N, H = desc.top_k, desc.n_experts, desc.hidden
    table = torch.tensor([[w["w_router"].data_ptr(), w["w_gate"].data_ptr(), w["w_up"].data_ptr(),
                           w["w_down"].data_ptr()] for w in layers], dtype=torch.int64, device=DEV)
    out = {
        "y": torch.full((T, L, H), float("nan"), dtype=torch.bfloat16, device=DEV),
        "idx": torch.full((L, T, K), -1, dtype=torch.int32, device=DEV),
        "w": torch.full((L, T, K), float("nan"), dtype=torch.float32, device=DEV),
        "state": torch.zeros(L, N, dtype=torch.int32, device=DEV),
        "ov": torch.full((L, T), 255, dtype=torch.uint8, device=DEV),
        "miss": torch.full((len(caps), L, T), 255, dtype=torch.uint8, device=DEV),
        "sum_ov": torch.zeros(L, dtype=torch.int64, device=DEV),
        "tot": torch.zeros(len(caps), L, dtype=torch.int64, device=DEV),
        "bytes": torch.zeros(len(caps), L, dtype=torch.int64, device=DEV),
    }
    ws = torch.zeros(remoe.remoe_decode_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    pos = 0
    for n in pieces:
        remoe.moe_decode(desc, table, x, pos, n, out["y"], out["idx"], out["w"], caps, expert_bytes, out["state"],
                         out["ov"], out["miss"], out["sum_ov"], out["tot"], out["bytes"], ws, spin_limit_us, order)
        torch.cuda.synchronize()
        pos += n
    assert pos == T
    out["abort"] = int(ws[128:132].view(torch.int32)[0])
    return out


def _check_decode(desc, layers, x, caps, expert_bytes, out, renorm):
    L, T = len(layers), x.shape[0]
    K, N = desc.top_k, desc.n_experts
    assert out["abort"] == 0, "a grid-barrier wait timed out"
    xc = x.cpu()
    worst = 0.0
    for l in range(L):
        wc = {k: v.cpu() for k, v in layers[l].items()}
        orc = oracle.route(xc, wc["w_router"], K, renorm, want_probs=True)
        _, exp_w = compare_routing(out["idx"][l], out["w"][l], orc, renorm)
        y_ref = oracle.experts_sparse(xc, out["idx"][l].cpu(), exp_w, wc)
        worst = max(worst, check_output(out["y"][:, l], y_ref, "bf16"))
    tr = out["idx"].cpu()
    rov, rsum = oracle.trace_reuse(tr, N)
    assert torch.equal(out["ov"].cpu(), rov) and torch.equal(out["sum_ov"].cpu(), rsum)
    for c, cap in enumerate(caps):
        rmiss, rtot, rbytes = oracle.lru_list(tr, N, cap, expert_bytes)
        assert torch.equal(out["miss"][c].cpu(), rmiss), f"LRU misses differ at capacity {cap}"
        assert torch.equal(out["tot"][c].cpu(), rtot) and torch.equal(out["bytes"][c].cpu(), rbytes)
    return worst


@pytest.mark.parametrize("order", [remoe.REMOE_DECODE_CHAINED, remoe.REMOE_DECODE_PIPELINED], ids=["chained", "pipelined"])
@pytest.mark.parametrize("L,T,H,N,I,K,renorm,caps,pieces", [
    (3, 40, 512, 16, 64, 4, True, [4, 8], [40]),
    (2, 33, 1024, 60, 128, 4, False, [12], [1, 1, 7, 24]),          # online: fed in pieces
    (4, 24, 2048, 128, 768, 8, True, [16, 32, 64], [10, 14]),       # the Qwen3-30B-A3B layer shape
    (1, 17, 512, 8, 64, 8, False, [2, 8, 9, 3], [17]),              # K = N, C < K, four capacities
    (20, 9, 512, 32, 128, 4, True, [8], [4, 5]),                    # groups of compute units with 3 and with 2 layers
    (64, 5, 512, 16, 64, 2, True, [4, 16], [5]),                    # the largest layer count
    (2, 6, 4096, 32, 128, 4, True, [8], [6]),                       # the widest row: two output rows per wavefront, two logit words per expert
    (2, 7, 1024, 16, 768, 4, False, [4, 8], [3, 4]),                # long down rows (12 chunks per lane) on a narrow layer
])
def test_decode_matches_oracle(L, T, H, N, I, K, renorm, caps, pieces, order):
    _say(f"decode order={order} L={L} T={T} H={H} N={N} I={I} K={K} caps={caps} pieces={pieces}")
    layers = _layers(70 + N, L, H, N, I, 0.05)
    x = wl.ar1_hidden_states(70 + N, 1, T, H, 0.9, torch.bfloat16, DEV)[0].contiguous()
    desc = remoe.LayerDesc(H, N, I, K, int(renorm), 0, 0, 1)
    out = _run_decode(desc, layers, x, caps, 3 * H * I * 2, pieces, order=order)
    err = _check_decode(desc, layers, x, caps, 3 * H * I * 2, out, renorm)
    _say(f"  worst rel L2 {err:.3e}")


@pytest.mark.parametrize("L,T,H,N,I,K", [
    (5, 12, 1024, 32, 256, 4),
    (2, 9, 4096, 16, 256, 2),      # two exchange words per expert in the chained order
    (3, 7, 2048, 128, 768, 8),     # the Qwen3-30B-A3B layer shape
])
def test_decode_orders_agree(L, T, H, N, I, K):
    """Chained and pipelined schedules compute the same arithmetic in the same order (fp32 router sums in
    runs of eight segments, bf16 activations, packed bf16 dot products): ids, gate weights, every
    statistic and the layer outputs agree bit for bit."""
    _say(f"decode orders L={L} T={T} H={H} N={N} I={I} K={K}")
    layers = _layers(90, L, H, N, I, 0.05)
    x = wl.ar1_hidden_states(90, 1, T, H, 0.7, torch.bfloat16, DEV)[0].contiguous()
    desc = remoe.LayerDesc(H, N, I, K, 1, 0, 0, 1)
    a = _run_decode(desc, layers, x, [6, 16], 7, [T - 5, 5], order=remoe.REMOE_DECODE_CHAINED)
    b = _run_decode(desc, layers, x, [6, 16], 7, [T], order=remoe.REMOE_DECODE_PIPELINED)
    assert a["abort"] == 0 and b["abort"] == 0
    for k in ("idx", "ov", "miss", "sum_ov", "tot", "bytes", "state"):
        assert torch.equal(a[k], b[k]), k
    assert torch.equal(a["w"].view(torch.int32), b["w"].view(torch.int32))
    assert torch.equal(a["y"].view(torch.int16), b["y"].view(torch.int16))


@pytest.mark.parametrize("order", [remoe.REMOE_DECODE_CHAINED, remoe.REMOE_DECODE_PIPELINED], ids=["chained", "pipelined"])
def test_decode_wait_limit_aborts_cleanly(order):
    """The smallest wait limit (1 us per wait) on a 16-layer stack.  Either every wait was met, and
    then every output equals the unlimited run's bit for bit, or a wait ran out, and then the abort
    word (byte 128 of the workspace) is 1, every workgroup has left the kernel (the stream
    synchronises), and the next call on the same device runs normally and reproduces the unlimited
    run."""
    L, T, H, N, I, K = 2, 4, 512, 16, 64, 4
    layers = _layers(81, L, H, N, I, 0.05) * 8
    x = wl.ar1_hidden_states(81, 1, T, H, 0.5, torch.bfloat16, DEV)[0].contiguous()
    desc = remoe.LayerDesc(H, N, I, K, 1, 0, 0, 1)
    keys = ("idx", "ov", "miss", "sum_ov", "tot", "bytes", "state")
    ref = _run_decode(desc, layers, x, [4], 1, [T], order=order)
    assert ref["abort"] == 0
    lim = _run_decode(desc, layers, x, [4], 1, [T], spin_limit_us=1, order=order)   # returns after a synchronize
    assert lim["abort"] in (0, 1)
    _say(f"  1 us wait limit: abort word {lim['abort']}")
    if lim["abort"] == 0:
        for k in keys:
            assert torch.equal(lim[k], ref[k]), k
        assert torch.equal(lim["y"].view(torch.int16), ref["y"].view(torch.int16))
    again = _run_decode(desc, layers, x, [4], 1, [T], order=order)
    assert again["abort"] == 0
    for k in keys:
        assert torch.equal(again[k], ref[k]), k
    assert torch.equal(again["y"].view(torch.int16), ref["y"].view(torch.int16))


def test_decode_rejects_unsupported_layers():
    x = torch.zeros(4, 768, dtype=torch.bfloat16, device=DEV)
    desc = remoe.LayerDesc(768, 16, 64, 4, 1, 0, 0, 1)
    ws = torch.zeros(8 << 20, dtype=torch.uint8, device=DEV)
    t = torch.zeros(1, 4, dtype=torch.int64, device=DEV)
    z = torch.zeros(64, dtype=torch.int64, device=DEV)
    with pytest.raises(remoe.RemoeError, match="hidden"):
        remoe.moe_decode(desc, t, x, 0, 4, x, z, z, [4], 1, z, z, z, z, z, z, ws)
    desc2 = remoe.LayerDesc(512, 16, 64, 4, 1, 64, 0, 1)
    x2 = torch.zeros(4, 512, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(remoe.RemoeError, match="shared"):
        remoe.moe_decode(desc2, t, x2, 0, 4, x2, z, z, [4], 1, z, z, z, z, z, z, ws)
    desc3 = remoe.LayerDesc(512, 16, 64, 4, 1, 0, 0, 1)
    with pytest.raises(remoe.RemoeError, match="layer_order"):
        remoe.moe_decode(desc3, t, x2, 0, 4, x2, z, z, [4], 1, z, z, z, z, z, z, ws, 0, 7)
