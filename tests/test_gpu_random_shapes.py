"""Seeded random shapes inside the documented limits, through the same checks as the fixed-shape parity
tests (oracle comparison at the tolerances of helpers.py, integer results bit for bit).  The fixed
cases aim at known seams (tile boundaries, ragged tails, extreme sizes); these sweep combinations
nobody thought of: expert counts around 32 / 64 / 128, token counts around the tile height, shared
experts with and without gate, decode shapes in both layer orders, traces under every cache policy.
"""
import random

import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe
import test_gpu_cache as tc
import test_gpu_decode as td
import test_gpu_parity as tp
import workload as wl
from helpers import check_output, to_oracle_weights

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("seed", [7, 21])
def test_random_layer_shapes_match_oracle(seed):
    rng = random.Random(seed)
    for it in range(12):
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        if dtype == "bf16":
            H, I = rng.choice([128, 256, 384, 512, 640, 1024]), rng.choice([64, 128, 192, 320, 448])
            Is = rng.choice([0, 0, 64, 128, 320])
        else:
            H, I, Is = rng.choice([32, 64, 96, 160]), rng.choice([8, 24, 40, 64]), rng.choice([0, 0, 16, 56])
        N = rng.choice([1, 2, 3, 5, 8, 16, 31, 33, 60, 64, 65, 100, 127, 128])
        K = rng.randint(1, min(8, N))
        T = rng.choice([1, 2, 7, 63, 64, 65, 255, 256, 257, 511, 1000, 1537])
        renorm, gate = rng.random() < 0.5, Is > 0 and rng.random() < 0.5
        _say(f"random layer [{seed}/{it}] dtype={dtype} T={T} H={H} N={N} I={I} K={K} renorm={renorm} Is={Is} gate={gate}")
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        w = tp._gen_layer(900 + it, H, N, I, Is, gate, dtype, std=0.05)
        x = wl.ar1_hidden_states(900 + it, 1, T, H, 0.8, tdt, DEV)[0].contiguous()
        desc = remoe.LayerDesc(H, N, I, K, int(renorm), Is, int(gate), 0 if dtype == "f32" else 1)
        y, idx, gw = tp._run_forward(desc, x, w)
        _, _, y_ref = tp.oracle_layer(x.cpu(), to_oracle_weights(w), K, renorm, idx, gw)
        check_output(y, y_ref, dtype)
        y2, idx2, gw2 = tp._run_forward(desc, x, w)
        bits = torch.int16 if dtype == "bf16" else torch.int32
        assert torch.equal(y.view(bits), y2.view(bits)) and torch.equal(idx, idx2) and torch.equal(gw, gw2)


def test_random_decode_shapes_match_oracle_in_both_orders():
    rng = random.Random(9)
    done = 0
    while done < 8:
        H = rng.choice([512, 1024, 2048, 4096])
        N = rng.choice([2, 8, 16, 24, 40, 64, 100, 128])
        I = rng.choice([64, 128, 192, 256, 512, 768])
        K = rng.randint(1, min(8, N))
        if N * H // 256 > 1024 or K * I > 6144:      # outside what the layer-overlapped order accepts
            continue
        L, T = rng.randint(1, 5), rng.randint(1, 12)
        renorm = rng.random() < 0.5
        caps = sorted(rng.sample(range(1, N + 1), min(rng.randint(1, 4), N)))
        cuts = sorted(rng.sample(range(1, T), min(rng.randint(0, 2), T - 1))) if T > 1 else []
        pieces = [b - a for a, b in zip([0] + cuts, cuts + [T])]
        _say(f"random decode [{done}] L={L} T={T} H={H} N={N} I={I} K={K} renorm={renorm} caps={caps} pieces={pieces}")
        layers = td._layers(300 + done, L, H, N, I, 0.05)
        x = wl.ar1_hidden_states(300 + done, 1, T, H, 0.9, torch.bfloat16, DEV)[0].contiguous()
        desc = remoe.LayerDesc(H, N, I, K, int(renorm), 0, 0, 1)
        outs = []
        for order in (remoe.REMOE_DECODE_CHAINED, remoe.REMOE_DECODE_PIPELINED):
            out = td._run_decode(desc, layers, x, caps, 3 * H * I * 2, pieces, order=order)
            td._check_decode(desc, layers, x, caps, 3 * H * I * 2, out, renorm)
            outs.append(out)
        assert torch.equal(outs[0]["y"].view(torch.int16), outs[1]["y"].view(torch.int16)), "the two layer orders differ"
        done += 1


def test_random_traces_match_oracle_under_every_policy():
    rng = random.Random(33)
    for it in range(16):
        N = rng.choice([1, 2, 5, 16, 33, 63, 64, 65, 100, 127, 128])
        K = rng.randint(1, min(N, rng.choice([2, 4, 8, 16, 64])))
        S, T = rng.randint(1, 5), rng.choice([1, 2, 17, 63, 64, 65, 130, 300, 777])
        C = rng.randint(1, N + 2)
        distinct, skew = rng.random() < 0.7, rng.choice([0.0, 0.5, 1.0])
        _say(f"random trace [{it}] S={S} T={T} K={K} N={N} C={C} distinct={distinct} skew={skew}")
        idx = tc._trace(1000 + it, S, T, K, N, distinct, skew)
        d = idx.to(DEV)
        ov = torch.full((S, T), 255, dtype=torch.uint8, device=DEV)
        sm = torch.full((S,), -1, dtype=torch.int64, device=DEV)
        remoe.trace_reuse(d, N, ov, sm)
        miss = torch.full((S, T), 255, dtype=torch.uint8, device=DEV)
        tot = torch.full((S,), -1, dtype=torch.int64, device=DEV)
        nb = torch.full((S,), -1, dtype=torch.int64, device=DEV)
        remoe.lru_simulate(d, N, C, 12345, 0, None, miss, tot, nb)
        torch.cuda.synchronize()
        rov, rs = oracle.trace_reuse(idx, N)
        rmiss, rtot, rnb = oracle.lru_list(idx, N, C, 12345)
        assert torch.equal(ov.cpu(), rov) and torch.equal(sm.cpu(), rs)
        assert torch.equal(miss.cpu(), rmiss) and torch.equal(tot.cpu(), rtot) and torch.equal(nb.cpu(), rnb)
        for p in tc.POLICY:
            got = tc._gpu_cache(idx, N, C, p, 777)
            ref = oracle.cache_policy(idx, N, C, p, 777)
            for k in ("miss", "uniq", "hit_tok", "total_miss", "total_uniq", "bytes"):
                assert torch.equal(got[k], ref[k]), (p, k)
        Kr, Cr = min(K, 16), min(C, N)
        pr = tc._probs(2000 + it, S, T, N)
        factor, renorm = rng.choice([1.0, 1.5, 2.718281828, 54.6]), rng.random() < 0.5
        ridx = torch.full((S, T, Kr), -1, dtype=torch.int32, device=DEV)
        rw = torch.zeros(S, T, Kr, dtype=torch.float32, device=DEV)
        rm = torch.full((S, T), 255, dtype=torch.uint8, device=DEV)
        rt = torch.full((S,), -1, dtype=torch.int64, device=DEV)
        remoe.reroute_lru(pr.to(DEV), Kr, Cr, factor, renorm, ridx, rw, rm, rt)
        torch.cuda.synchronize()
        ref = oracle.reroute_lru(pr, Kr, Cr, factor, renorm)
        assert torch.equal(ridx.cpu(), ref["idx"]) and torch.equal(rm.cpu(), ref["miss"]) and torch.equal(rt.cpu(), ref["total_miss"])
        assert torch.allclose(rw.cpu().double(), ref["w"], rtol=2e-6, atol=1e-12)
