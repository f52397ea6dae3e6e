"""Timings of the entry points built beyond the MoE-layer hot path, at the sizes of the Qwen3-30B-A3B
shaped prefill workload: 768 (sequence, layer) traces of 4096 steps for the cache simulator, 16
sequences of 4096 steps for the router regularisers, 65,536 tokens for the gate gradient.

    python bench_extras.py [--repeat 10]

Prints one JSON line per entry point: average milliseconds over `repeat` calls (HIP events on the
current stream), the algorithmic bytes or flops of one call and the rate they amount to.  Inputs
are seeded and synthetic (uniform draws of K distinct experts per step; softmaxes of AR(1) logits).
The hot path itself is measured by bench.py.
"""
import argparse
import json
import sys

import torch

import paper_2605_27081_amd as remoe

DEV = "cuda:0"


def timed(fn, repeat):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(repeat):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / repeat


def line(name, ms, **kw):
    d = {"entry_point": name, "ms": round(ms, 4)}
    d.update(kw)
    print(json.dumps(d), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--repeat", type=int, default=10)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("bench_extras.py needs a GPU", file=sys.stderr)
        return 2
    g = torch.Generator(device=DEV).manual_seed(5)
    N, K, H = 128, 8, 2048
    S_tr, T = 768, 4096          # traces of the prefill workload: 16 sequences x 48 layers
    C = 32
    expert_bytes = 3 * H * 768 * 2

    # K distinct experts per step: the K smallest of N random keys
    idx = torch.rand(S_tr, T, N, generator=g, device=DEV).topk(K, dim=-1, largest=False).indices.int().contiguous()
    miss = torch.empty(S_tr, T, dtype=torch.uint8, device=DEV)
    uniq = torch.empty_like(miss)
    hit = torch.empty_like(miss)
    tot = torch.empty(S_tr, dtype=torch.int64, device=DEV)
    totu = torch.empty_like(tot)
    byt = torch.empty_like(tot)
    trace_bytes = idx.numel() * 4
    for name, pol in (("lru", remoe.REMOE_CACHE_LRU), ("fifo", remoe.REMOE_CACHE_FIFO), ("lfu", remoe.REMOE_CACHE_LFU),
                      ("belady", remoe.REMOE_CACHE_BELADY)):
        nb = remoe.remoe_cache_workspace_bytes(S_tr, T, K, pol)
        ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=DEV) if nb else None
        ms = timed(lambda: remoe.cache_simulate(idx, N, C, pol, expert_bytes, miss, uniq, hit, tot, totu, byt, ws), args.repeat)
        line(f"cache_simulate[{name}]", ms, traces=S_tr, steps=T, capacity=C,
             trace_steps_per_s=round(S_tr * T / ms * 1e3), note="sequential in t per trace: latency-bound, one wavefront per trace")

    L, S = 48, 16
    out_all = torch.empty(S, T, dtype=torch.int16, device=DEV)
    hist = torch.empty(L * K + 1, dtype=torch.int64, device=DEV)
    pct = torch.empty(3, dtype=torch.int32, device=DEV)
    m3 = miss.view(L, S, T)
    ms = timed(lambda: remoe.step_miss_summary(m3, out_all, hist, pct), args.repeat)
    line("step_miss_summary", ms, bytes=m3.numel(), gb_per_s=round(m3.numel() / ms / 1e6, 1))

    load = torch.empty(S_tr, N, dtype=torch.int32, device=DEV)
    used = torch.empty(S_tr, dtype=torch.int32, device=DEV)
    ent = torch.empty(S_tr, dtype=torch.float64, device=DEV)
    cv = torch.empty(S_tr, dtype=torch.float64, device=DEV)
    ms = timed(lambda: remoe.routing_balance(idx, N, load, used, ent, cv), args.repeat)
    line("routing_balance", ms, bytes=trace_bytes, gb_per_s=round(trace_bytes / ms / 1e6, 1))

    # routing distributions: softmax of AR(1) logits
    z = torch.empty(S, T, N, device=DEV)
    z[:, 0] = torch.randn(S, N, generator=g, device=DEV)
    noise = torch.randn(S, T, N, generator=g, device=DEV)
    for t in range(1, T):
        z[:, t] = 0.8 * z[:, t - 1] + 0.6 * noise[:, t]
    P = torch.softmax(2.0 * z, -1).contiguous()
    Q = torch.softmax(2.0 * z + 0.2 * noise, -1).contiguous()
    pidx = torch.topk(P, K, -1).indices.int().contiguous()

    ridx = torch.empty(S, T, K, dtype=torch.int32, device=DEV)
    rw = torch.empty(S, T, K, device=DEV)
    rmiss = torch.empty(S, T, dtype=torch.uint8, device=DEV)
    rtot = torch.empty(S, dtype=torch.int64, device=DEV)
    ms = timed(lambda: remoe.reroute_lru(P, K, 4, 1.5, False, ridx, rw, rmiss, rtot), args.repeat)
    line("reroute_lru", ms, traces=S, steps=T, capacity=4, trace_steps_per_s=round(S * T / ms * 1e3),
         note="sequential in t per trace; 16 traces use 16 wavefronts")

    lags = [1, 2, 4, 8, 16]
    vals = torch.zeros(S, 6, dtype=torch.float64, device=DEV)
    ws = torch.empty(remoe.remoe_loss_workspace_bytes(S), dtype=torch.uint8, device=DEV)
    ms = timed(lambda: remoe.remoe_loss_forward(P, Q, pidx, lags, 64, vals, ws), args.repeat)
    line("remoe_loss_forward", ms, steps=S * T, experts=N, steps_per_s=round(S * T / ms * 1e3))
    dz = torch.empty(S, T, N, device=DEV)
    ws2 = torch.empty(remoe.remoe_loss_backward_workspace_bytes(S, T, N, 64), dtype=torch.uint8, device=DEV)
    ms = timed(lambda: remoe.remoe_loss_backward(P, Q, pidx, lags, 64, [1.0, 0.1, 0.5, 0.5, 0.2], vals, dz, ws2), args.repeat)
    line("remoe_loss_backward", ms, steps=S * T, experts=N, steps_per_s=round(S * T / ms * 1e3))

    x = torch.randn(S * T, H, generator=g, device=DEV).bfloat16()
    dw = torch.empty(N, H, device=DEV)
    ws3 = torch.empty(remoe.remoe_gate_grad_workspace_bytes(S * T, N, H), dtype=torch.uint8, device=DEV)
    ms = timed(lambda: remoe.remoe_gate_grad(dz.view(S * T, N), x, dw, ws3), args.repeat)
    flops = 2.0 * S * T * N * H
    line("remoe_gate_grad", ms, flops=flops, tflops=round(flops / ms / 1e9, 1), peak_tflops=157.3,
         frac=round(flops / ms / 1e9 / 157.3, 3), bound="mfma (fp32)")
    return 0


if __name__ == "__main__":
    sys.exit(main())
