"""Decode leg of bench.py: M = 1 steps of the Qwen3-30B-A3B-shaped stack through moe_decode.

One step is one token through all layers (router, top-k, the K selected experts' gather-GEMVs,
weighted sum) plus the online overlap / LRU statistics of that step.  Weights stay resident in HBM;
the kernel is bound by the bytes it must stream (router matrix + K experts per layer-step).
"""
from __future__ import annotations

import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def run_decode(args, cfg):
    import torch

    import paper_2605_27081_amd as remoe
    import workload as wl

    dev = torch.device("cuda:0")
    L = args.layers if args.layers > 0 else cfg.n_layers
    H, K, N, I = cfg.hidden, cfg.top_k, cfg.n_experts, cfg.inter
    T = cfg.seq_len
    rho = cfg.rhos[-1]
    caps = list(cfg.capacities)
    desc = remoe.LayerDesc.from_config(cfg)
    steps, warmup = args.steps, args.warmup
    if warmup + steps > T:
        print(f"bench: warmup + steps must not exceed {T}", file=sys.stderr)
        return 2

    t0 = time.perf_counter()
    x = wl.hidden_states(cfg, rho, device=dev).reshape(T, H).contiguous()
    weights = [wl.layer_weights(cfg, l, device=dev) for l in range(L)]
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    wbytes = sum(v.numel() * v.element_size() for w in weights for v in w.values() if v is not None)
    log(f"{cfg.name}: {L} layers, weights {wbytes / 2**30:.2f} GiB generated in {gen_s:.1f} s")
    table = torch.tensor([[w["w_router"].data_ptr(), w["w_gate"].data_ptr(), w["w_up"].data_ptr(),
                           w["w_down"].data_ptr()] for w in weights], dtype=torch.int64, device=dev)
    y = torch.empty(T, L, H, dtype=torch.bfloat16, device=dev)
    idx = torch.zeros(L, T, K, dtype=torch.int32, device=dev)
    gw = torch.zeros(L, T, K, dtype=torch.float32, device=dev)
    state = torch.zeros(L, N, dtype=torch.int32, device=dev)
    ov = torch.zeros(L, T, dtype=torch.uint8, device=dev)
    miss = torch.zeros(len(caps), L, T, dtype=torch.uint8, device=dev)
    sum_ov = torch.zeros(L, dtype=torch.int64, device=dev)
    tot = torch.zeros(len(caps), L, dtype=torch.int64, device=dev)
    nbytes = torch.zeros(len(caps), L, dtype=torch.int64, device=dev)
    ws = torch.zeros(remoe.remoe_decode_workspace_bytes(desc), dtype=torch.uint8, device=dev)

    order = remoe.REMOE_DECODE_CHAINED if getattr(args, "decode_chained", False) else remoe.REMOE_DECODE_PIPELINED

    def decode(step0, n):
        remoe.moe_decode(desc, table, x, step0, n, y, idx, gw, caps, cfg.expert_bytes, state, ov, miss, sum_ov,
                         tot, nbytes, ws, 0, order)

    chunk = 128                      # steps per launch: keeps a launch well under a second
    pos = 0
    while pos < warmup:
        n = min(chunk, warmup - pos)
        decode(pos, n)
        pos += n
    torch.cuda.synchronize()
    remoe.remoe_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    done = 0
    while done < steps:
        n = min(chunk, steps - done)
        decode(pos + done, n)
        done += n
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    remoe.remoe_profile_enable(False)
    ms_kernel, launches = remoe.remoe_profile_read(remoe.PROF_KINDS.index("decode"), reset=True)
    if int(ws[128:132].view(torch.int32)[0]) != 0:
        print("bench: the decode kernel reported a timed-out wait; results are invalid", file=sys.stderr)
        return 4

    tokens_per_s = steps / elapsed
    from bench import counter_traffic
    per_ls = counter_traffic("decode_pipelined", "bytes_per_layer_step") if order == remoe.REMOE_DECODE_PIPELINED else None
    bytes_step = cfg.decode_bytes_per_layer_step * L           # algorithmic bytes of one step
    ach = bytes_step * steps / (ms_kernel * 1e-3) / 1e9         # GB/s over the kernel's own time
    done_steps = warmup + steps
    eor = float(sum_ov.sum()) / (K * max(done_steps - 1, 1) * L)
    result = {
        "metric": "MoE-layer tokens/s (Qwen3-30B-A3B shape) + % of MFMA/HBM peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(elapsed / steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": L, "tokens_per_step": 1, "hidden": H, "n_experts": N,
                   "inter": I, "top_k": K, "rho": rho, "lru_capacities": caps, "seed": cfg.seed,
                   "steps_per_launch": chunk,
                   "layer_order": "chained" if order == remoe.REMOE_DECODE_CHAINED else "pipelined"},
        "roofline": {"bound": "hbm", "kernel": ("decode_kernel" if order == remoe.REMOE_DECODE_CHAINED else "decode_pipe_kernel") + " (router + K experts gather-GEMV)",
                     "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBS, 4),
                     "traffic": (None if per_ls is None else per_ls * L * chunk),
                     "traffic_unit": "HBM bytes per launch of %d steps (FETCH_SIZE + WRITE_SIZE scaled by a copy of known "
                                     "size), against %d algorithmic" % (chunk, bytes_step * chunk),
                     "avg_launch_ms": round(ms_kernel / max(launches, 1), 4), "launches": launches,
                     "bytes_per_step": bytes_step, "us_per_layer_step": round(ms_kernel * 1e3 / (steps * L), 3)},
        "trace": {"eor": round(eor, 5),
                  "lru_misses": {str(c): int(tot[i].sum()) for i, c in enumerate(caps)},
                  "bytes_fetched": {str(c): int(nbytes[i].sum()) for i, c in enumerate(caps)}},
        "setup": {"weights_gib": round(wbytes / 2**30, 2), "generate_s": round(gen_s, 1)},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline_decode(args, cfg, L, x, weights, y, idx, pos, steps)
    print(json.dumps(result), flush=True)
    return 0


def cpu_baseline_decode(args, cfg, L, x, weights, y, idx, step0, steps):
    """The oracle on a sample of the timed steps x first layers (router, experts, trace statistics)."""
    import torch

    import oracle

    K, N = cfg.top_k, cfg.n_experts
    n_tok = min(args.cpu_sample_tokens, steps)
    n_lay = min(args.cpu_sample_layers, L)
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    xs = x[step0:step0 + n_tok].cpu().contiguous()
    secs = t_trace = 0.0
    worst = 0.0
    for l in range(n_lay):
        wc = {k: (None if v is None else v.cpu()) for k, v in weights[l].items()}
        t0 = time.perf_counter()
        r = oracle.route(xs, wc["w_router"], K, cfg.renorm)
        ys = oracle.experts_sparse(xs, r["idx"], r["w"], wc)
        t1 = time.perf_counter()
        tr = idx[l, :step0 + n_tok].cpu()[None]
        oracle.trace_reuse(tr, N)
        for c in cfg.capacities:
            oracle.lru_list(tr, N, c, cfg.expert_bytes)
        t2 = time.perf_counter()
        secs += t1 - t0
        t_trace += t2 - t1
        same = (torch.sort(idx[l, step0:step0 + n_tok].cpu(), 1).values == torch.sort(r["idx"], 1).values).all(1)
        if same.any():
            yg = y[step0:step0 + n_tok, l].cpu().double()[same]
            worst = max(worst, float((yg - ys[same]).norm() / ys[same].norm()))
    value = n_tok * n_lay / cfg.n_layers / secs
    return {"value": round(value, 4), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": (f"{n_tok} consecutive steps x first {n_lay} layers of {cfg.name}: router + experts + "
                       f"combine in {secs:.1f} s ({n_tok * n_lay / secs:.1f} token-layers/s, scaled to "
                       f"{cfg.n_layers} layers); overlap + LRU ({len(cfg.capacities)} capacities) over those "
                       f"layers' traces took {t_trace:.2f} s more"),
            "sample_rel_l2_vs_gpu": round(worst, 5)}
