#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input: for every layer the
router, the token->expert sort, the grouped SwiGLU expert GEMMs (plus the shared expert) and the
weighted combine, followed by the routing-trace statistics (adjacent-step overlap and LRU cache
misses) over the expert ids of all layers.  All inputs and weights are generated on the GPU before
the timed region and stay resident in HBM.

Prints ONE JSON line: whole-job tokens/s (timed with the library's per-kernel event timing off), the
roofline figures of the dominant kernel (timed live with HIP events on the launch stream, in a
second short pass), for the headline workload the M = 1 decode figures of both layer orders on the
same resident weights, and the CPU oracle timed on a bounded sample of the same workload on the
host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
F32_VECTOR_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 5 batched passes, or 1024 decode steps)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps (default 1, or 32 decode steps)")
    ap.add_argument("--config", default="qwen3_prefill",
                    help="workload name (workload/configs.py); the headline is qwen3_prefill")
    ap.add_argument("--layers", type=int, default=0, help="use only the first N layers (0 = all; debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="before the run, copy this many MiB three times with the library's plain copy kernel "
                         "(the yardstick when the run is profiled with hardware byte counters)")
    ap.add_argument("--no-decode-leg", action="store_true",
                    help="qwen3_prefill only: skip the M = 1 decode measurement on the resident weights")
    ap.add_argument("--decode-steps", type=int, default=256,
                    help="qwen3_prefill only: timed decode steps per layer order (plus 32 warm-up and 128 profiled)")
    ap.add_argument("--data-dependence-probe", type=int, default=0, metavar="REPS",
                    help="batched configs: afterwards run layer 0 REPS times with its weights and REPS times with "
                         "all-zero expert weights (same routing, same instruction stream) and report both kernel "
                         "times: a matrix kernel that speeds up on zeros is held back by the clock the chip can "
                         "sustain on the operands' bit activity, not by its schedule")
    ap.add_argument("--cpu-sample-tokens", type=int, default=1024)
    ap.add_argument("--cpu-sample-layers", type=int, default=12)
    return ap.parse_args()


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def counter_traffic(kernel, field):
    """HBM bytes from the hardware-counter runs recorded in profiles/hbm_traffic.txt, or None when
    there is no record or the kernel's source has changed since the counters were taken."""
    import hashlib

    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if not parts or parts[0] != kernel:
            continue
        kv = dict(p.split("=", 1) for p in parts[1:])
        src = os.path.join(ROOT, kv.get("source", ""))
        if field not in kv or not os.path.isfile(src):
            return None
        if hashlib.sha256(open(src, "rb").read()).hexdigest() != kv.get("sha256"):
            return None
        return int(kv[field])
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this library measures ONE GPU; run with --gpus 1 (no sharding or collectives exist here)",
              file=sys.stderr)
        return 2

    import torch

    import paper_2605_27081_amd as remoe
    import workload as wl
    from paper_2605_27081_amd import build as hip_build

    if not hip_build.is_built():
        log("libremoe_hip.so missing: building")
        hip_build.build()
    remoe.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.zeros_like(src)
        for _ in range(3):
            remoe.remoe_copy_probe(dst, src)
        torch.cuda.synchronize()
        if not torch.equal(dst, src):
            print("bench.py: copy probe produced a wrong copy", file=sys.stderr)
            return 4
        del src, dst

    cfg = wl.get_config(args.config)
    if args.steps is None:
        args.steps = 1024 if cfg.decode else 5
    if args.warmup is None:
        args.warmup = 32 if cfg.decode else 1
    if cfg.decode:
        from bench_decode import run_decode  # M=1 decode has its own driver
        return run_decode(args, cfg)
    L = args.layers if args.layers > 0 else cfg.n_layers
    T, H, K, N = cfg.n_tokens, cfg.hidden, cfg.top_k, cfg.n_experts
    S, Ts = cfg.n_seq, cfg.seq_len
    rho = cfg.rhos[-1]
    capacity = cfg.capacities[0]
    desc = remoe.LayerDesc.from_config(cfg)
    tdt = desc.torch_dtype

    # ---- inputs and weights, resident in HBM (untimed) -----------------------------------------
    t0 = time.perf_counter()
    x = wl.hidden_states(cfg, rho, device=dev).reshape(T, H).contiguous()
    weights = [wl.layer_weights(cfg, l, device=dev) for l in range(L)]
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    wbytes = sum(v.numel() * v.element_size() for w in weights for v in w.values() if v is not None)
    log(f"{cfg.name}: {L} layers, {T} tokens, weights {wbytes / 2**30:.2f} GiB generated in {gen_s:.1f} s")

    y = torch.empty(L, T, H, dtype=tdt, device=dev)
    idx = torch.empty(L, T, K, dtype=torch.int32, device=dev)
    gw = torch.empty(L, T, K, dtype=torch.float32, device=dev)
    ws = torch.empty(remoe.remoe_workspace_bytes(desc, T), dtype=torch.uint8, device=dev)
    n_tr = L * S
    ov = torch.empty(n_tr, Ts, dtype=torch.uint8, device=dev)
    ov_sum = torch.empty(n_tr, dtype=torch.int64, device=dev)
    miss = torch.empty(n_tr, Ts, dtype=torch.uint8, device=dev)
    miss_tot = torch.empty(n_tr, dtype=torch.int64, device=dev)
    miss_bytes = torch.empty(n_tr, dtype=torch.int64, device=dev)

    def step():
        for l in range(L):
            w = weights[l]
            remoe.moe_forward(desc, x, w["w_router"], w["w_gate"], w["w_up"], w["w_down"], w["ws_gate"],
                              w["ws_up"], w["ws_down"], w["ws_scale"], y[l], idx[l], gw[l], ws)
        tr = idx.view(n_tr, Ts, K)
        remoe.trace_reuse(tr, N, ov, ov_sum)
        remoe.lru_simulate(tr, N, capacity, cfg.expert_bytes, 0, None, miss, miss_tot, miss_bytes)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: the library's per-kernel event timing is off, nothing but the path runs
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # second, short pass with the event timing on: per-kernel averages and the dominant kernel's
    # launch duration (HIP events on the launch stream)
    prof_steps = min(3, args.steps)
    remoe.remoe_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    elapsed_prof = time.perf_counter() - t0
    remoe.remoe_profile_enable(False)
    prof = {}
    for k, name in enumerate(remoe.PROF_KINDS):
        ms, n = remoe.remoe_profile_read(k, reset=True)
        if n:
            prof[name] = {"ms_total": ms, "launches": n, "ms_avg": ms / n}

    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = T / (elapsed / args.steps)      # tokens through the whole L-layer stack per second
    # whole-layer figure: useful flops of the routed + shared experts and router over wall time
    flops_step = cfg.flops_per_token_layer * T * L
    layer_tflops = flops_step / (elapsed / args.steps) / 1e12

    # ---- roofline of the dominant kernel: routed gate/up GEMM + SwiGLU ------------------------
    gate_up_flops = 2.0 * T * K * H * (2 * cfg.inter)       # algorithmic flops per launch
    dom = prof.get("gate_up")
    roofline = None
    if dom:
        ach = gate_up_flops / (dom["ms_avg"] * 1e-3) / 1e12
        peak = BF16_MFMA_PEAK_TFLOPS if cfg.dtype == "bf16" else F32_VECTOR_PEAK_TFLOPS
        roofline = {"bound": "mfma" if cfg.dtype == "bf16" else "alu", "kernel": "grouped_gemm (gate/up + SwiGLU)",
                    "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(ach / peak, 4),
                    "traffic": (counter_traffic("gate_up", "bytes_per_launch")
                                if (cfg.name == "qwen3_prefill" and cfg.dtype == "bf16") else None),
                    "traffic_source": "NOT measured in this run: replayed from profiles/hbm_traffic.txt, which records "
                                      "rocprofv3 FETCH_SIZE + WRITE_SIZE (scaled by a copy of known size) of an earlier "
                                      "run of the byte-identical kernel source; null once the source differs.  "
                                      "Bytes past the L2 per launch, against %d algorithmic"
                                      % int(T * H * 2 + 2 * N * cfg.inter * H * 2 + T * K * cfg.inter * 2),
                    "avg_launch_ms": round(dom["ms_avg"], 4), "launches": dom["launches"],
                    "timed_in": "a separate pass of %d steps with per-kernel HIP events on (%.3f ms per step)"
                                % (prof_steps, elapsed_prof / prof_steps * 1e3)}

    # the other kernels of a layer against the roofline that bounds each (algorithmic work per launch over
    # its average duration in the profiled pass); routed experts only, bf16 layers
    others = {}
    if cfg.dtype == "bf16":
        es = 2
        work = {
            "down": ("mfma", 2.0 * T * K * cfg.inter * H, BF16_MFMA_PEAK_TFLOPS, 1e12, "TFLOP/s"),
            # K (+1 with a shared expert) rows of H values read per token, one written
            "combine": ("hbm", float(T) * (K + (2 if cfg.shared_inter else 1)) * H * es, HBM_PEAK_GBS, 1e9, "GB/s"),
            # the hidden states once and the gate matrix once; the routing out
            "route": ("hbm", float(T) * H * es + N * H * 4.0 + T * K * 8.0, HBM_PEAK_GBS, 1e9, "GB/s"),
        }
        for name, (bound, amount, peak, scale, unit) in work.items():
            if name in prof:
                ach = amount / (prof[name]["ms_avg"] * 1e-3) / scale
                others[name] = {"bound": bound, "achieved": round(ach, 1), "peak": peak, "unit": unit,
                                "frac": round(ach / peak, 4), "avg_launch_ms": round(prof[name]["ms_avg"], 4)}

    eor = float(ov_sum.sum()) / (K * (Ts - 1) * n_tr) if Ts > 1 else float("nan")
    total_miss = int(miss_tot.sum())
    result = {
        "metric": "MoE-layer tokens/s (Qwen3-30B-A3B shape) + % of MFMA/HBM peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": L, "tokens": T, "n_seq": S, "seq_len": Ts, "hidden": H,
                   "n_experts": N, "inter": cfg.inter, "top_k": K, "shared_inter": cfg.shared_inter,
                   "rho": rho, "lru_capacity": capacity, "seed": cfg.seed},
        "roofline": roofline,
        "layer": {"useful_tflops": round(layer_tflops, 2),
                  "frac_of_bf16_mfma_peak": round(layer_tflops / BF16_MFMA_PEAK_TFLOPS, 4),
                  "kernels_ms_avg": {k: round(v["ms_avg"], 4) for k, v in prof.items()},
                  "other_kernels": others},
        "trace": {"eor": round(eor, 5), "lru_misses": total_miss,
                  "bytes_fetched": int(miss_bytes.sum())},
        "setup": {"weights_gib": round(wbytes / 2**30, 2), "generate_s": round(gen_s, 1)},
    }

    # ---- M = 1 decode on the same resident weights, both layer orders (chained first) -----------
    if cfg.name == "qwen3_prefill" and not args.no_decode_leg:
        result["decode"] = decode_leg(args, L, weights, desc)

    if args.data_dependence_probe > 0:
        result["data_dependence_probe"] = data_dependence_probe(args.data_dependence_probe, desc, x, weights[0],
                                                                y[0], idx[0], gw[0], ws)

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, cfg, L, x, weights, y, idx, gw)

    print(json.dumps(result), flush=True)
    return 0


def decode_leg(args, L, weights, desc):
    """The qwen3_decode workload (M = 1, rho = 0.9 input rows, capacities {16, 32, 64}) run on the layer
    stack that is already resident, so that one bench line carries both targets."""
    import torch

    import paper_2605_27081_amd as remoe
    import workload as wl
    from bench_decode import decode_figures

    dcfg = wl.get_config("qwen3_decode")
    dev = weights[0]["w_router"].device
    xd = wl.hidden_states(dcfg, dcfg.rhos[-1], device=dev).reshape(dcfg.seq_len, dcfg.hidden).contiguous()
    table = torch.tensor([[w["w_router"].data_ptr(), w["w_gate"].data_ptr(), w["w_up"].data_ptr(),
                           w["w_down"].data_ptr()] for w in weights], dtype=torch.int64, device=dev)
    try:
        figs, _, _ = decode_figures(remoe, torch, desc, table, xd, L, list(dcfg.capacities), dcfg.expert_bytes,
                                    dcfg.decode_bytes_per_layer_step, args.decode_steps, 32, 128)
    except RuntimeError as e:
        return {"error": str(e)}
    figs["workload"] = ("qwen3_decode input rows (seed %d, rho %.1f), M = 1, capacities %s, on the %d resident "
                        "qwen3_prefill layers (same shapes; weights of seed 3)"
                        % (dcfg.seed, dcfg.rhos[-1], list(dcfg.capacities), L))
    figs["target"] = "chained.roofline.frac >= 0.60 of the 8 TB/s HBM peak (<= 16 us per layer-step)"
    return figs


def data_dependence_probe(reps, desc, x, w, y, idx, gw, ws):
    """Layer 0, `reps` calls each: with its weights, then with a zeroed copy of the three expert tensors.
    The router weights and the input stay, so routing, tile lists and every kernel's instruction
    stream are identical; only the operand values of the two expert GEMMs (and what flows from them)
    change.  A third run zeroes the input as well.  Returns the per-kernel averages (HIP events)."""
    import torch

    import paper_2605_27081_amd as remoe

    def run(wg, wu, wd, xin=x):
        for _ in range(3):
            remoe.moe_forward(desc, xin, w["w_router"], wg, wu, wd, w["ws_gate"], w["ws_up"], w["ws_down"],
                              w["ws_scale"], y, idx, gw, ws)
        torch.cuda.synchronize()
        remoe.remoe_profile_enable(True)
        t0 = time.perf_counter()
        for _ in range(reps):
            remoe.moe_forward(desc, xin, w["w_router"], wg, wu, wd, w["ws_gate"], w["ws_up"], w["ws_down"],
                              w["ws_scale"], y, idx, gw, ws)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        remoe.remoe_profile_enable(False)
        out = {"ms_per_layer": round(ms, 4)}
        for k, name in enumerate(remoe.PROF_KINDS):
            t, n = remoe.remoe_profile_read(k, reset=True)
            if n:
                out[name] = round(t / n, 4)
        return out

    real = run(w["w_gate"], w["w_up"], w["w_down"])
    zg, zu, zd = (torch.zeros_like(w[k]) for k in ("w_gate", "w_up", "w_down"))
    zero = run(zg, zu, zd)
    # all operands zero: every token then routes to experts 0 .. K-1 (equal logits, ties to the lower id),
    # i.e. the same number of row tiles spread over K experts instead of N_r
    zero_all = run(zg, zu, zd, torch.zeros_like(x))
    del zg, zu, zd
    return {"reps": reps, "real_weights_ms": real, "zero_expert_weights_ms": zero, "all_zero_ms": zero_all,
            "gate_up_speedup_on_zeros": round(real["gate_up"] / zero["gate_up"], 3),
            "down_speedup_on_zeros": round(real["down"] / zero["down"], 3),
            "note": "same launches, tile lists and instructions in both runs; the zeros run leaves y = 0"}


def cpu_baseline(args, cfg, L, x, weights, y, idx, gw):
    """Time the oracle (as it stands) on sample tokens of the first layers, on the host cores."""
    import torch

    import oracle

    T, K, N = cfg.n_tokens, cfg.top_k, cfg.n_experts
    n_tok = min(args.cpu_sample_tokens, T)
    n_lay = min(args.cpu_sample_layers, L)
    tokens = [int(i * T // n_tok) for i in range(n_tok)]
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    xs = x[tokens].cpu().contiguous()
    t_route = t_exp = t_trace = 0.0
    worst = 0.0
    for l in range(n_lay):
        wc = {k: (None if v is None else v.cpu()) for k, v in weights[l].items()}
        t0 = time.perf_counter()
        r = oracle.route(xs, wc["w_router"], K, cfg.renorm)
        t1 = time.perf_counter()
        ys = oracle.experts_sparse(xs, r["idx"], r["w"], wc)
        t2 = time.perf_counter()
        tr = idx[l].view(cfg.n_seq, cfg.seq_len, K).cpu()
        oracle.trace_reuse(tr, N)
        oracle.lru_list(tr, N, cfg.capacities[0], cfg.expert_bytes)
        t3 = time.perf_counter()
        t_route += t1 - t0
        t_exp += t2 - t1
        t_trace += t3 - t2
        # the sample doubles as a spot check of the GPU result (tokens routed identically)
        same = (torch.sort(idx[l][tokens].cpu(), 1).values == torch.sort(r["idx"], 1).values).all(1)
        if same.any():
            yg = y[l][tokens].cpu().double()[same]
            worst = max(worst, float((yg - ys[same]).norm() / ys[same].norm()))
    token_layers = n_tok * n_lay
    secs = t_route + t_exp
    value = token_layers / cfg.n_layers / secs
    return {"value": round(value, 4), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": (f"{n_tok} evenly spaced tokens x first {n_lay} layers of {cfg.name}: router + experts + "
                       f"combine in {secs:.1f} s ({token_layers / secs:.1f} token-layers/s, scaled to "
                       f"{cfg.n_layers} layers); overlap + LRU over those layers' full traces took "
                       f"{t_trace:.2f} s more"),
            "sample_rel_l2_vs_gpu": round(worst, 5)}


if __name__ == "__main__":
    sys.exit(main())
