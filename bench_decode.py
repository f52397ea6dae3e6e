"""Decode leg of bench.py: M = 1 steps of the Qwen3-30B-A3B-shaped stack through moe_decode.

One step is one token through all layers (router, top-k, the K selected experts' gather-GEMVs,
weighted sum) plus the online overlap / LRU statistics of that step.  Weights stay resident in HBM;
the kernel is bound by the bytes it must stream (router matrix + K experts per layer-step).

Two layer orders are measured.  The headline is the CHAINED order: a layer starts only when the
previous layer of the step has finished everywhere, which is the dependency pattern of a decoder
(Sec. 3, the B = 1 regime).  The overlapped order runs the layers of a step concurrently; that is
legal here only because the synthetic layers all read the same input row, so its figure is reported
separately and is not a decoder's.
"""
from __future__ import annotations

import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0
STEPS_PER_LAUNCH = 128           # keeps a launch well under a second


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


class DecodeState:
    """Output and state buffers of one decode run (allocated once, outside every timed region)."""

    def __init__(self, torch, remoe, desc, L, T, caps, dev):
        H, K, N = desc.hidden, desc.top_k, desc.n_experts
        self.y = torch.empty(T, L, H, dtype=torch.bfloat16, device=dev)
        self.idx = torch.zeros(L, T, K, dtype=torch.int32, device=dev)
        self.gw = torch.zeros(L, T, K, dtype=torch.float32, device=dev)
        self.state = torch.zeros(L, N, dtype=torch.int32, device=dev)
        self.ov = torch.zeros(L, T, dtype=torch.uint8, device=dev)
        self.miss = torch.zeros(len(caps), L, T, dtype=torch.uint8, device=dev)
        self.sum_ov = torch.zeros(L, dtype=torch.int64, device=dev)
        self.tot = torch.zeros(len(caps), L, dtype=torch.int64, device=dev)
        self.nbytes = torch.zeros(len(caps), L, dtype=torch.int64, device=dev)
        self.ws = torch.zeros(remoe.remoe_decode_workspace_bytes(desc), dtype=torch.uint8, device=dev)


def measure_decode(remoe, torch, desc, table, x, L, caps, expert_bytes, bytes_per_layer_step, order, steps, warmup,
                   prof_steps):
    """`warmup` untimed steps, `steps` steps timed by the host clock with the library's event timing
    off, then `prof_steps` further steps with it on (the kernel's own launch duration).  Steps are
    consecutive positions of one run, so the online statistics stay those of one trace.
    Returns (figures, buffers, first timed step)."""
    dev = x.device
    T = x.shape[0]
    assert warmup + steps + prof_steps <= T
    st = DecodeState(torch, remoe, desc, L, T, caps, dev)

    def run(step0, n_total):
        done = 0
        while done < n_total:
            n = min(STEPS_PER_LAUNCH, n_total - done)
            remoe.moe_decode(desc, table, x, step0 + done, n, st.y, st.idx, st.gw, caps, expert_bytes, st.state, st.ov,
                             st.miss, st.sum_ov, st.tot, st.nbytes, st.ws, 0, order)
            done += n

    run(0, warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(warmup, steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kind = remoe.PROF_KINDS.index("decode")
    ms_kernel, launches = 0.0, 0
    if prof_steps > 0:
        remoe.remoe_profile_enable(True)
        run(warmup + steps, prof_steps)
        torch.cuda.synchronize()
        remoe.remoe_profile_enable(False)
        ms_kernel, launches = remoe.remoe_profile_read(kind, reset=True)
    if int(st.ws[128:132].view(torch.int32)[0]) != 0:
        raise RuntimeError("the decode kernel reported a timed-out wait; results are invalid")
    bytes_step = bytes_per_layer_step * L
    us_ls_wall = elapsed / steps / L * 1e6
    fig = {"tokens_per_s": round(steps / elapsed, 1), "ms_per_step": round(elapsed / steps * 1e3, 4),
           "us_per_layer_step": round(us_ls_wall, 3), "steps": steps, "warmup": warmup,
           "steps_per_launch": STEPS_PER_LAUNCH}
    if launches:
        ach = bytes_step * prof_steps / (ms_kernel * 1e-3) / 1e9          # GB/s over the kernel's own time
        fig["roofline"] = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": round(ach / HBM_PEAK_GBS, 4), "avg_launch_ms": round(ms_kernel / launches, 4),
                           "launches": launches, "steps_profiled": prof_steps,
                           "bytes_per_layer_step": bytes_per_layer_step,
                           "us_per_layer_step": round(ms_kernel * 1e3 / (prof_steps * L), 3)}
    return fig, st, warmup


CHAINED_NOTE = ("layers strictly one after the other: a layer starts when the previous layer of the step has "
                "finished on every compute unit (a decoder's dependency pattern)")
OVERLAPPED_NOTE = ("the layers of a step run concurrently, one layer per XCD at a time; possible only because the "
                   "synthetic layers all read the same input row, a decoder cannot do this")


def decode_figures(remoe, torch, desc, table, x, L, caps, expert_bytes, bytes_per_layer_step, steps, warmup, prof_steps):
    """Both layer orders, chained first.  Returns (dict for the JSON line, chained-run buffers, first timed step)."""
    from bench import counter_traffic

    ch, st, first = measure_decode(remoe, torch, desc, table, x, L, caps, expert_bytes, bytes_per_layer_step,
                                   remoe.REMOE_DECODE_CHAINED, steps, warmup, prof_steps)
    ch["kernel"] = "decode_kernel (router + K experts gather-GEMV, layers chained)"
    ch["note"] = CHAINED_NOTE
    pi, _, _ = measure_decode(remoe, torch, desc, table, x, L, caps, expert_bytes, bytes_per_layer_step,
                              remoe.REMOE_DECODE_PIPELINED, steps, warmup, prof_steps)
    pi["kernel"] = "decode_pipe_kernel (layers of a step overlapped)"
    pi["note"] = OVERLAPPED_NOTE
    per_ls = counter_traffic("decode_pipelined", "bytes_per_layer_step")
    if "roofline" in pi:
        pi["roofline"]["traffic"] = None if per_ls is None else per_ls * L * STEPS_PER_LAUNCH
        pi["roofline"]["traffic_source"] = ("replayed from profiles/hbm_traffic.txt (rocprofv3 FETCH_SIZE + WRITE_SIZE of an "
                                            "earlier run of the identical kernel source, scaled by a copy of known size); "
                                            "HBM bytes per launch of %d steps" % STEPS_PER_LAUNCH)
    if "roofline" in ch:
        per_ls_c = counter_traffic("decode_chained", "bytes_per_layer_step")
        ch["roofline"]["traffic"] = None if per_ls_c is None else per_ls_c * L * STEPS_PER_LAUNCH
        ch["roofline"]["traffic_source"] = pi["roofline"]["traffic_source"] if "roofline" in pi else None
    return {"chained": ch, "layers_overlapped": pi}, st, first


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
    prof_steps = min(steps, 256)
    if warmup + steps + prof_steps > T:
        print(f"bench: warmup + steps + {prof_steps} profiled steps must not exceed {T}", file=sys.stderr)
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
    try:
        figs, st, first = decode_figures(remoe, torch, desc, table, x, L, caps, cfg.expert_bytes,
                                         cfg.decode_bytes_per_layer_step, steps, warmup, prof_steps)
    except RuntimeError as e:
        print(f"bench: {e}", file=sys.stderr)
        return 4
    ch = figs["chained"]
    done_steps = warmup + steps + prof_steps
    eor = float(st.sum_ov.sum()) / (K * max(done_steps - 1, 1) * L)
    roof = dict(ch.get("roofline") or {})
    roof["kernel"] = ch["kernel"]
    result = {
        "metric": "MoE-layer tokens/s (Qwen3-30B-A3B shape) + % of MFMA/HBM peak",
        "value": ch["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ch["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": L, "tokens_per_step": 1, "hidden": H, "n_experts": N,
                   "inter": I, "top_k": K, "rho": rho, "lru_capacities": caps, "seed": cfg.seed,
                   "steps_per_launch": STEPS_PER_LAUNCH, "layer_order": "chained"},
        "roofline": roof,
        "decode": figs,
        "trace": {"eor": round(eor, 5),
                  "lru_misses": {str(c): int(st.tot[i].sum()) for i, c in enumerate(caps)},
                  "bytes_fetched": {str(c): int(st.nbytes[i].sum()) for i, c in enumerate(caps)}},
        "setup": {"weights_gib": round(wbytes / 2**30, 2), "generate_s": round(gen_s, 1)},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline_decode(args, cfg, L, x, weights, st.y, st.idx, first, steps)
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
