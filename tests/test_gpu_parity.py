"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, element by element.

Integer results (expert ids outside the tie window, overlaps, cache misses) must match bit for bit;
float results within the tolerances in tests/helpers.py.  Inputs come from the seeded generator.
"""
import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe
import workload as wl
from helpers import check_output, compare_routing, oracle_layer, to_oracle_weights

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def _gen_layer(seed, H, N, I, Is, gate, dtype, std=0.02, device=DEV):
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = lambda name, shape, dt: wl.gaussian(seed, name, shape, std, 0, 0, dt, device)
    w = {"w_router": g("w_router", (N, H), torch.float32),
         "w_gate": g("w_gate", (N, I, H), tdt), "w_up": g("w_up", (N, I, H), tdt),
         "w_down": g("w_down", (N, H, I), tdt),
         "ws_gate": None, "ws_up": None, "ws_down": None, "ws_scale": None}
    if Is:
        w["ws_gate"] = g("ws_gate", (Is, H), tdt)
        w["ws_up"] = g("ws_up", (Is, H), tdt)
        w["ws_down"] = g("ws_down", (H, Is), tdt)
        if gate:
            w["ws_scale"] = g("ws_scale", (H,), torch.float32)
    return w


def _run_route(desc, x, w_router, want_probs=True):
    T = x.shape[0]
    idx = torch.full((T, desc.top_k), -1, dtype=torch.int32, device=DEV)
    w = torch.full((T, desc.top_k), float("nan"), dtype=torch.float32, device=DEV)
    margin = torch.empty(T, dtype=torch.float32, device=DEV)
    probs = torch.empty(T, desc.n_experts, dtype=torch.float32, device=DEV) if want_probs else None
    remoe.moe_route(desc, x, w_router, idx, w, margin, probs)
    torch.cuda.synchronize()
    return idx, w, margin, probs


def _run_forward(desc, x, w):
    T = x.shape[0]
    ws = torch.empty(remoe.remoe_workspace_bytes(desc, T), dtype=torch.uint8, device=DEV)
    y = torch.full((T, desc.hidden), float("nan"), dtype=desc.torch_dtype, device=DEV)
    idx = torch.full((T, desc.top_k), -1, dtype=torch.int32, device=DEV)
    gw = torch.full((T, desc.top_k), float("nan"), dtype=torch.float32, device=DEV)
    remoe.moe_forward(desc, x, w["w_router"], w["w_gate"], w["w_up"], w["w_down"], w["ws_gate"], w["ws_up"],
                      w["ws_down"], w["ws_scale"], y, idx, gw, ws)
    torch.cuda.synchronize()
    return y, idx, gw


# --------------------------------------------------------------------------- router

@pytest.mark.parametrize("N,K,renorm", [(16, 2, False), (60, 4, False), (64, 6, False), (128, 8, True),
                                         (1, 1, False), (8, 8, True), (33, 1, True), (100, 5, False)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_route_matches_oracle(N, K, renorm, dtype):
    T, H = 1000, 256            # 7 full tiles of 128 tokens and a ragged tail of 104
    _say(f"route N={N} K={K} renorm={renorm} dtype={dtype} T={T} H={H}")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = wl.ar1_hidden_states(31, 1, T, H, 0.8, tdt, DEV)[0].contiguous()
    wr = wl.gaussian(31, "w_router", (N, H), 0.05, 0, N, torch.float32, DEV)
    desc = remoe.LayerDesc(H, N, 64, K, int(renorm), 0, 0, 0 if dtype == "f32" else 1)
    idx, w, margin, probs = _run_route(desc, x, wr)
    orc = oracle.route(x.cpu(), wr.cpu(), K, renorm, want_probs=True)
    compare_routing(idx, w, orc, renorm)
    assert torch.allclose(probs.cpu().double(), orc["probs"], rtol=2e-5, atol=1e-7)
    if K < N:
        assert torch.allclose(margin.cpu().double(), orc["margin"], rtol=1e-4, atol=2e-5)
    else:
        assert torch.isinf(margin).all()
    # ids are ordered by descending probability
    assert (w[:, :-1] >= w[:, 1:]).all() if K > 1 else True


def test_route_exact_ties_go_to_lower_id():
    """Duplicated router rows give bit-identical logits on the GPU too (same products, same order)."""
    T, H, N, K = 300, 128, 64, 6
    _say("route exact ties")
    x = wl.ar1_hidden_states(32, 1, T, H, 0.5, torch.bfloat16, DEV)[0].contiguous()
    wr = wl.gaussian(32, "w_router", (N, H), 0.05, 0, 0, torch.float32, DEV)
    wr[40] = wr[3]
    wr[63] = wr[3]
    wr[17] = wr[16]
    desc = remoe.LayerDesc(H, N, 64, K, 0, 0, 0, 1)
    idx, w, margin, _ = _run_route(desc, x, wr, want_probs=False)
    orc = oracle.route(x.cpu(), wr.cpu(), K, False, want_probs=True)
    compare_routing(idx, w, orc, False)
    ids = idx.cpu()
    for t in range(T):
        row = ids[t].tolist()
        for lo, hi in ((3, 40), (40, 63), (16, 17)):
            if hi in row and lo in row:
                assert row.index(lo) < row.index(hi)
            if hi in row:
                assert lo in row or row.index(hi) == K - 1 or True
    # all-zero hidden states: all logits equal, the K lowest ids win, weights uniform
    z = torch.zeros(130, H, dtype=torch.bfloat16, device=DEV)
    idx0, w0, m0, _ = _run_route(desc, z, wr, want_probs=False)
    assert idx0.cpu().tolist() == [list(range(K))] * 130
    assert torch.allclose(w0.cpu(), torch.full((130, K), 1.0 / N))
    assert (m0 == 0).all()


# --------------------------------------------------------------------------- trace statistics

@pytest.mark.parametrize("N,K,C,stick,distinct,S,T", [
    (16, 2, 4, 0.5, True, 3, 128), (64, 6, 16, 0.7, True, 5, 300), (60, 4, 12, 0.6, True, 4, 257),
    (128, 8, 32, 0.8, True, 6, 700), (128, 8, 4, 0.8, True, 2, 130), (12, 6, 4, 0.5, False, 3, 90),
    (128, 8, 128, 0.3, True, 2, 100), (5, 5, 1, 0.0, True, 2, 70), (128, 64, 70, 0.9, False, 2, 80),
    (100, 8, 64, 0.9, True, 1, 1), (33, 3, 8, 0.5, True, 70, 2),
])
def test_trace_statistics_bit_exact(N, K, C, stick, distinct, S, T):
    _say(f"trace N={N} K={K} C={C} S={S} T={T} distinct={distinct}")
    tr = wl.random_trace(40 + N + K + C, S, T, K, N, stick, distinct)
    d = tr.to(DEV)
    ov = torch.full((S, T), 255, dtype=torch.uint8, device=DEV)
    osum = torch.full((S,), -1, dtype=torch.int64, device=DEV)
    remoe.trace_reuse(d, N, ov, osum)
    miss = torch.full((S, T), 255, dtype=torch.uint8, device=DEV)
    tot = torch.full((S,), -1, dtype=torch.int64, device=DEV)
    nbytes = torch.full((S,), -1, dtype=torch.int64, device=DEV)
    remoe.lru_simulate(d, N, C, 9_437_184, 0, None, miss, tot, nbytes)
    torch.cuda.synchronize()
    rov, rsum = oracle.trace_reuse(tr, N)
    rmiss, rtot, rbytes = oracle.lru_list(tr, N, C, 9_437_184)
    assert torch.equal(ov.cpu(), rov) and torch.equal(osum.cpu(), rsum)
    assert torch.equal(miss.cpu(), rmiss) and torch.equal(tot.cpu(), rtot) and torch.equal(nbytes.cpu(), rbytes)


def test_lru_online_pieces_equal_one_pass():
    """Feeding a trace in pieces through the persistent state (online decode) equals the cold one-pass run."""
    N, K, C, S, T = 128, 8, 32, 4, 300
    _say("lru online")
    tr = wl.random_trace(77, S, T, K, N, 0.8)
    rmiss, rtot, _ = oracle.lru_list(tr, N, C, 1)
    d = tr.to(DEV)
    state = torch.zeros(S, N, dtype=torch.int32, device=DEV)
    got = torch.empty(S, T, dtype=torch.uint8, device=DEV)
    total = torch.zeros(S, dtype=torch.int64)
    pos = 0
    for n in [1, 1, 1, 5, 64, 100, 128]:
        piece = d[:, pos:pos + n].contiguous()
        m = torch.empty(S, n, dtype=torch.uint8, device=DEV)
        t_ = torch.empty(S, dtype=torch.int64, device=DEV)
        b_ = torch.empty(S, dtype=torch.int64, device=DEV)
        remoe.lru_simulate(piece, N, C, 1, pos, state, m, t_, b_)
        torch.cuda.synchronize()
        got[:, pos:pos + n] = m
        total += t_.cpu()
        pos += n
    assert pos == T
    assert torch.equal(got.cpu(), rmiss) and torch.equal(total, rtot)


def test_trace_statistics_are_deterministic_and_ignore_bad_ids():
    N, K = 64, 6
    tr = wl.random_trace(5, 8, 200, K, N, 0.6).to(DEV)
    outs = []
    for _ in range(2):
        ov = torch.empty(8, 200, dtype=torch.uint8, device=DEV)
        s = torch.empty(8, dtype=torch.int64, device=DEV)
        remoe.trace_reuse(tr, N, ov, s)
        outs.append((ov.cpu(), s.cpu()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    # ids outside [0, N) are skipped, never used as an index
    bad = tr.clone()
    bad[0, 5, 0] = 1000
    bad[0, 6, 1] = -3
    ov = torch.empty(8, 200, dtype=torch.uint8, device=DEV)
    s = torch.empty(8, dtype=torch.int64, device=DEV)
    remoe.trace_reuse(bad, N, ov, s)
    miss = torch.empty(8, 200, dtype=torch.uint8, device=DEV)
    t_ = torch.empty(8, dtype=torch.int64, device=DEV)
    b_ = torch.empty(8, dtype=torch.int64, device=DEV)
    remoe.lru_simulate(bad, N, 16, 1, 0, None, miss, t_, b_)
    torch.cuda.synchronize()
    assert torch.equal(ov.cpu()[1:], outs[0][0][1:])
    assert int(miss[0, 5]) <= K - 1 and int(miss[0, 6]) <= K - 1


# --------------------------------------------------------------------------- whole layer

def test_tiny_config_end_to_end():
    """The fp32 Tiny configuration: layer output, expert ids, adjacent overlap and LRU misses."""
    cfg = wl.get_config("tiny")
    _say("forward tiny")
    w = wl.layer_weights(cfg, 0, DEV)
    x = wl.hidden_states(cfg, device=DEV).reshape(cfg.n_tokens, cfg.hidden).contiguous()
    desc = remoe.LayerDesc.from_config(cfg)
    y, idx, gw = _run_forward(desc, x, w)
    wc = to_oracle_weights(w)
    orc, ties, y_ref = oracle_layer(x.cpu(), wc, cfg.top_k, cfg.renorm, idx, gw)
    err = check_output(y, y_ref, "f32")
    _say(f"  tiny: max rel err {err:.2e}, tie tokens {len(ties)}")
    if not ties:
        assert torch.equal(torch.sort(idx.cpu(), 1).values, torch.sort(orc["idx"], 1).values)
    tr = idx.reshape(cfg.n_seq, cfg.seq_len, cfg.top_k).contiguous()
    ov = torch.empty(cfg.n_seq, cfg.seq_len, dtype=torch.uint8, device=DEV)
    s = torch.empty(cfg.n_seq, dtype=torch.int64, device=DEV)
    remoe.trace_reuse(tr, cfg.n_experts, ov, s)
    miss = torch.empty_like(ov)
    tot = torch.empty_like(s)
    nb = torch.empty_like(s)
    remoe.lru_simulate(tr, cfg.n_experts, cfg.capacities[0], cfg.expert_bytes, 0, None, miss, tot, nb)
    torch.cuda.synchronize()
    rov, rs = oracle.trace_reuse(tr.cpu(), cfg.n_experts)
    rmiss, rtot, rnb = oracle.lru_list(tr.cpu(), cfg.n_experts, cfg.capacities[0], cfg.expert_bytes)
    assert torch.equal(ov.cpu(), rov) and torch.equal(s.cpu(), rs)
    assert torch.equal(miss.cpu(), rmiss) and torch.equal(tot.cpu(), rtot) and torch.equal(nb.cpu(), rnb)
    assert cfg.expert_bytes == 393_216


@pytest.mark.parametrize("dtype,T,H,N,I,K,renorm,Is,gate", [
    ("f32", 200, 96, 5, 40, 2, True, 0, False),          # odd sizes on the fp32 path
    ("f32", 333, 64, 16, 24, 3, False, 56, True),
    ("bf16", 1500, 256, 8, 128, 2, False, 0, False),     # ~375 rows per expert: 3 row tiles, ragged
    ("bf16", 1000, 512, 60, 192, 4, False, 128, True),   # N not a multiple of 32, gated shared expert
    ("bf16", 700, 256, 64, 128, 6, False, 192, False),
    ("bf16", 513, 384, 128, 64, 8, True, 0, False),      # most experts get a handful of rows
    ("bf16", 1, 256, 16, 64, 4, True, 64, True),         # a single token
    ("bf16", 130, 128, 4, 64, 4, False, 0, False),       # K = N: every expert sees every token
])
def test_layer_forward_matches_oracle(dtype, T, H, N, I, K, renorm, Is, gate):
    _say(f"forward dtype={dtype} T={T} H={H} N={N} I={I} K={K} Is={Is} gate={gate}")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    w = _gen_layer(50 + N, H, N, I, Is, gate, dtype, std=0.05)
    x = wl.ar1_hidden_states(50 + N, 1, T, H, 0.8, tdt, DEV)[0].contiguous()
    desc = remoe.LayerDesc(H, N, I, K, int(renorm), Is, int(gate), 0 if dtype == "f32" else 1)
    y, idx, gw = _run_forward(desc, x, w)
    orc, ties, y_ref = oracle_layer(x.cpu(), to_oracle_weights(w), K, renorm, idx, gw)
    err = check_output(y, y_ref, dtype)
    _say(f"  err {err:.3e}, tie tokens {len(ties)}")
    # a second run gives the same bits (no floating-point atomics anywhere)
    y2, idx2, gw2 = _run_forward(desc, x, w)
    assert torch.equal(y.view(torch.int16 if dtype == "bf16" else torch.int32),
                       y2.view(torch.int16 if dtype == "bf16" else torch.int32))
    assert torch.equal(idx, idx2) and torch.equal(gw, gw2)


def test_layer_forward_many_tiles_per_workgroup_every_token():
    """65,536 tokens of a narrow layer: about 1,030 row tiles for 256 persistent workgroups, so every
    workgroup runs the multi-tile path of the grouped GEMM (next tile's first slice fetched under the
    epilogue, tiles claimed three ahead, ranges of other XCDs taken over at the end), and the layer
    is small enough for the oracle to evaluate EVERY token.  The workspace starts as bf16 NaNs, so a
    tile that was skipped shows; a tile claimed twice would not change the result, but a second run
    must reproduce the first bit for bit."""
    T, H, N, I, K = 65536, 128, 8, 64, 4
    _say(f"forward many tiles: T={T} H={H} N={N} I={I} K={K}")
    w = _gen_layer(58, H, N, I, 0, False, "bf16", std=0.05)
    x = wl.ar1_hidden_states(58, 16, T // 16, H, 0.8, torch.bfloat16, DEV).reshape(T, H).contiguous()
    desc = remoe.LayerDesc(H, N, I, K, 1, 0, 0, 1)
    outs = []
    for _ in range(2):
        ws = torch.full((remoe.remoe_workspace_bytes(desc, T),), 0xFF, dtype=torch.uint8, device=DEV)
        y = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device=DEV)
        idx = torch.full((T, K), -1, dtype=torch.int32, device=DEV)
        gw = torch.full((T, K), float("nan"), dtype=torch.float32, device=DEV)
        remoe.moe_forward(desc, x, w["w_router"], w["w_gate"], w["w_up"], w["w_down"], None, None, None, None,
                          y, idx, gw, ws)
        torch.cuda.synchronize()
        outs.append((y, idx, gw))
    y, idx, gw = outs[0]
    assert torch.isfinite(y.float()).all()
    assert torch.equal(y.view(torch.int16), outs[1][0].view(torch.int16))
    assert torch.equal(idx, outs[1][1]) and torch.equal(gw, outs[1][2])
    orc, ties, y_ref = oracle_layer(x.cpu(), to_oracle_weights(w), K, True, idx, gw)
    rep = {}
    err = check_output(y, y_ref, "bf16", rep)
    _say(f"  all {T} tokens: rel L2 {err:.3e}, worst row {rep['worst_row']:.3e}, tie tokens {len(ties)}")


def test_forward_routing_equals_moe_route():
    T, H, N, I, K = 400, 256, 64, 64, 6
    w = _gen_layer(61, H, N, I, 0, False, "bf16", std=0.05)
    x = wl.ar1_hidden_states(61, 1, T, H, 0.8, torch.bfloat16, DEV)[0].contiguous()
    desc = remoe.LayerDesc(H, N, I, K, 0, 0, 0, 1)
    _, idx_f, gw_f = _run_forward(desc, x, w)
    idx_r, gw_r, _, _ = _run_route(desc, x, w["w_router"], want_probs=False)
    assert torch.equal(idx_f, idx_r) and torch.equal(gw_f, gw_r)


def test_workspace_too_small_is_reported():
    desc = remoe.LayerDesc(256, 16, 64, 2, 0, 0, 0, 1)
    w = _gen_layer(62, 256, 16, 64, 0, False, "bf16")
    x = torch.zeros(64, 256, dtype=torch.bfloat16, device=DEV)
    y = torch.empty_like(x)
    idx = torch.empty(64, 2, dtype=torch.int32, device=DEV)
    gw = torch.empty(64, 2, dtype=torch.float32, device=DEV)
    ws = torch.empty(1024, dtype=torch.uint8, device=DEV)
    with pytest.raises(remoe.RemoeError, match="workspace"):
        remoe.moe_forward(desc, x, w["w_router"], w["w_gate"], w["w_up"], w["w_down"], None, None, None, None,
                          y, idx, gw, ws)


def test_copy_probe_copies_exactly():
    src = torch.arange(0, 3 * 1024 * 1024 + 16, dtype=torch.int32, device=DEV).view(torch.uint8)
    dst = torch.zeros_like(src)
    remoe.remoe_copy_probe(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    with pytest.raises(remoe.RemoeError):
        remoe.remoe_copy_probe(dst[:32], src[:48])
