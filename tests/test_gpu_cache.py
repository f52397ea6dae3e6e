"""GPU parity of cache_simulate, step_miss_summary and routing_balance against the CPU oracle.

Integer results (misses, hits, totals, bytes, sums, histogram, percentiles, loads, experts used) are
compared bit for bit; the two fp64 balance figures to 1e-12 (the kernel adds the per-expert terms
in a tree, the oracle one after the other).
"""
import time

import pytest
import torch

import oracle
import paper_2605_27081_amd as remoe
import workload as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
POLICY = {"lru": remoe.REMOE_CACHE_LRU, "fifo": remoe.REMOE_CACHE_FIFO, "lfu": remoe.REMOE_CACHE_LFU,
          "belady": remoe.REMOE_CACHE_BELADY}


def _say(msg):
    print(msg, flush=True)


def _trace(seed, S, T, K, N, distinct=True, skew=0.0):
    g = torch.Generator().manual_seed(seed)
    if distinct:
        w = torch.arange(1, N + 1, dtype=torch.float64) ** (-skew)
        rows = torch.stack([torch.multinomial(w, K, replacement=False, generator=g) for _ in range(S * T)])
        return rows.reshape(S, T, K).to(torch.int32)
    return torch.randint(0, N, (S, T, K), generator=g, dtype=torch.int32)


def _gpu_cache(idx, N, C, policy, expert_bytes):
    S, T, K = idx.shape
    d = idx.to(DEV)
    out = {k: torch.full((S, T), 255, dtype=torch.uint8, device=DEV) for k in ("miss", "uniq", "hit_tok")}
    out.update({k: torch.full((S,), -1, dtype=torch.int64, device=DEV) for k in ("total_miss", "total_uniq", "bytes")})
    nb = remoe.remoe_cache_workspace_bytes(S, T, K, POLICY[policy])
    ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=DEV) if nb else None
    remoe.cache_simulate(d, N, C, POLICY[policy], expert_bytes, out["miss"], out["uniq"], out["hit_tok"],
                         out["total_miss"], out["total_uniq"], out["bytes"], ws)
    torch.cuda.synchronize()
    return {k: v.cpu() for k, v in out.items()}


@pytest.mark.parametrize("policy", ["lru", "fifo", "lfu", "belady"])
@pytest.mark.parametrize("S,T,K,N,C,distinct,skew", [
    (3, 50, 1, 6, 3, False, 0.0),       # one request per step
    (5, 130, 2, 16, 4, True, 0.0),      # several 64-step batches and a ragged tail
    (4, 200, 6, 64, 16, True, 1.0),     # DeepSeek-V2-Lite-shaped trace, skewed popularity
    (2, 300, 8, 128, 32, True, 0.5),    # Qwen3-shaped trace: both halves of the expert range
    (3, 90, 4, 60, 12, True, 0.0),      # Qwen1.5-shaped
    (2, 70, 4, 12, 5, False, 0.0),      # repeated ids inside a step
    (2, 40, 6, 20, 3, True, 0.0),       # C < K
    (2, 33, 4, 9, 9, True, 0.0),        # C = N_r
    (1, 1, 3, 8, 2, True, 0.0),         # a single step
])
def test_cache_policies_match_oracle(policy, S, T, K, N, C, distinct, skew):
    _say(f"cache {policy} S={S} T={T} K={K} N={N} C={C}")
    idx = _trace(S * 1000 + T + K, S, T, K, N, distinct, skew)
    got = _gpu_cache(idx, N, C, policy, 9437184)
    ref = oracle.cache_policy(idx, N, C, policy, 9437184)
    for k in ("miss", "uniq", "hit_tok", "total_miss", "total_uniq", "bytes"):
        assert torch.equal(got[k], ref[k]), k


def test_cache_lru_equals_lru_simulate():
    """The sequential LRU of cache_simulate and the parallel walk of lru_simulate are two kernels for one definition."""
    idx = _trace(77, 6, 500, 8, 128, True, 0.7).to(DEV)
    S, T, K = idx.shape
    a = _gpu_cache(idx.cpu(), 128, 32, "lru", 11)
    miss = torch.empty(S, T, dtype=torch.uint8, device=DEV)
    tot = torch.empty(S, dtype=torch.int64, device=DEV)
    nb = torch.empty(S, dtype=torch.int64, device=DEV)
    remoe.lru_simulate(idx, 128, 32, 11, 0, None, miss, tot, nb)
    torch.cuda.synchronize()
    assert torch.equal(a["miss"], miss.cpu()) and torch.equal(a["total_miss"], tot.cpu()) and torch.equal(a["bytes"], nb.cpu())


def test_cache_full_length_trace_sampled():
    """A full-length (4096-step) trace of the Qwen3-shaped configuration: totals of every policy against the
    oracle on a few traces, and Belady below the others on all of them."""
    cfg = wl.get_config("qwen3_prefill")
    idx = _trace(5, 4, cfg.seq_len, cfg.top_k, cfg.n_experts, True, 0.8)
    tot = {}
    for p in POLICY:
        got = _gpu_cache(idx, cfg.n_experts, 32, p, cfg.expert_bytes)
        t0 = time.perf_counter()
        ref = oracle.cache_policy(idx[:2], cfg.n_experts, 32, p, cfg.expert_bytes)
        dt = time.perf_counter() - t0
        # the oracle's rate on its two traces, to set beside bench_extras.py's figure for the kernel
        _say(f"oracle cache_policy[{p}]: {2 * cfg.seq_len / dt:.3g} trace-steps/s (2 traces x {cfg.seq_len} steps in {dt * 1e3:.1f} ms)")
        assert torch.equal(got["miss"][:2], ref["miss"]) and torch.equal(got["total_miss"][:2], ref["total_miss"])
        tot[p] = got["total_miss"]
    for p in ("lru", "fifo", "lfu"):
        assert (tot["belady"] <= tot[p]).all()


@pytest.mark.parametrize("policy", ["lru", "fifo", "lfu", "belady"])
def test_cache_policies_keep_the_served_step(policy):
    """App. A (step atomicity and admission) on the kernel's own output: with C >= K no policy evicts an
    expert of the step it has just served, so every step fetches at most K - |E_t n E_{t-1}| experts."""
    K, N, C = 8, 128, 16
    idx = _trace(31, 6, 700, K, N, True, 0.9)
    got = _gpu_cache(idx, N, C, policy, 1)
    ov, _ = oracle.trace_reuse(idx, N)
    assert (got["miss"][:, 1:].long() <= K - ov[:, 1:].long()).all()


def test_cache_rejects_bad_arguments():
    idx = torch.zeros(1, 4, 2, dtype=torch.int32, device=DEV)
    z8 = torch.zeros(1, 4, dtype=torch.uint8, device=DEV)
    z64 = torch.zeros(1, dtype=torch.int64, device=DEV)
    with pytest.raises(remoe.RemoeError, match="capacity"):
        remoe.cache_simulate(idx, 8, 0, 0, 1, z8, z8, z8, z64, z64, z64)
    with pytest.raises(remoe.RemoeError, match="policy"):
        remoe.cache_simulate(idx, 8, 2, 9, 1, z8, z8, z8, z64, z64, z64)
    with pytest.raises(remoe.RemoeError, match="workspace"):
        remoe.cache_simulate(idx, 8, 2, remoe.REMOE_CACHE_BELADY, 1, z8, z8, z8, z64, z64, z64, None)


@pytest.mark.parametrize("L,S,T,hist_len", [(3, 2, 50, 19), (26, 4, 64, 157), (48, 16, 500, 385), (1, 1, 7, 7), (4, 3, 9, 5)])
def test_step_summary_matches_oracle(L, S, T, hist_len):
    g = torch.Generator().manual_seed(L * S + T)
    miss = torch.randint(0, 7, (L, S, T), generator=g, dtype=torch.uint8)
    out_all = torch.zeros(S, T, dtype=torch.int16, device=DEV)
    hist = torch.full((hist_len,), -1, dtype=torch.int64, device=DEV)
    pct = torch.zeros(3, dtype=torch.int32, device=DEV)
    remoe.step_miss_summary(miss.to(DEV), out_all, hist, pct)
    torch.cuda.synchronize()
    rall, rhist, rpct = oracle.step_summary(miss, hist_len)
    assert torch.equal(out_all.cpu().to(torch.int32) & 0xFFFF, rall)
    assert torch.equal(hist.cpu(), rhist) and torch.equal(pct.cpu(), rpct)


def test_step_summary_of_gpu_misses_end_to_end():
    """Layers x sequences of LRU misses -> per-step sums and percentiles, all on the GPU, against the oracle chain."""
    L, S, T, K, N, C = 6, 3, 120, 4, 32, 8
    idx = _trace(3, L * S, T, K, N)
    d = idx.to(DEV)
    miss = torch.empty(L * S, T, dtype=torch.uint8, device=DEV)
    tot = torch.empty(L * S, dtype=torch.int64, device=DEV)
    nb = torch.empty(L * S, dtype=torch.int64, device=DEV)
    remoe.lru_simulate(d, N, C, 1, 0, None, miss, tot, nb)
    out_all = torch.zeros(S, T, dtype=torch.int16, device=DEV)
    hist = torch.zeros(L * K + 1, dtype=torch.int64, device=DEV)
    pct = torch.zeros(3, dtype=torch.int32, device=DEV)
    remoe.step_miss_summary(miss.view(L, S, T), out_all, hist, pct)
    torch.cuda.synchronize()
    rmiss, _, _ = oracle.lru_list(idx, N, C, 1)
    rall, rhist, rpct = oracle.step_summary(rmiss.view(L, S, T), L * K + 1)
    assert torch.equal(out_all.cpu().to(torch.int32) & 0xFFFF, rall) and torch.equal(hist.cpu(), rhist)
    assert torch.equal(pct.cpu(), rpct)


@pytest.mark.parametrize("S,T,K,N,skew", [(3, 100, 4, 20, 0.0), (4, 2048, 6, 64, 1.0), (2, 4096, 8, 128, 0.5),
                                          (2, 10, 1, 1, 0.0), (1, 5, 2, 60, 0.0)])
def test_balance_matches_oracle(S, T, K, N, skew):
    idx = _trace(S + T, S, T, K, N, True, skew)
    load = torch.zeros(S, N, dtype=torch.int32, device=DEV)
    used = torch.zeros(S, dtype=torch.int32, device=DEV)
    ent = torch.zeros(S, dtype=torch.float64, device=DEV)
    cv = torch.zeros(S, dtype=torch.float64, device=DEV)
    remoe.routing_balance(idx.to(DEV), N, load, used, ent, cv)
    torch.cuda.synchronize()
    rload, rused, rent, rcv = oracle.balance(idx, N)
    assert torch.equal(load.cpu().to(torch.int64), rload) and torch.equal(used.cpu(), rused)
    assert torch.allclose(ent.cpu(), rent, rtol=1e-12, atol=1e-14) and torch.allclose(cv.cpu(), rcv, rtol=1e-12, atol=1e-14)


def _probs(seed, S, T, N, temp=2.0):
    g = torch.Generator().manual_seed(seed)
    return torch.softmax(torch.randn(S, T, N, generator=g) * temp, -1).float().contiguous()


@pytest.mark.parametrize("S,T,N,K,C,factor,renorm", [
    (3, 40, 8, 2, 3, 1.0, False),          # no bonus: the plain router
    (4, 130, 64, 6, 4, 2.718281828, False),   # DeepSeek-V2-Lite shape, C = 4 < K as in the appendix, beta = 1
    (2, 200, 128, 8, 32, 7.389056099, True),  # Qwen3 shape, beta = 2, renormalised weights
    (3, 77, 60, 4, 12, 54.59815003, False),   # beta = 4
    (2, 50, 16, 16, 16, 3.0, True),        # K = N
    (2, 9, 5, 1, 1, 1e12, False),          # overwhelming bonus
])
def test_reroute_matches_oracle(S, T, N, K, C, factor, renorm):
    _say(f"reroute S={S} T={T} N={N} K={K} C={C} factor={factor}")
    p = _probs(S * T + N, S, T, N)
    idx = torch.full((S, T, K), -1, dtype=torch.int32, device=DEV)
    w = torch.zeros(S, T, K, dtype=torch.float32, device=DEV)
    miss = torch.full((S, T), 255, dtype=torch.uint8, device=DEV)
    tot = torch.full((S,), -1, dtype=torch.int64, device=DEV)
    remoe.reroute_lru(p.to(DEV), K, C, factor, renorm, idx, w, miss, tot)
    torch.cuda.synchronize()
    ref = oracle.reroute_lru(p, K, C, factor, renorm)
    assert torch.equal(idx.cpu(), ref["idx"]) and torch.equal(miss.cpu(), ref["miss"])
    assert torch.equal(tot.cpu(), ref["total_miss"])
    assert torch.allclose(w.cpu().double(), ref["w"], rtol=2e-6, atol=1e-12)


def test_reroute_of_router_probabilities_end_to_end():
    """moe_route's full probabilities fed to reroute_lru: with factor 1 the rerouted ids are the router's own
    and the misses are those of lru_simulate on them."""
    H, N, K, C, S, T = 256, 64, 6, 8, 2, 64
    x = wl.ar1_hidden_states(3, S, T, H, 0.8, torch.float32, DEV).reshape(S * T, H).contiguous()
    wr = wl.gaussian(3, "w_router", (N, H), 0.05, 0, 0, torch.float32, DEV)
    desc = remoe.LayerDesc(H, N, 64, K, 0, 0, 0, 0)
    ridx = torch.empty(S * T, K, dtype=torch.int32, device=DEV)
    rw = torch.empty(S * T, K, dtype=torch.float32, device=DEV)
    probs = torch.empty(S * T, N, dtype=torch.float32, device=DEV)
    remoe.moe_route(desc, x, wr, ridx, rw, None, probs)
    idx = torch.empty(S, T, K, dtype=torch.int32, device=DEV)
    w = torch.empty(S, T, K, dtype=torch.float32, device=DEV)
    miss = torch.empty(S, T, dtype=torch.uint8, device=DEV)
    tot = torch.empty(S, dtype=torch.int64, device=DEV)
    remoe.reroute_lru(probs.view(S, T, N), K, C, 1.0, False, idx, w, miss, tot)
    lmiss = torch.empty(S, T, dtype=torch.uint8, device=DEV)
    ltot = torch.empty(S, dtype=torch.int64, device=DEV)
    lb = torch.empty(S, dtype=torch.int64, device=DEV)
    remoe.lru_simulate(ridx.view(S, T, K), N, C, 1, 0, None, lmiss, ltot, lb)
    torch.cuda.synchronize()
    assert torch.equal(torch.sort(idx.cpu(), -1).values, torch.sort(ridx.view(S, T, K).cpu(), -1).values)
    assert torch.equal(miss.cpu(), lmiss.cpu()) and torch.equal(tot.cpu(), ltot.cpu())
    # a bonus can only be tried on the same probabilities: it must not lose to no bonus here
    remoe.reroute_lru(probs.view(S, T, N), K, C, 20.0, False, idx, w, miss, tot)
    torch.cuda.synchronize()
    assert int(tot.sum()) < int(ltot.sum())
