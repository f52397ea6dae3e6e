"""Pins of the CPU oracle against things other than itself.

Each test checks oracle/remoe_oracle.c against what the paper or the
mathematics fixes: a full sort, closed forms, library routines on special
cases, brute force on tiny inputs, the paper's fetch bounds (Prop. 3.1 and the
longer-horizon bound of App. A) and the accounting identity behind Table 2.
All of it runs on the CPU.
"""
import math
import os

import pytest
import torch
import torch.nn.functional as F

import oracle
import workload as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def _layer(seed, H, N, I, Is=0, gate=False, dtype=torch.float32, std=0.05):
    g = lambda name, shape, dt: wl.gaussian(seed, name, shape, std, 0, 0, dt)
    w = {"w_router": g("w_router", (N, H), torch.float32),
         "w_gate": g("w_gate", (N, I, H), dtype), "w_up": g("w_up", (N, I, H), dtype),
         "w_down": g("w_down", (N, H, I), dtype),
         "ws_gate": None, "ws_up": None, "ws_down": None, "ws_scale": None}
    if Is:
        w["ws_gate"] = g("ws_gate", (Is, H), dtype)
        w["ws_up"] = g("ws_up", (Is, H), dtype)
        w["ws_down"] = g("ws_down", (H, Is), dtype)
        if gate:
            w["ws_scale"] = g("ws_scale", (H,), torch.float32)
    return w


def _x(seed, T, H, dtype=torch.float32, rho=0.8):
    return wl.ar1_hidden_states(seed, 1, T, H, rho, dtype)[0]


# --------------------------------------------------------------------------- router

def test_topk_equals_full_stable_sort():
    """E_t = Top-K(P_t) (Sec. 3.1): the K first entries of a full sort by logit."""
    T, H, N, K = 64, 48, 60, 4
    x = _x(11, T, H)
    wr = _layer(11, H, N, 8)["w_router"]
    r = oracle.route(x, wr, K, False, want_probs=True, want_logits=True)
    z = x.double() @ wr.double().T                     # library matmul, fp64
    assert torch.allclose(r["logits"], z, rtol=1e-12, atol=1e-12)
    order = torch.sort(-z, dim=1, stable=True).indices  # ties -> lower id
    assert torch.equal(r["idx"].long(), order[:, :K])
    p = torch.softmax(z, dim=1)
    assert torch.allclose(r["probs"], p, rtol=1e-12, atol=1e-15)
    assert torch.allclose(r["w"], torch.gather(p, 1, order[:, :K]), rtol=1e-12)
    zs = torch.sort(z, dim=1, descending=True).values
    assert torch.allclose(r["margin"], zs[:, K - 1] - zs[:, K], rtol=0, atol=1e-12)
    # selecting on probabilities is the same as selecting on logits
    assert torch.equal(torch.sort(-p, dim=1, stable=True).indices[:, :K], order[:, :K])


def test_topk_ties_go_to_lower_id():
    """Duplicated router rows give exactly equal logits; the lower id must win."""
    T, H, N, K = 16, 32, 8, 3
    x = _x(12, T, H)
    wr = _layer(12, H, N, 8)["w_router"]
    wr[5] = wr[2]
    wr[7] = wr[2]
    wr[1] = wr[0]
    r = oracle.route(x, wr, K, True, want_logits=True)
    z = r["logits"]
    assert torch.equal(z[:, 5], z[:, 2]) and torch.equal(z[:, 1], z[:, 0])
    order = torch.sort(-z, dim=1, stable=True).indices[:, :K]
    assert torch.equal(r["idx"].long(), order)
    for t in range(T):
        ids = r["idx"][t].tolist()
        if 5 in ids:
            assert 2 in ids and ids.index(2) < ids.index(5)
        if 7 in ids:
            assert 5 in ids and ids.index(5) < ids.index(7)
        if 1 in ids:
            assert 0 in ids and ids.index(0) < ids.index(1)
    # all-zero input: every logit equal, the K lowest ids are chosen, in order
    r0 = oracle.route(torch.zeros(2, H), wr, K, False)
    assert r0["idx"].tolist() == [[0, 1, 2], [0, 1, 2]]
    assert torch.allclose(r0["w"], torch.full((2, K), 1.0 / N, dtype=torch.float64))
    assert torch.equal(r0["margin"], torch.zeros(2, dtype=torch.float64))


def test_softmax_weight_sums():
    T, H, N, K = 32, 40, 16, 2
    x = _x(13, T, H)
    wr = _layer(13, H, N, 8, std=0.3)["w_router"]
    a = oracle.route(x, wr, K, False, want_probs=True)
    b = oracle.route(x, wr, K, True, want_probs=True)
    one = torch.ones(T, dtype=torch.float64)
    assert torch.allclose(a["probs"].sum(1), one, atol=1e-14)
    assert torch.allclose(b["w"].sum(1), one, atol=1e-14)
    sel = torch.gather(a["probs"], 1, a["idx"].long()).sum(1)
    assert torch.allclose(a["w"].sum(1), sel, atol=1e-15)
    assert (a["w"].sum(1) < 1.0).all()
    assert torch.equal(a["idx"], b["idx"])
    assert torch.allclose(b["w"], a["w"] / sel[:, None], rtol=1e-13)
    # weights arrive in descending order of probability
    assert (a["w"][:, :-1] >= a["w"][:, 1:]).all()
    big = 1000.0 * x                                    # overflow-safe softmax
    c = oracle.route(big, wr, K, False, want_probs=True)
    assert torch.isfinite(c["probs"]).all()
    assert torch.allclose(c["probs"].sum(1), one, atol=1e-14)


def test_k_equals_n_margin_infinite():
    x = _x(14, 4, 24)
    wr = _layer(14, 24, 5, 8)["w_router"]
    r = oracle.route(x, wr, 5, False)
    assert torch.isinf(r["margin"]).all()
    assert torch.allclose(r["w"].sum(1), torch.ones(4, dtype=torch.float64), atol=1e-14)
    assert sorted(r["idx"][0].tolist()) == [0, 1, 2, 3, 4]


# --------------------------------------------------------------------------- experts

def _torch_layer(x, w, idx, gw):
    """Independent fp64 evaluation with library matmuls, expert-major and batched."""
    xd = x.double()
    N = w["w_gate"].shape[0]
    T, H = xd.shape
    what = torch.zeros(T, N, dtype=torch.float64)
    what.scatter_add_(1, idx.long(), gw.double())
    g = torch.einsum("th,eih->tei", xd, w["w_gate"].double())
    u = torch.einsum("th,eih->tei", xd, w["w_up"].double())
    h = F.silu(g) * u
    ye = torch.einsum("tei,eoi->teo", h, w["w_down"].double())
    y = (what[:, :, None] * ye).sum(1)
    if w.get("ws_gate") is not None:
        hs = F.silu(xd @ w["ws_gate"].double().T) * (xd @ w["ws_up"].double().T)
        ys = hs @ w["ws_down"].double().T
        if w.get("ws_scale") is not None:
            ys = ys * torch.sigmoid(xd @ w["ws_scale"].double())[:, None]
        y = y + ys
    return y


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("Is,gate", [(0, False), (24, False), (40, True)])
def test_layer_against_library_matmuls(dtype, Is, gate):
    """Steps 4-6 against torch einsum/silu/sigmoid in fp64 (different code, different loop order)."""
    T, H, N, I, K = 12, 32, 6, 20, 3
    x = _x(21, T, H, dtype)
    w = _layer(21, H, N, I, Is, gate, dtype, std=0.2)
    r = oracle.forward(x, w, K, renorm=True)
    ref = _torch_layer(x, w, r["idx"], r["w"])
    assert torch.allclose(r["y"], ref, rtol=1e-11, atol=1e-13)
    assert ref.abs().max() > 1e-3


def test_sparse_equals_dense_masked():
    T, H, N, I, K = 10, 24, 7, 12, 3
    x = _x(22, T, H)
    w = _layer(22, H, N, I, 16, True, std=0.2)
    r = oracle.forward(x, w, K, renorm=False)
    dense = oracle.experts_dense_masked(x, r["idx"], r["w"], w)
    assert torch.allclose(r["y"], dense, rtol=1e-12, atol=1e-14)
    # token subset addressing
    sub = oracle.experts_sparse(x, r["idx"], r["w"], w, tokens=[7, 2, 2])
    assert torch.equal(sub[0], r["y"][7]) and torch.equal(sub[1], r["y"][2]) and torch.equal(sub[2], r["y"][2])


def test_single_expert_is_plain_swiglu_mlp():
    """N = K = 1: the router weight is 1 and the layer is one SwiGLU MLP."""
    T, H, I = 9, 28, 17
    x = _x(23, T, H)
    w = _layer(23, H, 1, I, std=0.3)
    r = oracle.forward(x, w, 1, renorm=False)
    assert torch.equal(r["w"], torch.ones(T, 1, dtype=torch.float64))
    xd = x.double()
    ref = (F.silu(xd @ w["w_gate"][0].double().T) * (xd @ w["w_up"][0].double().T)) @ w["w_down"][0].double().T
    assert torch.allclose(r["y"], ref, rtol=1e-12, atol=1e-14)


def test_all_experts_selected_is_softmax_mixture():
    T, H, N, I = 6, 20, 4, 10
    x = _x(24, T, H)
    w = _layer(24, H, N, I, std=0.3)
    r = oracle.forward(x, w, N, renorm=False)
    p = torch.softmax(x.double() @ w["w_router"].double().T, 1)
    idx_all = torch.arange(N, dtype=torch.int32).repeat(T, 1)
    ref = _torch_layer(x, w, idx_all, p)
    assert torch.allclose(r["y"], ref, rtol=1e-11, atol=1e-13)


def test_zero_gate_scaling_and_relabelling():
    T, H, N, I, K = 8, 24, 6, 10, 2
    x = _x(25, T, H)
    w = _layer(25, H, N, I, std=0.3)
    base = oracle.forward(x, w, K, True)
    # silu(0) = 0: a zero gate projection silences the experts
    wz = dict(w); wz["w_gate"] = torch.zeros_like(w["w_gate"])
    assert torch.equal(oracle.forward(x, wz, K, True)["y"], torch.zeros(T, H, dtype=torch.float64))
    # linear in the down projection (power of two: exact in floating point)
    ws = dict(w); ws["w_down"] = w["w_down"] * 4.0
    assert torch.equal(oracle.forward(x, ws, K, True)["y"], 4.0 * base["y"])
    # relabel experts: permute router rows and expert tensors together
    perm = torch.tensor([3, 0, 5, 1, 4, 2])
    wp = {k: (v[perm] if k in ("w_router", "w_gate", "w_up", "w_down") else v) for k, v in w.items()}
    rp = oracle.forward(x, wp, K, True)
    assert torch.equal(perm[rp["idx"].long()].int(), base["idx"])
    assert torch.allclose(rp["y"], base["y"], rtol=1e-13, atol=1e-15)


def test_bf16_inputs_are_widened_exactly():
    T, H, N = 5, 16, 4
    x = _x(26, T, H, torch.bfloat16)
    wr = _layer(26, H, N, 4)["w_router"]
    r = oracle.route(x, wr, 1, False, want_logits=True)
    assert torch.allclose(r["logits"], x.double() @ wr.double().T, rtol=1e-13, atol=1e-15)
    xf = x.float()
    rf = oracle.route(xf, wr, 1, False, want_logits=True)
    assert torch.equal(r["logits"], rf["logits"])


# --------------------------------------------------------------------------- trace statistics

def _brute_lru(trace, N, C):
    """Recency keys (last step, id); residents before a step = the C largest keys so far."""
    T = len(trace)
    last = {}
    out = []
    for t in range(T):
        keys = sorted(((s, e) for e, s in last.items()), reverse=True)[:C]
        resident = {e for _, e in keys}
        U = set(trace[t])
        out.append(len(U - resident))
        for e in U:
            last[e] = t
    return out


def test_worked_example_by_hand():
    """N=6, K=2, C=3, worked by hand from the per-step definition M = |U_t \\ C_t| (App. E.2)."""
    tr = torch.tensor([[[0, 1], [1, 2], [3, 4], [0, 1], [1, 5]]], dtype=torch.int32)
    miss, tot, nbytes = oracle.lru_list(tr, 6, 3, expert_bytes=1000)
    assert miss[0].tolist() == [2, 1, 2, 2, 1]
    assert tot.tolist() == [8] and nbytes.tolist() == [8000]
    ov, s = oracle.trace_reuse(tr, 6)
    assert ov[0].tolist() == [0, 1, 0, 0, 1] and s.tolist() == [2]


@pytest.mark.parametrize("N,K,C,stick,distinct", [
    (8, 2, 3, 0.5, True), (16, 4, 4, 0.6, True), (16, 4, 9, 0.3, True), (12, 6, 4, 0.7, True),
    (10, 3, 5, 0.5, False), (128, 8, 32, 0.8, True), (5, 5, 2, 0.0, True), (6, 2, 1, 0.5, True),
])
def test_lru_list_equals_brute_force(N, K, C, stick, distinct):
    tr = wl.random_trace(100 + N + K + C, 3, 60, K, N, stick, distinct)
    miss, tot, _ = oracle.lru_list(tr, N, C)
    for s in range(tr.shape[0]):
        ref = _brute_lru(tr[s].tolist(), N, C)
        assert miss[s].tolist() == ref
        assert int(tot[s]) == sum(ref)


def test_overlap_properties():
    N, K = 16, 4
    tr = wl.random_trace(7, 4, 80, K, N, 0.5)
    ov, s = oracle.trace_reuse(tr, N)
    assert (ov[:, 0] == 0).all()
    assert (ov <= K).all()
    for q in range(tr.shape[0]):
        for t in range(1, tr.shape[1]):
            assert int(ov[q, t]) == len(set(tr[q, t].tolist()) & set(tr[q, t - 1].tolist()))
    assert torch.equal(s, ov.long().sum(1))
    # identical steps -> K, disjoint steps -> 0, symmetric in its two arguments
    same = torch.tensor([[[1, 2, 3, 4]] * 5], dtype=torch.int32)
    assert oracle.trace_reuse(same, N)[0][0].tolist() == [0, K, K, K, K]
    disj = torch.tensor([[[0, 1, 2, 3], [4, 5, 6, 7], [0, 1, 2, 3]]], dtype=torch.int32)
    assert oracle.trace_reuse(disj, N)[0][0].tolist() == [0, 0, 0]
    a, b = tr[0, 10], tr[0, 11]
    ab = oracle.trace_reuse(torch.stack([a, b])[None], N)[0][0, 1]
    ba = oracle.trace_reuse(torch.stack([b, a])[None], N)[0][0, 1]
    assert ab == ba
    # order inside a step and repeated ids do not matter (set semantics)
    rep = torch.tensor([[[2, 2, 5, 1], [5, 5, 5, 2]]], dtype=torch.int32)
    assert oracle.trace_reuse(rep, N)[0][0].tolist() == [0, 2]
    # sequences never see each other
    two = torch.cat([same, same])
    assert oracle.trace_reuse(two, N)[0][1, 0] == 0


def test_fetch_bound_tight_at_c_equals_k():
    """C = K: the cache holds exactly E_{t-1}, so misses = K - overlap (App. A, tightness)."""
    N, K = 32, 6
    tr = wl.random_trace(8, 5, 100, K, N, 0.6)
    ov, _ = oracle.trace_reuse(tr, N)
    miss, _, _ = oracle.lru_list(tr, N, K)
    assert (miss[:, 0] == K).all()                      # cold start (Sec. 3, request isolation)
    assert torch.equal(miss[:, 1:], K - ov[:, 1:])


@pytest.mark.parametrize("C", [6, 7, 10, 20])
def test_fetch_bounds_for_c_ge_k(C):
    """Prop. 3.1: N_fetch(t) <= K - |E_t ∩ E_{t-1}|, and the longer-horizon working-set bound."""
    N, K = 24, 6
    tr = wl.random_trace(9, 4, 120, K, N, 0.5)
    ov, _ = oracle.trace_reuse(tr, N)
    miss, _, _ = oracle.lru_list(tr, N, C)
    assert (miss[:, 1:] <= K - ov[:, 1:]).all()
    for s in range(tr.shape[0]):
        steps = [set(v) for v in tr[s].tolist()]
        for t in range(1, len(steps)):
            U, best = set(), set()
            for ell in range(1, t + 1):
                U = U | steps[t - ell]
                if len(U) > C:
                    break
                best = set(U)
            assert int(miss[s, t]) <= K - len(steps[t] & best)


def test_c_below_k_always_misses_at_least_k_minus_c():
    """Failure mode 1 of App. A: with C < K at least K - C experts miss at every step."""
    N, K, C = 16, 6, 4
    same = torch.tensor([[[0, 1, 2, 3, 4, 5]] * 6], dtype=torch.int32)
    miss, _, _ = oracle.lru_list(same, N, C)
    assert miss[0].tolist() == [6, 2, 2, 2, 2, 2]
    tr = wl.random_trace(10, 3, 80, K, N, 0.7)
    miss, _, _ = oracle.lru_list(tr, N, C)
    assert (miss >= K - C).all()


def test_big_cache_counts_distinct_experts_and_monotone_in_c():
    N, K = 20, 4
    tr = wl.random_trace(11, 4, 90, K, N, 0.4)
    totals = []
    for C in range(1, N + 3):
        _, tot, _ = oracle.lru_list(tr, N, C)
        totals.append(tot)
    for a, b in zip(totals, totals[1:]):
        assert (b <= a).all()                           # LRU is a stack algorithm
    distinct = torch.tensor([len(set(tr[s].flatten().tolist())) for s in range(tr.shape[0])])
    assert torch.equal(totals[N - 1], distinct)
    assert torch.equal(totals[-1], distinct)


def test_table2_accounting_identity():
    """Table 2: #uMiss = (1 - uHR) * (prompts * steps * layers * K) for every LRU row.

    This fixes the accounting the oracle must follow: cold-start misses are
    counted, every layer-step contributes exactly K unique requests at B = 1,
    and uHR = 1 - #uMiss / sum |U|.  The same identity is then checked on the
    oracle's own counts for a synthetic trace of the paper's shape.
    """
    prompts, steps, layers, K, N = 128, 64, 26, 6, 64
    requests = prompts * steps * layers * K
    assert requests == 1_277_952
    rows = []
    with open(os.path.join(HERE, "golden", "paper_table2_lru.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([float(v) for v in line.split()])
    assert [int(r[0]) for r in rows] == [4, 6, 8, 12]
    for C, hr_b, hr_r, m_b, m_r in rows:
        assert abs((1 - hr_b) * requests / 1e6 - m_b) < 1.5e-4
        assert abs((1 - hr_r) * requests / 1e6 - m_r) < 1.5e-4
    S = prompts * layers
    tr = wl.random_trace(12, 64, steps, K, N, 0.5)      # a slice of the shape keeps the test quick
    for C in (4, 6, 8, 12):
        miss, tot, nbytes = oracle.lru_list(tr, N, C, expert_bytes=17_301_504)
        hits = 0
        for s in range(tr.shape[0]):
            ref = _brute_lru(tr[s].tolist(), N, C)
            hits += sum(K - m for m in ref)
        total_req = tr.shape[0] * steps * K
        assert int(tot.sum()) + hits == total_req
        assert (miss[:, 0] == K).all()
        assert torch.equal(nbytes, tot * 17_301_504)
    assert S * steps * K == requests


def test_out_of_range_ids_are_rejected():
    bad = torch.tensor([[[0, 9]]], dtype=torch.int32)
    with pytest.raises(RuntimeError):
        oracle.trace_reuse(bad, 8)
    with pytest.raises(RuntimeError):
        oracle.lru_list(bad, 8, 2)
    with pytest.raises(RuntimeError):
        oracle.lru_list(torch.zeros(1, 1, 1, dtype=torch.int32), 8, 0)


# --------------------------------------------------------------------------- workload sanity

def test_overlap_statistics_of_the_synthetic_workload():
    """At rho = 0 consecutive Top-K sets are independent: E|E_t ∩ E_{t-1}| = K^2 / N (hypergeometric
    mean); overlap grows with the AR(1) correlation."""
    H, N, K, T = 128, 60, 4, 3000
    wr = wl.gaussian(2, "w_router", (N, H), 0.02)
    means = []
    for rho in (0.0, 0.5, 0.9):
        x = wl.ar1_hidden_states(2, 1, T, H, rho)[0]
        idx = oracle.route(x, wr, K, False)["idx"]
        ov, s = oracle.trace_reuse(idx[None], N)
        means.append(float(s[0]) / (T - 1))
    assert abs(means[0] - K * K / N) < 0.05
    assert means[0] < means[1] < means[2]
    assert means[2] > 4 * means[0]


def test_generator_is_deterministic_and_chunk_invariant():
    a = wl.gaussian(3, "w_gate", (5, 7, 11), 0.02)
    b = wl.gaussian(3, "w_gate", (5 * 7 * 11,), 0.02)
    assert torch.equal(a.flatten(), b)
    c = wl.gaussian(4, "w_gate", (5, 7, 11), 0.02)
    assert not torch.equal(a, c)
    x1 = wl.ar1_hidden_states(5, 3, 40, 8, 0.8)
    x2 = wl.ar1_hidden_states(5, 2, 40, 8, 0.8)
    assert torch.equal(x1[:2], x2)
    big = wl.gaussian(6, "x", (200_000,), 1.0, dtype=torch.float64)
    assert abs(float(big.mean())) < 0.01 and abs(float(big.std()) - 1) < 0.01
    xs = wl.ar1_hidden_states(7, 1, 20_000, 4, 0.8, torch.float64)[0]
    r1 = float((xs[1:] * xs[:-1]).mean())
    assert abs(r1 - 0.8) < 0.03 and abs(float(xs.var()) - 1) < 0.06


# ---- the oracle's C code under the address and undefined-behaviour sanitizers --------------------
def test_oracle_is_clean_under_sanitizers():
    """Every oracle function on small inputs (one token, one expert, K = N_r, C < K, repeated ids, empty
    traces, short histograms, long lags) in a build with -fsanitize=address,undefined: an access past
    the end of an exactly sized buffer, a signed overflow or a misaligned access ends the run."""
    import subprocess

    from oracle import build as oracle_build

    exe = oracle_build.build_sanitized()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "sanitize_check ok" in r.stdout, r.stdout + r.stderr
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
