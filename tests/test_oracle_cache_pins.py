"""Pins of the cache-policy, step-summary and balance oracles (CPU only).

Each pin fixes the oracle to something other than itself: textbook single-request simulations
written here with Python containers, the list LRU of the first oracle file, exhaustive search for
the least possible number of misses, the paper's own table, numpy's percentile, closed forms.
"""
import collections
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _trace(seed, S, T, K, N, distinct=True):
    g = torch.Generator().manual_seed(seed)
    if distinct:
        rows = [torch.randperm(N, generator=g)[:K] for _ in range(S * T)]
        return torch.stack(rows).reshape(S, T, K).to(torch.int32)
    return torch.randint(0, N, (S, T, K), generator=g, dtype=torch.int32)


# ---- LRU through the generic rule == the list form of the first file ---------------------------
@pytest.mark.parametrize("K,N,C", [(1, 6, 3), (2, 9, 4), (4, 16, 4), (6, 20, 3), (3, 8, 8)])
def test_lru_policy_equals_list_lru(K, N, C):
    idx = _trace(K * 100 + C, 3, 60, K, N, distinct=(K > 1))
    a = oracle.cache_policy(idx, N, C, "lru", 7)
    miss, tot, nbytes = oracle.lru_list(idx, N, C, 7)
    assert torch.equal(a["miss"], miss) and torch.equal(a["total_miss"], tot) and torch.equal(a["bytes"], nbytes)


# ---- FIFO / LFU at one request per step == the textbook algorithms ------------------------------
def _textbook_fifo(seq, C):
    q, miss = collections.deque(), []
    for e in seq:
        if e in q:
            miss.append(0)
            continue
        miss.append(1)
        q.append(e)
        if len(q) > C:
            q.popleft()
    return miss


def _textbook_lfu(seq, C):
    """LFU with request counts kept for the whole sequence, least-recently-used among equals: on a miss
    with a full cache the victim is chosen among the pages already held, then the new page comes in."""
    cache, freq, last, miss = set(), collections.Counter(), {}, []
    for t, e in enumerate(seq):
        miss.append(0 if e in cache else 1)
        if e not in cache and len(cache) == C:
            cache.remove(min(cache, key=lambda x: (freq[x], last[x], x)))
        freq[e] += 1
        last[e] = t
        cache.add(e)
    return miss


@pytest.mark.parametrize("N,C", [(5, 2), (8, 3), (12, 5)])
def test_fifo_lfu_single_request_match_textbook(N, C):
    idx = _trace(N + C, 4, 200, 1, N, distinct=False)
    fifo = oracle.cache_policy(idx, N, C, "fifo")
    lfu = oracle.cache_policy(idx, N, C, "lfu")
    for s in range(idx.shape[0]):
        seq = idx[s, :, 0].tolist()
        assert fifo["miss"][s].tolist() == _textbook_fifo(seq, C)
        assert lfu["miss"][s].tolist() == _textbook_lfu(seq, C)


def test_fifo_hit_does_not_renew():
    # C = 2: 0, 1, then 0 again (hit), then 2 evicts 0 (the oldest arrival) under FIFO but 1 under LRU
    idx = torch.tensor([[[0], [1], [0], [2], [0], [1]]], dtype=torch.int32)
    assert oracle.cache_policy(idx, 3, 2, "fifo")["miss"][0].tolist() == [1, 1, 0, 1, 1, 1]
    assert oracle.cache_policy(idx, 3, 2, "lru")["miss"][0].tolist() == [1, 1, 0, 1, 0, 1]


# ---- the in-step rules, hand-worked at K = 2 --------------------------------------------------------
def test_fifo_two_requests_per_step_hand_worked():
    """FIFO, N = 5, K = 2, C = 3.  Two experts fetched in the same step have the same age; the lower id
    counts as the earlier arrival and leaves first.
      t0 {0,1}: cold, 2 misses.                      held {0,1}
      t1 {2,3}: 2 misses; 4 held > 3; candidates outside the step: 0, 1 (both fetched at t0) -> 0 leaves.
                                                      held {1,2,3}
      t2 {1,4}: 1 hits, 4 misses -> 1 (had 1 left instead of 0 this would be 2).
                4 held; candidates 2, 3 (both fetched at t1) -> 2 leaves.   held {1,3,4}
      t3 {3,0}: 3 hits, 0 misses -> 1 (had 3 left instead of 2 this would be 2).
                candidates 1 (t0), 4 (t2) -> 1 leaves.                      held {0,3,4}
      t4 {4,1}: 4 hits, 1 misses -> 1."""
    idx = torch.tensor([[[0, 1], [2, 3], [1, 4], [3, 0], [4, 1]]], dtype=torch.int32)
    assert oracle.cache_policy(idx, 5, 3, "fifo")["miss"][0].tolist() == [2, 2, 1, 1, 1]


def test_fifo_keeps_what_the_step_requested():
    """FIFO, C = K = 2: t0 {0,1}; t1 {0,2}: 0 hits, 2 misses, and the expert that leaves is 1, the only
    one the step did not ask for -- not 0, although 0 is the oldest arrival (App. A: an expert used in a
    step is not evicted before the step is over).  t2 {0,2} then hits twice: miss_t <= K - overlap_t = 0."""
    idx = torch.tensor([[[0, 1], [0, 2], [0, 2]]], dtype=torch.int32)
    assert oracle.cache_policy(idx, 3, 2, "fifo")["miss"][0].tolist() == [2, 1, 0]
    assert oracle.cache_policy(idx, 3, 2, "lfu")["miss"][0].tolist() == [2, 1, 0]


def test_lfu_two_requests_per_step_hand_worked():
    """LFU, N = 5, K = 2, C = 4; counts are kept across evictions, equal counts go by last use, equal last
    use by id (lower id leaves first).
      t0 {0,1}: 2 misses.  counts 0:1 1:1                        held {0,1}
      t1 {0,2}: 0 hits, 2 misses -> 1.  counts 0:2 1:1 2:1         held {0,1,2}
      t2 {3,4}: 2 misses; 5 held > 4; outside the step: 0 (count 2), 1 (count 1, last t0), 2 (count 1, last t1)
                -> 1 leaves.                                      held {0,2,3,4}
      t3 {1,2}: 1 misses, 2 hits -> 1.  counts 1:2 2:2; outside the step: 0 (2), 3 (1, last t2), 4 (1, last t2)
                -> equal count and last use: 3 leaves.            held {0,1,2,4}
      t4 {4,0}: both hit -> 0 (had 4 left instead of 3 this would be 1).
      t5 {3,4}: 3 misses -> 1."""
    idx = torch.tensor([[[0, 1], [0, 2], [3, 4], [1, 2], [4, 0], [3, 4]]], dtype=torch.int32)
    assert oracle.cache_policy(idx, 5, 4, "lfu")["miss"][0].tolist() == [2, 1, 2, 1, 0, 1]


@pytest.mark.parametrize("policy", list(oracle.POLICIES))
@pytest.mark.parametrize("K,N,C", [(2, 6, 2), (2, 9, 3), (4, 16, 4), (6, 20, 8), (8, 128, 32)])
def test_every_policy_keeps_the_served_step(policy, K, N, C):
    """App. A: with C >= K every policy keeps E_t for the next step, so Prop. 3.1's bound
    miss_t <= K - |E_t n E_{t-1}| holds for t >= 2 whatever the policy."""
    idx = _trace(K * 7 + C, 4, 150, K, N)
    miss = oracle.cache_policy(idx, N, C, policy)["miss"].long()
    ov, _ = oracle.trace_reuse(idx, N)
    assert (miss[:, 1:] <= K - ov[:, 1:].long()).all()


# ---- Belady == the least number of misses any replacement choice can reach ----------------------
def _least_misses(steps, C):
    """Exhaustive search over every replacement choice of a cache that serves and keeps each step's
    request (App. A): after a step the resident set is any subset of resident | requested of size
    <= C that contains the request (or, when the request alone exceeds C, any C of the requested)."""
    best = {frozenset(): 0}
    for req in steps:
        nxt = {}
        for res, m in best.items():
            m2 = m + len(req - res)
            cand = res | req
            if len(cand) <= C:
                keeps = [cand]
            elif len(req) <= C:
                keeps = [req | frozenset(c) for c in itertools.combinations(cand - req, C - len(req))]
            else:
                keeps = [frozenset(c) for c in itertools.combinations(req, C)]
            for k in keeps:
                if k not in nxt or nxt[k] > m2:
                    nxt[k] = m2
        best = nxt
    return min(best.values())


@pytest.mark.parametrize("seed,K,N,C,T", [(1, 1, 4, 2, 10), (2, 2, 5, 2, 8), (3, 2, 5, 3, 9), (4, 3, 6, 3, 7),
                                          (5, 2, 6, 4, 9), (6, 1, 5, 3, 12), (7, 2, 7, 3, 10), (8, 3, 7, 4, 8)])
def test_belady_is_optimal_on_tiny_traces(seed, K, N, C, T):
    idx = _trace(seed, 6, T, K, N, distinct=(K > 1))
    got = oracle.cache_policy(idx, N, C, "belady")["total_miss"].tolist()
    for s in range(idx.shape[0]):
        steps = [frozenset(idx[s, t].tolist()) for t in range(T)]
        assert got[s] == _least_misses(steps, C)


@pytest.mark.parametrize("K,N,C", [(2, 16, 4), (6, 64, 12), (8, 128, 32), (4, 60, 12)])
def test_belady_never_worse_and_all_bounded(K, N, C):
    idx = _trace(K + N, 4, 300, K, N)
    tot = {p: oracle.cache_policy(idx, N, C, p)["total_miss"] for p in oracle.POLICIES}
    for p in ("lru", "fifo", "lfu"):
        assert (tot["belady"] <= tot[p]).all()
    # every policy pays at least the compulsory (first-use) misses and at most K per step
    for s in range(idx.shape[0]):
        first_use = len(set(idx[s].reshape(-1).tolist()))
        for p in oracle.POLICIES:
            assert first_use <= int(tot[p][s]) <= 300 * K


# ---- accounting (App. E.2): hits + misses = requests; token hits; capacity >= N_r ---------------
@pytest.mark.parametrize("policy", list(oracle.POLICIES))
def test_accounting_identities(policy):
    idx = _trace(11, 3, 80, 4, 12, distinct=False)          # repeated ids inside a step allowed
    o = oracle.cache_policy(idx, 12, 5, policy, 1000)
    assert torch.equal(o["total_miss"], o["miss"].sum(1)) and torch.equal(o["total_uniq"], o["uniq"].sum(1))
    assert torch.equal(o["bytes"], o["total_miss"] * 1000)
    assert (o["miss"] <= o["uniq"]).all() and (o["uniq"] <= 4).all() and (o["hit_tok"] <= 4).all()
    # with distinct ids in every step, token hits are exactly the unique hits
    idx2 = _trace(12, 3, 80, 4, 12, distinct=True)
    o2 = oracle.cache_policy(idx2, 12, 5, policy)
    assert torch.equal(o2["hit_tok"], o2["uniq"] - o2["miss"])
    # a cache that holds every expert only pays first uses
    o3 = oracle.cache_policy(idx2, 12, 12, policy)
    for s in range(3):
        assert int(o3["total_miss"][s]) == len(set(idx2[s].reshape(-1).tolist()))
    # cold start: the first step misses all of its distinct experts
    assert torch.equal(o["miss"][:, 0], o["uniq"][:, 0])


def test_paper_full_cache_table_identity():
    """#uMiss = (1 - uHR) * (prompts * steps * layers * K) for the LFU / FIFO rows as well, and Belady's
    counts lie below the LRU counts of the same capacity (App. F.1)."""
    requests = 128 * 64 * 26 * 6
    lru = {4: (1.0150, 0.9746), 6: (0.8707, 0.8068)}
    with open(os.path.join(HERE, "golden", "paper_cache_policies.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    seen = 0
    for r in rows:
        if r[0] in ("LFU", "FIFO", "LRU"):
            for uhr, um in ((float(r[2]), float(r[4])), (float(r[3]), float(r[5]))):
                assert abs((1.0 - uhr) * requests / 1e6 - um) < 6e-5 * requests / 1e6 + 5e-5
            seen += 1
        else:
            c = int(r[1])
            assert int(r[2]) < lru[c][0] * 1e6 and int(r[3]) < lru[c][1] * 1e6
            seen += 1
    assert seen == 5


# ---- per-step sums over layers and percentiles ------------------------------------------------------
@pytest.mark.parametrize("L,S,T", [(3, 2, 50), (26, 4, 64), (1, 1, 7)])
def test_step_summary_matches_numpy(L, S, T):
    g = torch.Generator().manual_seed(L * S)
    miss = torch.randint(0, 7, (L, S, T), generator=g, dtype=torch.uint8)
    allm, hist, pct = oracle.step_summary(miss, L * 6 + 1)
    ref = miss.to(torch.int64).sum(0)
    assert torch.equal(allm.to(torch.int64), ref)
    assert torch.equal(hist, torch.bincount(ref.reshape(-1), minlength=L * 6 + 1))
    want = [int(np.percentile(ref.numpy().reshape(-1), p, method="inverted_cdf")) for p in (50, 95, 99)]
    assert pct.tolist() == want


def test_step_summary_sums_beyond_the_table_share_its_last_bin():
    """A histogram shorter than the largest per-step sum: every sum >= hist_len - 1 is counted in the last
    bin (numpy: clip, then bincount), the per-step sums themselves are unchanged, and a percentile that
    falls into that bin reads hist_len - 1."""
    g = torch.Generator().manual_seed(77)
    L, S, T, hist_len = 9, 3, 120, 5
    miss = torch.randint(0, 4, (L, S, T), generator=g, dtype=torch.uint8)
    allm, hist, pct = oracle.step_summary(miss, hist_len)
    ref = miss.to(torch.int64).sum(0)
    assert int(ref.max()) >= hist_len + 3                      # the overflow rule is exercised
    assert torch.equal(allm.to(torch.int64), ref)
    want = np.bincount(np.clip(ref.numpy().reshape(-1), 0, hist_len - 1), minlength=hist_len)
    assert hist.tolist() == want.tolist() and int(hist.sum()) == S * T
    cum = np.cumsum(want)
    for k, p in enumerate((50, 95, 99)):
        assert int(pct[k]) == int(np.searchsorted(100 * cum, p * S * T, side="left"))
    assert int(pct[2]) == hist_len - 1


# ---- balance: closed forms ----------------------------------------------------------------------
def test_balance_closed_forms():
    N = 8
    even = torch.arange(N, dtype=torch.int32).repeat(5).reshape(1, 20, 2)       # every expert 5 times
    load, used, ent, cv = oracle.balance(even, N)
    assert load[0].tolist() == [5] * N and int(used[0]) == N
    assert abs(float(ent[0]) - 1.0) < 1e-15 and abs(float(cv[0])) < 1e-15
    one = torch.full((1, 10, 1), 3, dtype=torch.int32)                           # one expert only
    load, used, ent, cv = oracle.balance(one, N)
    assert int(used[0]) == 1 and float(ent[0]) == 0.0
    assert abs(float(cv[0]) - math.sqrt(N - 1)) < 1e-14                         # std / mean of a one-hot load
    two = torch.tensor([[[0, 1]] * 6], dtype=torch.int32)                        # two experts, evenly
    _, used, ent, cv = oracle.balance(two, 4)
    assert int(used[0]) == 2 and abs(float(ent[0]) - 0.5) < 1e-15 and abs(float(cv[0]) - 1.0) < 1e-15


def test_balance_matches_numpy():
    idx = _trace(5, 3, 100, 4, 20)
    load, used, ent, cv = oracle.balance(idx, 20)
    for s in range(3):
        c = np.bincount(idx[s].reshape(-1).numpy(), minlength=20).astype(np.float64)
        p = c[c > 0] / c.sum()
        assert load[s].tolist() == c.astype(int).tolist() and int(used[s]) == int((c > 0).sum())
        assert abs(float(ent[s]) - float(-(p * np.log(p)).sum() / np.log(20))) < 1e-14
        assert abs(float(cv[s]) - float(c.std() / c.mean())) < 1e-14


# ---- cache-aware rerouting (App. G) -----------------------------------------------------------------
def _probs(seed, S, T, N):
    g = torch.Generator().manual_seed(seed)
    return torch.softmax(torch.randn(S, T, N, generator=g) * 2.0, -1).float().contiguous()


@pytest.mark.parametrize("K,N,C", [(2, 8, 3), (6, 64, 16), (8, 128, 32)])
def test_reroute_without_bonus_is_plain_topk_and_lru(K, N, C):
    p = _probs(K, 3, 60, N)
    o = oracle.reroute_lru(p, K, C, 1.0, False)
    want = torch.sort(torch.topk(p, K, dim=-1).indices, -1).values
    assert torch.equal(torch.sort(o["idx"].long(), -1).values, want)
    miss, tot, _ = oracle.lru_list(o["idx"], N, C, 0)
    assert torch.equal(o["miss"], miss) and torch.equal(o["total_miss"], tot)
    assert torch.allclose(o["w"], torch.gather(p.double(), -1, o["idx"].long()))


def test_reroute_with_overwhelming_bonus_locks_onto_the_cache():
    """When the bonus outweighs every score gap and C >= K, every step after the first is served from the cache:
    K cold misses and none afterwards; with renormalisation the gate weights still sum to one."""
    K, N, C = 4, 32, 6
    p = _probs(9, 2, 50, N).clamp_min(1e-6)
    p = (p / p.sum(-1, keepdim=True)).float()
    o = oracle.reroute_lru(p, K, C, 1e12, True)
    assert o["miss"][:, 0].tolist() == [K, K] and int(o["miss"][:, 1:].sum()) == 0
    assert o["total_miss"].tolist() == [K, K]
    assert torch.allclose(o["w"].sum(-1), torch.ones(2, 50, dtype=torch.float64))
    # the resident set can only ever be the first step's choice, so every later step repeats that set
    first = torch.sort(o["idx"][:, :1], -1).values
    assert torch.equal(torch.sort(o["idx"], -1).values, first.expand(-1, 50, -1))


def test_reroute_hand_worked():
    # N = 4, K = 1, C = 1, factor 3: step 0 picks 0 (0.5); step 1 scores (0.2*3, 0.5, ..) = 0.6 > 0.5 keeps 0;
    # step 2 scores (0.1*3, 0.6, ..) = 0.3 < 0.6 switches to 1 (miss); step 3 ties 0.3*... : (0.3, 0.1*3=0.3) -> lower id 0 wins
    p = torch.tensor([[[0.5, 0.3, 0.1, 0.1], [0.2, 0.5, 0.2, 0.1], [0.1, 0.6, 0.2, 0.1], [0.3, 0.1, 0.3, 0.3]]])
    o = oracle.reroute_lru(p.float(), 1, 1, 3.0, False)
    assert o["idx"][0, :, 0].tolist() == [0, 0, 1, 0]
    assert o["miss"][0].tolist() == [1, 0, 1, 1]


def test_reroute_bonus_raises_hits_on_average():
    p = _probs(21, 8, 200, 64)
    tot = [int(oracle.reroute_lru(p, 6, 8, f, False)["total_miss"].sum()) for f in (1.0, 2.0, 8.0, 64.0)]
    assert tot[0] > tot[1] > tot[2] > tot[3]
