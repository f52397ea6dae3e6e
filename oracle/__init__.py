"""Python face of the CPU oracle (oracle/remoe_oracle.c, loaded through ctypes).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
benchmark's CPU-baseline leg.  It never imports the HIP package and the HIP
package never imports it.  Arguments are CPU torch tensors (torch is used as a
typed buffer only, which gives bf16 storage); results are fp64 / integer CPU
tensors.  All arithmetic happens in the C file.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence

import torch

from .build import ensure_built

_lib = None

_c_i64 = ctypes.c_int64
_c_int = ctypes.c_int
_c_ptr = ctypes.c_void_p


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(ensure_built())
        _lib.oracle_route.restype = _c_int
        _lib.oracle_route.argtypes = [_c_ptr, _c_int, _c_i64, _c_int, _c_ptr, _c_int, _c_int, _c_int,
                                      _c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_ptr]
        _lib.oracle_experts_sparse.restype = _c_int
        _lib.oracle_experts_sparse.argtypes = [_c_ptr, _c_int, _c_int, _c_int, _c_int, _c_int,
                                               _c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_ptr,
                                               _c_int, _c_ptr, _c_ptr, _c_ptr, _c_ptr,
                                               _c_ptr, _c_i64, _c_ptr]
        _lib.oracle_experts_dense_masked.restype = _c_int
        _lib.oracle_experts_dense_masked.argtypes = [_c_ptr, _c_int, _c_i64, _c_int, _c_int, _c_int, _c_int,
                                                     _c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_ptr,
                                                     _c_int, _c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_ptr]
        _lib.oracle_trace_reuse.restype = _c_int
        _lib.oracle_trace_reuse.argtypes = [_c_ptr, _c_i64, _c_i64, _c_int, _c_int, _c_ptr, _c_ptr]
        _lib.oracle_lru_list.restype = _c_int
        _lib.oracle_lru_list.argtypes = [_c_ptr, _c_i64, _c_i64, _c_int, _c_int, _c_int, ctypes.c_uint64,
                                         _c_ptr, _c_ptr, _c_ptr]
        _lib.oracle_cache_policy.restype = _c_int
        _lib.oracle_cache_policy.argtypes = [_c_ptr, _c_i64, _c_i64, _c_int, _c_int, _c_int, _c_int, ctypes.c_uint64,
                                             _c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_ptr]
        _lib.oracle_step_summary.restype = _c_int
        _lib.oracle_step_summary.argtypes = [_c_ptr, _c_i64, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_i64, _c_ptr]
        _lib.oracle_balance.restype = _c_int
        _lib.oracle_balance.argtypes = [_c_ptr, _c_i64, _c_i64, _c_int, _c_int, _c_ptr, _c_ptr, _c_ptr, _c_ptr]
        _lib.oracle_reroute_lru.restype = _c_int
        _lib.oracle_reroute_lru.argtypes = [_c_ptr, _c_i64, _c_i64, _c_int, _c_int, _c_int, ctypes.c_float, _c_int,
                                            _c_ptr, _c_ptr, _c_ptr, _c_ptr]
        _lib.oracle_remoe_losses.restype = _c_int
        _lib.oracle_remoe_losses.argtypes = [_c_ptr, _c_ptr, _c_ptr, _c_i64, _c_i64, _c_int, _c_int, _c_ptr, _c_int,
                                             _c_int, _c_ptr]
        _lib.oracle_remoe_loss_grad.restype = _c_int
        _lib.oracle_remoe_loss_grad.argtypes = [_c_ptr, _c_ptr, _c_ptr, _c_i64, _c_i64, _c_int, _c_int, _c_ptr, _c_int,
                                                _c_int, _c_ptr, _c_ptr]
        _lib.oracle_gate_grad.restype = _c_int
        _lib.oracle_gate_grad.argtypes = [_c_ptr, _c_ptr, _c_i64, _c_int, _c_int, _c_ptr, _c_i64, _c_ptr]
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise TypeError(f"oracle: unsupported dtype {t.dtype}")


def _chk(t: Optional[torch.Tensor], dtype=None) -> Optional[torch.Tensor]:
    if t is None:
        return None
    if t.device.type != "cpu":
        raise ValueError("oracle takes CPU tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"oracle: expected {dtype}, got {t.dtype}")
    return t.contiguous()


def _p(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def route(x: torch.Tensor, w_router: torch.Tensor, top_k: int, renorm: bool,
          want_probs: bool = False, want_logits: bool = False):
    """Router of Sec. 3.1 for tokens x [T,H]: returns dict(idx, w, margin[, probs][, logits])."""
    x = _chk(x)
    w_router = _chk(w_router, torch.float32)
    T, H = x.shape
    N = w_router.shape[0]
    assert w_router.shape[1] == H
    idx = torch.empty(T, top_k, dtype=torch.int32)
    w = torch.empty(T, top_k, dtype=torch.float64)
    margin = torch.empty(T, dtype=torch.float64)
    probs = torch.empty(T, N, dtype=torch.float64) if want_probs else None
    logits = torch.empty(T, N, dtype=torch.float64) if want_logits else None
    rc = lib().oracle_route(_p(x), _dtype_code(x), T, H, _p(w_router), N, top_k, int(bool(renorm)),
                            _p(idx), _p(w), _p(margin), _p(probs), _p(logits))
    if rc != 0:
        raise RuntimeError(f"oracle_route failed ({rc})")
    out = {"idx": idx, "w": w, "margin": margin}
    if want_probs:
        out["probs"] = probs
    if want_logits:
        out["logits"] = logits
    return out


def _expert_args(x, weights):
    wg = _chk(weights["w_gate"]); wu = _chk(weights["w_up"]); wd = _chk(weights["w_down"])
    for m in (wg, wu, wd):
        if m.dtype != x.dtype:
            raise TypeError("oracle: x and expert weights must share a dtype")
    N, I, H = wg.shape
    assert wu.shape == (N, I, H) and wd.shape == (N, H, I) and x.shape[1] == H
    sg = _chk(weights.get("ws_gate")); su = _chk(weights.get("ws_up")); sd = _chk(weights.get("ws_down"))
    sc = _chk(weights.get("ws_scale"), torch.float32) if weights.get("ws_scale") is not None else None
    Is = 0 if sg is None else sg.shape[0]
    if Is:
        assert sg.shape == (Is, H) and su.shape == (Is, H) and sd.shape == (H, Is)
        assert sg.dtype == x.dtype and su.dtype == x.dtype and sd.dtype == x.dtype
    keep = (wg, wu, wd, sg, su, sd, sc)
    return N, I, H, Is, keep


def experts_sparse(x: torch.Tensor, idx: torch.Tensor, w: torch.Tensor, weights: dict,
                   tokens: Optional[Sequence[int]] = None) -> torch.Tensor:
    """y[t] = sum_j w[t,j] * expert_{idx[t,j]}(x[t]) + shared(x[t]) for the listed tokens (fp64)."""
    x = _chk(x)
    idx = _chk(idx, torch.int32)
    w = _chk(w.to(torch.float64))
    N, I, H, Is, (wg, wu, wd, sg, su, sd, sc) = _expert_args(x, weights)
    K = idx.shape[1]
    tok = None
    n_sel = x.shape[0]
    if tokens is not None:
        tok = torch.as_tensor(list(tokens), dtype=torch.int64).contiguous()
        n_sel = tok.numel()
    y = torch.empty(n_sel, H, dtype=torch.float64)
    rc = lib().oracle_experts_sparse(_p(x), _dtype_code(x), H, N, I, K, _p(idx), _p(w),
                                     _p(wg), _p(wu), _p(wd), Is, _p(sg), _p(su), _p(sd), _p(sc),
                                     _p(tok), n_sel, _p(y))
    if rc != 0:
        raise RuntimeError(f"oracle_experts_sparse failed ({rc})")
    return y


def experts_dense_masked(x: torch.Tensor, idx: torch.Tensor, w: torch.Tensor, weights: dict) -> torch.Tensor:
    """Dense check form: all N experts evaluated, combined with masked gate weights (fp64)."""
    x = _chk(x)
    idx = _chk(idx, torch.int32)
    w = _chk(w.to(torch.float64))
    N, I, H, Is, (wg, wu, wd, sg, su, sd, sc) = _expert_args(x, weights)
    T, K = idx.shape
    y = torch.empty(T, H, dtype=torch.float64)
    rc = lib().oracle_experts_dense_masked(_p(x), _dtype_code(x), T, H, N, I, K, _p(idx), _p(w),
                                           _p(wg), _p(wu), _p(wd), Is, _p(sg), _p(su), _p(sd), _p(sc), _p(y))
    if rc != 0:
        raise RuntimeError(f"oracle_experts_dense_masked failed ({rc})")
    return y


def forward(x: torch.Tensor, weights: dict, top_k: int, renorm: bool,
            tokens: Optional[Sequence[int]] = None):
    """Whole layer: route every token, evaluate the experts for `tokens` (all if None)."""
    r = route(x, weights["w_router"], top_k, renorm)
    r["y"] = experts_sparse(x, r["idx"], r["w"], weights, tokens)
    return r


def trace_reuse(idx: torch.Tensor, n_experts: int):
    """Adjacent-step overlap |E_t ∩ E_{t-1}| per trace: idx int32 [S,T,K] -> (ov uint8 [S,T], sum uint64 [S])."""
    idx = _chk(idx, torch.int32)
    S, T, K = idx.shape
    ov = torch.empty(S, T, dtype=torch.uint8)
    tot = torch.empty(S, dtype=torch.int64)
    rc = lib().oracle_trace_reuse(_p(idx), S, T, K, n_experts, _p(ov), _p(tot))
    if rc != 0:
        raise RuntimeError(f"oracle_trace_reuse failed ({rc})")
    return ov, tot


def lru_list(idx: torch.Tensor, n_experts: int, capacity: int, expert_bytes: int = 0):
    """Cold-start LRU misses per trace: (miss uint8 [S,T], total int64 [S], bytes int64 [S])."""
    idx = _chk(idx, torch.int32)
    S, T, K = idx.shape
    miss = torch.empty(S, T, dtype=torch.uint8)
    tot = torch.empty(S, dtype=torch.int64)
    nbytes = torch.empty(S, dtype=torch.int64)
    rc = lib().oracle_lru_list(_p(idx), S, T, K, n_experts, capacity, expert_bytes,
                               _p(miss), _p(tot), _p(nbytes))
    if rc != 0:
        raise RuntimeError(f"oracle_lru_list failed ({rc})")
    return miss, tot, nbytes


POLICIES = {"lru": 0, "fifo": 1, "lfu": 2, "belady": 3}


def cache_policy(idx: torch.Tensor, n_experts: int, capacity: int, policy: str, expert_bytes: int = 0):
    """Expert cache of one replacement policy per trace (App. E.2; Belady: App. F.1).  idx [S, T, K] int32.
    Returns dict: miss, uniq, hit_tok uint8 [S, T]; total_miss, total_uniq, bytes int64 [S]."""
    idx = _chk(idx, torch.int32)
    S, T, K = idx.shape
    out = {k: torch.zeros(S, T, dtype=torch.uint8) for k in ("miss", "uniq", "hit_tok")}
    out.update({k: torch.zeros(S, dtype=torch.int64) for k in ("total_miss", "total_uniq", "bytes")})
    rc = lib().oracle_cache_policy(_p(idx), S, T, K, n_experts, capacity, POLICIES[policy], expert_bytes,
                                   _p(out["miss"]), _p(out["uniq"]), _p(out["hit_tok"]), _p(out["total_miss"]),
                                   _p(out["total_uniq"]), _p(out["bytes"]))
    if rc != 0:
        raise ValueError(f"oracle_cache_policy failed ({rc})")
    return out


def step_summary(miss: torch.Tensor, hist_len: int):
    """Per-step sums over layers and their P50/P95/P99 (App. E.2).  miss uint8 [L, S, T].
    Returns (all uint16-valued int32 [S, T], hist int64 [hist_len], pct int32 [3])."""
    miss = _chk(miss, torch.uint8)
    L, S, T = miss.shape
    allm = torch.zeros(S, T, dtype=torch.int16)
    hist = torch.zeros(hist_len, dtype=torch.int64)
    pct = torch.zeros(3, dtype=torch.int32)
    rc = lib().oracle_step_summary(_p(miss), L, S, T, _p(allm), _p(hist), hist_len, _p(pct))
    if rc != 0:
        raise ValueError(f"oracle_step_summary failed ({rc})")
    return allm.to(torch.int32) & 0xFFFF, hist, pct


def balance(idx: torch.Tensor, n_experts: int):
    """Expert-load balance per trace: load int64 [S, N], used int32 [S], entropy, cv fp64 [S]."""
    idx = _chk(idx, torch.int32)
    S, T, K = idx.shape
    load = torch.zeros(S, n_experts, dtype=torch.int32)
    used = torch.zeros(S, dtype=torch.int32)
    ent = torch.zeros(S, dtype=torch.float64)
    cv = torch.zeros(S, dtype=torch.float64)
    rc = lib().oracle_balance(_p(idx), S, T, K, n_experts, _p(load), _p(used), _p(ent), _p(cv))
    if rc != 0:
        raise ValueError(f"oracle_balance failed ({rc})")
    return load.to(torch.int64), used, ent, cv


def reroute_lru(probs: torch.Tensor, top_k: int, capacity: int, factor: float, renorm: bool):
    """Cache-aware rerouting (App. G): probs fp32 [S, T, N]; factor = exp(beta) as an fp32 value.
    Returns dict idx int32 [S,T,K], w fp64 [S,T,K], miss uint8 [S,T], total_miss int64 [S]."""
    probs = _chk(probs, torch.float32)
    S, T, N = probs.shape
    out = {"idx": torch.zeros(S, T, top_k, dtype=torch.int32), "w": torch.zeros(S, T, top_k, dtype=torch.float64),
           "miss": torch.zeros(S, T, dtype=torch.uint8), "total_miss": torch.zeros(S, dtype=torch.int64)}
    rc = lib().oracle_reroute_lru(_p(probs), S, T, N, top_k, capacity, float(factor), int(renorm), _p(out["idx"]),
                                  _p(out["w"]), _p(out["miss"]), _p(out["total_miss"]))
    if rc != 0:
        raise ValueError(f"oracle_reroute_lru failed ({rc})")
    return out


LOSS_NAMES = ("rho", "reuse", "trust", "smooth", "lag", "ws")


def remoe_losses(probs: torch.Tensor, probs_ref: torch.Tensor, idx: torch.Tensor, lags: Sequence[int], window: int):
    """Forward values of ReMoE's router regularisers (Eq. 2-12) per sequence: fp64 [S, 6] in the order of
    LOSS_NAMES.  probs, probs_ref fp32 [S, T, N]; idx int32 [S, T, K]."""
    probs, probs_ref, idx = _chk(probs, torch.float32), _chk(probs_ref, torch.float32), _chk(idx, torch.int32)
    S, T, N = probs.shape
    lg = torch.tensor(list(lags), dtype=torch.int32)
    out = torch.zeros(S, 6, dtype=torch.float64)
    rc = lib().oracle_remoe_losses(_p(probs), _p(probs_ref), _p(idx), S, T, N, idx.shape[2], _p(lg), len(lags), window,
                                   _p(out))
    if rc != 0:
        raise ValueError(f"oracle_remoe_losses failed ({rc})")
    return out


def remoe_loss_grad(probs: torch.Tensor, probs_ref: torch.Tensor, idx: torch.Tensor, lags: Sequence[int], window: int,
                    coef: Sequence[float]):
    """d(sum_i coef[i] L_i)/d(logits) per sequence, L_i in the order Reuse, Trust, Smooth, Lag, WS
    (Eq. 3, 6-12 through the softmax): fp64 [S, T, N]."""
    probs, probs_ref, idx = _chk(probs, torch.float32), _chk(probs_ref, torch.float32), _chk(idx, torch.int32)
    S, T, N = probs.shape
    lg = torch.tensor(list(lags), dtype=torch.int32)
    cf = torch.tensor(list(coef), dtype=torch.float64)
    assert cf.numel() == 5
    out = torch.zeros(S, T, N, dtype=torch.float64)
    rc = lib().oracle_remoe_loss_grad(_p(probs), _p(probs_ref), _p(idx), S, T, N, idx.shape[2], _p(lg), len(lags), window,
                                      _p(cf), _p(out))
    if rc != 0:
        raise ValueError(f"oracle_remoe_loss_grad failed ({rc})")
    return out


def gate_grad(dz: torch.Tensor, x: torch.Tensor, pick: Optional[torch.Tensor] = None):
    """dL/dW_r = dz^T x (router without bias, Sec. 3.1): fp64 [N, H], or the picked (e, h) entries only."""
    dz, x = _chk(dz, torch.float32), _chk(x.float(), torch.float32)
    T, N = dz.shape
    H = x.shape[1]
    assert x.shape[0] == T
    if pick is not None:
        pick = _chk(pick, torch.int32)
        out = torch.zeros(pick.shape[0], dtype=torch.float64)
        rc = lib().oracle_gate_grad(_p(dz), _p(x), T, N, H, _p(pick), pick.shape[0], _p(out))
    else:
        out = torch.zeros(N, H, dtype=torch.float64)
        rc = lib().oracle_gate_grad(_p(dz), _p(x), T, N, H, None, 0, _p(out))
    if rc != 0:
        raise ValueError(f"oracle_gate_grad failed ({rc})")
    return out
