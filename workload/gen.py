"""Counter-based seeded generator for hidden states, weights and routing traces.

Every element of every tensor is a pure function of (seed, tensor id, layer,
stream, element index): a SplitMix64-style 64-bit mixer (Steele, Lea & Flood,
"Fast splittable pseudorandom number generators", OOPSLA 2014) produces 64
bits, whose two 32-bit halves feed a Box-Muller transform evaluated in fp64.
Tensors are therefore reproducible in any chunking and on any torch device.
Integer hashing is exact everywhere; fp64 add / multiply / sqrt are correctly
rounded everywhere; only log and cos may differ by an ulp between devices, so a
run generates each tensor once and hands the same bits to every consumer.

No arithmetic of the MoE layer or of the cache statistics lives here.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import torch

from .configs import MoEConfig

TENSOR_IDS = {
    "x": 1, "w_router": 2, "w_gate": 3, "w_up": 4, "w_down": 5,
    "ws_gate": 6, "ws_up": 7, "ws_down": 8, "ws_scale": 9, "trace": 10,
}

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(v: int) -> int:
    """Reinterpret an unsigned 64-bit integer as the signed value torch.int64 holds."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix_py(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 (torch's >> is arithmetic)."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix_t(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def stream_key(seed: int, tensor_id: int, layer: int = 0, stream: int = 0) -> int:
    """64-bit key of one tensor's random stream."""
    k = _mix_py(seed + 0x51ED270B)
    k = _mix_py(k ^ (tensor_id * 0x100000001B3))
    k = _mix_py(k ^ (layer * 0xD6E8FEB86659FD93))
    k = _mix_py(k ^ (stream * 0xA0761D6478BD642F))
    return k


def raw_bits(key: int, start: int, n: int, device="cpu") -> torch.Tensor:
    """64 pseudo-random bits (as int64) for counters start .. start+n-1."""
    ctr = torch.arange(start, start + n, dtype=torch.int64, device=device)
    return _mix_t(ctr * _s64(_GOLDEN) + _s64(key))


def standard_normal(key: int, start: int, n: int, device="cpu") -> torch.Tensor:
    """n draws of N(0,1) in fp64 for counters start .. start+n-1 (Box-Muller, cosine branch)."""
    bits = raw_bits(key, start, n, device)
    hi = _lsr(bits, 32).to(torch.float64)
    lo = (bits & 0xFFFFFFFF).to(torch.float64)
    u1 = (hi + 1.0) * (1.0 / 4294967296.0)          # (0, 1]
    u2 = lo * (1.0 / 4294967296.0)                  # [0, 1)
    r = torch.sqrt(-2.0 * torch.log(u1))
    return r * torch.cos((2.0 * math.pi) * u2)


_CHUNK = 1 << 24


def gaussian(seed: int, name: str, shape, std: float = 1.0, layer: int = 0, stream: int = 0,
             dtype=torch.float32, device="cpu") -> torch.Tensor:
    """Tensor of N(0, std^2) draws, generated in fp64 and rounded once to `dtype`."""
    key = stream_key(seed, TENSOR_IDS[name], layer, stream)
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=dtype, device=device)
    for a in range(0, n, _CHUNK):
        m = min(_CHUNK, n - a)
        out[a:a + m] = (standard_normal(key, a, m, device) * std).to(dtype)
    return out.reshape(*shape)


def ar1_hidden_states(seed: int, n_seq: int, seq_len: int, hidden: int, rho: float,
                      dtype=torch.float32, device="cpu", stream: int = 0) -> torch.Tensor:
    """Hidden states [n_seq, seq_len, hidden] from a stationary AR(1) process.

    Independently for every sequence and hidden component, along the token
    axis: x_0 = eps_0 and x_t = rho * x_{t-1} + sqrt(1 - rho^2) * eps_t with
    eps ~ N(0,1), so every x_t is N(0,1) and adjacent tokens correlate by rho.
    The recurrence runs in fp64; the result is rounded once to `dtype`.
    """
    key = stream_key(seed, TENSOR_IDS["x"], 0, stream)
    out = torch.empty(n_seq, seq_len, hidden, dtype=dtype, device=device)
    c = math.sqrt(1.0 - rho * rho)
    per_seq = seq_len * hidden
    group = max(1, min(n_seq, (1 << 27) // max(per_seq, 1)))   # sequences advanced together
    for s0 in range(0, n_seq, group):
        g = min(group, n_seq - s0)
        eps = torch.empty(g, seq_len, hidden, dtype=torch.float64, device=device)
        flat = eps.view(-1)
        for a in range(0, g * per_seq, _CHUNK):
            m = min(_CHUNK, g * per_seq - a)
            flat[a:a + m] = standard_normal(key, s0 * per_seq + a, m, device)
        if rho != 0.0:
            prev = eps[:, 0].clone()
            for t in range(1, seq_len):
                prev = rho * prev + c * eps[:, t]
                eps[:, t] = prev
        out[s0:s0 + g] = eps.to(dtype)
    return out


def layer_weights(cfg: MoEConfig, layer: int, device="cpu") -> Dict[str, Optional[torch.Tensor]]:
    """All weight tensors of one MoE layer, N(0, weight_std^2).

    Matrices are [out_features, in_features] row-major.  The router matrix and
    the shared-expert scale vector are always fp32; expert matrices have the
    configuration's dtype.
    """
    wdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    H, N, I, Is = cfg.hidden, cfg.n_experts, cfg.inter, cfg.shared_inter
    g = lambda name, shape, dt: gaussian(cfg.seed, name, shape, cfg.weight_std, layer, 0, dt, device)
    w = {
        "w_router": g("w_router", (N, H), torch.float32),
        "w_gate": g("w_gate", (N, I, H), wdt),
        "w_up": g("w_up", (N, I, H), wdt),
        "w_down": g("w_down", (N, H, I), wdt),
        "ws_gate": None, "ws_up": None, "ws_down": None, "ws_scale": None,
    }
    if Is > 0:
        w["ws_gate"] = g("ws_gate", (Is, H), wdt)
        w["ws_up"] = g("ws_up", (Is, H), wdt)
        w["ws_down"] = g("ws_down", (H, Is), wdt)
        if cfg.shared_gate:
            w["ws_scale"] = g("ws_scale", (H,), torch.float32)
    return w


def hidden_states(cfg: MoEConfig, rho: Optional[float] = None, device="cpu") -> torch.Tensor:
    """The configuration's input [n_seq, seq_len, hidden] in its dtype."""
    rho = cfg.rhos[0] if rho is None else rho
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    stream = int(round(rho * 1000))
    return ar1_hidden_states(cfg.seed, cfg.n_seq, cfg.seq_len, cfg.hidden, rho, dt, device, stream)


def random_trace(seed: int, n_seq: int, n_steps: int, top_k: int, n_experts: int,
                 stickiness: float = 0.0, distinct: bool = True, stream: int = 0) -> torch.Tensor:
    """Synthetic routing trace int32 [n_seq, n_steps, top_k] of expert ids.

    Each step keeps every expert of the previous step with probability
    `stickiness` and redraws the others uniformly; with `distinct` the K ids of
    a step are pairwise different (as a Top-K produces), otherwise repeats may
    occur (as a batched step's flattened request list would have).
    Small helper for tests of the trace statistics; host-side Python loops.
    """
    key = stream_key(seed, TENSOR_IDS["trace"], 0, stream)
    out = torch.empty(n_seq, n_steps, top_k, dtype=torch.int32)
    ctr = 0

    def draw() -> int:
        nonlocal ctr
        v = _mix_py((ctr * _GOLDEN + key) & _M64)
        ctr += 1
        return v

    for s in range(n_seq):
        prev: list = []
        for t in range(n_steps):
            cur: list = []
            for e in prev:
                if (draw() >> 11) * (1.0 / (1 << 53)) < stickiness and (not distinct or e not in cur):
                    cur.append(e)
            while len(cur) < top_k:
                e = draw() % n_experts
                if distinct and e in cur:
                    continue
                cur.append(e)
            out[s, t] = torch.tensor(cur[:top_k], dtype=torch.int32)
            prev = cur[:top_k]
    return out
