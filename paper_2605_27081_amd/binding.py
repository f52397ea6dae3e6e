"""ctypes binding of include/remoe.h: same names, argument marshalling only.

torch supplies device memory and the current HIP stream; nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libremoe_hip.so")
_lib: Optional[ctypes.CDLL] = None

REMOE_F32, REMOE_BF16 = 0, 1
REMOE_DECODE_CHAINED, REMOE_DECODE_PIPELINED = 0, 1
REMOE_CACHE_LRU, REMOE_CACHE_FIFO, REMOE_CACHE_LFU, REMOE_CACHE_BELADY = 0, 1, 2, 3


class RemoeError(RuntimeError):
    """A C-ABI call returned a negative status."""


class LayerDesc(ctypes.Structure):
    """Mirror of remoe_layer_desc."""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("hidden", "n_experts", "inter", "top_k", "renorm", "shared_inter", "shared_gate", "dtype")]

    @classmethod
    def from_config(cls, cfg) -> "LayerDesc":
        return cls(cfg.hidden, cfg.n_experts, cfg.inter, cfg.top_k, int(cfg.renorm), cfg.shared_inter,
                   int(cfg.shared_gate), REMOE_F32 if cfg.dtype == "f32" else REMOE_BF16)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == REMOE_F32 else torch.bfloat16


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libremoe_hip.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RemoeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2605_27081_amd.build` "
                         "(hipcc, gfx950); there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    P, I64, I32, U64, SZ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_size_t
    D = ctypes.POINTER(LayerDesc)
    lib.remoe_version.restype = I32
    lib.remoe_version.argtypes = []
    lib.remoe_last_error.restype = ctypes.c_char_p
    lib.remoe_last_error.argtypes = []
    lib.remoe_workspace_bytes.restype = SZ
    lib.remoe_workspace_bytes.argtypes = [D, I64]
    lib.moe_route.restype = ctypes.c_int
    lib.moe_route.argtypes = [D, P, I64, P, P, P, P, P, P]
    lib.moe_forward.restype = ctypes.c_int
    lib.moe_forward.argtypes = [D, P, I64, P, P, P, P, P, P, P, P, P, P, P, P, SZ, P]
    lib.trace_reuse.restype = ctypes.c_int
    lib.trace_reuse.argtypes = [P, I64, I64, I32, I32, P, P, P]
    lib.lru_simulate.restype = ctypes.c_int
    lib.lru_simulate.argtypes = [P, I64, I64, I32, I32, I32, U64, I64, P, P, P, P, P]
    lib.remoe_decode_workspace_bytes.restype = SZ
    lib.remoe_decode_workspace_bytes.argtypes = [D]
    lib.moe_decode.restype = ctypes.c_int
    lib.moe_decode.argtypes = [D, I32, P, P, I64, I64, I64, P, P, P, I32, ctypes.POINTER(I32), U64,
                               P, P, P, P, P, P, P, SZ, U64, I32, P]
    lib.remoe_decode_static_bytes.restype = SZ
    lib.remoe_decode_static_bytes.argtypes = []
    lib.moe_decode_static.restype = ctypes.c_int
    lib.moe_decode_static.argtypes = [D, I32, P, P, I64, I64, I64, P, P, P, I32, ctypes.POINTER(I32), U64,
                                      P, P, P, P, P, P, P, U64, I32, P]
    lib.remoe_copy_probe.restype = ctypes.c_int
    lib.remoe_copy_probe.argtypes = [P, P, SZ, P]
    lib.remoe_profile_enable.restype = ctypes.c_int
    lib.remoe_profile_enable.argtypes = [I32]
    lib.remoe_profile_read.restype = ctypes.c_int
    lib.remoe_profile_read.argtypes = [I32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(I64), I32]
    lib.remoe_cache_workspace_bytes.restype = SZ
    lib.remoe_cache_workspace_bytes.argtypes = [I64, I64, I32, I32]
    lib.cache_simulate.restype = ctypes.c_int
    lib.cache_simulate.argtypes = [P, I64, I64, I32, I32, I32, I32, U64, P, P, P, P, P, P, P, SZ, P]
    lib.step_miss_summary.restype = ctypes.c_int
    lib.step_miss_summary.argtypes = [P, I64, I64, I64, P, P, I64, P, P]
    lib.routing_balance.restype = ctypes.c_int
    lib.routing_balance.argtypes = [P, I64, I64, I32, I32, P, P, P, P, P]
    lib.reroute_lru.restype = ctypes.c_int
    lib.reroute_lru.argtypes = [P, I64, I64, I32, I32, I32, ctypes.c_float, I32, P, P, P, P, P]
    lib.remoe_loss_workspace_bytes.restype = SZ
    lib.remoe_loss_workspace_bytes.argtypes = [I64]
    lib.remoe_loss_forward.restype = ctypes.c_int
    lib.remoe_loss_forward.argtypes = [P, P, P, I64, I64, I32, I32, ctypes.POINTER(I32), I32, I32, P, P, SZ, P]
    lib.remoe_loss_backward_workspace_bytes.restype = SZ
    lib.remoe_loss_backward_workspace_bytes.argtypes = [I64, I64, I32, I32]
    lib.remoe_loss_backward.restype = ctypes.c_int
    lib.remoe_loss_backward.argtypes = [P, P, P, I64, I64, I32, I32, ctypes.POINTER(I32), I32, I32,
                                        ctypes.POINTER(ctypes.c_double), P, P, P, SZ, P]
    lib.remoe_gate_grad_workspace_bytes.restype = SZ
    lib.remoe_gate_grad_workspace_bytes.argtypes = [I64, I32, I32]
    lib.remoe_gate_grad.restype = ctypes.c_int
    lib.remoe_gate_grad.argtypes = [P, P, I32, I64, I32, I32, P, P, SZ, P]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise RemoeError(f"remoe status {status}: {remoe_last_error()}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise RemoeError("the library takes device tensors")
    if not t.is_contiguous():
        raise RemoeError("tensors must be contiguous")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def remoe_version() -> int:
    return int(load_library().remoe_version())


def remoe_last_error() -> str:
    return load_library().remoe_last_error().decode()


PROF_KINDS = ("route", "permute", "gate_up", "down", "shared_gate_up", "shared_down", "combine",
              "trace_reuse", "lru", "decode", "cache")


def remoe_profile_enable(on: bool) -> None:
    _check(load_library().remoe_profile_enable(int(bool(on))))


def remoe_profile_read(kind: int, reset: bool = True):
    """(total milliseconds, launches) of one kernel kind; synchronise the device first."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(load_library().remoe_profile_read(kind, ctypes.byref(ms), ctypes.byref(n), int(bool(reset))))
    return ms.value, n.value


def remoe_workspace_bytes(desc: LayerDesc, n_tokens: int) -> int:
    n = int(load_library().remoe_workspace_bytes(ctypes.byref(desc), n_tokens))
    if n == 0 and n_tokens != 0:
        raise RemoeError(f"remoe_workspace_bytes: {remoe_last_error()}")
    return n


def moe_route(desc: LayerDesc, x: torch.Tensor, w_router: torch.Tensor, out_idx: torch.Tensor,
              out_w: torch.Tensor, out_margin: Optional[torch.Tensor] = None,
              out_probs: Optional[torch.Tensor] = None) -> None:
    n_tokens = x.shape[0]
    _check(load_library().moe_route(ctypes.byref(desc), _ptr(x), n_tokens, _ptr(w_router), _ptr(out_idx),
                                    _ptr(out_w), _ptr(out_margin), _ptr(out_probs), _stream()))


def moe_forward(desc: LayerDesc, x: torch.Tensor, w_router, w_gate, w_up, w_down, ws_gate, ws_up, ws_down,
                ws_scale, y: torch.Tensor, out_idx: torch.Tensor, out_w: torch.Tensor,
                workspace: torch.Tensor) -> None:
    n_tokens = x.shape[0]
    _check(load_library().moe_forward(ctypes.byref(desc), _ptr(x), n_tokens, _ptr(w_router), _ptr(w_gate),
                                      _ptr(w_up), _ptr(w_down), _ptr(ws_gate), _ptr(ws_up), _ptr(ws_down),
                                      _ptr(ws_scale), _ptr(y), _ptr(out_idx), _ptr(out_w), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream()))


def trace_reuse(idx: torch.Tensor, n_experts: int, out_overlap: torch.Tensor, out_sum: torch.Tensor) -> None:
    n_seq, n_steps, top_k = idx.shape
    _check(load_library().trace_reuse(_ptr(idx), n_seq, n_steps, top_k, n_experts, _ptr(out_overlap),
                                      _ptr(out_sum), _stream()))


def lru_simulate(idx: torch.Tensor, n_experts: int, capacity: int, expert_bytes: int, step0: int,
                 state: Optional[torch.Tensor], out_miss: torch.Tensor, out_total_miss: torch.Tensor,
                 out_bytes: torch.Tensor) -> None:
    n_seq, n_steps, top_k = idx.shape
    _check(load_library().lru_simulate(_ptr(idx), n_seq, n_steps, top_k, n_experts, capacity, expert_bytes,
                                       step0, _ptr(state), _ptr(out_miss), _ptr(out_total_miss),
                                       _ptr(out_bytes), _stream()))


def remoe_copy_probe(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain copy of src into dst (same byte size): the yardstick for hardware byte counters."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise RemoeError("remoe_copy_probe: dst and src differ in size")
    _check(load_library().remoe_copy_probe(_ptr(dst), _ptr(src), nbytes, _stream()))


def remoe_decode_workspace_bytes(desc: LayerDesc) -> int:
    n = int(load_library().remoe_decode_workspace_bytes(ctypes.byref(desc)))
    if n == 0:
        raise RemoeError(f"remoe_decode_workspace_bytes: {remoe_last_error()}")
    return n


def moe_decode(desc: LayerDesc, layer_weights: torch.Tensor, x: torch.Tensor, step0: int, n_steps: int,
               y: torch.Tensor, out_idx: torch.Tensor, out_w: torch.Tensor, capacities, expert_bytes: int,
               lru_state: torch.Tensor, out_overlap: torch.Tensor, out_miss: Optional[torch.Tensor],
               sum_overlap: torch.Tensor, total_miss: Optional[torch.Tensor],
               bytes_fetched: Optional[torch.Tensor], workspace: torch.Tensor, spin_limit_us: int = 0,
               layer_order: int = 1) -> None:
    """layer_weights: int64 device tensor [n_layers, 4] of data_ptr()s (w_router, w_gate, w_up, w_down).
    layer_order: REMOE_DECODE_CHAINED (0) or REMOE_DECODE_PIPELINED (1)."""
    n_layers = layer_weights.shape[0]
    steps_total = x.shape[0]
    caps = (ctypes.c_int32 * max(len(capacities), 1))(*capacities)
    _check(load_library().moe_decode(ctypes.byref(desc), n_layers, _ptr(layer_weights), _ptr(x), steps_total,
                                     step0, n_steps, _ptr(y), _ptr(out_idx), _ptr(out_w), len(capacities), caps,
                                     expert_bytes, _ptr(lru_state), _ptr(out_overlap), _ptr(out_miss),
                                     _ptr(sum_overlap), _ptr(total_miss), _ptr(bytes_fetched), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), spin_limit_us, layer_order,
                                     _stream()))


def remoe_decode_static_bytes() -> int:
    return int(load_library().remoe_decode_static_bytes())


def moe_decode_static(desc: LayerDesc, layer_weights: torch.Tensor, x: torch.Tensor, step0: int, n_steps: int,
                      y: torch.Tensor, out_idx: torch.Tensor, out_w: torch.Tensor, capacities, expert_bytes: int,
                      lru_state: torch.Tensor, out_overlap: torch.Tensor, out_miss: Optional[torch.Tensor],
                      sum_overlap: torch.Tensor, total_miss: Optional[torch.Tensor],
                      bytes_fetched: Optional[torch.Tensor], out_abort: torch.Tensor, spin_limit_us: int = 0,
                      layer_order: int = 0) -> None:
    """moe_decode without a workspace (scratch in a static device array); out_abort: one int32 on the device."""
    n_layers = layer_weights.shape[0]
    steps_total = x.shape[0]
    caps = (ctypes.c_int32 * max(len(capacities), 1))(*capacities)
    _check(load_library().moe_decode_static(ctypes.byref(desc), n_layers, _ptr(layer_weights), _ptr(x), steps_total,
                                            step0, n_steps, _ptr(y), _ptr(out_idx), _ptr(out_w), len(capacities),
                                            caps, expert_bytes, _ptr(lru_state), _ptr(out_overlap), _ptr(out_miss),
                                            _ptr(sum_overlap), _ptr(total_miss), _ptr(bytes_fetched),
                                            _ptr(out_abort), spin_limit_us, layer_order, _stream()))


def remoe_cache_workspace_bytes(n_seq: int, n_steps: int, top_k: int, policy: int) -> int:
    return int(load_library().remoe_cache_workspace_bytes(n_seq, n_steps, top_k, policy))


def cache_simulate(idx: torch.Tensor, n_experts: int, capacity: int, policy: int, expert_bytes: int,
                   out_miss: torch.Tensor, out_uniq: torch.Tensor, out_hit_tok: torch.Tensor,
                   out_total_miss: torch.Tensor, out_total_uniq: torch.Tensor, out_bytes: torch.Tensor,
                   workspace: Optional[torch.Tensor] = None) -> None:
    n_seq, n_steps, top_k = idx.shape
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().cache_simulate(_ptr(idx), n_seq, n_steps, top_k, n_experts, capacity, policy, expert_bytes,
                                         _ptr(out_miss), _ptr(out_uniq), _ptr(out_hit_tok), _ptr(out_total_miss),
                                         _ptr(out_total_uniq), _ptr(out_bytes), _ptr(workspace), ws_bytes, _stream()))


def step_miss_summary(miss: torch.Tensor, out_all: torch.Tensor, out_hist: torch.Tensor, out_pct: torch.Tensor) -> None:
    """miss uint8 [L, S, T]; out_all int16 [S, T] (holds uint16); out_hist int64 [hist_len]; out_pct int32 [3]."""
    n_layers, n_seq, n_steps = miss.shape
    _check(load_library().step_miss_summary(_ptr(miss), n_layers, n_seq, n_steps, _ptr(out_all), _ptr(out_hist),
                                            out_hist.numel(), _ptr(out_pct), _stream()))


def routing_balance(idx: torch.Tensor, n_experts: int, out_load: torch.Tensor, out_used: torch.Tensor,
                    out_entropy: torch.Tensor, out_cv: torch.Tensor) -> None:
    n_seq, n_steps, top_k = idx.shape
    _check(load_library().routing_balance(_ptr(idx), n_seq, n_steps, top_k, n_experts, _ptr(out_load), _ptr(out_used),
                                          _ptr(out_entropy), _ptr(out_cv), _stream()))


def reroute_lru(probs: torch.Tensor, top_k: int, capacity: int, factor: float, renorm: bool, out_idx: torch.Tensor,
                out_w: torch.Tensor, out_miss: torch.Tensor, out_total_miss: torch.Tensor) -> None:
    """probs fp32 [S, T, N]; factor = exp(beta)."""
    n_seq, n_steps, n_experts = probs.shape
    _check(load_library().reroute_lru(_ptr(probs), n_seq, n_steps, n_experts, top_k, capacity, factor, int(renorm),
                                      _ptr(out_idx), _ptr(out_w), _ptr(out_miss), _ptr(out_total_miss), _stream()))


def remoe_loss_workspace_bytes(n_seq: int) -> int:
    return int(load_library().remoe_loss_workspace_bytes(n_seq))


def remoe_loss_forward(probs: torch.Tensor, probs_ref: torch.Tensor, idx: torch.Tensor, lags, window: int,
                       out: torch.Tensor, workspace: torch.Tensor) -> None:
    """probs, probs_ref fp32 [S, T, N]; idx int32 [S, T, K]; out fp64 [S, 6] (rho, reuse, trust, smooth, lag, ws)."""
    n_seq, n_steps, n_experts = probs.shape
    lg = (ctypes.c_int32 * max(len(lags), 1))(*lags)
    _check(load_library().remoe_loss_forward(_ptr(probs), _ptr(probs_ref), _ptr(idx), n_seq, n_steps, n_experts,
                                             idx.shape[2], lg, len(lags), window, _ptr(out), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream()))


def remoe_loss_backward_workspace_bytes(n_seq: int, n_steps: int, n_experts: int, window: int) -> int:
    return int(load_library().remoe_loss_backward_workspace_bytes(n_seq, n_steps, n_experts, window))


def remoe_loss_backward(probs: torch.Tensor, probs_ref: torch.Tensor, idx: torch.Tensor, lags, window: int, coef,
                        loss_values: torch.Tensor, dlogits: torch.Tensor, workspace: torch.Tensor) -> None:
    """coef: 5 host floats (Reuse, Trust, Smooth, Lag, WS); loss_values fp64 [S, 6] from remoe_loss_forward;
    dlogits fp32 [S, T, N] (written)."""
    n_seq, n_steps, n_experts = probs.shape
    lg = (ctypes.c_int32 * max(len(lags), 1))(*lags)
    cf = (ctypes.c_double * 5)(*[float(c) for c in coef])
    _check(load_library().remoe_loss_backward(_ptr(probs), _ptr(probs_ref), _ptr(idx), n_seq, n_steps, n_experts,
                                              idx.shape[2], lg, len(lags), window, cf, _ptr(loss_values), _ptr(dlogits),
                                              _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def remoe_gate_grad_workspace_bytes(n_tokens: int, n_experts: int, hidden: int) -> int:
    return int(load_library().remoe_gate_grad_workspace_bytes(n_tokens, n_experts, hidden))


def remoe_gate_grad(dlogits: torch.Tensor, x: torch.Tensor, dw: torch.Tensor, workspace: torch.Tensor) -> None:
    """dlogits fp32 [T, N]; x [T, H] fp32 or bf16; dw fp32 [N, H] (overwritten)."""
    n_tokens, n_experts = dlogits.shape
    hidden = x.shape[1]
    code = REMOE_BF16 if x.dtype == torch.bfloat16 else REMOE_F32
    _check(load_library().remoe_gate_grad(_ptr(dlogits), _ptr(x), code, n_tokens, n_experts, hidden, _ptr(dw),
                                          _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))
