"""Shared helpers of the GPU parity tests: tolerances and the tie-window comparison."""
from __future__ import annotations

import torch

import oracle

TIE_WINDOW = 1e-4        # tokens whose K-th and (K+1)-th logits are closer than this may go either way
W_RTOL, W_ATOL = 2e-5, 1e-7
F32_MAX_REL = 1e-4       # max |diff| / max |ref| per layer, fp32 layers
BF16_REL_L2 = 2e-2       # ||diff||_2 / ||ref||_2 per layer, bf16 layers


def to_oracle_weights(weights: dict) -> dict:
    return {k: (None if v is None else v.cpu()) for k, v in weights.items()}


def compare_routing(gpu_idx: torch.Tensor, gpu_w: torch.Tensor, orc: dict, renorm: bool):
    """Check GPU routing against the oracle's (which must hold 'probs').

    Expert sets must be identical except for tokens inside the tie window, which are returned
    (and printed) as a list; gate weights are compared against the oracle's probabilities of the
    ids the GPU picked.  Returns (tie_tokens, expected_w) with expected_w in the GPU's id order.
    """
    gi = gpu_idx.cpu().long()
    gw = gpu_w.cpu().double()
    oi = orc["idx"].long()
    T, K = gi.shape
    same_order = (gi == oi).all(1)
    same_set = torch.sort(gi, 1).values.eq(torch.sort(oi, 1).values).all(1)
    ties = []
    for t in torch.nonzero(~same_set).flatten().tolist():
        assert float(orc["margin"][t]) < TIE_WINDOW, (
            f"token {t}: expert sets differ outside the tie window: gpu {gi[t].tolist()} "
            f"oracle {oi[t].tolist()} margin {float(orc['margin'][t]):.3e}")
        ties.append(t)
    if ties:
        print(f"[tie window] {len(ties)} of {T} tokens differ within {TIE_WINDOW}: {ties[:8]}")
    # order inside the top-k may legitimately differ only where two selected logits nearly tie
    assert int((~same_order & same_set).sum()) <= max(4, T // 1000), "top-k order differs too often"
    assert (gi >= 0).all() and (gi < orc["probs"].shape[1]).all()
    assert (torch.sort(gi, 1).values[:, 1:] != torch.sort(gi, 1).values[:, :-1]).all(), "duplicate expert ids"
    exp_w = torch.gather(orc["probs"], 1, gi)
    if renorm:
        exp_w = exp_w / exp_w.sum(1, keepdim=True)
    assert torch.allclose(gw, exp_w, rtol=W_RTOL, atol=W_ATOL), (
        f"gate weights differ: max abs {float((gw - exp_w).abs().max()):.3e}")
    return ties, exp_w


BF16_COL_BLOCK = 256     # columns of one output tile of the down projection


def check_output(y_gpu: torch.Tensor, y_ref: torch.Tensor, dtype: str, report: dict = None):
    """fp32: max |diff| / max |ref| over the layer.  bf16: the relative L2 error over the layer, and the
    same bound for every token (row) on its own and for every (row, 256-column block) cell, so that one
    wrong row or one wrong 16-byte piece of a row cannot hide in the layer's norm.  Returns the layer
    figure; `report` (if given) receives the worst row and the worst cell."""
    yg = y_gpu.cpu().double()
    diff = yg - y_ref
    if dtype == "f32":
        err = float(diff.abs().max() / y_ref.abs().max())
        assert err <= F32_MAX_REL, f"fp32 max relative error {err:.3e} > {F32_MAX_REL}"
        return err
    err = float(diff.norm() / y_ref.norm())
    assert err <= BF16_REL_L2, f"bf16 relative L2 error {err:.3e} > {BF16_REL_L2}"
    if diff.dim() == 2 and diff.shape[0] > 0:
        row_err = diff.norm(dim=1) / y_ref.norm(dim=1)
        worst_row = int(row_err.argmax())
        assert float(row_err[worst_row]) <= BF16_REL_L2, (
            f"row {worst_row}: bf16 relative L2 error {float(row_err[worst_row]):.3e} > {BF16_REL_L2}")
        H = diff.shape[1]
        nb = (H + BF16_COL_BLOCK - 1) // BF16_COL_BLOCK
        pad = nb * BF16_COL_BLOCK - H
        d2 = torch.nn.functional.pad(diff, (0, pad)).reshape(-1, nb, BF16_COL_BLOCK)
        r2 = torch.nn.functional.pad(y_ref, (0, pad)).reshape(-1, nb, BF16_COL_BLOCK)
        cell = d2.norm(dim=2) / r2.norm(dim=2).clamp_min(1e-300)
        worst_cell = float(cell.max())
        assert worst_cell <= BF16_REL_L2, f"a (row, column-block) cell is off by {worst_cell:.3e} > {BF16_REL_L2}"
        if report is not None:
            report.update(worst_row=float(row_err[worst_row]), worst_cell=worst_cell)
    return err


def slot_aimed_tokens(idx: torch.Tensor, n_experts: int, tile: int = 256, experts: int = 16, boundaries: int = 4):
    """Tokens that sit where the grouped GEMM is most likely to go wrong, worked out on the host from the
    expert ids alone: the (token, j) pairs are sorted by expert, stable in pair order (the slot order of
    the sort step), and for `experts` evenly spaced experts the tokens of the first and last slot and of
    the slots either side of up to `boundaries` tile boundaries (the first and the last ones) are taken.
    Returns a sorted tensor of distinct token numbers."""
    T, K = idx.shape
    flat = idx.reshape(-1).long().cpu()
    order = torch.sort(flat, stable=True).indices          # slot -> pair index
    counts = torch.bincount(flat, minlength=n_experts)
    offs = torch.cumsum(counts, 0) - counts
    picked = []
    busy = [e for e in range(n_experts) if int(counts[e]) > 0]
    step = max(1, len(busy) // experts)
    chosen = busy[::step][:experts]
    if busy and busy[-1] not in chosen:
        chosen.append(busy[-1])
    for e in chosen:
        lo, n = int(offs[e]), int(counts[e])
        slots = {lo, lo + n - 1}
        cuts = list(range(tile, n, tile))
        for b in cuts[:boundaries // 2] + cuts[-(boundaries - boundaries // 2):]:
            slots.update((lo + b - 1, lo + b))
        picked += [int(order[s]) // K for s in slots]
    return torch.tensor(sorted(set(picked)), dtype=torch.int64)


def oracle_layer(x_cpu, weights_cpu, top_k, renorm, gpu_idx, gpu_w, tokens=None):
    """Oracle routing for all tokens plus expert outputs (for `tokens`) evaluated on the GPU's
    expert choice with the oracle's own gate weights for it."""
    orc = oracle.route(x_cpu, weights_cpu["w_router"], top_k, renorm, want_probs=True)
    ties, exp_w = compare_routing(gpu_idx, gpu_w, orc, renorm)
    y_ref = oracle.experts_sparse(x_cpu, gpu_idx.cpu().int(), exp_w, weights_cpu, tokens)
    return orc, ties, y_ref
