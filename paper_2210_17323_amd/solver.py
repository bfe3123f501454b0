"""Convenience driver: allocates the device buffers with PyTorch and walks one layer -- or the linear layers
of one transformer block -- through the C-ABI calls.  Every arithmetic step happens inside the library's HIP
kernels."""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as B


@dataclass
class LayerResult:
    codes: torch.Tensor          # [r, n] uint8
    scales: torch.Tensor         # [r, G] float32
    zeros: torch.Tensor          # [r, G] int32
    half_E2_rows: torch.Tensor   # [r] float64
    Wq: torch.Tensor | None      # [r, n] float32 (optional)
    packed: torch.Tensor | None  # [r, ceil(n*bits/32)] int32 (optional)


def new_hessian(n: int, device="cuda") -> torch.Tensor:
    return torch.zeros((n, n), dtype=torch.float32, device=device)


def accumulate(H: torch.Tensor, X: torch.Tensor, chunk: int | None = None) -> None:
    """H += 2 X X^T, optionally walking the token axis in chunks (multiples of 8 tokens)."""
    n, t = X.shape
    step = t if chunk is None or chunk >= t else chunk
    nbytes = max(B.gptq_hessian_accumulate_workspace_bytes(n, c, X.dtype) for c in {step, t % step or step})
    ws = torch.empty(nbytes, dtype=torch.uint8, device=X.device) if nbytes else None
    for c0 in range(0, t, step):
        B.gptq_hessian_accumulate(H, X[:, c0:min(c0 + step, t)], ws)


def cholesky_inverse(H: torch.Tensor, percdamp: float = 0.01, check: bool = True) -> torch.Tensor:
    """In place H -> U; returns H (now U).  Raises GptqError if a pivot is not positive."""
    n = H.shape[0]
    ws = torch.empty(B.gptq_damp_cholesky_inverse_workspace_bytes(n), dtype=torch.uint8, device=H.device)
    info = torch.zeros(1, dtype=torch.int32, device=H.device)
    B.gptq_damp_cholesky_inverse(H, percdamp, ws, info)
    if check:
        B.gptq_check_info(info)
    return H


def cholesky_factor(H: torch.Tensor, percdamp: float = 0.01, check: bool = True) -> torch.Tensor:
    """In place H -> R with H + lambda I = R R^T (no inverse); returns H (now R)."""
    n = H.shape[0]
    ws = torch.empty(B.gptq_damp_cholesky_workspace_bytes(n), dtype=torch.uint8, device=H.device)
    info = torch.zeros(1, dtype=torch.int32, device=H.device)
    B.gptq_damp_cholesky(H, percdamp, ws, info)
    if check:
        B.gptq_check_info(info)
    return H


def quantize(W: torch.Tensor, U: torch.Tensor, bits: int, grid: str = "minmax", block: int = 128, group: int = 0,
             want_Wq: bool = False, pack: bool = False, ws: torch.Tensor | None = None, from_factor: bool = False) -> LayerResult:
    """Alg. 1 + optional packing.  from_factor: `U` is the factor R of cholesky_factor (one grid per row, or groups of
    32, 64 or 128 columns: B.gptq_quantize_layer_from_factor_supports)."""
    r, n = W.shape
    dev = W.device
    G = n // group if group else 1
    codes = torch.empty((r, n), dtype=torch.uint8, device=dev)
    scales = torch.empty((r, G), dtype=torch.float32, device=dev)
    zeros = torch.empty((r, G), dtype=torch.int32, device=dev)
    half = torch.zeros(r, dtype=torch.float64, device=dev)
    Wq = torch.empty((r, n), dtype=torch.float32, device=dev) if want_Wq else None
    if ws is None:
        ws = torch.empty(B.gptq_quantize_layer_workspace_bytes(r, n, block, group), dtype=torch.uint8, device=dev)
    gid = B.GPTQ_GRID_TERNARY if grid == "ternary" else B.GPTQ_GRID_MINMAX
    B.gptq_quantize_layer(W, U, bits, gid, block, group, codes, scales, zeros, ws, Wq, half, from_factor=from_factor)
    packed = None
    if pack:
        pbits = 2 if grid == "ternary" else bits
        packed = torch.empty((r, B.packed_words_per_row(n, pbits)), dtype=torch.int32, device=dev)
        B.gptq_pack(codes, pbits, packed)
    return LayerResult(codes, scales, zeros, half, Wq, packed)


def solve_block(groups, bits: int | None = None, chunk: int | None = None, want_Wq: bool = False, timings: dict | None = None,
                factors: dict | None = None, form: str = "auto", overlap: bool = False, stack: bool = True):
    """The layers of one block, quantized in sequence (Section 4, Setup: a block's inputs are collected, its
    layers quantized, then the next block).  `groups` is a list of (X, layers): X [n x m] are the input
    activations shared by `layers`, a list of (name, W, settings) with settings an object carrying
    bits / grid / block / group / percdamp (e.g. workloads.configs.Layer).  Layers that share an input share
    one Hessian and one factor.  Returns {name: LayerResult}; if `timings` is a dict it receives, per group,
    the milliseconds of the Hessian and of the factorisation, and per layer those of Alg. 1 plus packing
    (CUDA events; with overlap the phases of different groups run at the same time, so they do not add up to the
    wall time, which is returned under "total").  If `factors` is a dict it receives {group index: the factor
    each group's layers were quantized with} (otherwise it is freed as soon as the group is done).
    chunk: tokens per gptq_hessian_accumulate call (None: a group's whole input in one call, which lets the library
    split or slice the token range itself).
    form: "inverse" factors every group into U = Cholesky((H + lambda I)^-1)^T; "factor" into R with
    H + lambda I = R R^T and runs Alg. 1 from R (no triangular inverse; one grid per row or groups of 32, 64 or 128
    columns); "auto" takes the factor form for the groups all of whose layers it is offered for.
    overlap: the Hessian of group k+1 is accumulated on a second stream while group k is factored and quantized
    (the factorisation's serial chains leave most of the chip idle).
    stack: layers of a group with the same bits, grid, block, group size and weight type are quantized as one matrix of
    stacked rows (their results are row slices of the stack's; their time is reported under "a+b+c:quantize_pack")."""
    out = {}
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream() if overlap else main
    t_begin, t_end = ev(), ev()
    t_begin.record(main)

    def hessian_of(gi):
        X = groups[gi][0]
        e0, e1 = ev(), ev()
        with torch.cuda.stream(side):
            e0.record()
            H = new_hessian(X.shape[0], X.device)
            accumulate(H, X, chunk)
            e1.record()
        marks.append((f"group{gi}:hessian", e0, e1))
        return H, e1

    if overlap:
        side.wait_stream(main)
    pending = hessian_of(0)
    for gi, (X, layers) in enumerate(groups):
        n = X.shape[0]
        H, h_done = pending
        main.wait_event(h_done)
        if gi + 1 < len(groups):
            pending = hessian_of(gi + 1)          # with overlap: runs beside this group's factorisation and Alg. 1
        e = [ev(), ev()]
        e[0].record()
        from_factor = form == "factor" or (form == "auto" and all(B.gptq_quantize_layer_from_factor_supports(lay.group) for _, _, lay in layers))
        U = (cholesky_factor if from_factor else cholesky_inverse)(H, layers[0][2].percdamp)
        e[1].record()
        marks.append((f"group{gi}:damp_cholesky_inverse", e[0], e[1]))
        ws = None
        # Rows are independent in Alg. 1 (Section 2: the objective is a sum over rows), so layers that share the factor and
        # the grid settings go through it as ONE matrix of stacked rows: one pass over the columns instead of one per
        # layer, with three times the rows per kernel for q, k, v.
        stacks = []
        for name, W, lay in layers:
            key = (lay.bits if bits is None else bits, lay.grid, lay.block, lay.group, W.dtype)
            for st in stacks:
                if stack and st[0] == key:
                    st[1].append((name, W, lay))
                    break
            else:
                stacks.append((key, [(name, W, lay)]))
        for (b, grid, block, group, _), members in stacks:
            Ws = members[0][1] if len(members) == 1 else torch.cat([W for _, W, _ in members], dim=0)
            need = B.gptq_quantize_layer_workspace_bytes(Ws.shape[0], n, block, group)
            if ws is None or ws.numel() < need:
                ws = None
                ws = torch.empty(need, dtype=torch.uint8, device=X.device)
            q0, q1 = ev(), ev()
            q0.record()
            res = quantize(Ws, U, b, grid, block, group, want_Wq=want_Wq, pack=True, ws=ws, from_factor=from_factor)
            q1.record()
            r0 = 0
            for name, W, _ in members:
                r1 = r0 + W.shape[0]
                out[name] = res if len(members) == 1 else LayerResult(
                    res.codes[r0:r1], res.scales[r0:r1], res.zeros[r0:r1], res.half_E2_rows[r0:r1],
                    None if res.Wq is None else res.Wq[r0:r1], None if res.packed is None else res.packed[r0:r1])
                r0 = r1
            marks.append(("+".join(name for name, _, _ in members) + ":quantize_pack", q0, q1))
            del Ws, res
        if factors is not None:
            factors[gi] = U
        if overlap:
            H.record_stream(main)
        del H, U, ws
    t_end.record(main)
    if timings is not None:
        torch.cuda.synchronize()
        for key, a, b in marks:
            timings[key] = a.elapsed_time(b)
        timings["total"] = t_begin.elapsed_time(t_end)
    return out
