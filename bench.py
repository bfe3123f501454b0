#!/usr/bin/env python3
"""Benchmark of the GPTQ layer solve on one MI355X.

One step = one pass of the whole hot path over one synthetic layer: zero H, accumulate
H += 2 X X^T over all calibration tokens (in chunks), damp + Cholesky of the inverse, Algorithm 1
(block quantizer + trailing updates), bit packing.  Inputs are resident in HBM before timing starts.
Prints ONE JSON line: metric, value (TFLOP/s over the algorithmic flops of the whole solve), ms_per_step, per-phase
times, rates and fractions of peak, the roofline of the dominant kernel (the fp16 SYRK) and of the float32 GEMM, the same
figures for the other workload shapes from one short run each, and the CPU oracle baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_F16_MFMA_TFLOPS = 2516.6      # MI355X dense fp16/bf16 matrix-core peak
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM-side bytes of ONE syrk_f16_dma_kernel launch: a STORED reading, not measured in this run (hardware counters need
# rocprofv3 around the process).  From rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what the same counter reads
# for a plain 1 GiB copy kernel (factors 2.000 and 1.000): profiles/layer_solve_opt175b_fc2_pmc_counters.txt.  The fetch
# reading varies from one collection to the next; the entry is the one tabulated there, the note gives the range seen.
# Keyed by (n, tokens per launch); other shapes: not collected.
MEASURED_SYRK_TRAFFIC = {(49152, 32768): {"bytes": (6.4375e7 * 2.0 + 9.1801e6 * 1.0) * 1024,
                                          "note": "stored rocprofv3 reading (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000), not collected in "
                                                  "this run; nine collections of this launch gave 135-283 GB against 12.9 GB algorithmic "
                                                  "(X slice read once, upper triangle of H read and written once) plus the 6.4 GB of the "
                                                  "next slice's repack, which the launch does in its tail"}}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--layer", default="opt175b_fc2", help="opt175b_fc2 (headline) | opt175b_fc1 | opt6.7b_attn | bloom176b_qkv_2bit_g128 | "
                         "bloom176b_out_ternary_g128 | opt175b_q | tiny | opt175b_block (all six linears of a block)")
    ap.add_argument("--tokens", type=int, default=0, help="calibration tokens (default: the layer's own, 262144)")
    ap.add_argument("--chunk", type=int, default=0,
                    help="tokens per gptq_hessian_accumulate call (default: all of them in one call; the library splits the token "
                         "range of matrices with few tiles and walks long calls on large matrices in slices of 32768)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--form", choices=["auto", "factor", "inverse"], default="auto",
                    help="steps 2 and 3.  factor: gptq_damp_cholesky + gptq_quantize_layer_from_factor (Alg. 1 driven by the Cholesky "
                         "factor of H + lambda I itself, no triangular inverse; one grid per row or groups of 32, 64 or 128).  inverse: "
                         "gptq_damp_cholesky_inverse + gptq_quantize_layer (U = Cholesky of the inverse, any grid).  auto: factor "
                         "where the library offers it for the layer's grid, else inverse")
    ap.add_argument("--no-other-layers", action="store_true",
                    help="skip the short runs of the other workload shapes that the default (opt175b_fc2) line carries as extra keys")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the timed region, run one plain 1 GiB device-to-device copy kernel (dst = src * 1: known "
                         "traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled)")
    return ap.parse_args()


def pick_layer(name: str, tokens: int):
    from workloads import configs
    m = tokens or configs.TOKENS
    table = {
        "opt175b_fc2": lambda: configs.config3(m)[1],
        "opt175b_fc1": lambda: configs.config3(m)[0],
        "opt6.7b_attn": lambda: configs.config2(m)[0],
        "bloom176b_qkv_2bit_g128": lambda: configs.config4(m)[0],
        "bloom176b_out_ternary_g128": lambda: configs.config4(m)[3],
        "opt175b_q": lambda: configs.config5(m)[0],
        "tiny": lambda: configs.config1()[0],
    }
    return table[name]()


def flop_model(r: int, n: int, m: int, B: int = 128):
    """Algorithmic flops of each step: what the mathematics needs, not what the kernels execute."""
    trailing = sum(2 * r * min(B, n - i) * (n - i - min(B, n - i)) for i in range(0, n, B))
    inblock = sum(r * min(B, n - i) * (min(B, n - i) - 1) for i in range(0, n, B))
    return {
        "hessian": float(n) * (n + 1) * m,            # SYRK: n(n+1)/2 outputs, 2 flops per token
        "cholesky": float(n) ** 3 / 3.0,              # factorisation
        "tri_inverse": float(n) ** 3 / 3.0,           # triangular inverse
        "quantize": float(trailing + inblock),
    }


def cpu_baseline(lay, flops):
    """The float64 NumPy oracle, as it stands, timed on the host cores on a bounded sample of the
    same workload; each step is timed on a reduced problem and scaled by its flop count."""
    import numpy as np
    from oracle import gptq_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    n_h, t_h = min(lay.n, 6144), min(lay.x.m, 32768)
    X = lay.x.tile(nrows=n_h, ncols=t_h).double().numpy()
    t0 = time.perf_counter(); H = O.hessian(X); th = time.perf_counter() - t0
    full_h = th * flops["hessian"] / (float(n_h) * (n_h + 1) * t_h)
    t0 = time.perf_counter(); U = O.hinv_cholesky_upper(O.damp(H, lay.percdamp)); tc = time.perf_counter() - t0
    full_c = tc * (lay.n / n_h) ** 3
    r_q = min(lay.r, 128)
    W = lay.weights(nrows=r_q).double().numpy()[:, :n_h]
    t0 = time.perf_counter(); out = O.gptq_quantize(W, U, lay.bits, lay.grid, lay.block, 0 if not lay.group else lay.group); tq = time.perf_counter() - t0
    full_q = tq * (lay.r / r_q) * (lay.n / n_h) ** 2
    t0 = time.perf_counter(); O.pack_codes(out["codes"], 2 if lay.grid == "ternary" else lay.bits); tp = time.perf_counter() - t0
    full_p = tp * (lay.r / r_q) * (lay.n / n_h)
    total = full_h + full_c + full_q + full_p
    return {
        "value": sum(flops.values()) / total / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
        "sample": (f"float64 NumPy oracle timed on: Hessian {n_h}x{t_h} tokens ({th:.2f}s), damp+inverse+Cholesky n={n_h} ({tc:.2f}s), "
                   f"Alg.1 {r_q} rows x {n_h} cols ({tq:.2f}s), pack ({tp:.3f}s); each scaled by flop count to the full layer: "
                   f"EXTRAPOLATED layer solve {total:.0f} s"),
    }


def bench_block(a):
    """--layer opt175b_block: the six linears of one OPT-175B-shaped decoder block in sequence (q, k, v share one
    Hessian), 3-bit and 4-bit, with and without the next group's Hessian overlapped with the current group's
    factorisation and Alg. 1; prints per-layer times and the block totals as one JSON line."""
    import torch
    import paper_2210_17323_amd as g
    from paper_2210_17323_amd import solver as S
    from workloads import configs
    g.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    m = a.tokens or configs.TOKENS
    layers = configs.config5(m)
    by_x = {}
    for lay in layers:
        by_x.setdefault(lay.x.tensor_id, []).append(lay)
    groups = []
    for xid, lays in by_x.items():
        _, X = configs.materialize(replace_rows(lays[0], 1), dev)          # X only; weights come per layer below
        members = []
        for lay in lays:
            W = torch.empty((lay.r, lay.n), dtype=lay.dtype, device=dev)
            rows = max(1, (1 << 27) // lay.n)
            for r0 in range(0, lay.r, rows):
                W[r0:r0 + rows] = lay.weights(row0=r0, nrows=min(rows, lay.r - r0), device=dev)
            members.append((lay.name, W, lay))
        groups.append((X, members))
    chunk = min(a.chunk or m, m)
    form = "auto" if a.form == "auto" else a.form
    runs = {}
    for bits in (3, 4):
        for overlap in (False, True):
            S.solve_block(groups, bits=bits, chunk=chunk, form=form, overlap=overlap)            # warm-up
            torch.cuda.synchronize()
            t = {}
            t0 = time.perf_counter()
            S.solve_block(groups, bits=bits, chunk=chunk, form=form, overlap=overlap, timings=t)
            torch.cuda.synchronize()
            t["wall"] = (time.perf_counter() - t0) * 1e3
            runs[(bits, overlap)] = t
    def named(t):
        out = {}
        for gi, (_, members) in enumerate(groups):
            names = "+".join(nm for nm, _, _ in members)
            out[f"{names}:hessian"] = round(t[f"group{gi}:hessian"], 3)
            out[f"{names}:factorisation"] = round(t[f"group{gi}:damp_cholesky_inverse"], 3)
        for key, v in t.items():
            if key.endswith(":quantize_pack"):
                out[key] = round(v, 3)          # layers that share a factor go through Alg. 1 as one matrix of stacked rows
        return out
    total3 = min(runs[(3, False)]["total"], runs[(3, True)]["total"])
    out = {
        "metric": "gptq_block_solve_ms", "value": total3, "unit": "ms", "n_gpus": 1, "steps": 1, "warmup": 1,
        "ms_per_step": total3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 inputs, f32 accumulate (Hessian); f32 (Cholesky, Alg. 1: the large rank-1024 updates as products of three "
                 "bf16 pieces per f32 element, exact piece products accumulated in f32); u8 codes", "data": "synthetic",
        "config": {"workload": f"one OPT-175B-shaped decoder block: q, k, v, out 12288x12288, fc1 49152x12288, fc2 12288x49152, "
                               f"{m} tokens, per-row grids, B=128; q/k/v share one Hessian, one factor and one pass of Alg. 1 (stacked rows)",
                   "steps_2_and_3": form, "tokens_per_accumulate_call": chunk},
        "per_layer_ms_3bit_sequential": named(runs[(3, False)]),
        "per_layer_ms_4bit_sequential": named(runs[(4, False)]),
        "block_total_ms": {"3bit_sequential": round(runs[(3, False)]["total"], 3), "3bit_hessian_overlapped": round(runs[(3, True)]["total"], 3),
                           "4bit_sequential": round(runs[(4, False)]["total"], 3), "4bit_hessian_overlapped": round(runs[(4, True)]["total"], 3)},
    }
    print(json.dumps(out))


def replace_rows(lay, r):
    from dataclasses import replace
    return replace(lay, r=r)


class LayerBench:
    """Device buffers of one layer solve and the step that walks them through the four C-ABI calls."""

    def __init__(self, lay, chunk_arg: int, dev, factor_form: bool = False):
        import torch
        import paper_2210_17323_amd as g
        from workloads import configs
        self.g, self.torch, self.lay = g, torch, lay
        # factor_form: steps 2 and 3 through gptq_damp_cholesky + gptq_quantize_layer_from_factor (no triangular inverse)
        self.factor_form = factor_form
        r, n, m = lay.r, lay.n, lay.x.m
        self.W, self.X = configs.materialize(lay, dev)
        self.H = torch.empty((n, n), dtype=torch.float32, device=dev)
        self.chol_ws = torch.empty(g.gptq_damp_cholesky_inverse_workspace_bytes(n), dtype=torch.uint8, device=dev)
        self.info = torch.zeros(1, dtype=torch.int32, device=dev)
        self.q_ws = torch.empty(g.gptq_quantize_layer_workspace_bytes(r, n, lay.block, lay.group), dtype=torch.uint8, device=dev)
        G = n // lay.group if lay.group else 1
        self.codes = torch.empty((r, n), dtype=torch.uint8, device=dev)
        self.scales = torch.empty((r, G), dtype=torch.float32, device=dev)
        self.zeros = torch.empty((r, G), dtype=torch.int32, device=dev)
        self.half = torch.empty(r, dtype=torch.float64, device=dev)
        self.pbits = 2 if lay.grid == "ternary" else lay.bits
        self.packed = torch.empty((r, g.packed_words_per_row(n, self.pbits)), dtype=torch.int32, device=dev)
        self.grid = g.GPTQ_GRID_TERNARY if lay.grid == "ternary" else g.GPTQ_GRID_MINMAX
        # one call over all tokens: the library splits short matrices' token range and walks long ones slice by slice
        self.chunk = min(chunk_arg or m, m)
        self.chunks = [(c0, min(c0 + self.chunk, m)) for c0 in range(0, m, self.chunk)]
        h_bytes = g.gptq_hessian_accumulate_workspace_bytes(n, self.chunk, lay.x.dtype)
        self.h_ws = torch.empty(h_bytes, dtype=torch.uint8, device=dev) if h_bytes else None
        self.syrk_events, self.phase_events = [], []

    def step(self, record: bool):
        g, lay, torch = self.g, self.lay, self.torch
        ev = lambda: torch.cuda.Event(enable_timing=True)
        marks = [ev() for _ in range(5)] if record else None
        if record: marks[0].record()
        self.H.zero_()
        for (c0, c1) in self.chunks:
            if record:
                e0, e1 = ev(), ev(); e0.record()
            g.gptq_hessian_accumulate(self.H, self.X[:, c0:c1], self.h_ws)
            if record:
                e1.record(); self.syrk_events.append((e0, e1, c1 - c0))
        if record: marks[1].record()
        if self.factor_form:
            g.gptq_damp_cholesky(self.H, lay.percdamp, self.chol_ws, self.info)
        else:
            g.gptq_damp_cholesky_inverse(self.H, lay.percdamp, self.chol_ws, self.info)
        if record: marks[2].record()
        g.gptq_quantize_layer(self.W, self.H, lay.bits, self.grid, lay.block, lay.group, self.codes, self.scales, self.zeros,
                              self.q_ws, None, self.half, from_factor=self.factor_form)
        if record: marks[3].record()
        g.gptq_pack(self.codes, self.pbits, self.packed)
        if record:
            marks[4].record(); self.phase_events.append(marks)

    def run(self, steps: int, warmup: int):
        """`warmup` untimed steps, then exactly `steps` timed ones between two device synchronisations."""
        torch, g = self.torch, self.g
        for _ in range(warmup):
            self.step(False)
        torch.cuda.synchronize()
        if g.gptq_check_info(self.info) != 0:
            raise RuntimeError("Cholesky reported a non-positive pivot")
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(True)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
        names = ["hessian", "damp_cholesky_inverse", "quantize_layer", "pack"]
        phases = {nm: sum(mk[i].elapsed_time(mk[i + 1]) for mk in self.phase_events) / len(self.phase_events)
                  for i, nm in enumerate(names)}
        return ms_per_step, phases


def phase_rates(flops, phases, r, n, packed_numel, factor_form=False):
    chol_flops = flops["cholesky"] + (0.0 if factor_form else flops["tri_inverse"])
    tf = {
        "hessian_syrk": flops["hessian"] / (phases["hessian"] * 1e-3) / 1e12,
        "cholesky_plus_inverse_f32": chol_flops / (phases["damp_cholesky_inverse"] * 1e-3) / 1e12,
        "quantize_f32": flops["quantize"] / (phases["quantize_layer"] * 1e-3) / 1e12,
    }
    frac = {
        "hessian_of_fp16_mfma_peak": tf["hessian_syrk"] / PEAK_F16_MFMA_TFLOPS,
        "cholesky_plus_inverse_of_fp32_peak": tf["cholesky_plus_inverse_f32"] / PEAK_F32_TFLOPS,
        "quantize_of_fp32_peak": tf["quantize_f32"] / PEAK_F32_TFLOPS,
        "pack_of_hbm_peak": (r * n + packed_numel * 4) / (phases["pack"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
    }
    return tf, frac


FORM_NAME = {True: "gptq_damp_cholesky + gptq_quantize_layer_from_factor (Alg. 1 driven by the factor R of H + lambda I; no triangular inverse)",
             False: "gptq_damp_cholesky_inverse + gptq_quantize_layer (U = Cholesky((H + lambda I)^-1)^T)"}
OTHER_LAYERS = ["opt175b_fc1", "opt175b_q", "bloom176b_qkv_2bit_g128", "bloom176b_out_ternary_g128", "opt6.7b_attn"]


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the solver is a single-GPU path; --gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    if a.layer == "opt175b_block":
        return bench_block(a)
    import torch
    import paper_2210_17323_amd as g
    g.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    lay = pick_layer(a.layer, a.tokens)
    r, n, m = lay.r, lay.n, lay.x.m
    flops = flop_model(r, n, m, lay.block)
    if a.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)        # an elementwise kernel (a same-dtype copy_ would be a DMA transfer, not a kernel)
        torch.cuda.synchronize()
        del src, dst
    factor_form = a.form == "factor" or (a.form == "auto" and g.gptq_quantize_layer_from_factor_supports(lay.group))
    lb = LayerBench(lay, a.chunk, dev, factor_form=factor_form)
    ms_per_step, phases = lb.run(a.steps, a.warmup)
    chunk = lb.chunk
    ev = lambda: torch.cuda.Event(enable_timing=True)

    # per launch of the SYRK kernel: a call's event time over the launches the library says the call makes
    launches = sum(g.gptq_hessian_accumulate_launches(n, t, lay.x.dtype) for (_, _, t) in lb.syrk_events)
    syrk_avg_ms = sum(e0.elapsed_time(e1) for (e0, e1, _) in lb.syrk_events) / launches
    syrk_flops_per_launch = sum(float(n) * (n + 1) * t for (_, _, t) in lb.syrk_events) / launches
    tokens_per_launch = int(round(sum(t for (_, _, t) in lb.syrk_events) / launches))
    achieved = syrk_flops_per_launch / (syrk_avg_ms * 1e-3) / 1e12
    if factor_form:
        flops = dict(flops, tri_inverse=0.0)            # this form has no triangular inverse: not counted
    total_flops = sum(flops.values())
    tf, frac = phase_rates(flops, phases, r, n, lb.packed.numel(), factor_form)

    def timed(fn, reps):
        fn(); torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # Consumers of the packed layer (outside the timed step): batch-1 product and full decompression
    packed, scales, zeros, pbits = lb.packed, lb.scales, lb.zeros, lb.pbits
    xv = torch.randn(n, device=dev).half()
    yv = torch.empty(r, dtype=torch.float32, device=dev)
    Wd = torch.empty((r, n), dtype=torch.float16, device=dev)
    mv_ms = timed(lambda: g.gptq_matvec_packed(packed, n, pbits, scales, zeros, lay.group, xv, yv), 50)
    dq_ms = timed(lambda: g.gptq_dequantize_packed(packed, n, pbits, scales, zeros, lay.group, Wd), 10)
    grid_bytes = scales.numel() * 8
    mv_bytes = packed.numel() * 4 + grid_bytes + n * 2 + r * 4
    dq_bytes = packed.numel() * 4 + grid_bytes + r * n * 2
    del Wd

    # The deferred rank-1024 update that carries the larger share of the step (factorisation and Alg. 1), timed alone at the
    # shape of Alg. 1's median deferred update of this layer, W[r x n/2] -= E[r x 1024] U[1024 x n/2], operands taken
    # from the buffers of the solve: through the split products the solvers use at this size (bf16 matrix cores, six piece
    # products per float32 product; the time includes splitting both operands) and through the float32 kernel.
    gemm = split_gemm = None
    kk, nc = min(1024, n), (n // 2) // 256 * 256
    if nc >= 256 and r >= 256:
        Wt = torch.zeros((r, nc), dtype=torch.float32, device=dev)
        Et = torch.randn((r, kk), dtype=torch.float32, device=dev)
        Ut = lb.H[:kk, n - nc:]                                     # rows of the factor right of their diagonal block
        g_ms = timed(lambda: g.gptq_trailing_update(Wt, Et, Ut), 10)
        g_flops = 2.0 * r * nc * kk
        gemm = {"kernel": f"gemm_f32_dma_kernel (gptq_trailing_update: W[{r}x{nc}] -= E[{r}x{kk}] U[{kk}x{nc}])", "bound": "mfma",
                "achieved": g_flops / (g_ms * 1e-3) / 1e12, "peak": PEAK_F32_TFLOPS, "unit": "TFLOP/s",
                "frac": g_flops / (g_ms * 1e-3) / 1e12 / PEAK_F32_TFLOPS, "avg_launch_ms": g_ms, "flops_per_launch": g_flops,
                "traffic": None}
        if kk == 1024 and r % 256 == 0:
            sws = torch.empty(g.gptq_trailing_update_split_workspace_bytes(r, nc), dtype=torch.uint8, device=dev)
            s_ms = timed(lambda: g.gptq_trailing_update_split(Wt, Et, Ut, sws), 10)
            split_gemm = {"kernel": f"gemm_split_kernel + split_rows_kernel + split_cols_kernel (gptq_trailing_update_split, same shape)",
                          "bound": "mfma", "achieved": 6 * g_flops / (s_ms * 1e-3) / 1e12, "peak": PEAK_F16_MFMA_TFLOPS, "unit": "TFLOP/s",
                          "frac": 6 * g_flops / (s_ms * 1e-3) / 1e12 / PEAK_F16_MFMA_TFLOPS, "avg_launch_ms": s_ms,
                          "flops_per_launch": 6 * g_flops,
                          "float32_equivalent_tflops": g_flops / (s_ms * 1e-3) / 1e12,
                          "float32_equivalent_of_fp32_peak": g_flops / (s_ms * 1e-3) / 1e12 / PEAK_F32_TFLOPS,
                          "note": "bf16 matrix-core flops: six piece products per float32 product, priced against the bf16 peak; "
                                  "float32_equivalent counts the float32 product's own flops",
                          "traffic": None}
            del sws
        del Wt, Et, Ut

    traffic = MEASURED_SYRK_TRAFFIC.get((n, tokens_per_launch)) if lay.x.dtype != torch.float32 else None
    out = {
        "metric": "gptq_layer_solve_tflops", "value": total_flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 inputs, f32 accumulate (Hessian); f32 (Cholesky, Alg. 1: the large rank-1024 updates as products of three "
                 "bf16 pieces per f32 element, exact piece products accumulated in f32); u8 codes",
        "data": "synthetic",
        "value_note": "all algorithmic flops of the solve (fp16 SYRK + fp32 factorisation, inverse and Alg. 1) over the step "
                      "time: a throughput of the whole job, comparable with no single peak; see phase_frac_of_peak",
        "config": {"workload": f"{lay.name}: W {r}x{n} {str(lay.dtype).split('.')[-1]}, X {n}x{m} {str(lay.x.dtype).split('.')[-1]}, "
                               f"{lay.bits}-bit {lay.grid} grid, group {lay.group or 'per-row'}, B={lay.block}, damp {lay.percdamp}",
                   "tokens_per_accumulate_call": chunk,
                   "steps_2_and_3": FORM_NAME[factor_form]},
        "phases_ms": {k: round(v, 3) for k, v in phases.items()},
        "phase_tflops": tf,
        "phase_frac_of_peak": frac,
        "phase_frac_note": "Cholesky and Alg. 1: the float32 flops of the phase against the float32 matrix-core peak; their large updates "
                           "run as split products on the bf16 matrix cores (roofline_split_gemm), which is how a phase can pass 1",
        "pack_GBps": (r * n + packed.numel() * 4) / (phases["pack"] * 1e-3) / 1e9,
        "algorithmic_flops": flops,
        "packed_consumers": {"matvec_us": mv_ms * 1e3, "matvec_GBps": mv_bytes / (mv_ms * 1e-3) / 1e9,
                             "matvec_frac_of_hbm_peak": mv_bytes / (mv_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                             "dequantize_f16_ms": dq_ms, "dequantize_GBps": dq_bytes / (dq_ms * 1e-3) / 1e9,
                             "dequantize_frac_of_hbm_peak": dq_bytes / (dq_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "roofline": {"kernel": "syrk_f16_dma_kernel (HIP events around a gptq_hessian_accumulate call, divided by the launches of the kernel "
                               "the call makes; a launch repacks the next slice of the token range in its tail)",
                     "launches_per_call": launches // len(lb.syrk_events), "tokens_per_launch": tokens_per_launch,
                     "bound": "mfma", "achieved": achieved,
                     "peak": PEAK_F16_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_F16_MFMA_TFLOPS,
                     "avg_launch_ms": syrk_avg_ms, "flops_per_launch": syrk_flops_per_launch,
                     "traffic": traffic["bytes"] if traffic else None,
                     "traffic_unit": "bytes per launch",
                     "traffic_note": traffic["note"] if traffic else "not collected for this shape"},
        "roofline_f32_gemm": gemm,
        "roofline_split_gemm": split_gemm,
    }
    # The other workload shapes, one short run each (1 warm-up + 2 timed steps): per-layer time and per-phase fraction of peak
    if a.layer == "opt175b_fc2" and not a.no_other_layers:
        # the same layer through the other pair of calls (2 timed steps), on the buffers of the headline run
        if factor_form and a.form == "auto":
            lb.factor_form, lb.syrk_events, lb.phase_events = False, [], []
            ims, iph = lb.run(2, 1)
            ifl = flop_model(r, n, m, lay.block)
            itf, ifr = phase_rates(ifl, iph, r, n, lb.packed.numel(), False)
            out["same_layer_inverse_form"] = {"steps_2_and_3": FORM_NAME[False], "ms_per_step": round(ims, 3),
                                              "phases_ms": {k: round(v, 3) for k, v in iph.items()},
                                              "phase_tflops": {k: round(v, 2) for k, v in itf.items()},
                                              "phase_frac_of_peak": {k: round(v, 4) for k, v in ifr.items()}}
        del lb, packed, scales, zeros, xv, yv
        torch.cuda.empty_cache()
        others = {}
        for name in OTHER_LAYERS:
            ol = pick_layer(name, a.tokens)
            off = g.gptq_quantize_layer_from_factor_supports(ol.group)
            ob = LayerBench(ol, 0, dev, factor_form=off)
            oms, oph = ob.run(2, 1)
            ofl = flop_model(ol.r, ol.n, ol.x.m, ol.block)
            otf, ofr = phase_rates(ofl, oph, ol.r, ol.n, ob.packed.numel(), off)
            others[name] = {"workload": f"W {ol.r}x{ol.n}, X {ol.n}x{ol.x.m}, {ol.bits}-bit {ol.grid}, group {ol.group or 'per-row'}",
                            "steps_2_and_3": FORM_NAME[off],
                            "ms_per_step": round(oms, 3), "phases_ms": {k: round(v, 3) for k, v in oph.items()},
                            "phase_tflops": {k: round(v, 2) for k, v in otf.items()},
                            "phase_frac_of_peak": {k: round(v, 4) for k, v in ofr.items()}}
            del ob
            torch.cuda.empty_cache()
        out["other_layers"] = others
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(lay, flops)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
