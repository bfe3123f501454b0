"""Comparison of an Alg. 1 result (codes, zero points, scales from the GPU path) with the CPU oracle, written
so that a red test means a wrong kernel and never an unlucky rounding tie.

The bar (Section 2: quant rounds to the nearest grid value; Alg. 1): levels `code - zero` agree on at least
99.9 % of the weights and the rest differ by one grid step at rounding ties.  Two arithmetics can only differ
where w/scale lies next to a half-integer, but one such flip changes every later weight of its row a little, so
a handful of later decisions of that row flip too.  The audit therefore has two legs:

  raw      the oracle's own free run against the result: agreement of the levels.
  forced   the oracle takes every decision on the RESULT's history (teacher forcing: it decides, reports its
           decision, then continues from the result's level).  No flip can cascade, so every differing decision
           must be a near-tie, |frac(w/scale) - 1/2| <= tie_tol, one step wide, and there may be at most 0.1 % of
           them.  A kernel that rounds wrongly, reads a wrong element of U or drops an update differs at
           decisions that are nowhere near a tie and fails here.

The raw agreement has to reach 99.9 % as well unless every row that disagrees does so from a column on at which
the forced leg found a near-tie (the first difference of a row is always such a decision: up to there both runs
have the same history).
"""
import numpy as np

from oracle import gptq_oracle as O


def levels(codes, zero, gsz):
    return np.asarray(codes).astype(np.int64) - np.repeat(np.asarray(zero).astype(np.int64), gsz, axis=1)


def tie_distance(frac):
    f = np.asarray(frac, dtype=np.float64)
    return np.abs(np.abs(f - np.floor(f)) - 0.5)


def audit_alg1(W64, U, bits, grid, block, group, codes_g, zero_g, scale_g, decision_dtype,
               tie_tol=1e-3, say=print, tag="alg1", free=None, scale_rtol=1e-5):
    """Asserts the bar described in the module docstring; returns a dict of what was measured, with the
    oracle's free run under "free"."""
    W64 = np.asarray(W64, dtype=np.float64)
    r, n = W64.shape
    gsz = group if group else n
    lev_g = levels(codes_g, zero_g, gsz)
    if free is None:
        free = O.gptq_quantize(W64, U, bits, grid, block, group, decision_dtype=decision_dtype)
    lev_o = levels(free["codes"], free["zero"], gsz)
    raw_diff = np.abs(lev_g - lev_o)
    raw = float((raw_diff == 0).mean()) if raw_diff.size else 1.0
    out = dict(raw=raw, raw_max_step=int(raw_diff.max()) if raw_diff.size else 0, forced=1.0, n_forced_diff=0,
               max_tie_dist=0.0, cascade_rows=0, free=free)
    name = np.dtype(decision_dtype).name
    if raw == 1.0:
        assert np.allclose(scale_g, free["scale"], rtol=scale_rtol)
        say(f"  {tag} [{name} decisions]: raw agreement 1.00000")
        return out
    forced = O.gptq_quantize(W64, U, bits, grid, block, group, decision_dtype=decision_dtype, teacher_levels=lev_g)
    # grids of the forced run are taken on the result's history: scales agree to float32 rounding
    assert np.allclose(scale_g, forced["scale"], rtol=scale_rtol), "grid scales differ beyond rounding"
    # A zero point may itself fall on the other side of a tie of rint(-lo/scale).  That is a legitimate difference
    # between two arithmetics if -lo/scale is next to a half-integer; it moves the clamping range of that row's
    # group by one step, so decisions there may differ where one side clamps -- and only there.
    zmis = forced["zero"] != np.asarray(zero_g)
    zdiff = float(zmis.mean())
    if zmis.any():
        assert np.abs(forced["zero"] - np.asarray(zero_g)).max() <= 1
        assert tie_distance(forced["zero_real"][zmis]).max() <= tie_tol, "a zero point differs that is not a rounding tie"
    maxq = O.grid_maxq(bits, grid)
    lev_f = levels(forced["codes"], forced["zero"], gsz)
    fdiff = np.abs(lev_f - lev_g)
    codes_g = np.asarray(codes_g).astype(np.int64)
    clamped = (forced["codes"] == 0) | (forced["codes"] == maxq) | (codes_g == 0) | (codes_g == maxq)
    excused = np.repeat(zmis, gsz, axis=1) & clamped & (fdiff == 1)
    nz = (fdiff != 0) & ~excused
    out["forced"] = float((~nz).mean())
    out["n_forced_diff"] = int(nz.sum())
    if nz.any():
        out["max_tie_dist"] = float(tie_distance(forced["frac"][nz]).max())
    rows = np.flatnonzero(raw_diff.any(axis=1))
    first_raw = np.array([np.flatnonzero(raw_diff[i])[0] for i in rows], dtype=np.int64)
    # ... or lies in or behind a group whose zero point was such a tie (audited above)
    explained = np.array([nz[i, c] or zmis[i, :c // gsz + 1].any() for i, c in zip(rows, first_raw)], dtype=bool)
    out["cascade_rows"] = int(len(rows))
    say(f"  {tag} [{name} decisions]: raw agreement {raw:.5f} (max step {out['raw_max_step']}, {len(rows)} rows differ), "
        f"forced agreement {out['forced']:.6f} ({out['n_forced_diff']} decisions differ, farthest from a tie "
        f"{out['max_tie_dist']:.2e}), zero points differing {zdiff:.5f}")
    assert fdiff.max() <= 1, "a forced decision differs by more than one grid step"
    assert excused.mean() <= 1e-3, "too many decisions differ behind zero-point ties"
    assert out["forced"] >= 0.999, "more than 0.1 % of the decisions differ on the same history"
    assert out["max_tie_dist"] <= tie_tol, "a decision differs that is not a rounding tie"
    assert zdiff <= 5e-3 or zmis.sum() <= 1, "too many zero points differ"
    assert out["raw_max_step"] <= 1, "levels differ by more than one grid step"
    assert explained.all(), "a row diverges from the oracle at a decision that is not a rounding tie"
    if raw < 0.999:
        say(f"  {tag}: raw agreement below 99.9 %: all {len(rows)} differing rows start at an audited near-tie (cascade)")
    return out


def compare_quant(res, W64, U64, Hd, bits, grid, group, tag, tie_tol=1e-3, say=print):
    """`res` holds GPU tensors codes / zeros / scales / half_E2_rows / Wq (solver.LayerResult).  The GPU result against the oracle's Alg. 1 on (W64, U64), with the decision w -> code taken in float64
    (the oracle proper) and in float32 (the precision of the kernel): at least 99.9 % of the levels equal and every
    difference a one-step rounding tie, audited on the GPU's own history (tests/parity_util.py); layer error within
    1 %; the kernel's closed-form (1/2) sum e^2 within 1 % of the real error."""
    codes = res.codes.cpu().numpy().astype(np.int64)
    zero = res.zeros.cpu().numpy().astype(np.int64)
    scale = res.scales.cpu().numpy()
    n = np.asarray(W64).shape[1]
    gsz = group if group else n
    lev_g = levels(codes, zero, gsz)
    Qg = np.repeat(scale.astype(np.float64), gsz, axis=1) * lev_g
    eg = O.layer_error_H(W64, Qg, Hd)
    half = float(res.half_E2_rows.sum().item())
    raws = []
    for dd in (np.float64, np.float32):
        a = audit_alg1(W64, U64, bits, grid, 128, group, codes, zero, scale, dd, tie_tol=tie_tol, say=say, tag=tag)
        ora = a["free"]
        eo = O.layer_error_H(W64, ora["Q"], Hd)
        say(f"  {tag}: err_gpu={eg:.6e} err_oracle={eo:.6e} halfE2={half:.6e}")
        assert abs(eg - eo) <= 0.01 * eo
        assert abs(half - 0.5 * np.sum(ora["E"] ** 2)) <= 0.01 * 0.5 * np.sum(ora["E"] ** 2)
        raws.append(a["raw"])
    assert abs(half - eg) <= 0.01 * eg                       # the kernel's closed-form error is the real one
    if res.Wq is not None:
        assert np.allclose(res.Wq.double().cpu().numpy(), Qg, rtol=1e-6, atol=1e-12)
    return min(raws)
