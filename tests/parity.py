"""Shared helpers of the GPU parity tests: run the oracle on a workload, run
the HIP path on the same tensors, and compare to the stated bars.

Bars (the target statement of this build): routing indices, counts, offsets,
permutation, flag numbering and fence counts bit-exact.  bf16 outputs:

 (i)  against the exact (fp64-accumulating) oracle: max relative error 2e-2 with
      an absolute floor of 1e-3, read per row: max_n |g - r| / max(max_n |r|, 1e-3).
 (ii) the paper's criterion (section 6.2 "Correctness": error rate below 1%),
      element by element, |g - r| <= max(1e-3, 2e-2 |r|), against the
      bf16-faithful oracle (same arithmetic, h / y / out rounded to bf16 where
      a bf16 MFMA pipeline must round): fewer than 0.1% of elements outside.
      Against the exact oracle the same count is only reported and bounded by
      8%: h has to be rounded to bf16 to become an MFMA operand, which alone
      puts an error of about 1.5e-3 rms(y) on every y; an element then misses a
      2% RELATIVE bound whenever |r| < 0.07 rms(y), i.e. for about 5% of
      Gaussian-distributed outputs, whatever the kernel does.
 (iii) against the bf16-faithful oracle, per row, in units of the spacing of
      bf16 numbers (8 significant bits: ulp(v) = 2^(floor(log2 |v|) - 7), between
      2^-8 and 2^-7 of v): a row of staging may differ by one flipped rounding,
      max_n |g - r| <= 1.25 ulp(max_n |r|) (the quarter ulp covers what fp32
      accumulation and flipped roundings of h move the sum before it is rounded);
      a row of out by what its k staging rows may differ, weighted, plus one
      flipped rounding of its own: sum_j w_j 1.25 ulp(max |staging_j|) + ulp(max |out|).
fp32 problems: row-normalised 1e-4.
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2605_00686_amd import workloads as W

REL, ABS_FLOOR = 2e-2, 1e-3
RATE_FAITHFUL, RATE_EXACT = 1e-3, 0.08
# Against the EXACT oracle the elementwise rate is bounded per full-size workload by what an ideal bf16 pipeline
# gives there (measured on the committed seeds) plus one point; RATE_EXACT is the bound for everything else.
RATE_EXACT_BY_WORKLOAD = {"cfg1": 0.01, "cfg2": 0.0142, "cfg3": 0.0593, "cfg4": 0.0678, "cfg5": 0.0633, "cfg6": 0.0479,
                          "cfg7": 0.0635, "cfg8": 0.0143}
REL_F32 = 1e-4
FAITHFUL_REL = 8e-3  # rows without a per-row bound (see faithful_bounds): two bf16 ulps of a row maximum near 2^n
STAGING_ULPS = 1.25  # one flipped rounding, plus what moves the sum before it is rounded


def bf16_ulp(v):
    """spacing of bf16 numbers around |v| (8 significant bits): 2^(floor(log2 |v|) - 7); 0 where v == 0"""
    v = np.abs(np.asarray(v, np.float64))
    out = np.zeros_like(v)
    nz = v > 0
    out[nz] = np.exp2(np.floor(np.log2(v[nz])) - 7.0)
    return out


def faithful_bounds(st_f, out_f, w):
    """Per-row absolute bounds on |GPU - bf16-faithful oracle|: (staging rows [T*k], out rows [T]); st_f is the
    faithful staging [T*k, d] of the same tokens in slot order, w their gate weights [T, k]."""
    T, k = w.shape
    st_b = STAGING_ULPS * bf16_ulp(np.abs(st_f).max(axis=1))
    out_b = (w.astype(np.float64) * st_b.reshape(T, k)).sum(axis=1) + bf16_ulp(np.abs(out_f).max(axis=1))
    return st_b, out_b


def oracle_arrays(inp):
    return {n: W.as_oracle_array(inp.get(n)) for n in ("x", "Wg", "gate_bias", "W1", "W3", "W2", "topk_idx", "topk_w")}


def oracle_routing(inp):
    """idx, w (and margin) for a workload: computed, or taken from the inputs."""
    cfg = inp["cfg"]
    o = oracle_arrays(inp)
    if cfg["prerouted"] is None:
        idx, w, margin = oracle.route(o["x"], o["Wg"], cfg["k"], o["gate_bias"])
    else:
        idx, w, margin = o["topk_idx"], o["topk_w"], None
    return idx, w, margin


def row_err(got, ref):
    """per-row max |got - ref| normalised by max(row max |ref|, floor)."""
    scale = np.maximum(np.abs(ref).max(axis=1), ABS_FLOOR)
    return np.abs(got.astype(np.float64) - ref.astype(np.float64)).max(axis=1) / scale


def violation_rate(got, ref, rel=REL):
    bad = np.abs(got.astype(np.float64) - ref) > np.maximum(ABS_FLOOR, rel * np.abs(ref))
    return float(bad.mean())


def check_outputs(name, got, ref, ref_faithful, is_f32, rate_exact=None, row_bound=None):
    """-> dict of metrics; raises AssertionError with the numbers when a bar fails."""
    m = {"row_err": float(row_err(got, ref).max()), "viol_rate": violation_rate(got, ref)}
    if is_f32:
        assert m["row_err"] <= REL_F32, f"{name}: fp32 row error {m['row_err']:.3e}"
        return m
    assert m["row_err"] <= REL, f"{name}: row-normalised error {m['row_err']:.3e} > {REL}"
    bound = RATE_EXACT if rate_exact is None else rate_exact
    assert m["viol_rate"] < bound, f"{name}: {m['viol_rate']:.4%} of elements outside tolerance (exact oracle, bound {bound})"
    if ref_faithful is not None:
        m["row_err_faithful"] = float(row_err(got, ref_faithful).max())
        m["viol_rate_faithful"] = violation_rate(got, ref_faithful)
        if row_bound is None:
            assert m["row_err_faithful"] <= FAITHFUL_REL, f"{name}: vs bf16-faithful oracle {m['row_err_faithful']:.3e}"
        else:
            err = np.abs(got.astype(np.float64) - ref_faithful.astype(np.float64)).max(axis=1)
            ratio = np.where(row_bound > 0, err / np.where(row_bound > 0, row_bound, 1.0), np.where(err > 0, np.inf, 0.0))
            m["row_bound_ratio_faithful"] = float(ratio.max())
            assert m["row_bound_ratio_faithful"] <= 1.0, \
                f"{name}: row {int(ratio.argmax())} is {m['row_bound_ratio_faithful']:.3f} x its bound against the bf16-faithful oracle"
        assert m["viol_rate_faithful"] < RATE_FAITHFUL, \
            f"{name}: {m['viol_rate_faithful']:.4%} of elements outside tolerance (bf16-faithful oracle)"
    return m


def expected_fences(plan, signal_mode, group_size=0):
    """Release fences issued right before flag stores: one per publish tile in
    the coupled mode; in the decoupled mode one per non-empty destination, or,
    with a group size g, one per group of g flags of a destination:
    sum over r of ceil(n_r / g) (section 4.1, granularity of Algorithm 1)."""
    if signal_mode == 0:
        return plan["fences_per_tile"]
    if group_size == 0:
        return plan["fences_per_dest"]
    from oracle import accounting
    n_r = np.diff(plan["dest_flag_begin"].astype(np.int64))
    return int(sum(accounting.fence_count(int(n), group_size) for n in n_r if n > 0))
