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
 (iii) against the bf16-faithful oracle the row-normalised error is at most two
      bf16 ulps of the row maximum (8e-3).
fp32 problems: row-normalised 1e-4.
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2605_00686_amd import workloads as W

REL, ABS_FLOOR = 2e-2, 1e-3
RATE_FAITHFUL, RATE_EXACT = 1e-3, 0.08
REL_F32 = 1e-4
FAITHFUL_REL = 8e-3  # two bf16 ulps of the row maximum (2 * 2^-8)


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


def check_outputs(name, got, ref, ref_faithful, is_f32):
    """-> dict of metrics; raises AssertionError with the numbers when a bar fails."""
    m = {"row_err": float(row_err(got, ref).max()), "viol_rate": violation_rate(got, ref)}
    if is_f32:
        assert m["row_err"] <= REL_F32, f"{name}: fp32 row error {m['row_err']:.3e}"
        return m
    assert m["row_err"] <= REL, f"{name}: row-normalised error {m['row_err']:.3e} > {REL}"
    assert m["viol_rate"] < RATE_EXACT, f"{name}: {m['viol_rate']:.4%} of elements outside tolerance (exact oracle)"
    if ref_faithful is not None:
        m["row_err_faithful"] = float(row_err(got, ref_faithful).max())
        m["viol_rate_faithful"] = violation_rate(got, ref_faithful)
        assert m["row_err_faithful"] <= FAITHFUL_REL, f"{name}: vs bf16-faithful oracle {m['row_err_faithful']:.3e}"
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
