"""Closed-form figures of the paper -- TEST INFRASTRUCTURE ONLY (see __init__).

Each function restates one counting rule from the paper so that tests can hold
it against the numbers the paper prints (tests/golden/paper_figures.txt).
"""
from __future__ import annotations


def flops_per_row(H: int, I: int) -> int:
    """Gated MLP: three H x I matrices, 2 FLOPs per multiply-add => 6*H*I per
    (token, expert) pair (section 3.1 footnote: 'gated MLP factor x6')."""
    return 6 * H * I


def compute_to_comm_ratio(H: int, I: int, k: int = 1) -> float:
    """Section 3.1 footnote: per-token FLOPs (k rows of 6*H*I) over the
    communication volume, quoted as TFLOPs/GB.  The printed values (4.6, 17.3,
    49.2) are reproduced when the volume of a routed row is counted as its H
    elements, one direction: ratio = k*6*H*I / (k*H) * 1e-12 / 1e-9."""
    flops = k * flops_per_row(H, I)
    volume = k * H
    return flops / volume * 1e-12 / 1e-9


def message_bytes(S: int, k: int, E: int, H: int) -> float:
    """Per-expert message M = EC * H * 2 with EC = S*k/E (appendix A)."""
    return S * k / E * H * 2


def tile_bytes(rows: int, cols: int, elem: int = 2) -> int:
    """Bytes of one tile (section 3.3: a 128 x 64 bf16 tile is 16 KB)."""
    return rows * cols * elem


def concurrent_transfers(P: int, P_local: int, E: int) -> int:
    """(P - P_local) * E / P transfers per dispatch through one proxy channel
    (section 3.2)."""
    return (P - P_local) * (E // P)


def fence_count(n_transfers: int, group_size: int) -> int:
    """One fence per group of signals (section 4.1, Algorithm 1 and its
    granularity footnote: 112 remote experts at group size 4 -> 28 fences)."""
    return -(-n_transfers // group_size)


def zipf_pmf(n: int, s: float):
    """pmf over ranks 1..n proportional to rank^-s (section 6.4)."""
    wts = [r ** (-s) for r in range(1, n + 1)]
    tot = sum(wts)
    return [v / tot for v in wts]
