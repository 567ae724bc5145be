"""CPU oracle for the MoE hot path -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline``
leg may import this package.  The product (``paper_2605_00686_amd``) never does,
and this package never imports the product's HIP binding: the two share no code.

``moe_oracle.c`` holds the arithmetic (plain C, double accumulators);
this module only marshals numpy arrays into it.  ``accounting.py`` holds the
paper's closed-form figures (FLOPs, message sizes, transfer and fence counts).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_publish_plan.restype = ctypes.c_int64
        _lib.orc_num_threads.restype = ctypes.c_int
        _lib.orc_round_bf16.restype = ctypes.c_float
        _lib.orc_round_bf16.argtypes = [ctypes.c_float]
    return _lib


def round_bf16(v: float) -> float:
    """The rounding the bf16-faithful mode applies (nearest, ties to even), on one fp32 value."""
    return float(lib().orc_round_bf16(ctypes.c_float(v)))


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dt(a: np.ndarray) -> int:
    """fp32 arrays are values; uint16 arrays are raw bf16 bit patterns."""
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle tensors are float32 or uint16 (bf16 bits), got {a.dtype}")


def _c(a, dtype=None):
    a = np.ascontiguousarray(a)
    if dtype is not None and a.dtype != dtype:
        a = a.astype(dtype)
    return a


def route(x, Wg, k, bias=None, want_logits=False):
    """-> idx[T,k] int32, w[T,k] f32, margin[T] f64 (, logits[T,E] f64)."""
    x, Wg = _c(x), _c(Wg)
    T, d = x.shape
    E = Wg.shape[1]
    assert Wg.shape[0] == d and _dt(x) == _dt(Wg) and 1 <= k <= E
    idx = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float32)
    margin = np.empty(T, np.float64)
    logits = np.empty((T, E), np.float64) if want_logits else None
    b = None if bias is None else _c(bias, np.float32)
    lib().orc_route(T, d, E, k, _dt(x), _p(x), _p(Wg), _p(b), _p(idx), _p(w), _p(logits), _p(margin))
    return (idx, w, margin, logits) if want_logits else (idx, w, margin)


def dispatch(idx, E, capacity=0):
    """-> counts[E], offsets[E+1], perm, inv_perm[N] (all int32).
    capacity == 0: the ragged (dropless) order, perm[N].  capacity = C > 0: the padded layout of
    balanced routing (paper section 6.1, expert capacity EC = S*k/E): expert e owns the C sorted
    positions from e*C, its slots fill the first counts[e] of them in the same (stable) order,
    offsets[e] = e*C, perm[E*C] holds -1 in unused positions.  Nothing is dropped: counts beyond C
    raise."""
    flat = _c(idx, np.int32).reshape(-1)
    N = flat.size
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(N, np.int32)
    inv = np.empty(N, np.int32)
    lib().orc_dispatch(N, E, _p(flat), _p(counts), _p(offsets), _p(perm), _p(inv))
    if capacity > 0:
        if counts.max() > capacity:
            raise ValueError(f"an expert has {counts.max()} rows, capacity is {capacity}")
        padded_off = (np.arange(E + 1, dtype=np.int64) * capacity).astype(np.int32)
        rank = inv - offsets[flat]                      # position of slot s among its expert's slots
        inv_c = (padded_off[flat] + rank).astype(np.int32)
        perm_c = np.full(E * capacity, -1, np.int32)
        perm_c[inv_c] = np.arange(N, dtype=np.int32)
        return counts, padded_off, perm_c, inv_c
    return counts, offsets, perm, inv


def gather(x, perm, k):
    """x_perm[p] = x[perm[p] / k]; positions with perm[p] < 0 (padded layout) are zero rows."""
    x = _c(x)
    perm = _c(perm, np.int32)
    out = np.empty((perm.size, x.shape[1]), x.dtype)
    lib().orc_gather(int(perm.size), k, x.shape[1], _dt(x), _p(x), _p(np.maximum(perm, 0)), _p(out))
    out[perm < 0] = 0
    return out


def experts_sorted(x, W1, W3, W2, offsets, perm, k, faithful=False):
    """y[N,d] f32 in sorted order."""
    x, W1, W3, W2 = _c(x), _c(W1), _c(W3), _c(W2)
    E, d, f = W1.shape
    assert W3.shape == (E, d, f) and W2.shape == (E, f, d) and x.shape[1] == d
    N = perm.size
    y = np.empty((N, d), np.float32)
    lib().orc_experts_sorted(N, k, d, E, f, _dt(x), _p(x), _p(W1), _p(W3), _p(W2),
                             _p(_c(offsets, np.int32)), _p(_c(perm, np.int32)), int(faithful), _p(y))
    return y


def stage(y, inv_perm):
    y = _c(y, np.float32)
    out = np.empty_like(y)
    lib().orc_stage(y.shape[0], y.shape[1], _p(y), _p(_c(inv_perm, np.int32)), _p(out))
    return out


def combine(staging, w, faithful=False):
    w = _c(w, np.float32)
    T, k = w.shape
    staging = _c(staging, np.float32).reshape(T * k, -1)
    d = staging.shape[1]
    out = np.empty((T, d), np.float32)
    lib().orc_combine(T, k, d, _p(staging), _p(w), int(faithful), _p(out))
    return out


def forward_tokens(x, W1, W3, W2, idx, w, tokens, faithful=False):
    """Layer restricted to ``tokens`` -> staging_rows[n*k,d], out_rows[n,d]."""
    x, W1, W3, W2 = _c(x), _c(W1), _c(W3), _c(W2)
    idx, w = _c(idx, np.int32), _c(w, np.float32)
    tokens = _c(tokens, np.int32)
    E, d, f = W1.shape
    k = idx.shape[1]
    n = tokens.size
    st = np.empty((n * k, d), np.float32)
    out = np.empty((n, d), np.float32)
    lib().orc_forward_tokens(k, d, f, _dt(x), _p(x), _p(W1), _p(W3), _p(W2), _p(idx), _p(w),
                             n, _p(tokens), int(faithful), _p(st), _p(out))
    return st, out


def publish_plan(idx, offsets, inv_perm, E, R, d, tile_m, tile_n):
    """Flag layout of the publish step; see ``orc_publish_plan`` in the C file."""
    idx = _c(idx, np.int32)
    T, k = idx.shape
    assert T % R == 0
    seg_begin = np.empty(E * R, np.int32)
    seg_cnt = np.empty(E * R, np.int32)
    flag_base = np.empty(R * E, np.int32)
    slot_flag = np.empty(T * k, np.int32)
    dest_begin = np.empty(R + 1, np.int32)
    fa = ctypes.c_int64(0)
    fb = ctypes.c_int64(0)
    n = lib().orc_publish_plan(T, k, E, R, d, tile_m, tile_n, _p(idx), _p(_c(offsets, np.int32)),
                               _p(_c(inv_perm, np.int32)), _p(seg_begin), _p(seg_cnt), _p(flag_base),
                               _p(slot_flag), _p(dest_begin), ctypes.byref(fa), ctypes.byref(fb))
    return dict(n_flags=int(n), seg_begin=seg_begin.reshape(E, R), seg_cnt=seg_cnt.reshape(E, R),
                flag_base=flag_base.reshape(R, E), slot_flag=slot_flag, dest_flag_begin=dest_begin,
                fences_per_tile=int(fa.value), fences_per_dest=int(fb.value))


def forward(x, Wg, W1, W3, W2, k, bias=None, idx=None, w=None, faithful=False, capacity=0):
    """Whole layer through the sorted layout: route (unless idx/w are given),
    dispatch, experts, stage, combine.  Returns a dict of every intermediate.  The layout of the
    sorted order (ragged or padded to `capacity` rows per expert) changes where rows sit, i.e.
    offsets / perm / inv_perm as dispatch() returns them, and nothing that is computed."""
    if idx is None:
        idx, w, margin = route(x, Wg, k, bias)
    else:
        idx, w, margin = _c(idx, np.int32), _c(w, np.float32), None
    E = W1.shape[0]
    counts, offsets, perm, inv = dispatch(idx, E)
    y = experts_sorted(x, W1, W3, W2, offsets, perm, k, faithful)
    st = stage(y, inv)
    out = combine(st, w, faithful)
    if capacity > 0:
        counts, offsets, perm, inv = dispatch(idx, E, capacity)
    return dict(idx=idx, w=w, margin=margin, counts=counts, offsets=offsets, perm=perm,
                inv_perm=inv, y=y, staging=st, out=out)
