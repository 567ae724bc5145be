"""Pins for the CPU oracle: everything here checks `oracle/` against something
other than itself -- brute force, textbook / library routines, invariants, and
the figures the paper prints (tests/golden/paper_figures.txt).  CPU only."""
import itertools
import math

import numpy as np
import pytest
import scipy.special

import oracle
from oracle import accounting


def rng(seed):
    return np.random.default_rng(seed)


def to_bf16_bits(a):
    """fp32 -> bf16 bit patterns by numpy bit arithmetic (round to nearest even)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (b.astype(np.uint32) << 16).view(np.float32)


# ------------------------------------------------------------------ route
@pytest.mark.parametrize("T,d,E,k,seed", [(8, 16, 6, 2, 0), (5, 8, 7, 3, 1), (8, 32, 5, 5, 2), (3, 4, 4, 1, 3)])
def test_route_brute_force(T, d, E, k, seed):
    r = rng(seed)
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = r.standard_normal((d, E)).astype(np.float32)
    bias = r.standard_normal(E).astype(np.float32)
    idx, w, margin, logits = oracle.route(x, Wg, k, bias, want_logits=True)
    ref_logits = x.astype(np.float64) @ Wg.astype(np.float64) + bias.astype(np.float64)
    np.testing.assert_allclose(logits, ref_logits, rtol=0, atol=1e-12)
    for t in range(T):
        # the chosen set maximises the summed score over all C(E,k) subsets
        best = max(itertools.combinations(range(E), k), key=lambda s: sum(ref_logits[t, e] for e in s))
        assert set(idx[t]) == set(best)
        assert len(set(idx[t])) == k and all(0 <= e < E for e in idx[t])
        sc = ref_logits[t, idx[t]]
        assert all(sc[j] >= sc[j + 1] for j in range(k - 1))  # descending
        order = np.argsort(-ref_logits[t], kind="stable")[:k]  # full sort cross-check
        assert list(order) == list(idx[t])
        # softmax over the full row, renormalised over the chosen k
        p = scipy.special.softmax(ref_logits[t])
        np.testing.assert_allclose(w[t], p[idx[t]] / p[idx[t]].sum(), rtol=1e-6)
        assert abs(float(w[t].astype(np.float64).sum()) - 1.0) < 1e-6
        srt = np.sort(ref_logits[t])[::-1]
        gaps = srt[: (k + 1 if k < E else k)]
        assert margin[t] == pytest.approx(np.min(gaps[:-1] - gaps[1:]), abs=1e-12)


def test_route_special_cases():
    r = rng(7)
    T, d, E = 6, 12, 5
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = r.standard_normal((d, E)).astype(np.float32)
    # k = E: weights are the textbook softmax of the logits
    idx, w, _, logits = oracle.route(x, Wg, E, want_logits=True)
    for t in range(T):
        np.testing.assert_allclose(w[t], scipy.special.softmax(logits[t])[idx[t]], rtol=1e-6)
        assert sorted(idx[t]) == list(range(E))
    # k = 1: weight exactly 1, index = argmax
    idx1, w1, _ = oracle.route(x, Wg, 1)
    assert np.all(w1 == 1.0)
    assert np.array_equal(idx1[:, 0], np.argmax(logits, axis=1))
    # equal logits: 1/k each, lowest ids first
    idx0, w0, m0 = oracle.route(np.zeros((2, d), np.float32), Wg, 3)
    assert np.array_equal(idx0, np.tile(np.arange(3, dtype=np.int32), (2, 1)))
    np.testing.assert_allclose(w0, 1.0 / 3.0, rtol=1e-7)
    assert np.all(m0 == 0.0)


def test_route_column_permutation_equivariance():
    r = rng(9)
    T, d, E, k = 16, 24, 9, 3
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = r.standard_normal((d, E)).astype(np.float32)
    bias = r.standard_normal(E).astype(np.float32)
    idx, w, _ = oracle.route(x, Wg, k, bias)
    pi = r.permutation(E)  # new column c holds old expert pi[c]
    idx2, w2, _ = oracle.route(x, Wg[:, pi].copy(), k, bias[pi].copy())
    assert np.array_equal(pi[idx2], idx)
    np.testing.assert_allclose(w2, w, rtol=1e-6)


def test_route_bf16_inputs_are_read_exactly():
    r = rng(10)
    T, d, E, k = 4, 64, 8, 2
    xb = to_bf16_bits(r.standard_normal((T, d)))
    Wb = to_bf16_bits(r.standard_normal((d, E)) * 0.02)
    _, _, _, logits = oracle.route(xb, Wb, k, want_logits=True)
    ref = bf16_bits_to_f32(xb).astype(np.float64) @ bf16_bits_to_f32(Wb).astype(np.float64)
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-13)


# --------------------------------------------------------------- dispatch
@pytest.mark.parametrize("T,k,E,seed", [(64, 2, 8, 0), (37, 4, 16, 1), (8, 1, 4, 2), (50, 3, 3, 3)])
def test_dispatch_against_library_sort(T, k, E, seed):
    r = rng(seed)
    idx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    counts, offsets, perm, inv = oracle.dispatch(idx, E)
    flat = idx.reshape(-1)
    N = T * k
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    assert counts.sum() == N and offsets[0] == 0 and offsets[E] == N
    assert np.array_equal(offsets[1:], np.cumsum(counts))
    assert np.array_equal(perm, np.argsort(flat, kind="stable"))
    assert sorted(perm.tolist()) == list(range(N))  # bijection
    assert np.array_equal(inv[perm], np.arange(N))
    srt = flat[perm]
    assert np.all(srt[1:] >= srt[:-1])
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)


def test_dispatch_empty_experts_and_gather():
    idx = np.array([[3], [3], [0], [3]], np.int32)
    counts, offsets, perm, inv = oracle.dispatch(idx, 5)
    assert counts.tolist() == [1, 0, 0, 3, 0]
    assert offsets.tolist() == [0, 1, 1, 1, 4, 4]
    assert perm.tolist() == [2, 0, 1, 3]
    x = np.arange(4 * 3, dtype=np.float32).reshape(4, 3)
    xp = oracle.gather(x, perm, 1)
    assert np.array_equal(xp, x[perm])
    xb = to_bf16_bits(x)
    assert np.array_equal(oracle.gather(xb, perm, 1), xb[perm])


# ---------------------------------------------------------------- experts
def dense_swiglu(x, W1, W3, W2):
    x, W1, W3, W2 = (a.astype(np.float64) for a in (x, W1, W3, W2))
    g = x @ W1
    u = x @ W3
    return (g * scipy.special.expit(g) * u) @ W2


def test_dispatch_padded_layout_balanced_routing_has_no_padding():
    """Balanced routing (paper section 6.1): token t picks experts (t*k + j) mod E, so every expert gets
    exactly EC = T*k/E slots; with capacity = EC the padded layout IS the ragged one."""
    T, k, E = 48, 4, 16
    idx = ((np.arange(T)[:, None] * k + np.arange(k)[None, :]) % E).astype(np.int32)
    EC = T * k // E
    ragged = oracle.dispatch(idx, E)
    padded = oracle.dispatch(idx, E, capacity=EC)
    assert np.all(ragged[0] == EC)
    for a, b in zip(ragged, padded):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("T,k,E,C,seed", [(40, 2, 6, 0, 1), (100, 3, 7, 64, 2), (17, 1, 3, 0, 3)])
def test_dispatch_padded_layout_against_enumeration(T, k, E, C, seed):
    """Padded layout, by its definition: expert e's slots, ascending, at positions e*C ..; -1 behind them."""
    rng = np.random.default_rng(seed)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    flat = idx.reshape(-1)
    cmax = int(np.bincount(flat, minlength=E).max())
    C = C or cmax  # (C = 0 in the parameters: the tightest capacity that drops nothing)
    counts, offsets, perm, inv = oracle.dispatch(idx, E, capacity=C)
    assert np.array_equal(offsets, np.arange(E + 1) * C)
    want = np.full(E * C, -1, np.int64)
    for e in range(E):
        slots = [s for s in range(T * k) if flat[s] == e]
        assert counts[e] == len(slots)
        want[e * C:e * C + len(slots)] = slots
    assert np.array_equal(perm, want)
    assert np.array_equal(perm[inv], np.arange(T * k))
    assert (perm < 0).sum() == E * C - T * k
    # rows of unused positions are zero, the others are the token's row
    x = rng.standard_normal((T, 5)).astype(np.float32)
    xp = oracle.gather(x, perm, k)
    assert np.array_equal(xp[perm >= 0], x[perm[perm >= 0] // k]) and not xp[perm < 0].any()
    with pytest.raises(ValueError):
        oracle.dispatch(idx, E, capacity=cmax - 1)


def test_forward_does_not_depend_on_the_layout():
    rng = np.random.default_rng(5)
    T, d, E, k, f = 24, 16, 4, 2, 8
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = rng.standard_normal((d, E)).astype(np.float32)
    W1, W3 = (0.1 * rng.standard_normal((E, d, f)).astype(np.float32) for _ in range(2))
    W2 = 0.1 * rng.standard_normal((E, f, d)).astype(np.float32)
    a = oracle.forward(x, Wg, W1, W3, W2, k)
    b = oracle.forward(x, Wg, W1, W3, W2, k, capacity=int(a["counts"].max()) + 3)
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["staging"], b["staging"])
    assert np.array_equal(b["perm"][b["inv_perm"]], np.arange(T * k))


def test_experts_single_expert_is_a_dense_mlp():
    r = rng(20)
    T, d, f = 10, 24, 40
    x = r.standard_normal((T, d)).astype(np.float32)
    W1 = (r.standard_normal((1, d, f)) * 0.3).astype(np.float32)
    W3 = (r.standard_normal((1, d, f)) * 0.3).astype(np.float32)
    W2 = (r.standard_normal((1, f, d)) * 0.3).astype(np.float32)
    idx = np.zeros((T, 1), np.int32)
    res = oracle.forward(x, None, W1, W3, W2, 1, idx=idx, w=np.ones((T, 1), np.float32))
    ref = dense_swiglu(x, W1[0], W3[0], W2[0])
    np.testing.assert_allclose(res["y"], ref, rtol=2e-6, atol=1e-6)
    np.testing.assert_allclose(res["out"], ref, rtol=2e-6, atol=1e-6)  # k = 1, w = 1: out is the y row
    # W1 and W3 are distinguishable (a swapped operand changes the result)
    assert np.abs(dense_swiglu(x, W3[0], W1[0], W2[0]) - ref).max() > 1e-3


def test_experts_multi_expert_against_per_expert_dense():
    r = rng(21)
    T, d, f, E, k = 24, 16, 20, 4, 2
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = r.standard_normal((d, E)).astype(np.float32)
    W1 = (r.standard_normal((E, d, f)) * 0.3).astype(np.float32)
    W3 = (r.standard_normal((E, d, f)) * 0.3).astype(np.float32)
    W2 = (r.standard_normal((E, f, d)) * 0.3).astype(np.float32)
    res = oracle.forward(x, Wg, W1, W3, W2, k)
    idx, w = res["idx"], res["w"]
    ref_out = np.zeros((T, d))
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            y = dense_swiglu(x[t:t + 1], W1[e], W3[e], W2[e])[0]
            np.testing.assert_allclose(res["staging"][t * k + j], y, rtol=2e-6, atol=1e-6)
            ref_out[t] += float(w[t, j]) * y
    np.testing.assert_allclose(res["out"], ref_out, rtol=3e-6, atol=1e-6)
    # the token-restricted path is the same function of the same inputs
    tok = np.array([0, 5, 23], np.int32)
    st, out = oracle.forward_tokens(x, W1, W3, W2, idx, w, tok)
    assert np.array_equal(out, res["out"][tok])
    assert np.array_equal(st.reshape(3, k, d), res["staging"].reshape(T, k, d)[tok])


def test_experts_zero_scale_and_equivariance():
    r = rng(22)
    T, d, f, E, k = 12, 8, 12, 3, 2
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = r.standard_normal((d, E)).astype(np.float32)
    W1 = (r.standard_normal((E, d, f)) * 0.5).astype(np.float32)
    W3 = (r.standard_normal((E, d, f)) * 0.5).astype(np.float32)
    W2 = (r.standard_normal((E, f, d)) * 0.5).astype(np.float32)
    base = oracle.forward(x, Wg, W1, W3, W2, k)
    assert np.all(oracle.forward(x, Wg, W1, W3, np.zeros_like(W2), k)["out"] == 0)
    assert np.all(oracle.forward(x, Wg, np.zeros_like(W1), W3, W2, k)["out"] == 0)
    np.testing.assert_allclose(oracle.forward(x, Wg, W1, W3, 2.0 * W2, k)["out"], 2.0 * base["out"], rtol=1e-6)
    # token permutation equivariance
    pt = r.permutation(T)
    np.testing.assert_allclose(oracle.forward(x[pt].copy(), Wg, W1, W3, W2, k)["out"], base["out"][pt], rtol=1e-6,
                               atol=1e-7)
    # relabelling the experts leaves the layer output unchanged
    pe = r.permutation(E)
    rel = oracle.forward(x, Wg[:, pe].copy(), W1[pe].copy(), W3[pe].copy(), W2[pe].copy(), k)
    np.testing.assert_allclose(rel["out"], base["out"], rtol=1e-6, atol=1e-7)


def test_faithful_mode_rounds_to_bf16_and_stays_close():
    r = rng(23)
    T, d, f, E, k = 16, 64, 96, 4, 2
    x = to_bf16_bits(r.standard_normal((T, d)))
    Wg = to_bf16_bits(r.standard_normal((d, E)) * 0.02)
    W1 = to_bf16_bits(r.standard_normal((E, d, f)) * 0.1)
    W3 = to_bf16_bits(r.standard_normal((E, d, f)) * 0.1)
    W2 = to_bf16_bits(r.standard_normal((E, f, d)) * 0.1)
    a = oracle.forward(x, Wg, W1, W3, W2, k)
    b = oracle.forward(x, Wg, W1, W3, W2, k, faithful=True)
    # every faithful output is representable in bf16 ...
    assert np.array_equal(bf16_bits_to_f32(to_bf16_bits(b["out"])), b["out"])
    assert np.array_equal(bf16_bits_to_f32(to_bf16_bits(b["staging"])), b["staging"])
    # ... and within a few bf16 ulps of the exact result, measured per row
    scale = np.abs(a["out"]).max(axis=1, keepdims=True)
    assert (np.abs(a["out"] - b["out"]) / scale).max() < 2e-2


def _f32(bits):
    return float(np.array([bits], np.uint32).view(np.float32)[0])


# (input bits, expected bf16 bits): derived by hand from the definition "nearest representable value, ties to the
# one whose last kept bit is 0".  bf16 keeps the upper 16 bits of the fp32 pattern; the lower 16 decide.
ROUND_BF16_TABLE = [
    (0x3F800000, 0x3F80),  # 1.0 is representable
    (0x3F807FFF, 0x3F80),  # just below the midpoint: down
    (0x3F808001, 0x3F81),  # just above the midpoint: up (truncation would give 0x3F80)
    (0x3F808000, 0x3F80),  # midpoint, lower neighbour even: down (round-half-up would give 0x3F81)
    (0x3F818000, 0x3F82),  # midpoint, lower neighbour odd: up to the even one
    (0x3FFFFFFF, 0x4000),  # mantissa overflows: carry into the exponent, 2.0
    (0x3FFF8000, 0x4000),  # midpoint below 2.0, lower neighbour odd: carry into the exponent
    (0x3FFE8000, 0x3FFE),  # midpoint, lower neighbour even: stays
    (0xBF808000, 0xBF80),  # negative values: the sign does not take part
    (0xBF818000, 0xBF82),
    (0xBF808001, 0xBF81),
    (0xBF807FFF, 0xBF80),
    (0xC0FFC000, 0xC100),  # -7.9921875 -> -8.0: carry into the exponent, negative
    (0x00000000, 0x0000),
    (0x80000000, 0x8000),
    (0x3A83126F, 0x3A83),  # 0.001: lower half 0x126F < 0x8000, down
    (0x3DCCCCCD, 0x3DCD),  # 0.1: lower half 0xCCCD > 0x8000, up
]


@pytest.mark.parametrize("bits,want", ROUND_BF16_TABLE)
def test_round_bf16_table(bits, want):
    got = np.array([oracle.round_bf16(_f32(bits))], np.float32).view(np.uint32)[0]
    assert got == (want << 16), f"{bits:#010x} -> {got:#010x}, expected {want << 16:#010x}"


def numpy_faithful_layer(x, W1, W3, W2, idx, w):
    """The layer with the roundings a bf16 matrix-core pipeline cannot avoid (section 6.2, 'Correctness'), rebuilt
    with numpy matmuls and this file's own integer rounding: g, u rounded to fp32; h = silu(g) * u to bf16; y to
    fp32, then bf16; out to fp32, then bf16.  Inputs are bf16 bit patterns.  Every dot product here is a sum of
    products of short mantissas whose exponents span far less than 53 bits, so fp64 sums are exact in any order and
    the comparison with the oracle can be bit for bit."""
    xf, W1f, W3f, W2f = (bf16_bits_to_f32(a).astype(np.float64) for a in (x, W1, W3, W2))
    T, k = idx.shape
    d = xf.shape[1]
    staging = np.empty((T * k, d), np.float32)
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            g = (xf[t] @ W1f[e]).astype(np.float32).astype(np.float64)
            u = (xf[t] @ W3f[e]).astype(np.float32).astype(np.float64)
            h = np.array([gj / (1.0 + math.exp(-gj)) * uj for gj, uj in zip(g, u)], np.float64)
            h = bf16_bits_to_f32(to_bf16_bits(h.astype(np.float32))).astype(np.float64)
            y = (h @ W2f[e]).astype(np.float32)
            staging[t * k + j] = bf16_bits_to_f32(to_bf16_bits(y))
    acc = (w.astype(np.float64)[:, :, None] * staging.reshape(T, k, d).astype(np.float64)).sum(axis=1)
    out = bf16_bits_to_f32(to_bf16_bits(acc.astype(np.float32)))
    return staging, out


@pytest.mark.parametrize("T,d,f,E,k,seed", [(16, 64, 96, 4, 2, 23), (9, 32, 48, 3, 3, 24), (12, 128, 64, 5, 1, 25)])
def test_faithful_mode_bit_exact_against_numpy_rebuild(T, d, f, E, k, seed):
    r = rng(seed)
    x = to_bf16_bits(r.standard_normal((T, d)))
    Wg = to_bf16_bits(r.standard_normal((d, E)) * 0.02)
    W1 = to_bf16_bits(r.standard_normal((E, d, f)) * 0.1)
    W3 = to_bf16_bits(r.standard_normal((E, d, f)) * 0.1)
    W2 = to_bf16_bits(r.standard_normal((E, f, d)) * 0.1)
    res = oracle.forward(x, Wg, W1, W3, W2, k, faithful=True)
    st, out = numpy_faithful_layer(x, W1, W3, W2, res["idx"], res["w"])
    assert np.array_equal(res["staging"].view(np.uint32), st.view(np.uint32))
    assert np.array_equal(res["out"].view(np.uint32), out.view(np.uint32))
    # the exact mode differs from it (else the comparison above would say nothing about the roundings)
    exact = oracle.forward(x, Wg, W1, W3, W2, k)
    assert not np.array_equal(exact["staging"], st) and not np.array_equal(exact["out"], out)
    # the token-restricted entry point takes the same roundings
    tok = np.array(sorted({0, T // 2, T - 1}), np.int32)
    st_t, out_t = oracle.forward_tokens(x, W1, W3, W2, res["idx"], res["w"], tok, faithful=True)
    assert np.array_equal(out_t.view(np.uint32), out[tok].view(np.uint32))
    assert np.array_equal(st_t.reshape(len(tok), k, d).view(np.uint32), st.reshape(T, k, d)[tok].view(np.uint32))
    # and the stand-alone combine
    cmb = oracle.combine(st, res["w"], faithful=True)
    assert np.array_equal(cmb.view(np.uint32), out.view(np.uint32))


def test_faithful_rebuild_notices_a_missing_rounding_of_h():
    """The pin above is sharp: the same rebuild WITHOUT the rounding of h to bf16 (a planted mistake, on the CPU)
    does not reproduce the oracle's faithful output."""
    r = rng(23)
    T, d, f, E, k = 16, 64, 96, 4, 2
    x = to_bf16_bits(r.standard_normal((T, d)))
    Wg = to_bf16_bits(r.standard_normal((d, E)) * 0.02)
    W1 = to_bf16_bits(r.standard_normal((E, d, f)) * 0.1)
    W3 = to_bf16_bits(r.standard_normal((E, d, f)) * 0.1)
    W2 = to_bf16_bits(r.standard_normal((E, f, d)) * 0.1)
    res = oracle.forward(x, Wg, W1, W3, W2, k, faithful=True)
    xf, W1f, W3f, W2f = (bf16_bits_to_f32(a).astype(np.float64) for a in (x, W1, W3, W2))
    e = res["idx"][0, 0]
    g = (xf[0] @ W1f[e]).astype(np.float32).astype(np.float64)
    u = (xf[0] @ W3f[e]).astype(np.float32).astype(np.float64)
    h = g / (1.0 + np.exp(-g)) * u  # not rounded
    y = bf16_bits_to_f32(to_bf16_bits((h @ W2f[e]).astype(np.float32)))
    assert not np.array_equal(y, res["staging"][0])


# ---------------------------------------------------------------- combine
def test_combine_identity_experts_return_x():
    r = rng(30)
    T, d, E, k = 20, 16, 6, 3
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = r.standard_normal((d, E)).astype(np.float32)
    _, w, _ = oracle.route(x, Wg, k)
    staging = np.repeat(x, k, axis=0)  # every chosen expert returns the token itself
    np.testing.assert_allclose(oracle.combine(staging, w), x, rtol=1e-6, atol=1e-6)
    # distinct weights matter: a hand-computed two-expert case
    st = np.array([[1.0, 2.0], [10.0, 20.0]], np.float32)
    out = oracle.combine(st, np.array([[0.25, 0.75]], np.float32))
    np.testing.assert_allclose(out, [[7.75, 15.5]], rtol=1e-7)


def test_stage_is_the_inverse_permutation():
    y = np.arange(12, dtype=np.float32).reshape(6, 2)
    perm = np.array([4, 0, 5, 1, 3, 2], np.int32)
    inv = np.empty(6, np.int32)
    inv[perm] = np.arange(6)
    st = oracle.stage(y, inv)
    assert np.array_equal(st[perm], y)  # sorted row p goes to slot perm[p]


# ---------------------------------------------------------------- publish
def brute_publish(idx, E, R, d, tm, tn):
    """Independent re-count: enumerate slots, collect tiles in a python set."""
    T, k = idx.shape
    flat = idx.reshape(-1)
    perm = np.argsort(flat, kind="stable")
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size)
    off = np.concatenate([[0], np.cumsum(np.bincount(flat, minlength=E))])
    ncb = -(-d // tn)
    tiles = set()
    for s in range(T * k):
        e, r = flat[s], (s // k) // (T // R)
        q = inv[s] - off[e]
        for c in range(ncb):
            tiles.add((r, e, q // tm, c))
    order = {t: i for i, t in enumerate(sorted(tiles))}
    slot_flag = np.array([order[((s // k) // (T // R), flat[s], (inv[s] - off[flat[s]]) // tm, 0)]
                          for s in range(T * k)], np.int32)
    return len(tiles), slot_flag, len({t[0] for t in tiles})


@pytest.mark.parametrize("T,k,E,R,d,tm,tn,seed", [(32, 2, 4, 4, 128, 4, 64, 0), (64, 4, 8, 8, 200, 8, 64, 1),
                                                   (16, 2, 16, 16, 64, 32, 64, 2), (48, 1, 3, 2, 96, 5, 32, 3)])
def test_publish_plan_against_enumeration(T, k, E, R, d, tm, tn, seed):
    r = rng(seed)
    idx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    _, offsets, _, inv = oracle.dispatch(idx, E)
    plan = oracle.publish_plan(idx, offsets, inv, E, R, d, tm, tn)
    n, slot_flag, nd = brute_publish(idx, E, R, d, tm, tn)
    assert plan["n_flags"] == n
    assert np.array_equal(plan["slot_flag"], slot_flag)
    assert plan["fences_per_tile"] == n  # coupled: one fence per published tile
    assert plan["fences_per_dest"] == nd  # decoupled, per-destination groups
    assert plan["dest_flag_begin"][0] == 0 and plan["dest_flag_begin"][R] == n
    assert plan["seg_cnt"].sum() == T * k
    # upper bound the library's flag allocation relies on
    assert n <= (-(-T * k // tm) + E * R) * -(-d // tn)


# ---------------------------------------------- the figures the paper prints
def test_paper_flop_and_message_figures(golden):
    g = golden
    assert accounting.flops_per_row(1, 1) == g["flop_factor_gated_mlp"]
    for name, key in (("qwen3", "ratio_qwen3"), ("gptoss", "ratio_gptoss")):
        H, I = int(g[f"{name}_H"]), int(g[f"{name}_I"])
        assert round(accounting.compute_to_comm_ratio(H, I, int(g[f"{name}_k"])), 1) == g[key]
    assert round(accounting.compute_to_comm_ratio(5120, 8192), 1) == g["ratio_llama4"]
    for name in ("qwen3", "gptoss"):
        H, E, k = int(g[f"{name}_H"]), int(g[f"{name}_E"]), int(g[f"{name}_k"])
        assert accounting.message_bytes(1024, k, E, H) == 1024 * g[f"msg_bytes_per_S_{name}"]
    assert accounting.tile_bytes(int(g["tile_rows"]), int(g["tile_cols"])) == g["tile_kbytes_bf16"] * 1024


def test_paper_transfer_and_fence_counts(golden):
    g = golden
    E = int(g["qwen3_E"])
    for P, key in ((16, "16gpu_4node"), (32, "32gpu_8node"), (8, "8gpu_2node")):
        n = accounting.concurrent_transfers(P, 4, E)  # 4 PEs per node on that machine
        assert n == g[f"transfers_{key}"]
        per_pe = E // P  # one group per remote PE
        assert accounting.fence_count(n, per_pe) == g[f"fences_{key.split('_')[0]}_per_pe"]
    assert accounting.fence_count(112, 4) == g["fences_112_group4"]
    assert accounting.fence_count(112, 28) == g["fences_112_group28"]
    assert g["transfers_16gpu_4node"] / g["fences_16gpu_per_pe"] == g["fence_reduction_factor_qwen3"]
    assert accounting.fence_count(7, 3) == 3  # ragged last group still needs its fence


def test_paper_zipf_mass(golden):
    g = golden
    pmf = accounting.zipf_pmf(int(g["zipf_experts"]), g["zipf_exponent"])
    assert abs(sum(pmf) - 1.0) < 1e-12
    assert round(sum(pmf[: int(g["zipf_top"])]), 2) == g["zipf_top_mass"]
    assert all(a > b for a, b in zip(pmf, pmf[1:]))
    assert math.isclose(accounting.zipf_pmf(4, 0.0)[2], 0.25)
