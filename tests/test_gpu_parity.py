"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Sizes here finish in seconds on the CPU yet span
several tiles, ragged tails, empty segments and both signaling modes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_00686_amd import workloads as W
from tests import parity

pytestmark = pytest.mark.gpu


def _binding():
    from paper_2605_00686_amd import binding as B
    return B


def _dev(inp, names):
    return {n: (inp[n].cuda() if inp.get(n) is not None else None) for n in names}


def _problem(B, cfg, signal_mode=1, fence_scope=0, epoch=1, group_size=0, scheduler=0, capacity=0, wait_ticks=0,
             fuse_ffn=0):
    return B.problem(cfg["T"], cfg["d"], cfg["E"], cfg["k"], cfg["f"], cfg["R"], cfg["dtype"], tile_m=cfg["tile_m"],
                     tile_n=cfg["tile_n"], signal_mode=signal_mode, fence_scope=fence_scope, epoch=epoch,
                     group_size=group_size, scheduler=scheduler, capacity=capacity, wait_ticks=wait_ticks,
                     fuse_ffn=fuse_ffn)


def run_forward(B, inp, signal_mode, fence_scope, epoch=1, buf=None, group_size=0, scheduler=0, capacity=0,
                wait_ticks=0, fuse_ffn=0):
    cfg = inp["cfg"]
    p = _problem(B, cfg, signal_mode, fence_scope, epoch, group_size, scheduler, capacity, wait_ticks, fuse_ffn)
    buf = buf or B.Buffers(p)
    d = _dev(inp, ("x", "Wg", "gate_bias", "W1", "W3", "W2"))
    if cfg["prerouted"] is not None:
        buf.topk_idx.copy_(inp["topk_idx"])
        buf.topk_w.copy_(inp["topk_w"])
    buf.staging.fill_(float("nan"))  # poison: a row read before its flag would show
    buf.out.fill_(float("nan"))
    B.forward(p, buf, d["x"], d["Wg"], d["gate_bias"], d["W1"], d["W3"], d["W2"])
    torch.cuda.synchronize()
    return p, buf


def check_against_oracle(B, inp, p, buf, signal_mode, ref=None):
    cfg = inp["cfg"]
    o = parity.oracle_arrays(inp)
    idx, w, margin = parity.oracle_routing(inp)
    if ref is None:
        ref = oracle.forward(o["x"], o["Wg"], o["W1"], o["W3"], o["W2"], cfg["k"], idx=idx, w=w, capacity=p.capacity)
    stats = buf.stats.cpu().numpy()
    assert stats[7] == 0, f"device status {stats[7]} ({B.status_string(int(stats[7]))}), timeouts {stats[6]}"
    # integer work: bit-exact
    assert np.array_equal(buf.topk_idx.cpu().numpy(), idx), f"routing differs (min margin {None if margin is None else margin.min()})"
    np.testing.assert_allclose(buf.topk_w.cpu().numpy(), w, rtol=1e-5, atol=1e-7)
    assert np.array_equal(buf.counts.cpu().numpy(), ref["counts"])
    assert np.array_equal(buf.offsets.cpu().numpy(), ref["offsets"])
    assert np.array_equal(buf.perm.cpu().numpy(), ref["perm"])
    assert np.array_equal(buf.inv_perm.cpu().numpy(), ref["inv_perm"])
    plan = oracle.publish_plan(idx, ref["offsets"], ref["inv_perm"], cfg["E"], cfg["R"], cfg["d"], cfg["tile_m"],
                               cfg["tile_n"])
    assert np.array_equal(buf.slot_flag.cpu().numpy(), plan["slot_flag"])
    nfl = plan["n_flags"]
    assert nfl <= B.moe_num_flags(p)
    flags = buf.flags.cpu().numpy().view(np.uint32)
    assert np.all(flags[:nfl] == p.epoch), "a published tile has no flag"
    assert stats[0] == parity.expected_fences(plan, signal_mode, p.group_size), \
        (stats, plan["fences_per_tile"], plan["fences_per_dest"], p.group_size)
    assert stats[1] == nfl and stats[2] == nfl
    # floating point
    is_f32 = cfg["dtype"] == "f32"
    faithful = None
    if not is_f32:
        faithful = oracle.forward(o["x"], o["Wg"], o["W1"], o["W3"], o["W2"], cfg["k"], idx=idx, w=w, faithful=True)
    st = buf.staging.float().cpu().numpy()
    out = buf.out.float().cpu().numpy()
    assert not np.isnan(st).any() and not np.isnan(out).any(), "poison survived: a row was never written"
    st_b = out_b = None
    if faithful is not None:
        st_b, out_b = parity.faithful_bounds(faithful["staging"], faithful["out"], w)
    m1 = parity.check_outputs("staging", st, ref["staging"], None if faithful is None else faithful["staging"], is_f32,
                              row_bound=st_b)
    m2 = parity.check_outputs("out", out, ref["out"], None if faithful is None else faithful["out"], is_f32,
                              row_bound=out_b)
    print(f"[{cfg}] staging {m1} out {m2} stats {stats.tolist()}")
    return ref


@pytest.mark.parametrize("name", ["mini_f32", "mini_bf16", "mini_skew", "mini_pre", "mini_decode", "mini_large", "mini_odd"])
@pytest.mark.parametrize("signal_mode", [0, 1])
def test_megakernel_parity(name, signal_mode):
    B = _binding()
    print(f"case {name} signal_mode {signal_mode}", flush=True)
    inp = W.make_inputs(name)
    p, buf = run_forward(B, inp, signal_mode, 0)
    check_against_oracle(B, inp, p, buf, signal_mode)


@pytest.mark.parametrize("name", ["mini_bf16", "mini_decode", "mini_pre"])
def test_megakernel_fence_group_size(name):
    """Decoupled signaling at several granularities (section 4.1: one fence per
    group of g signals).  Same buffers for every g, rising epochs: outputs and
    flags as always, fences = sum over destinations of ceil(flags / g)."""
    B = _binding()
    inp = W.make_inputs(name)
    ref, buf = None, None
    for epoch, g in enumerate([0, 3, 1, 64, 100000, 8, 0], start=2):
        print(f"case {name} group_size {g}", flush=True)
        if buf is None:  # (one workspace serves every granularity)
            buf = B.Buffers(_problem(B, inp["cfg"], 1, 0, 1))
        p, buf = run_forward(B, inp, 1, 0, epoch=epoch, buf=buf, group_size=g)
        ref = check_against_oracle(B, inp, p, buf, 1, ref)


@pytest.mark.parametrize("name", ["mini_f32", "mini_bf16", "mini_skew", "mini_pre", "mini_decode", "mini_large", "mini_odd"])
def test_megakernel_ready_queue_scheduler(name):
    """The ready-queue scheduler (section 2.3: tasks enqueued when their inputs are there) against the
    oracle, in both signaling modes and with fence groups, on one set of buffers with rising epochs (so
    every queue must have emptied itself for the next call).  Every GEMM2 tile and every combine task
    goes through a queue exactly once."""
    B = _binding()
    inp = W.make_inputs(name)
    buf = B.Buffers(_problem(B, inp["cfg"], 1, 0, 1))
    ref = None
    for epoch, (mode, g) in enumerate([(1, 0), (0, 0), (1, 5), (1, 0)], start=2):
        print(f"case {name} ready queue, signal_mode {mode} group_size {g}", flush=True)
        p, buf = run_forward(B, inp, mode, 0, epoch=epoch, buf=buf, group_size=g, scheduler=1)
        ref = check_against_oracle(B, inp, p, buf, mode, ref)
        stats = buf.stats.cpu().numpy()
        n_comb = int(stats[16]) - int(stats[5])  # combine tasks: equal shares of every destination's tokens
        cfg = inp["cfg"]
        assert n_comb >= cfg["R"] and (cfg["T"] // cfg["R"]) % (n_comb // cfg["R"]) == 0 and n_comb % cfg["R"] == 0, stats.tolist()
    # and the static scheduler again on the same workspace
    p, buf = run_forward(B, inp, 1, 0, epoch=9, buf=buf, group_size=0, scheduler=0)
    check_against_oracle(B, inp, p, buf, 1, ref)
    assert buf.stats.cpu().numpy()[16] == 0


@pytest.mark.parametrize("E", [96, 70])
def test_megakernel_gate_many_experts_and_ties(E):
    """Gate with E >= 64 (the path that screens in bf16 and decides on exact fp64 logits of the
    candidates only).  Some rows of x are zero, so all 96 logits of those tokens are equal: more
    candidates than that path keeps, which sends the task down the exact path for all experts;
    the tie-break (lower expert first, equal weights) must come out as the oracle's.  E = 70: a row of
    the gate weights is not a whole number of 16-byte pieces."""
    B = _binding()
    cfg = dict(T=192, d=256, E=E, k=4, f=128, R=4, dtype="bf16", seed=21)
    inp = W.make_inputs(cfg)
    inp["x"][5] = 0
    inp["x"][40:44] = 0
    inp["x"][191] = 0
    for mode in (1, 0):
        print(f"case gate E={E} with ties, signal_mode {mode}", flush=True)
        p, buf = run_forward(B, inp, mode, 0)
        check_against_oracle(B, inp, p, buf, mode)
    idx = buf.topk_idx.cpu().numpy()
    assert idx[5].tolist() == [0, 1, 2, 3] and idx[191].tolist() == [0, 1, 2, 3]
    np.testing.assert_allclose(buf.topk_w.cpu().numpy()[40:44], 0.25, rtol=1e-6)


@pytest.mark.parametrize("cfg", [
    # k = E, destinations that are not whole token blocks, 64 x 128 publish tile
    dict(T=200, d=128, E=5, k=5, f=192, R=4, dtype="bf16", seed=31, tile_m=64, tile_n=128),
    # odd everything, one expert per token, fp32
    dict(T=130, d=64, E=3, k=1, f=64, R=2, dtype="f32", seed=32),
    # one destination, 32-row publish tile with many rows per expert (256-row compute tiles)
    dict(T=512, d=256, E=2, k=2, f=128, R=1, dtype="bf16", seed=33, tile_m=32),
    # more destinations than a wavefront has lanes, tiny segments
    dict(T=256, d=128, E=16, k=2, f=64, R=128, dtype="bf16", seed=34, tile_m=32),
    # three blocks of 16 tokens and a long reduction: the gate is split ten ways over the reduction
    dict(T=48, d=4096, E=24, k=3, f=128, R=3, dtype="bf16", seed=35, tile_m=32, bias_std=0.5),
    # the same in fp32 (two slices)
    dict(T=40, d=1024, E=12, k=2, f=64, R=2, dtype="f32", seed=36),
    # one expert, every token its own destination
    dict(T=16, d=64, E=1, k=1, f=64, R=16, dtype="bf16", seed=37, tile_m=32),
    # a decode-sized batch with many experts: the split gate takes precedence over the bf16 screen
    dict(T=128, d=2048, E=128, k=8, f=64, R=8, dtype="bf16", seed=40, tile_m=32, bias_std=0.5),
    # 128 blocks of 16 tokens, 64 experts: half of the workgroups get a gate task (the bf16 screen)
    dict(T=2048, d=1024, E=64, k=2, f=64, R=8, dtype="bf16", seed=41),
    # fp32 rows of h of 64 bytes: two row blocks share a cache line wherever an expert starts at an odd row
    dict(T=40, d=1024, E=200, k=2, f=16, R=1, dtype="f32", seed=43055, bias_std=0.5, tile_m=64),
    # 32 experts per token (the most the interface allows), of 40 and of 256
    dict(T=66, d=128, E=40, k=32, f=64, R=2, dtype="bf16", seed=42, tile_m=64),
    dict(T=48, d=1024, E=256, k=32, f=64, R=3, dtype="bf16", seed=43, bias_std=0.5),
    # the most destinations the interface allows, one token each
    dict(T=1024, d=64, E=16, k=2, f=64, R=1024, dtype="bf16", seed=44, tile_m=32),
    # a single token
    dict(T=1, d=128, E=4, k=2, f=64, R=1, dtype="bf16", seed=38, tile_m=32),
    # a single token, fp32
    dict(T=1, d=64, E=2, k=2, f=64, R=1, dtype="f32", seed=39),
], ids=["k_eq_E", "odd_f32", "one_dest", "many_dest", "split_gate", "split_gate_f32", "one_expert",
        "split_gate_many_experts", "gate_128_blocks", "h_rows_share_lines", "k_32_of_40", "k_32_of_256", "max_dest", "one_token", "one_token_f32"])
@pytest.mark.parametrize("signal_mode", [0, 1])
def test_megakernel_odd_shapes(cfg, signal_mode):
    B = _binding()
    print(f"case {cfg} signal_mode {signal_mode}", flush=True)
    inp = W.make_inputs(cfg)
    p, buf = run_forward(B, inp, signal_mode, 0)
    check_against_oracle(B, inp, p, buf, signal_mode)


def test_megakernel_system_scope_and_reuse():
    """Same buffers, three calls in a row with rising epochs, both scopes and
    both modes: the workspace must come back clean each time."""
    B = _binding()
    inp = W.make_inputs("mini_skew")
    print("case mini_skew reuse", flush=True)
    ref, buf = None, None
    for epoch, (mode, scope) in enumerate([(1, 1), (0, 1), (1, 0), (0, 0)], start=3):
        p, buf = run_forward(B, inp, mode, scope, epoch=epoch, buf=buf)
        ref = check_against_oracle(B, inp, p, buf, mode, ref)


@pytest.mark.parametrize("name", ["mini_f32", "mini_bf16", "mini_skew", "mini_decode"])
def test_route_parity(name):
    B = _binding()
    print(f"case route {name}", flush=True)
    inp = W.make_inputs(name, with_weights=False)
    cfg = inp["cfg"]
    p = _problem(B, cfg)
    d = _dev(inp, ("x", "Wg", "gate_bias"))
    idx = torch.empty((cfg["T"], cfg["k"]), dtype=torch.int32, device="cuda")
    w = torch.empty((cfg["T"], cfg["k"]), dtype=torch.float32, device="cuda")
    B.moe_route(p, d["x"], d["Wg"], d["gate_bias"], idx, w)
    torch.cuda.synchronize()
    ridx, rw, margin = parity.oracle_routing(inp)
    assert np.array_equal(idx.cpu().numpy(), ridx), f"min margin {margin.min()}"
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=1e-5, atol=1e-7)
    s = w.cpu().numpy().astype(np.float64).sum(axis=1)
    assert np.abs(s - 1).max() < 1e-6
    assert all(len(set(r)) == cfg["k"] for r in idx.cpu().numpy().tolist())


def test_route_equal_logits_tie_break():
    """All logits equal: the k lowest expert ids, weights 1/k (degenerate case)."""
    B = _binding()
    T, d, E, k = 32, 64, 12, 3
    p = B.problem(T, d, E, k, 64, 1, "bf16")
    x = torch.zeros((T, d), dtype=torch.bfloat16, device="cuda")
    Wg = torch.randn((d, E), device="cuda").to(torch.bfloat16)
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    w = torch.empty((T, k), dtype=torch.float32, device="cuda")
    B.moe_route(p, x, Wg, None, idx, w)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), np.tile(np.arange(k, dtype=np.int32), (T, 1)))
    np.testing.assert_allclose(w.cpu().numpy(), 1.0 / k, rtol=1e-6)


@pytest.mark.parametrize("name", ["mini_f32", "mini_bf16", "mini_skew", "mini_pre", "mini_decode"])
def test_dispatch_parity(name):
    B = _binding()
    print(f"case dispatch {name}", flush=True)
    inp = W.make_inputs(name, with_weights=False)
    cfg = inp["cfg"]
    p = _problem(B, cfg)
    ridx, _, _ = parity.oracle_routing(inp)
    buf = B.Buffers(p)
    x = inp["x"].cuda()
    idx = torch.from_numpy(ridx).cuda()
    x_perm = torch.full((cfg["T"] * cfg["k"], cfg["d"]), float("nan"), dtype=x.dtype, device="cuda")
    for rep in range(2):  # twice: the workspace must be reusable
        B.moe_dispatch(p, x, idx, buf.counts, buf.offsets, buf.perm, buf.inv_perm, x_perm, None, buf.workspace)
        torch.cuda.synchronize()
        counts, offsets, perm, inv = oracle.dispatch(ridx, cfg["E"])
        assert np.array_equal(buf.counts.cpu().numpy(), counts)
        assert np.array_equal(buf.offsets.cpu().numpy(), offsets)
        assert np.array_equal(buf.perm.cpu().numpy(), perm)
        assert np.array_equal(buf.inv_perm.cpu().numpy(), inv)
        ref_xp = oracle.gather(W.as_oracle_array(inp["x"]), perm, cfg["k"])
        assert np.array_equal(W.as_oracle_array(x_perm), ref_xp)  # byte-exact row copy
    # indices only
    B.moe_dispatch(p, None, idx, buf.counts, buf.offsets, buf.perm, buf.inv_perm, None, None, buf.workspace)
    torch.cuda.synchronize()
    assert np.array_equal(buf.perm.cpu().numpy(), perm)


def test_dispatch_empty_experts():
    """Every token picks experts 2 and 5 only: six experts stay empty."""
    B = _binding()
    T, d, E, k = 100, 64, 8, 2
    p = B.problem(T, d, E, k, 64, 4, "bf16")
    buf = B.Buffers(p)
    ridx = np.tile(np.array([[5, 2]], np.int32), (T, 1))
    B.moe_dispatch(p, None, torch.from_numpy(ridx).cuda(), buf.counts, buf.offsets, buf.perm, buf.inv_perm, None, None,
                   buf.workspace)
    torch.cuda.synchronize()
    counts, offsets, perm, inv = oracle.dispatch(ridx, E)
    assert np.array_equal(buf.counts.cpu().numpy(), counts)
    assert np.array_equal(buf.offsets.cpu().numpy(), offsets)
    assert np.array_equal(buf.perm.cpu().numpy(), perm)


@pytest.mark.parametrize("name", ["mini_bf16", "mini_skew", "mini_decode", "mini_odd", "mini_f32"])
def test_megakernel_padded_layout(name):
    """The padded layout of balanced routing (section 6.1: every expert owns `capacity` rows of the sorted
    order): same outputs, offsets = e * capacity, perm with -1 in unused rows.  Capacity = the largest
    expert's rows (nothing spare) and something larger; both signaling modes; then a capacity that is too
    small: reported, and the workspace still good for the next call."""
    B = _binding()
    inp = W.make_inputs(name)
    idx, _, _ = parity.oracle_routing(inp)
    cmax = int(np.bincount(idx.reshape(-1), minlength=inp["cfg"]["E"]).max())
    for mode, cap in [(1, cmax), (0, cmax + 37)]:
        print(f"case {name} padded layout, capacity {cap}, signal_mode {mode}", flush=True)
        p, buf = run_forward(B, inp, mode, 0, capacity=cap)
        check_against_oracle(B, inp, p, buf, mode)
    print(f"case {name} padded layout with the ready-queue scheduler and fence groups", flush=True)
    p, buf = run_forward(B, inp, 1, 0, capacity=cmax + 1, scheduler=1, group_size=7)
    check_against_oracle(B, inp, p, buf, 1)
    print(f"case {name} capacity {cmax - 1}: too small", flush=True)
    p, buf = run_forward(B, inp, 1, 0, capacity=cmax - 1)
    assert int(buf.stats.cpu().numpy()[7]) == B.MOE_ERR_CAPACITY
    assert np.array_equal(buf.counts.cpu().numpy(), np.bincount(idx.reshape(-1), minlength=inp["cfg"]["E"]))
    # the same buffers again, with routing given that fits: the failed call left the workspace usable
    T, k, E = inp["cfg"]["T"], inp["cfg"]["k"], inp["cfg"]["E"]
    if T * k % E == 0 and T * k // E <= cmax - 1:
        inp2 = dict(inp)
        inp2["cfg"] = dict(inp["cfg"], prerouted=dict(kind="given"))
        inp2["Wg"], inp2["gate_bias"] = None, None
        inp2["topk_idx"] = ((torch.arange(T)[:, None] * k + torch.arange(k)[None, :]) % E).to(torch.int32)
        inp2["topk_w"] = torch.full((T, k), 1.0 / k)
        p, buf = run_forward(B, inp2, 1, 0, epoch=2, buf=buf, capacity=cmax - 1)
        check_against_oracle(B, inp2, p, buf, 1)


@pytest.mark.parametrize("name", ["mini_bf16", "mini_decode"])
def test_dispatch_padded_layout(name):
    B = _binding()
    inp = W.make_inputs(name, with_weights=False)
    cfg = inp["cfg"]
    ridx, _, _ = parity.oracle_routing(inp)
    cmax = int(np.bincount(ridx.reshape(-1), minlength=cfg["E"]).max())
    x = inp["x"].cuda()
    idx = torch.from_numpy(ridx).cuda()
    for cap in (cmax, cmax + 5):
        print(f"case dispatch {name} capacity {cap}", flush=True)
        p = _problem(B, cfg, capacity=cap)
        buf = B.Buffers(p)
        x_perm = torch.full((cfg["E"] * cap, cfg["d"]), float("nan"), dtype=x.dtype, device="cuda")
        B.moe_dispatch(p, x, idx, buf.counts, buf.offsets, buf.perm, buf.inv_perm, x_perm, None, buf.workspace)
        torch.cuda.synchronize()
        counts, offsets, perm, inv = oracle.dispatch(ridx, cfg["E"], capacity=cap)
        assert np.array_equal(buf.counts.cpu().numpy(), counts)
        assert np.array_equal(buf.offsets.cpu().numpy(), offsets)
        assert np.array_equal(buf.perm.cpu().numpy(), perm)
        assert np.array_equal(buf.inv_perm.cpu().numpy(), inv)
        assert np.array_equal(W.as_oracle_array(x_perm), oracle.gather(W.as_oracle_array(inp["x"]), perm, cfg["k"]))
    # too small: counts are exact, nothing else is written
    p = _problem(B, cfg, capacity=cmax - 1)
    buf = B.Buffers(p)
    buf.perm.fill_(-7)
    x_perm = torch.full((cfg["E"] * (cmax - 1), cfg["d"]), 3.0, dtype=x.dtype, device="cuda")
    B.moe_dispatch(p, x, idx, buf.counts, buf.offsets, buf.perm, buf.inv_perm, x_perm, None, buf.workspace)
    torch.cuda.synchronize()
    assert np.array_equal(buf.counts.cpu().numpy(), counts)
    assert (buf.perm == -7).all().item() and (x_perm == 3.0).all().item()


def test_dispatch_many_blocks_and_experts():
    """Indices only, at a size whose block histograms (T/64 x E) do not fit the short form's LDS: the
    form with the single-workgroup plan runs.  Random distinct experts per token, seeded."""
    B = _binding()
    T, d, E, k = 8192, 64, 256, 4
    p = B.problem(T, d, E, k, 64, 8, "bf16")
    buf = B.Buffers(p)
    g = torch.Generator().manual_seed(77)
    ridx = torch.rand((T, E), generator=g).argsort(dim=1)[:, :k].to(torch.int32).contiguous()
    for rep in range(2):
        B.moe_dispatch(p, None, ridx.cuda(), buf.counts, buf.offsets, buf.perm, buf.inv_perm, None, None, buf.workspace)
        torch.cuda.synchronize()
        counts, offsets, perm, inv = oracle.dispatch(ridx.numpy(), E)
        assert np.array_equal(buf.counts.cpu().numpy(), counts)
        assert np.array_equal(buf.offsets.cpu().numpy(), offsets)
        assert np.array_equal(buf.perm.cpu().numpy(), perm)
        assert np.array_equal(buf.inv_perm.cpu().numpy(), inv)
    # the padded layout through the same form
    cap = int(counts.max()) + 1
    p = B.problem(T, d, E, k, 64, 8, "bf16", capacity=cap)
    buf = B.Buffers(p)
    B.moe_dispatch(p, None, ridx.cuda(), buf.counts, buf.offsets, buf.perm, buf.inv_perm, None, None, buf.workspace)
    torch.cuda.synchronize()
    counts, offsets, perm, inv = oracle.dispatch(ridx.numpy(), E, capacity=cap)
    assert np.array_equal(buf.offsets.cpu().numpy(), offsets)
    assert np.array_equal(buf.perm.cpu().numpy(), perm)
    assert np.array_equal(buf.inv_perm.cpu().numpy(), inv)


def test_dispatch_then_megakernel_share_a_workspace():
    """A standalone dispatch between two passes of the megakernel on the same buffers leaves the
    workspace as the megakernel needs it."""
    B = _binding()
    inp = W.make_inputs("mini_skew")
    p, buf = run_forward(B, inp, 1, 0, epoch=1)
    ref = check_against_oracle(B, inp, p, buf, 1)
    idx = buf.topk_idx.clone()
    B.moe_dispatch(p, inp["x"].cuda(), idx, buf.counts, buf.offsets, buf.perm, buf.inv_perm, None, None, buf.workspace)
    torch.cuda.synchronize()
    assert np.array_equal(buf.perm.cpu().numpy(), ref["perm"])
    p, buf = run_forward(B, inp, 0, 0, epoch=2, buf=buf)
    check_against_oracle(B, inp, p, buf, 0, ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_combine_identity_experts_return_x(dtype):
    """Every chosen expert returns the token itself => out = x (combine alone)."""
    B = _binding()
    T, d, E, k = 192, 512, 8, 4
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    p = B.problem(T, d, E, k, 64, 4, dtype)
    g = torch.Generator().manual_seed(5)
    x = torch.randn((T, d), generator=g).to(tdt)
    wraw = torch.rand((T, k), generator=g) + 0.1
    w = (wraw / wraw.sum(dim=1, keepdim=True)).float()
    staging = x.repeat_interleave(k, dim=0).contiguous()
    out = torch.empty((T, d), dtype=tdt, device="cuda")
    B.moe_combine(p, staging.cuda(), None, None, w.cuda(), out, None)
    torch.cuda.synchronize()
    ref = oracle.combine(staging.float().numpy(), w.numpy())
    got = out.float().cpu().numpy()
    tol = 1e-6 if dtype == "f32" else 2.0 ** -8
    assert np.abs(got - ref).max() <= tol * np.abs(ref).max()
    assert np.abs(got - x.float().numpy()).max() <= (2e-6 if dtype == "f32" else 2.0 ** -7) * np.abs(ref).max()


def test_combine_reports_missing_flag():
    B = _binding()
    T, d, E, k = 64, 256, 4, 2
    p = B.problem(T, d, E, k, 64, 2, "bf16", epoch=9)
    ncb = d // 64
    staging = torch.zeros((T * k, d), dtype=torch.bfloat16, device="cuda")
    w = torch.full((T, k), 0.5, device="cuda")
    out = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    slot_flag = (torch.arange(T * k, dtype=torch.int32, device="cuda") * ncb).contiguous()
    flags = torch.full((T * k * ncb,), 9, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.moe_combine(p, staging, flags, slot_flag, w, out, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    flags[37] = 8  # one tile of the previous epoch
    B.moe_combine(p, staging, flags, slot_flag, w, out, status)
    torch.cuda.synchronize()
    assert int(status.item()) == B.MOE_ERR_NOT_READY


def test_bad_routing_is_reported_not_followed():
    """An expert id outside [0, E) in precomputed routing: device status says
    so and nothing is written out of bounds (the call still terminates)."""
    B = _binding()
    inp = W.make_inputs("mini_pre")
    inp["topk_idx"] = inp["topk_idx"].clone()
    inp["topk_idx"][17, 0] = 99
    p, buf = run_forward(B, inp, 1, 0)
    assert int(buf.stats.cpu().numpy()[7]) == B.MOE_ERR_BAD_ROUTING
    # the workspace is clean again: a good call right after works
    good = W.make_inputs("mini_pre")
    p, buf = run_forward(B, good, 1, 0, epoch=2, buf=buf)
    check_against_oracle(B, good, p, buf, 1)


def test_dispatch_reports_bad_routing_and_gathers_nothing():
    """moe_dispatch alone with one expert id outside [0, E): the status says so, counts leave the slot out,
    and neither perm nor x_perm is written (x_perm keeps its poison), in the short form (block histograms) and
    in the long one (histograms too large for one workgroup's LDS: the plan form)."""
    B = _binding()
    cases = [("short", dict(T=256, d=256, E=8, k=2, f=64, R=4, dtype="bf16", seed=71)),
             ("long", dict(T=8192, d=64, E=200, k=2, f=64, R=4, dtype="bf16", seed=72))]
    for form, cfg in cases:
        print(f"case bad id, {form} form", flush=True)
        cfg = W.config(cfg)
        inp = W.make_inputs(cfg, with_weights=False)
        T, d, E, k = cfg["T"], cfg["d"], cfg["E"], cfg["k"]
        r = np.random.default_rng(cfg["seed"])
        ridx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
        good = ridx.copy()
        ridx[T // 3, 1] = E + 5
        p = _problem(B, cfg)
        buf = B.Buffers(p)
        x = inp["x"].cuda()
        x_perm = torch.full((T * k, d), float("nan"), dtype=x.dtype, device="cuda")
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        buf.perm.fill_(-7)
        B.moe_dispatch(p, x, torch.from_numpy(ridx).cuda(), buf.counts, buf.offsets, buf.perm, buf.inv_perm, x_perm,
                       status, buf.workspace)
        torch.cuda.synchronize()
        assert int(status.item()) == B.MOE_ERR_BAD_ROUTING, (form, int(status.item()))
        want = np.bincount(ridx.reshape(-1)[ridx.reshape(-1) < E], minlength=E)
        assert np.array_equal(buf.counts.cpu().numpy(), want)
        assert torch.isnan(x_perm).all().item(), "rows were gathered although the routing is invalid"
        # the same buffers and workspace right after, valid routing: status untouched, result right
        status.zero_()
        B.moe_dispatch(p, x, torch.from_numpy(good).cuda(), buf.counts, buf.offsets, buf.perm, buf.inv_perm, x_perm,
                       status, buf.workspace)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        counts, offsets, perm, inv = oracle.dispatch(good, E)
        assert np.array_equal(buf.counts.cpu().numpy(), counts) and np.array_equal(buf.perm.cpu().numpy(), perm)
        assert np.array_equal(buf.inv_perm.cpu().numpy(), inv)
        xp = oracle.gather(W.as_oracle_array(inp["x"]), perm, k)
        assert np.array_equal(x_perm.cpu().view(torch.uint16).numpy(), xp)
    # over capacity (padded layout) is reported the same way
    cfg = W.config(cases[0][1])
    p = _problem(B, cfg, capacity=8)
    buf = B.Buffers(p)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    skew = np.zeros((cfg["T"], cfg["k"]), np.int32)
    skew[:, 1] = 1
    B.moe_dispatch(p, None, torch.from_numpy(skew).cuda(), buf.counts, buf.offsets, buf.perm, buf.inv_perm, None, status,
                   buf.workspace)
    torch.cuda.synchronize()
    assert int(status.item()) == B.MOE_ERR_CAPACITY


def test_epoch_reuse_needs_zeroed_flags():
    """Epochs 1, 2, then 1 again with other routing, on one set of buffers: legal only because the flags are zeroed
    before the value is reused (a flag the second call set and the third does not publish would otherwise still say
    2, and one the first call set would read as ready).  Every call is checked in full, flags beyond those in use
    included."""
    B = _binding()
    a = W.make_inputs("mini_skew")
    b = W.make_inputs(dict(W.CONFIGS["mini_skew"], seed=113, bias_std=0.2))
    p, buf = run_forward(B, a, 1, 0, epoch=1)
    check_against_oracle(B, a, p, buf, 1)
    p, buf = run_forward(B, b, 1, 0, epoch=2, buf=buf)
    check_against_oracle(B, b, p, buf, 1)
    buf.flags.zero_()
    p, buf = run_forward(B, a, 0, 0, epoch=1, buf=buf)
    check_against_oracle(B, a, p, buf, 0)
    idx, _, _ = parity.oracle_routing(a)
    _, offsets, _, inv = oracle.dispatch(idx, a["cfg"]["E"])
    nfl = oracle.publish_plan(idx, offsets, inv, a["cfg"]["E"], a["cfg"]["R"], a["cfg"]["d"], a["cfg"]["tile_m"],
                              a["cfg"]["tile_n"])["n_flags"]
    assert not buf.flags[nfl:].any().item(), "a flag outside the tiles of this call was touched"


def _random_cases(seed, n):
    """Seeded draw of small valid problems with a random mix of options."""
    import random
    rng = random.Random(seed)
    for case in range(n):
        dtype = rng.choice(["bf16", "bf16", "f32"])
        step = 64 if dtype == "bf16" else 16
        R = rng.choice([1, 1, 2, 3, 4, 5, 8, 16])
        per = rng.choice([1, 2, 7, 16, 33, 64, 100, 129])
        if dtype == "f32":
            per = min(per, 40)
        T = R * per
        E = rng.choice([1, 2, 3, 5, 8, 13, 16, 31, 32, 33, 64, 65, 100, 128])
        k = rng.randint(1, min(E, 8))
        d = step * rng.randint(1, 6 if dtype == "bf16" else 12)
        f = step * rng.randint(1, 7 if dtype == "bf16" else 10)
        tile_m, tile_n = rng.choice([0, 32, 64, 128]), rng.choice([0, 64, 128])
        cfg = dict(T=T, d=d, E=E, k=k, f=f, R=R, dtype=dtype, seed=1000 * seed + case, bias_std=rng.choice([0.0, 0.5, 2.0]))
        if tile_m:
            cfg["tile_m"] = tile_m
        if tile_n:
            cfg["tile_n"] = tile_n
        mode = rng.choice([0, 1])
        g = rng.choice([0, 0, 1, 3, 50]) if mode == 1 else 0
        yield cfg, mode, g, rng.choice([0, 1]), rng.choice([0, 0, T])


def test_megakernel_random_shapes():
    """Forty seeded random problems (token counts that are no multiple of anything, 1 to 128 experts,
    k up to 8, every publish tile, both dtypes) with random signaling mode, fence group size, scheduler
    and layout, each run twice on its buffers and checked against the oracle like every other case.
    The one combination the library declines (fp32 with a 128-column publish tile: its compute tiles
    are 64 columns wide) must be declined on the host."""
    B = _binding()
    ran = 0
    for cfg, mode, g, sched, cap in _random_cases(2, 40):
        print(f"case {cfg} signal_mode {mode} group_size {g} scheduler {sched} capacity {cap}", flush=True)
        inp = W.make_inputs(cfg)
        p = _problem(B, inp["cfg"], mode, 0, 1, g, sched, cap)
        if cfg["dtype"] == "f32" and cfg.get("tile_n") == 128:
            with pytest.raises(Exception, match="unsupported"):
                B.Buffers(p)
            continue
        buf, ref = B.Buffers(p), None
        for epoch in (1, 2):
            p, buf = run_forward(B, inp, mode, 0, epoch=epoch, buf=buf, group_size=g, scheduler=sched, capacity=cap)
            ref = check_against_oracle(B, inp, p, buf, mode, ref)
        ran += 1
    assert ran >= 30


def test_standalone_entry_points_random_shapes():
    """Thirty seeded random problems through moe_route, moe_dispatch (the oracle's routing or a skewed one
    that leaves experts empty; ragged and padded layout; with and without the row gather; twice on one
    workspace) and moe_combine, against the oracle."""
    import random
    B = _binding()
    rng = random.Random(7)
    for case in range(30):
        dtype = rng.choice(["bf16", "bf16", "f32"])
        step = 64 if dtype == "bf16" else 16
        R = rng.choice([1, 2, 3, 4, 8, 16])
        T = R * rng.choice([1, 2, 7, 16, 33, 64, 100, 129, 500, 1111])
        E = rng.choice([1, 2, 3, 5, 8, 13, 16, 31, 32, 33, 64, 65, 70, 100, 128, 200, 256])
        k = rng.randint(1, min(E, 8))
        d = step * rng.randint(1, 8 if dtype == "bf16" else 16)
        cfg = dict(T=T, d=d, E=E, k=k, f=64, R=R, dtype=dtype, seed=7000 + case, bias_std=rng.choice([0.0, 0.5, 2.0]))
        print(f"case {cfg}", flush=True)
        inp = W.make_inputs(cfg, with_weights=False)
        p = _problem(B, inp["cfg"])
        dv = _dev(inp, ("x", "Wg", "gate_bias"))
        idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
        w = torch.empty((T, k), dtype=torch.float32, device="cuda")
        B.moe_route(p, dv["x"], dv["Wg"], dv["gate_bias"], idx, w)
        torch.cuda.synchronize()
        ridx, rw, margin = parity.oracle_routing(inp)
        assert np.array_equal(idx.cpu().numpy(), ridx), f"min margin {margin.min()}"
        np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=1e-5, atol=1e-7)
        if rng.random() < 0.5 and E > k:  # a few experts take every row
            hot = rng.sample(range(E), min(E, k + rng.randint(0, 2)))
            sel = torch.rand((T, len(hot)), generator=torch.Generator().manual_seed(case)).argsort(dim=1)[:, :k]
            ridx = np.ascontiguousarray(torch.tensor(hot, dtype=torch.int32)[sel].numpy())
        cmax = int(np.bincount(ridx.reshape(-1), minlength=E).max())
        for cap in (0, rng.choice([cmax, cmax + 3])):
            pc = _problem(B, inp["cfg"], capacity=cap)
            buf = B.Buffers(pc)
            with_x = rng.random() < 0.7
            x_perm = (torch.full((E * cap if cap else T * k, d), float("nan"), dtype=dv["x"].dtype, device="cuda")
                      if with_x else None)
            counts, offsets, perm, inv = oracle.dispatch(ridx, E, capacity=cap)
            for rep in range(2):
                B.moe_dispatch(pc, dv["x"] if with_x else None, torch.from_numpy(ridx).cuda(), buf.counts, buf.offsets,
                               buf.perm, buf.inv_perm, x_perm, None, buf.workspace)
                torch.cuda.synchronize()
                assert np.array_equal(buf.counts.cpu().numpy(), counts)
                assert np.array_equal(buf.offsets.cpu().numpy(), offsets)
                assert np.array_equal(buf.perm.cpu().numpy(), perm)
                assert np.array_equal(buf.inv_perm.cpu().numpy(), inv)
                if with_x:
                    assert np.array_equal(W.as_oracle_array(x_perm), oracle.gather(W.as_oracle_array(inp["x"]), perm, k))
        staging = torch.randn((T * k, d), generator=torch.Generator().manual_seed(100 + case)).to(dv["x"].dtype)
        out = torch.empty((T, d), dtype=dv["x"].dtype, device="cuda")
        wt = torch.from_numpy(rw).float()
        B.moe_combine(p, staging.cuda(), None, None, wt.cuda(), out, None)
        torch.cuda.synchronize()
        ref = oracle.combine(staging.float().numpy(), wt.numpy())
        tol = 1e-6 if dtype == "f32" else 2.0 ** -8  # one rounding of the fp32 sum to the output type
        assert np.all(np.abs(out.float().cpu().numpy() - ref) <= tol * np.maximum(np.abs(ref), 1e-3) + 1e-7)


@pytest.mark.parametrize("scheduler", [0, 1])
def test_repeat_launches_are_bit_identical(scheduler):
    """Every sum in the path has a fixed order, so a launch repeated on the same inputs must reproduce
    staging, out, routing and permutation bit for bit, on reused and on fresh buffers: a race between
    workgroups would show as a difference."""
    B = _binding()
    cases = ["mini_skew", "mini_odd",
             dict(T=40, d=1024, E=200, k=2, f=16, R=1, dtype="f32", seed=43055, bias_std=0.5, tile_m=64),
             dict(T=128, d=2048, E=128, k=8, f=64, R=8, dtype="bf16", seed=40, tile_m=32, bias_std=0.5)]
    names = ("staging", "out", "perm", "inv_perm", "topk_idx", "topk_w", "slot_flag")
    for c in cases:
        print(f"case {c} scheduler {scheduler}", flush=True)
        inp = W.make_inputs(c)
        p, buf = run_forward(B, inp, 1, 0, epoch=1, scheduler=scheduler)
        check_against_oracle(B, inp, p, buf, 1)
        ref = {n: getattr(buf, n).clone() for n in names}
        for rep in range(12):
            p, buf = run_forward(B, inp, 1, 0, epoch=2 + rep, buf=None if rep % 4 == 3 else buf, scheduler=scheduler)
            assert int(buf.stats.cpu().numpy()[7]) == 0
            for n in names:
                assert torch.equal(getattr(buf, n).view(torch.uint8), ref[n].view(torch.uint8)), (c, rep, n)


@pytest.mark.parametrize("scheduler", [0, 1])
def test_expired_waits_drain_the_kernel(scheduler):
    """The time-out path, forced from the host: a call whose bound of the in-kernel waits is one tick
    (moe_problem_t.wait_ticks; nothing global changes): the plan's wait for the gate gives up, the error spreads,
    every workgroup leaves in the ordinary way and the call reports MOE_ERR_TIMEOUT.  With the workspace
    initialised again, the same buffers give the right result in a call with the default bound."""
    B = _binding()
    inp = W.make_inputs("mini_bf16")
    p, buf = run_forward(B, inp, 1, 0, epoch=1, scheduler=scheduler)
    ref = check_against_oracle(B, inp, p, buf, 1)
    print(f"case mini_bf16 scheduler {scheduler}, wait limit 1 tick", flush=True)
    p, buf = run_forward(B, inp, 1, 0, epoch=2, buf=buf, scheduler=scheduler, wait_ticks=1)
    stats = buf.stats.cpu().numpy()
    assert int(stats[7]) == B.MOE_ERR_TIMEOUT and stats[6] > 0, stats.tolist()
    B.moe_workspace_init(p, buf.workspace)
    buf.flags.zero_()
    p, buf = run_forward(B, inp, 1, 0, epoch=3, buf=buf, scheduler=scheduler)
    check_against_oracle(B, inp, p, buf, 1, ref)


def test_probe_mfma_runs_and_keeps_its_work():
    """The measurement aid: launches, writes one float per thread, and the sums are what 16 products per round of the
    given fragments add up to (all-ones operands: every accumulator element gains 16 per product)."""
    B = _binding()
    frag = torch.ones(4096, dtype=torch.bfloat16, device="cuda")
    sink = torch.full((8 * 256,), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_probe_mfma(frag, 3, 8, sink)
    torch.cuda.synchronize()
    # a lane holds 16 accumulator values of each of the 16 independent products; each value = rounds * K(16) * 1 * 1
    assert torch.equal(sink, torch.full_like(sink, 3 * 16.0 * 16 * 16))
    with pytest.raises(B.MoeError):
        B.moe_probe_mfma(frag, 0, 8, sink)


def test_megakernel_replayed_from_a_captured_graph():
    """A serving loop launches the layer from a captured HIP graph: the library only launches kernels on the stream it
    is given (no allocation, no memset, no synchronisation; kernel attributes are set by the first eager call), and the
    megakernel leaves its workspace ready for the next launch.  The graph holds what one step needs: flags cleared
    by a fill kernel (the epoch is baked into the captured launch), outputs poisoned, one forward.  Every replay,
    with eager launches and synchronisations of the program's own in between, must reproduce the eager result bit
    for bit."""
    B = _binding()
    inp = W.make_inputs("mini_bf16")
    cfg = inp["cfg"]
    d = _dev(inp, ("x", "Wg", "gate_bias", "W1", "W3", "W2"))
    p, buf = run_forward(B, inp, 1, 0, epoch=5)  # eager: reference result, and the one-time host-side set-up
    check_against_oracle(B, inp, p, buf, 1)
    want = {n: getattr(buf, n).clone() for n in ("out", "staging", "topk_idx", "perm", "counts")}
    other = B.Buffers(p)  # the program's own eager work between replays uses other buffers
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        buf.flags.zero_()
        buf.staging.fill_(float("nan"))
        buf.out.fill_(float("nan"))
        B.forward(p, buf, d["x"], d["Wg"], d["gate_bias"], d["W1"], d["W3"], d["W2"])
    torch.cuda.synchronize()
    for rep in range(4):
        print(f"case graph replay {rep}", flush=True)
        buf.out.fill_(0.25)  # whatever the last replay left must not be what this one is checked on
        buf.perm.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        for n, ref in want.items():
            got = getattr(buf, n)
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), (rep, n)
        assert int(buf.stats[7].item()) == 0
        p2 = _problem(B, cfg, 1, 0, epoch=100 + rep)
        other.flags.zero_()
        B.forward(p2, other, d["x"], d["Wg"], d["gate_bias"], d["W1"], d["W3"], d["W2"])
        torch.cuda.synchronize()
        assert torch.equal(other.out.view(torch.uint8), want["out"].view(torch.uint8))


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("to_lds", [0, 1])
def test_probe_stream_reads_what_it_says(waves, to_lds):
    """The streaming measurement aid reads exactly the pieces its contract names: the word a thread leaves in `sink`
    is rebuilt on the CPU from the buffer (register form: XOR of every word the lane loaded; LDS form: XOR of the
    four words that ended up at byte 16 * thread of the workgroup's LDS, i.e. of a piece of the last batch)."""
    B = _binding()
    span, stride, wgs, depth = 1 << 20, 4096 + 48, 5, 8
    per_wg = waves * 1024 * (3 * depth + 5)  # rounds down to three batches of eight loads per wavefront
    rng = np.random.default_rng(17)
    host = rng.integers(0, 1 << 32, size=span // 4, dtype=np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).cuda()
    nt = waves * 64
    sink = torch.full((wgs * nt,), -1, dtype=torch.int32, device="cuda")
    B.moe_probe_stream(buf, span, stride, per_wg, wgs, waves, to_lds, sink)
    torch.cuda.synchronize()
    got = sink.cpu().numpy().view(np.uint32).reshape(wgs, nt)
    n_instr = 3 * depth

    def piece(off):  # XOR of the four words at byte offset off
        w = host[off // 4: off // 4 + 4]
        return int(w[0] ^ w[1] ^ w[2] ^ w[3])

    for w in range(wgs):
        start = (w * stride) % span
        for tid in range(nt):
            if to_lds:
                at = tid * 16  # byte of the workgroup's LDS: ring of wavefront at // 8192, load at % 8192 // 1024 of a batch
                wave, u, lane = at // (depth * 1024), (at % (depth * 1024)) // 1024, (at % 1024) // 16
                want = piece((start + (n_instr - depth + u) * waves * 1024 + wave * 1024 + lane * 16) % span)
            else:
                wave, lane = tid // 64, tid % 64
                want = 0
                for i in range(n_instr):
                    want ^= piece((start + i * waves * 1024 + wave * 1024 + lane * 16) % span)
            assert int(got[w, tid]) == want, (w, tid)
    for bad in (dict(waves=3), dict(span=span + 8), dict(stride=8), dict(span=1024)):
        with pytest.raises(B.MoeError):
            B.moe_probe_stream(buf, bad.get("span", span), bad.get("stride", stride), per_wg, wgs, bad.get("waves", waves),
                               to_lds, sink)


@pytest.mark.parametrize("name,tile_m", [("mini_decode", 32), ("mini_bf16", 64), ("mini_skew", 64), ("mini_skew", 32),
                                         ("mini_odd", 64), ("mini_pre", 32), ("mini_large", 64)])
@pytest.mark.parametrize("signal_mode", [0, 1])
def test_megakernel_fused_ffn(name, tile_m, signal_mode):
    """The fused FFN (a workgroup takes a row block through both GEMMs, h stays in LDS): same results as the
    oracle to the same bars, both row-block heights, both signaling modes, reused buffers; and bit-identical
    staging and out to the unfused path (same products, same order of accumulation per element)."""
    B = _binding()
    inp = W.make_inputs(dict(W.CONFIGS[name], tile_m=tile_m))
    print(f"case fused {name} tile_m {tile_m} mode {signal_mode}", flush=True)
    p, buf = run_forward(B, inp, signal_mode, 0, fuse_ffn=1)
    ref = check_against_oracle(B, inp, p, buf, signal_mode)
    st, out = buf.staging.clone(), buf.out.clone()
    p, buf = run_forward(B, inp, signal_mode, 0, epoch=2, buf=buf, fuse_ffn=1)
    check_against_oracle(B, inp, p, buf, signal_mode, ref)
    p, buf = run_forward(B, inp, signal_mode, 0, epoch=3, buf=buf, fuse_ffn=0)
    check_against_oracle(B, inp, p, buf, signal_mode, ref)
    assert torch.equal(buf.staging.view(torch.int16), st.view(torch.int16)) and torch.equal(buf.out.view(torch.int16), out.view(torch.int16))


def test_fused_ffn_limits():
    B = _binding()
    # declined when the problem is planned: publish tile taller than the row block, ready-queue scheduler, fp32
    for kw in (dict(tile_m=128), dict(tile_m=32, scheduler=1), dict(tile_m=32, dtype="f32")):
        p = B.problem(128, 1024, 16, 4, 512, 8, kw.get("dtype", "bf16"), tile_m=kw["tile_m"], scheduler=kw.get("scheduler", 0),
                      fuse_ffn=1)
        assert B.moe_workspace_bytes(p) == 0, kw
    # declined at the launch: h of a row block (32 rows x 2048) does not fit the LDS beside the stage buffers
    p = B.problem(128, 1024, 16, 4, 2048, 8, "bf16", tile_m=32, fuse_ffn=1)
    buf = B.Buffers(p)
    x = torch.zeros((128, 1024), dtype=torch.bfloat16, device="cuda")
    Wg = torch.zeros((1024, 16), dtype=torch.bfloat16, device="cuda")
    W1 = torch.zeros((16, 1024, 2048), dtype=torch.bfloat16, device="cuda")
    W2 = torch.zeros((16, 2048, 1024), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.MoeError) as e:
        B.forward(p, buf, x, Wg, None, W1, W1, W2)
    assert e.value.status == B.MOE_ERR_UNSUPPORTED
