"""The entry point that allocates nothing (moe_dispatch_noalloc: scratch in a static device array of the
library) against moe_dispatch (scratch in the caller's workspace), through the C ABI: two calls in a row, the
second with a smaller input, bit for bit; and its size limit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_00686_amd import workloads as W

pytestmark = pytest.mark.gpu


def _routing(T, E, k, seed):
    r = np.random.default_rng(seed)
    return np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)


def _both(B, cfg, seed):
    cfg = W.config(cfg)
    T, d, E, k = cfg["T"], cfg["d"], cfg["E"], cfg["k"]
    p = B.problem(T, d, E, k, cfg["f"], cfg["R"], cfg["dtype"])
    x = W.make_inputs(cfg, with_weights=False)["x"].cuda()
    idx = torch.from_numpy(_routing(T, E, k, seed)).cuda()
    buf = B.Buffers(p)  # workspace for the reference call only
    N = T * k
    i32 = dict(dtype=torch.int32, device="cuda")
    got = dict(counts=torch.full((E,), -1, **i32), offsets=torch.full((E + 1,), -1, **i32),
               perm=torch.full((N,), -1, **i32), inv_perm=torch.full((N,), -1, **i32),
               x_perm=torch.full((N, d), float("nan"), dtype=x.dtype, device="cuda"))
    ref_xp = torch.full((N, d), float("nan"), dtype=x.dtype, device="cuda")
    status = torch.zeros(1, **i32)
    torch.cuda.synchronize()
    print(f"case no-alloc dispatch T={T} E={E} k={k} d={d}", flush=True)
    B.moe_dispatch_noalloc(p, x, idx, got["counts"], got["offsets"], got["perm"], got["inv_perm"], got["x_perm"], status)
    torch.cuda.synchronize()
    B.moe_dispatch(p, x, idx, buf.counts, buf.offsets, buf.perm, buf.inv_perm, ref_xp, None, buf.workspace)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    for name, ref in (("counts", buf.counts), ("offsets", buf.offsets), ("perm", buf.perm), ("inv_perm", buf.inv_perm)):
        assert torch.equal(got[name], ref), name
    assert torch.equal(got["x_perm"].view(torch.uint8), ref_xp.view(torch.uint8))
    # and both against the oracle's stable counting sort
    counts, offsets, perm, inv = oracle.dispatch(idx.cpu().numpy(), E)
    assert np.array_equal(got["perm"].cpu().numpy(), perm) and np.array_equal(got["counts"].cpu().numpy(), counts)


def test_noalloc_dispatch_two_calls_second_smaller():
    from paper_2605_00686_amd import binding as B
    # the first two are large enough for the form of the dispatch that keeps block histograms in the scratch
    # array (T*k slots x T/16 workgroups above 64 Mi); the array keeps the first call's data for the second
    _both(B, dict(T=32768, d=64, E=8, k=8, f=64, R=8, dtype="bf16", seed=201), 1)
    _both(B, dict(T=16384, d=128, E=8, k=8, f=64, R=4, dtype="bf16", seed=202), 2)
    _both(B, dict(T=7680, d=64, E=128, k=32, f=64, R=4, dtype="bf16", seed=204), 4)
    # small problems take the single-launch form, which needs no scratch at all
    _both(B, dict(T=320, d=256, E=24, k=3, f=64, R=4, dtype="bf16", seed=205), 5)
    _both(B, dict(T=1000, d=64, E=8, k=2, f=64, R=4, dtype="f32", seed=203), 3)


def test_noalloc_dispatch_rejects_sizes_beyond_its_scratch():
    from paper_2605_00686_amd import binding as B
    p = B.problem(16384, 64, 128, 2, 64, 8, "bf16")  # 256 blocks x 128 experts: histograms of 128 KB
    i32 = dict(dtype=torch.int32, device="cuda")
    z = torch.zeros(16384 * 2, **i32)
    with pytest.raises(B.MoeError) as e:
        B.moe_dispatch_noalloc(p, None, z, z, z, z, z, None, None)
    assert e.value.status == B.MOE_ERR_UNSUPPORTED
