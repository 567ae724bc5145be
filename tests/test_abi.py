"""Host-only checks of the C ABI: the library loads, exports every function
include/moe.h declares, and rejects bad problems before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2605_00686_amd", "libmoe_hip.so")


@pytest.fixture(scope="module")
def B():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    from paper_2605_00686_amd import binding
    return binding


def declared_functions():
    src = open(os.path.join(ROOT, "include", "moe.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(B):
    names = declared_functions()
    assert set(names) == set(B.EXPORTS), names
    lib = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(B):
    seen = {B.status_string(s) for s in range(0, -8, -1)}
    assert len(seen) == 8 and "ok" in seen
    assert B.status_string(-99) == "unknown status"


def test_workspace_and_flag_sizes(B):
    p = B.problem(4096, 2048, 128, 8, 768, 8, "bf16")
    ws = B.moe_workspace_bytes(p)
    assert ws >= 4096 * 8 * 768 * 2  # holds h[N, f]
    assert ws % 256 == 0
    # (ceil(N / tile_m) + E*R) * ceil(d / tile_n) with the default 128 x 64 tile
    assert B.moe_num_flags(p) == (256 + 1024) * 32
    p5 = B.problem(128, 7168, 32, 8, 2048, 64, "bf16", tile_m=32)
    assert B.moe_num_flags(p5) == (32 + 2048) * 112
    # one workspace serves every signaling mode, fence granularity and scheduler of a problem shape
    for kw in (dict(signal_mode=0), dict(group_size=1), dict(group_size=64), dict(scheduler=1), dict(fence_scope=1)):
        assert B.moe_workspace_bytes(B.problem(4096, 2048, 128, 8, 768, 8, "bf16", **kw)) == ws, kw
    # the padded layout holds E * capacity rows of h instead of N
    wc = B.moe_workspace_bytes(B.problem(4096, 2048, 128, 8, 768, 8, "bf16", capacity=512))
    assert wc - ws == (128 * 512 - 4096 * 8) * 768 * 2


@pytest.mark.parametrize("kw", [dict(k=9, E=8), dict(T=100, R=8), dict(T=0), dict(dtype=5), dict(signal_mode=3),
                                dict(fence_scope=2), dict(tile_m=-1), dict(group_size=-1, signal_mode=1),
                                dict(group_size=4, signal_mode=0), dict(scheduler=2), dict(scheduler=-1), dict(capacity=-1)])
def test_invalid_problems_are_rejected_on_the_host(B, kw):
    base = dict(T=256, d=512, E=8, k=2, f=1024, R=2, dtype=1)
    base.update(kw)
    p = B.MoeProblem(base["T"], base["d"], base["E"], base["k"], base["f"], base["R"], base["dtype"],
                     base.get("tile_m", 0), 0, base.get("signal_mode", 0), base.get("fence_scope", 0), 1,
                     base.get("group_size", 0), base.get("scheduler", 0), base.get("capacity", 0))
    assert B.moe_workspace_bytes(p) == 0 and B.moe_num_flags(p) == 0
    lib = ctypes.CDLL(LIB)
    rc = lib.moe_route(ctypes.byref(p), None, None, None, None, None, None)
    assert rc == B.MOE_ERR_INVALID_ARG


@pytest.mark.parametrize("kw", [dict(d=100), dict(tile_m=48), dict(tile_n=32), dict(E=300, k=2), dict(E=64, k=33), dict(T=2048, R=2048),
                                # fp32 compute tiles are 64 columns wide: a 128-column publish tile would span two
                                dict(dtype=0, tile_n=128)])
def test_unsupported_problems(B, kw):
    base = dict(T=256, d=512, E=8, k=2, f=1024, R=2, tile_m=0, tile_n=0)
    base.update(kw)
    p = B.MoeProblem(base["T"], base["d"], base["E"], base["k"], base["f"], base["R"], base.get("dtype", 1), base["tile_m"],
                     base["tile_n"], 0, 0, 1)
    lib = ctypes.CDLL(LIB)
    assert lib.moe_combine(ctypes.byref(p), None, None, None, None, None, None, None) == B.MOE_ERR_UNSUPPORTED


def test_null_pointers_and_zero_epoch(B):
    p = B.problem(256, 512, 8, 2, 1024, 2, "bf16")
    lib = ctypes.CDLL(LIB)
    assert lib.moe_route(ctypes.byref(p), None, None, None, None, None, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_dispatch(ctypes.byref(p), *([None] * 10)) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_megakernel_forward(ctypes.byref(p), *([None] * 19)) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_combine(ctypes.byref(p), *([None] * 7)) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_workspace_init(ctypes.byref(p), None, None) == B.MOE_ERR_WORKSPACE
    fake = ctypes.c_void_p(0x1008)  # misaligned workspace is refused before any launch
    assert lib.moe_workspace_init(ctypes.byref(p), fake, None) == B.MOE_ERR_WORKSPACE


def test_header_is_plain_c_and_links_from_c(B, tmp_path):
    """The boundary is a C ABI: include/moe.h compiles as strict C99 (no C++ in it), a C program links against the
    library without anything else on its link line, and what it gets from the host-only calls is what the Python
    binding gets."""
    import subprocess
    src = tmp_path / "abi.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "moe.h"
int main(void) {
    moe_problem_t p;
    memset(&p, 0, sizeof p);
    p.T = 4096; p.d = 2048; p.E = 128; p.k = 8; p.f = 768; p.R = 8;
    p.dtype = MOE_DT_BF16; p.signal_mode = MOE_SIGNAL_PER_DEST; p.fence_scope = MOE_SCOPE_AGENT; p.epoch = 1;
    printf("%zu %zu %s|%s\n", moe_workspace_bytes(&p), moe_num_flags(&p), moe_status_string(MOE_OK),
           moe_status_string(MOE_ERR_UNSUPPORTED));
    p.k = 200;  /* more experts per token than experts: no workspace size */
    printf("%zu\n", moe_workspace_bytes(&p));
    /* a compute entry point refuses a missing problem before it touches a device */
    printf("%d\n", moe_combine(NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL));
    return 0;
}
''')
    exe = tmp_path / "abi"
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, str(src), "-o", str(exe), LIB,
                    "-Wl,-rpath," + os.path.dirname(LIB)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    p = B.problem(4096, 2048, 128, 8, 768, 8, "bf16")
    assert out[0] == f"{B.moe_workspace_bytes(p)} {B.moe_num_flags(p)} ok|unsupported problem"
    assert out[1] == "0"
    assert int(out[2]) == B.MOE_ERR_INVALID_ARG
