#!/usr/bin/env python3
"""Benchmark of the MoE hot path on one MI355X.

One step = one pass of the whole path (gate, dispatch, grouped SwiGLU GEMM,
publish with flags, combine) in one persistent-kernel launch over one batch of
seeded synthetic input already resident in HBM.  Prints ONE JSON line.

Default workload: cfg4, the largest single-GPU configuration (few large
experts), whose grouped GEMM is bound by the bf16 matrix cores: its `roofline`
is FFN FLOPs / kernel time against the published dense bf16 MFMA peak.  The
same line carries, under `hbm_workload`, the Qwen3-30B-A3B-shaped cfg2, whose
layer streams weights and is bound by HBM.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4]
                  [--signal-mode per_dest|per_tile] [--scope agent|system] [--group-size G]
                  [--scheduler static|ready_queue] [--capacity C] [--ops] [--no-cpu] [--no-secondary]
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

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published
MFMA_BF16_PEAK_TF = 2500.0  # dense bf16 MFMA, published
DEFAULT_WORKLOAD = "cfg4"
SECONDARY_WORKLOAD = "cfg2"

# HBM bytes per launch of k_megakernel as hardware counters read them (rocprofv3 --pmc FETCH_SIZE, then
# WRITE_SIZE, each scaled by what the counter reads for a plain copy of known size).  Not measured by this
# script: taken from the named summary under profiles/; a workload without one reports null.
MEASURED_TRAFFIC = {
    "cfg2": (1.849e9, "profiles/megakernel_cfg2_hbm_traffic.txt"),
    "cfg4": (2.063e10, "profiles/megakernel_cfg4_hbm_traffic.txt"),
}


def elem_bytes(cfg) -> int:
    return 4 if cfg["dtype"] == "f32" else 2


def algorithmic_bytes(cfg) -> int:
    """Bytes one launch must move through HBM: every weight once, x once, the
    intermediate h written and read once, every expert output row written to
    staging and read back by combine, out written once, plus routing metadata.
    (The permuted copy of x is never materialised, so it is not counted.)"""
    T, d, E, k, f = cfg["T"], cfg["d"], cfg["E"], cfg["k"], cfg["f"]
    sz = elem_bytes(cfg)
    N = T * k
    weights = 3 * E * d * f * sz + (d * E * sz if cfg["prerouted"] is None else 0)
    return weights + T * d * sz + 2 * N * f * sz + 2 * N * d * sz + T * d * sz + 24 * N


def ffn_flops(cfg) -> int:
    """The grouped GEMM's algorithmic work: 6 d f per routed row (gated MLP, three matrices)."""
    return cfg["T"] * cfg["k"] * 6 * cfg["d"] * cfg["f"]


def gate_flops(cfg) -> int:
    return 2 * cfg["T"] * cfg["d"] * cfg["E"] if cfg["prerouted"] is None else 0


def bound_of(cfg) -> str:
    """Which roofline bounds the layer: with at least ~314 rows per expert (machine balance 2.5 PFLOP/s over
    8 TB/s, 3 d f weights of 2 bytes against 6 d f FLOPs per row) the bf16 matrix cores, else HBM (weights)."""
    return "mfma" if cfg["dtype"] == "bf16" and cfg["T"] * cfg["k"] / cfg["E"] >= 314 else "hbm"


def cpu_baseline(inp, budget_tokens: int):
    """The CPU oracle, as it stands, on the first `budget_tokens` tokens of the
    same workload (gate, dispatch, experts, combine), timed once."""
    import oracle
    from paper_2605_00686_amd import workloads as W
    cfg = inp["cfg"]
    n = min(budget_tokens, cfg["T"])
    o = {k: W.as_oracle_array(inp[k]) for k in ("x", "Wg", "gate_bias", "W1", "W3", "W2", "topk_idx", "topk_w")}
    x = o["x"][:n]
    t0 = time.perf_counter()
    if cfg["prerouted"] is None:
        oracle.forward(x, o["Wg"], o["W1"], o["W3"], o["W2"], cfg["k"], bias=o["gate_bias"])
    else:
        oracle.forward(x, None, o["W1"], o["W3"], o["W2"], cfg["k"], idx=o["topk_idx"][:n], w=o["topk_w"][:n])
    dt = time.perf_counter() - t0
    how = "whole workload" if n == cfg["T"] else "extrapolated from a token subset"
    return {"value": n / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {n} of {cfg['T']} tokens of the same workload ({how}), whole path, {dt:.1f} s"}


def standalone_ops(B, torch, p, buf, dev, cfg, steps):
    """Average duration of each standalone entry point (HIP events on the launch stream) and the
    rate at which it moves its algorithmic bytes.  buf holds the routing of the last full pass."""
    T, d, E, k = cfg["T"], cfg["d"], cfg["E"], cfg["k"]
    sz = elem_bytes(cfg)
    N = T * k
    x_perm = torch.empty((p.E * p.capacity if p.capacity > 0 else N, d), dtype=dev["x"].dtype, device="cuda")
    idx2, w2 = torch.empty_like(buf.topk_idx), torch.empty_like(buf.topk_w)

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for e0, e1 in evs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        return sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps

    def rates(ms, nbytes):
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"ms": ms, "algorithmic_bytes": nbytes, "GB/s": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}

    out = {}
    if dev["Wg"] is not None:
        ms = timed(lambda: B.moe_route(p, dev["x"], dev["Wg"], dev["gate_bias"], idx2, w2))
        out["moe_route"] = {"ms": ms, "fp64_tflops": 2.0 * T * d * E / (ms * 1e-3) / 1e12}
    ms = timed(lambda: B.moe_dispatch(p, dev["x"], buf.topk_idx, buf.counts, buf.offsets, buf.perm, buf.inv_perm,
                                      x_perm, None, buf.workspace))
    # what a dispatch must move: every token row read once, every routed row written once, the ids read, perm and
    # inv_perm written.  ("requested": the same with every routed row also read, as a gather by sorted position does.)
    out["moe_dispatch"] = rates(ms, T * d * sz + N * d * sz + 12 * N)
    out["moe_dispatch"]["requested_bytes"] = 2 * N * d * sz + 12 * N
    ms = timed(lambda: B.moe_combine(p, buf.staging, None, None, buf.topk_w, buf.out, None))
    out["moe_combine"] = rates(ms, N * d * sz + T * d * sz + 4 * N)  # staging rows read, out written, weights read
    return out


def mfma_ceiling(B, torch):
    """What the matrix cores of THIS box deliver, for holding the grouped GEMM's fraction of the published peak
    against: (a) the library's probe kernel, nothing but independent bf16 MFMAs at one wavefront per SIMD, on
    all-zero operands and on operands with the workloads' value distributions (x ~ N(0,1), W ~ N(0,0.02)): the
    clock the chip holds under matrix-core load depends on its power limit and on the operand bits; (b) the
    vendor library's GEMM (torch.matmul) on one cfg4 expert's two products with the same distributions."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(cus * 256, dtype=torch.float32, device="cuda")
    gen = torch.Generator(device="cpu").manual_seed(99)
    gauss = torch.cat([torch.randn(2048, generator=gen), torch.randn(2048, generator=gen) * 0.02]).to(torch.bfloat16).cuda()
    iters = 40000  # x 16 products of 32 cycles each: about 14 ms at 1.5 GHz

    def timed(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in evs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        return sum(e0.elapsed_time(e1) for e0, e1 in evs) / reps

    out = {"peak_tflops": MFMA_BF16_PEAK_TF, "compute_units": cus}
    for label, frag in (("probe_zero_operands", torch.zeros(4096, dtype=torch.bfloat16, device="cuda")),
                        ("probe_gaussian_operands", gauss)):
        ms = timed(lambda: B.moe_probe_mfma(frag, iters, cus, sink), 20)
        tf = cus * 4 * iters * 16 * 32768 / (ms * 1e-3) / 1e12
        out[label] = {"ms": ms, "tflops": tf, "frac_of_peak": tf / MFMA_BF16_PEAK_TF}
    T, d, f = 4096, 4096, 14336  # rows of one cfg4 expert, model and FFN dims
    x = torch.randn(T, d, generator=gen).to(torch.bfloat16).cuda()
    w1 = (torch.randn(d, f, generator=gen) * 0.02).to(torch.bfloat16).cuda()
    h = (torch.randn(T, f, generator=gen) * 0.3).to(torch.bfloat16).cuda()
    w2 = (torch.randn(f, d, generator=gen) * 0.02).to(torch.bfloat16).cuda()
    for label, (a, b) in (("vendor_gemm_x_w1", (x, w1)), ("vendor_gemm_h_w2", (h, w2))):
        ms = timed(lambda: torch.matmul(a, b), 20)
        tf = 2.0 * T * d * f / (ms * 1e-3) / 1e12
        out[label] = {"ms": ms, "tflops": tf, "frac_of_peak": tf / MFMA_BF16_PEAK_TF, "shape": list(a.shape) + [b.shape[1]]}
    return out


def stream_ceiling(B, torch):
    """What the CUs of this machine pull in when they do nothing else (the library's probe kernel): bytes/s by source
    (HBM: every workgroup its own 8 MB of a 2 GB buffer; memory-side cache: all inside 128 MB; L2: all workgroups
    read the same 2 MB) and by wavefronts per CU.  The megakernel runs 4 wavefronts per CU."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    buf = torch.ones(2 << 30, dtype=torch.uint8, device="cuda")
    sink = torch.empty(cus * 1024, dtype=torch.int32, device="cuda")
    per_wg = 8 << 20
    out = {"compute_units": cus, "bytes_per_workgroup": per_wg, "hbm_peak_gbs": HBM_PEAK_GBS, "rows": []}
    for source, span, stride in (("hbm", 2 << 30, per_wg), ("memory_side_cache", 128 << 20, 1 << 20), ("l2", 2 << 20, 0)):
        for waves in (4, 8, 16):
            for to_lds in (1, 0):
                fn = lambda: B.moe_probe_stream(buf, span, stride, per_wg, cus, waves, to_lds, sink)
                for _ in range(2):
                    fn()
                torch.cuda.synchronize()
                evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
                for e0, e1 in evs:
                    e0.record()
                    fn()
                    e1.record()
                torch.cuda.synchronize()
                ms = sum(e0.elapsed_time(e1) for e0, e1 in evs) / len(evs)
                gbs = cus * per_wg / (ms * 1e-3) / 1e9
                out["rows"].append({"source": source, "wavefronts_per_cu": waves, "into": "lds" if to_lds else "registers",
                                    "ms": round(ms, 4), "gbs": round(gbs, 1), "gbs_per_cu": round(gbs / cus, 2)})
    return out


def run_workload(name, args, B, torch, W, steps, warmup, with_cpu, with_ops, calibrate=False):
    """Time `steps` launches of the megakernel on workload `name`; -> dict of everything measured."""
    cfg = W.config(name)
    # tens of GB of weights are drawn in GPU memory (seconds instead of minutes on the host)
    big = 3 * cfg["E"] * cfg["d"] * cfg["f"] * elem_bytes(cfg) > 8e9
    inp = W.make_inputs(dict(W.CONFIGS[name], tile_m=args.tile_m) if args.tile_m else name,
                        device="cuda" if big and cfg["prerouted"] is None else "cpu")
    cfg = inp["cfg"]
    mode = B.MOE_SIGNAL_PER_DEST if args.signal_mode == "per_dest" else B.MOE_SIGNAL_PER_TILE
    scope = B.MOE_SCOPE_AGENT if args.scope == "agent" else B.MOE_SCOPE_SYSTEM

    def make_problem(capacity):
        return B.problem(cfg["T"], cfg["d"], cfg["E"], cfg["k"], cfg["f"], cfg["R"], cfg["dtype"], tile_m=cfg["tile_m"],
                         tile_n=cfg["tile_n"], signal_mode=mode, fence_scope=scope, epoch=1, group_size=args.group_size,
                         scheduler=1 if args.scheduler == "ready_queue" else 0, capacity=capacity,
                         fuse_ffn=1 if args.fuse_ffn else 0)

    def fresh_buffers(p):
        buf = B.Buffers(p)
        if cfg["prerouted"] is not None:
            buf.topk_idx.copy_(inp["topk_idx"])
            buf.topk_w.copy_(inp["topk_w"])
        torch.cuda.synchronize()
        return buf

    capacity = args.capacity
    p = make_problem(max(capacity, 0))
    buf = fresh_buffers(p)
    dev = {n: (inp[n].cuda() if inp[n] is not None else None) for n in ("x", "Wg", "gate_bias", "W1", "W3", "W2")}
    torch.cuda.synchronize()
    if capacity < 0:
        # one untimed pass in the ragged layout tells how many rows the largest expert gets
        B.forward(p, buf, dev["x"], dev["Wg"], dev["gate_bias"], dev["W1"], dev["W3"], dev["W2"])
        torch.cuda.synchronize()
        capacity = (int(buf.counts.max().item()) + 63) // 64 * 64
        p = make_problem(capacity)
        buf = fresh_buffers(p)

    def step():
        p.epoch += 1
        B.forward(p, buf, dev["x"], dev["Wg"], dev["gate_bias"], dev["W1"], dev["W3"], dev["W2"])

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # per-launch durations: events on the stream the kernel is launched on (torch's current stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    avg_ms = sum(kern_ms) / len(kern_ms)
    stats = buf.stats.cpu().tolist()
    if stats[7] != 0:
        print(f"bench.py: device status {stats[7]} ({B.status_string(stats[7])})", file=sys.stderr)
        sys.exit(1)
    if calibrate:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = wall * 1e3 / steps
    abytes, flops = algorithmic_bytes(cfg), ffn_flops(cfg)
    gbs = abytes / (avg_ms * 1e-3) / 1e9
    tfs = flops / (avg_ms * 1e-3) / 1e12
    traffic, traffic_src = MEASURED_TRAFFIC.get(name, (None, None))
    timing = {"kernel": "k_megakernel", "kernel_ms_avg": avg_ms, "kernel_ms_median": kern_ms[len(kern_ms) // 2],
              "kernel_ms_min": kern_ms[0], "traffic": traffic, "traffic_source": traffic_src}
    hbm = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
           "algorithmic_bytes": abytes}
    mfma = {"bound": "mfma", "achieved": tfs, "peak": MFMA_BF16_PEAK_TF, "unit": "TFLOP/s", "frac": tfs / MFMA_BF16_PEAK_TF,
            "algorithmic_flops": flops, "gate_flops_not_counted": gate_flops(cfg)}
    bound = bound_of(cfg)
    res = {
        "workload": f"{name}: T={cfg['T']} d={cfg['d']} E={cfg['E']} k={cfg['k']} f={cfg['f']} "
                    f"R={cfg['R']} tile={cfg['tile_m']}x{cfg['tile_n']}",
        "tokens_per_s": cfg["T"] / (ms_per_step * 1e-3), "ms_per_step": ms_per_step, "capacity": capacity,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
        "roofline": dict(mfma if bound == "mfma" else hbm, **timing),
        "other_roofline": hbm if bound == "mfma" else mfma,
        "signaling": {"fences": stats[0], "flags": stats[1], "publish_tiles": stats[2], "writer_releases": stats[3],
                      "gemm1_tiles": stats[4], "gemm2_tiles": stats[5]},
        "scheduling": {"ready_queue_tasks": stats[16], "gemm2_tiles_run_ahead_of_waiting_gemm1_tiles": stats[17]},
        "timeline_us": {"gate_end": stats[8] / 1e3, "plan_end": stats[9] / 1e3, "perm_end": stats[10] / 1e3,
                        "gemm1_end": stats[11] / 1e3, "gemm2_end": stats[12] / 1e3, "combine_end": stats[13] / 1e3,
                        "wait_sum": stats[14] / 1e3, "workgroups": stats[15]},
    }
    if with_ops:
        res["standalone_ops"] = standalone_ops(B, torch, p, buf, dev, cfg, steps)
    if with_cpu:
        n_cpu = args.cpu_tokens or max(16, min(cfg["T"], int(4e11 / (cfg["k"] * 3 * cfg["d"] * cfg["f"]))))
        res["cpu_baseline"] = cpu_baseline(inp, n_cpu)
    del dev, buf, inp
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--signal-mode", default="per_dest", choices=["per_dest", "per_tile"])
    ap.add_argument("--scope", default="agent", choices=["agent", "system"])
    ap.add_argument("--group-size", type=int, default=0,
                    help="per_dest only: flags per fence group (0 = all flags of a destination)")
    ap.add_argument("--scheduler", default="static", choices=["static", "ready_queue"],
                    help="order of expert tiles and combine tasks: dependency-ordered lists, or ready queues")
    ap.add_argument("--capacity", type=int, default=0,
                    help="rows per expert in the padded layout of the sorted order (0 = ragged layout; -1 = the largest "
                         "expert's row count of this workload, rounded up to a multiple of 64)")
    ap.add_argument("--fuse-ffn", action="store_true",
                    help="a workgroup takes a row block through both GEMMs with h in LDS (f <= 768, tile_m <= 64; see "
                         "--tile-m) instead of two tile passes with h in the workspace")
    ap.add_argument("--tile-m", type=int, default=0, help="publish tile rows (0 = the workload's own)")
    ap.add_argument("--cpu-tokens", type=int, default=0, help="tokens for the CPU baseline (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help=f"skip the HBM-bound workload ({SECONDARY_WORKLOAD}) that the default run reports beside the headline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic) so that hardware byte "
                         "counters collected around this command can be scaled")
    ap.add_argument("--stream-ceiling", action="store_true",
                    help="also measure what this box's CUs stream from HBM, the memory-side cache and L2 with 4, 8 and 16 "
                         "wavefronts each (the library's probe kernel; 'stream_ceiling')")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="also measure what this box's matrix cores deliver with no memory traffic (the library's "
                         "probe kernel) and what the vendor GEMM reaches on one cfg4 expert's shapes ('mfma_ceiling')")
    ap.add_argument("--ops", action="store_true",
                    help="also time the standalone entry points (moe_route, moe_dispatch, moe_combine) on the same "
                         "workload and add them to the JSON line as 'standalone_ops'")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_00686_amd import binding as B
    from paper_2605_00686_amd import workloads as W

    torch.cuda.set_device(0)
    main_res = run_workload(args.workload, args, B, torch, W, args.steps, args.warmup, not args.no_cpu, args.ops,
                            calibrate=args.calibrate_copy)
    res = {
        "metric": "moe_layer_tokens_per_s", "value": main_res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res["dtype"], "data": "synthetic",
        "config": {"workload": main_res["workload"], "signal_mode": args.signal_mode, "fence_scope": args.scope,
                   "group_size": args.group_size, "scheduler": args.scheduler, "capacity": main_res["capacity"],
                   "launches_per_step": 1},
        "roofline": main_res["roofline"],
    }
    for key in ("other_roofline", "signaling", "scheduling", "timeline_us", "standalone_ops"):
        if key in main_res:
            res[key] = main_res[key]
    if args.workload == DEFAULT_WORKLOAD and not args.no_secondary:
        # the weight-streaming (HBM-bound) layer beside the headline, same launch configuration, no CPU leg
        sec = run_workload(SECONDARY_WORKLOAD, args, B, torch, W, max(args.steps, 20), max(args.warmup, 5), False, args.ops)
        res["hbm_workload"] = {k: sec[k] for k in ("workload", "tokens_per_s", "ms_per_step", "roofline", "other_roofline",
                                                   "signaling", "timeline_us", "standalone_ops") if k in sec}
    if args.mfma_ceiling:
        res["mfma_ceiling"] = mfma_ceiling(B, torch)
    if args.stream_ceiling:
        res["stream_ceiling"] = stream_ceiling(B, torch)
    if "cpu_baseline" in main_res:
        res["cpu_baseline"] = main_res["cpu_baseline"]
    print(json.dumps(res))


if __name__ == "__main__":
    main()
