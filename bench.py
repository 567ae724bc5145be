#!/usr/bin/env python3
"""Benchmark of the MoE hot path on one MI355X.

One step = one pass of the whole path (gate, dispatch, grouped SwiGLU GEMM,
publish with flags, combine) in one persistent-kernel launch over one batch of
seeded synthetic input already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2]
                  [--signal-mode per_dest|per_tile] [--scope agent|system] [--group-size G] [--scheduler static|ready_queue] [--capacity C]
                  [--ops] [--no-cpu]
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

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (profiles/megakernel_cfg2_hbm_traffic.txt), keyed by workload; None = not measured.
MEASURED_TRAFFIC_BYTES = {"cfg2": 1.853e9}


def algorithmic_bytes(cfg) -> int:
    """Bytes one launch must move through HBM: every weight once, x once, the
    intermediate h written and read once, every expert output row written to
    staging and read back by combine, out written once, plus routing metadata.
    (The permuted copy of x is never materialised, so it is not counted.)"""
    T, d, E, k, f = cfg["T"], cfg["d"], cfg["E"], cfg["k"], cfg["f"]
    sz = 4 if cfg["dtype"] == "f32" else 2
    N = T * k
    weights = 3 * E * d * f * sz + (d * E * sz if cfg["prerouted"] is None else 0)
    return weights + T * d * sz + 2 * N * f * sz + 2 * N * d * sz + T * d * sz + 24 * N


def layer_flops(cfg) -> int:
    T, d, E, k, f = cfg["T"], cfg["d"], cfg["E"], cfg["k"], cfg["f"]
    gate = 2 * T * d * E if cfg["prerouted"] is None else 0
    return T * k * 6 * d * f + gate


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
    return {"value": n / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {n} of {cfg['T']} tokens of the same workload, whole path, {dt:.1f} s"}


def standalone_ops(B, torch, p, buf, dev, cfg, steps):
    """Average duration of each standalone entry point (HIP events on the launch stream) and the
    rate at which it moves its algorithmic bytes.  buf holds the routing of the last full pass."""
    T, d, E, k = cfg["T"], cfg["d"], cfg["E"], cfg["k"]
    sz = 4 if cfg["dtype"] == "f32" else 2
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

    out = {}
    if dev["Wg"] is not None:
        ms = timed(lambda: B.moe_route(p, dev["x"], dev["Wg"], dev["gate_bias"], idx2, w2))
        out["moe_route"] = {"ms": ms, "fp64_tflops": 2.0 * T * d * E / (ms * 1e-3) / 1e12}
    ms = timed(lambda: B.moe_dispatch(p, dev["x"], buf.topk_idx, buf.counts, buf.offsets, buf.perm, buf.inv_perm,
                                      x_perm, None, buf.workspace))
    nbytes = 2 * N * d * sz + 12 * N  # rows read and written once, indices read, perm and inv_perm written
    out["moe_dispatch"] = {"ms": ms, "algorithmic_bytes": nbytes, "GB/s": nbytes / (ms * 1e-3) / 1e9,
                           "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    ms = timed(lambda: B.moe_combine(p, buf.staging, None, None, buf.topk_w, buf.out, None))
    nbytes = N * d * sz + T * d * sz + 4 * N  # staging rows read, out written, weights read
    out["moe_combine"] = {"ms": ms, "algorithmic_bytes": nbytes, "GB/s": nbytes / (ms * 1e-3) / 1e9,
                          "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--signal-mode", default="per_dest", choices=["per_dest", "per_tile"])
    ap.add_argument("--scope", default="agent", choices=["agent", "system"])
    ap.add_argument("--group-size", type=int, default=0,
                    help="per_dest only: flags per fence group (0 = all flags of a destination)")
    ap.add_argument("--scheduler", default="static", choices=["static", "ready_queue"],
                    help="order of expert tiles and combine tasks: dependency-ordered lists, or ready queues")
    ap.add_argument("--capacity", type=int, default=0,
                    help="rows per expert in the padded layout of the sorted order (0 = ragged layout; -1 = the largest "
                         "expert's row count of this workload, rounded up to a multiple of 64)")
    ap.add_argument("--cpu-tokens", type=int, default=0, help="tokens for the CPU baseline (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic) so that hardware byte "
                         "counters collected around this command can be scaled")
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
    cfg = W.config(args.workload)
    # tens of GB of weights are drawn in GPU memory (seconds instead of minutes on the host)
    big = 3 * cfg["E"] * cfg["d"] * cfg["f"] * (4 if cfg["dtype"] == "f32" else 2) > 8e9
    inp = W.make_inputs(args.workload, device="cuda" if big and cfg["prerouted"] is None else "cpu")
    cfg = inp["cfg"]
    mode = B.MOE_SIGNAL_PER_DEST if args.signal_mode == "per_dest" else B.MOE_SIGNAL_PER_TILE
    scope = B.MOE_SCOPE_AGENT if args.scope == "agent" else B.MOE_SCOPE_SYSTEM
    def make_problem(capacity):
        return B.problem(cfg["T"], cfg["d"], cfg["E"], cfg["k"], cfg["f"], cfg["R"], cfg["dtype"], tile_m=cfg["tile_m"],
                         tile_n=cfg["tile_n"], signal_mode=mode, fence_scope=scope, epoch=1, group_size=args.group_size,
                         scheduler=1 if args.scheduler == "ready_queue" else 0, capacity=capacity)

    capacity = args.capacity
    p = make_problem(max(capacity, 0))
    buf = B.Buffers(p)
    dev = {n: (inp[n].cuda() if inp[n] is not None else None) for n in ("x", "Wg", "gate_bias", "W1", "W3", "W2")}
    if cfg["prerouted"] is not None:
        buf.topk_idx.copy_(inp["topk_idx"])
        buf.topk_w.copy_(inp["topk_w"])
    torch.cuda.synchronize()
    if capacity < 0:
        # one untimed pass in the ragged layout tells how many rows the largest expert gets
        B.forward(p, buf, dev["x"], dev["Wg"], dev["gate_bias"], dev["W1"], dev["W3"], dev["W2"])
        torch.cuda.synchronize()
        capacity = (int(buf.counts.max().item()) + 63) // 64 * 64
        p = make_problem(capacity)
        buf = B.Buffers(p)
        if cfg["prerouted"] is not None:
            buf.topk_idx.copy_(inp["topk_idx"])
            buf.topk_w.copy_(inp["topk_w"])
        torch.cuda.synchronize()

    def step():
        p.epoch += 1
        B.forward(p, buf, dev["x"], dev["Wg"], dev["gate_bias"], dev["W1"], dev["W3"], dev["W2"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # per-launch durations: events on the stream the kernel is launched on (torch's current stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
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

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
    ms_per_step = wall * 1e3 / args.steps
    abytes = algorithmic_bytes(cfg)
    flops = layer_flops(cfg)
    achieved = abytes / (avg_ms * 1e-3) / 1e9
    res = {
        "metric": "moe_layer_tokens_per_s", "value": cfg["T"] / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: T={cfg['T']} d={cfg['d']} E={cfg['E']} k={cfg['k']} f={cfg['f']} "
                               f"R={cfg['R']} tile={cfg['tile_m']}x{cfg['tile_n']}",
                   "signal_mode": args.signal_mode, "fence_scope": args.scope, "group_size": args.group_size,
                   "scheduler": args.scheduler, "capacity": capacity,
                   "launches_per_step": 1},
        "roofline": {"bound": "hbm", "kernel": "k_megakernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
                     "algorithmic_bytes": abytes, "kernel_ms_avg": avg_ms, "kernel_ms_median": kern_ms[len(kern_ms) // 2],
                     "kernel_ms_min": kern_ms[0]},
        "mfma": {"tflops": flops / (avg_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TF,
                 "frac": flops / (avg_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF, "flops": flops},
        "signaling": {"fences": stats[0], "flags": stats[1], "publish_tiles": stats[2], "writer_releases": stats[3],
                      "gemm1_tiles": stats[4], "gemm2_tiles": stats[5]},
        "scheduling": {"ready_queue_tasks": stats[16], "gemm2_tiles_run_ahead_of_waiting_gemm1_tiles": stats[17]},
        "timeline_us": {"gate_end": stats[8] / 1e3, "plan_end": stats[9] / 1e3, "perm_end": stats[10] / 1e3,
                        "gemm1_end": stats[11] / 1e3, "gemm2_end": stats[12] / 1e3, "combine_end": stats[13] / 1e3,
                        "wait_sum": stats[14] / 1e3, "workgroups": stats[15]},
    }
    if args.ops:
        res["standalone_ops"] = standalone_ops(B, torch, p, buf, dev, cfg, args.steps)
    if not args.no_cpu:
        n_cpu = args.cpu_tokens or max(16, min(cfg["T"], int(4e11 / (cfg["k"] * 3 * cfg["d"] * cfg["f"]))))
        res["cpu_baseline"] = cpu_baseline(inp, n_cpu)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
