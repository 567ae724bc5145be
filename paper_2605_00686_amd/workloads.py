"""Seeded synthetic workloads shaped like the paper's MoE layers.

This module only draws random numbers and names shapes.  It holds none of the
method's arithmetic (no routing, no sorting, no expert math), so both the HIP
path and the CPU oracle may be fed from it without sharing code.

Shapes follow Table 1 of the paper (H, I, E, k): Qwen3-30B-A3B
(2048, 768, 128, 8), DeepSeek-V3 (7168, 2048, 256, 8) and GPT-OSS-120B
(2880, 2880, 128, 4), plus a compute-bound
few-large-experts layer in the role the paper gives Llama4 (section 3.1) and a
decode-sized batch (section 8, 'small S resembles decode').  Skewed routing
follows section 6.4 (Zipf popularity, no token drops).
"""
from __future__ import annotations

import numpy as np
import torch

# name -> recipe.  'bias_std' adds a per-expert fp32 offset to the gate logits;
# 'prerouted' means topk_idx / topk_w are inputs (one arriving row per slot).
CONFIGS = {
    # toy layer, fp32, oracle runs in seconds
    "cfg1": dict(T=256, d=512, E=8, k=2, f=1024, R=2, dtype="f32", seed=0),
    # Qwen3-30B-A3B-shaped, all 128 experts local, load skewed by a gate bias
    "cfg2": dict(T=4096, d=2048, E=128, k=8, f=768, R=8, dtype="bf16", seed=2, bias_std=0.5),
    # DeepSeek-V3-shaped share of one rank of EP-64: 4 local experts, rows arrive pre-routed
    "cfg3": dict(T=8192, d=7168, E=4, k=1, f=2048, R=64, dtype="bf16", seed=3,
                 prerouted=dict(global_experts=256, zipf=1.1, topk=8)),
    # few large experts, compute-bound
    "cfg4": dict(T=16384, d=4096, E=8, k=2, f=14336, R=8, dtype="bf16", seed=4),
    # decode-sized batch, many tiny signaled tiles
    "cfg5": dict(T=128, d=7168, E=32, k=8, f=2048, R=64, dtype="bf16", seed=5, tile_m=32),
    # third shape of Table 1 (2880, 2880, 128, 4): dimensions that are not powers of two, ragged column tiles
    "cfg6": dict(T=4096, d=2880, E=128, k=4, f=2880, R=8, dtype="bf16", seed=6),
    # DeepSeek-V3-shaped layer with all 256 experts local (Table 1, second shape): every weight tensor has more
    # than 2^31 elements (7.5 GB), which is what this one is for
    "cfg7": dict(T=2048, d=7168, E=256, k=8, f=2048, R=8, dtype="bf16", seed=7, bias_std=0.5),
    # decode-sized batch on the Qwen3-30B-A3B-shaped layer: few tokens AND many experts
    "cfg8": dict(T=128, d=2048, E=128, k=8, f=768, R=8, dtype="bf16", seed=8, tile_m=32, bias_std=0.5),
    # --- reduced shapes for parity tests: several tiles plus ragged tails ---
    "mini_f32": dict(T=96, d=192, E=6, k=2, f=320, R=4, dtype="f32", seed=11),
    "mini_bf16": dict(T=384, d=512, E=8, k=2, f=640, R=4, dtype="bf16", seed=12, bias_std=0.5),
    "mini_skew": dict(T=512, d=256, E=16, k=4, f=384, R=8, dtype="bf16", seed=13, bias_std=1.5),
    "mini_pre": dict(T=640, d=512, E=4, k=1, f=256, R=16, dtype="bf16", seed=14,
                     prerouted=dict(global_experts=256, zipf=1.1, topk=8)),
    "mini_large": dict(T=2048, d=512, E=4, k=2, f=384, R=8, dtype="bf16", seed=16),
    "mini_decode": dict(T=64, d=1024, E=16, k=4, f=512, R=32, dtype="bf16", seed=15, tile_m=32),
    "mini_odd": dict(T=320, d=320, E=8, k=4, f=448, R=4, dtype="bf16", seed=17),
}

W_STD = 0.02  # N(0, 0.02): 0.02 is the standard deviation


def config(name_or_cfg) -> dict:
    cfg = dict(CONFIGS[name_or_cfg]) if isinstance(name_or_cfg, str) else dict(name_or_cfg)
    cfg.setdefault("tile_m", 128)
    cfg.setdefault("tile_n", 64)
    cfg.setdefault("bias_std", 0.0)
    cfg.setdefault("prerouted", None)
    return cfg


def torch_dtype(cfg) -> torch.dtype:
    return torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16


def _normal(gen, shape, std, dtype):
    """N(0, std) drawn in fp32 on the generator's device, then rounded once to ``dtype``.
    Leading-dimension chunks bound the fp32 temporary for multi-GB tensors."""
    out = torch.empty(shape, dtype=dtype, device=gen.device)
    if len(shape) == 3:
        for e in range(shape[0]):
            out[e] = (torch.randn(shape[1:], generator=gen, dtype=torch.float32, device=gen.device) * std).to(dtype)
    else:
        out.copy_((torch.randn(shape, generator=gen, dtype=torch.float32, device=gen.device) * std).to(dtype))
    return out


def make_inputs(name_or_cfg, with_weights: bool = True, device: str = "cpu") -> dict:
    """Tensors for one workload: x[T,d], Wg[d,E], gate_bias[E] or None,
    W1/W3[E,d,f], W2[E,f,d] in the config dtype; for pre-routed configs also
    topk_idx[T,1] int32 and topk_w[T,1] fp32 (and no Wg).  Drawn on the CPU by
    default; ``device="cuda"`` draws them in GPU memory with that device's
    seeded generator (other values than the CPU's for the same seed; tens of GB
    of weights then take seconds instead of minutes)."""
    cfg = config(name_or_cfg)
    T, d, E, k, f = cfg["T"], cfg["d"], cfg["E"], cfg["k"], cfg["f"]
    dt = torch_dtype(cfg)
    gen = torch.Generator(device=device).manual_seed(int(cfg["seed"]))
    out = {"cfg": cfg}
    out["x"] = _normal(gen, (T, d), 1.0, dt)
    pre = cfg["prerouted"]
    if pre is None:
        out["Wg"] = _normal(gen, (d, E), W_STD, dt)
        out["gate_bias"] = (torch.randn(E, generator=gen, dtype=torch.float32, device=gen.device) * cfg["bias_std"]
                            if cfg["bias_std"] > 0 else None)
        out["topk_idx"] = None
        out["topk_w"] = None
    else:
        assert k == 1 and device == "cpu"
        # popularity of the local experts: global ranks 1..E of a Zipf law over all experts
        ranks = torch.arange(1, E + 1, dtype=torch.float64)
        pmf = ranks.pow(-float(pre["zipf"]))
        ids = torch.multinomial(pmf / pmf.sum(), T, replacement=True, generator=gen)
        out["topk_idx"] = ids.to(torch.int32).reshape(T, 1).contiguous()
        # the weight this row carries is one share of a normalised top-k gate:
        # first of `topk` positive numbers summing to one
        shares = torch.rand(T, int(pre["topk"]), generator=gen, dtype=torch.float32) + 0.05
        out["topk_w"] = (shares[:, :1] / shares.sum(dim=1, keepdim=True)).contiguous()
        out["Wg"] = None
        out["gate_bias"] = None
    if with_weights:
        out["W1"] = _normal(gen, (E, d, f), W_STD, dt)
        out["W3"] = _normal(gen, (E, d, f), W_STD, dt)
        out["W2"] = _normal(gen, (E, f, d), W_STD, dt)
    return out


def as_oracle_array(t):
    """torch CPU tensor -> numpy array the oracle accepts: fp32 values, or the
    raw 16-bit patterns of a bf16 tensor (no rounding happens here)."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.uint16).numpy()
    return t.numpy()


def sample_tokens(cfg, n: int, seed: int = 1234) -> np.ndarray:
    """n distinct token ids spread over the whole batch (first, last and a
    seeded random draw), for sampled full-size parity."""
    T = cfg["T"]
    n = min(n, T)
    rng = np.random.default_rng(seed)
    picks = {0, T - 1}
    while len(picks) < n:
        picks.add(int(rng.integers(0, T)))
    return np.array(sorted(picks), dtype=np.int32)
