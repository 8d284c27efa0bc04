"""Seeded input generators for the router-gated decode path.

This module only draws random numbers and names shapes.  It implements none of the
method's arithmetic (no norm, no projection, no router, no attention): both the CPU oracle
and the HIP library are handed the buffers made here and neither imports the other.

Recipe (synthetic stand-ins for the paper's LLaMA checkpoints and dataset prompts, which
only fix shapes, lengths and the mask as far as decode cost is concerned):
  * projection / embedding / LM-head weights ~ N(0, 0.02^2) in fp32, then (bf16 models)
    rounded to nearest-even bf16; RMSNorm gains are exactly 1;
  * router weights ~ N(0, 0.02^2), fp32, one D-vector per layer, no bias;
  * prompt ids uniform in [0, vocab);
  * benchmark skip masks: k distinct layers drawn uniformly from {1..L-2} (first and last
    layer always kept, like the trained routers in the paper's layer-wise skip tables).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np
import torch


@dataclass(frozen=True)
class ModelDesc:
    """Geometry of a Llama-style decoder (pre-norm, RoPE, GQA, SwiGLU, untied LM head)."""
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # storage type of weights and KV cache: "bf16" or "fp32"
    rope_base: float = 10000.0
    rms_eps: float = 1e-5

    @property
    def layer_params(self) -> int:
        d, hq, hkv, hd, f = self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.d_ffn
        return 2 * d * hq * hd + 2 * d * hkv * hd + 3 * d * f

    @property
    def bytes_per_elem(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    def with_(self, **kw) -> "ModelDesc":
        return replace(self, **kw)


# The model geometries named by the benchmark configurations.
CONFIGS: Dict[str, ModelDesc] = {
    "tiny": ModelDesc(4, 256, 4, 4, 64, 688, 1024, dtype="fp32"),
    "1b": ModelDesc(16, 2048, 32, 8, 64, 8192, 32000, dtype="bf16"),
    "8b": ModelDesc(32, 4096, 32, 8, 128, 14336, 128256, dtype="bf16"),
    "3b": ModelDesc(28, 3072, 24, 8, 128, 8192, 128256, dtype="bf16"),        # geometry of the paper's second model
    # reduced shapes for fast parity tests: ragged FFN / vocab sizes, GQA group 4
    "mini_bf16": ModelDesc(4, 512, 8, 2, 64, 1416, 2003, dtype="bf16"),
    "mini_fp32": ModelDesc(3, 256, 4, 2, 64, 696, 1001, dtype="fp32"),
    "mini_hd128": ModelDesc(3, 512, 4, 1, 128, 1032, 1500, dtype="bf16"),
    "mini_8b_heads": ModelDesc(2, 512, 32, 8, 128, 1032, 1500, dtype="bf16"),    # the 8B head geometry (32 query / 8 KV heads) on a narrow model
    # widths that are multiples of 2048: shapes the persistent whole-step decode kernel accepts
    "step_hd128": ModelDesc(3, 2048, 16, 4, 128, 4096, 5003, dtype="bf16"),
    "step_hd64": ModelDesc(2, 2048, 32, 8, 64, 2048, 3001, dtype="bf16"),
    "step_g2": ModelDesc(2, 2048, 16, 8, 128, 2048, 2999, dtype="bf16"),
    "step_mha": ModelDesc(2, 2048, 16, 16, 128, 2048, 2999, dtype="bf16"),
    "step_3k": ModelDesc(2, 1536, 12, 4, 128, 2560, 3001, dtype="bf16"),          # widths that are not multiples of 2048
}

# Workloads: (model, batch, prompt length(s), decode steps, skipped-layer count(s)).
WORKLOADS: Dict[str, dict] = {
    "cfg1_tiny": dict(model="tiny", batch=1, prompt=32, decode=16, skip=[2, 0, 4], seed=1),
    "cfg2_1b": dict(model="1b", batch=1, prompt=512, decode=128, skip=[4], seed=2),
    "cfg3_8b": dict(model="8b", batch=1, prompt=1024, decode=256, skip=[0, 8, 16], seed=3),
    "cfg3_3b": dict(model="3b", batch=1, prompt=1024, decode=256, skip=[0, 7, 14], seed=6),
    "cfg4_8b_b16": dict(model="8b", batch=16, prompt=(256, 2048), decode=128, skip="U[0,0.5]", seed=4),
    "cfg5_8b_16k": dict(model="8b", batch=4, prompt=16384, decode=256, skip=[12], seed=5),
}


def torch_dtype(desc: ModelDesc) -> torch.dtype:
    return torch.bfloat16 if desc.dtype == "bf16" else torch.float32


def _gen(seed: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(shape, std: float, gen: torch.Generator, device: str, dtype: torch.dtype) -> torch.Tensor:
    """N(0, std^2) drawn in fp32 then rounded (nearest-even) to the storage type.
    Large tensors are drawn in row chunks so the fp32 staging copy stays small."""
    rows = shape[0]
    out = torch.empty(shape, dtype=dtype, device=device)
    per_row = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    chunk = max(1, (64 << 20) // max(1, per_row))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        t = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=gen, device=device,
                        dtype=torch.float32) * std
        out[r0:r1] = t.to(dtype)
    return out


def make_weights(desc: ModelDesc, seed: int, device: str = "cpu") -> dict:
    """All dense weights of the decoder, row-major [out_features, in_features]."""
    gen = _gen(1000 + seed, device)
    dt = torch_dtype(desc)
    d, hq, hkv, hd, f, v = (desc.d_model, desc.n_q_heads, desc.n_kv_heads, desc.head_dim,
                            desc.d_ffn, desc.vocab)
    ones = lambda: torch.ones(d, dtype=torch.float32, device=device)
    w = {
        "embed": _normal((v, d), 0.02, gen, device, dt),
        "lm_head": _normal((v, d), 0.02, gen, device, dt),
        "final_norm": ones(),
        "layers": [],
    }
    for _ in range(desc.n_layers):
        w["layers"].append({
            "attn_norm": ones(),
            "wq": _normal((hq * hd, d), 0.02, gen, device, dt),
            "wk": _normal((hkv * hd, d), 0.02, gen, device, dt),
            "wv": _normal((hkv * hd, d), 0.02, gen, device, dt),
            "wo": _normal((d, hq * hd), 0.02, gen, device, dt),
            "mlp_norm": ones(),
            "w_gate": _normal((f, d), 0.02, gen, device, dt),
            "w_up": _normal((f, d), 0.02, gen, device, dt),
            "w_down": _normal((d, f), 0.02, gen, device, dt),
        })
    return w


def make_router(desc: ModelDesc, seed: int, device: str = "cpu", std: float = 0.02) -> torch.Tensor:
    """Router weights [L, D] fp32, one bias-free D->1 linear per layer."""
    gen = _gen(2000 + seed, device)
    return torch.randn((desc.n_layers, desc.d_model), generator=gen, device=device,
                       dtype=torch.float32) * std


def make_prompt(vocab: int, n: int, seed: int) -> torch.Tensor:
    """n token ids uniform in [0, vocab), int32, on the CPU."""
    rng = np.random.Generator(np.random.PCG64(3000 + int(seed)))
    return torch.from_numpy(rng.integers(0, vocab, size=int(n), dtype=np.int32))


def make_skip_mask(n_layers: int, n_skip: int, seed: int) -> torch.Tensor:
    """uint8 [L] keep mask (1 = layer runs) with n_skip zeros placed uniformly among the
    interior layers 1..L-2."""
    if n_skip < 0 or n_skip > max(0, n_layers - 2):
        raise ValueError("n_skip must lie in [0, L-2]")
    rng = np.random.Generator(np.random.PCG64(4000 + int(seed)))
    mask = np.ones(n_layers, dtype=np.uint8)
    if n_skip:
        idx = rng.choice(np.arange(1, n_layers - 1), size=n_skip, replace=False)
        mask[idx] = 0
    return torch.from_numpy(mask)


def make_interval_mask(n_layers: int, n_skip: int) -> torch.Tensor:
    """uint8 [L] keep mask with n_skip zeros at (as nearly as integers allow) equal intervals over the interior layers
    1..L-2: the fixed-interval rule of the paper's baselines (Section 5.1)."""
    if n_skip < 0 or n_skip > max(0, n_layers - 2):
        raise ValueError("n_skip must lie in [0, L-2]")
    mask = np.ones(n_layers, dtype=np.uint8)
    inner = n_layers - 2
    for i in range(n_skip):
        mask[1 + ((2 * i + 1) * inner) // (2 * n_skip)] = 0
    assert int((mask == 0).sum()) == n_skip
    return torch.from_numpy(mask)


def to_device(weights: dict, device: str) -> dict:
    """Copy of a weight dict on another device (plumbing only)."""
    out = {k: (v.to(device) if torch.is_tensor(v) else v) for k, v in weights.items() if k != "layers"}
    out["layers"] = [{k: v.to(device) for k, v in lw.items()} for lw in weights["layers"]]
    return out
