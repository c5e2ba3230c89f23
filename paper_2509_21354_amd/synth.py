"""Seeded synthetic inputs for the gated chunked-KV decode path.

This module holds no arithmetic of the method: it only draws random tensors
with the shapes, dtypes and value distributions of the workloads.  Both the
HIP path (through the binding) and the CPU oracle (through the tests and the
bench) are fed from here, so that they consume identical bytes.

Recipe (synthetic token sequences stand in for the robot datasets, as in the
paper's own long-context cost measurement, section 4.2):
  * Q, K, V      ~ N(0, 1) i.i.d., drawn in fp32, cast to the storage dtype;
  * every weight ~ U(-1/sqrt(fan_in), +1/sqrt(fan_in)), drawn in fp32, cast:
      pool MLP  W1,b1 fan_in = d;  W2,b2 fan_in = d_sum   (one set for K, one for V)
      LSTM      W_ih fan_in = 2d;  W_hh, b_ih, b_hh, w_s, b_s fan_in = d_g
  * seed of a tensor = 20250921 + 1000 * config number + tensor id.
Weights exist once per layer and are shared by all batch rows and heads.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict

import torch

BASE_SEED = 20250921

TENSOR_ID = {
    "Q": 1, "K": 2, "V": 3,
    "W1K": 4, "b1K": 5, "W2K": 6, "b2K": 7,
    "W1V": 8, "b1V": 9, "W2V": 10, "b2V": 11,
    "W_ih": 12, "W_hh": 13, "b_ih": 14, "b_hh": 15, "w_s": 16, "b_s": 17,
    "Q_stream": 18,
}


@dataclasses.dataclass(frozen=True)
class Config:
    """One workload: the symbols follow the paper (C chunk length, W recent
    window, d_sum aggregator hidden width, d_g gate hidden width)."""
    number: int
    name: str
    dtype: str          # "f32" or "bf16": storage type of Q/K/V, summaries and weights
    L: int              # layers batched in one call
    B: int              # batch rows
    H: int              # heads
    d: int              # head dimension
    T: int              # tokens in the cache
    C: int              # chunk length
    k: int              # chunks kept by top-k
    W: int              # raw recent window (tokens)
    d_sum: int
    d_g: int
    Tq: int             # query tokens per sequence
    steps: int = 1      # streaming steps (frames appended); 1 = one-shot
    frame: int = 0      # tokens appended per streaming step
    decode_per_step: int = 1
    H_kv: int = 0       # key-value heads (grouped-query attention); 0 = H

    @property
    def kv_heads(self) -> int:
        return self.H_kv or self.H

    @property
    def N(self) -> int:
        return self.T // self.C

    @property
    def N_cand(self) -> int:
        return max(0, self.T - self.W) // self.C

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[int, Config] = {
    1: Config(1, "cfg1_tiny_f32", "f32", L=1, B=1, H=4, d=64, T=1024, C=16, k=16, W=64,
              d_sum=128, d_g=64, Tq=1),
    2: Config(2, "cfg2_llama7b_layer_b1", "bf16", L=1, B=1, H=32, d=128, T=4096, C=32, k=32,
              W=256, d_sum=128, d_g=256, Tq=1),
    3: Config(3, "cfg3_llama7b_32layers_b8", "bf16", L=32, B=8, H=32, d=128, T=8192, C=32,
              k=64, W=256, d_sum=128, d_g=256, Tq=1),
    4: Config(4, "cfg4_stream_b16", "bf16", L=1, B=16, H=32, d=128, T=16384, C=32, k=64,
              W=256, d_sum=128, d_g=256, Tq=1, steps=64, frame=256, decode_per_step=8),
    5: Config(5, "cfg5_multiquery_b64", "bf16", L=1, B=64, H=32, d=128, T=32768, C=64,
              k=128, W=512, d_sum=128, d_g=512, Tq=256),
}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _normal(shape, dtype, device, seed):
    """N(0,1) drawn in fp32 and cast; the leading axis is filled slab by slab so
    that a 17 GB tensor never needs an fp32 copy of itself."""
    g = _gen(device, seed)
    out = torch.empty(shape, dtype=dtype, device=device)
    if out.numel() == 0:
        return out
    for i in range(shape[0]):
        out[i].copy_(torch.randn(shape[1:], generator=g, dtype=torch.float32, device=device))
    return out


def _uniform(shape, bound, dtype, device, seed):
    g = _gen(device, seed)
    x = torch.rand(shape, generator=g, dtype=torch.float32, device=device)
    return ((x * 2.0 - 1.0) * bound).to(dtype)


def seed_of(cfg: Config, tensor: str) -> int:
    return BASE_SEED + 1000 * cfg.number + TENSOR_ID[tensor]


def make_weights(cfg: Config, device="cpu") -> Dict[str, torch.Tensor]:
    """Per-layer aggregator and gate weights, row-major [out, in]."""
    dt, L, d, ds, dg = cfg.torch_dtype, cfg.L, cfg.d, cfg.d_sum, cfg.d_g
    w = {}
    for kv in ("K", "V"):
        w["W1" + kv] = _uniform((L, ds, d), 1 / math.sqrt(d), dt, device, seed_of(cfg, "W1" + kv))
        w["b1" + kv] = _uniform((L, ds), 1 / math.sqrt(d), dt, device, seed_of(cfg, "b1" + kv))
        w["W2" + kv] = _uniform((L, d, ds), 1 / math.sqrt(ds), dt, device, seed_of(cfg, "W2" + kv))
        w["b2" + kv] = _uniform((L, d), 1 / math.sqrt(ds), dt, device, seed_of(cfg, "b2" + kv))
    w["W_ih"] = _uniform((L, 4 * dg, 2 * d), 1 / math.sqrt(2 * d), dt, device, seed_of(cfg, "W_ih"))
    w["W_hh"] = _uniform((L, 4 * dg, dg), 1 / math.sqrt(dg), dt, device, seed_of(cfg, "W_hh"))
    w["b_ih"] = _uniform((L, 4 * dg), 1 / math.sqrt(dg), dt, device, seed_of(cfg, "b_ih"))
    w["b_hh"] = _uniform((L, 4 * dg), 1 / math.sqrt(dg), dt, device, seed_of(cfg, "b_hh"))
    w["w_s"] = _uniform((L, dg), 1 / math.sqrt(dg), dt, device, seed_of(cfg, "w_s"))
    w["b_s"] = _uniform((L,), 1 / math.sqrt(dg), dt, device, seed_of(cfg, "b_s"))
    return w


def make_qkv(cfg: Config, device="cpu", T_cap: int | None = None) -> Dict[str, torch.Tensor]:
    """Q [L,B,H,Tq,d]; K, V [L,B,H_kv,T_cap,d] with the first T tokens drawn (the
    rest, if T_cap > T, is filled from the same stream: never read by the path)."""
    T_cap = cfg.T if T_cap is None else T_cap
    dt = cfg.torch_dtype
    out = {
        "Q": _normal((cfg.L, cfg.B, cfg.H, cfg.Tq, cfg.d), dt, device, seed_of(cfg, "Q")),
        "K": _normal((cfg.L, cfg.B, cfg.kv_heads, T_cap, cfg.d), dt, device, seed_of(cfg, "K")),
        "V": _normal((cfg.L, cfg.B, cfg.kv_heads, T_cap, cfg.d), dt, device, seed_of(cfg, "V")),
    }
    return out


def make_stream_queries(cfg: Config, device="cpu") -> torch.Tensor:
    """Streaming workload: decode_per_step distinct queries for every step,
    [steps, decode_per_step, L, B, H, 1, d]."""
    return _normal((cfg.steps, cfg.decode_per_step, cfg.L, cfg.B, cfg.H, 1, cfg.d),
                   cfg.torch_dtype, device, seed_of(cfg, "Q_stream"))


def make_inputs(cfg: Config, device="cpu") -> Dict[str, torch.Tensor]:
    out = make_qkv(cfg, device)
    out.update(make_weights(cfg, device))
    return out
