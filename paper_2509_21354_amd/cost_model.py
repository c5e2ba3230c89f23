"""The paper's closed-form cost model (section 3.3, Eq. 4-7), for reporting beside
measured numbers.  Nothing on the GPU path depends on it.

Symbols as in the paper: B batch, n cached tokens, d_model, H heads, d_k head
width, d_ff FFN width, W raw window, M kept summaries, C chunk size, d_sum the
aggregator's hidden width, d_g the gate's hidden width; n' = W + M.
"""
from __future__ import annotations

from dataclasses import dataclass


@dataclass(frozen=True)
class ModelDims:
    d_model: int = 4096
    H: int = 32
    d_k: int = 128
    d_ff: int = 11008


def flops_base_attention(B: int, n: int, m: ModelDims = ModelDims()) -> float:
    """Eq. 4: four d_model x d_model projections over n tokens plus QK^T and PV over n x n."""
    return 4.0 * B * n * m.d_model ** 2 + 2.0 * B * m.H * float(n) ** 2 * m.d_k


def flops_ffn(B: int, n: int, m: ModelDims = ModelDims()) -> float:
    """Eq. 5: the SwiGLU feed-forward block."""
    return 3.0 * B * n * m.d_model * m.d_ff


def flops_kv_efficient(B: int, n: int, W: int, M: float, C: int, d_sum: int, d_g: int,
                       m: ModelDims = ModelDims()) -> float:
    """Eq. 6: Eq. 4 at the shortened length n' = W + M, plus per chunk and head the
    aggregator MLP and the recurrent gate."""
    n_eff = W + M
    per_chunk = 4.0 * d_sum * m.d_model + 4.0 * d_g * m.d_model + 4.0 * d_g ** 2
    return (4.0 * B * n_eff * m.d_model ** 2 + 2.0 * B * m.H * n_eff ** 2 * m.d_k
            + (n / C) * B * m.H * per_chunk)


def speed_up(flops_base: float, flops_ffn_: float, flops_kv_eff: float) -> float:
    """Eq. 7: ratio of per-layer work with the FFN unchanged."""
    return (flops_base + flops_ffn_) / (flops_kv_eff + flops_ffn_)


def memory_ratio(n: int, W: int, M: float) -> float:
    """Section 3.3, last paragraph: rows of cache kept, n / (W + M)."""
    return n / (W + M)


def report(B: int, n: int, W: int, M: float, C: int, d_sum: int, d_g: int, m: ModelDims = ModelDims()) -> dict:
    base, ffn = flops_base_attention(B, n, m), flops_ffn(B, n, m)
    eff = flops_kv_efficient(B, n, W, M, C, d_sum, d_g, m)
    return {"flops_base_attention": base, "flops_ffn": ffn, "flops_kv_efficient": eff,
            "speed_up_eq7": speed_up(base, ffn, eff), "memory_ratio": memory_ratio(n, W, M),
            "attention_only_flops_ratio": base / eff}
