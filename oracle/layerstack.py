"""CPU oracle of one layer of the layer-stack stand-in: dense GEMM then paged attention.

TEST INFRASTRUCTURE ONLY.  The paper has no layer stack; the stand-in is
``y = x . W`` (bf16 inputs, exact products, fp64 sums, result rounded to bf16 with
round-to-nearest-even), ``q = y[:, :Hq*d]`` viewed as [B, Hq, d], then the attention
of ``paged_attention`` on that layer's own KV cache.
"""
from __future__ import annotations

import numpy as np

from .paged_attention import paged_attention


def _bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp64 -> bf16 bit patterns, round to nearest, ties to even (finite inputs).

    Goes through fp32 first; the fp64 sums of bf16 products handled here carry far
    more than 24 significant bits only below the fp32 rounding step, so the double
    rounding can move a result by at most one bf16 ulp in exact-tie cases.
    """
    f32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f32.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = u + 0x7FFF + lsb
    return (u >> 16).astype(np.uint16)


def layer_gemm_bf16(x_bits: np.ndarray, w_bits: np.ndarray) -> np.ndarray:
    """y = x . W in fp64 from bf16 bit patterns; returns bf16 bit patterns [B, N]."""
    x = _bf16_bits_to_f64(x_bits)
    w = _bf16_bits_to_f64(w_bits)
    return round_to_bf16_bits(x @ w)


def layerstack_layer(x_bits, w_bits, k_cache, v_cache, block_tables, context_lens, scale,
                     num_q_heads, head_dim, pairs=None):
    """(y_bits [B,N], out fp64) of one layer; ``pairs`` as in ``paged_attention``."""
    y = layer_gemm_bf16(x_bits, w_bits)
    B = y.shape[0]
    q = np.ascontiguousarray(y[:, : num_q_heads * head_dim]).reshape(B, num_q_heads, head_dim)
    out = paged_attention(q, k_cache, v_cache, block_tables, context_lens, scale, "bf16", pairs)
    return y, out
