"""Seeded synthetic inputs for paged-KV decode attention.

This module holds no attention arithmetic: it only draws shapes, lengths, block
tables and N(0,1) tensors.  Both the test oracle and the HIP path are fed from it.

The shapes follow the workloads the paper evaluates (Section 4.1: batch 1..128,
512 input + 512..8192 output tokens, 16-token blocks, head_dim 128, MHA and GQA
models) as fixed by this repository's benchmark configurations.  Physical block ids
are a random permutation of a pool 25 % larger than needed, so consecutive logical
blocks of a sequence are far apart in HBM (the fragmented access pattern of
Section 2).
"""
from __future__ import annotations

import math

import numpy as np
import torch

BASE_SEED = 20250406

CONFIGS = [
    dict(name="tiny", B=2, Hq=4, Hkv=4, d=64, bs=16, lens=[37, 128], dtype="f16"),
    dict(name="llama3_8b_decode", B=64, Hq=32, Hkv=8, d=128, bs=16, len_range=(1024, 8192),
         dtype="bf16"),
    dict(name="long_context_decode", B=8, Hq=32, Hkv=8, d=128, bs=16, lens=[32768] * 8,
         dtype="bf16"),
    dict(name="llama3_70b_decode", B=32, Hq=64, Hkv=8, d=128, bs=32, len_range=(512, 16384),
         dtype="bf16"),
    dict(name="layer_stack", B=128, Hq=32, Hkv=8, d=128, bs=16, len_range=(2048, 4096),
         dtype="bf16", layers=32, gemm_k=4096, gemm_n=14336),
]

TORCH_DTYPES = {"f16": torch.float16, "bf16": torch.bfloat16}


def config_seed(index: int, layer: int = 0) -> int:
    return BASE_SEED + index + 1000 * layer


def context_lengths(cfg: dict, seed: int) -> np.ndarray:
    """Per-sequence context lengths: fixed list, or uniform integers in [lo, hi]."""
    if "lens" in cfg:
        return np.asarray(cfg["lens"], dtype=np.int32)
    lo, hi = cfg["len_range"]
    rng = np.random.Generator(np.random.PCG64(seed))
    u = rng.random(cfg["B"])
    return (lo + np.floor(u * (hi - lo + 1))).astype(np.int32)


def block_tables(lens: np.ndarray, bs: int, seed: int, slack: float = 1.25, width: int | None = None):
    """Random paging of every sequence.

    Returns (tables int32 [B, MB], NBLK, poison_id).  Needed entries are distinct ids
    drawn without replacement from a shuffled pool; entries past a sequence's last
    block all name ``poison_id`` (= NBLK - 1), a block no sequence owns.
    """
    lens = np.asarray(lens, dtype=np.int64)
    need = (np.maximum(lens, 0) + bs - 1) // bs
    total = int(need.sum())
    pool = int(math.ceil(slack * total)) + 1
    poison_id = pool  # one extra block after the pool
    nblk = pool + 1
    mb = int(need.max()) if width is None else int(width)
    mb = max(mb, 1)
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    perm = rng.permutation(pool)
    tables = np.full((len(lens), mb), poison_id, dtype=np.int32)
    pos = 0
    for b, nb in enumerate(need):
        tables[b, :nb] = perm[pos:pos + nb]
        pos += nb
    return tables, nblk, poison_id


def randn16(shape, dtype: str, seed: int, device) -> torch.Tensor:
    """N(0,1) values rounded to fp16 / bf16, drawn on ``device`` from a seeded generator."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=TORCH_DTYPES[dtype])


def make_case(cfg: dict, seed: int, device="cpu", poison: bool = False, table_width: int | None = None,
              lens=None, data_seed: int | None = None) -> dict:
    """All tensors of one attention call.

    Lengths and paging come from ``seed``; the N(0,1) values from ``data_seed`` (default ``seed``), so
    the layers of a stack can share one block table and hold different data.

    poison=True writes NaN into every cache slot no sequence owns (the unowned pool
    blocks, the poison block, and the tail of each sequence's last block); a correct
    implementation never reads them.
    """
    lens = context_lengths(cfg, seed) if lens is None else np.asarray(lens, dtype=np.int32)
    B, Hq, Hkv, d, bs = len(lens), cfg["Hq"], cfg["Hkv"], cfg["d"], cfg["bs"]
    tables, nblk, poison_id = block_tables(lens, bs, seed, width=table_width)
    dt = cfg["dtype"]
    ds = seed if data_seed is None else data_seed
    q = randn16((B, Hq, d), dt, ds + 1, device)
    k_cache = randn16((nblk, Hkv, bs, d), dt, ds + 2, device)
    v_cache = randn16((nblk, Hkv, bs, d), dt, ds + 3, device)
    if poison:
        owned = torch.zeros(nblk, dtype=torch.bool)
        tail_mask = torch.zeros((nblk, bs), dtype=torch.bool)
        for b, n in enumerate(lens):
            nb = (max(int(n), 0) + bs - 1) // bs
            ids = torch.from_numpy(tables[b, :nb].astype(np.int64))
            owned[ids] = True
            if nb and n % bs:
                tail_mask[int(tables[b, nb - 1]), int(n % bs):] = True
        dead = (~owned)[:, None] | tail_mask            # [nblk, bs]
        dead = dead.to(device)[:, None, :, None]
        nan = torch.tensor(float("nan"), dtype=TORCH_DTYPES[dt], device=device)
        k_cache = torch.where(dead, nan, k_cache)
        v_cache = torch.where(dead, nan, v_cache)
    return dict(
        q=q, k_cache=k_cache, v_cache=v_cache,
        block_tables=torch.from_numpy(tables).to(device),
        context_lens=torch.from_numpy(lens.astype(np.int32)).to(device),
        scale=1.0 / math.sqrt(d), dtype=dt, num_kv_heads=Hkv, block_size=bs,
        lens=lens, poison_id=poison_id,
    )


def to_fp8_codes(x: torch.Tensor, scale: float) -> torch.Tensor:
    """Nearest OCP FP8 E4M3 codes (uint8) of x / scale; NaN stays NaN (code 0x7f / 0xff)."""
    return (x.to(torch.float32) / scale).to(torch.float8_e4m3fn).view(torch.uint8)


def make_case_kv8(cfg: dict, seed: int, device="cpu", poison: bool = False, lens=None, k_scale: float = 1.0,
                  v_scale: float = 1.0, table_width: int | None = None, data_seed: int | None = None) -> dict:
    """As :func:`make_case` with the caches quantised to FP8 E4M3 codes: the values attended to are
    ``k_scale * decode(k_cache)`` and ``v_scale * decode(v_cache)``."""
    c = make_case(cfg, seed, device, poison=poison, table_width=table_width, lens=lens, data_seed=data_seed)
    c["k_cache"] = to_fp8_codes(c["k_cache"], k_scale)
    c["v_cache"] = to_fp8_codes(c["v_cache"], v_scale)
    c["k_scale"], c["v_scale"] = float(k_scale), float(v_scale)
    return c


def kv_bytes(lens, Hkv: int, d: int, elem_bytes: int = 2) -> int:
    """Algorithmic K+V bytes one attention call must move."""
    return int(np.maximum(np.asarray(lens, dtype=np.int64), 0).sum()) * Hkv * d * 2 * elem_bytes
