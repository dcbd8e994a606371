"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI, run the
CPU oracle on the same bits, compare to the stated tolerance."""
import numpy as np
import torch

import oracle
import paper_2504_06319_amd as kv

MAX_ABS_TOL = 1e-2      # tolerance of the benchmark contract: max-abs <= 1e-2 ...
MEAN_ABS_TOL = 1e-3     # ... and mean-abs <= 1e-3 on N(0,1) inputs with scale 1/sqrt(d)


def run_hip(c, prefetch_distance=1, out=None, stream=None):
    out = torch.full_like(c["q"], float("nan")) if out is None else out
    kv.kv_decode_attn(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], out,
                      c["scale"], c["num_kv_heads"], c["block_size"], prefetch_distance, stream)
    torch.cuda.synchronize()
    return out


def host_bits(c):
    """One device->host copy of the inputs as raw bit patterns for the oracle."""
    return dict(q=oracle.bits_of(c["q"]), k=oracle.bits_of(c["k_cache"]), v=oracle.bits_of(c["v_cache"]),
                bt=c["block_tables"].cpu().numpy(), cl=c["context_lens"].cpu().numpy())


def run_oracle(c, pairs=None, bits=None):
    h = host_bits(c) if bits is None else bits
    return oracle.paged_attention(h["q"], h["k"], h["v"], h["bt"], h["cl"], c["scale"], c["dtype"], pairs)


def compare(got, want, what=""):
    got = got.detach().to(torch.float64).cpu().numpy() if isinstance(got, torch.Tensor) else got
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want)
    assert err.max() <= MAX_ABS_TOL, f"{what}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS_TOL, f"{what}: mean-abs {err.mean():.3e}"
    return float(err.max()), float(err.mean())


def check_case(c, prefetch_distance=1, what=""):
    got = run_hip(c, prefetch_distance)
    return compare(got, run_oracle(c), what)
