"""Parity of kv_decode_attn_kv8 (8-bit FP8 E4M3 KV cache) with the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_06319_amd as kv
from paper_2504_06319_amd import synth
from kvcheck import compare

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_hip(c, pd=2, out=None):
    out = torch.full_like(c["q"], float("nan")) if out is None else out
    kv.kv_decode_attn_kv8(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], out,
                          c["scale"], c["k_scale"], c["v_scale"], c["num_kv_heads"], c["block_size"], pd)
    torch.cuda.synchronize()
    return out


def run_oracle(c, pairs=None):
    return oracle.paged_attention_kv8(oracle.bits_of(c["q"]), c["k_cache"].cpu().numpy(), c["v_cache"].cpu().numpy(),
                                      c["block_tables"].cpu().numpy(), c["context_lens"].cpu().numpy(), c["scale"],
                                      c["dtype"], c["k_scale"], c["v_scale"], pairs)


def test_every_fp8_code_is_widened_as_the_oracle_decodes_it():
    """A context of one token returns v_scale * V exactly: put all 254 finite codes into one V row per kv head."""
    for dtype in ("bf16", "f16"):
        cfg = dict(Hq=2, Hkv=2, d=128, bs=16, dtype=dtype)
        c = synth.make_case_kv8(cfg, 5, DEV, lens=[1])
        codes = torch.arange(256, dtype=torch.uint8)
        codes[0x7f] = 0
        codes[0xff] = 0x80
        blk = int(c["block_tables"][0, 0])
        c["v_cache"][blk, :, 0, :] = codes.reshape(2, 128).to(DEV)
        got = run_hip(c).to(torch.float64).cpu().numpy()
        want = oracle.fp8e4m3_to_f64(codes.numpy()).reshape(2, 128)
        # the oracle's values are exactly representable in the output type only above its subnormal range
        # (f16: every E4M3 value is); compare after rounding the oracle's values to the output type
        want_r = torch.from_numpy(want).to(synth.TORCH_DTYPES[dtype]).to(torch.float64).numpy()
        assert np.array_equal(want_r, want)
        assert np.array_equal(got[0], want)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("d,bs", [(128, 16), (128, 32), (64, 16), (64, 32)])
@pytest.mark.parametrize("G", [1, 4, 7, 8])
def test_shapes_groups_and_query_types(dtype, d, bs, G):
    Hkv = 2
    cfg = dict(Hq=Hkv * G, Hkv=Hkv, d=d, bs=bs, dtype=dtype)
    lens = [1, 15, 16, 17, 100, 333, 0, 1000]
    c = synth.make_case_kv8(cfg, 100 + G + d + bs, DEV, poison=True, lens=lens, k_scale=0.5, v_scale=2.0)
    compare(run_hip(c), run_oracle(c), f"{dtype} d{d} bs{bs} G{G}")


@pytest.mark.parametrize("d,bs", [(128, 16), (128, 32), (64, 16), (64, 32)])
def test_lengths_around_the_32_token_tiles(d, bs):
    """The 8-bit kernel walks 32-token tiles, which span two 16-token KV blocks: contexts that end in the first or
    the second block of their last tile, on and next to every boundary, with poisoned slack and table entries."""
    cfg = dict(Hq=8, Hkv=2, d=d, bs=bs, dtype="bf16")
    lens = [16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 2, 0, 95, 96, 97, 1023, 1040]
    c = synth.make_case_kv8(cfg, 77 + d + bs, DEV, poison=True, lens=lens, k_scale=0.75, v_scale=1.25)
    for pd in (0, 2):
        got = run_hip(c, pd)
        compare(got, run_oracle(c), f"d{d} bs{bs} distance {pd}")
        assert not got[12].any()


@pytest.mark.parametrize("pd", list(range(0, kv.KV_MAX_PREFETCH_DISTANCE + 1)))
def test_every_prefetch_distance_gives_the_same_bits(pd):
    cfg = dict(Hq=8, Hkv=2, d=128, bs=16, dtype="bf16")
    rng = np.random.default_rng(7)
    lens = rng.integers(1, 3000, 12).tolist()
    c = synth.make_case_kv8(cfg, 21, DEV, poison=True, lens=lens, k_scale=1.5, v_scale=0.75)
    kv.kv_decode_set_waves_per_cu(2)        # the cuts depend on the worker count: one that fits the LDS at every distance
    try:
        got = run_hip(c, pd)
        ref = run_hip(c, 0)
    finally:
        kv.kv_decode_set_waves_per_cu(0)
    assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
    compare(got, run_oracle(c), f"distance {pd}")


@pytest.mark.parametrize("waves", [1, 3, 8, 16])
@pytest.mark.parametrize("d", [128, 64])
def test_worker_counts(waves, d):
    cfg = dict(Hq=8, Hkv=4, d=d, bs=16, dtype="bf16")
    lens = np.random.default_rng(waves).integers(0, 2500, 20).tolist()
    c = synth.make_case_kv8(cfg, 31 + waves, DEV, poison=True, lens=lens)
    kv.kv_decode_set_waves_per_cu(waves)
    try:
        for pd in (0, 2):
            compare(run_hip(c, pd), run_oracle(c), f"{waves} waves, distance {pd}")
    finally:
        kv.kv_decode_set_waves_per_cu(0)


def test_empty_batch_rows_single_tokens_and_one_long_sequence():
    cfg = dict(Hq=4, Hkv=1, d=128, bs=16, dtype="bf16")
    c = synth.make_case_kv8(cfg, 41, DEV, poison=True, lens=[0, 0, 1, 0])
    got = run_hip(c)
    assert not got[0].any() and not got[1].any() and not got[3].any()
    compare(got, run_oracle(c), "mostly empty")
    c = synth.make_case_kv8(cfg, 43, DEV, poison=True, lens=[70001])      # one unit spread over every worker
    compare(run_hip(c), run_oracle(c), "one long sequence")


@pytest.mark.parametrize("index", [1, 2, 3])
def test_benchmark_configurations_at_full_size_every_row(index):
    """The benchmark configurations with an 8-bit cache at full size, at the distance bench.py times (1) and
    without look-ahead; every (sequence, head) row on the oracle."""
    cfg = synth.CONFIGS[index]
    c = synth.make_case_kv8(cfg, synth.config_seed(index), DEV)
    want = run_oracle(c)
    assert want.shape == (cfg["B"], cfg["Hq"], cfg["d"])
    for pd in (1, 0):
        print(f"{cfg['name']}, 8-bit cache: prefetch distance {pd}", flush=True)
        got = run_hip(c, pd)
        compare(got, want, f"{cfg['name']}, 8-bit cache, distance {pd}")


def test_wrong_cache_type_and_scales_are_rejected():
    cfg = dict(Hq=4, Hkv=2, d=128, bs=16, dtype="bf16")
    c = synth.make_case_kv8(cfg, 51, DEV, lens=[40, 3])
    out = torch.empty_like(c["q"])
    c16 = synth.make_case(cfg, 51, DEV, lens=[40, 3])
    with pytest.raises(kv.KVError) as e:            # 16-bit caches through the 8-bit entry point
        kv.kv_decode_attn_kv8(c["q"], c16["k_cache"], c16["v_cache"], c["block_tables"], c["context_lens"], out,
                              c["scale"], 1.0, 1.0, 2, 16, 1)
    assert e.value.status == 1
    with pytest.raises(kv.KVError) as e:            # 8-bit caches through the 16-bit entry point
        kv.kv_decode_attn(c["q"], c["k_cache"].view(torch.float8_e4m3fn), c["v_cache"].view(torch.float8_e4m3fn),
                          c["block_tables"], c["context_lens"], out, c["scale"], 2, 16, 1)
    assert e.value.status == 1
    for ks, vs in ((0.0, 1.0), (1.0, -2.0), (float("nan"), 1.0), (1.0, float("inf"))):
        with pytest.raises(kv.KVError) as e:
            kv.kv_decode_attn_kv8(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], out,
                                  c["scale"], ks, vs, 2, 16, 1)
        assert e.value.status == 1


def test_strided_cache_views_and_a_side_stream():
    """Caches that are slices of a larger pool (block and head strides larger than dense, still multiples of 16
    bytes), q and out as column slices, launched on a non-default stream."""
    cfg = dict(Hq=8, Hkv=2, d=128, bs=16, dtype="f16")
    c = synth.make_case_kv8(cfg, 61, DEV, poison=True, lens=[500, 31, 1200], v_scale=0.25)
    nblk = c["k_cache"].shape[0]
    big_k = torch.full((nblk, 3, 16, 128), 0x7f, dtype=torch.uint8, device=DEV)     # NaN codes around the real heads
    big_v = torch.full((nblk, 3, 16, 128), 0xff, dtype=torch.uint8, device=DEV)
    big_k[:, :2] = c["k_cache"]
    big_v[:, :2] = c["v_cache"]
    qbig = torch.zeros((3, 8, 256), dtype=torch.float16, device=DEV)
    qbig[:, :, 64:192] = c["q"]
    obig = torch.full((3, 8, 256), float("nan"), dtype=torch.float16, device=DEV)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        kv.kv_decode_attn_kv8(qbig[:, :, 64:192], big_k[:, :2], big_v[:, :2], c["block_tables"], c["context_lens"],
                              obig[:, :, 64:192], c["scale"], c["k_scale"], c["v_scale"], 2, 16, 2)
    s.synchronize()
    assert torch.isnan(obig[:, :, :64]).all() and torch.isnan(obig[:, :, 192:]).all()
    compare(obig[:, :, 64:192], run_oracle(c), "strided views")
