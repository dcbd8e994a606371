"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2504_06319_amd as kv
from paper_2504_06319_amd import synth
from kvcheck import check_case, compare, host_bits, run_hip, run_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cfg(Hq, Hkv, d, bs, dtype):
    return dict(Hq=Hq, Hkv=Hkv, d=d, bs=bs, dtype=dtype)


def test_tiny_config_matches_oracle():
    """Benchmark configuration 0: batch 2, MHA 4 heads, d 64, lengths {37, 128}, fp16."""
    c = synth.make_case(synth.CONFIGS[0], synth.config_seed(0), DEV, poison=True)
    for pd in (0, 1, 2):
        check_case(c, pd, f"tiny pd={pd}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("d,bs", [(128, 16), (128, 32), (64, 16), (64, 32)])
@pytest.mark.parametrize("G", [1, 2, 4, 5, 7, 8])
def test_shapes_groups_and_dtypes(dtype, d, bs, G):
    """Several tiles per wave, ragged tails, every supported (d, block_size), the GQA ratios of
    the paper's four models (1, 4, 5, 7) and more."""
    Hkv = 2
    lens = [1, bs - 1, bs, bs + 1, 5 * bs + 3, 333, 700, 64 * bs]
    c = synth.make_case(_cfg(Hkv * G, Hkv, d, bs, dtype), 100 + G, DEV, poison=True, lens=lens)
    for pd in (0, 1, 3):
        check_case(c, pd, f"G={G} d={d} bs={bs} {dtype} pd={pd}")


@pytest.mark.parametrize("pd", list(range(0, kv.KV_MAX_PREFETCH_DISTANCE + 1)))
def test_every_prefetch_distance_gives_the_same_result(pd):
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 7, DEV, poison=True, lens=[3000, 17, 2049, 1024])
    kv.kv_decode_set_waves_per_cu(2)       # fits the LDS at every distance: same worker count, hence the same cuts
    try:
        ref = run_hip(c, 0)
        got = run_hip(c, pd)
    finally:
        kv.kv_decode_set_waves_per_cu(0)
    compare(got, run_oracle(c), f"pd={pd}")
    assert torch.equal(got, ref), "prefetching must not change any value"


def test_missing_workspace_is_reported():
    """Every call needs the registered split-KV scratch; without it the call fails before any launch."""
    from paper_2504_06319_amd import binding
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 3, DEV, lens=[50, 70])
    lib = kv.load_library()
    assert lib.kv_decode_set_workspace(None, 0) == 0
    binding._registered.clear()
    descs = [binding.describe(t) for t in (c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"],
                                           torch.empty_like(c["q"]))]
    import ctypes
    rc = lib.kv_decode_attn(*[ctypes.byref(d) for d in descs], c["scale"], 2, 16, 1, None)
    assert rc == 4 and "workspace" in kv.kv_last_error()
    check_case(c, 1, "after re-registration")          # the binding registers its buffer again


def test_calls_on_two_streams_take_separate_slices_of_the_workspace():
    """Calls enqueued on different streams may overlap in time; each stream gets its own slice of the registered
    workspace, so both results equal the ones computed alone.  Long launches (units cut over every worker) are
    enqueued alternately on two streams, several deep, without any wait in between."""
    a = synth.make_case(_cfg(32, 8, 128, 16, "bf16"), 401, DEV, lens=[60000, 17, 45000, 3000])
    b = synth.make_case(_cfg(32, 8, 128, 16, "bf16"), 402, DEV, lens=[30000, 52000, 1, 9000])
    want_a, want_b = run_hip(a, 2), run_hip(b, 2)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    s1.wait_stream(torch.cuda.current_stream())
    s2.wait_stream(torch.cuda.current_stream())
    outs_a = [torch.full_like(a["q"], float("nan")) for _ in range(6)]
    outs_b = [torch.full_like(b["q"], float("nan")) for _ in range(6)]
    for oa, ob in zip(outs_a, outs_b):
        run_args = lambda c, o, s: kv.kv_decode_attn(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], o,
                                                     c["scale"], c["num_kv_heads"], c["block_size"], 2, s)
        run_args(a, oa, s1)
        run_args(b, ob, s2)
    torch.cuda.synchronize()
    for oa, ob in zip(outs_a, outs_b):
        assert torch.equal(oa.view(torch.int16), want_a.view(torch.int16))
        assert torch.equal(ob.view(torch.int16), want_b.view(torch.int16))


def test_a_stream_that_finds_no_room_in_the_workspace_is_told_so():
    """With a workspace that holds one call's slice, a second stream's call returns status 4 and enqueues nothing;
    registering again releases the slices."""
    import ctypes
    from paper_2504_06319_amd import binding
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 403, DEV, lens=[5000, 700])
    want = run_hip(c, 2)
    lib = kv.load_library()
    need = 4096 + 256 * kv.kv_decode_get_waves_per_cu(2, 128) * 2 * 4 * 132 * 4          # ticket words + this launch's pieces
    small = torch.empty(need + 512, dtype=torch.uint8, device=DEV)
    torch.cuda.synchronize()
    out = torch.full_like(c["q"], 7.0)
    descs = [binding.describe(t) for t in (c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], out)]
    call = lambda stream: lib.kv_decode_attn(*[ctypes.byref(d) for d in descs], c["scale"], 2, 16, 2, ctypes.c_void_p(stream))
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        assert lib.kv_decode_set_workspace(ctypes.c_void_p(small.data_ptr()), small.numel()) == 0
        assert call(s1.cuda_stream) == 0
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16))
        out.fill_(7.0)
        assert call(s2.cuda_stream) == 4 and "stream" in kv.kv_last_error()
        torch.cuda.synchronize()
        assert (out == 7.0).all()
        assert call(s1.cuda_stream) == 0                     # the stream that holds the slice goes on
        torch.cuda.synchronize()
        assert lib.kv_decode_set_workspace(ctypes.c_void_p(small.data_ptr()), small.numel()) == 0
        assert call(s2.cuda_stream) == 0                     # released by the new registration
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    finally:
        torch.cuda.synchronize()
        lib.kv_decode_set_workspace(None, 0)
        binding._registered.clear()
    check_case(c, 1, "after re-registration")


def test_lengths_around_worker_range_boundaries():
    """Contexts whose tile counts straddle the equal shares of the flat tile space, an empty one included."""
    lens = [511, 512, 513, 3 * 512 + 17, 8 * 512, 1, 0, 5 * 512 - 16]
    for d in (128, 64):
        c = synth.make_case(_cfg(8, 2, d, 16, "bf16"), 11, DEV, poison=True, lens=lens)
        got = run_hip(c, 1)
        compare(got, run_oracle(c), f"d={d}")
        assert (got[6] == 0).all()          # empty context -> zero row


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("waves", [1, 3, 8, 16])
@pytest.mark.parametrize("pd", [0, 1, 4])
def test_other_worker_counts_cut_units_differently(waves, pd, d):
    """The number of persistent workers decides where units are cut into pieces;
    every cut must give the same result.  One long sequence spans hundreds of workers, short
    ones are covered whole, empty ones get zero rows."""
    kv.kv_decode_set_waves_per_cu(waves)
    try:
        lens = [40000, 0, 5, 16, 17, 3000, 0, 1, 12345, 640, 0]
        c = synth.make_case(_cfg(8, 2, d, 16, "bf16"), 43 + waves, DEV, poison=True, lens=lens)
        got = run_hip(c, pd)
        compare(got, run_oracle(c), f"waves={waves} pd={pd} d={d}")
        for b, n in enumerate(lens):
            if n == 0:
                assert (got[b] == 0).all()
    finally:
        kv.kv_decode_set_waves_per_cu(0)


@pytest.mark.parametrize("skew", [0, 20, 256])
def test_skewed_shares_of_even_and_odd_workers(skew):
    """Even workers take 1024 + skew parts of the tile space and odd ones 1024 - skew (the two XCDs of a pair
    differ in delivered bandwidth); every skew cuts the units elsewhere and must give the same result."""
    lens = [60000, 0, 33, 45000, 17, 30000, 1, 7000]
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 59, DEV, poison=True, lens=lens)
    trace = torch.zeros((4096, 4), dtype=torch.int64, device=DEV)
    kv.kv_decode_set_waves_per_cu(1)
    kv.kv_decode_set_xcd_skew(skew)
    kv.kv_decode_set_worker_trace(trace)
    try:
        got = run_hip(c, 2)
    finally:
        kv.kv_decode_set_worker_trace(None)
        kv.kv_decode_set_xcd_skew(10)
        kv.kv_decode_set_waves_per_cu(0)
    compare(got, run_oracle(c), f"skew={skew}")
    tiles = trace.cpu().numpy()[:256, 3] & 0xffffffff
    T = sum((n + 15) // 16 for n in lens) * 2
    assert T >= 64 * 256 and tiles.sum() == T
    share = T / 256 / 1024
    assert abs(tiles[0::2].mean() - share * (1024 + skew)) < 1 and abs(tiles[1::2].mean() - share * (1024 - skew)) < 1


def test_single_unit_spanning_every_worker():
    c = synth.make_case(_cfg(4, 1, 128, 32, "f16"), 47, DEV, poison=True, lens=[70001])
    check_case(c, 2, "one unit")


def test_more_sequences_than_lanes_in_the_length_scan():
    rng = np.random.default_rng(5)
    lens = rng.integers(0, 200, 300).tolist()
    c = synth.make_case(_cfg(4, 2, 128, 16, "bf16"), 53, DEV, poison=True, lens=lens)
    check_case(c, 1, "300 sequences")


@pytest.mark.parametrize("G,d", [(16, 128), (12, 128), (16, 64), (3, 64)])
def test_wide_query_groups(G, d):
    """Up to 16 query heads per kv head fill every row of the 16-wide MFMA tile."""
    c = synth.make_case(_cfg(G, 1, d, 16, "bf16"), 200 + G, DEV, poison=True, lens=[1, 17, 400, 2500])
    check_case(c, 2, f"G={G} d={d}")


def test_lengths_beyond_the_table_are_clamped_to_it():
    """context_lens larger than MB * block_size attend over the MB * block_size tokens the table can name."""
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 59, DEV, lens=[160, 320, 48])       # table width 20 blocks
    want = run_oracle(c)
    c2 = dict(c)
    c2["block_tables"] = c["block_tables"][:, :10].contiguous()                           # now 160 tokens at most
    c2["context_lens"] = torch.tensor([160, 10 ** 9, 48], dtype=torch.int32, device=DEV)
    got = run_hip(c2, 1)
    c3 = dict(c, context_lens=torch.tensor([160, 160, 48], dtype=torch.int32, device=DEV))
    want3 = run_oracle(c3)
    compare(got, want3, "clamped")
    compare(got[[0, 2]], want[[0, 2]], "untouched rows")


def test_profile_events_sample_every_nth_call():
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 61, DEV, lens=[600, 900])
    out = torch.empty_like(c["q"])
    kv.kv_profile_enable(3, 2)
    try:
        for _ in range(5):
            run_hip(c, 1, out=out)
        ms, n = kv.kv_profile_read()
        assert n == 3 and 0 < ms / n < 5.0
        ms, n = kv.kv_profile_read()
        assert n == 0
    finally:
        kv.kv_profile_enable(0, 1)


def test_empty_and_single_token_contexts():
    c = synth.make_case(_cfg(4, 4, 64, 16, "f16"), 17, DEV, poison=True, lens=[0, 1, 0, 2])
    got = run_hip(c, 1)
    compare(got, run_oracle(c), "empty")
    assert (got[0] == 0).all() and (got[2] == 0).all()
    blk = int(c["block_tables"][1, 0])
    assert torch.equal(got[1], c["v_cache"][blk, :, 0, :])        # context of one returns V exactly


def test_wide_table_with_poison_entries_and_negative_length():
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 19, DEV, poison=True, lens=[100, 900, 31], table_width=200)
    want = run_oracle(c)
    compare(run_hip(c, 2), want, "wide table")
    c["context_lens"][2] = -5                                      # treated as empty
    got = run_hip(c, 2)
    assert (got[2] == 0).all()
    compare(got[:2], want[:2], "negative length neighbours")


def test_garbage_ids_in_unused_table_entries_are_never_dereferenced():
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 23, DEV, poison=True, lens=[40, 513, 16], table_width=64)
    want = run_oracle(c)
    bt = c["block_tables"]
    for b, n in enumerate(c["lens"]):
        nb = -(-int(n) // 16)
        bt[b, nb:] = torch.tensor([-1, 2 ** 31 - 1, -2 ** 31, 10 ** 9] * 16, dtype=torch.int32, device=DEV)[: 64 - nb]
    compare(run_hip(c, 3), want, "garbage table tail")


def test_validate_inputs_names_the_first_bad_entry():
    """The synchronising checker accepts what the generators make (garbage in unused table entries included) and names
    the first length or block id the kernels would have clamped."""
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 27, DEV, lens=[40, 513, 0, 16], table_width=40)
    nblk = c["k_cache"].shape[0]
    bt = c["block_tables"]
    for b, n in enumerate(c["lens"]):
        bt[b, -(-int(n) // 16):] = -7                       # unused entries may hold anything
    kv.kv_validate_inputs(bt, c["context_lens"], nblk, 16)
    bad = bt.clone(); bad[1, 3] = nblk
    with pytest.raises(kv.KVError) as e:
        kv.kv_validate_inputs(bad, c["context_lens"], nblk, 16)
    assert e.value.status == 1 and "block_tables[1, 3]" in str(e.value)
    lens = c["context_lens"].clone(); lens[3] = 40 * 16 + 1
    with pytest.raises(kv.KVError) as e:
        kv.kv_validate_inputs(bt, lens, nblk, 16)
    assert "context_lens[3]" in str(e.value)
    lens[3] = -1
    with pytest.raises(kv.KVError):
        kv.kv_validate_inputs(bt, lens, nblk, 16)
    with pytest.raises(kv.KVError):
        kv.kv_validate_inputs(bt.to(torch.int64), c["context_lens"], nblk, 16)


def test_permuting_physical_block_ids_changes_nothing():
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 29, DEV, lens=[700, 33, 1500])
    a = run_hip(c, 1)
    nblk = c["k_cache"].shape[0]
    perm = torch.randperm(nblk, generator=torch.Generator().manual_seed(1)).to(DEV)
    c2 = dict(c)
    c2["k_cache"] = torch.empty_like(c["k_cache"]); c2["k_cache"][perm] = c["k_cache"]
    c2["v_cache"] = torch.empty_like(c["v_cache"]); c2["v_cache"][perm] = c["v_cache"]
    c2["block_tables"] = perm[c["block_tables"].long()].to(torch.int32)
    assert torch.equal(run_hip(c2, 1), a)


def test_strided_q_out_and_cache_views_on_a_side_stream():
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 31, DEV, poison=True, lens=[70, 1300])
    want = run_oracle(c)
    qbig = torch.zeros(2, 8, 256, dtype=torch.bfloat16, device=DEV); qbig[:, :, :128] = c["q"]
    obig = torch.zeros(2, 16, 128, dtype=torch.bfloat16, device=DEV)
    kbig = torch.zeros(c["k_cache"].shape[0], 3, 16, 128, dtype=torch.bfloat16, device=DEV)
    vbig = torch.zeros_like(kbig)
    kbig[:, 1:] = c["k_cache"]; vbig[:, 1:] = c["v_cache"]
    c2 = dict(c, q=qbig[:, :, :128], k_cache=kbig[:, 1:], v_cache=vbig[:, 1:])
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        run_hip(c2, 1, out=obig[:, ::2], stream=s)
    compare(obig[:, ::2], want, "strided")
    assert (obig[:, 1::2] == 0).all()


def test_identical_keys_return_mean_of_values():
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 37, DEV, lens=[256, 100])
    c["k_cache"][:] = c["k_cache"][0, 0, 0]
    got = run_hip(c, 1).to(torch.float64).cpu().numpy()
    v = c["v_cache"].to(torch.float64).cpu().numpy(); bt = c["block_tables"].cpu().numpy()
    for b, n in enumerate(c["lens"]):
        rows = np.stack([v[bt[b, t // 16], :, t % 16] for t in range(n)]).mean(0)     # [Hkv, d]
        assert np.abs(got[b].reshape(2, 4, 128) - rows[:, None, :]).max() < 2e-3


def test_large_logits_do_not_overflow():
    c = synth.make_case(_cfg(4, 1, 128, 16, "bf16"), 41, DEV, poison=True, lens=[600])
    c["scale"] = 4.0                       # logits of magnitude ~50: softmax close to one-hot
    check_case(c, 1, "large logits")


@pytest.mark.parametrize("step", [0.05, 0.25, 0.5, -0.5])
@pytest.mark.parametrize("pd", [0, 2])
def test_logits_that_keep_growing_or_falling(step, pd):
    """The running maximum creeps up by less than the kernel's rescale slack per tile, or by more, or never moves
    after the first token: the accumulators are rescaled only now and then, and the result must not care."""
    n = 700
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 43, DEV, poison=True, lens=[n, 333])
    bt = c["block_tables"].cpu().numpy()
    ramp = (torch.arange(n, dtype=torch.float32) * step / 16.0)
    for t in range(n):
        blk = int(bt[0, t // 16])
        c["k_cache"][blk, :, t % 16, :] = 0
        c["k_cache"][blk, :, t % 16, 0] = ramp[t]
    c["q"][0] = 0
    c["q"][0, :, 0] = 16.0                   # logit of token t = step * t (natural log units), before bf16 rounding of K
    c["scale"] = 1.0
    check_case(c, pd, f"ramp {step}")


def test_one_million_token_context():
    """A single unit of 65 537 tiles: every worker holds one piece of it and the merge kernel sees 1 536 pieces."""
    n = (1 << 20) + 7
    c = synth.make_case(_cfg(4, 1, 128, 16, "bf16"), 71, DEV, lens=[n])
    got = run_hip(c, 2)
    pairs = np.array([(0, 0), (0, 3)], np.int32)
    compare(got[0, [0, 3]], run_oracle(c, pairs), "1M tokens")
    assert torch.isfinite(got.float()).all()


def test_four_thousand_short_sequences():
    """A batch far wider than a wave: the length scan runs over 64 chunks and most units are a single tile."""
    rng = np.random.default_rng(9)
    lens = rng.integers(0, 40, 4096).tolist()
    c = synth.make_case(_cfg(4, 2, 64, 16, "f16"), 73, DEV, poison=True, lens=lens)
    check_case(c, 1, "4096 sequences")


# ---------------------------------------------------------------- benchmark configurations at full size
@pytest.mark.parametrize("index", [1, 2, 3])
def test_full_size_configuration_every_row(index):
    """Full benchmark shapes in the launch configurations bench.py times (prefetch distance 2 and 0 at their
    automatic occupancies, which cut the units differently); the oracle computes every (sequence, head) row."""
    cfg = synth.CONFIGS[index]
    c = synth.make_case(cfg, synth.config_seed(index), DEV)
    bits = host_bits(c)
    want = run_oracle(c, bits=bits)
    assert want.shape == (cfg["B"], cfg["Hq"], cfg["d"])
    for pd in (2, 0):
        print(f"{cfg['name']}: prefetch distance {pd}, {kv.kv_decode_get_waves_per_cu(pd, cfg['d'])} waves per compute unit", flush=True)
        got = run_hip(c, pd)
        e_max, e_mean = compare(got, want, f"{cfg['name']} distance {pd}")
        print(f"{cfg['name']}: max-abs {e_max:.2e} mean-abs {e_mean:.2e} over {want.size} elements", flush=True)


@pytest.mark.parametrize("d,bs", [(128, 16), (128, 32), (64, 16), (64, 32)])
def test_fetch_probe_runs_the_fetch_stream_and_writes_nothing(d, bs):
    lens = [700, 0, 33, 1500, 16, 4000, 257, 1]
    c = synth.make_case(_cfg(8, 2, d, bs, "bf16"), 71, DEV, poison=True, lens=lens)
    out = torch.full_like(c["q"], 7.0)
    for pd in range(0, kv.KV_MAX_PREFETCH_DISTANCE + 1):
        kv.kv_decode_fetch_probe(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], out,
                                 c["scale"], c["num_kv_heads"], c["block_size"], pd)
    torch.cuda.synchronize()
    assert (out == 7.0).all()
    check_case(c, 2, "attention after the probe")


@pytest.mark.parametrize("d,bs", [(128, 16), (128, 32), (64, 16), (64, 32)])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_l2_touch_wave_changes_no_bit(d, bs, dtype):
    """The comparison mode with a second wave per worker touching tiles into L2 ahead of it: the worker's own
    arithmetic is that of prefetch_distance 0, so every group size gives the bits of the plain call."""
    lens = [700, 0, 33, 1500, 16, 4000, 257, 1, 2048, 5]
    c = synth.make_case(_cfg(8, 2, d, bs, dtype), 83, DEV, poison=True, lens=lens)
    plain = run_hip(c, 0)
    compare(plain, run_oracle(c), "plain")
    ahead = run_hip(c, 2)                       # taken with the mode off: other distances must ignore the setting
    try:
        for tiles in (1, 3, 8):
            kv.kv_decode_set_l2_touch(tiles)
            got = run_hip(c, 0)
            assert torch.equal(got.view(torch.int16), plain.view(torch.int16)), f"group of {tiles}"
            assert torch.equal(run_hip(c, 2).view(torch.int16), ahead.view(torch.int16)), f"distance 2, group of {tiles}"
    finally:
        kv.kv_decode_set_l2_touch(0)


def test_l2_touch_wave_on_a_full_size_configuration():
    cfg = synth.CONFIGS[1]
    c = synth.make_case(cfg, synth.config_seed(1), DEV)
    try:
        for waves in (2, 6):
            kv.kv_decode_set_waves_per_cu(waves)
            kv.kv_decode_set_l2_touch(0)
            ref = run_hip(c, 0)
            kv.kv_decode_set_l2_touch(4)
            got = run_hip(c, 0)
            assert torch.equal(got.view(torch.int16), ref.view(torch.int16)), f"{waves} waves"
    finally:
        kv.kv_decode_set_l2_touch(0)
        kv.kv_decode_set_waves_per_cu(0)


def test_automatic_prefetch_distance_is_the_measured_best_one():
    """KV_PREFETCH_AUTO resolves to distance 2 on a 16-bit cache and to distance 1 on an 8-bit one: the bits of those
    explicit calls."""
    cfg = _cfg(8, 2, 128, 16, "bf16")
    lens = [900, 0, 17, 2500, 64, 1]
    c = synth.make_case(cfg, 311, DEV, poison=True, lens=lens)
    assert torch.equal(run_hip(c, kv.KV_PREFETCH_AUTO).view(torch.int16), run_hip(c, 2).view(torch.int16))
    c8 = synth.make_case_kv8(cfg, 311, DEV, poison=True, lens=lens, k_scale=0.5, v_scale=2.0)
    outs = []
    for pd in (kv.KV_PREFETCH_AUTO, 1):
        out = torch.full_like(c8["q"], float("nan"))
        kv.kv_decode_attn_kv8(c8["q"], c8["k_cache"], c8["v_cache"], c8["block_tables"], c8["context_lens"], out, c8["scale"],
                              c8["k_scale"], c8["v_scale"], 2, 16, pd)
        torch.cuda.synchronize()
        outs.append(out)
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    with pytest.raises(kv.KVError):
        run_hip(c, -2)


def test_fetches_without_the_non_temporal_hint_change_no_bit():
    """The cache-policy comparison mode (plain KV fetches) is built for the benchmark shapes: same bits as the default,
    and a clear refusal for shapes it was not built for."""
    c = synth.make_case(_cfg(32, 8, 128, 16, "bf16"), 313, DEV, poison=True, lens=[3000, 0, 17, 700, 8192, 1])
    small = synth.make_case(_cfg(4, 4, 64, 16, "f16"), 314, DEV, lens=[100, 30])
    want = {pd: run_hip(c, pd) for pd in (0, 2)}
    kv.kv_decode_set_fetch_policy(kv.KV_FETCH_PLAIN)
    try:
        for pd in (0, 2):
            assert torch.equal(run_hip(c, pd).view(torch.int16), want[pd].view(torch.int16)), f"distance {pd}"
        for case, pd in ((c, 1), (small, 2)):
            with pytest.raises(kv.KVError) as e:
                run_hip(case, pd)
            assert e.value.status == 2 and "KV_FETCH_PLAIN" in str(e.value)
    finally:
        kv.kv_decode_set_fetch_policy(kv.KV_FETCH_NON_TEMPORAL)
    compare(run_hip(small, 2), run_oracle(small), "default policy again")


def test_worker_timeline_accounts_for_every_tile():
    """Every worker reports its entry / range-located / exit clock readings and its tile count: the counts add
    up to the tiles of the batch (per kv head), the readings are ordered, and the result is unchanged."""
    cfg = dict(Hq=8, Hkv=2, d=128, bs=16, dtype="bf16")
    lens = [700, 0, 33, 1500, 16, 4000, 257, 1]
    case = synth.make_case(cfg, 97, DEV, poison=True, lens=lens)
    trace = torch.zeros((4096, 4), dtype=torch.int64, device=DEV)
    kv.kv_decode_set_worker_trace(trace)
    try:
        got = run_hip(case, 2)
        torch.cuda.synchronize()
    finally:
        kv.kv_decode_set_worker_trace(None)
    t = trace.cpu().numpy()
    active = t[t[:, 3] > 0]
    first_wait = (active[:, 3] >> 40) & 0xffff
    xcd, active[:, 3] = (active[:, 3] >> 32) & 0xf, active[:, 3] & 0xffffffff
    assert (first_wait > 0).all() and (first_wait < 0xffff).all()      # the first tile pair took between 10 ns and 0.65 ms
    assert ((xcd >= 0) & (xcd < 8)).all()
    tiles = sum((n + 15) // 16 for n in lens) * cfg["Hkv"]
    assert active[:, 3].sum() == tiles
    assert len(active) == min(tiles, 256 * kv.kv_decode_get_waves_per_cu(2, 128))
    assert (active[:, 0] <= active[:, 1]).all() and (active[:, 1] <= active[:, 2]).all()
    compare(got, run_oracle(case), "traced launch")
    # unregistered again: a later launch leaves the buffer alone
    trace.zero_()
    run_hip(case, 2)
    torch.cuda.synchronize()
    assert int(trace.abs().sum()) == 0


def test_calls_can_be_captured_into_a_graph_and_replayed():
    """kv_decode_attn and kv_decode_attn_kv8 enqueue only kernels on the caller's stream (no allocation, no
    memset, no host synchronisation), so a stream capture records them; every replay, with new inputs copied
    into the captured tensors and eager work in between, must equal the eager result bit for bit."""
    cfg = dict(Hq=8, Hkv=2, d=128, bs=16, dtype="bf16")
    lens = [900, 0, 17, 2500, 64, 1]
    a = synth.make_case(cfg, 211, DEV, poison=True, lens=lens)
    a8 = synth.make_case_kv8(cfg, 211, DEV, poison=True, lens=lens, k_scale=0.5, v_scale=2.0)
    out, out8 = torch.empty_like(a["q"]), torch.empty_like(a["q"])

    def enqueue():
        kv.kv_decode_attn(a["q"], a["k_cache"], a["v_cache"], a["block_tables"], a["context_lens"], out, a["scale"],
                          a["num_kv_heads"], a["block_size"], 2)
        kv.kv_decode_attn_kv8(a8["q"], a8["k_cache"], a8["v_cache"], a8["block_tables"], a8["context_lens"], out8,
                              a8["scale"], a8["k_scale"], a8["v_scale"], a8["num_kv_heads"], a8["block_size"], 1)

    enqueue()                                   # eager warm-up: the workspace is allocated and registered here
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    for rep in range(3):
        # new values, same paging (and so the same poisoned slots)
        b = synth.make_case(cfg, 211, DEV, poison=True, lens=lens, data_seed=300 + rep)
        b8 = synth.make_case_kv8(cfg, 211, DEV, poison=True, lens=lens, k_scale=0.5, v_scale=2.0, data_seed=300 + rep)
        for key in ("q", "k_cache", "v_cache"):
            a[key].copy_(b[key])
            a8[key].copy_(b8[key])
        want, want8 = torch.empty_like(out), torch.empty_like(out8)
        kv.kv_decode_attn(b["q"], b["k_cache"], b["v_cache"], a["block_tables"], a["context_lens"], want, a["scale"],
                          a["num_kv_heads"], a["block_size"], 2)
        kv.kv_decode_attn_kv8(b8["q"], b8["k_cache"], b8["v_cache"], a8["block_tables"], a8["context_lens"], want8,
                              a8["scale"], a8["k_scale"], a8["v_scale"], a8["num_kv_heads"], a8["block_size"], 1)
        torch.cuda.synchronize()
        out.fill_(float("nan"))
        out8.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"replay {rep}"
        assert torch.equal(out8.view(torch.int16), want8.view(torch.int16)), f"replay {rep}, 8-bit cache"
        assert torch.isfinite(out.float()).all() and torch.isfinite(out8.float()).all()
    compare(out, run_oracle(a), "last replay")


@pytest.mark.parametrize("seed", list(range(12)))
def test_randomised_shapes_lengths_and_launch_settings(seed):
    """Seeded random draws over everything a caller can vary: batch, group size, kv heads, head_dim, block size,
    type, length mix (including empty and one-token sequences), table width, prefetch distance, waves per compute
    unit, and the 16-bit or 8-bit cache."""
    rng = np.random.default_rng(1000 + seed)
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16]))
    Hkv = int(rng.choice([1, 2, 4, 8]))
    d = int(rng.choice([64, 128]))
    bs = int(rng.choice([16, 32]))
    dtype = str(rng.choice(["bf16", "f16"]))
    B = int(rng.integers(1, 40))
    kind = rng.integers(0, 3)
    if kind == 0:
        lens = rng.integers(0, 60, B)                       # tiny contexts, many empty
    elif kind == 1:
        lens = rng.integers(1, 3000, B)
    else:
        lens = np.where(rng.random(B) < 0.2, rng.integers(3000, 20000, B), rng.integers(0, 200, B))   # a few long ones
    lens = lens.astype(np.int64).tolist()
    pd = int(rng.integers(0, kv.KV_MAX_PREFETCH_DISTANCE + 1))
    waves = int(rng.choice([0, 1, 2, 3, 5, 6, 8, 11, 16]))
    width = (max(lens) + bs - 1) // bs + int(rng.integers(0, 5))
    cfg = dict(Hq=G * Hkv, Hkv=Hkv, d=d, bs=bs, dtype=dtype)
    kv8 = bool(rng.integers(0, 2))
    what = f"seed {seed}: B {B} G {G} Hkv {Hkv} d {d} bs {bs} {dtype} pd {pd} waves {waves} kv8 {kv8} kind {kind}"
    print(what, flush=True)
    kv.kv_decode_set_waves_per_cu(waves)
    try:
        if kv8:
            c = synth.make_case_kv8(cfg, 2000 + seed, DEV, poison=True, lens=lens, k_scale=0.75, v_scale=1.5,
                                    table_width=max(width, 1))
            out = torch.full_like(c["q"], float("nan"))
            kv.kv_decode_attn_kv8(c["q"], c["k_cache"], c["v_cache"], c["block_tables"], c["context_lens"], out,
                                  c["scale"], c["k_scale"], c["v_scale"], Hkv, bs, pd)
            torch.cuda.synchronize()
            want = oracle.paged_attention_kv8(oracle.bits_of(c["q"]), c["k_cache"].cpu().numpy(), c["v_cache"].cpu().numpy(),
                                              c["block_tables"].cpu().numpy(), c["context_lens"].cpu().numpy(), c["scale"],
                                              dtype, c["k_scale"], c["v_scale"])
            compare(out, want, what)
        else:
            c = synth.make_case(cfg, 2000 + seed, DEV, poison=True, lens=lens, table_width=max(width, 1))
            compare(run_hip(c, pd), run_oracle(c), what)
    finally:
        kv.kv_decode_set_waves_per_cu(0)
