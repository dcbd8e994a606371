"""Parity of the two-phase variant of kv_decode_attn (logits of a chunk first, then the V tiles: the form of the
kernel the paper patches) with the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2504_06319_amd as kv
from paper_2504_06319_amd import synth
from kvcheck import compare, run_hip, run_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True)
def two_phase_variant():
    kv.kv_decode_set_variant(kv.KV_VARIANT_TWO_PHASE)
    yield
    kv.kv_decode_set_variant(kv.KV_VARIANT_ONE_PASS)
    kv.kv_decode_set_waves_per_cu(0)


def _cfg(Hq, Hkv, d, bs, dtype):
    return dict(Hq=Hq, Hkv=Hkv, d=d, bs=bs, dtype=dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("d,bs", [(128, 16), (128, 32), (64, 16), (64, 32)])
@pytest.mark.parametrize("G", [1, 4, 7, 16])
def test_shapes_groups_and_dtypes(dtype, d, bs, G):
    lens = [1, 15, 16, 17, 100, 333, 0, 1000, 511, 512, 513]
    c = synth.make_case(_cfg(2 * G, 2, d, bs, dtype), 200 + G + d + bs, DEV, poison=True, lens=lens)
    got = run_hip(c, 2)
    compare(got, run_oracle(c), f"{dtype} d{d} bs{bs} G{G}")
    assert not got[6].any()                     # empty context -> zero row


@pytest.mark.parametrize("pd", list(range(0, kv.KV_MAX_PREFETCH_DISTANCE + 1)))
def test_every_prefetch_distance_gives_the_same_bits(pd):
    """Chunks of 32 tiles: lengths on and next to the chunk boundaries, several chunks per unit."""
    lens = [511, 512, 513, 1023, 1024, 1025, 3 * 512 + 17, 5000, 1, 0, 31 * 16, 33 * 16]
    c = synth.make_case(_cfg(8, 2, 128, 16, "bf16"), 211, DEV, poison=True, lens=lens)
    kv.kv_decode_set_waves_per_cu(2)            # the cuts depend on the worker count: keep it fixed
    got = run_hip(c, pd)
    ref = run_hip(c, 0)
    assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
    compare(got, run_oracle(c), f"distance {pd}")


@pytest.mark.parametrize("waves", [1, 2, 3, 4])
@pytest.mark.parametrize("d", [128, 64])
def test_worker_counts_cut_units_and_chunks_differently(waves, d):
    lens = [40000, 0, 5, 16, 17, 3000, 0, 1, 12345, 640, 0]
    c = synth.make_case(_cfg(8, 2, d, 16, "bf16"), 220 + waves, DEV, poison=True, lens=lens)
    kv.kv_decode_set_waves_per_cu(waves)
    for pd in (0, 1, 3):
        got = run_hip(c, pd)
        compare(got, run_oracle(c), f"{waves} waves, distance {pd}, d {d}")
        for b, n in enumerate(lens):
            if n == 0:
                assert not got[b].any()


def test_single_unit_spanning_every_worker_and_tiny_batches():
    c = synth.make_case(_cfg(4, 1, 128, 32, "f16"), 231, DEV, poison=True, lens=[70001])
    compare(run_hip(c, 2), run_oracle(c), "one long sequence")
    c = synth.make_case(_cfg(4, 1, 128, 16, "bf16"), 232, DEV, poison=True, lens=[0, 0, 1, 0])
    got = run_hip(c, 1)
    assert not got[0].any() and not got[1].any() and not got[3].any()
    compare(got, run_oracle(c), "mostly empty")


def test_identical_keys_return_mean_of_values_and_large_logits_stay_finite():
    cfg = _cfg(4, 2, 128, 16, "bf16")
    c = synth.make_case(cfg, 233, DEV, lens=[700, 64])
    c["k_cache"][:] = c["k_cache"][0, 0, 0]      # every key equal: uniform weights
    got = run_hip(c, 2)
    compare(got, run_oracle(c), "identical keys")
    c = synth.make_case(cfg, 234, DEV, lens=[900, 33])
    c["q"] *= 40.0
    got = run_hip(c, 2)
    assert torch.isfinite(got.float()).all()
    compare(got, run_oracle(c), "large logits")


@pytest.mark.parametrize("index", [1, 2, 3])
def test_benchmark_configurations_at_full_size_sampled(index):
    cfg = synth.CONFIGS[index]
    c = synth.make_case(cfg, synth.config_seed(index), DEV)
    rng = np.random.default_rng(index)
    lens = c["lens"]
    seqs = sorted({int(np.argmin(lens)), int(np.argmax(lens))} | set(rng.integers(0, cfg["B"], 4).tolist()))
    pairs = np.array([(b, int(h)) for b in seqs for h in rng.choice(cfg["Hq"], 3, replace=False)], np.int32)
    want = run_oracle(c, pairs)
    for pd in (2, 0):
        got = run_hip(c, pd)
        assert torch.isfinite(got.float()).all()
        sub = got[torch.from_numpy(pairs[:, 0]).long().to(DEV), torch.from_numpy(pairs[:, 1]).long().to(DEV)]
        compare(sub, want, f"{cfg['name']}, two-phase, distance {pd}")


def test_one_pass_and_two_phase_agree_to_rounding():
    c = synth.make_case(_cfg(32, 8, 128, 16, "bf16"), 241, DEV, lens=np.random.default_rng(5).integers(1, 6000, 24).tolist())
    two = run_hip(c, 2).float()
    kv.kv_decode_set_variant(kv.KV_VARIANT_ONE_PASS)
    one = run_hip(c, 2).float()
    assert (one - two).abs().max() <= 2e-2


def test_group_sizes_in_any_order_at_the_deepest_look_ahead():
    """The LDS a worker needs grows with the query heads per kv head; the kernel's dynamic-LDS limit is raised once,
    to what the widest group needs, so a narrower group (15 heads: 67 584 bytes at distance 4) followed by the widest
    (16 heads: 69 632 bytes) both launch."""
    for G in (15, 16, 14, 16):
        c = synth.make_case(_cfg(G, 1, 128, 16, "bf16"), 260 + G, DEV, poison=True, lens=[900, 0, 17, 2500])
        compare(run_hip(c, 4), run_oracle(c), f"G = {G} at distance 4")


def test_large_lds_launch_and_graph_capture():
    """G = 16 at prefetch distance 4 needs 68 KB of LDS per worker (beyond the default limit of dynamic LDS, which
    the launch raises once), and the comparison modes enqueue only kernels, so a stream capture records them:
    the two-phase call and a call with the L2 touch wave are captured (eager warm-up first) and every replay must
    equal the eager result bit for bit."""
    cfg = _cfg(32, 2, 128, 16, "bf16")
    lens = [900, 0, 17, 2500, 64, 1]
    a = synth.make_case(cfg, 251, DEV, poison=True, lens=lens)
    out, out_t = torch.empty_like(a["q"]), torch.empty_like(a["q"])

    def enqueue(o2, ot):
        kv.kv_decode_set_variant(kv.KV_VARIANT_TWO_PHASE)
        run_args = (a["q"], a["k_cache"], a["v_cache"], a["block_tables"], a["context_lens"])
        kv.kv_decode_attn(*run_args, o2, a["scale"], a["num_kv_heads"], a["block_size"], 4)
        kv.kv_decode_set_variant(kv.KV_VARIANT_ONE_PASS)
        kv.kv_decode_set_l2_touch(2)
        kv.kv_decode_attn(*run_args, ot, a["scale"], a["num_kv_heads"], a["block_size"], 0)
        kv.kv_decode_set_l2_touch(0)

    try:
        enqueue(out, out_t)
        torch.cuda.synchronize()
        compare(out, run_oracle(a), "eager, 68 KB of LDS per worker")
        compare(out_t, run_oracle(a), "eager, L2 touch wave")
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                enqueue(out, out_t)
        torch.cuda.synchronize()
        for rep in range(3):
            b = synth.make_case(cfg, 251, DEV, poison=True, lens=lens, data_seed=400 + rep)
            for key in ("q", "k_cache", "v_cache"):
                a[key].copy_(b[key])
            want, want_t = torch.empty_like(out), torch.empty_like(out)
            enqueue(want, want_t)
            torch.cuda.synchronize()
            out.fill_(float("nan"))
            out_t.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"replay {rep}, two-phase"
            assert torch.equal(out_t.view(torch.int16), want_t.view(torch.int16)), f"replay {rep}, L2 touch"
        compare(out, run_oracle(a), "last replay")
    finally:
        kv.kv_decode_set_l2_touch(0)
