"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, evaluates the paper's closed forms, and rejects bad
arguments before any kernel launch."""
import ctypes
import os
import re

import pytest
import torch

import paper_2504_06319_amd as kv
from paper_2504_06319_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "kvprefetch.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kv_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = kv.load_library()
    names = _declared_functions()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(binding.EXPORTS)


def test_version_and_error_text():
    assert kv.kv_version() >= 100
    assert isinstance(kv.kv_last_error(), str)


def test_closed_forms_match_the_paper_worked_example():
    # Section 3.3: Eq. 1 gives 4 KB, Eq. 2 gives 512 KB for Table 3's hyper-parameters at batch 1
    assert kv.kv_block_bytes(2, 128, 16) == 4096
    assert kv.kv_iter_working_set_bytes(4096, 128 // 32, 32, 1) == 512 * 1024
    assert (60 << 20) // kv.kv_iter_working_set_bytes(4096, 4, 32, 1) == 120
    assert kv.kv_block_bytes(0, 128, 16) == 0


def test_workspace_size_formula():
    # two partial pieces of min(Hq, 16) rows of d + 4 floats for each of at most 4096 workers
    # 4096 bytes of dense-layer ticket words, then two pieces of min(Hq, 16) rows of d + 4 floats per worker
    assert kv.kv_decode_workspace_bytes(8, 32, 128, 32768, 16) == 4096 + 4096 * 2 * 16 * 132 * 4
    assert kv.kv_decode_workspace_bytes(1, 4, 128, 16, 16) == 4096 + 4096 * 2 * 4 * 132 * 4
    assert kv.kv_decode_workspace_bytes(2, 4, 64, 128, 16) == 4096 + 4096 * 2 * 4 * 68 * 4
    assert kv.kv_decode_workspace_bytes(2, 4, 96, 128, 16) == 0
    # the layer stack with weights in operand order adds two fp32 tiles of 128 x 128 per 128 columns
    assert kv.kv_layerstack_workspace_bytes(32, 128, 14336) == kv.kv_decode_workspace_bytes(1, 32, 128, 16, 16) + 112 * 2 * 128 * 128 * 4
    assert kv.kv_layerstack_workspace_bytes(32, 128, 100) == 0


def test_waves_per_cu_follow_the_lds_budget():
    # automatic choice: many waves with little or no look-ahead, few with deep look-ahead (32-48 KB of KV in
    # flight per compute unit), never fewer than four at head_dim 64
    assert [kv.kv_decode_get_waves_per_cu(d, 128) for d in range(5)] == [6, 6, 2, 2, 2]
    assert [kv.kv_decode_get_waves_per_cu(d, 64) for d in range(5)] == [8, 8, 4, 4, 4]
    # an explicit request is capped by LDS: a worker holds (distance + 1) x 12 KB at head_dim 128 (a stage of 8 KB
    # and a query image of 4 KB; 6 KB at head_dim 64; 8-bit caches: 8 KB and 4 KB), a compute unit has 160 KB
    # 8-bit cache: tile pairs of the same bytes (32 tokens), twice the arithmetic per byte: more waves
    assert [kv.kv_decode_get_waves_per_cu_kv8(d, 128) for d in range(5)] == [6, 3, 3, 3, 2]
    assert [kv.kv_decode_get_waves_per_cu_kv8(d, 64) for d in range(5)] == [8, 8, 8, 6, 4]
    kv.kv_decode_set_waves_per_cu(16)
    try:
        assert [kv.kv_decode_get_waves_per_cu_kv8(d, 128) for d in range(5)] == [13, 6, 4, 3, 2]
        assert [kv.kv_decode_get_waves_per_cu(d, 128) for d in range(5)] == [13, 6, 4, 3, 2]
        assert [kv.kv_decode_get_waves_per_cu(d, 64) for d in range(5)] == [16, 13, 8, 6, 5]
        with pytest.raises(kv.KVError):
            kv.kv_decode_set_waves_per_cu(17)
    finally:
        kv.kv_decode_set_waves_per_cu(0)


def _fake(shape, dtype, ptr=0x1000):
    """A descriptor with a made-up aligned pointer: validation must reject before any launch."""
    t = torch.empty(shape, dtype=dtype)
    d = binding.describe(t)
    d.data = ptr
    return d


def _call(q, k, v, bt, cl, out, scale=0.1, hkv=2, bs=16, pd=1):
    lib = kv.load_library()
    ref = lambda d: ctypes.byref(d) if d is not None else None
    return lib.kv_decode_attn(ref(q), ref(k), ref(v), ref(bt), ref(cl), ref(out), scale, hkv, bs, pd, None)


def _good():
    f = torch.bfloat16
    return dict(q=_fake((3, 8, 128), f), k=_fake((10, 2, 16, 128), f), v=_fake((10, 2, 16, 128), f),
                bt=_fake((3, 4), torch.int32), cl=_fake((3,), torch.int32), out=_fake((3, 8, 128), f))


@pytest.mark.parametrize("mutate,status,needle", [
    (lambda a: a.update(q=None), 1, "null"),
    (lambda a: setattr(a["k"], "data", 0), 1, "null data"),
    (lambda a: a.update(q=_fake((3, 8, 128), torch.float32)), 2, "dtype"),
    (lambda a: a.update(v=_fake((10, 2, 16, 128), torch.float16)), 1, "share one dtype"),
    (lambda a: a.update(bt=_fake((3, 4), torch.float32)), 1, "int32"),
    (lambda a: a.update(q=_fake((3, 7, 128), torch.bfloat16), out=_fake((3, 7, 128), torch.bfloat16)), 1, "divisible"),
    (lambda a: a.update(out=_fake((3, 8, 64), torch.bfloat16)), 1, "out shape"),
    (lambda a: a.update(k=_fake((10, 2, 32, 128), torch.bfloat16)), 1, "differ"),
    (lambda a: a.update(bt=_fake((2, 4), torch.int32)), 1, "batch"),
    (lambda a: a.update(q=_fake((3, 8, 128, 1), torch.bfloat16)), 1, "rank"),
    (lambda a: setattr(a["q"], "data", 0x1002), 1, "aligned"),
    (lambda a: a["k"].stride.__setitem__(2, 256), 1, "dense"),
    (lambda a: a.update(q=_fake((3, 8, 96), torch.bfloat16), out=_fake((3, 8, 96), torch.bfloat16),
                        k=_fake((10, 2, 16, 96), torch.bfloat16), v=_fake((10, 2, 16, 96), torch.bfloat16)), 2, "head_dim"),
])
def test_invalid_arguments_are_rejected_before_launch(mutate, status, needle):
    a = _good()
    mutate(a)
    rc = _call(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["out"])
    assert rc == status, kv.kv_last_error()
    assert needle in kv.kv_last_error()


def test_scalar_arguments_are_checked():
    a = _good()
    assert _call(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["out"], pd=-2) == 1      # -1 is KV_PREFETCH_AUTO
    assert _call(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["out"], pd=kv.KV_MAX_PREFETCH_DISTANCE + 1) == 1
    assert _call(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["out"], hkv=0) == 1
    f = torch.bfloat16
    a.update(k=_fake((10, 2, 8, 128), f), v=_fake((10, 2, 8, 128), f))
    assert _call(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["out"], bs=8) == 2


def test_kv8_entry_point_checks_cache_type_scales_and_alignment():
    lib = kv.load_library()
    ref = ctypes.byref
    f8 = torch.float8_e4m3fn

    def call(a, ks=1.0, vs=1.0):
        return lib.kv_decode_attn_kv8(ref(a["q"]), ref(a["k"]), ref(a["v"]), ref(a["bt"]), ref(a["cl"]), ref(a["out"]),
                                      0.1, ks, vs, 2, 16, 1, None)

    a = _good()
    assert call(a) == 1 and "FP8" in kv.kv_last_error()                    # 16-bit caches
    a.update(k=_fake((10, 2, 16, 128), f8), v=_fake((10, 2, 16, 128), f8))
    for ks, vs in ((0.0, 1.0), (1.0, -1.0), (float("inf"), 1.0), (1.0, float("nan"))):
        assert call(a, ks, vs) == 1 and "scale" in kv.kv_last_error()
    a["k"].stride[0] = 2 * 16 * 128 + 8                                    # block stride not a multiple of 16 bytes
    assert call(a) == 1 and "aligned" in kv.kv_last_error()
    a = _good()
    a.update(k=_fake((10, 2, 16, 128), f8), v=_fake((10, 2, 16, 128), f8))
    assert _call(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["out"]) == 1  # 8-bit caches through the 16-bit entry point
    # valid arguments get past validation: without a GPU the device query fails (3), with one the missing
    # workspace is reported (4); nothing is launched either way
    lib.kv_decode_set_workspace(None, 0)
    binding._registered.clear()
    assert call(a) in (3, 4)


def test_workspace_registration_arguments_are_checked():
    lib = kv.load_library()
    assert lib.kv_decode_set_workspace(None, 0) == 0
    assert lib.kv_decode_set_workspace(ctypes.c_void_p(0x1000), 0) == 1
    assert lib.kv_decode_set_workspace(None, 64) == 1
    assert lib.kv_decode_set_workspace(ctypes.c_void_p(0x1004), 64) == 1
    binding._registered.clear()


def test_worker_trace_registration_arguments_are_checked():
    lib = kv.load_library()
    assert lib.kv_decode_set_worker_trace(None, 0) == 0
    assert lib.kv_decode_set_worker_trace(ctypes.c_void_p(0x1000), 0) == 1
    assert lib.kv_decode_set_worker_trace(None, 64) == 1
    assert lib.kv_decode_set_worker_trace(ctypes.c_void_p(0x1004), 64) == 1


def test_variant_switch_and_its_occupancy():
    lib = kv.load_library()
    assert lib.kv_decode_set_variant(2) == 1 and lib.kv_decode_set_variant(-1) == 1
    try:
        kv.kv_decode_set_variant(kv.KV_VARIANT_TWO_PHASE)
        # a worker holds 2 d + 1 tiles of 4 KB (head_dim 128) and 32 x G x 64 bytes of logits
        assert [kv.kv_decode_get_waves_per_cu_for(d, 128, 4) for d in range(5)] == [12, 6, 4, 4, 3]
        assert [kv.kv_decode_get_waves_per_cu_for(d, 128, 16) for d in range(5)] == [4, 3, 3, 2, 2]
        assert [kv.kv_decode_get_waves_per_cu(d, 128) for d in range(5)] == [4, 3, 3, 2, 2]
        assert kv.kv_decode_get_waves_per_cu_for(0, 128, 17) == 0 and kv.kv_decode_get_waves_per_cu_for(0, 96, 4) == 0
    finally:
        kv.kv_decode_set_variant(kv.KV_VARIANT_ONE_PASS)
    assert [kv.kv_decode_get_waves_per_cu_for(d, 128, 4) for d in range(5)] == [6, 6, 2, 2, 2]


def test_l2_touch_range_is_checked():
    lib = kv.load_library()
    assert lib.kv_decode_set_l2_touch(-1) == 1 and lib.kv_decode_set_l2_touch(9) == 1
    assert lib.kv_decode_set_l2_touch(4) == 0 and lib.kv_decode_set_l2_touch(0) == 0


def test_validate_inputs_checks_its_descriptors_first():
    lib = kv.load_library()
    a = _good()
    ref = ctypes.byref
    assert lib.kv_validate_inputs(None, None, 10, 16, None) == 1
    assert lib.kv_validate_inputs(ref(a["bt"]), ref(a["cl"]), 0, 16, None) == 1          # no blocks
    assert lib.kv_validate_inputs(ref(a["bt"]), ref(a["cl"]), 10, 8, None) == 1          # block size
    assert lib.kv_validate_inputs(ref(a["q"]), ref(a["cl"]), 10, 16, None) == 1          # not an int32 table


def test_fetch_policy_is_checked():
    lib = kv.load_library()
    assert lib.kv_decode_set_fetch_policy(2) == 1 and lib.kv_decode_set_fetch_policy(-1) == 1
    assert lib.kv_decode_set_fetch_policy(kv.KV_FETCH_PLAIN) == 0 and lib.kv_decode_set_fetch_policy(kv.KV_FETCH_NON_TEMPORAL) == 0


def test_xcd_skew_range_is_checked():
    lib = kv.load_library()
    assert lib.kv_decode_set_xcd_skew(-1) == 1 and lib.kv_decode_set_xcd_skew(257) == 1
    assert lib.kv_decode_set_xcd_skew(0) == 0 and lib.kv_decode_set_xcd_skew(10) == 0


def test_operand_order_packing_places_every_element():
    # Wp[t, ks, nb, l, j] = W[32 ks + 8 (l // 16) + j, 64 t + 16 nb + l % 16], checked element by element
    import torch
    K, N = 64, 128
    w = torch.arange(K * N, dtype=torch.int32).reshape(K, N).to(torch.float32)
    wp = kv.pack_weights(w, "operand")
    assert tuple(wp.shape) == (N // 64, K // 32, 4, 64, 8) and wp.is_contiguous()
    for t in range(N // 64):
        for ks in range(K // 32):
            for nb in range(4):
                for l in range(64):
                    for j in range(8):
                        assert wp[t, ks, nb, l, j] == w[32 * ks + 8 * (l // 16) + j, 64 * t + 16 * nb + l % 16]
    tile = kv.pack_weights(w, "tile")
    assert tuple(tile.shape) == (1, K, 128) and torch.equal(tile[0], w)
    with pytest.raises(kv.KVError):
        kv.pack_weights(w, "columns")
