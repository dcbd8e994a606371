"""Pins of the CPU oracle against things other than itself.

Every check here runs without a GPU.  Together they are chosen so that a plausible
mistake in the oracle (dropped scale, wrong sign in the exponent, wrong kv-head map,
wrong block/slot indexing, K and V swapped, missing normalisation, wrong 16-bit
decoding) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2504_06319_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_kv(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                out[k.strip()] = v.strip()
    return out


def _bits(x, dtype):
    return oracle.bits_of(torch.as_tensor(np.asarray(x, dtype=np.float64)).to(synth.TORCH_DTYPES[dtype]))


def _page(K, V, bs, rng, dtype, extra_blocks=3):
    """Scatter contiguous K,V [B,Hkv,n,d] (float64, exactly representable) into a paged cache."""
    B, Hkv, n, d = K.shape
    nb = (n + bs - 1) // bs
    nblk = B * nb + extra_blocks
    perm = rng.permutation(nblk)
    tables = np.zeros((B, nb), dtype=np.int32)
    kc = rng.standard_normal((nblk, Hkv, bs, d))
    vc = rng.standard_normal((nblk, Hkv, bs, d))
    pos = 0
    for b in range(B):
        for j in range(nb):
            blk = perm[pos]; pos += 1
            tables[b, j] = blk
            t0, t1 = j * bs, min(n, (j + 1) * bs)
            kc[blk, :, : t1 - t0] = K[b, :, t0:t1]
            vc[blk, :, : t1 - t0] = V[b, :, t0:t1]
    return _bits(kc, dtype), _bits(vc, dtype), tables


def _rounded(x, dtype):
    return torch.as_tensor(x).to(synth.TORCH_DTYPES[dtype]).to(torch.float64).numpy()


# ----------------------------------------------------------------------------- decoding
def test_fp16_decoding_matches_numpy_on_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen_bits(bits, "f16")
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == want[~nan]).all()
    assert (np.signbit(got[~nan]) == np.signbit(want[~nan])).all()


def test_bf16_decoding_matches_torch_on_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen_bits(bits, "bf16")
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == want[~nan]).all()


# ----------------------------------------------------------------------------- closed forms
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_hand_worked_two_token_example(dtype):
    g = _read_kv(os.path.join(GOLDEN, "hand_worked_attention.txt"))
    vec = lambda k: np.array([float(x) for x in g[k].split()])
    q = _bits(vec("q").reshape(1, 1, 2), dtype)
    kc = _bits(np.stack([vec("k0"), vec("k1")]).reshape(1, 1, 2, 2), dtype)
    vc = _bits(np.stack([vec("v0"), vec("v1")]).reshape(1, 1, 2, 2), dtype)
    tables = np.zeros((1, 1), np.int32)
    lens = np.array([2], np.int32)
    scale = math.log(float(g["scale_is_ln"]))
    out = oracle.paged_attention(q, kc, vc, tables, lens, scale, dtype)
    _, probs = oracle.paged_attention_probs(q, kc, vc, tables, lens, scale, dtype, 0, 0)
    np.testing.assert_allclose(probs, vec("probs"), rtol=0, atol=1e-15)
    np.testing.assert_allclose(out[0, 0], vec("out"), rtol=0, atol=1e-14)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("G", [1, 4, 7])
def test_matches_non_paged_library_attention(dtype, G):
    """Paged oracle == torch's fp64 scaled_dot_product_attention on the contiguous K, V."""
    rng = np.random.default_rng(5 + G)
    B, Hkv, d, bs, n = 3, 2, 32, 16, 75          # 75 = 4 full blocks + ragged tail of 11
    Hq = Hkv * G
    K = _rounded(rng.standard_normal((B, Hkv, n, d)), dtype)
    V = _rounded(rng.standard_normal((B, Hkv, n, d)), dtype)
    Q = _rounded(rng.standard_normal((B, Hq, d)), dtype)
    kc, vc, tables = _page(K, V, bs, rng, dtype)
    lens = np.full(B, n, np.int32)
    scale = 0.37
    got = oracle.paged_attention(_bits(Q, dtype), kc, vc, tables, lens, scale, dtype)
    Kt = torch.from_numpy(K).repeat_interleave(G, dim=1)      # head h uses kv head h // G
    Vt = torch.from_numpy(V).repeat_interleave(G, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[:, :, None, :], Kt, Vt, scale=scale)[:, :, 0, :].numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_matches_scipy_softmax_with_mixed_lengths():
    from scipy.special import softmax
    rng = np.random.default_rng(11)
    B, Hkv, G, d, bs = 4, 2, 2, 16, 16
    lens = np.array([1, 16, 17, 50], np.int32)
    nmax = 50
    K = _rounded(rng.standard_normal((B, Hkv, nmax, d)), "bf16")
    V = _rounded(rng.standard_normal((B, Hkv, nmax, d)), "bf16")
    Q = _rounded(rng.standard_normal((B, Hkv * G, d)), "bf16")
    kc, vc, tables = _page(K, V, bs, rng, "bf16")
    scale = 1 / math.sqrt(d)
    got = oracle.paged_attention(_bits(Q, "bf16"), kc, vc, tables, lens, scale, "bf16")
    for b in range(B):
        n = lens[b]
        for h in range(Hkv * G):
            p = softmax(scale * (K[b, h // G, :n] @ Q[b, h]))
            np.testing.assert_allclose(got[b, h], p @ V[b, h // G, :n], rtol=0, atol=1e-12)


def _tiny_case(poison=False, seed=3):
    c = synth.make_case(synth.CONFIGS[0], seed, "cpu", poison=poison)
    a = dict(q=oracle.bits_of(c["q"]), k=oracle.bits_of(c["k_cache"]), v=oracle.bits_of(c["v_cache"]),
             bt=c["block_tables"].numpy(), cl=c["context_lens"].numpy(), scale=c["scale"], dt=c["dtype"])
    return c, a


def _run(a, **over):
    a = {**a, **over}
    return oracle.paged_attention(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["scale"], a["dt"])


def test_softmax_rows_sum_to_one_and_are_positive():
    _, a = _tiny_case()
    for b in range(2):
        for h in range(4):
            _, p = oracle.paged_attention_probs(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["scale"], a["dt"], b, h)
            assert p.shape == (a["cl"][b],)
            assert (p > 0).all()
            assert abs(p.sum() - 1.0) < 1e-12


def test_context_of_one_returns_v_exactly():
    c, a = _tiny_case()
    lens = np.array([1, 1], np.int32)
    out = _run(a, cl=lens)
    for b in range(2):
        blk = a["bt"][b, 0]
        want = c["v_cache"][blk, :, 0, :].to(torch.float64).numpy()   # [Hkv, d], MHA here
        assert (out[b] == want).all()


def test_identical_keys_give_mean_of_v():
    c, a = _tiny_case()
    k = c["k_cache"].clone()
    k[:] = k[0, 0, 0]                       # every key row identical
    out = _run(a, k=oracle.bits_of(k))
    v = c["v_cache"].to(torch.float64).numpy()
    for b, n in enumerate(a["cl"]):
        rows = np.stack([v[a["bt"][b, t // 16], :, t % 16] for t in range(n)])   # [n, Hkv, d]
        np.testing.assert_allclose(out[b], rows.mean(0), rtol=0, atol=1e-12)


def test_zero_query_gives_mean_of_v():
    c, a = _tiny_case()
    out = _run(a, q=oracle.bits_of(torch.zeros_like(c["q"])))
    v = c["v_cache"].to(torch.float64).numpy()
    for b, n in enumerate(a["cl"]):
        rows = np.stack([v[a["bt"][b, t // 16], :, t % 16] for t in range(n)])
        np.testing.assert_allclose(out[b], rows.mean(0), rtol=0, atol=1e-12)


def test_invariant_under_permuting_physical_block_ids():
    c, a = _tiny_case()
    nblk = a["k"].shape[0]
    perm = np.random.default_rng(1).permutation(nblk)      # new id of old block i is perm[i]
    k2 = np.empty_like(a["k"]); v2 = np.empty_like(a["v"])
    k2[perm] = a["k"]; v2[perm] = a["v"]
    bt2 = perm[a["bt"]].astype(np.int32)
    assert (_run(a) == _run(a, k=k2, v=v2, bt=bt2)).all()


def test_one_hot_limit_selects_one_value_row():
    rng = np.random.default_rng(2)
    d, n, bs = 16, 40, 16
    K = np.zeros((1, 1, n, d)); V = _rounded(rng.standard_normal((1, 1, n, d)), "f16")
    for t in range(n):
        K[0, 0, t, 1 + t % (d - 1)] = 1.0          # orthogonal to e_0
    hit = 23
    K[0, 0, hit] = 0; K[0, 0, hit, 0] = 64.0
    Q = np.zeros((1, 1, d)); Q[0, 0, 0] = 1.0
    kc, vc, tables = _page(K, V, bs, rng, "f16")
    out = oracle.paged_attention(_bits(Q, "f16"), kc, vc, tables, np.array([n], np.int32), 1.0, "f16")
    np.testing.assert_allclose(out[0, 0], V[0, 0, hit], rtol=0, atol=1e-20)


def test_adding_a_constant_to_every_logit_changes_nothing():
    rng = np.random.default_rng(4)
    d, n, bs = 16, 33, 16
    K = _rounded(rng.standard_normal((1, 1, n, d)), "bf16"); V = _rounded(rng.standard_normal((1, 1, n, d)), "bf16")
    Q = _rounded(rng.standard_normal((1, 1, d)), "bf16")
    K0 = K.copy(); K0[..., 0] = 0; Q0 = Q.copy(); Q0[..., 0] = 0
    K1 = K0.copy(); K1[..., 0] = 1.0; Q1 = Q0.copy(); Q1[..., 0] = 8.0    # +8 on every logit
    lens = np.array([n], np.int32)
    kc0, vc0, t0 = _page(K0, V, bs, np.random.default_rng(9), "bf16")
    kc1, vc1, t1 = _page(K1, V, bs, np.random.default_rng(9), "bf16")
    o0 = oracle.paged_attention(_bits(Q0, "bf16"), kc0, vc0, t0, lens, 1.0, "bf16")
    o1 = oracle.paged_attention(_bits(Q1, "bf16"), kc1, vc1, t1, lens, 1.0, "bf16")
    np.testing.assert_allclose(o0, o1, rtol=0, atol=1e-13)


def test_gqa_with_duplicated_kv_heads_equals_mha():
    rng = np.random.default_rng(6)
    B, Hkv, G, d, bs, n = 2, 2, 3, 16, 16, 45
    K = _rounded(rng.standard_normal((B, Hkv, n, d)), "bf16"); V = _rounded(rng.standard_normal((B, Hkv, n, d)), "bf16")
    Q = _rounded(rng.standard_normal((B, Hkv * G, d)), "bf16")
    lens = np.full(B, n, np.int32)
    kc, vc, t = _page(K, V, bs, np.random.default_rng(1), "bf16")
    gqa = oracle.paged_attention(_bits(Q, "bf16"), kc, vc, t, lens, 0.25, "bf16")
    kcm, vcm, tm = _page(np.repeat(K, G, 1), np.repeat(V, G, 1), bs, np.random.default_rng(1), "bf16")
    mha = oracle.paged_attention(_bits(Q, "bf16"), kcm, vcm, tm, lens, 0.25, "bf16")
    assert (gqa == mha).all()


def test_poisoned_unowned_slots_and_table_entries_are_never_read():
    clean, a = _tiny_case(poison=False)
    dirty, p = _tiny_case(poison=True)
    assert torch.isnan(dirty["k_cache"]).any()
    # widen the table with entries that name the poison block
    wide = np.full((2, 12), clean["poison_id"], np.int32); wide[:, : a["bt"].shape[1]] = p["bt"]
    out = _run(p, bt=wide)
    assert np.isfinite(out).all()
    assert (out == _run(a)).all()


def test_empty_context_gives_zero_row():
    _, a = _tiny_case()
    out = _run(a, cl=np.array([0, 128], np.int32))
    assert (out[0] == 0).all() and np.isfinite(out).all()
    assert (out[1] == _run(a)[1]).all()


def test_split_ranges_merge_by_log_sum_exp():
    """Attention over [0,n) equals the log-sum-exp merge of attention over [0,m) and [m,n)."""
    rng = np.random.default_rng(8)
    d, n, m, bs = 32, 96, 32, 16
    K = _rounded(rng.standard_normal((1, 1, n, d)), "bf16"); V = _rounded(rng.standard_normal((1, 1, n, d)), "bf16")
    Q = _rounded(rng.standard_normal((1, 1, d)), "bf16")
    scale = 1 / math.sqrt(d)
    full_kc, full_vc, full_t = _page(K, V, bs, np.random.default_rng(0), "bf16")
    full = oracle.paged_attention(_bits(Q, "bf16"), full_kc, full_vc, full_t, np.array([n], np.int32), scale, "bf16")[0, 0]
    parts = []
    for lo, hi in ((0, m), (m, n)):
        kc, vc, t = _page(K[:, :, lo:hi], V[:, :, lo:hi], bs, np.random.default_rng(lo + 1), "bf16")
        o = oracle.paged_attention(_bits(Q, "bf16"), kc, vc, t, np.array([hi - lo], np.int32), scale, "bf16")[0, 0]
        s = scale * (K[0, 0, lo:hi] @ Q[0, 0])
        parts.append((o, s.max(), np.exp(s - s.max()).sum()))
    mstar = max(p[1] for p in parts)
    num = sum(o * l * math.exp(mx - mstar) for o, mx, l in parts)
    den = sum(l * math.exp(mx - mstar) for _, mx, l in parts)
    np.testing.assert_allclose(full, num / den, rtol=0, atol=1e-13)


def test_pairs_subset_equals_rows_of_full_result():
    _, a = _tiny_case()
    full = _run(a)
    pairs = np.array([[1, 3], [0, 0], [1, 0]], np.int32)
    sub = oracle.paged_attention(a["q"], a["k"], a["v"], a["bt"], a["cl"], a["scale"], a["dt"], pairs)
    for i, (b, h) in enumerate(pairs):
        assert (sub[i] == full[b, h]).all()


def test_block_id_out_of_range_is_an_error():
    _, a = _tiny_case()
    bt = a["bt"].copy(); bt[0, 0] = a["k"].shape[0]
    with pytest.raises(RuntimeError):
        _run(a, bt=bt)


# ----------------------------------------------------------------------------- Section 3.3
def test_working_set_worked_example_of_the_paper():
    g = {k: int(v) for k, v in _read_kv(os.path.join(GOLDEN, "paper_working_set.txt")).items()}
    mb = oracle.block_bytes(g["bytes_per_element"], g["head_dim"], g["tokens_per_block"])
    assert mb == g["m_block"] == 4 * 1024
    mt = oracle.iteration_working_set_bytes(mb, g["threads_per_block"], g["heads"], g["batch"])
    assert mt == g["m_total"] == 512 * 1024
    assert g["l2_cache_bytes"] == 60 * 1024 * 1024
    assert oracle.max_resident_batches(g["l2_cache_bytes"], mt) == g["max_resident_batches"]


# ----------------------------------------------------------------------------- Algorithm 1
@pytest.mark.parametrize("first,end,warps", [(0, 1, 4), (0, 4, 4), (3, 22, 4), (5, 5, 2), (0, 64, 8), (7, 40, 3)])
@pytest.mark.parametrize("distance", [0, 1, 2, 3])
def test_alg1_block_sets(first, end, warps, distance):
    """Algorithm 1 as sets: between them the warps use every block of the range exactly once; what a warp fetches
    ahead is exactly what it uses `distance` of its own iterations later (so: everything it uses but its first
    `distance` blocks, each fetched once); nothing at or past the range end is ever named."""
    everything = []
    for rank in range(warps):
        used = oracle.blocks_used(first, end, warps, rank)
        assert used == sorted(used) and all(b % warps == (first + rank) % warps for b in used)
        ahead = oracle.fetches_in_flight(first, end, warps, rank, distance)
        assert list(ahead) == used
        fetched = [t for t in ahead.values() if t is not None]
        assert fetched == (used[distance:] if distance else [])
        for block, target in ahead.items():
            if target is not None:
                assert target == block + distance * warps and first <= target < end
            else:
                assert distance == 0 or block + distance * warps >= end        # only the guard suppresses a fetch
        everything += used
    assert sorted(everything) == list(range(first, end))


# ----------------------------------------------------------------------------- layer stack
def test_bf16_rounding_matches_torch_including_ties():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 3, [1.00390625, 1.01171875, -1.00390625, 0.0, 65280.0]])
    got = oracle.round_to_bf16_bits(x)
    want = oracle.bits_of(torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16))
    assert (got == want).all()


def test_layer_gemm_on_small_integers_is_exact():
    rng = np.random.default_rng(1)
    x = rng.integers(-4, 5, (5, 12)).astype(np.float64)
    w = rng.integers(-4, 5, (12, 7)).astype(np.float64)
    y = oracle.layer_gemm_bf16(_bits(x, "bf16"), _bits(w, "bf16"))
    want = np.zeros((5, 7))
    for i in range(5):
        for j in range(7):
            want[i, j] = sum(x[i, k] * w[k, j] for k in range(12))    # |sums| <= 192: exact in bf16
    assert (oracle.widen_bits(y, "bf16") == want).all()


def test_layerstack_layer_uses_leading_columns_as_queries():
    rng = np.random.default_rng(2)
    cfg = dict(Hq=2, Hkv=1, d=16, bs=16, dtype="bf16")
    c = synth.make_case(cfg, 5, "cpu", lens=[20, 33])
    xb = _bits(rng.standard_normal((2, 24)), "bf16"); wb = _bits(rng.standard_normal((24, 40)) * 0.2, "bf16")
    y, out = oracle.layerstack_layer(xb, wb, oracle.bits_of(c["k_cache"]), oracle.bits_of(c["v_cache"]),
                                     c["block_tables"].numpy(), c["context_lens"].numpy(), c["scale"], 2, 16)
    q = y[:, :32].reshape(2, 2, 16)
    want = oracle.paged_attention(q, oracle.bits_of(c["k_cache"]), oracle.bits_of(c["v_cache"]),
                                  c["block_tables"].numpy(), c["context_lens"].numpy(), c["scale"], "bf16")
    assert (out == want).all() and y.shape == (2, 40)
