"""Pins of the 8-bit-KV-cache oracle against things other than itself (no GPU).

The FP8 E4M3 decoder is checked on all 256 codes against torch's float8_e4m3fn; the attention on an FP8
cache against (i) torch's fp64 scaled_dot_product_attention on the decoded, scaled K and V and (ii) the
16-bit oracle (itself pinned elsewhere) on the same values written as bf16, which holds every E4M3 value
exactly.  A decoder with the wrong bias, a dropped or swapped scale, or a scale applied on the wrong
side of the softmax fails at least one of them.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2504_06319_amd import synth


def _bits(x, dtype):
    return oracle.bits_of(torch.as_tensor(np.asarray(x, dtype=np.float64)).to(synth.TORCH_DTYPES[dtype]))


def _fp8_codes(x):
    """float64 array -> nearest E4M3 codes (torch's conversion on the CPU)."""
    return torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_fp8_decoding_matches_torch_on_every_code():
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.fp8e4m3_to_f64(codes)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.isnan(got).sum() == 2                      # 0x7f and 0xff, no infinities
    ok = ~np.isnan(got)
    assert np.array_equal(got[ok], want[ok])
    assert got[0x7e] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6 and got[0x38] == 1.0
    assert np.array_equal(np.signbit(got[ok]), codes[ok] >= 128)


def _case(rng, B=3, Hkv=2, G=4, d=32, bs=16, n=75):
    Hq = Hkv * G
    nb = (n + bs - 1) // bs
    nblk = B * nb + 3
    kcode = _fp8_codes(rng.standard_normal((nblk, Hkv, bs, d)))
    vcode = _fp8_codes(rng.standard_normal((nblk, Hkv, bs, d)))
    tables = rng.permutation(nblk)[: B * nb].reshape(B, nb).astype(np.int32)
    Q = torch.as_tensor(rng.standard_normal((B, Hq, d))).to(torch.bfloat16).to(torch.float64).numpy()
    lens = np.array([n, n - 20, 1], np.int32)[:B]
    return dict(B=B, Hkv=Hkv, G=G, Hq=Hq, d=d, bs=bs, Q=Q, kcode=kcode, vcode=vcode, tables=tables, lens=lens)


def _contiguous(c, codes, b):
    """decoded [Hkv, n_b, d] rows of sequence b"""
    n = int(c["lens"][b])
    dec = oracle.fp8e4m3_to_f64(codes)
    rows = [dec[c["tables"][b, t // c["bs"]], :, t % c["bs"], :] for t in range(n)]
    return np.stack(rows, axis=1)


@pytest.mark.parametrize("k_scale,v_scale", [(1.0, 1.0), (0.5, 2.0), (1.7, 0.3)])
def test_matches_library_attention_on_decoded_scaled_values(k_scale, v_scale):
    rng = np.random.default_rng(17)
    c = _case(rng)
    scale = 0.41
    got = oracle.paged_attention_kv8(_bits(c["Q"], "bf16"), c["kcode"], c["vcode"], c["tables"], c["lens"], scale,
                                     "bf16", k_scale, v_scale)
    for b in range(c["B"]):
        K = torch.from_numpy(k_scale * _contiguous(c, c["kcode"], b)).repeat_interleave(c["G"], dim=0)
        V = torch.from_numpy(v_scale * _contiguous(c, c["vcode"], b)).repeat_interleave(c["G"], dim=0)
        q = torch.from_numpy(c["Q"][b])[:, None, :]
        want = torch.nn.functional.scaled_dot_product_attention(q, K, V, scale=scale)[:, 0, :].numpy()
        np.testing.assert_allclose(got[b], want, rtol=0, atol=1e-12)


def test_equals_the_16_bit_oracle_on_the_same_values():
    """bf16 holds every E4M3 value exactly, so the two definitions must agree to rounding of the sums."""
    rng = np.random.default_rng(23)
    c = _case(rng, G=7, n=50)
    kb = _bits(oracle.fp8e4m3_to_f64(c["kcode"]), "bf16")
    vb = _bits(oracle.fp8e4m3_to_f64(c["vcode"]), "bf16")
    scale = 0.3
    want = oracle.paged_attention(_bits(c["Q"], "bf16"), kb, vb, c["tables"], c["lens"], scale, "bf16")
    got = oracle.paged_attention_kv8(_bits(c["Q"], "bf16"), c["kcode"], c["vcode"], c["tables"], c["lens"], scale, "bf16")
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    # k_scale acts like the softmax scale, v_scale multiplies the output
    a = oracle.paged_attention_kv8(_bits(c["Q"], "bf16"), c["kcode"], c["vcode"], c["tables"], c["lens"], scale, "bf16", 2.0, 3.0)
    b = oracle.paged_attention(_bits(c["Q"], "bf16"), kb, vb, c["tables"], c["lens"], 2.0 * scale, "bf16")
    np.testing.assert_allclose(a, 3.0 * b, rtol=0, atol=1e-12)


def test_fp16_queries_pairs_and_empty_rows():
    rng = np.random.default_rng(29)
    c = _case(rng)
    c["lens"][1] = 0
    qh = oracle.bits_of(torch.as_tensor(c["Q"]).to(torch.float16))
    full = oracle.paged_attention_kv8(qh, c["kcode"], c["vcode"], c["tables"], c["lens"], 0.2, "f16")
    assert not full[1].any()
    pairs = [(2, 5), (0, 0), (0, 7)]
    sub = oracle.paged_attention_kv8(qh, c["kcode"], c["vcode"], c["tables"], c["lens"], 0.2, "f16", pairs=pairs)
    for i, (b, h) in enumerate(pairs):
        assert np.array_equal(sub[i], full[b, h])
    # context of one returns the scaled V row exactly
    v0 = 1.5 * oracle.fp8e4m3_to_f64(c["vcode"])[c["tables"][2, 0], :, 0, :]
    one = oracle.paged_attention_kv8(qh, c["kcode"], c["vcode"], c["tables"], c["lens"], 0.2, "f16", 1.0, 1.5)
    for h in range(c["Hq"]):
        assert np.array_equal(one[2, h], v0[h // c["G"]])


def test_unowned_codes_are_never_read_and_bad_ids_are_errors():
    rng = np.random.default_rng(31)
    c = _case(rng)
    base = oracle.paged_attention_kv8(_bits(c["Q"], "bf16"), c["kcode"], c["vcode"], c["tables"], c["lens"], 0.2, "bf16")
    kc, vc = c["kcode"].copy(), c["vcode"].copy()
    owned = np.zeros(kc.shape[0] * kc.shape[2], bool).reshape(kc.shape[0], kc.shape[2])
    for b in range(c["B"]):
        for t in range(int(c["lens"][b])):
            owned[c["tables"][b, t // c["bs"]], t % c["bs"]] = True
    unowned = np.broadcast_to(~owned[:, None, :, None], kc.shape)
    kc[unowned] = 0x7f                                  # NaN code in every slot nobody owns
    vc[unowned] = 0xff
    again = oracle.paged_attention_kv8(_bits(c["Q"], "bf16"), kc, vc, c["tables"], c["lens"], 0.2, "bf16")
    assert np.array_equal(base, again)
    bad = c["tables"].copy(); bad[0, 0] = kc.shape[0]
    with pytest.raises(RuntimeError):
        oracle.paged_attention_kv8(_bits(c["Q"], "bf16"), kc, vc, bad, c["lens"], 0.2, "bf16")
