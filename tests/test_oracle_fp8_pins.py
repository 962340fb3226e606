"""Pins of the 8-bit KV-cache oracle against things other than itself: the E4M3 format's defining
values, a library's own E4M3 conversion, brute force over all codes, and reductions to the plain
attention oracle."""
import numpy as np
import pytest
import torch

from oracle import fp8_cache as f8
from oracle import nfd_oracle as orc

ALL = np.arange(256, dtype=np.uint8)
FINITE = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)


def test_decode_matches_the_format_definition():
    d = f8.e4m3_decode(ALL)
    # landmarks of OCP E4M3: bias 7, no infinities, one NaN magnitude
    assert d[0x00] == 0.0 and d[0x38] == 1.0 and d[0x40] == 2.0 and d[0x30] == 0.5
    assert d[0x7E] == 448.0 and d[0x08] == 2.0 ** -6 and d[0x01] == 2.0 ** -9 and d[0x07] == 7 * 2.0 ** -9
    assert d[0x39] == 1.125 and d[0xB8] == -1.0 and d[0xFE] == -448.0
    assert np.isnan(d[0x7F]) and np.isnan(d[0xFF])
    assert np.all(np.diff(d[:0x7F]) > 0)               # magnitudes strictly increase with the code
    assert np.array_equal(d[0x80:0xFF], -d[0x00:0x7F])


def test_decode_matches_a_library_conversion():
    lib = torch.from_numpy(FINITE.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(f8.e4m3_decode(FINITE), lib)


def test_encode_inverts_decode_on_every_code():
    assert np.array_equal(f8.e4m3_encode(f8.e4m3_decode(FINITE).astype(np.float32)), FINITE)


def test_ties_go_to_the_even_code_and_large_values_saturate():
    x = np.array([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, 432.0, 448.0, 1e6, -1e6, np.inf, -0.0, -2.0 ** -11],
                 dtype=np.float32)
    want = [0x38, 0x3A, 0x00, 0x02, 0x7E, 0x7E, 0x7E, 0xFE, 0x7E, 0x80, 0x80]
    # 1.0625 is midway 1.0|1.125 -> 1.0 (0x38, even); 1.1875 midway 1.125|1.25 -> 1.25 (0x3A);
    # 2^-10 midway 0|2^-9 -> 0; 3*2^-10 midway 2^-9|2^-8 -> 2^-8 (0x02); 432 midway 416|448 -> 448 (0x7E)
    assert f8.e4m3_encode(x).tolist() == want


def test_encode_is_the_nearest_value_by_brute_force():
    rng = np.random.default_rng(7)
    x = np.concatenate([rng.standard_normal(4000) * s for s in (1e-3, 0.02, 1.0, 30.0, 300.0)]).astype(np.float32)
    vals = f8.e4m3_decode(FINITE)
    got = f8.e4m3_decode(f8.e4m3_encode(x))
    xc = np.clip(x.astype(np.float64), -448.0, 448.0)
    best = np.abs(vals[None, :] - xc[:, None]).min(axis=1)
    assert np.array_equal(np.abs(got - xc), best)
    assert np.array_equal(np.signbit(got), np.signbit(x))


def test_encode_matches_a_library_conversion_in_range():
    rng = np.random.default_rng(8)
    x = np.concatenate([rng.standard_normal(20000) * s for s in (1e-3, 0.05, 1.0, 100.0)]).astype(np.float32)
    x = x[np.abs(x) <= 448.0]
    mids = (f8.e4m3_decode(np.arange(0, 0x7E, dtype=np.uint8)) + f8.e4m3_decode(np.arange(1, 0x7F, dtype=np.uint8))) / 2
    x = np.concatenate([x, mids.astype(np.float32), -mids.astype(np.float32)])  # every exact tie as well
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(f8.e4m3_encode(x), lib)


def test_quantize_with_power_of_two_scales_is_a_shift_of_the_input():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, 3, 5, 8)).astype(np.float32)
    for k in (-3, 0, 2):
        s = np.full((2, 3, 1, 1), 2.0 ** k, dtype=np.float32)
        assert np.array_equal(f8.quantize(x, s), f8.e4m3_encode(x * np.float32(2.0 ** -k)))
    # and the value read back is within half a step of E4M3 (relative 2^-4) of the input
    s = np.float32(0.05)
    back = f8.e4m3_decode(f8.quantize(x, s)) * float(s)
    big = np.abs(x) > 2.0 ** -6 * float(s)
    assert np.all(np.abs(back - x)[big] <= np.abs(x)[big] * 2.0 ** -4 * (1 + 1e-6))


def test_append_places_codes_and_stores_v_feature_major():
    B, H, T, D, F = 1, 2, 5, 8, 4
    rng = np.random.default_rng(10)
    k8 = np.full((B, H, F * T, D), 0x7F, dtype=np.uint8)
    v8t = np.full((B, H, D, F * T), 0x7F, dtype=np.uint8)
    kn = rng.standard_normal((B, H, 2 * T, D)).astype(np.float32)
    vn = rng.standard_normal((B, H, 2 * T, D)).astype(np.float32)
    ks = np.array([[0.5, 0.01]], dtype=np.float32)
    vs = np.array([[1.0, 0.125]], dtype=np.float32)
    f8.kvcache_append_fp8(k8, v8t, kn, vn, T, 1, ks, vs)
    assert np.all(k8[:, :, :T] == 0x7F) and np.all(k8[:, :, 3 * T:] == 0x7F)
    assert np.all(v8t[:, :, :, :T] == 0x7F) and np.all(v8t[:, :, :, 3 * T:] == 0x7F)
    for h in range(H):
        for tok in (0, 3, 2 * T - 1):
            for d in (0, 5):
                assert k8[0, h, T + tok, d] == f8.e4m3_encode(np.float32(kn[0, h, tok, d]) * (np.float32(1) / ks[0, h]))
                assert v8t[0, h, d, T + tok] == f8.e4m3_encode(np.float32(vn[0, h, tok, d]) * (np.float32(1) / vs[0, h]))
    with pytest.raises(ValueError):
        f8.kvcache_append_fp8(k8, v8t, kn, vn, T, 3, ks, vs)


def test_attention_on_representable_values_is_the_plain_oracle():
    """Inputs that are E4M3 values already (scale 1) lose nothing: the 8-bit path must return what the
    plain attention oracle returns on the same numbers.  Power-of-two scales are exact as well."""
    B, H, T, D, kvf, qf = 1, 2, 6, 8, 4, 2
    rng = np.random.default_rng(11)
    codes = lambda shape: FINITE[rng.integers(0, len(FINITE), size=shape)]
    k = f8.e4m3_decode(codes((B, H, kvf * T, D))) / 64.0
    v = f8.e4m3_decode(codes((B, H, kvf * T, D))) / 64.0
    q = rng.standard_normal((B, H, qf * T, D))
    k8 = np.zeros((B, H, kvf * T + 3, D), dtype=np.uint8)
    v8t = np.zeros((B, H, D, kvf * T + 3), dtype=np.uint8)
    ks = np.array([[2.0 ** -6, 2.0 ** -3]], dtype=np.float32)
    vs = np.array([[2.0 ** -8, 2.0 ** -6]], dtype=np.float32)
    k8[:, :, :kvf * T] = f8.quantize(k, ks[:, :, None, None])
    v8t[:, :, :, :kvf * T] = np.swapaxes(f8.quantize(v, vs[:, :, None, None]), 2, 3)
    k8[:, :, kvf * T:] = 0x7F   # capacity rows hold NaN codes: they must not matter
    v8t[:, :, :, kvf * T:] = 0x7F
    kk, vv = f8.dequantize(k8[:, :, :kvf * T], v8t[:, :, :, :kvf * T], ks, vs)
    # every value survives unless the division pushed it below the subnormal grid or above 448
    ok_k = (np.abs(k) / ks[:, :, None, None] <= 448) & (np.abs(k) / ks[:, :, None, None] >= 2.0 ** -6)
    assert np.array_equal(kk[ok_k], k[ok_k]) and ok_k.mean() > 0.5
    got = f8.block_causal_attn_fp8kv(q, k8, v8t, ks, vs, T, kvf, qf)
    ref = orc.block_causal_attn(q, kk, vv, T, kv_frames=kvf, q_frames=qf)
    assert np.array_equal(got, ref)
    # scaling K's scale by 2 and the queries by 1/2 changes nothing
    got2 = f8.block_causal_attn_fp8kv(q * 0.5, k8, v8t, ks * 2, vs, T, kvf, qf)
    assert np.allclose(got2, ref, rtol=1e-13, atol=1e-15)
    # V's scale is linear in the output
    got3 = f8.block_causal_attn_fp8kv(q, k8, v8t, ks, vs * 4, T, kvf, qf)
    assert np.allclose(got3, 4 * ref, rtol=1e-13, atol=1e-15)


def test_quantisation_error_of_the_attention_output_is_bounded():
    """N(0,1) K and V at a scale that maps 6 sigma to the top of the range: the output over the 8-bit
    cache stays within a few percent (relative L2) of the output over the exact cache - a sanity
    bound on the whole chain, not a parity tolerance."""
    B, H, T, D, kvf = 1, 2, 16, 64, 6
    rng = np.random.default_rng(12)
    q, k, v = (rng.standard_normal((B, H, kvf * T, D)) for _ in range(3))
    s = np.full((B, H), 6.0 / 448.0, dtype=np.float32)
    k8 = f8.quantize(k, s[:, :, None, None])
    v8t = np.swapaxes(f8.quantize(v, s[:, :, None, None]), 2, 3).copy()
    got = f8.block_causal_attn_fp8kv(q, k8, v8t, s, s, T, kvf, kvf)
    ref = orc.block_causal_attn(q, k, v, T, kv_frames=kvf, q_frames=kvf)
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert 1e-3 < rel < 6e-2, rel
