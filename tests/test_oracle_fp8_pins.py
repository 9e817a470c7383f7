"""Pins for the oracle's E4M3 decode and its attention over an fp8 cache (a cache format the paper
does not mention; the attention itself is the paper's: Preliminaries, "Speculative Decoding").

The decode is pinned by the format's closed forms and by the tensor library's own conversion; the
float64 dense-numpy attention is pinned by the C oracle's loop version of the same definition on
inputs both can take, and the multipliers by the identities they must obey."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def test_decode_closed_forms():
    d = oracle.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert d[0x00] == 0.0 and d[0x80] == 0.0 and np.signbit(d[0x80])
    assert d[0x38] == 1.0 and d[0xB8] == -1.0
    assert d[0x7E] == 448.0                       # largest finite value
    assert d[0x01] == 2.0 ** -9                   # smallest subnormal
    assert d[0x07] == 7 * 2.0 ** -9               # largest subnormal
    assert d[0x08] == 2.0 ** -6                   # smallest normal
    assert d[0x40] == 2.0 and d[0x3C] == 1.5 and d[0x39] == 1.125
    assert np.isnan(d[0x7F]) and np.isnan(d[0xFF])
    assert np.isfinite(np.delete(d, [0x7F, 0xFF])).all()
    assert np.all(np.diff(d[:0x7F]) > 0)          # magnitude codes are ordered
    np.testing.assert_array_equal(d[0x80:0xFF], -d[0x00:0x7F])


def test_decode_equals_library_conversion():
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = oracle.e4m3_decode(codes.numpy())
    np.testing.assert_array_equal(np.isnan(lib), np.isnan(ours))
    keep = ~np.isnan(lib)
    np.testing.assert_array_equal(lib[keep], ours[keep])


def test_quantizer_round_trip_is_nearest():
    r = np.random.default_rng(0)
    x = r.standard_normal((2, 3, 50, 16)).astype(np.float32)
    codes, mult = si.quantize_e4m3(x)
    table = oracle.e4m3_decode(np.arange(256, dtype=np.uint8))
    finite = table[~np.isnan(table)]
    y = x / mult[:, :, None, None]
    got = oracle.e4m3_decode(codes)
    best = np.abs(y[..., None] - finite).min(axis=-1)
    np.testing.assert_allclose(np.abs(got - y), best, atol=1e-6)
    assert np.abs(got).max() == 448.0


def _case(seed, B=2, ql=3, H=4, Hkv=2, d=16, ctx=21):
    r = np.random.default_rng(seed)
    q = r.standard_normal((B, ql, H, d)).astype(np.float32)
    k = r.standard_normal((B, Hkv, ctx + ql, d)).astype(np.float32)
    v = r.standard_normal((B, Hkv, ctx + ql, d)).astype(np.float32)
    return q, k, v, ctx


def test_dense_float64_attention_equals_loop_version():
    q, k, v, ctx = _case(1)
    o1, l1 = oracle.attention(q, k, v, ctx)
    o2, l2 = oracle._attention64(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), ctx, None)
    np.testing.assert_allclose(o2, o1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l2, l1, rtol=1e-12, atol=1e-14)


def test_fp8_attention_is_attention_of_the_decoded_cache():
    # multipliers that are powers of two keep multiplier * code exact in float32, so the C oracle
    # can take the dequantised cache directly
    q, k, v, ctx = _case(2)
    kc, _ = si.quantize_e4m3(k)
    vc, _ = si.quantize_e4m3(v)
    ks = np.array([[0.5, 2.0], [0.125, 1.0]], np.float32)
    vs = np.array([[4.0, 0.25], [1.0, 0.0625]], np.float32)
    kd = (oracle.e4m3_decode(kc) * ks[:, :, None, None]).astype(np.float32)
    vd = (oracle.e4m3_decode(vc) * vs[:, :, None, None]).astype(np.float32)
    o1, l1 = oracle.attention(q, kd, vd, ctx)
    o2, l2 = oracle.attention_fp8kv(q, kc, vc, ks, vs, ctx)
    np.testing.assert_allclose(o2, o1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l2, l1, rtol=1e-12, atol=1e-14)
    # planted mistake: the two multipliers exchanged
    o3, _ = oracle.attention_fp8kv(q, kc, vc, vs, ks, ctx)
    assert np.abs(o3 - o1).max() > 1e-2


def test_multiplier_identities():
    q, k, v, ctx = _case(3)
    kc, km = si.quantize_e4m3(k)
    vc, vm = si.quantize_e4m3(v)
    base, lse = oracle.attention_fp8kv(q, kc, vc, km, vm, ctx, 0.2)
    # a K multiplier c is a softmax scale c (c a power of two, so the fp32 multiplier stays exact)
    o, l = oracle.attention_fp8kv(q, kc, vc, km * 4, vm, ctx, 0.2 / 4)
    np.testing.assert_allclose(o, base, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(l, lse, rtol=1e-10, atol=1e-12)
    # the output is linear in the V multiplier, per (batch element, KV head)
    f = np.array([[2.0, 0.5], [3.0, 1.0]])
    o, _ = oracle.attention_fp8kv(q, kc, vc, km, vm * f.astype(np.float32), ctx, 0.2)
    G = q.shape[2] // kc.shape[1]
    np.testing.assert_allclose(o, base * np.repeat(f, G, axis=1)[:, None, :, None], rtol=1e-6)
    # V codes all 1.0: every output element equals the V multiplier
    ones = np.full_like(vc, 0x38)
    o, _ = oracle.attention_fp8kv(q, kc, ones, km, vm, ctx)
    np.testing.assert_allclose(o, np.broadcast_to(np.repeat(vm, G, axis=1)[:, None, :, None], o.shape), rtol=1e-12)


def test_quantizer_closed_forms_and_ties():
    # one head whose maximum is exactly 448: the multiplier is 1 and x itself is encoded
    x = np.zeros((1, 1, 1, 16), np.float32)
    x[0, 0, 0, :12] = [448.0, 1.0, 1.0625, 1.1875, 1.03, -1.09, 2.0 ** -9, 2.0 ** -10, 1.5 * 2.0 ** -9, 0.0, -0.0, 464.0 - 448.0]
    codes, mult = oracle.quantize_e4m3(x)
    assert mult[0, 0] == 1.0
    c = codes[0, 0, 0]
    assert c[0] == 0x7E and c[1] == 0x38
    assert c[2] == 0x38            # 1.0625 lies midway between 1.0 (0x38) and 1.125 (0x39): the even code
    assert c[3] == 0x3A            # 1.1875 lies midway between 1.125 (0x39) and 1.25 (0x3a): the even code
    assert c[4] == 0x38 and c[5] == 0xB9
    assert c[6] == 0x01            # the smallest subnormal
    assert c[7] == 0x00            # half of it: a tie between 0 and 0x01, the even code
    assert c[8] == 0x02            # 1.5 subnormal steps: a tie between 0x01 and 0x02
    assert c[9] == 0x00 and c[10] == 0x80
    assert c[11] == 0x58           # 16.0
    # an all-zero head keeps multiplier 1
    z, m = oracle.quantize_e4m3(np.zeros((1, 2, 3, 16), np.float32))
    assert np.all(z == 0) and np.all(m == 1.0)


def test_quantizer_equals_library_conversion():
    r = np.random.default_rng(5)
    x = (r.standard_normal((2, 3, 257, 64)) * r.uniform(0.01, 50, (2, 3, 1, 1))).astype(np.float32)
    x[0, 0, :5] = 0.0
    codes, mult = oracle.quantize_e4m3(x)
    amax = np.abs(x).max(axis=(2, 3))
    np.testing.assert_array_equal(mult, (amax / np.float32(448.0)).astype(np.float32))
    y = torch.from_numpy((x / mult[:, :, None, None]).astype(np.float32))
    lib = y.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(codes, lib)
    # and the input generator's quantiser is the same function
    c2, m2 = si.quantize_e4m3(x)
    np.testing.assert_array_equal(c2, codes)
    np.testing.assert_array_equal(m2, mult)
    # every code is a nearest neighbour
    table = oracle.e4m3_decode(np.arange(256, dtype=np.uint8))
    finite = table[~np.isnan(table)]
    yv = y.numpy().astype(np.float64)
    best = np.abs(yv[..., None][:1, :1, :50] - finite).min(axis=-1)
    np.testing.assert_allclose(np.abs(oracle.e4m3_decode(codes)[:1, :1, :50] - yv[:1, :1, :50]), best, atol=0)
