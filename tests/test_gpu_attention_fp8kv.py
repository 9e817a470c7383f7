"""GPU parity: hippo_verify_attention_fp8kv / hippo_draft_attention_fp8kv (through the C ABI) vs the
CPU oracle's attention over the dequantised cache.  The arithmetic is the bf16 path's (codes convert
to bf16 exactly, the multipliers are fp32 factors), so the bf16 tolerances apply unchanged."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import assert_close, dev, host, prep

pytestmark = pytest.mark.gpu


def codes_dev(c: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(c)).cuda()


def run_case(hippo, q, k, v, ctx, num_splits=0, scale=0.0, fn="verify", what=""):
    q = prep(q, "bf16")
    kc, km = si.quantize_e4m3(k)
    vc, vm = si.quantize_e4m3(v)
    f = hippo.hippo_verify_attention_fp8kv if fn == "verify" else hippo.hippo_draft_attention_fp8kv
    out, lse = f(dev(q, "bf16"), codes_dev(kc), codes_dev(vc), torch.from_numpy(km).cuda(),
                 torch.from_numpy(vm).cuda(), ctx, softmax_scale=scale, num_splits=num_splits, want_lse=True)
    torch.cuda.synchronize()
    ro, rl = oracle.attention_fp8kv(q, kc, vc, km, vm, ctx, scale if scale > 0 else None)
    assert_close(host(out), ro, "bf16", what + " out")
    np.testing.assert_allclose(host(lse), rl, rtol=2.0 ** -9, atol=2.0 ** -9, err_msg=what + " lse")
    return host(out)


def rand_case(seed, B, ql, H, Hkv, d, ctx, qscale=1.0):
    r = np.random.default_rng(seed)
    q = r.standard_normal((B, ql, H, d)) * qscale
    k = r.standard_normal((B, Hkv, ctx + ql, d))
    # unequal magnitudes per (batch element, KV head), so the multipliers differ
    v = r.standard_normal((B, Hkv, ctx + ql, d)) * r.uniform(0.3, 3.0, (B, Hkv, 1, 1))
    return q, k, v


@pytest.mark.parametrize("shape", [
    # B, q_len, H, Hkv, d, ctx
    (1, 1, 4, 4, 64, 1),          # single context row, MHA
    (2, 3, 8, 2, 64, 37),         # ragged, barely more than one tile
    (1, 9, 7, 1, 128, 333),       # R = 63, one KV head
    (2, 5, 16, 2, 128, 1000),     # R = 40
    (1, 6, 28, 4, 128, 2049),     # headline head geometry, tile-boundary tail
    (1, 2, 6, 2, 64, 0),          # empty context: rows see only the new tokens
    (1, 12, 16, 2, 64, 515),      # R = 96 > 64: more than one row chunk
    (1, 1, 28, 4, 128, 832),      # the draft call's shape
])
def test_random_shapes_sharp_softmax(hippo, shape):
    B, ql, H, Hkv, d, ctx = shape
    q, k, v = rand_case(hash(shape) % 1000, B, ql, H, Hkv, d, ctx, qscale=3.0)
    # library-chosen slices, one slice (long slices: the four-group variant), and a few
    for s in (0, 1, 3):
        run_case(hippo, q, k, v, ctx, s, what="%s S=%d" % (shape, s))
    run_case(hippo, q, k, v, ctx, 0, fn="draft", what="%s draft" % (shape,))


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("shape", [
    # q_len, G, ctx, forced slices: slices of at least 24 32-token tiles (four token groups, two stages)
    (1, 7, 4096, 1),              # R = 7: one 16-row block
    (1, 7, 4096, 2),
    (5, 4, 2048, 1),              # R = 20: two row blocks
    (9, 7, 3072, 2),              # R = 63: four row blocks
    (3, 14, 1700, 1),             # R = 42: three row blocks, ragged last tile
])
def test_long_slices_every_row_block_count(hippo, shape, d):
    ql, G, ctx, S = shape
    q, k, v = rand_case(ql * 1000 + G + d, 1, ql, 2 * G, 2, d, ctx, qscale=3.0 if d == 64 else 2.5)
    run_case(hippo, q, k, v, ctx, S, what="fp8 long slices %s d=%d" % (shape, d))


def test_causal_mask_probe_with_one_hot_values(hippo):
    # V = identity (code 0x38 = 1.0): the output IS the probability row; mass beyond ctx+i must be 0
    B, ql, H, Hkv, d, ctx = 1, 6, 4, 2, 128, 100
    n = ctx + ql
    q, k, _ = rand_case(5, B, ql, H, Hkv, d, ctx)
    v = np.zeros((B, Hkv, n, d), np.float32)
    v[:, :, np.arange(n), np.arange(n)] = 1.0
    out = run_case(hippo, q, k, v, ctx, what="probe")
    for i in range(ql):
        assert np.all(out[0, i, :, ctx + i + 1:] == 0.0)
        np.testing.assert_allclose(out[0, i].sum(-1), 1.0, atol=2e-2)
    ones = run_case(hippo, q, k, np.ones_like(v), ctx, what="rows sum to 1")
    np.testing.assert_allclose(ones, 1.0, atol=8e-3)


def test_token_order_probe(hippo):
    # the fp8 path permutes tile rows between the K operand and the V read: give every token its own
    # value vector and a query that picks exactly one token, for every token of two tiles and a tail
    B, H, Hkv, d, n = 1, 2, 1, 64, 75
    r = np.random.default_rng(3)
    k = r.standard_normal((B, Hkv, n, d)).astype(np.float32)
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = r.standard_normal((B, Hkv, n, d)).astype(np.float32)
    kc, km = si.quantize_e4m3(k)
    vc, vm = si.quantize_e4m3(v)
    kdec = oracle.e4m3_decode(kc) * km[:, :, None, None]
    vdec = oracle.e4m3_decode(vc) * vm[:, :, None, None]
    for t in range(n - 1):
        q = np.zeros((B, 1, H, d), np.float32)
        q[0, 0, :, :] = 200.0 * kdec[0, 0, t] / np.linalg.norm(kdec[0, 0, t])
        q = prep(q, "bf16")
        out = hippo.hippo_verify_attention_fp8kv(dev(q, "bf16"), codes_dev(kc), codes_dev(vc),
                                                 torch.from_numpy(km).cuda(), torch.from_numpy(vm).cuda(), n - 1)
        ro, _ = oracle.attention_fp8kv(q, kc, vc, km, vm, n - 1)
        assert_close(host(out), ro, "bf16", "token %d" % t)
    assert np.abs(ro[0, 0, 0] - vdec[0, 0, n - 2]).max() < 0.2     # the probe does isolate one token


def test_strided_caches_and_custom_scale(hippo):
    # K and V interleaved in one allocation ([B,Hkv,N_alloc,2,d]): stride_n = 2d, oversized stride_h
    B, ql, H, Hkv, d, ctx = 2, 4, 6, 3, 64, 150
    q, k, v = rand_case(11, B, ql, H, Hkv, d, ctx)
    q = prep(q, "bf16")
    kc, km = si.quantize_e4m3(k)
    vc, vm = si.quantize_e4m3(v)
    n, n_alloc = ctx + ql, ctx + ql + 13
    buf = torch.zeros((B, Hkv, n_alloc, 2, d), dtype=torch.uint8, device="cuda")
    buf[:, :, :n, 0] = codes_dev(kc)
    buf[:, :, :n, 1] = codes_dev(vc)
    kd, vd = buf[:, :, :, 0], buf[:, :, :, 1]
    assert kd.stride(2) == 2 * d
    out = hippo.hippo_verify_attention_fp8kv(dev(q, "bf16"), kd, vd, torch.from_numpy(km).cuda(),
                                             torch.from_numpy(vm).cuda(), ctx, softmax_scale=0.21)
    torch.cuda.synchronize()
    ro, _ = oracle.attention_fp8kv(q, kc, vc, km, vm, ctx, 0.21)
    assert_close(host(out), ro, "bf16", "strided")


def test_split_count_does_not_change_the_result(hippo):
    q, k, v = rand_case(12, 1, 5, 28, 4, 128, 3000)
    outs = [run_case(hippo, q, k, v, 3000, s, what="S=%d" % s) for s in (1, 2, 5, 33)]
    for o in outs[1:]:
        assert np.max(np.abs(o - outs[0])) <= 2 ** -7 * np.max(np.abs(outs[0])) + 1e-6


@pytest.mark.parametrize("name", ["c3_16k", "c4_long"])
def test_full_size(hippo, name):
    """The benchmark shapes with their caches quantised, in the launch configuration bench.py times."""
    cfg = si.CONFIGS[name]
    x = si.make_inputs(cfg, 0)
    run_case(hippo, x["q_new"], x["k"], x["v"], cfg.ctx_len, 0, what=name)


def test_prune_then_draft_attention_on_an_fp8_cache(hippo):
    """The draft path with an 8-bit cache end to end: the gather copies the kept rows' codes (bit
    exact, the per-head multipliers stay valid), and the draft attention over the pruned codes equals
    the oracle's attention over the same rows of the dequantised cache."""
    cfg = si.CONFIGS["draft"]
    x = si.make_inputs(cfg, 4)
    n = cfg.ctx_len + 1                                   # context + the draft token's own row
    kc, km = si.quantize_e4m3(x["k"][:, :, :n])
    vc, vm = si.quantize_e4m3(x["v"][:, :, :n])
    r = np.random.default_rng(0)
    scores = r.standard_normal((cfg.batch, cfg.n_visual)).astype(np.float32)
    k_keep = (cfg.n_visual * cfg.keep_pct + 99) // 100
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    idx, kp, vp = hippo.hippo_select_gather_kv(torch.from_numpy(scores).cuda(), k_keep, codes_dev(kc), codes_dev(vc),
                                               vid, cfg.n_q_heads)
    torch.cuda.synchronize()
    ridx = oracle.topk(scores, k_keep)
    np.testing.assert_array_equal(idx.cpu().numpy(), ridx)
    rows = np.concatenate([np.arange(cfg.n_prefix), cfg.n_prefix + ridx[0],
                           np.arange(cfg.n_prefix + cfg.n_visual, n)])
    assert cfg.batch == 1
    np.testing.assert_array_equal(kp.cpu().numpy(), kc[:, :, rows])
    np.testing.assert_array_equal(vp.cpu().numpy(), vc[:, :, rows])
    q = prep(x["q_new"][:, :1], "bf16")
    ctx = len(rows) - 1
    out = hippo.hippo_draft_attention_fp8kv(dev(q, "bf16"), kp, vp, torch.from_numpy(km).cuda(),
                                            torch.from_numpy(vm).cuda(), ctx)
    torch.cuda.synchronize()
    ro, _ = oracle.attention_fp8kv(q, kc[:, :, rows], vc[:, :, rows], km, vm, ctx)
    assert_close(host(out), ro, "bf16", "draft attention over the pruned fp8 cache")


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("shape", [(1, 1, 1, 64), (2, 3, 77, 64), (1, 4, 1670, 128), (2, 2, 5000, 128)])
def test_quantize_kv_bit_exact(hippo, dtype, shape):
    """The library's writer of the 8-bit format against the oracle's: codes and multipliers bit for bit
    (values spread over eight octaves per head, planted zeros, ties and the subnormal range)."""
    B, Hkv, N, d = shape
    r = np.random.default_rng(N)
    mag = np.exp2(r.uniform(-9, 8, (B, Hkv, N, d)))
    k = prep(r.standard_normal(shape) * mag, dtype)
    v = prep(r.standard_normal(shape) * r.uniform(0.05, 20, (B, Hkv, 1, 1)), dtype)
    k[:, :, ::7, ::5] = 0.0
    v[0, 0] = 0.0                                           # an all-zero head: multiplier 1, codes 0
    if N > 8:
        # one head whose maximum is exactly 448: the values themselves are encoded, ties included
        k[0, -1] = np.clip(k[0, -1], -400, 400)
        k[0, -1, 0, :8] = [448.0, 1.0625, 1.1875, -1.0625, 2.0 ** -10, 1.5 * 2.0 ** -9, 2.5 * 2.0 ** -9, -0.0]
    kd, vd = dev(k, dtype), dev(v, dtype)
    kc, vc, ks, vs = hippo.hippo_quantize_kv_e4m3(kd, vd)
    torch.cuda.synchronize()
    rk, rkm = oracle.quantize_e4m3(k)
    rv, rvm = oracle.quantize_e4m3(v)
    np.testing.assert_array_equal(ks.cpu().numpy(), rkm)
    np.testing.assert_array_equal(vs.cpu().numpy(), rvm)
    np.testing.assert_array_equal(kc.cpu().numpy(), rk)
    np.testing.assert_array_equal(vc.cpu().numpy(), rv)


def test_quantize_strided_prefix_then_attend(hippo):
    """Quantise the first n rows of caches that sit interleaved in one allocation, into a larger code
    buffer, then attend over the codes: equals the oracle's attention over its own quantisation."""
    B, ql, H, Hkv, d, ctx = 2, 3, 8, 2, 128, 300
    q, k, v = rand_case(21, B, ql, H, Hkv, d, ctx)
    q, k, v = prep(q, "bf16"), prep(k, "bf16"), prep(v, "bf16")
    n = ctx + ql
    buf = torch.zeros((B, Hkv, n + 9, 2, d), dtype=torch.bfloat16, device="cuda")
    buf[:, :, :n, 0] = dev(k, "bf16")
    buf[:, :, :n, 1] = dev(v, "bf16")
    buf[:, :, n:] = 1000.0                                   # rows beyond n must not reach the maximum
    codes = torch.full((B, Hkv, n + 20, 2, d), 0x7F, dtype=torch.uint8, device="cuda")
    kc, vc, ks, vs = hippo.hippo_quantize_kv_e4m3(buf[:, :, :, 0], buf[:, :, :, 1], n_rows=n,
                                                  k_codes=codes[:, :, :, 0], v_codes=codes[:, :, :, 1])
    out = hippo.hippo_verify_attention_fp8kv(dev(q, "bf16"), kc, vc, ks, vs, ctx)
    torch.cuda.synchronize()
    rk, rkm = oracle.quantize_e4m3(k)
    rv, rvm = oracle.quantize_e4m3(v)
    np.testing.assert_array_equal(kc[:, :, :n].cpu().numpy(), rk)
    np.testing.assert_array_equal(ks.cpu().numpy(), rkm)
    assert torch.all(codes[:, :, n:] == 0x7F)                # nothing written past n_rows
    ro, _ = oracle.attention_fp8kv(q, rk, rv, rkm, rvm, ctx)
    assert_close(host(out), ro, "bf16", "attention over the library's own quantisation")
