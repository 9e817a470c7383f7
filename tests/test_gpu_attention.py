"""GPU parity: hippo_verify_attention / hippo_draft_attention (through the C ABI) vs the CPU oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import assert_close, dev, host, prep

pytestmark = pytest.mark.gpu


def run_case(hippo, q, k, v, ctx, dtype, num_splits=0, scale=0.0, fn="verify", check_lse=True, what=""):
    q, k, v = prep(q, dtype), prep(k, dtype), prep(v, dtype)
    f = hippo.hippo_verify_attention if fn == "verify" else hippo.hippo_draft_attention
    out, lse = f(dev(q, dtype), dev(k, dtype), dev(v, dtype), ctx, softmax_scale=scale, num_splits=num_splits,
                 want_lse=True)
    torch.cuda.synchronize()
    ro, rl = oracle.attention(q, k, v, ctx, scale if scale > 0 else None)
    assert_close(host(out), ro, dtype, what + " out")
    if check_lse:
        # bf16 path: the denominator sums the bf16-rounded probabilities the PV product uses
        # (relative 2^-9 each), so ln(denominator) is off by at most 2^-9
        tol = 2e-5 if dtype == "fp32" else 2.0 ** -9
        np.testing.assert_allclose(host(lse), rl, rtol=tol, atol=tol, err_msg=what + " lse")
    return host(out)


def rand_case(seed, B, ql, H, Hkv, d, ctx, qscale=1.0, extra_rows=0):
    r = np.random.default_rng(seed)
    q = r.standard_normal((B, ql, H, d)) * qscale
    n = ctx + ql + extra_rows
    k = r.standard_normal((B, Hkv, n, d))
    v = r.standard_normal((B, Hkv, n, d))
    return q, k, v


@pytest.mark.parametrize("name", ["tiny", "draft"])
@pytest.mark.parametrize("num_splits", [0, 1, 3, 16])
def test_verify_on_configs(hippo, name, num_splits):
    cfg = si.CONFIGS[name]
    x = si.make_inputs(cfg, 0)
    run_case(hippo, x["q_new"], x["k"], x["v"], cfg.ctx_len, cfg.dtype, num_splits, what=name)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("shape", [
    # B, q_len, H, Hkv, d, ctx
    (1, 1, 4, 4, 64, 1),          # single context row, MHA
    (2, 3, 8, 2, 64, 37),         # ragged, shorter than one tile
    (1, 9, 7, 1, 128, 333),       # R = 63, one KV head
    (2, 5, 16, 2, 128, 1000),     # R = 40
    (1, 6, 28, 4, 128, 2049),     # headline head geometry, tile-boundary tail
    (1, 2, 6, 2, 64, 0),          # empty context: rows see only the new tokens
    (1, 12, 16, 2, 64, 515),      # R = 96 > 64: more than one row chunk
])
def test_verify_random_shapes_sharp_softmax(hippo, dtype, shape):
    B, ql, H, Hkv, d, ctx = shape
    # logits of std ~3: a handful of keys dominate each row, so a wrong mask or a dropped tile shows
    q, k, v = rand_case(hash(shape) % 1000, B, ql, H, Hkv, d, ctx, qscale=3.0)
    for s in (0, 2):
        run_case(hippo, q, k, v, ctx, dtype, s, what="%s %s S=%d" % (dtype, shape, s))


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("shape", [
    # q_len, G, ctx, forced slices: slices of at least 24 32-token tiles, the long-slice launch shape
    (1, 7, 4096, 1),              # R = 7: one 16-row block (draft attention over an unpruned cache)
    (1, 7, 4096, 2),
    (5, 4, 2048, 1),              # R = 20: two row blocks
    (9, 7, 3072, 2),              # R = 63: four row blocks
    (3, 14, 1700, 1),             # R = 42: three row blocks, ragged last tile
])
def test_verify_long_slices_every_row_block_count(hippo, shape, d):
    ql, G, ctx, S = shape
    q, k, v = rand_case(ql * 1000 + G + d, 1, ql, 2 * G, 2, d, ctx, qscale=3.0 if d == 64 else 2.5)
    run_case(hippo, q, k, v, ctx, "bf16", S, what="long slices %s d=%d" % (shape, d))
    if ql == 1:
        run_case(hippo, q, k, v, ctx, "bf16", S, fn="draft", what="long slices %s d=%d draft" % (shape, d))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_causal_mask_probe_with_one_hot_values(hippo, dtype):
    # V = identity: the output IS the probability row.  Mass beyond ctx+i must be exactly zero.
    B, ql, H, Hkv, d, ctx = 1, 6, 4, 2, 128, 100
    n = ctx + ql
    q, k, _ = rand_case(5, B, ql, H, Hkv, d, ctx)
    v = np.zeros((B, Hkv, n, d), np.float32)
    v[:, :, np.arange(n), np.arange(n)] = 1.0
    out = run_case(hippo, q, k, v, ctx, dtype, what="probe")
    for i in range(ql):
        assert np.all(out[0, i, :, ctx + i + 1:] == 0.0)
        np.testing.assert_allclose(out[0, i].sum(-1), 1.0, atol=2e-2 if dtype == "bf16" else 1e-5)
    ones = run_case(hippo, q, k, np.ones_like(v), ctx, dtype, what="rows sum to 1")
    np.testing.assert_allclose(ones, 1.0, atol=8e-3 if dtype == "bf16" else 1e-6)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_gamma0_is_single_token_decode_and_rows_match_truncated_calls(hippo, dtype):
    B, ql, H, Hkv, d, ctx = 1, 5, 8, 2, 64, 300
    q, k, v = rand_case(7, B, ql, H, Hkv, d, ctx, qscale=2.0)
    full = run_case(hippo, q, k, v, ctx, dtype, what="full")
    for i in range(ql):
        for fn in ("verify", "draft"):
            one = run_case(hippo, q[:, i:i + 1], k[:, :, :ctx + i + 1], v[:, :, :ctx + i + 1], ctx + i, dtype,
                           fn=fn, what="row %d via %s" % (i, fn))
            assert_close(one[:, 0], full[:, i].astype(np.float64), dtype, "row %d vs verify row" % i)


def test_split_count_does_not_change_the_result(hippo):
    cfg = si.CONFIGS["draft"]
    x = si.make_inputs(cfg, 1)
    outs = [run_case(hippo, x["q_new"], x["k"], x["v"], cfg.ctx_len, cfg.dtype, s, what="S=%d" % s)
            for s in (1, 2, 5, 33, 132)]
    for o in outs[1:]:
        assert np.max(np.abs(o - outs[0])) <= 2 ** -7 * np.max(np.abs(outs[0])) + 1e-6


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_strided_caches_and_custom_scale(hippo, dtype):
    # K and V interleaved in one allocation ([B,Hkv,N_alloc,2,d]): stride_n = 2d, oversized stride_h
    B, ql, H, Hkv, d, ctx = 2, 4, 6, 3, 64, 150
    q, k, v = rand_case(11, B, ql, H, Hkv, d, ctx)
    q, k, v = prep(q, dtype), prep(k, dtype), prep(v, dtype)
    n, n_alloc = ctx + ql, ctx + ql + 13
    buf = torch.zeros((B, Hkv, n_alloc, 2, d), dtype=dev(q, dtype).dtype, device="cuda")
    buf[:, :, :n, 0] = dev(k, dtype)
    buf[:, :, :n, 1] = dev(v, dtype)
    kd, vd = buf[:, :, :, 0], buf[:, :, :, 1]
    assert kd.stride(2) == 2 * d
    out = hippo.hippo_verify_attention(dev(q, dtype), kd, vd, ctx, softmax_scale=0.21)
    torch.cuda.synchronize()
    ro, _ = oracle.attention(q, k, v, ctx, 0.21)
    assert_close(host(out), ro, dtype, "strided")


def test_draft_attention_on_full_keep_equals_unpruned(hippo):
    cfg = si.CONFIGS["draft"]
    x = si.make_inputs(cfg, 2)
    dt = cfg.dtype
    kd, vd = dev(x["k"], dt), dev(x["v"], dt)
    q1 = dev(x["q_new"][:, :1], dt)
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    scores = torch.zeros((cfg.batch, cfg.n_visual), dtype=torch.float32, device="cuda")
    n = cfg.ctx_len + 1
    idx, kp, vp = hippo.hippo_select_gather_kv(scores, cfg.n_visual, kd[:, :, :n], vd[:, :, :n], vid, cfg.n_q_heads)
    a = hippo.hippo_draft_attention(q1, kp, vp, cfg.ctx_len)
    b = hippo.hippo_draft_attention(q1, kd, vd, cfg.ctx_len)
    torch.cuda.synchronize()
    assert torch.equal(kp, kd[:, :, :n]) and torch.equal(a, b)


@pytest.mark.parametrize("name", ["c3_16k", "c4_long"])
def test_verify_full_size(hippo, name):
    """The benchmark shapes, in the launch configuration bench.py times (library-chosen splits)."""
    cfg = si.CONFIGS[name]
    x = si.make_inputs(cfg, 0)
    run_case(hippo, x["q_new"], x["k"], x["v"], cfg.ctx_len, cfg.dtype, 0, what=name)


def test_verify_full_size_large_share(hippo):
    """Batch 4 x 8 KV heads x 37K rows, every batch element against the oracle."""
    cfg = si.CONFIGS["c5_large"]
    x = si.make_inputs(cfg, 0)
    dt = cfg.dtype
    out = hippo.hippo_verify_attention(dev(x["q_new"], dt), dev(x["k"], dt), dev(x["v"], dt), cfg.ctx_len)
    torch.cuda.synchronize()
    got = host(out)
    for b in range(cfg.batch):
        ro, _ = oracle.attention(x["q_new"][b:b + 1], x["k"][b:b + 1], x["v"][b:b + 1], cfg.ctx_len)
        assert_close(got[b:b + 1], ro, dt, "c5 batch %d" % b)


# ---------------------------------------------------------------------------------------------
# appended-row fusion: the new rows come from the projection's output and reach the cache in the
# same launch
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("fn", ["verify", "draft"])
@pytest.mark.parametrize("shape", [
    # B, q_len, H, Hkv, d, ctx, num_splits
    (1, 1, 4, 4, 64, 1, 0),
    (2, 3, 8, 2, 64, 37, 0),
    (1, 9, 7, 1, 128, 333, 4),       # new rows inside the last of four slices
    (2, 6, 28, 4, 128, 2049, 0),     # the new rows straddle a tile boundary (2049 = 64 * 32 + 1)
    (1, 12, 16, 2, 64, 515, 3),      # two row chunks
    (1, 40, 4, 2, 64, 24, 2),        # more new rows than context: they span both slices
    (1, 2, 6, 2, 64, 0, 0),          # empty context
    (2, 4, 16, 4, 128, 1900, 2),     # long slices (rotated start): the new rows sit in the middle of the walk
])
def test_append_fusion(hippo, dtype, fn, shape):
    B, ql, H, Hkv, d, ctx, ns = shape
    q, k, v = rand_case(sum(shape), B, ql, H, Hkv, d, ctx, extra_rows=3)
    q, k, v = prep(q, dtype), prep(k, dtype), prep(v, dtype)
    f = hippo.hippo_verify_attention if fn == "verify" else hippo.hippo_draft_attention
    # reference run: the new rows already in the cache
    kd, vd = dev(k, dtype), dev(v, dtype)
    want = f(dev(q, dtype), kd, vd, ctx, num_splits=ns)
    # fused run: cache rows >= ctx hold garbage, the new rows arrive as [B, q_len, Hkv, d]
    k_poison, v_poison = k.copy(), v.copy()
    k_poison[:, :, ctx:] = 1e30
    v_poison[:, :, ctx:] = -1e30
    kc, vc = dev(k_poison, dtype), dev(v_poison, dtype)
    k_new = dev(np.ascontiguousarray(k[:, :, ctx:ctx + ql].transpose(0, 2, 1, 3)), dtype)
    v_new = dev(np.ascontiguousarray(v[:, :, ctx:ctx + ql].transpose(0, 2, 1, 3)), dtype)
    got = f(dev(q, dtype), kc, vc, ctx, num_splits=ns, k_new=k_new, v_new=v_new)
    torch.cuda.synchronize()
    assert torch.equal(got, want)                        # same data through the same arithmetic
    ro, _ = oracle.attention(q, k, v, ctx)
    assert_close(host(got), ro, dtype, "append %s %s" % (fn, shape))
    # the cache now holds the new rows, bit for bit; nothing else moved
    np.testing.assert_array_equal(host(kc[:, :, :ctx + ql]), host(kd[:, :, :ctx + ql]))
    np.testing.assert_array_equal(host(vc[:, :, :ctx + ql]), host(vd[:, :, :ctx + ql]))
    np.testing.assert_array_equal(host(kc[:, :, ctx + ql:]), host(dev(k_poison, dtype)[:, :, ctx + ql:]))


def test_append_fusion_decode_chain(hippo):
    """Three consecutive verify calls at growing context, each appending its own rows: the third
    sees what the first two wrote."""
    cfg = si.CONFIGS["draft"]
    x = si.make_inputs(cfg, 4)
    dt, n = cfg.dtype, cfg.ctx_len
    r = np.random.default_rng(0)
    steps, ql = 3, 4
    extra_k = prep(r.standard_normal((cfg.batch, cfg.n_kv_heads, steps * ql, cfg.head_dim)) / 8, dt)
    extra_v = prep(r.standard_normal((cfg.batch, cfg.n_kv_heads, steps * ql, cfg.head_dim)) / 8, dt)
    k_full = np.concatenate([x["k"][:, :, :n], extra_k], 2)
    v_full = np.concatenate([x["v"][:, :, :n], extra_v], 2)
    kc = dev(np.concatenate([x["k"][:, :, :n], np.zeros_like(extra_k)], 2), dt)
    vc = dev(np.concatenate([x["v"][:, :, :n], np.zeros_like(extra_v)], 2), dt)
    for s in range(steps):
        ctx = n + s * ql
        q = prep(r.standard_normal((cfg.batch, ql, cfg.n_q_heads, cfg.head_dim)), dt)
        k_new = dev(np.ascontiguousarray(k_full[:, :, ctx:ctx + ql].transpose(0, 2, 1, 3)), dt)
        v_new = dev(np.ascontiguousarray(v_full[:, :, ctx:ctx + ql].transpose(0, 2, 1, 3)), dt)
        out = hippo.hippo_verify_attention(dev(q, dt), kc[:, :, :ctx + ql], vc[:, :, :ctx + ql], ctx, k_new=k_new,
                                           v_new=v_new)
        torch.cuda.synchronize()
        ro, _ = oracle.attention(q, k_full[:, :, :ctx + ql], v_full[:, :, :ctx + ql], ctx)
        assert_close(host(out), ro, dt, "chain step %d" % s)
    np.testing.assert_array_equal(host(kc), prep(k_full, dt))
    np.testing.assert_array_equal(host(vc), prep(v_full, dt))


# ---------------------------------------------------------------------------------------------
# paged cache: the same rows scattered over a page pool
# ---------------------------------------------------------------------------------------------

def to_pages(x, page_size, n_pool, rng):
    """[B, Hkv, N, d] -> (pool [n_pool, page_size, Hkv, d], table [B, max_pages]); pages in random
    pool slots, unused slots and the tail of the last page filled with garbage."""
    B, Hkv, N, d = x.shape
    max_pages = (N + page_size - 1) // page_size
    assert B * max_pages <= n_pool
    slots = rng.permutation(n_pool)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
    pool = np.full((n_pool, page_size, Hkv, d), 3e4, dtype=np.float32)
    for b in range(B):
        for pg in range(max_pages):
            rows = x[b, :, pg * page_size:(pg + 1) * page_size]          # [Hkv, <=page, d]
            pool[slots[b, pg], :rows.shape[1]] = rows.transpose(1, 0, 2)
    return pool, slots


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("shape", [
    # B, q_len, H, Hkv, d, ctx, page_size, num_splits
    (1, 1, 4, 4, 64, 1, 16, 0),
    (2, 3, 8, 2, 64, 37, 16, 0),
    (1, 9, 7, 1, 128, 333, 32, 4),
    (2, 6, 28, 4, 128, 2049, 64, 0),      # headline head geometry
    (1, 12, 16, 2, 64, 515, 256, 3),      # pages larger than a slice
    (1, 6, 28, 4, 128, 5000, 16, 0),      # many small pages
    (1, 2, 6, 2, 64, 0, 16, 0),           # empty context
    (2, 4, 16, 4, 128, 1900, 16, 2),      # long slices (rotated start) over small pages
    (1, 3, 8, 4, 64, 3000, 128, 1),       # one long slice per KV head, each head at its own phase
])
def test_paged_cache(hippo, dtype, shape):
    B, ql, H, Hkv, d, ctx, ps, ns = shape
    q, k, v = rand_case(sum(shape), B, ql, H, Hkv, d, ctx)
    q, k, v = prep(q, dtype), prep(k, dtype), prep(v, dtype)
    rng = np.random.default_rng(7)
    n_pool = B * ((ctx + ql + ps - 1) // ps) + 5
    k_pool, table = to_pages(k, ps, n_pool, rng)
    v_pool, _ = to_pages(v, ps, n_pool, np.random.default_rng(7))        # same slots
    for fn, plain, paged in (("verify", hippo.hippo_verify_attention, hippo.hippo_verify_attention_paged),
                             ("draft", hippo.hippo_draft_attention, hippo.hippo_draft_attention_paged)):
        want, want_lse = plain(dev(q, dtype), dev(k, dtype), dev(v, dtype), ctx, num_splits=ns, want_lse=True)
        got, got_lse = paged(dev(q, dtype), dev(k_pool, dtype), dev(v_pool, dtype), torch.from_numpy(table).cuda(),
                             ctx, num_splits=ns, want_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(got, want) and torch.equal(got_lse, want_lse), (fn, shape)
    ro, _ = oracle.attention(q, k, v, ctx)
    assert_close(host(got), ro, dtype, "paged %s" % (shape,))


def test_paged_cache_full_size(hippo):
    """The 16K headline configuration through 16-token pages, in the heuristic's own launch shape."""
    cfg = si.CONFIGS["c3_16k"]
    x = si.make_inputs(cfg, 0)
    dt, n = cfg.dtype, cfg.ctx_len
    rng = np.random.default_rng(1)
    n_pool = (n + cfg.q_len + 15) // 16 + 9
    k_pool, table = to_pages(prep(x["k"], dt), 16, n_pool, rng)
    v_pool, _ = to_pages(prep(x["v"], dt), 16, n_pool, np.random.default_rng(1))
    q = dev(x["q_new"], dt)
    want = hippo.hippo_verify_attention(q, dev(x["k"], dt), dev(x["v"], dt), n)
    got = hippo.hippo_verify_attention_paged(q, dev(k_pool, dt), dev(v_pool, dt), torch.from_numpy(table).cuda(), n)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    # a table entry outside the pool is clamped into it: garbage out, but no access leaves the pool
    bad = table.copy()
    bad[0, 3] = 10 ** 9
    bad[0, 4] = -5
    hippo.hippo_verify_attention_paged(q, dev(k_pool, dt), dev(v_pool, dt), torch.from_numpy(bad).cuda(), n)
    torch.cuda.synchronize()
