"""Pins for the CPU oracle: closed forms, invariants, library routines and brute force.

Nothing here touches the HIP library.  Each test ties one piece of ``oracle/hippo_oracle.c`` to
something other than itself: the paper's equations worked by hand (tests/golden), a textbook
identity, scipy/numpy dense routines on tiny shapes, or an exhaustive sort.
"""
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import oracle
import synth_inputs as si

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":")
            out[key.strip()] = np.array([float(x) for x in vals.split()])
    return out


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------------------------------
# Eq. 2  s_attn
# ------------------------------------------------------------------------------------------

def _cache_from_vis(k_vis, vis_off=3, tail=2, seed=9):
    """embed visual keys [B,Hkv,Nv,d] in a longer cache with random text rows around them"""
    B, Hkv, Nv, d = k_vis.shape
    k = rng(seed).standard_normal((B, Hkv, vis_off + Nv + tail, d)).astype(np.float32)
    k[:, :, vis_off:vis_off + Nv] = k_vis
    return k, vis_off


def test_s_attn_matches_library_softmax_gqa():
    r = rng(0)
    B, L, H, Hkv, d, Nv = 2, 5, 6, 2, 8, 37
    q = r.standard_normal((B, L, H, d)).astype(np.float32) * 2
    kv = r.standard_normal((B, Hkv, Nv, d)).astype(np.float32)
    k, off = _cache_from_vis(kv)
    got = oracle.s_attn(q, k, off, Nv)
    G = H // Hkv
    ref = np.zeros((B, Nv))
    for b in range(B):
        for h in range(H):
            z = q[b, :, h, :].astype(np.float64) @ kv[b, h // G].astype(np.float64).T / math.sqrt(d)
            ref[b] += softmax(z, axis=-1).sum(axis=0)
    ref /= H * L
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-15)


def test_s_attn_sums_to_one_and_ignores_text_rows():
    r = rng(1)
    q = r.standard_normal((1, 4, 4, 16)).astype(np.float32) * 3
    kv = r.standard_normal((1, 2, 50, 16)).astype(np.float32)
    k1, off = _cache_from_vis(kv, seed=1)
    k2, _ = _cache_from_vis(kv, seed=2)          # different text rows, same visual rows
    a1, a2 = oracle.s_attn(q, k1, off, 50), oracle.s_attn(q, k2, off, 50)
    assert abs(a1.sum() - 1.0) < 1e-13
    np.testing.assert_array_equal(a1, a2)


def test_s_attn_uniform_when_keys_equal():
    r = rng(2)
    q = r.standard_normal((1, 3, 2, 8)).astype(np.float32)
    kv = np.tile(r.standard_normal((1, 1, 1, 8)).astype(np.float32), (1, 1, 20, 1))
    k, off = _cache_from_vis(kv)
    np.testing.assert_allclose(oracle.s_attn(q, k, off, 20), 1.0 / 20, rtol=1e-13)


def test_s_attn_scale_is_inverse_sqrt_dk():
    # one query, two keys whose logits differ by exactly ln 3 after the 1/sqrt(d_k) scale -> 3/4, 1/4
    d = 16
    q = np.zeros((1, 1, 1, d), np.float32)
    q[..., 0] = 4.0
    kv = np.zeros((1, 1, 2, d), np.float32)
    kv[0, 0, 0, 0] = np.float32(math.log(3.0))       # q.k/sqrt(16) = ln3 (up to fp32 rounding of ln3)
    k, off = _cache_from_vis(kv)
    got = oracle.s_attn(q, k, off, 2)[0]
    l3 = float(np.float32(math.log(3.0)))
    np.testing.assert_allclose(got, [math.exp(l3) / (1 + math.exp(l3)), 1 / (1 + math.exp(l3))], rtol=1e-14)
    assert abs(got[0] - 0.75) < 1e-7


def test_s_attn_large_logits_do_not_overflow():
    q = np.full((1, 1, 1, 4), 300.0, np.float32)
    kv = np.zeros((1, 1, 3, 4), np.float32)
    kv[0, 0, 1] = 300.0
    k, off = _cache_from_vis(kv)
    got = oracle.s_attn(q, k, off, 3)[0]
    assert np.all(np.isfinite(got)) and abs(got[1] - 1.0) < 1e-12


# ------------------------------------------------------------------------------------------
# Eq. 3-4  s_temp
# ------------------------------------------------------------------------------------------

def test_s_temp_golden_three_frames():
    g = read_golden("eq34_three_frames.txt")
    t = math.radians(g["theta_deg"][0])
    emb = np.zeros((1, 3, 4), np.float64)
    emb[0, 0, 0] = 1
    emb[0, 1, 0], emb[0, 1, 1] = math.cos(t), math.sin(t)
    emb[0, 2, 1] = 1
    got = oracle.s_temp(emb * np.array([2.0, 0.5, 7.0])[None, :, None], 3)[0]   # norms must not matter
    np.testing.assert_allclose(got, g["s_temp"], atol=2e-7)                    # fp32 inputs


def test_s_temp_closed_forms():
    r = rng(3)
    P, de = 6, 10
    base = r.standard_normal((1, P, de)).astype(np.float32)
    same = np.concatenate([base] * 4, axis=1)
    np.testing.assert_allclose(oracle.s_temp(same, 4), 0.0, atol=1e-12)
    flip = np.concatenate([base, -base, base], axis=1)
    np.testing.assert_allclose(oracle.s_temp(flip, 3), 2.0, atol=1e-12)
    np.testing.assert_allclose(oracle.s_temp(base, 1), 1.0, atol=0)             # F = 1: no neighbour
    orth = np.zeros((1, 3 * P, 3), np.float32)
    for f in range(3):
        orth[0, f * P:(f + 1) * P, f] = 1.0 + f
    np.testing.assert_allclose(oracle.s_temp(orth, 3), 1.0, atol=1e-12)


def test_s_temp_matches_numpy_definition():
    r = rng(4)
    F, P, de = 5, 7, 12
    emb = r.standard_normal((2, F * P, de)).astype(np.float32)
    got = oracle.s_temp(emb, F)
    e = emb.astype(np.float64).reshape(2, F, P, de)
    e = e / np.linalg.norm(e, axis=-1, keepdims=True)
    ref = np.zeros((2, F, P))
    for f in range(F):
        nb = [g for g in (f - 1, f + 1) if 0 <= g < F]
        ref[:, f] = 1.0 - sum((e[:, f] * e[:, g]).sum(-1) for g in nb) / len(nb)
    np.testing.assert_allclose(got, ref.reshape(2, -1), rtol=1e-12, atol=1e-14)


def test_zero_norm_embedding_gives_zero_cosine():
    emb = np.ones((1, 2, 4), np.float32)
    emb[0, 0] = 0
    np.testing.assert_allclose(oracle.s_temp(emb, 2), 1.0)


# ------------------------------------------------------------------------------------------
# Eq. 5-6  s_spa
# ------------------------------------------------------------------------------------------

def test_s_spa_golden_small_crops():
    g = read_golden("eq6_small_crops.txt")
    t = math.radians(g["two_token_theta_deg"][0])
    emb = np.array([[[3.0, 0.0], [0.5 * math.cos(t), 0.5 * math.sin(t)]]])
    np.testing.assert_allclose(oracle.s_spa(emb, 1, 1, 2, 5, 5)[0], g["two_token_s_spa"], atol=1e-7)
    dup = np.array([[[1.0, 0, 0], [2.0, 0, 0], [0, 0, 5.0]]])
    np.testing.assert_allclose(oracle.s_spa(dup, 1, 1, 3, 5, 5)[0], g["dup_s_spa"], atol=1e-14)
    for M, want in zip(g["orthonormal_M"].astype(int), g["orthonormal_s_spa"]):
        emb = (np.eye(M) * np.arange(1, M + 1))[None]
        h, w = (5, 5) if M == 25 else (1, M)
        if M == 10:
            h, w = 2, 5
        np.testing.assert_allclose(oracle.s_spa(emb, 1, h, w, 5, 5)[0], want, atol=1e-14)


def test_s_spa_tiling_is_anchored_tiles_with_truncated_edges():
    # 12 x 16 grid, 5 x 5 crops -> row bands 5,5,2 and column bands 5,5,5,1.  Give every token a
    # one-hot code of its position inside its expected crop: each crop is then an orthonormal set
    # and s_spa must be (M_c - 1)/M_c^2 with the crop's true size.  Any other tiling mixes equal
    # codes into one crop and breaks the closed form.
    gh, gw, F = 12, 16, 2
    emb = np.zeros((1, F * gh * gw, 25), np.float32)
    want = np.zeros(F * gh * gw)
    for f in range(F):
        for y in range(gh):
            for x in range(gw):
                emb[0, f * gh * gw + y * gw + x, (y % 5) * 5 + (x % 5)] = 1.0
                mh = 5 if y < 10 else 2
                mw = 5 if x < 15 else 1
                M = mh * mw
                want[f * gh * gw + y * gw + x] = (M - 1) / M ** 2
    np.testing.assert_allclose(oracle.s_spa(emb, F, gh, gw, 5, 5)[0], want, atol=1e-14)


def test_s_spa_matches_numpy_definition_and_is_scale_invariant():
    r = rng(5)
    F, gh, gw, de = 2, 7, 6, 9
    emb = r.standard_normal((1, F * gh * gw, de)).astype(np.float32)
    got = oracle.s_spa(emb, F, gh, gw, 3, 4)
    e = emb[0].astype(np.float64).reshape(F, gh, gw, de)
    e = e / np.linalg.norm(e, axis=-1, keepdims=True)
    ref = np.zeros((F, gh, gw))
    for f in range(F):
        for y0 in range(0, gh, 3):
            for x0 in range(0, gw, 4):
                E = e[f, y0:y0 + 3, x0:x0 + 4].reshape(-1, de)
                S = E @ E.T
                ref[f, y0:y0 + 3, x0:x0 + 4] = S.var(axis=1).reshape(ref[f, y0:y0 + 3, x0:x0 + 4].shape)
    np.testing.assert_allclose(got[0], ref.reshape(-1), rtol=1e-11, atol=1e-14)
    scaled = emb * np.float32(4.0)          # exact in fp32
    np.testing.assert_allclose(oracle.s_spa(scaled, F, gh, gw, 3, 4), got, rtol=1e-12, atol=1e-15)


def test_s_spa_identical_crop_is_zero():
    emb = np.tile(rng(6).standard_normal((1, 1, 8)).astype(np.float32), (1, 25, 1))
    np.testing.assert_allclose(oracle.s_spa(emb, 1, 5, 5, 5, 5), 0.0, atol=1e-14)


# ------------------------------------------------------------------------------------------
# Eq. 7  fusion
# ------------------------------------------------------------------------------------------

def test_fuse_golden():
    g = read_golden("eq7_zscore_worked.txt")
    s = g["s"][None]
    zero = np.zeros_like(s)
    np.testing.assert_allclose(oracle.fuse(s, zero, zero, 1, oracle.FLAG_ATTN)[0], g["zhat"], rtol=1e-15)
    np.testing.assert_allclose(oracle.fuse(zero, s, zero, 1, oracle.FLAG_TEMP)[0], g["zhat"], rtol=1e-15)
    np.testing.assert_allclose(oracle.fuse(zero, zero, s, 1, oracle.FLAG_SPA)[0], g["zhat"], rtol=1e-15)
    mirror = s[:, ::-1].copy()
    np.testing.assert_allclose(oracle.fuse(s, mirror, zero, 1, oracle.FLAG_ATTN | oracle.FLAG_TEMP)[0],
                               g["fused_with_mirror"], atol=1e-15)
    # all three flags with a constant third term: sigma = 0 contributes nothing
    np.testing.assert_allclose(oracle.fuse(s, s, np.ones_like(s), 1)[0], 2 * g["zhat"], rtol=1e-15)


def test_fuse_is_per_frame_and_matches_numpy():
    r = rng(7)
    B, F, P = 2, 3, 11
    a, t, s = (r.standard_normal((B, F * P)) * sc + off for sc, off in ((1e-4, 1e-3), (0.1, 0.4), (0.02, 0.05)))
    got = oracle.fuse(a, t, s, F)
    ref = np.zeros((B, F, P))
    for x in (a, t, s):
        x = x.reshape(B, F, P)
        ref += (x - x.mean(-1, keepdims=True)) / x.std(-1, keepdims=True)     # numpy std: population
    np.testing.assert_allclose(got, ref.reshape(B, -1), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(got.reshape(B, F, P).sum(-1), 0.0, atol=1e-11)   # every frame sums to 0
    # a term scaled by a positive constant (e.g. the 1/(N_L H L_txt) of Eq. 2) does not change the result
    np.testing.assert_allclose(oracle.fuse(a * 37.0, t, s, F), got, rtol=1e-10, atol=1e-11)


# ------------------------------------------------------------------------------------------
# top-k
# ------------------------------------------------------------------------------------------

def brute_topk(row, k):
    def key(i):
        x = row[i]
        if np.isnan(x):
            return (1, 0.0, i)
        return (0, -float(x), i)         # -0.0 == 0.0 in tuple comparison, so +-0 tie by index
    return sorted(sorted(range(len(row)), key=key)[:k])


@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force(seed):
    r = rng(100 + seed)
    n = int(r.integers(1, 60))
    k = int(r.integers(1, n + 1))
    s = si.random_scores(3, n, seed, n_distinct=(0 if seed % 2 else 5))
    if seed == 4:
        s[0, ::3] = np.nan
        s[1, ::2] = 0.0
        s[1, 1::4] = -0.0
    got = oracle.topk(s, k)
    for b in range(3):
        assert got[b].tolist() == brute_topk(s[b], k)


def test_topk_special_cases():
    s = si.random_scores(2, 40, 0)
    np.testing.assert_array_equal(oracle.topk(s, 40), np.tile(np.arange(40, dtype=np.int32), (2, 1)))
    np.testing.assert_array_equal(oracle.topk(np.ones((1, 30), np.float32), 7)[0], np.arange(7))
    # ties straddling the threshold: values 5,5,5,5 and k leaves room for two of them
    s = np.array([[1, 5, 9, 5, 0, 5, 9, 5]], np.float32)
    np.testing.assert_array_equal(oracle.topk(s, 4)[0], [1, 2, 3, 6])
    # NaN below every number, even -inf
    s = np.array([[np.nan, -np.inf, np.nan, 1.0]], np.float32)
    np.testing.assert_array_equal(oracle.topk(s, 2)[0], [1, 3])
    np.testing.assert_array_equal(oracle.topk(s, 3)[0], [0, 1, 3])


def test_keep_count_rounding():
    g = read_golden("keep_count.txt")
    for n, k in zip(g["n_visual"].astype(int), g["k_at_10pct"].astype(int)):
        assert (n * 10 + 99) // 100 == k
    assert si.CONFIGS["tiny"].n_visual == 768 and si.CONFIGS["tiny"].k_keep == 77
    assert si.CONFIGS["tiny"].ctx_len == 832
    assert si.CONFIGS["c3_16k"].ctx_len == 16640 and si.CONFIGS["c3_16k"].k_keep == 1639


# ------------------------------------------------------------------------------------------
# gather
# ------------------------------------------------------------------------------------------

def test_gather_rows_and_identity():
    r = rng(8)
    B, Hkv, N, d, off, Nv = 2, 3, 30, 4, 5, 20
    src = r.standard_normal((B, Hkv, N, d)).astype(np.float32)
    full = np.tile(np.arange(Nv, dtype=np.int32), (B, 1))
    np.testing.assert_array_equal(oracle.gather(src, off, Nv, full), src)        # keep 100 %
    idx = np.array([[0, 7, 19], [3, 4, 5]], np.int32)
    dst = oracle.gather(src, off, Nv, idx)
    assert dst.shape == (B, Hkv, N - Nv + 3, d)
    for b in range(B):
        np.testing.assert_array_equal(dst[b, :, :off], src[b, :, :off])
        np.testing.assert_array_equal(dst[b, :, off:off + 3], src[b][:, off + idx[b]])
        np.testing.assert_array_equal(dst[b, :, off + 3:], src[b, :, off + Nv:])


# ------------------------------------------------------------------------------------------
# attention
# ------------------------------------------------------------------------------------------

def textbook_attention(q, k, v, ctx_len, scale):
    """softmax(scale QK^T + mask) V through scipy/numpy dense routines, float64."""
    B, ql, H, d = q.shape
    Hkv = k.shape[1]
    G = H // Hkv
    n = ctx_len + ql
    out = np.zeros((B, ql, H, d))
    lse = np.zeros((B, H, ql))
    mask = np.where(np.arange(n)[None, :] <= ctx_len + np.arange(ql)[:, None], 0.0, -np.inf)
    for b in range(B):
        for h in range(H):
            z = scale * q[b, :, h].astype(np.float64) @ k[b, h // G, :n].astype(np.float64).T + mask
            out[b, :, h] = softmax(z, axis=-1) @ v[b, h // G, :n].astype(np.float64)
            lse[b, h] = logsumexp(z, axis=-1)
    return out, lse


def _attn_case(seed, B=2, ql=4, H=6, Hkv=3, d=8, ctx=21, extra=0, qscale=2.0):
    r = rng(seed)
    q = (r.standard_normal((B, ql, H, d)) * qscale).astype(np.float32)
    k = r.standard_normal((B, Hkv, ctx + ql + extra, d)).astype(np.float32)
    v = r.standard_normal((B, Hkv, ctx + ql + extra, d)).astype(np.float32)
    return q, k, v, ctx


def test_attention_matches_textbook():
    q, k, v, ctx = _attn_case(10, extra=3)       # rows beyond ctx+q_len must be ignored
    out, lse = oracle.attention(q, k, v, ctx)
    ro, rl = textbook_attention(q, k, v, ctx, 1 / math.sqrt(q.shape[-1]))
    np.testing.assert_allclose(out, ro, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, rl, rtol=1e-13)
    out2, _ = oracle.attention(q, k, v, ctx, scale=0.3)
    np.testing.assert_allclose(out2, textbook_attention(q, k, v, ctx, 0.3)[0], rtol=1e-12, atol=1e-14)


def test_attention_rows_sum_to_one_and_mask_is_causal():
    q, k, v, ctx = _attn_case(11, B=1, ql=5, H=2, Hkv=1, d=4, ctx=9)
    n = ctx + 5
    out, _ = oracle.attention(q, k, np.ones_like(v), ctx)
    np.testing.assert_allclose(out, 1.0, rtol=1e-13)
    # one-hot V (d = n) reads the probabilities back out
    d = n
    r = rng(12)
    q = r.standard_normal((1, 5, 2, d)).astype(np.float32)
    k = r.standard_normal((1, 1, n, d)).astype(np.float32)
    v = np.eye(n, dtype=np.float32)[None, None]
    p, _ = oracle.attention(q, k, v, ctx)
    for i in range(5):
        assert np.all(p[0, i, :, ctx + i + 1:] == 0.0)          # nothing from the future rows
        assert np.all(p[0, i, :, :ctx + i + 1] > 0.0)
        np.testing.assert_allclose(p[0, i].sum(-1), 1.0, rtol=1e-13)


def test_verify_row_equals_single_token_decode_on_truncated_cache():
    q, k, v, ctx = _attn_case(13, ql=5)
    out, lse = oracle.attention(q, k, v, ctx)
    for i in range(5):
        oi, li = oracle.attention(q[:, i:i + 1], k[:, :, :ctx + i + 1], v[:, :, :ctx + i + 1], ctx + i)
        np.testing.assert_array_equal(oi[:, 0], out[:, i])        # gamma = 0 call == row i
        np.testing.assert_array_equal(li[:, :, 0], lse[:, :, i])


def test_attention_permutation_invariance_and_closed_form():
    q, k, v, ctx = _attn_case(14, ql=1)
    perm = rng(15).permutation(ctx)
    k2, v2 = k.copy(), v.copy()
    k2[:, :, :ctx], v2[:, :, :ctx] = k[:, :, perm], v[:, :, perm]
    a, _ = oracle.attention(q, k, v, ctx)
    b, _ = oracle.attention(q, k2, v2, ctx)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    # two entries, logits differ by ln 3 under the default 1/sqrt(d) scale: out = 3/4 v0 + 1/4 v1
    d = 4
    q = np.zeros((1, 1, 1, d), np.float32); q[..., 0] = 2.0
    k = np.zeros((1, 1, 2, d), np.float32); k[0, 0, 0, 0] = np.float32(math.log(3.0))
    v = np.zeros((1, 1, 2, d), np.float32); v[0, 0, 0, 1] = 1.0; v[0, 0, 1, 2] = 1.0
    o, l = oracle.attention(q, k, v, 1)
    np.testing.assert_allclose(o[0, 0, 0], [0, 0.75, 0.25, 0], atol=1e-7)
    np.testing.assert_allclose(l[0, 0, 0], math.log(4.0), atol=1e-7)


def test_keep_100_percent_reproduces_unpruned_attention():
    cfg = si.CONFIGS["tiny"]
    x = si.make_inputs(cfg, 0)
    full = np.tile(np.arange(cfg.n_visual, dtype=np.int32), (cfg.batch, 1))
    kd = oracle.gather(x["k"], cfg.n_prefix, cfg.n_visual, full)
    vd = oracle.gather(x["v"], cfg.n_prefix, cfg.n_visual, full)
    a, _ = oracle.attention(x["q_new"][:, :1], x["k"], x["v"], cfg.ctx_len)
    b, _ = oracle.attention(x["q_new"][:, :1], kd, vd, cfg.ctx_len)
    np.testing.assert_array_equal(a, b)


# ------------------------------------------------------------------------------------------
# end-to-end on the Tiny configuration + generator sanity
# ------------------------------------------------------------------------------------------

def test_tiny_pipeline_shapes_and_invariants():
    cfg = si.CONFIGS["tiny"]
    x = si.make_inputs(cfg, 0)
    scores, comp = oracle.score_tokens(x["q_txt"], x["k"], cfg.n_prefix, cfg.n_frames, cfg.grid_h, cfg.grid_w)
    assert scores.shape == (1, 768) and comp.shape == (3, 1, 768)
    assert abs(comp[0].sum() - 1.0) < 1e-12
    P = cfg.grid_h * cfg.grid_w
    np.testing.assert_allclose(scores.reshape(cfg.n_frames, P).sum(-1), 0.0, atol=1e-9)
    idx = oracle.topk(scores.astype(np.float32), cfg.k_keep)
    assert idx.shape == (1, 77) and np.all(np.diff(idx[0]) > 0)
    kd = oracle.gather(x["k"], cfg.n_prefix, cfg.n_visual, idx)
    assert kd.shape[2] == cfg.ctx_len + cfg.q_len - cfg.n_visual + 77


def test_generator_is_seeded_and_bf16_exact():
    cfg = si.CONFIGS["draft"]
    a, b = si.make_inputs(cfg, 3), si.make_inputs(cfg, 3)
    for key in a:
        np.testing.assert_array_equal(a[key], b[key])
        np.testing.assert_array_equal(si.round_to_bf16(a[key]), a[key])           # already bf16 values
        np.testing.assert_array_equal(si.bf16_bits_to_f32(si.bf16_bits(a[key])), a[key])
    c = si.make_inputs(cfg, 4)
    assert not np.array_equal(a["k"], c["k"])
    # bf16 rounding is round-to-nearest-even: 1 + 2^-8 is a tie -> 1.0 ; 1 + 3*2^-8 -> 1 + 2^-6
    t = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20], np.float32)
    np.testing.assert_array_equal(si.round_to_bf16(t), np.array([1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7], np.float32))


def test_generator_position_bias_shows_in_attention_only_selection():
    # the boundary ring (about 23 % of a 16x16 grid) must be over-represented in the attention-only
    # top 10 % and less so after fusion -- the effect the paper's motivation section reports
    cfg = si.CONFIGS["draft"]
    x = si.make_inputs(cfg, 0)
    scores, comp = oracle.score_tokens(x["q_txt"], x["k"], cfg.n_prefix, cfg.n_frames, cfg.grid_h, cfg.grid_w)
    ring = np.zeros((cfg.grid_h, cfg.grid_w), bool)
    ring[0], ring[-1], ring[:, 0], ring[:, -1] = True, True, True, True
    ring = np.tile(ring.reshape(-1), cfg.n_frames)
    only_attn = oracle.topk(comp[0].astype(np.float32), cfg.k_keep)[0]
    fused = oracle.topk(scores.astype(np.float32), cfg.k_keep)[0]
    share_attn, share_fused = ring[only_attn].mean(), ring[fused].mean()
    assert share_attn > 0.4 > ring.mean()
    assert share_fused < share_attn
