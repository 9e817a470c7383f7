"""GPU parity: hippo_score_tokens and hippo_select_gather_kv (through the C ABI) vs the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import assert_close, assert_fused_close, assert_indices_consistent, dev, host, prep

pytestmark = pytest.mark.gpu


def score_case(hippo, q_txt, k, vis_off, F, gh, gw, dtype, ch=5, cw=5, emb=None, flags=7, what="", emb_pad=0):
    q_txt, k = prep(q_txt, dtype), prep(k, dtype)
    emb_h = None if emb is None else prep(emb, dtype)
    vid = hippo.video_desc(F, gh, gw, vis_off, ch, cw)
    emb_d = None if emb is None else dev(emb_h, dtype)
    if emb_pad:                                    # the same values as a view into rows emb_pad channels wider
        wide = torch.zeros(emb_d.shape[:2] + (emb_d.shape[2] + emb_pad,), dtype=emb_d.dtype, device="cuda")
        wide[..., :emb_d.shape[2]] = emb_d
        emb_d = wide[..., :emb_d.shape[2]]
    scores, comps = hippo.hippo_score_tokens(dev(q_txt, dtype), dev(k, dtype), vid, emb=emb_d, flags=flags,
                                             want_components=True)
    torch.cuda.synchronize()
    rs, rc = oracle.score_tokens(q_txt, k, vis_off, F, gh, gw, ch, cw, emb=emb_h, flags=flags)
    names = ["s_attn", "s_temp", "s_spa"]
    for t in range(3):
        if flags & (1 << t):
            assert_close(host(comps[t]), rc[t], dtype, "%s %s" % (what, names[t]))
    # the fused score is a sum of z-scores of O(1); its error is judged against O(1), i.e. the
    # tolerance's rms floor (z-scores cross zero), in fp32 plus what Eq. 7's division by the per-frame
    # deviation makes of the raw terms' own bound
    assert_fused_close(host(scores), rs, rc, F, dtype, what + " fused", flags)
    return host(scores), rs


@pytest.mark.parametrize("name", ["tiny", "draft"])
def test_score_on_configs(hippo, name):
    cfg = si.CONFIGS[name]
    x = si.make_inputs(cfg, 0)
    n = cfg.ctx_len
    score_case(hippo, x["q_txt"], x["k"][:, :, :n], cfg.n_prefix, cfg.n_frames, cfg.grid_h, cfg.grid_w,
               cfg.dtype, what=name)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("shape", [
    # B, L, H, Hkv, d, F, gh, gw, vis_off, tail, crop
    (1, 3, 2, 1, 64, 1, 5, 5, 0, 0, (5, 5)),       # one frame: s_temp = 1 everywhere -> sigma 0
    (2, 7, 6, 2, 64, 2, 7, 9, 3, 2, (5, 5)),       # two frames: every frame has one neighbour
    (1, 33, 8, 2, 128, 5, 6, 11, 17, 5, (4, 3)),   # odd everything, 4x3 crops
    (1, 70, 7, 1, 128, 3, 13, 21, 8, 8, (5, 5)),   # 819 tokens: several tiles and a ragged tail
    (2, 5, 4, 4, 64, 4, 8, 8, 1, 0, (8, 8)),       # 64-token crops (the maximum)
    (1, 4, 4, 2, 64, 2, 33, 32, 5, 3, (5, 5)),     # 1056-token frames: beyond the register-resident fusion
    (2, 9, 8, 2, 128, 5, 16, 16, 6, 4, (5, 5)),    # 256-token frames: one token tile each
    (2, 6, 4, 2, 64, 3, 16, 32, 0, 1, (5, 5)),     # 512-token frames: two tiles per frame
    (1, 5, 4, 1, 64, 3, 32, 32, 2, 0, (4, 8)),     # 1024-token frames: four tiles, two values per thread
    (1, 9, 4, 2, 64, 3, 13, 15, 3, 2, (6, 7)),     # 42-token crops (three 16-row blocks), ragged: 6+6+1 by 7+7+1
    (2, 5, 8, 2, 128, 4, 12, 16, 0, 1, (6, 8)),    # 48-token crops tiling the grid exactly
    (1, 6, 4, 1, 128, 2, 14, 17, 5, 0, (6, 8)),    # 48-token crops cut by both edges (2-row and 1-column rests)
    (1, 4, 2, 1, 64, 3, 10, 14, 1, 1, (5, 7)),     # 35-token crops: barely past the two-block kernel
    (1, 96, 16, 2, 64, 85, 16, 16, 5, 3, (5, 5)),  # 170 key tiles x 12 row chunks: the sweeps cut the rows in three runs
    (1, 40, 14, 2, 64, 33, 16, 16, 0, 0, (5, 5)),  # 66 key tiles x 5 row chunks: two runs of 3 and 2 chunks
])
def test_score_random_shapes(hippo, dtype, shape):
    B, L, H, Hkv, d, F, gh, gw, off, tail, (ch, cw) = shape
    r = np.random.default_rng(sum(shape[:10]))
    nv = F * gh * gw
    q = r.standard_normal((B, L, H, d)) * 1.5
    k = r.standard_normal((B, Hkv, off + nv + tail, d))
    # correlate neighbouring frames and neighbouring patches a little so the terms have structure
    kv = k[:, :, off:off + nv].reshape(B, Hkv, F, gh, gw, d)
    kv += 0.8 * np.roll(kv, 1, axis=2) + 0.5 * np.roll(kv, 1, axis=4)
    score_case(hippo, q, k, off, F, gh, gw, dtype, ch, cw, what="%s %s" % (dtype, shape))


def test_score_is_repeatable_bit_for_bit(hippo):
    """The 16K configuration and a four-layer call, repeated: every partial result has one writer and
    the sums have a fixed order, so each repetition must give the same bits whatever the order in
    which blocks run."""
    cfg = si.CONFIGS["c3_16k"]
    x = si.make_inputs(cfg, 3)
    dt, n = cfg.dtype, cfg.ctx_len
    q, k = dev(x["q_txt"], dt), dev(x["k"][:, :, :n], dt)
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    first = hippo.hippo_score_tokens(q, k, vid).clone()
    first4 = hippo.hippo_score_tokens_layers([q] * 4, [k] * 4, vid, emb_layer=0).clone()
    for _ in range(25):
        assert torch.equal(hippo.hippo_score_tokens(q, k, vid), first)
        assert torch.equal(hippo.hippo_score_tokens_layers([q] * 4, [k] * 4, vid, emb_layer=0), first4)
    rs, _ = oracle.score_tokens(x["q_txt"], x["k"][:, :, :n], cfg.n_prefix, cfg.n_frames, cfg.grid_h, cfg.grid_w)
    assert_close(host(first), rs, dt, "16K fused")


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_score_explicit_embedding_and_flags(hippo, dtype):
    B, L, H, Hkv, d, F, gh, gw, off = 1, 9, 4, 2, 64, 3, 6, 7, 4
    r = np.random.default_rng(21)
    nv = F * gh * gw
    q = r.standard_normal((B, L, H, d))
    k = r.standard_normal((B, Hkv, off + nv + 3, d))
    emb = r.standard_normal((B, nv, 200))         # 200 channels: 3 chunks of 64 and a tail of 8
    emb[:, gh * gw:2 * gh * gw] += 0.7 * emb[:, :gh * gw]
    for flags in (7, 1, 2, 4, 6, 5):
        score_case(hippo, q, k, off, F, gh, gw, dtype, emb=emb, flags=flags, what="flags %d" % flags)


@pytest.mark.parametrize("case", [
    # B, F, gh, gw, crop, channels, flags: what the frame-run kernel of the embedding terms can be handed
    (1, 130, 10, 10, (5, 5), 72, 6),     # 520 (crop, frame) pairs: runs of 2 frames; 72 channels: two waves, one ragged
    (1, 87, 8, 12, (4, 4), 512, 6),      # 6 crops x 87 frames: runs of 2, the last run a single frame; all 512 channels
    (2, 100, 10, 10, (5, 5), 136, 7),    # batch 2: runs of 3 frames, 100 = 33 x 3 + 1; riding in pass 1's launch
    (1, 520, 6, 5, (5, 5), 64, 6),       # two crops per frame (one of them a single row): runs of 4 frames
    (1, 9, 10, 10, (5, 5), 520, 6),      # 520 channels: beyond the frame-run kernel, a block per crop
    (1, 9, 10, 10, (5, 5), 520, 7),      # ... and riding in pass 1's launch, two crops per block
])
def test_embedding_terms_over_runs_of_frames(hippo, case):
    """Eq. 3-6 on bf16 embeddings with small crops: a block owns one crop position over a run of
    consecutive frames; run lengths, a short last run, ragged channel counts and the boundary to
    the wider-embedding kernels."""
    B, F, gh, gw, (ch, cw), de, flags = case
    r = np.random.default_rng(F + de)
    nv = F * gh * gw
    L, H, Hkv, d, off = 3, 2, 1, 64, 2
    q = r.standard_normal((B, L, H, d))
    k = r.standard_normal((B, Hkv, off + nv + 1, d))
    emb = r.standard_normal((B, F, gh * gw, de))
    emb[:, 1:] += 0.8 * emb[:, :-1]                  # neighbouring frames resemble each other
    emb[:, 3 % F, 7] = 0.0                           # a zero-norm token: its cosines are defined as 0
    score_case(hippo, q, k, off, F, gh, gw, "bf16", ch, cw, emb=emb.reshape(B, nv, de), flags=flags,
               what="runs %s" % (case,), emb_pad=24 if de == 136 else 0)   # one case with a token stride > channels


def test_score_layer_accumulation(hippo):
    """Outer layer sum of Eq. 2: two ACCUMULATE_ONLY-style calls; the last one fuses."""
    cfg = si.CONFIGS["tiny"]
    xs = [si.make_inputs(cfg, s) for s in (0, 1)]
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    mass = torch.zeros((cfg.batch, cfg.n_visual), dtype=torch.float32, device="cuda")
    k0 = dev(xs[0]["k"], cfg.dtype)
    hippo.hippo_score_tokens(dev(xs[0]["q_txt"], cfg.dtype), k0, vid, flags=hippo.SCORE_ACCUMULATE_ONLY,
                             attn_mass_inout=mass)
    # second layer: its own queries/keys for the attention term; embeddings come from this call's keys
    scores, comps = hippo.hippo_score_tokens(dev(xs[1]["q_txt"], cfg.dtype), dev(xs[1]["k"], cfg.dtype), vid,
                                             attn_mass_inout=mass, want_components=True)
    torch.cuda.synchronize()
    sa = sum(oracle.s_attn(x["q_txt"], x["k"], cfg.n_prefix, cfg.n_visual) for x in xs)
    assert_close(host(mass), sa, "fp32", "accumulated mass")
    emb = oracle.keys_as_embedding(xs[1]["k"], cfg.n_prefix, cfg.n_visual)
    ref = oracle.fuse(sa, oracle.s_temp(emb, cfg.n_frames),
                      oracle.s_spa(emb, cfg.n_frames, cfg.grid_h, cfg.grid_w), cfg.n_frames)
    assert_fused_close(host(scores), ref, (sa, oracle.s_temp(emb, cfg.n_frames),
                                           oracle.s_spa(emb, cfg.n_frames, cfg.grid_h, cfg.grid_w)),
                       cfg.n_frames, "fp32", "fused after accumulation")


# ---------------------------------------------------------------------------------------------
# selection + gather: bit exact
# ---------------------------------------------------------------------------------------------

def select_case(hippo, scores: np.ndarray, k: int):
    B, n = scores.shape
    vid = hippo.video_desc(1, 1, n, 0)
    dummy = torch.zeros((B, 1, n, 64), dtype=torch.float32, device="cuda")
    idx, _, _ = hippo.hippo_select_gather_kv(torch.from_numpy(scores).cuda(), k, dummy, dummy, vid, gather=False)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.topk(scores, k))


@pytest.mark.parametrize("n,k", [(1, 1), (63, 7), (64, 64), (1025, 100), (4096, 410), (16384, 1639),
                                 (36864, 3687), (36864, 36863), (5000, 1), (40960, 4096), (40961, 7),
                                 (70001, 7001)])
def test_topk_bit_exact(hippo, n, k):
    select_case(hippo, si.random_scores(2, n, n + k), k)


@pytest.mark.parametrize("n,k,distinct", [(1000, 100, 3), (4096, 2048, 2), (777, 776, 1), (20000, 5000, 17),
                                          (50000, 20000, 5)])
def test_topk_with_many_ties(hippo, n, k, distinct):
    select_case(hippo, si.random_scores(3, n, n, n_distinct=distinct), k)


@pytest.mark.parametrize("n,k,others", [(3000, 300, 0), (4096, 1000, 0), (4097, 1000, 0), (4200, 150, 104),
                                        (16384, 1639, 37), (33000, 3300, 5000), (40960, 40000, 1)])
def test_topk_scores_sharing_the_first_digit(hippo, n, k, others):
    """Scores whose keys agree in sign, exponent and the top three mantissa bits: the radix select's first digit
    does not separate them.  The sizes put 3000, exactly 4096, 4097 and many more keys into that one bin (the
    boundary of the in-LDS candidate list and the register sweeps beyond it); `others` scores lie elsewhere, above
    and below, so the wanted key is in the crowded bin for some cases and next to it for others."""
    rng = np.random.default_rng(n + k)
    s = (1.0 + rng.random((2, n)) * 0.0624).astype(np.float32)          # [1, 1.0625): one 12-bit digit
    s[1] = np.round(s[1] * 64) / 64                                       # second row: a handful of distinct values
    if others:
        at = rng.choice(n, size=others, replace=False)
        s[:, at] = (rng.standard_normal((2, others)) * 3).astype(np.float32)
    select_case(hippo, s, k)


def test_topk_special_values(hippo):
    s = si.random_scores(4, 3000, 9)
    s[0, ::5] = np.nan
    s[0, 1::7] = -np.inf
    s[1, ::2] = 0.0
    s[1, 1::4] = -0.0
    s[2, :] = np.inf
    s[3, ::3] = np.float32(1e-45)          # denormals order like any other number
    s[3, 1::3] = -np.float32(1e-45)
    for k in (1, 299, 1500, 2999, 3000):
        select_case(hippo, s, k)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_gather_bit_exact(hippo, dtype):
    B, Hkv, d, F, gh, gw, off, tail, k = 2, 3, 128, 3, 5, 7, 6, 9, 31
    nv = F * gh * gw
    r = np.random.default_rng(3)
    ks = prep(r.standard_normal((B, Hkv, off + nv + tail, d)), dtype)
    vs = prep(r.standard_normal((B, Hkv, off + nv + tail, d)), dtype)
    scores = si.random_scores(B, nv, 4, n_distinct=11)
    vid = hippo.video_desc(F, gh, gw, off)
    idx, kd, vd = hippo.hippo_select_gather_kv(torch.from_numpy(scores).cuda(), k, dev(ks, dtype), dev(vs, dtype), vid)
    torch.cuda.synchronize()
    ridx = oracle.topk(scores, k)
    np.testing.assert_array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_array_equal(host(kd), oracle.gather(ks, off, nv, ridx))
    np.testing.assert_array_equal(host(vd), oracle.gather(vs, off, nv, ridx))


# ---------------------------------------------------------------------------------------------
# end to end: score -> select -> gather -> draft attention on the pruned cache
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["tiny", "draft", "c3_16k"])
def test_prune_pipeline(hippo, name):
    cfg = si.CONFIGS[name]
    x = si.make_inputs(cfg, 0)
    dt = cfg.dtype
    n = cfg.ctx_len
    kd, vd = dev(x["k"][:, :, :n], dt), dev(x["v"][:, :, :n], dt)
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    scores = hippo.hippo_score_tokens(dev(x["q_txt"], dt), kd, vid)
    idx, kp, vp = hippo.hippo_select_gather_kv(scores, cfg.k_keep, kd, vd, vid, cfg.n_q_heads)
    torch.cuda.synchronize()
    # selection is bit exact given the GPU's own fp32 scores ...
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.topk(host(scores), cfg.k_keep))
    # ... and agrees with the all-oracle selection except for near-ties at the threshold
    rs, rc = oracle.score_tokens(x["q_txt"], x["k"][:, :, :n], cfg.n_prefix, cfg.n_frames, cfg.grid_h, cfg.grid_w)
    assert_fused_close(host(scores), rs, rc, cfg.n_frames, dt, name + " scores")
    ridx = oracle.topk(rs.astype(np.float32), cfg.k_keep)
    assert_indices_consistent(idx.cpu().numpy(), rs, ridx, tol=1e-4 if dt == "fp32" else 5e-2)
    # the pruned cache is what the oracle builds from the same indices
    np.testing.assert_array_equal(host(kp), oracle.gather(x["k"][:, :, :n], cfg.n_prefix, cfg.n_visual, idx.cpu().numpy()))
    # draft decode over it: the draft cache holds the pruned context plus the new token's own row
    kpn = torch.cat([kp, dev(x["k"][:, :, n:n + 1], dt)], dim=2)
    vpn = torch.cat([vp, dev(x["v"][:, :, n:n + 1], dt)], dim=2)
    out = hippo.hippo_draft_attention(dev(x["q_new"][:, :1], dt), kpn, vpn, kp.shape[2])
    torch.cuda.synchronize()
    ro, _ = oracle.attention(x["q_new"][:, :1], host(kpn), host(vpn), kp.shape[2])
    assert_close(host(out), ro, dt, name + " draft attention")


# ---------------------------------------------------------------------------------------------
# Eq. 2's sum over layers inside one call
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name,n_layers", [("tiny", 3), ("draft", 4), ("draft", 1)])
def test_score_layers_in_one_call(hippo, name, n_layers):
    cfg = si.CONFIGS[name]
    dt, n = cfg.dtype, cfg.ctx_len
    xs = [si.make_inputs(cfg, 10 + l) for l in range(n_layers)]
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    qs = [dev(x["q_txt"], dt) for x in xs]
    ks = [dev(x["k"][:, :, :n], dt) for x in xs]
    emb_layer = n_layers - 1
    scores, comps = hippo.hippo_score_tokens_layers(qs, ks, vid, emb_layer=emb_layer, want_components=True)
    torch.cuda.synchronize()
    sa = sum(oracle.s_attn(x["q_txt"], x["k"][:, :, :n], cfg.n_prefix, cfg.n_visual) for x in xs)
    emb = oracle.keys_as_embedding(xs[emb_layer]["k"][:, :, :n], cfg.n_prefix, cfg.n_visual)
    st = oracle.s_temp(emb, cfg.n_frames)
    ss = oracle.s_spa(emb, cfg.n_frames, cfg.grid_h, cfg.grid_w)
    assert_close(host(comps[0]), sa, dt, "layer-summed s_attn")
    assert_close(host(comps[1]), st, dt, "s_temp")
    ref = oracle.fuse(sa, st, ss, cfg.n_frames)
    assert_fused_close(host(scores), ref, (sa, st, ss), cfg.n_frames, dt, "fused over %d layers" % n_layers)
    # the same through per-layer calls with the accumulate flag (what the batched call replaces)
    mass = torch.zeros((cfg.batch, cfg.n_visual), dtype=torch.float32, device="cuda")
    for l in range(n_layers - 1):
        hippo.hippo_score_tokens(qs[l], ks[l], vid, flags=hippo.SCORE_ACCUMULATE_ONLY, attn_mass_inout=mass)
    seq = hippo.hippo_score_tokens(qs[-1], ks[-1], vid, attn_mass_inout=mass)
    torch.cuda.synchronize()
    # two fp32 paths to the same number: each within the propagated bound of the oracle's
    if dt == "fp32":
        assert_fused_close(host(seq), ref, (sa, st, ss), cfg.n_frames, dt, "accumulated calls, %d layers" % n_layers)
    else:
        assert_close(host(seq), host(scores).astype(np.float64), dt, "batched vs accumulated")
