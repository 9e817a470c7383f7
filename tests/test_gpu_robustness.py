"""GPU checks beyond plain parity: determinism (the race check), independence from workspace
contents, exact workspace sizes, strided inputs, and the remaining full-size configurations."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import assert_close, assert_fused_close, assert_indices_consistent, dev, host, prep

pytestmark = pytest.mark.gpu


def _ws(nbytes, fill):
    t = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    t.fill_(fill)
    return t


@pytest.mark.parametrize("name", ["tiny", "draft"])
def test_results_are_bit_stable_and_ignore_workspace_contents(hippo, name):
    """Every kernel is deterministic: repeated runs, with the caller's workspace holding different
    garbage each time (all-ones bits = NaN patterns, zeros), give identical bits.  The workspace is
    exactly as large as hippo_workspace_bytes says."""
    cfg = si.CONFIGS[name]
    x = si.make_inputs(cfg, 5)
    dt, n = cfg.dtype, cfg.ctx_len
    k, v, q = dev(x["k"], dt), dev(x["v"], dt), dev(x["q_new"], dt)
    q_txt = dev(x["q_txt"], dt)
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    kvd = hippo.kv_desc(k, cfg.n_q_heads)
    need_v = hippo.workspace_bytes(hippo.CALL_VERIFY_ATTENTION, kvd, None, cfg.q_len, n + cfg.q_len)
    need_s = hippo.workspace_bytes(hippo.CALL_SCORE_TOKENS, kvd, vid, cfg.l_txt, n)
    outs = []
    for fill in (0xFF, 0x00, 0x7F):
        o = hippo.hippo_verify_attention(q, k, v, n, workspace=_ws(need_v, fill))
        s = hippo.hippo_score_tokens(q_txt, k[:, :, :n], vid, workspace=_ws(need_s, fill))
        idx, kp, vp = hippo.hippo_select_gather_kv(s, cfg.k_keep, k[:, :, :n], v[:, :, :n], vid, cfg.n_q_heads)
        torch.cuda.synchronize()
        outs.append((o.clone(), s.clone(), idx.clone(), kp.clone()))
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)


def test_workspace_one_byte_short_is_refused(hippo):
    cfg = si.CONFIGS["tiny"]
    x = si.make_inputs(cfg, 0)
    k, v, q = dev(x["k"], "fp32"), dev(x["v"], "fp32"), dev(x["q_new"], "fp32")
    kvd = hippo.kv_desc(k, cfg.n_q_heads)
    need = hippo.workspace_bytes(hippo.CALL_VERIFY_ATTENTION, kvd, None, cfg.q_len, cfg.ctx_len + cfg.q_len)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    with pytest.raises(hippo.HippoError) as e:
        hippo.hippo_verify_attention(q, k, v, cfg.ctx_len, workspace=ws[:need - 256])
    assert e.value.status == hippo.ERR_WORKSPACE_TOO_SMALL


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_scoring_and_gather_on_strided_caches(hippo, dtype):
    """K and V interleaved in one allocation (row stride 2d, oversized head stride); the gathered
    draft cache is written into a strided view as well."""
    B, L, H, Hkv, d, F, gh, gw, off, tail = 2, 6, 4, 2, 64, 3, 6, 5, 7, 4
    r = np.random.default_rng(77)
    nv = F * gh * gw
    n = off + nv + tail
    q = prep(r.standard_normal((B, L, H, d)), dtype)
    k = prep(r.standard_normal((B, Hkv, n, d)), dtype)
    v = prep(r.standard_normal((B, Hkv, n, d)), dtype)
    tdt = dev(q, dtype).dtype
    buf = torch.zeros((B, Hkv, n + 9, 2, d), dtype=tdt, device="cuda")
    buf[:, :, :n, 0], buf[:, :, :n, 1] = dev(k, dtype), dev(v, dtype)
    kd, vd = buf[:, :, :n, 0], buf[:, :, :n, 1]
    vid = hippo.video_desc(F, gh, gw, off)
    scores = hippo.hippo_score_tokens(dev(q, dtype), kd, vid)
    kk = 17
    dst = torch.zeros((B, Hkv, n - nv + kk + 3, 2, d), dtype=tdt, device="cuda")
    idx, kp, vp = hippo.hippo_select_gather_kv(scores, kk, kd, vd, vid, H, k_dst=dst[:, :, :n - nv + kk, 0],
                                               v_dst=dst[:, :, :n - nv + kk, 1])
    torch.cuda.synchronize()
    rs, rc = oracle.score_tokens(q, k, off, F, gh, gw)
    assert_fused_close(host(scores), rs, rc, F, dtype, "strided scores")
    ridx = oracle.topk(host(scores), kk)
    np.testing.assert_array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_array_equal(host(kp), oracle.gather(k, off, nv, ridx))
    np.testing.assert_array_equal(host(vp), oracle.gather(v, off, nv, ridx))
    assert torch.all(dst[:, :, n - nv + kk:] == 0)            # nothing written past the draft cache


@pytest.mark.parametrize("shape", [(1, 9, 7, 1, 64, 700), (2, 4, 16, 1, 64, 129), (1, 8, 8, 1, 128, 40)])
def test_verify_four_row_blocks_both_head_dims(hippo, shape):
    B, ql, H, Hkv, d, ctx = shape        # R = 63, 64, 64: the 4-row-block instantiations
    r = np.random.default_rng(ql * 100 + d)
    q = r.standard_normal((B, ql, H, d)) * 2.5
    k = r.standard_normal((B, Hkv, ctx + ql, d))
    v = r.standard_normal((B, Hkv, ctx + ql, d))
    q, k, v = prep(q, "bf16"), prep(k, "bf16"), prep(v, "bf16")
    for s in (0, 1, 3):
        out = hippo.hippo_verify_attention(dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), ctx, num_splits=s)
        torch.cuda.synchronize()
        ro, _ = oracle.attention(q, k, v, ctx)
        assert_close(host(out), ro, "bf16", "%s S=%d" % (shape, s))


def test_prune_pipeline_long_video(hippo):
    """33K-token configuration, keep ratios 5 / 10 / 25 %."""
    cfg0 = si.CONFIGS["c4_long"]
    x = si.make_inputs(cfg0, 0)
    dt, n = cfg0.dtype, cfg0.ctx_len
    kd, vd = dev(x["k"][:, :, :n], dt), dev(x["v"][:, :, :n], dt)
    vid = hippo.video_desc(cfg0.n_frames, cfg0.grid_h, cfg0.grid_w, cfg0.n_prefix)
    scores = hippo.hippo_score_tokens(dev(x["q_txt"], dt), kd, vid)
    torch.cuda.synchronize()
    rs, _ = oracle.score_tokens(x["q_txt"], x["k"][:, :, :n], cfg0.n_prefix, cfg0.n_frames, cfg0.grid_h, cfg0.grid_w)
    assert_close(host(scores), rs, dt, "c4 scores")
    for pct in (5, 10, 25):
        cfg = cfg0.with_keep(pct)
        idx, kp, vp = hippo.hippo_select_gather_kv(scores, cfg.k_keep, kd, vd, vid, cfg.n_q_heads)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(idx.cpu().numpy(), oracle.topk(host(scores), cfg.k_keep))
        assert_indices_consistent(idx.cpu().numpy(), rs, oracle.topk(rs.astype(np.float32), cfg.k_keep), tol=5e-2)
        np.testing.assert_array_equal(host(vp), oracle.gather(x["v"][:, :, :n], cfg.n_prefix, cfg.n_visual,
                                                              idx.cpu().numpy()))


def test_prune_pipeline_large_share(hippo):
    """Batch 4 x 64 heads x 36864 visual tokens: the GPU scores all four sequences in one call; the
    oracle re-computes every batch element (scores, selection, gathered rows)."""
    cfg = si.CONFIGS["c5_large"]
    x = si.make_inputs(cfg, 0)
    dt, n = cfg.dtype, cfg.ctx_len
    kd, vd = dev(x["k"][:, :, :n], dt), dev(x["v"][:, :, :n], dt)
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    scores = hippo.hippo_score_tokens(dev(x["q_txt"], dt), kd, vid)
    idx, kp, vp = hippo.hippo_select_gather_kv(scores, cfg.k_keep, kd, vd, vid, cfg.n_q_heads)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.topk(host(scores), cfg.k_keep))
    for b in range(cfg.batch):
        rs, _ = oracle.score_tokens(x["q_txt"][b:b + 1], x["k"][b:b + 1, :, :n], cfg.n_prefix, cfg.n_frames,
                                    cfg.grid_h, cfg.grid_w)
        assert_close(host(scores)[b:b + 1], rs, dt, "c5 scores, batch element %d" % b)
        np.testing.assert_array_equal(host(kp)[b:b + 1], oracle.gather(x["k"][b:b + 1, :, :n], cfg.n_prefix,
                                                                       cfg.n_visual, idx.cpu().numpy()[b:b + 1]))
