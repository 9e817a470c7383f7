"""The pruning criteria the paper compares HIPPO with, expressed through the same two entry points
(Experiments, ablation of the score terms; App., comparison of pruning criteria): attention-only
selection (the criterion of earlier video-SD work), HIPPO without the temporal or the spatial term,
random retention and uniform frame dropping.  The first three are `flags`; the last two are
caller-made score vectors handed to hippo_select_gather_kv, which is all a selection rule is to
the library.  Checked against the oracle, plus the observable the paper's motivation section
reports: attention-only selection crowds onto the position-biased border, fusion spreads it."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import assert_close, assert_fused_close, dev, host

pytestmark = pytest.mark.gpu


def ring_share(idx, cfg):
    pos = idx % (cfg.grid_h * cfg.grid_w)
    y, x = pos // cfg.grid_w, pos % cfg.grid_w
    return float(((y == 0) | (y == cfg.grid_h - 1) | (x == 0) | (x == cfg.grid_w - 1)).mean())


@pytest.mark.parametrize("name", ["draft", "c3_16k"])
def test_ablation_modes_and_border_share(hippo, name):
    cfg = si.CONFIGS[name]
    x = si.make_inputs(cfg, 1)
    dt, n = cfg.dtype, cfg.ctx_len
    kd, vd = dev(x["k"][:, :, :n], dt), dev(x["v"][:, :, :n], dt)
    q = dev(x["q_txt"], dt)
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    emb = oracle.keys_as_embedding(x["k"][:, :, :n], cfg.n_prefix, cfg.n_visual)
    sa = oracle.s_attn(x["q_txt"], x["k"][:, :, :n], cfg.n_prefix, cfg.n_visual)
    st = oracle.s_temp(emb, cfg.n_frames)
    ss = oracle.s_spa(emb, cfg.n_frames, cfg.grid_h, cfg.grid_w)
    share = {}
    for label, flags in (("attention only", 1), ("without temporal", 5), ("without spatial", 3), ("full", 7)):
        scores = hippo.hippo_score_tokens(q, kd, vid, flags=flags)
        idx, kp, _ = hippo.hippo_select_gather_kv(scores, cfg.k_keep, kd, vd, vid, cfg.n_q_heads)
        torch.cuda.synchronize()
        ref = oracle.fuse(sa, st, ss, cfg.n_frames, flags)
        assert_fused_close(host(scores), ref, (sa, st, ss), cfg.n_frames, dt, "%s %s" % (name, label), flags)
        np.testing.assert_array_equal(idx.cpu().numpy(), oracle.topk(host(scores), cfg.k_keep))
        assert kp.shape[2] == n - cfg.n_visual + cfg.k_keep
        share[label] = ring_share(idx.cpu().numpy(), cfg)
    border = 1 - (cfg.grid_h - 2) * (cfg.grid_w - 2) / (cfg.grid_h * cfg.grid_w)     # 23 % of a 16 x 16 grid
    assert share["attention only"] > 0.40 > border        # the position bias the paper measures (44-58 %)
    assert share["full"] < share["attention only"] - 0.05  # holistic fusion pulls the selection inward


def test_random_and_uniform_frame_retention(hippo):
    cfg = si.CONFIGS["draft"]
    x = si.make_inputs(cfg, 2)
    dt, n = cfg.dtype, cfg.ctx_len
    kd, vd = dev(x["k"][:, :, :n], dt), dev(x["v"][:, :, :n], dt)
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    P = cfg.grid_h * cfg.grid_w
    # random retention: the caller's random numbers are the scores
    r = si.random_scores(cfg.batch, cfg.n_visual, 5)
    idx, kp, vp = hippo.hippo_select_gather_kv(torch.from_numpy(r).cuda(), cfg.k_keep, kd, vd, vid, cfg.n_q_heads)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.topk(r, cfg.k_keep))
    np.testing.assert_array_equal(host(kp), oracle.gather(x["k"][:, :, :n], cfg.n_prefix, cfg.n_visual, idx.cpu().numpy()))
    assert 0.1 < ring_share(idx.cpu().numpy(), cfg) < 0.35          # no position preference
    # uniform frame dropping: keep every fourth frame whole -> score = 1 on kept frames, 0 elsewhere,
    # k = number of tokens in the kept frames (ties inside a frame resolve to ascending index)
    keep = np.arange(cfg.n_frames) % 4 == 0
    s = np.repeat(keep.astype(np.float32), P)[None].repeat(cfg.batch, 0)
    k = int(keep.sum()) * P
    idx, kp, vp = hippo.hippo_select_gather_kv(torch.from_numpy(s).cuda(), k, kd, vd, vid, cfg.n_q_heads)
    torch.cuda.synchronize()
    want = np.nonzero(np.repeat(keep, P))[0].astype(np.int32)
    np.testing.assert_array_equal(idx.cpu().numpy(), np.broadcast_to(want, (cfg.batch, k)))
    np.testing.assert_array_equal(host(vp), oracle.gather(x["v"][:, :, :n], cfg.n_prefix, cfg.n_visual, idx.cpu().numpy()))
