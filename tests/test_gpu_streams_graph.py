"""Draft and verify attention on two concurrent streams, eagerly and as a replayed HIP graph.

The replays are interleaved with eager work and synchronisations, inputs change between replays,
and every replay is compared with the eager result and the oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from gpu_util import assert_close, dev, host

pytestmark = pytest.mark.gpu


def test_two_stream_round_eager_and_graph(hippo):
    cfg = si.CONFIGS["draft"]
    xs = [si.make_inputs(cfg, s) for s in (0, 1, 2)]
    dt, n = cfg.dtype, cfg.ctx_len
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    k, v = dev(xs[0]["k"], dt), dev(xs[0]["v"], dt)
    q, q1 = dev(xs[0]["q_new"], dt), dev(xs[0]["q_new"][:, :1], dt)
    scores = hippo.hippo_score_tokens(dev(xs[0]["q_txt"], dt), k[:, :, :n], vid)
    n_d = n - cfg.n_visual + cfg.k_keep
    kp = torch.zeros((cfg.batch, cfg.n_kv_heads, n_d + 1, cfg.head_dim), dtype=k.dtype, device="cuda")
    vp = torch.zeros_like(kp)
    idx, _, _ = hippo.hippo_select_gather_kv(scores, cfg.k_keep, k[:, :, :n], v[:, :, :n], vid, cfg.n_q_heads,
                                             k_dst=kp[:, :, :n_d], v_dst=vp[:, :, :n_d])
    kp[:, :, n_d], vp[:, :, n_d] = k[:, :, n], v[:, :, n]
    kvd = hippo.kv_desc(k, cfg.n_q_heads)
    ws_v = torch.empty(hippo.workspace_bytes(hippo.CALL_VERIFY_ATTENTION, kvd, None, cfg.q_len, n + cfg.q_len),
                       dtype=torch.uint8, device="cuda")
    ws_d = torch.empty(hippo.workspace_bytes(hippo.CALL_DRAFT_ATTENTION, hippo.kv_desc(kp, cfg.n_q_heads), None, 1,
                                             n_d + 1), dtype=torch.uint8, device="cuda")
    out_v, out_d = torch.empty_like(q), torch.empty_like(q1)
    sB = torch.cuda.Stream()

    def round_():
        cur = torch.cuda.current_stream()
        sB.wait_stream(cur)
        hippo.hippo_verify_attention(q, k, v, n, out=out_v, workspace=ws_v)
        hippo.hippo_draft_attention(q1, kp, vp, n_d, out=out_d, workspace=ws_d, stream=sB)
        cur.wait_stream(sB)

    def reference(x):
        rv, _ = oracle.attention(x["q_new"], host(k), host(v), n)
        rd, _ = oracle.attention(x["q_new"][:, :1], host(kp), host(vp), n_d)
        return rv, rd

    round_()
    torch.cuda.synchronize()
    rv, rd = reference(xs[0])
    assert_close(host(out_v), rv, dt, "eager verify")
    assert_close(host(out_d), rd, dt, "eager draft")
    eager_v, eager_d = out_v.clone(), out_d.clone()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        round_()
    for rep, x in enumerate([xs[0], xs[1], xs[2], xs[0]]):
        # new queries in place (the graph reads the same buffers), eager work between replays
        q.copy_(dev(x["q_new"], dt))
        q1.copy_(dev(x["q_new"][:, :1], dt))
        out_v.zero_()
        out_d.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        rv, rd = reference(x)
        assert_close(host(out_v), rv, dt, "replay %d verify" % rep)
        assert_close(host(out_d), rd, dt, "replay %d draft" % rep)
        if rep in (0, 3):
            assert torch.equal(out_v, eager_v) and torch.equal(out_d, eager_d)
