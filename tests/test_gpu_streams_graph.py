"""Draft and verify attention on two concurrent streams, eagerly and as a replayed HIP graph.

The replays are interleaved with eager work and synchronisations, inputs change between replays,
and every replay is compared with the eager result and the oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import assert_close, dev, host

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


def test_two_non_default_streams_with_wrapper_allocated_buffers(hippo):
    """Verify and draft on two side streams while the binding allocates workspace, outputs and lse
    itself: those buffers must belong to the stream the kernels run on, or the allocator may hand
    them to the allocations made here, between the calls, while the kernels still use them."""
    cfg = si.CONFIGS["draft"]
    x = si.make_inputs(cfg, 3)
    dt, n = cfg.dtype, cfg.ctx_len
    k, v = dev(x["k"], dt), dev(x["v"], dt)
    q, q1 = dev(x["q_new"], dt), dev(x["q_new"][:, :1], dt)
    rv, rlv = oracle.attention(x["q_new"], x["k"], x["v"], n)
    rd, rld = oracle.attention(x["q_new"][:, :1], x["k"][:, :, :n + 1], x["v"][:, :, :n + 1], n)
    sA, sB = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(6):
        outs = []
        for _ in range(4):                      # several calls in flight per stream, no workspace passed
            ov = hippo.hippo_verify_attention(q, k, v, n, want_lse=True, stream=sA)
            # allocations on the current (default) stream between the calls: what a recycled block would go to
            junk = [torch.full((1 << 18,), float(rep), device="cuda") for _ in range(8)]
            od = hippo.hippo_draft_attention(q1, k[:, :, :n + 1], v[:, :, :n + 1], n, want_lse=True, stream=sB)
            outs.append((ov, od))
            del junk
        torch.cuda.synchronize()
        for (ov, lv), (od, ld) in outs:
            assert_close(host(ov), rv, dt, "verify on a side stream, rep %d" % rep)
            assert_close(host(od), rd, dt, "draft on a side stream, rep %d" % rep)
            np.testing.assert_allclose(host(lv), rlv, rtol=2.0 ** -9, atol=2.0 ** -9)
            np.testing.assert_allclose(host(ld), rld, rtol=2.0 ** -9, atol=2.0 ** -9)
