"""The whole decoding round under the library's control logic, on the GPU: the state machine plans a
round; the target's verification attention (q_len = verify_len + 1 over the full cache) and the draft
model's decode attention (q_len = 1 over the pruned cache, on a second stream) run concurrently;
hippo_spec_verify (greedy, the paper's evaluation setting) gives the verdict; the state machine
commits it.  There is no model here: position t of the generation has fixed synthetic target and
draft logits and fixed K/V rows, which is all the control flow and the kernels can see.

Checked: every verification's attention output and verdict against the oracle (at that round's
cache length and width), the emitted sequence against plain greedy decoding with the target
(losslessness), and the final counters against the reference timeline driven by the same verdicts."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import assert_close, dev, host, prep
from oracle import vpsd_ref

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("gamma,buffer,closeness", [(5, 0, 0.35), (3, 0, 0.8), (4, 7, 0.2)])
def test_vpsd_rounds_on_two_streams(hippo, gamma, buffer, closeness):
    cfg = si.CONFIGS["draft"]
    dt, n_ctx = cfg.dtype, cfg.ctx_len
    x = si.make_inputs(cfg, 3)
    n_gen, V = 48, 4096
    B, H, Hkv, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    r = np.random.default_rng(gamma)
    n_new = n_gen + 80                                       # look-ahead drafts run past the end
    k_all = np.concatenate([x["k"][:, :, :n_ctx], r.standard_normal((B, Hkv, n_new, d)).astype(np.float32) / np.sqrt(d)], 2)
    v_all = np.concatenate([x["v"][:, :, :n_ctx], r.standard_normal((B, Hkv, n_new, d)).astype(np.float32) / np.sqrt(d)], 2)
    q_all = r.standard_normal((B, n_new, H, d)).astype(np.float32)
    k_all, v_all, q_all = prep(k_all, dt), prep(v_all, dt), prep(q_all, dt)
    P, Q, _ = si.make_logits(B, n_new, V, 11, closeness)     # P[:, t]: target row of position t; Q[:, t]: draft row
    P, Q = prep(P, dt), prep(Q, dt)
    draft_tok = Q.argmax(-1).astype(np.int32)                # a greedy draft model
    target_tok = P.argmax(-1)

    kd, vd, qd = dev(k_all, dt), dev(v_all, dt), dev(q_all, dt)
    Pd, tokd = dev(P, dt), torch.from_numpy(draft_tok).cuda()
    # the draft model's pruned cache and one decode query (the draft side only has to run concurrently)
    vid = hippo.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    scores = hippo.hippo_score_tokens(dev(x["q_txt"], dt), kd[:, :, :n_ctx], vid)
    _, kp, vp = hippo.hippo_select_gather_kv(scores, cfg.k_keep, kd[:, :, :n_ctx], vd[:, :, :n_ctx], vid, H)
    n_d = kp.shape[2] - 1
    out_d = torch.empty((B, 1, H, d), dtype=kd.dtype, device="cuda")
    sB = torch.cuda.Stream()

    state = hippo.vpsd_init(gamma, buffer)
    c = 0                                                    # positions committed so far
    emitted, verdicts = [], []
    while state.n_emitted < n_gen:
        rnd = hippo.vpsd_plan(state)
        v = rnd.verify_len
        cur = torch.cuda.current_stream()
        sB.wait_stream(cur)
        # target: the last committed token and the v drafts, appended at rows n_ctx + c ..
        q_round = qd[:, c:c + v + 1].contiguous()
        out_v = hippo.hippo_verify_attention(q_round, kd[:, :, :n_ctx + c + v + 1], vd[:, :, :n_ctx + c + v + 1], n_ctx + c)
        n_acc, nxt = hippo.hippo_spec_verify(Pd[:, c:c + v + 1].contiguous(), None, tokd[:, c:c + v].contiguous(),
                                             None, None, 0.0)
        # draft: draft_parallel single-token decodes, concurrently
        for _ in range(rnd.draft_parallel):
            hippo.hippo_draft_attention(qd[:, c:c + 1].contiguous(), kp, vp, n_d, out=out_d, stream=sB)
        cur.wait_stream(sB)
        a = int(n_acc.cpu()[0])                              # the verdict crosses to the host here
        ro, _ = oracle.attention(q_all[:, c:c + v + 1], k_all[:, :, :n_ctx + c + v + 1], v_all[:, :, :n_ctx + c + v + 1], n_ctx + c)
        assert_close(host(out_v), ro, dt, "verify width %d at position %d" % (v + 1, c))
        r_acc, r_nxt, _ = oracle.spec_verify(P[:, c:c + v + 1], None, draft_tok[:, c:c + v], np.zeros((B, v)), np.zeros(B), 0.0)
        assert a == r_acc[0] and int(nxt.cpu()[0]) == r_nxt[0]
        verdicts += [1] * a + ([0] if a < v else [])
        if a == v:
            emitted += draft_tok[0, c:c + v].tolist()
            hippo.vpsd_commit(state, rnd, a)
            c += v
        else:
            emitted += draft_tok[0, c:c + a].tolist() + [int(nxt.cpu()[0])]
            hippo.vpsd_commit(state, rnd, a, min(rnd.draft_parallel, 2))
            c += a + 1
        assert state.n_emitted == len(emitted) == c
    torch.cuda.synchronize()
    # lossless: exactly what greedy decoding with the target alone would have produced
    assert emitted == target_tok[0, :len(emitted)].tolist()
    assert 0 < sum(verdicts) < len(verdicts)                 # both outcomes occurred
    # the counters agree with the reference timeline fed the same verdicts (times: T_t = 2 T_d so
    # that two look-ahead drafts fit before a rejecting verdict, as committed above)
    ref = vpsd_ref.vpsd(gamma, 1.0, 2.0, verdicts, n_gen, buffer)
    assert (state.n_emitted, state.n_rounds, state.n_target_calls, state.n_mode_switches) == \
        (ref.emitted, ref.rounds, ref.target_calls, ref.mode_switches)
    assert state.n_draft_tokens == ref.draft_tokens
    assert state.n_draft_wasted + state.n_pending == ref.draft_wasted
