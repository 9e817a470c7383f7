"""hippo_verify_attention_static (the entry point that allocates nothing: its split partials live in
the library's static device array) against hippo_verify_attention, through the C ABI: two calls in a
row on the same GPU, the second on a smaller input, plus the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import assert_close, dev, host

pytestmark = pytest.mark.gpu


def _both(hippo, q, k, v, ctx, num_splits=0):
    """outputs and lse of the workspace call and of the static call, all buffers caller-made"""
    lib = hippo.load()
    B, q_len, H, d = q.shape
    kv = hippo.kv_desc(k, H)
    ws = torch.empty(hippo.workspace_bytes(hippo.CALL_VERIFY_ATTENTION, kv, None, q_len, ctx + q_len, 0, num_splits),
                     dtype=torch.uint8, device="cuda")
    out_a, out_b = torch.zeros_like(q), torch.zeros_like(q)
    lse_a = torch.zeros((B, H, q_len), dtype=torch.float32, device="cuda")
    lse_b = torch.zeros_like(lse_a)
    st = torch.cuda.current_stream().cuda_stream or None
    rc = lib.hippo_verify_attention(q.data_ptr(), q_len, k.data_ptr(), v.data_ptr(), C.byref(kv), ctx, 0.0, num_splits,
                                    out_a.data_ptr(), lse_a.data_ptr(), ws.data_ptr(), ws.numel(), st)
    assert rc == hippo.OK
    rc = lib.hippo_verify_attention_static(q.data_ptr(), q_len, k.data_ptr(), v.data_ptr(), C.byref(kv), ctx, 0.0,
                                           num_splits, out_b.data_ptr(), lse_b.data_ptr(), st)
    assert rc == hippo.OK, hippo.status_string(rc)
    torch.cuda.synchronize()
    return out_a, lse_a, out_b, lse_b


def test_static_scratch_matches_the_workspace_call_twice_in_a_row(hippo):
    assert hippo.load().hippo_static_scratch_init() == hippo.OK
    # first the 16K headline shape (64 slices per KV head, 2.9 MB of partials), then a much smaller one
    # whose partials cover only the front of the array the first call filled
    big, small = si.CONFIGS["c3_16k"], si.CONFIGS["draft"]
    for cfg, splits in ((big, 0), (small, 0), (small, 5), (big, 0)):
        x = si.make_inputs(cfg, 1)
        dt = cfg.dtype
        q, k, v = dev(x["q_new"], dt), dev(x["k"], dt), dev(x["v"], dt)
        out_a, lse_a, out_b, lse_b = _both(hippo, q, k, v, cfg.ctx_len, splits)
        # same kernels, same slices, same arithmetic: the two calls agree bit for bit
        assert torch.equal(out_a, out_b), cfg.name
        assert torch.equal(lse_a, lse_b), cfg.name
        if cfg is small:                                    # and both are right (oracle in seconds)
            ro, rl = oracle.attention(x["q_new"], x["k"], x["v"], cfg.ctx_len)
            assert_close(host(out_b), ro, dt, "static-scratch verify")
            np.testing.assert_allclose(host(lse_b), rl, rtol=2.0 ** -9, atol=2.0 ** -9)


def test_static_scratch_fp32_and_size_limit(hippo):
    lib = hippo.load()
    cfg = si.CONFIGS["tiny"]
    x = si.make_inputs(cfg, 0)
    q, k, v = dev(x["q_new"], "fp32"), dev(x["k"], "fp32"), dev(x["v"], "fp32")
    out_a, lse_a, out_b, lse_b = _both(hippo, q, k, v, cfg.ctx_len)
    assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)
    ro, _ = oracle.attention(x["q_new"], x["k"], x["v"], cfg.ctx_len)
    assert_close(host(out_b), ro, "fp32", "static-scratch verify, fp32")
    # beyond the array: refused with its own status, nothing enqueued, output untouched
    B, Hkv, H, d, n = 4, 8, 64, 128, 4096
    kq = torch.zeros((B, Hkv, n + 6, d), dtype=torch.bfloat16, device="cuda")
    qq = torch.zeros((B, 6, H, d), dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(qq, 7.0)
    kv = hippo.kv_desc(kq, H)
    assert hippo.workspace_bytes(hippo.CALL_VERIFY_ATTENTION, kv, None, 6, n + 6, 0, 64) > lib.hippo_static_scratch_bytes()
    rc = lib.hippo_verify_attention_static(qq.data_ptr(), 6, kq.data_ptr(), kq.data_ptr(), C.byref(kv), n, 0.0, 64,
                                           out.data_ptr(), None, None)
    assert rc == hippo.ERR_STATIC_SCRATCH_LIMIT
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
