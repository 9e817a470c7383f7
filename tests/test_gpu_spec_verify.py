"""GPU parity: hippo_spec_verify (through the C ABI) vs the CPU oracle of Eq. 1 and the resampling
rule.

What is compared, and how:
  alpha       fp32 vs fp64: |alpha - ref| <= 1e-5 * max(ref, rms) (the library forms the ratio in
              double from fp32 row sums, whose relative error is a few 1e-7).
  n_accept    an integer decided by `u < alpha`: identical whenever no u of the sequence lies within
              2e-5 * alpha of its alpha (both sides decide in their own precision; a u that close to
              the threshold is a coin the paper does not define) -- such sequences are skipped and
              must stay rare.
  next_token  an integer decided by where u * sum falls in a running sum: the GPU's word must be a
              valid inverse-CDF answer for the oracle's fp64 running sum C, i.e. it carries mass
              and C[t-1] - tol <= u * C[-1] <= C[t] + tol with tol = 2e-5 * C[-1]; and it must be
              the oracle's very word in the vast majority of cases.
  greedy      everything is integer work on identical inputs: bit exact.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity_util import dev, host, prep

pytestmark = pytest.mark.gpu


def softmax64(x, T):
    z = np.asarray(x, dtype=np.float64) / T
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def run_case(hippo, pl, ql, tok, ua, us, T, dtype, pad=0, what=""):
    pl, ql = prep(pl, dtype), prep(ql, dtype)
    B, g1, V = pl.shape
    gamma = g1 - 1
    ua32, us32 = ua.astype(np.float32), us.astype(np.float32)

    def padded(x):
        if pad == 0:
            return dev(x, dtype)
        full = np.full(x.shape[:2] + (V + pad,), 77.0, dtype=np.float32)    # garbage beyond the vocabulary
        full[..., :V] = x
        return dev(full, dtype)[..., :V]
    n_acc, nxt, alpha = hippo.hippo_spec_verify(
        padded(pl), padded(ql) if gamma > 0 or T > 0 else None, torch.from_numpy(tok.astype(np.int32)).cuda(),
        torch.from_numpy(ua32).cuda(), torch.from_numpy(us32).cuda(), T, want_alpha=True)
    torch.cuda.synchronize()
    n_acc, nxt, alpha = n_acc.cpu().numpy(), nxt.cpu().numpy(), host(alpha).astype(np.float64)
    r_acc, r_nxt, r_alpha = oracle.spec_verify(pl, ql, tok, ua32, us32, T)

    rms = float(np.sqrt(np.mean(r_alpha ** 2))) if r_alpha.size else 0.0
    assert np.all(np.abs(alpha - r_alpha) <= 1e-5 * np.maximum(r_alpha, rms)), (what, np.abs(alpha - r_alpha).max())

    ambiguous = (np.abs(ua32.astype(np.float64) - r_alpha) <= 2e-5 * r_alpha).any(axis=1) if gamma else np.zeros(B, bool)
    assert ambiguous.mean() <= 0.02, what
    ok = ~ambiguous
    np.testing.assert_array_equal(n_acc[ok], r_acc[ok], err_msg=what)

    p = softmax64(pl, T)
    q = softmax64(ql, T) if gamma else None
    same = 0
    for b in np.nonzero(ok)[0]:
        j = r_acc[b]
        r = p[b, j] if j == gamma else np.maximum(p[b, j] - q[b, j], 0.0)
        if r.sum() == 0:
            r = p[b, j]
        C = np.cumsum(r)
        t = int(nxt[b])
        assert 0 <= t < V and r[t] > 0, (what, b, t)
        target, tol = float(us32[b]) * C[-1], 2e-5 * C[-1]
        assert (C[t - 1] if t else 0.0) - tol <= target <= C[t] + tol, (what, b, t, int(r_nxt[b]))
        same += int(t == r_nxt[b])
    assert same >= 0.98 * ok.sum(), (what, same, int(ok.sum()))
    return n_acc, nxt


def synth_logits(B, gamma, V, seed, closeness):
    return si.make_logits(B, gamma, V, seed, closeness)


def draw_from(q_logits, T, r):
    q = softmax64(q_logits, T)
    u = r.random(q.shape[:-1])[..., None]
    return np.minimum((np.cumsum(q, -1) < u).sum(-1), q.shape[-1] - 1).astype(np.int32)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("B,gamma,V,T,pad", [
    (64, 5, 1000, 1.0, 0),          # one segment, ragged
    (48, 3, 8192, 0.7, 0),          # exactly one segment
    (32, 5, 8200, 1.3, 8),          # a second segment holding 8 words; padded rows
    (24, 8, 40003, 1.0, 5 + 8),     # five segments, odd length (scalar tail), odd padding -> multiple of 8 with V
    (8, 5, 151936, 0.8, 0),         # the 7B-class vocabulary
    (16, 1, 32000, 1.0, 0),         # conservative mode: x_1 alone
    (16, 0, 32000, 1.0, 0),         # no draft: plain sampling from p_0
])
def test_sampling_parity(hippo, dtype, B, gamma, V, T, pad):
    if (V + pad) % 8:
        pad += 8 - (V + pad) % 8
    pl, ql, r = synth_logits(B, gamma, V, B + gamma + V, 0.6)
    tok = draw_from(ql, T, r) if gamma else np.zeros((B, 0), np.int32)
    ua, us = r.random((B, gamma)), r.random(B)
    n_acc, _ = run_case(hippo, pl, ql, tok, ua, us, T, dtype, pad, "%s B%d g%d V%d" % (dtype, B, gamma, V))
    if gamma >= 3:
        assert 0 < n_acc.mean() < gamma          # the inputs exercise both outcomes


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_masked_words_edge_uniforms_and_bad_tokens(hippo, dtype):
    B, gamma, V, T = 40, 4, 20000, 1.0
    pl, ql, r = synth_logits(B, gamma, V, 5, 0.5)
    pl[:, :, ::3] = -np.inf                       # a third of the vocabulary masked for the target
    ql[:, :, 1::3] = -np.inf                      # another third for the draft
    pl[:, :, 17000:] = -np.inf                    # the last segment has target mass nowhere
    tok = draw_from(ql, T, r)
    tok[0, 0] = -1                                # not a word -> rejected at once
    tok[1, 1] = V
    tok[2, 0] = 1                                 # q = 0 there, p >= q -> alpha 1
    ua, us = r.random((B, gamma)), r.random(B)
    us[:8] = 0.0
    us[8:16] = np.nextafter(np.float32(1), np.float32(0))
    ua[16:20] = 0.0
    ql_ref, tok_ref = ql.copy(), tok.copy()
    # the oracle has no notion of a non-word: give it a word with p = 0 < q there (alpha 0 as well)
    for b, i in ((0, 0), (1, 1)):
        tok_ref[b, i] = 0
        ql_ref[b, i, 0] = 0.0
    pl_d, ql_d = prep(pl, dtype), prep(ql, dtype)
    n_acc, nxt, alpha = hippo.hippo_spec_verify(dev(pl_d, dtype), dev(ql_d, dtype), torch.from_numpy(tok).cuda(),
                                                torch.from_numpy(ua.astype(np.float32)).cuda(),
                                                torch.from_numpy(us.astype(np.float32)).cuda(), T, want_alpha=True)
    torch.cuda.synchronize()
    n_acc, nxt, alpha = n_acc.cpu().numpy(), nxt.cpu().numpy(), host(alpha)
    assert n_acc[0] == 0 and alpha[0, 0] == 0 and alpha[1, 1] == 0 and n_acc[1] <= 1
    assert alpha[2, 0] == 1.0
    p, q = softmax64(pl_d, T), softmax64(ql_d, T)
    for b in range(B):
        j = n_acc[b]
        res = p[b, j] if j == gamma else np.maximum(p[b, j] - q[b, j], 0)
        assert res[nxt[b]] > 0 and nxt[b] % 3 != 0 and nxt[b] < 17000, (b, j, nxt[b])
        if b < 8 and b > 2:                        # u_sample = 0: the first word with mass
            assert nxt[b] == np.nonzero(res > 0)[0][0]
        if 8 <= b < 16:                            # u_sample just below 1: at most a few ulps from the last
            C = np.cumsum(res)
            assert C[nxt[b]] >= (1 - 1e-5) * C[-1]
    # everything else against the oracle, on the rows without non-words
    keep = np.arange(3, B)
    r_acc, r_nxt, r_alpha = oracle.spec_verify(pl_d[keep], ql_d[keep], tok[keep], ua[keep], us[keep], T)
    np.testing.assert_allclose(alpha[keep], r_alpha, rtol=1e-5, atol=1e-30)
    np.testing.assert_array_equal(n_acc[keep], r_acc)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("B,gamma,V", [(64, 5, 1000), (16, 8, 40003), (4, 5, 151936), (8, 1, 8193), (8, 0, 5000)])
def test_greedy_bit_exact(hippo, dtype, B, gamma, V):
    r = np.random.default_rng(V + gamma)
    pl = prep(r.standard_normal((B, gamma + 1, V)).astype(np.float32), dtype)
    if V > 9000:
        pl[:, :, 8192 + 7] = pl.max(-1)              # a tie across segments: the lower index wins
        pl[:, :, 3] = pl.max(-1)
    tok = pl.argmax(-1)[:, :gamma].astype(np.int32)
    flip = r.random((B, gamma)) < 0.25
    tok[flip] = r.integers(0, V, int(flip.sum()))
    full = np.full((B, gamma + 1, (V + 7) // 8 * 8), 1e30, dtype=np.float32)   # row padding must not be read
    full[..., :V] = pl
    n_acc, nxt, alpha = hippo.hippo_spec_verify(dev(full, dtype)[..., :V], None, torch.from_numpy(tok).cuda(), None,
                                                None, 0.0, want_alpha=True)
    torch.cuda.synchronize()
    r_acc, r_nxt, r_alpha = oracle.spec_verify(pl, None, tok, np.zeros((B, gamma)), np.zeros(B), 0.0)
    np.testing.assert_array_equal(n_acc.cpu().numpy(), r_acc)
    np.testing.assert_array_equal(nxt.cpu().numpy(), r_nxt)
    np.testing.assert_array_equal(host(alpha), r_alpha)


def test_identical_models_accept_all(hippo):
    B, gamma, V = 16, 5, 30000
    pl, _, r = synth_logits(B, gamma, V, 2, 0.0)
    tok = draw_from(pl[:, :gamma], 1.0, r)
    ua = np.full((B, gamma), np.nextafter(np.float32(1), np.float32(0)))
    n_acc, nxt, alpha = hippo.hippo_spec_verify(dev(pl, "fp32"), dev(pl[:, :gamma].copy(), "fp32"),
                                                torch.from_numpy(tok).cuda(), torch.from_numpy(ua.astype(np.float32)).cuda(),
                                                torch.from_numpy(r.random(B).astype(np.float32)).cuda(), 1.0, want_alpha=True)
    torch.cuda.synchronize()
    assert (host(alpha) == 1.0).all() and (n_acc.cpu().numpy() == gamma).all()


def test_emitted_token_follows_target_on_gpu(hippo):
    """Losslessness measured on the GPU path itself (gamma = 1, 6-word vocabulary, stratified
    uniforms): the first emitted token is distributed as the target's p."""
    V, T, n = 6, 1.0, 100
    r = np.random.default_rng(4)
    p_log = (r.standard_normal(V) * 1.5).astype(np.float32)
    q_log = (r.standard_normal(V) * 1.5).astype(np.float32)
    p, q = softmax64(p_log, T), softmax64(q_log, T)
    X, UA, US = np.meshgrid(np.arange(V), (np.arange(n) + 0.5) / n, (np.arange(n) + 0.5) / n, indexing="ij")
    B = X.size
    Vp = 8
    pl = np.full((B, 2, Vp), -np.inf, np.float32); pl[:, :, :V] = p_log
    ql = np.full((B, 1, Vp), -np.inf, np.float32); ql[:, :, :V] = q_log
    n_acc, nxt = hippo.hippo_spec_verify(torch.from_numpy(pl).cuda(), torch.from_numpy(ql).cuda(),
                                         torch.from_numpy(X.reshape(B, 1).astype(np.int32)).cuda(),
                                         torch.from_numpy(UA.reshape(B, 1).astype(np.float32)).cuda(),
                                         torch.from_numpy(US.reshape(B).astype(np.float32)).cuda(), T)
    torch.cuda.synchronize()
    first = np.where(n_acc.cpu().numpy() >= 1, X.reshape(B), nxt.cpu().numpy())
    dist = np.bincount(first, weights=q[X.reshape(B)] / (n * n), minlength=Vp)[:V]
    np.testing.assert_allclose(dist, p, atol=1.0 / n)
