"""The comparison helpers the GPU parity tests rely on must themselves reject mistakes: planted errors on the CPU
(in copies of the oracle's own results) have to fail, rounding-sized perturbations have to pass."""
import numpy as np
import pytest

import oracle
import synth_inputs as si
from parity_util import assert_close, assert_fused_close


def _tiny_scores():
    cfg = si.CONFIGS["tiny"]
    x = si.make_inputs(cfg, 0)
    n = cfg.ctx_len
    rs, rc = oracle.score_tokens(x["q_txt"], x["k"][:, :, :n], cfg.n_prefix, cfg.n_frames, cfg.grid_h, cfg.grid_w)
    return cfg, rs, rc


def test_fused_fp32_bound_passes_rounding_and_rejects_planted_mistakes():
    cfg, rs, rc = _tiny_scores()
    F = cfg.n_frames
    # fp32 rounding of the raw terms, pushed through Eq. 7 by the oracle itself: must pass
    rounded = [t.astype(np.float32).astype(np.float64) for t in rc]
    assert_fused_close(oracle.fuse(*rounded, F), rs, rc, F, "fp32", "fp32-rounded terms")
    # a raw attention term off by a relative 1e-3 (a wrong scale, a dropped head) moves the fused score far
    # outside the propagated bound ...
    wrong = oracle.fuse(rc[0] * (1 + 1e-3 * np.sign(rc[0] - rc[0].mean())), rc[1], rc[2], F)
    with pytest.raises(AssertionError):
        assert_fused_close(wrong, rs, rc, F, "fp32", "scaled attention term")
    # ... so does a term left out of the sum, one token shifted by a position, or a z-score without its mean
    with pytest.raises(AssertionError):
        assert_fused_close(oracle.fuse(rc[0], rc[1], rc[2], F, flags=3), rs, rc, F, "fp32", "dropped spatial term")
    with pytest.raises(AssertionError):
        assert_fused_close(np.roll(rs, 1, axis=1), rs, rc, F, "fp32", "shifted by one token")
    with pytest.raises(AssertionError):
        assert_fused_close(rs + 1e-3, rs, rc, F, "fp32", "constant offset")
    # a single element wrong by 1e-3 of its own size is enough
    one = rs.copy()
    i = np.unravel_index(np.argmax(np.abs(rs)), rs.shape)
    one[i] *= 1 + 1e-3
    with pytest.raises(AssertionError):
        assert_fused_close(one, rs, rc, F, "fp32", "one element")


def test_fused_bound_is_no_wider_than_the_terms_allow():
    """The bound is the raw terms' 1e-5 pushed through Eq. 7, not a blanket tolerance: where a frame's term
    varies as much as it is large (|mean| ~ sigma) the allowance stays within a few 1e-5."""
    B, F, P = 1, 2, 64
    rng = np.random.default_rng(5)
    terms = [rng.standard_normal((B, F * P)) for _ in range(3)]        # mean ~ 0, sigma ~ 1
    ref = oracle.fuse(*terms, F)
    assert_fused_close(ref + 2e-5, ref, terms, F, "fp32", "rounding-sized")   # (|x|+|mu|)/sigma + |z| ~ 2 per term
    with pytest.raises(AssertionError):
        assert_fused_close(ref + 5e-4, ref, terms, F, "fp32", "far outside")


def test_bf16_bound_rejects_what_it_should():
    r = np.random.default_rng(1).standard_normal((4, 64)) * 1e-2
    assert_close(r * (1 + 2.0 ** -8), r, "bf16", "two bf16 roundings")
    with pytest.raises(AssertionError):
        assert_close(r * 1.05, r, "bf16", "5 % off")
    with pytest.raises(AssertionError):       # the absolute term alone would let this through on small outputs
        assert_close(r + 3e-3, r, "bf16", "offset of a third of the rms")
