"""Pins of the speculative-sampling oracle (Eq. 1 and the resampling rule) to things it does not
compute itself: the losslessness theorem of speculative sampling (the emitted token is distributed
exactly as the target's p, whatever q is), the closed form of the acceptance rate
(sum_x min(p, q) = 1 - total variation), a hand-worked 4-word example, inverse-CDF boundaries,
the greedy limit by brute force, and planted-mistake checks that show the pins have teeth."""
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def logits_of(prob):
    with np.errstate(divide="ignore"):
        return np.log(np.asarray(prob, dtype=np.float64)).astype(np.float32)    # prob 0 -> -inf (a masked word)


def softmax(x, T):
    z = np.asarray(x, dtype=np.float64) / T
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def first_token_distribution(p_log, q_log, T, n_u=300, n_s=300, emit=None):
    """Integrate the oracle over x ~ q, u_accept ~ U, u_sample ~ U on midpoint grids (gamma = 1)
    and return the distribution of the first token the step emits."""
    V = p_log.shape[-1]
    q = softmax(q_log, T)
    ua = (np.arange(n_u) + 0.5) / n_u
    us = (np.arange(n_s) + 0.5) / n_s
    X, UA, US = np.meshgrid(np.arange(V), ua, us, indexing="ij")
    B = X.size
    pl = np.broadcast_to(np.stack([p_log, p_log]), (B, 2, V))     # row 1 (the extra token) is irrelevant here
    ql = np.broadcast_to(q_log[None, None], (B, 1, V))
    n_acc, nxt, _ = (emit or oracle.spec_verify)(pl, ql, X.reshape(B, 1), UA.reshape(B, 1), US.reshape(B), T)
    first = np.where(n_acc >= 1, X.reshape(B), nxt)
    w = (q[X.reshape(B)] / (n_u * n_s))
    return np.bincount(first, weights=w, minlength=V), float(np.sum(w * (n_acc >= 1)))


@pytest.mark.parametrize("seed,T", [(0, 1.0), (1, 0.6), (2, 1.7)])
def test_emitted_token_follows_target_distribution(seed, T):
    r = np.random.default_rng(seed)
    V = 7
    p_log = (r.standard_normal(V) * 1.5).astype(np.float32)
    q_log = (r.standard_normal(V) * 1.5).astype(np.float32)
    dist, acc = first_token_distribution(p_log, q_log, T)
    p, q = softmax(p_log, T), softmax(q_log, T)
    # midpoint grids: each of the V accept thresholds and V CDF steps is off by at most half a cell
    np.testing.assert_allclose(dist, p, atol=1.0 / 300)
    # acceptance rate = sum min(p, q) = 1 - TV(p, q)
    assert abs(acc - np.minimum(p, q).sum()) <= 1.0 / 300
    assert abs(acc - (1 - 0.5 * np.abs(p - q).sum())) <= 1.0 / 300


def test_planted_mistakes_break_losslessness():
    """The losslessness pin fails for the plausible slips: ratio upside down, residual with the
    operands swapped, residual without the clamp (i.e. resampling from p)."""
    r = np.random.default_rng(5)
    V, T = 6, 1.0
    p_log = (r.standard_normal(V) * 1.5).astype(np.float32)
    q_log = (r.standard_normal(V) * 1.5).astype(np.float32)
    p, q = softmax(p_log, T), softmax(q_log, T)

    def variant(alpha_fn, resid_fn):
        def run(pl, ql, tok, ua, us, T):
            B = tok.shape[0]
            x = tok[:, 0]
            a = alpha_fn(p[x], q[x])
            acc = ua[:, 0] < a
            res = resid_fn(p, q)
            cdf = np.cumsum(res / res.sum())
            nxt = np.minimum(np.searchsorted(cdf, us, side="right"), V - 1)
            return acc.astype(np.int32), nxt.astype(np.int32), a[:, None]
        return run

    good = variant(lambda a, b: np.minimum(1, a / b), lambda a, b: np.maximum(0, a - b))
    d, _ = first_token_distribution(p_log, q_log, T, emit=good)
    np.testing.assert_allclose(d, p, atol=1 / 300)                       # the harness itself is sound
    for bad in (variant(lambda a, b: np.minimum(1, b / a), lambda a, b: np.maximum(0, a - b)),
                variant(lambda a, b: np.minimum(1, a / b), lambda a, b: np.maximum(0, b - a)),
                variant(lambda a, b: np.minimum(1, a / b), lambda a, b: a)):
        d, _ = first_token_distribution(p_log, q_log, T, emit=bad)
        assert np.abs(d - p).max() > 0.02


def test_hand_worked_example():
    rows = [l for l in open(os.path.join(HERE, "golden", "eq1_hand_worked.txt")) if not l.startswith("#")]
    p_log = logits_of([0.5, 0.3, 0.2, 0.0])
    q_log = logits_of([0.2, 0.6, 0.1, 0.1])
    for line in rows:
        lhs, rhs = line.split("|")
        x, ua, us = lhs.split()
        acc, alpha, emitted = rhs.split()
        n_acc, nxt, a = oracle.spec_verify(np.stack([p_log, p_log])[None], q_log[None, None],
                                           np.array([[int(x)]]), np.array([[float(ua)]]), np.array([float(us)]), 1.0)
        assert int(n_acc[0]) == int(acc), line
        assert abs(a[0, 0] - float(alpha)) < 1e-6, line
        assert (int(x) if n_acc[0] == 1 else int(nxt[0])) == int(emitted), line


def test_identical_models_accept_everything_and_extra_token_is_inverse_cdf():
    prob = np.array([0.1, 0.2, 0.3, 0.4])
    lg = logits_of(prob)
    gamma = 3
    us = np.array([0.0, 0.05, 0.0999, 0.1001, 0.29, 0.31, 0.59, 0.61, 0.999], dtype=np.float32)
    want = np.array([0, 0, 0, 1, 1, 2, 2, 3, 3])
    B = us.size
    pl = np.broadcast_to(lg, (B, gamma + 1, 4))
    ql = np.broadcast_to(lg, (B, gamma, 4))
    tok = np.random.default_rng(0).integers(0, 4, (B, gamma))
    ua = np.full((B, gamma), 0.999999, dtype=np.float32)
    n_acc, nxt, a = oracle.spec_verify(pl, ql, tok, ua, us, 1.0)
    assert (n_acc == gamma).all() and (a == 1.0).all()
    np.testing.assert_array_equal(nxt, want)


def test_disjoint_support_rejects_and_resamples_from_target():
    p_log = logits_of([0.25, 0.75, 0, 0])
    q_log = logits_of([0, 0, 0.5, 0.5])
    us = np.array([0.1, 0.24, 0.26, 0.9], dtype=np.float32)
    B = 4
    n_acc, nxt, a = oracle.spec_verify(np.broadcast_to(p_log, (B, 3, 4)), np.broadcast_to(q_log, (B, 2, 4)),
                                       np.array([[2, 3]] * B), np.zeros((B, 2)), us, 1.0)
    assert (n_acc == 0).all() and np.all(a == 0)
    np.testing.assert_array_equal(nxt, [0, 0, 1, 1])


def test_chain_stops_at_first_rejection_and_ignores_the_rest():
    r = np.random.default_rng(3)
    B, gamma, V, T = 64, 5, 11, 0.9
    pl = r.standard_normal((B, gamma + 1, V)).astype(np.float32)
    ql = (pl[:, :gamma] + 0.7 * r.standard_normal((B, gamma, V))).astype(np.float32)
    tok = r.integers(0, V, (B, gamma))
    ua = r.random((B, gamma), dtype=np.float32)
    us = r.random(B, dtype=np.float32)
    n_acc, nxt, a = oracle.spec_verify(pl, ql, tok, ua, us, T)
    # independent recomputation of alpha with a library softmax
    p, q = softmax(pl, T), softmax(ql, T)
    px = np.take_along_axis(p[:, :gamma], tok[..., None], -1)[..., 0]
    qx = np.take_along_axis(q, tok[..., None], -1)[..., 0]
    np.testing.assert_allclose(a, np.minimum(1.0, px / qx), rtol=1e-12)
    rej = ~(ua < a)
    want = np.where(rej.any(1), rej.argmax(1), gamma)
    np.testing.assert_array_equal(n_acc, want)
    assert 0 < (n_acc == gamma).sum() < B               # both outcomes occur
    # whatever follows the first rejection cannot matter
    pl2, ql2, tok2, ua2 = pl.copy(), ql.copy(), tok.copy(), ua.copy()
    for b in range(B):
        j = n_acc[b]
        if j < gamma:
            pl2[b, j + 1:] = r.standard_normal((gamma - j, V))
            ql2[b, j + 1:] = r.standard_normal((gamma - j - 1, V))
            tok2[b, j + 1:] = r.integers(0, V, gamma - j - 1)
            ua2[b, j + 1:] = r.random(gamma - j - 1)
    n2, x2, _ = oracle.spec_verify(pl2, ql2, tok2, ua2, us, T)
    np.testing.assert_array_equal(n2, n_acc)
    np.testing.assert_array_equal(x2, nxt)
    # the replacement always has positive residual mass; the extra token positive target mass
    for b in range(B):
        j = n_acc[b]
        if j < gamma:
            assert p[b, j, nxt[b]] > q[b, j, nxt[b]]
        else:
            assert p[b, gamma, nxt[b]] > 0


def test_temperature_rescales_logits():
    prob = np.array([0.64, 0.16, 0.16, 0.04])
    lg = logits_of(prob)                       # T = 2 -> proportional to sqrt: 0.4 0.2 0.2 0.1 -> /1.0 ... normalised
    want = np.sqrt(prob) / np.sqrt(prob).sum()
    dist, _ = first_token_distribution(lg, logits_of([0.25] * 4), 2.0)
    np.testing.assert_allclose(dist, want, atol=1 / 300)


def test_greedy_is_argmax_agreement():
    r = np.random.default_rng(9)
    B, gamma, V = 200, 4, 13
    pl = r.standard_normal((B, gamma + 1, V)).astype(np.float32)
    pl[:, :, 5] = pl[:, :, 2]                               # ties: the lower index is the argmax
    am = pl.argmax(-1)                                      # numpy returns the first maximum
    tok = am[:, :gamma].copy()
    flip = r.random((B, gamma)) < 0.3
    tok[flip] = r.integers(0, V, flip.sum())
    n_acc, nxt, a = oracle.spec_verify(pl, None, tok, r.random((B, gamma)), r.random(B), 0.0)
    for b in range(B):
        j = 0
        while j < gamma and tok[b, j] == am[b, j]:
            j += 1
        assert n_acc[b] == j and nxt[b] == am[b, j]
    np.testing.assert_array_equal(a, (tok == am[:, :gamma]).astype(np.float64))


def test_low_temperature_approaches_greedy():
    r = np.random.default_rng(10)
    B, gamma, V = 50, 3, 9
    pl = r.standard_normal((B, gamma + 1, V)).astype(np.float32)
    ql = r.standard_normal((B, gamma, V)).astype(np.float32)
    tok = ql.argmax(-1)                                     # a greedy draft
    ua, us = r.random((B, gamma)) * 0.98 + 0.01, r.random(B) * 0.98 + 0.01
    g = oracle.spec_verify(pl, None, tok, ua, us, 0.0)
    s = oracle.spec_verify(pl, ql, tok, ua, us, 1e-3)
    np.testing.assert_array_equal(g[0], s[0])
    np.testing.assert_array_equal(g[1], s[1])
