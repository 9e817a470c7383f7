"""Host-side control of video parallel speculative decoding: no GPU.

The reference timeline (oracle/vpsd_ref.py) is pinned to the numbers the paper prints and to closed
forms; the library's state machine and timing model are then compared with it on random acceptance
streams, counter by counter."""
import ctypes as C

import numpy as np
import pytest

import paper_2601_08273_amd as h
from oracle import vpsd_ref as ref


# ---- pins of the reference: what the paper prints, and closed forms ------------------------------

def test_paper_toy_speedups_of_serial_sd():
    """Motivated Experiments, "Non-negligible Draft Latency": T_target = 3 T_draft, gamma = 3:
    speedup 2 if all three drafts are accepted, 0.5 if the first is rejected."""
    td, tt, g = 1.0, 3.0, 3
    all_ok = ref.serial_sd(g, td, tt, [1] * 300, 400)
    assert all_ok.emitted == 400 and all_ok.rounds == 100
    assert all_ok.speedup_over(tt) == pytest.approx(2.0, abs=1e-12)
    none_ok = ref.serial_sd(g, td, tt, [0] * 400, 400)
    assert none_ok.rounds == 400 and none_ok.draft_wasted == 1200
    assert none_ok.speedup_over(tt) == pytest.approx(0.5, abs=1e-12)
    assert ref.autoregressive(50, tt).speedup_over(tt) == pytest.approx(1.0)


def test_paper_prefill_buffer_example():
    """"Synchronous Draft-Target Prefill": 0.8 s vs 0.2 s at 50 ms per draft token -> about 12."""
    assert h.vpsd_prefill_buffer(0.8, 0.2, 0.05) == 12
    assert h.vpsd_prefill_buffer(0.2, 0.8, 0.05) == 0
    assert h.vpsd_prefill_buffer(0.8, 0.2, 0.07) == 8
    assert h.vpsd_prefill_buffer(0.8, 0.2, 0.0) == -1
    assert h.vpsd_prefill_buffer(float("nan"), 0.2, 0.05) == -1


def test_vpsd_closed_forms():
    td, tt, g = 1.0, 3.0, 3
    # every draft accepted: after the conservative start each round emits gamma tokens per
    # max(T_t, gamma T_d) -> speedup -> gamma * T_t / max(T_t, gamma T_d) = 3
    n = 3000
    a = ref.vpsd(g, td, tt, [], n)
    assert a.mode_switches == 1
    # start: T_d + max(T_t, 2 T_d) for x_1, then rounds of 2, 3, 3, ... tokens each max(3, 3) = 3
    assert a.time == pytest.approx(4.0 + 3.0 * (a.rounds - 1))
    assert a.speedup_over(tt) == pytest.approx(3.0, rel=2e-3)
    assert a.draft_wasted == a.draft_tokens - a.emitted      # only the final look-ahead batch is left over
    # every first token rejected: one token per T_d + T_t -> 0.75 (serial SD: 0.5, see above)
    r = ref.vpsd(g, td, tt, [0] * 1000, 1000)
    assert r.rounds == 1000 and r.mode_switches == 0
    assert r.speedup_over(tt) == pytest.approx(3.0 / 4.0, abs=1e-12)
    # a slower draft model bounds the optimistic rate: gamma T_d > T_t
    s = ref.vpsd(4, 1.0, 2.0, [], 4000)
    assert s.speedup_over(2.0) == pytest.approx(4 * 2.0 / 4.0, rel=2e-3)
    # the prefill buffer is verified in one go and saves the serial first draft
    b = ref.vpsd(g, td, tt, [], 12 + 3, n_prefill_buffer=12)
    assert b.rounds == 2 and b.emitted == 15 and b.time == pytest.approx(6.0) and b.mode_switches == 0


def test_vpsd_beats_serial_sd_when_the_two_models_are_balanced():
    """With gamma T_draft close to T_target (the regime the parallel schedule is built for: neither
    model waits long for the other) it wins at every acceptance rate.  It is NOT a theorem for a
    target many times slower than a whole draft batch: there conservative mode spends a full target
    forward on x_1 alone."""
    r = np.random.default_rng(0)
    for rate in (0.2, 0.5, 0.8, 0.95):
        flags = (r.random(4000) < rate).astype(int).tolist()
        for g, td, tt in ((3, 1.0, 3.0), (5, 1.0, 2.5), (5, 1.0, 5.0), (8, 1.0, 6.0)):
            sd = ref.serial_sd(g, td, tt, flags, 1000)
            vp = ref.vpsd(g, td, tt, flags, 1000)
            assert vp.speedup_over(tt) > sd.speedup_over(tt)


# ---- the library against the reference ----------------------------------------------------------

FIELDS = [("n_emitted", "emitted"), ("n_rounds", "rounds"), ("n_target_calls", "target_calls"),
          ("n_draft_tokens", "draft_tokens"), ("n_draft_wasted", "draft_wasted"),
          ("n_mode_switches", "mode_switches"), ("n_flags_used", "flags_used")]


@pytest.mark.parametrize("seed", range(6))
def test_simulation_matches_reference(seed):
    r = np.random.default_rng(seed)
    for _ in range(40):
        g = int(r.integers(1, 9))
        td = float(r.uniform(0.2, 2.0))
        tt = float(r.uniform(0.5, 6.0))
        rate = float(r.uniform(0.05, 0.98))
        n = int(r.integers(1, 400))
        buf = int(r.integers(0, 14)) if r.random() < 0.5 else 0
        flags = (r.random(int(r.integers(0, 1200))) < rate).astype(int).tolist()
        got = h.vpsd_simulate(h.POLICY_VPSD, g, td, tt, flags, n, buf)
        want = ref.vpsd(g, td, tt, flags, n, buf)
        for a, b in FIELDS:
            assert getattr(got, a) == getattr(want, b), (a, g, td, tt, n, buf)
        assert got.time == pytest.approx(want.time, rel=1e-12)
        assert got.speedup == pytest.approx(want.speedup_over(tt), rel=1e-12)
        got = h.vpsd_simulate(h.POLICY_SERIAL_SD, g, td, tt, flags, n)
        want = ref.serial_sd(g, td, tt, flags, n)
        for a, b in FIELDS:
            if b != "mode_switches":
                assert getattr(got, a) == getattr(want, b), (a, g, n)
        assert got.time == pytest.approx(want.time, rel=1e-12)
    ar = h.vpsd_simulate(h.POLICY_AUTOREGRESSIVE, 3, 1.0, 3.0, [], 77)
    assert ar.n_emitted == 77 and ar.speedup == pytest.approx(1.0) and ar.time == pytest.approx(231.0)


def test_library_reproduces_the_paper_numbers():
    assert h.vpsd_simulate(h.POLICY_SERIAL_SD, 3, 1.0, 3.0, [1] * 300, 400).speedup == pytest.approx(2.0)
    assert h.vpsd_simulate(h.POLICY_SERIAL_SD, 3, 1.0, 3.0, [0] * 400, 400).speedup == pytest.approx(0.5)
    assert h.vpsd_simulate(h.POLICY_VPSD, 3, 1.0, 3.0, [0] * 400, 400).speedup == pytest.approx(0.75)
    assert h.vpsd_simulate(h.POLICY_VPSD, 3, 1.0, 3.0, [], 30000).speedup == pytest.approx(3.0, rel=1e-3)


def test_state_machine_round_by_round():
    s = h.vpsd_init(5)
    assert s.mode == h.VPSD_CONSERVATIVE and s.n_pending == 0
    r = h.vpsd_plan(s)
    assert (r.draft_serial, r.verify_len, r.draft_parallel) == (1, 1, 4)      # x_1 alone, x_2..x_5 meanwhile
    h.vpsd_commit(s, r, 1)                                                    # accepted
    assert s.mode == h.VPSD_OPTIMISTIC and s.n_pending == 4 and s.n_emitted == 1
    r = h.vpsd_plan(s)
    assert (r.draft_serial, r.verify_len, r.draft_parallel) == (0, 4, 5)
    h.vpsd_commit(s, r, 4)                                                    # all accepted: next batch is ready
    assert s.mode == h.VPSD_OPTIMISTIC and s.n_pending == 5 and s.n_emitted == 5
    r = h.vpsd_plan(s)
    assert (r.verify_len, r.draft_parallel) == (5, 5)
    h.vpsd_commit(s, r, 2, 3)                                                 # rejection at the third token
    assert s.mode == h.VPSD_CONSERVATIVE and s.n_pending == 0 and s.n_emitted == 5 + 3
    assert s.n_draft_wasted == 3 + 3 and s.n_mode_switches == 2
    r = h.vpsd_plan(s)
    assert (r.draft_serial, r.verify_len, r.draft_parallel) == (1, 1, 4)
    h.vpsd_commit(s, r, 0, 2)                                                 # x_1 rejected, drafting aborted
    assert s.mode == h.VPSD_CONSERVATIVE and s.n_emitted == 9 and s.n_draft_wasted == 6 + 1 + 2
    # with a prefill buffer generation starts optimistic and verifies the whole buffer at once
    s = h.vpsd_init(5, 12)
    r = h.vpsd_plan(s)
    assert s.mode == h.VPSD_OPTIMISTIC and (r.verify_len, r.draft_parallel) == (12, 5)


def test_state_machine_errors():
    lib = h.load()
    s, r = h.VpsdState(), h.VpsdRound()
    assert lib.hippo_vpsd_init(None, 5, 0) == h.ERR_NULL_ARG
    assert lib.hippo_vpsd_init(C.byref(s), 0, 0) == h.ERR_BAD_SHAPE
    assert lib.hippo_vpsd_init(C.byref(s), 65, 0) == h.ERR_BAD_SHAPE
    assert lib.hippo_vpsd_init(C.byref(s), 5, -1) == h.ERR_BAD_SHAPE
    assert lib.hippo_vpsd_init(C.byref(s), 5, 0) == h.OK
    assert lib.hippo_vpsd_plan(C.byref(s), None) == h.ERR_NULL_ARG
    assert lib.hippo_vpsd_plan(C.byref(s), C.byref(r)) == h.OK
    assert lib.hippo_vpsd_commit(C.byref(s), C.byref(r), 2, 4) == h.ERR_BAD_SHAPE      # more than were verified
    assert lib.hippo_vpsd_commit(C.byref(s), C.byref(r), 1, 5) == h.ERR_BAD_SHAPE      # more than were asked for
    assert lib.hippo_vpsd_commit(C.byref(s), C.byref(r), 1, 2) == h.ERR_BAD_SHAPE      # kept batch incomplete
    stale = h.VpsdRound(h.VPSD_OPTIMISTIC, 0, 5, 5)
    assert lib.hippo_vpsd_commit(C.byref(s), C.byref(stale), 5, 5) == h.ERR_BAD_SHAPE  # not this state's round
    # a round of the right mode whose other fields differ from the planned one is refused too
    for bad in (h.VpsdRound(r.mode, r.draft_serial + 1, r.verify_len, r.draft_parallel),
                h.VpsdRound(r.mode, r.draft_serial, r.verify_len + 1, r.draft_parallel),
                h.VpsdRound(r.mode, r.draft_serial, r.verify_len, r.draft_parallel + 1)):
        assert lib.hippo_vpsd_commit(C.byref(s), C.byref(bad), 0, 0) == h.ERR_BAD_SHAPE
    res = h.VpsdResult()
    assert lib.hippo_vpsd_simulate(7, 3, 1.0, 3.0, 0, None, 0, 10, C.byref(res)) == h.ERR_BAD_SHAPE
    assert lib.hippo_vpsd_simulate(2, 3, 0.0, 3.0, 0, None, 0, 10, C.byref(res)) == h.ERR_BAD_SHAPE
    assert lib.hippo_vpsd_simulate(2, 3, 1.0, 3.0, 0, None, 5, 10, C.byref(res)) == h.ERR_NULL_ARG
    assert lib.hippo_vpsd_simulate(2, 3, 1.0, 3.0, 0, None, 0, 10, None) == h.ERR_NULL_ARG


def test_refused_commit_leaves_the_state_unchanged():
    lib = h.load()
    for gamma, buf in ((5, 0), (5, 12), (1, 0)):
        s = h.vpsd_init(gamma, buf)
        r = h.vpsd_plan(s)
        before = bytes(s)
        refused = [(r, r.verify_len + 1, r.draft_parallel), (r, -1, 0), (r, r.verify_len, r.draft_parallel + 1),
                   (h.VpsdRound(1 - r.mode, r.draft_serial, r.verify_len, r.draft_parallel), 0, 0),
                   (h.VpsdRound(r.mode, r.draft_serial, r.verify_len + 2, r.draft_parallel), 0, 0)]
        if r.draft_parallel > 0:
            refused.append((r, r.verify_len, r.draft_parallel - 1))     # fully accepted, kept batch incomplete
        for rnd, n_acc, n_par in refused:
            assert lib.hippo_vpsd_commit(C.byref(s), C.byref(rnd), n_acc, n_par) == h.ERR_BAD_SHAPE
            assert bytes(s) == before, (gamma, buf, n_acc, n_par)
        h.vpsd_commit(s, r, r.verify_len)                               # and the planned round still commits
        assert s.n_rounds == 1
