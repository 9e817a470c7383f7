"""Reference timeline of the decoding schedules the paper compares (TEST INFRASTRUCTURE ONLY).

A deliberately literal, token-by-token event model of
  * plain autoregressive decoding with the target model,
  * serial speculative decoding (Motivated Experiments, "Non-negligible Draft Latency"),
  * video parallel speculative decoding with optimistic / conservative switching
    (Method, "Video Parallel Speculative Decoding"),
written independently of the library's state machine: it keeps two clocks (when each model becomes
free) and explicit token lists instead of counters.  Draft token number i (in the order tokens are
looked at by the target) is accepted iff accept[i]; flags past the end count as accepted.

Readings (shared with the library, since the paper leaves them open): in the parallel modes a fully
accepted verification emits exactly the verified tokens (the draft has already run past the
position the extra token would take); one verification takes the whole buffer; a rejection ends
concurrent drafting at the moment the verdict arrives.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence


@dataclass
class Timeline:
    time: float = 0.0
    emitted: int = 0
    rounds: int = 0
    target_calls: int = 0
    draft_tokens: int = 0
    draft_wasted: int = 0
    mode_switches: int = 0
    flags_used: int = 0

    @property
    def speedup_over(self):
        return lambda t_target: self.emitted * t_target / self.time


class _Flags:
    def __init__(self, accept: Sequence[int]):
        self.a, self.i = list(accept), 0

    def next(self) -> bool:
        ok = bool(self.a[self.i]) if self.i < len(self.a) else True
        self.i += 1
        return ok


def autoregressive(n_tokens: int, t_target: float) -> Timeline:
    tl = Timeline()
    for _ in range(n_tokens):
        tl.time += t_target
        tl.emitted += 1
        tl.target_calls += 1
        tl.rounds += 1
    return tl


def serial_sd(gamma: int, t_draft: float, t_target: float, accept: Sequence[int], n_tokens: int) -> Timeline:
    tl, fl = Timeline(), _Flags(accept)
    while tl.emitted < n_tokens:
        drafts = ["d"] * gamma
        tl.time += gamma * t_draft                 # the target waits for all gamma drafts ...
        tl.draft_tokens += gamma
        tl.time += t_target                        # ... and the draft model waits for the verdict
        tl.target_calls += 1
        kept = 0
        for _ in drafts:
            if not fl.next():
                break
            kept += 1
        tl.emitted += kept + 1                     # accepted drafts + the target's own token
        tl.draft_wasted += gamma - kept
        tl.rounds += 1
    tl.flags_used = fl.i
    return tl


def vpsd(gamma: int, t_draft: float, t_target: float, accept: Sequence[int], n_tokens: int,
         n_prefill_buffer: int = 0) -> Timeline:
    tl, fl = Timeline(), _Flags(accept)
    buffer: List[str] = ["b"] * n_prefill_buffer          # drafted, not yet verified
    tl.draft_tokens += n_prefill_buffer
    optimistic = n_prefill_buffer > 0
    now = 0.0
    while tl.emitted < n_tokens:
        tl.rounds += 1
        if optimistic:
            to_verify, ahead = list(buffer), gamma
            start = now
        else:
            assert not buffer
            now += t_draft                                # x_1 first
            tl.draft_tokens += 1
            to_verify, ahead = ["x1"], gamma - 1
            start = now
        verdict_at = start + t_target
        tl.target_calls += 1
        kept = 0
        for _ in to_verify:
            if not fl.next():
                break
            kept += 1
        if kept == len(to_verify):
            drafted_at = start + ahead * t_draft
            now = max(verdict_at, drafted_at)
            tl.draft_tokens += ahead
            tl.emitted += kept
            buffer = ["n"] * ahead
            new_mode = ahead > 0
        else:
            done = min(ahead, int((t_target / t_draft) * (1 + 1e-12)))   # drafts finished before the verdict
            tl.draft_tokens += done
            tl.draft_wasted += (len(to_verify) - kept) + done
            now = verdict_at
            tl.emitted += kept + 1                         # the target's replacement token
            buffer = []
            new_mode = False
        if new_mode != optimistic:
            tl.mode_switches += 1
            optimistic = new_mode
    tl.draft_wasted += len(buffer)
    tl.time = now
    tl.flags_used = fl.i
    return tl
