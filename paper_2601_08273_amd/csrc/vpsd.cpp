// Host-side control logic of video parallel speculative decoding (paper: Method, "Video Parallel
// Speculative Decoding": synchronous draft-target prefill and adaptive decoding strategy
// switching).  No device code: a small state machine that tells a serving loop what to enqueue on
// the draft and the target stream in each round and how to account for the verification outcome,
// plus a timing model of it (and of serial speculative decoding and plain autoregressive decoding,
// the paper's motivation example) for capacity planning and tests.
#include <math.h>
#include <string.h>

#include "hippo.h"

namespace {

inline void count_switch(hippo_vpsd_state* s, int new_mode) {
  if (s->mode != new_mode) {
    s->mode = new_mode;
    s->n_mode_switches += 1;
  }
}

// outcome of verifying `len` draft tokens against the flag stream: number accepted; consumes one
// flag per token looked at (the rejected one included)
inline int verify_against_flags(const uint8_t* accept, int64_t n_flags, int64_t* cursor, int len) {
  int n = 0;
  while (n < len) {
    const bool ok = (*cursor < n_flags) ? accept[*cursor] != 0 : true;
    *cursor += 1;
    if (!ok) break;
    n += 1;
  }
  return n;
}

}  // namespace

extern "C" {

int32_t hippo_vpsd_prefill_buffer(double t_prefill_target, double t_prefill_draft, double t_draft_token) {
  if (!(t_draft_token > 0.0) || !(t_prefill_target >= 0.0) || !(t_prefill_draft >= 0.0)) return -1;
  const double slack = t_prefill_target - t_prefill_draft;
  if (slack <= 0.0) return 0;
  const double n = floor(slack / t_draft_token * (1.0 + 1e-12));   // 0.6 / 0.05 must count as 12
  return n > 1e9 ? 1000000000 : (int32_t)n;
}

int hippo_vpsd_init(hippo_vpsd_state* s, int32_t gamma, int32_t n_prefill_buffer) {
  if (s == nullptr) return HIPPO_ERR_NULL_ARG;
  if (gamma < 1 || gamma > 64 || n_prefill_buffer < 0 || n_prefill_buffer > 64) return HIPPO_ERR_BAD_SHAPE;
  memset(s, 0, sizeof(*s));
  s->gamma = gamma;
  s->n_pending = n_prefill_buffer;
  s->mode = n_prefill_buffer > 0 ? HIPPO_VPSD_OPTIMISTIC : HIPPO_VPSD_CONSERVATIVE;
  s->n_draft_tokens = n_prefill_buffer;
  return HIPPO_OK;
}

int hippo_vpsd_plan(const hippo_vpsd_state* s, hippo_vpsd_round* r) {
  if (s == nullptr || r == nullptr) return HIPPO_ERR_NULL_ARG;
  if (s->gamma < 1 || s->gamma > 64 || s->n_pending < 0 || s->n_pending > 64) return HIPPO_ERR_BAD_SHAPE;
  r->mode = s->mode;
  if (s->mode == HIPPO_VPSD_OPTIMISTIC) {
    if (s->n_pending < 1) return HIPPO_ERR_BAD_SHAPE;
    r->draft_serial = 0;
    r->verify_len = s->n_pending;          // the whole buffer goes to the target ...
    r->draft_parallel = s->gamma;          // ... while the draft model runs one batch ahead
  } else if (s->mode == HIPPO_VPSD_CONSERVATIVE) {
    if (s->n_pending != 0) return HIPPO_ERR_BAD_SHAPE;
    r->draft_serial = 1;                   // x_1 first,
    r->verify_len = 1;                     // verified alone ...
    r->draft_parallel = s->gamma - 1;      // ... while x_2..x_gamma are drafted
  } else {
    return HIPPO_ERR_BAD_SHAPE;
  }
  return HIPPO_OK;
}

int hippo_vpsd_commit(hippo_vpsd_state* s, const hippo_vpsd_round* r, int32_t n_accept, int32_t n_drafted_parallel) {
  if (s == nullptr || r == nullptr) return HIPPO_ERR_NULL_ARG;
  // every check comes before the first change of the state: a refused commit leaves it as it was.
  // The round must be the one hippo_vpsd_plan derives from this state, field by field.
  hippo_vpsd_round planned;
  const int rc = hippo_vpsd_plan(s, &planned);
  if (rc != HIPPO_OK) return rc;
  if (r->mode != planned.mode || r->draft_serial != planned.draft_serial || r->verify_len != planned.verify_len ||
      r->draft_parallel != planned.draft_parallel)
    return HIPPO_ERR_BAD_SHAPE;
  if (n_accept < 0 || n_accept > r->verify_len || n_drafted_parallel < 0 || n_drafted_parallel > r->draft_parallel)
    return HIPPO_ERR_BAD_SHAPE;
  const bool all_accepted = n_accept == r->verify_len;
  if (all_accepted && n_drafted_parallel != r->draft_parallel) return HIPPO_ERR_BAD_SHAPE;   // a kept batch must be whole
  s->n_rounds += 1;
  s->n_target_calls += 1;
  s->n_draft_tokens += r->draft_serial + n_drafted_parallel;
  if (all_accepted) {
    // everything verified was right: the tokens drafted meanwhile become the next buffer
    s->n_emitted += n_accept;
    s->n_pending = r->draft_parallel;
    if (s->n_pending > 0) count_switch(s, HIPPO_VPSD_OPTIMISTIC);
    else count_switch(s, HIPPO_VPSD_CONSERVATIVE);           // gamma = 1: nothing was drafted ahead
  } else {
    // a rejection: the accepted prefix plus the target's replacement token; every other draft dies
    s->n_emitted += n_accept + 1;
    s->n_draft_wasted += (r->verify_len - n_accept) + n_drafted_parallel;
    s->n_pending = 0;
    count_switch(s, HIPPO_VPSD_CONSERVATIVE);
  }
  return HIPPO_OK;
}

int hippo_vpsd_simulate(int32_t policy, int32_t gamma, double t_draft, double t_target, int32_t n_prefill_buffer,
                        const uint8_t* accept, int64_t n_flags, int64_t n_tokens, hippo_vpsd_result* out) {
  if (out == nullptr || (accept == nullptr && n_flags > 0)) return HIPPO_ERR_NULL_ARG;
  if (gamma < 1 || gamma > 64 || !(t_draft > 0.0) || !(t_target > 0.0) || n_tokens < 1 || n_flags < 0)
    return HIPPO_ERR_BAD_SHAPE;
  memset(out, 0, sizeof(*out));
  int64_t cursor = 0;
  double t = 0.0;
  if (policy == HIPPO_POLICY_AUTOREGRESSIVE) {
    out->n_emitted = n_tokens;
    out->n_target_calls = n_tokens;
    out->n_rounds = n_tokens;
    t = (double)n_tokens * t_target;
  } else if (policy == HIPPO_POLICY_SERIAL_SD) {
    // draft gamma tokens, then verify them; the target always contributes one token
    while (out->n_emitted < n_tokens) {
      const int n_acc = verify_against_flags(accept, n_flags, &cursor, gamma);
      t += gamma * t_draft + t_target;
      out->n_emitted += n_acc + 1;
      out->n_draft_tokens += gamma;
      out->n_draft_wasted += gamma - n_acc;
      out->n_target_calls += 1;
      out->n_rounds += 1;
    }
  } else if (policy == HIPPO_POLICY_VPSD) {
    hippo_vpsd_state s;
    int rc = hippo_vpsd_init(&s, gamma, n_prefill_buffer);
    if (rc != HIPPO_OK) return rc;
    while (s.n_emitted < n_tokens) {
      hippo_vpsd_round r;
      if ((rc = hippo_vpsd_plan(&s, &r)) != HIPPO_OK) return rc;
      const int n_acc = verify_against_flags(accept, n_flags, &cursor, r.verify_len);
      int drafted = r.draft_parallel;
      double dt = r.draft_serial * t_draft;
      if (n_acc == r.verify_len) {
        dt += fmax(t_target, r.draft_parallel * t_draft);      // both must finish
      } else {
        dt += t_target;                                        // drafting is cut when the verdict arrives
        const double could = floor(t_target / t_draft * (1.0 + 1e-12));
        if (could < drafted) drafted = (int)could;
      }
      t += dt;
      if ((rc = hippo_vpsd_commit(&s, &r, n_acc, drafted)) != HIPPO_OK) return rc;
    }
    out->n_emitted = s.n_emitted;
    out->n_rounds = s.n_rounds;
    out->n_target_calls = s.n_target_calls;
    out->n_draft_tokens = s.n_draft_tokens;
    out->n_draft_wasted = s.n_draft_wasted + s.n_pending;      // a buffer left over at the end is waste too
    out->n_mode_switches = s.n_mode_switches;
  } else {
    return HIPPO_ERR_BAD_SHAPE;
  }
  out->time = t;
  out->speedup = (double)out->n_emitted * t_target / t;
  out->n_flags_used = cursor;
  return HIPPO_OK;
}

}  // extern "C"
