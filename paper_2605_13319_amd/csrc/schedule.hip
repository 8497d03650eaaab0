// Edge-side scheduling of a speculative round: host code only (no kernel, no HIP call).
//
// Token batching (Sec. 3.2): N draft tokens leave the edge in K batches; batch k starts at token
// b_k.  Generating a token takes gamma, sending a batch of n tokens alpha + beta n; a batch is
// sent once it has been generated and the link has finished the batch before it.  The time of a
// batching is Eq. (6); the best batching is a shortest path over the link's states, optimal by the
// argument of Sec. 4.1 (Theorem 1).
// NAV trigger (Sec. 3.3): a round ends at the draft token whose confidence brings the running
// product to R1 or below, or is itself R2 or below.
#include <math.h>

#include <new>
#include <vector>

#include "../../include/pipesd.h"

namespace {

constexpr int32_t kMaxScheduleTokens = 1 << 14;  // the table walk is quadratic in the window

bool cost_ok(double v) { return v >= 0.0 && isfinite(v); }

}  // namespace

// Eqs. (2)-(6).  Generation never pauses (Eq. (4)), so the k-th batch is complete at gamma times
// the number of tokens up to its end; the link takes the batches in order (Eq. (5)).
extern "C" int pipesd_batching_time(int32_t n_tokens, const int32_t* first, int32_t n_batches, double alpha, double beta,
                                    double gamma, double* time_out) {
  if (!first || !time_out || n_tokens < 1 || n_batches < 1 || n_batches > n_tokens) return PIPESD_EINVAL;
  if (!cost_ok(alpha) || !cost_ok(beta) || !cost_ok(gamma)) return PIPESD_EINVAL;
  if (first[0] != 1 || first[n_batches - 1] > n_tokens) return PIPESD_EINVAL;
  for (int32_t k = 1; k < n_batches; ++k)
    if (first[k] <= first[k - 1]) return PIPESD_EINVAL;
  double link_free = 0.0;
  for (int32_t k = 0; k < n_batches; ++k) {
    const int32_t end = k + 1 < n_batches ? first[k + 1] - 1 : n_tokens;  // last token of the batch
    const double ready = gamma * (double)end;
    const double start = (k > 0 && link_free > ready) ? link_free : ready;
    link_free = start + (alpha + beta * (double)(end - first[k] + 1));
  }
  *time_out = link_free;  // tau_ag of the first batch is 0
  return PIPESD_OK;
}

// Shortest path over link states (the model of Sec. 3.2, Eqs. (1)-(6)).  State s = "tokens 1..s have
// been delivered", reached at time free_at[s] (state 0 at time 0).  From state s a batch of len
// tokens leads to state s + len: it can start when the link is free (free_at[s]) and its last token
// exists (gamma (s + len), generation never pausing), and occupies the link for alpha + beta len.
// The states are settled in increasing s (every edge goes forward), each one relaxing all the
// states it can reach; T of Eq. (6) for the best batching is free_at[N].  A later state only
// replaces a predecessor that is strictly better, and predecessors are visited in increasing s, so
// among equally good batchings the one whose last batch starts earliest (is longest) is kept, and so
// on towards the front.  Theorem 1's optimum is what the tests hold this to, by enumeration.
extern "C" int pipesd_batching_optimal(int32_t n_tokens, double alpha, double beta, double gamma, int32_t* first_out,
                                       int32_t* n_batches_out, double* time_out) {
  if (!first_out || !n_batches_out || !time_out || n_tokens < 1 || n_tokens > kMaxScheduleTokens) return PIPESD_EINVAL;
  if (!cost_ok(alpha) || !cost_ok(beta) || !cost_ok(gamma)) return PIPESD_EINVAL;
  std::vector<double> free_at;
  std::vector<int32_t> from;  // the state the best way into a state comes from
  try {
    free_at.assign((size_t)n_tokens + 1, INFINITY);
    from.assign((size_t)n_tokens + 1, 0);
  } catch (const std::bad_alloc&) {
    return PIPESD_ENOMEM;
  }
  free_at[0] = 0.0;
  for (int32_t s = 0; s < n_tokens; ++s) {
    const double link_free = free_at[s];  // final: every edge into s has been relaxed
    for (int32_t len = 1; s + len <= n_tokens; ++len) {
      const int32_t to = s + len;
      const double generated = gamma * (double)to;
      const double arrival = (link_free > generated ? link_free : generated) + (alpha + beta * (double)len);
      if (arrival < free_at[to]) {
        free_at[to] = arrival;
        from[to] = s;
      }
    }
  }
  int32_t n_batches = 0;
  for (int32_t s = n_tokens; s > 0; s = from[s]) ++n_batches;
  for (int32_t s = n_tokens, k = n_batches; s > 0; s = from[s]) first_out[--k] = from[s] + 1;
  *n_batches_out = n_batches;
  *time_out = free_at[n_tokens];
  return PIPESD_OK;
}

extern "C" int pipesd_trigger_rounds(const double* confidence, int64_t n, double r1, double r2, int32_t max_len,
                                     int32_t* lengths_out, int64_t lengths_cap, int64_t* n_rounds_out,
                                     int64_t* consumed_out) {
  if (n < 0 || (n > 0 && !confidence) || !n_rounds_out || !consumed_out || max_len < 1 || lengths_cap < 0 ||
      (lengths_cap > 0 && !lengths_out))
    return PIPESD_EINVAL;
  if (!(r1 >= 0.0 && r1 <= 1.0) || !(r2 >= 0.0 && r2 <= 1.0)) return PIPESD_EINVAL;
  for (int64_t i = 0; i < n; ++i)
    if (!(confidence[i] >= 0.0 && confidence[i] <= 1.0)) return PIPESD_EINVAL;
  int64_t rounds = 0, consumed = 0;
  double running = 1.0;  // product of the confidences drafted since the last NAV
  int32_t len = 0;
  for (int64_t i = 0; i < n; ++i) {
    const double p = confidence[i];
    running *= p;
    ++len;
    if (running <= r1 || p <= r2 || len >= max_len) {
      if (rounds == lengths_cap) break;  // no room to report this round: stop in front of it
      lengths_out[rounds++] = len;
      consumed = i + 1;
      running = 1.0;
      len = 0;
    }
  }
  *n_rounds_out = rounds;
  *consumed_out = consumed;
  return PIPESD_OK;
}
