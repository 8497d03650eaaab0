// Edge-side scheduling of a speculative round: host code only (no kernel, no HIP call).
//
// Token batching (Sec. 3.2): N draft tokens leave the edge in K batches; batch k starts at token
// b_k.  Generating a token takes gamma, sending a batch of n tokens alpha + beta n; a batch is
// sent once it has been generated and the link has finished the batch before it.  The time of a
// batching is Eq. (6); the best batching comes from the dynamic programme of Sec. 4.1 (Theorem 1).
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

// done[j]: earliest time the link can have delivered tokens 1..j; the last batch {i+1..j} starts
// when tokens 1..i are delivered and token j exists.  Ties keep the smallest i (the longest last
// batch), so the batching returned is the one with the fewest, latest boundaries among the best.
extern "C" int pipesd_batching_optimal(int32_t n_tokens, double alpha, double beta, double gamma, int32_t* first_out,
                                       int32_t* n_batches_out, double* time_out) {
  if (!first_out || !n_batches_out || !time_out || n_tokens < 1 || n_tokens > kMaxScheduleTokens) return PIPESD_EINVAL;
  if (!cost_ok(alpha) || !cost_ok(beta) || !cost_ok(gamma)) return PIPESD_EINVAL;
  std::vector<double> done;
  std::vector<int32_t> cut;
  try {
    done.assign((size_t)n_tokens + 1, 0.0);
    cut.assign((size_t)n_tokens + 1, 0);
  } catch (const std::bad_alloc&) {
    return PIPESD_ENOMEM;
  }
  for (int32_t j = 1; j <= n_tokens; ++j) {
    const double ready = gamma * (double)j;
    double best = INFINITY;
    int32_t arg = 0;
    for (int32_t i = 0; i < j; ++i) {
      const double start = done[i] > ready ? done[i] : ready;
      const double t = start + (alpha + beta * (double)(j - i));
      if (t < best) {
        best = t;
        arg = i;
      }
    }
    done[j] = best;
    cut[j] = arg;
  }
  int32_t n_batches = 0;
  for (int32_t p = n_tokens; p > 0; p = cut[p]) ++n_batches;
  int32_t k = n_batches;
  for (int32_t p = n_tokens; p > 0; p = cut[p]) first_out[--k] = cut[p] + 1;
  *n_batches_out = n_batches;
  *time_out = done[n_tokens];
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
