// Token-Deposit (Section 3.2, "SLO-aware Token-Deposit") and the profile-mismatch trigger of the
// Adaptive Controller (Section 3.4), host only.
//
// Deposit rule: a generated token is appended to a CPU FIFO of 4-byte ids.  While the FIFO is
// non-empty exactly one token is delivered per SLO interval; when it is empty the next token is
// delivered as soon as it is generated (only then can a violation be seen by the user); once the
// request finishes everything left is delivered in one burst.
#pragma once

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <deque>

namespace orbit {

struct Deposit {
  double slo = 0.0;
  double last_delivery = -1.0;  // < 0: nothing delivered yet
  bool finished = false;
  double finish_time = 0.0;
  std::deque<int32_t> tok;
  std::deque<double> gen;
  int64_t delivered = 0, visible_violations = 0, max_size = 0;

  void push(int32_t token, double now) {
    tok.push_back(token);
    gen.push_back(now);
    max_size = std::max<int64_t>(max_size, (int64_t)tok.size());
  }
  // Time at which the head token is due (+inf if the FIFO is empty).
  double head_due() const {
    if (tok.empty()) return INFINITY;
    double due = last_delivery < 0 ? gen.front() : std::max(gen.front(), last_delivery + slo);
    if (finished) due = std::min(due, std::max(finish_time, gen.front()));
    return due;
  }
  // Pops the head if it is due by `now`; returns false otherwise.
  bool pop_due(double now, int32_t *token, double *when) {
    const double due = head_due();
    if (!(due <= now)) return false;
    if (last_delivery >= 0 && due - last_delivery > slo * (1.0 + 1e-12)) ++visible_violations;
    *token = tok.front();
    *when = due;
    tok.pop_front();
    gen.pop_front();
    last_delivery = due;
    ++delivered;
    return true;
  }
};

// SLO accounting of one request over a run of decode steps (Section 2.1 "SLO Metrics", Section 3.2):
// step k ends with one token; the clock starts at the delivery of the request's previous token with an
// empty deposit.  Runs the FIFO above over the implied generation times.
struct SloReport {
  int64_t tokens = 0, backend_violations = 0, visible_violations = 0, max_deposit = 0;
  double tpot = 0.0, max_visible_gap = 0.0;
  bool tpot_violated = false;
};
inline SloReport slo_replay(const double *step_latency, int64_t n, double slo, bool finish_at_end) {
  SloReport rep;
  rep.tokens = n;
  if (n <= 0) return rep;
  Deposit d;
  d.slo = slo;
  d.last_delivery = 0.0;  // the previous token went out at the clock's origin
  double now = 0.0, last_out = 0.0;
  auto drain = [&](double until) {
    int32_t tok;
    double when;
    while (!d.tok.empty() && d.pop_due(until, &tok, &when)) {
      rep.max_visible_gap = std::max(rep.max_visible_gap, when - last_out);
      last_out = when;
    }
  };
  for (int64_t k = 0; k < n; ++k) {
    if (step_latency[k] > slo * (1.0 + 1e-12)) ++rep.backend_violations;
    now += step_latency[k];
    d.push((int32_t)k, now);
    if (k == n - 1 && finish_at_end) {
      d.finished = true;
      d.finish_time = now;
    }
    if (k + 1 < n && step_latency[k + 1] == 0.0) continue;  // tokens of one instant are looked at together
    drain(now);  // whatever is due by this generation instant leaves first
    rep.max_deposit = std::max<int64_t>(rep.max_deposit, (int64_t)d.tok.size());
  }
  drain(INFINITY);
  rep.visible_violations = d.visible_violations;
  rep.tpot = now / (double)n;
  rep.tpot_violated = rep.tpot > slo * (1.0 + 1e-12);
  return rep;
}

// |predicted - observed| > fraction * predicted  (Section 3.4, profile-mismatch trigger)
inline bool profile_mismatch(double predicted, double observed, double fraction) {
  return std::fabs(predicted - observed) > fraction * predicted;
}
// exponentially weighted moving average refresh of a profile: p <- (1 - w) p + w observed
inline void profile_ewma(double *profile, const double *observed, int64_t n, double weight) {
  for (int64_t i = 0; i < n; ++i) profile[i] = (1.0 - weight) * profile[i] + weight * observed[i];
}

}  // namespace orbit
