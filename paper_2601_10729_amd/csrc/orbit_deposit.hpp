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

// |predicted - observed| > fraction * predicted  (Section 3.4, profile-mismatch trigger)
inline bool profile_mismatch(double predicted, double observed, double fraction) {
  return std::fabs(predicted - observed) > fraction * predicted;
}
// exponentially weighted moving average refresh of a profile: p <- (1 - w) p + w observed
inline void profile_ewma(double *profile, const double *observed, int64_t n, double weight) {
  for (int64_t i = 0; i < n; ++i) profile[i] = (1.0 - weight) * profile[i] + weight * observed[i];
}

}  // namespace orbit
