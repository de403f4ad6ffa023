// Host-side cost model and pruned plan search (no GPU work).
//
//  * distance-driven candidates: a request offloads every N-th layer; the candidates are the
//    distinct values of floor(L/k), k = 2..L (Section 3.3.2, "Pruning the Search Space").
//  * latency model: the prefetch rules that Algorithm 1 models (Section 3.3.1, "Scheduling KV
//    Prefetching") run as an event-driven simulation: layers strictly in order, a layer starts
//    when its KV is present, one stream and at most one layer in flight per request, the next
//    fetch of a request starts once its previously fetched layer has been executed, active
//    streams share the link evenly and a finished stream's share is redistributed.  This
//    reproduces the stall totals 9 and 12 of the paper's example (Section 2.3), counted in
//    block-transfer units; the algorithm as printed gives 9 and 11.
//  * search: minimum modelled latency subject to Eq. (1); exhaustive over the pruned space when
//    it is small (9^4 = 6561 for L = 32 and four requests), coordinate descent otherwise.
#pragma once

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

namespace orbit {

inline std::vector<int> distance_counts(int L) {  // descending, e.g. 16 10 8 6 5 4 3 2 1 for L = 32
  std::vector<int> v;
  for (int k = 2; k <= L; ++k) v.push_back(L / k);
  std::sort(v.begin(), v.end(), [](int a, int b) { return a > b; });
  v.erase(std::unique(v.begin(), v.end()), v.end());
  return v;
}

// x[l] = 1 keeps layer l (0-based) on the GPU.  count 0 keeps all, count L offloads all; otherwise
// the largest distance N with floor(L/N) == count is used and 1-based layers l with l % N == 0 go.
inline bool distance_pattern(int L, int count, uint8_t *x) {
  for (int l = 0; l < L; ++l) x[l] = 1;
  if (count <= 0) return true;
  int n = 0;
  for (int k = 1; k <= L; ++k)
    if (L / k == count) n = k;
  if (n == 0) return false;
  for (int l = 1; l <= L; ++l)
    if (l % n == 0) x[l - 1] = 0;
  return true;
}

// T_batch; stall[l] (may be null) receives the stall time in front of layer l.
inline double simulate_prefetch(int n_req, int L, const uint8_t *x, const int64_t *b, double bandwidth,
                                const double *comp, double *stall_out) {
  std::vector<double> remaining(n_req, 0.0);
  std::vector<int> target(n_req, 0);
  std::vector<uint8_t> active(n_req, 0), was(n_req, 0);
  auto advance = [&](double limit, int need_layer) -> double {
    double passed = 0.0;
    for (;;) {
      int live = 0;
      bool needed = false;
      for (int r = 0; r < n_req; ++r)
        if (active[r]) {
          ++live;
          needed |= target[r] == need_layer;
        }
      if (limit < 0 && !needed) return passed;
      if (live == 0 || (limit >= 0 && passed >= limit)) return limit < 0 ? passed : limit;
      const double rate = bandwidth / live;
      double least = std::numeric_limits<double>::infinity();
      for (int r = 0; r < n_req; ++r)
        if (active[r]) least = std::min(least, remaining[r]);
      double dt = least / rate;
      if (limit >= 0 && passed + dt > limit) {
        dt = limit - passed;
        for (int r = 0; r < n_req; ++r)
          if (active[r]) remaining[r] -= rate * dt;
        return limit;
      }
      was = active;  // same size: no allocation
      for (int r = 0; r < n_req; ++r)
        if (was[r]) remaining[r] -= rate * dt;
      passed += dt;
      for (int r = 0; r < n_req; ++r)
        if (was[r] && remaining[r] <= 1e-12 * std::max(1.0, (double)b[r])) {
          remaining[r] = 0.0;
          active[r] = 0;
        }
    }
  };
  double total = 0.0;
  for (int layer = 1; layer <= L; ++layer) {
    for (int r = 0; r < n_req; ++r) {
      if (active[r] || target[r] >= layer) continue;
      for (int l = layer; l <= L; ++l)
        if (!x[(size_t)r * L + l - 1]) {
          target[r] = l;
          remaining[r] = (double)b[r];
          active[r] = remaining[r] > 0;
          break;
        }
    }
    const double stall = advance(-1.0, layer);
    if (stall_out) stall_out[layer - 1] = stall;
    advance(comp[layer - 1], layer);
    total += stall + comp[layer - 1];
    for (int r = 0; r < n_req; ++r)
      if (target[r] == layer && !active[r]) target[r] = 0;
  }
  return total;
}

struct SearchResult {
  double t = std::numeric_limits<double>::infinity();
  std::vector<uint8_t> x;  // [n_req][L]
  int64_t evals = 0;
  bool exhaustive = false;
};

inline bool eq1_fits(int n_req, int L, const uint8_t *x, const int64_t *b, int64_t gpu_blocks, int slots) {
  int64_t resident = 0, buffer = 0;
  for (int l = 0; l < L; ++l) {
    int64_t off = 0;
    for (int r = 0; r < n_req; ++r) {
      if (x[(size_t)r * L + l]) resident += b[r];
      else off += b[r];
    }
    buffer = std::max(buffer, off);
  }
  return resident + (int64_t)slots * buffer <= gpu_blocks;
}

// stagger: request r takes its pattern rotated right by r layers, so that requests do not all
// offload the same layers (an extension of the paper's space: same counts and distances, a
// smaller prefetch buffer and a smoother link load).
inline SearchResult plan_search(int n_req, int L, const int64_t *b, int64_t gpu_blocks, int slots, double bandwidth,
                                const double *comp, int64_t max_evals, bool stagger = false) {
  SearchResult res;
  std::vector<int> cands{0};
  {
    std::vector<int> d = distance_counts(L);
    std::sort(d.begin(), d.end());
    cands.insert(cands.end(), d.begin(), d.end());
    if (L > 1) cands.push_back(L);
  }
  const int nc = (int)cands.size();
  std::vector<std::vector<uint8_t>> pat(nc, std::vector<uint8_t>(L));
  for (int i = 0; i < nc; ++i) distance_pattern(L, cands[i], pat[i].data());
  std::vector<uint8_t> x((size_t)n_req * L);
  auto put = [&](std::vector<uint8_t> &dst, int r, int i) {  // row r <- candidate i, rotated if staggered
    const int shift = stagger ? r % L : 0;
    for (int l = 0; l < L; ++l) dst[(size_t)r * L + (l + shift) % L] = pat[i][l];
  };
  auto eval = [&](const std::vector<int> &choice) -> double {
    for (int r = 0; r < n_req; ++r) put(x, r, choice[r]);
    if (!eq1_fits(n_req, L, x.data(), b, gpu_blocks, slots)) return std::numeric_limits<double>::infinity();
    ++res.evals;
    return simulate_prefetch(n_req, L, x.data(), b, bandwidth, comp, nullptr);
  };
  auto keep = [&](const std::vector<int> &choice, double t) {
    res.t = t;
    res.x.assign((size_t)n_req * L, 1);
    for (int r = 0; r < n_req; ++r) put(res.x, r, choice[r]);
  };
  double space = 1.0;
  for (int r = 0; r < n_req; ++r) space *= nc;
  std::vector<int> choice(n_req, 0);
  if (n_req == 0) {
    res.t = 0;
    for (int l = 0; l < L; ++l) res.t += comp[l];
    res.exhaustive = true;
    return res;
  }
  if (space <= (double)max_evals) {
    res.exhaustive = true;
    for (;;) {  // odometer with request 0 as the most significant digit: lexicographic order
      const double t = eval(choice);
      if (t < res.t - 1e-12) keep(choice, t);
      int r = n_req - 1;
      while (r >= 0 && ++choice[r] == nc) choice[r--] = 0;
      if (r < 0) break;
    }
    return res;
  }
  // coordinate descent from the best uniform plan; it stops, keeping the best plan found, once
  // max_evals placements have been simulated (the uniform plans are always tried)
  int best_u = -1;
  for (int i = 0; i < nc; ++i) {
    std::fill(choice.begin(), choice.end(), i);
    const double t = eval(choice);
    if (t < res.t - 1e-12) {
      keep(choice, t);
      best_u = i;
    }
  }
  if (best_u < 0) return res;
  std::fill(choice.begin(), choice.end(), best_u);
  for (int sweep = 0; sweep < 8 && res.evals < max_evals; ++sweep) {
    bool improved = false;
    for (int r = 0; r < n_req && res.evals < max_evals; ++r) {
      const int cur = choice[r];
      int best_i = cur;
      for (int i = 0; i < nc && res.evals < max_evals; ++i) {
        if (i == cur) continue;
        choice[r] = i;
        const double t = eval(choice);
        if (t < res.t - 1e-12) {
          keep(choice, t);
          best_i = i;
          improved = true;
        }
      }
      choice[r] = best_i;
    }
    if (!improved) break;
  }
  return res;
}

// Pause-Resume fallback of Section 3.4 in its capacity form: while no placement of the remaining
// requests satisfies Eq. (1), the request with the largest sum of KV blocks and deposited tokens
// leaves the batch (ties: the later request), and the search runs again.  paused[r] = 1 marks the
// victims; res.x has one row per ORIGINAL request (rows of paused requests are all 1 and unused).
struct FallbackResult {
  SearchResult res;
  std::vector<uint8_t> paused;
  int n_paused = 0;
};

inline FallbackResult plan_search_or_pause(int n_req, int L, const int64_t *b, const int64_t *deposited, int64_t gpu_blocks,
                                           int slots, double bandwidth, const double *comp, int64_t max_evals, bool stagger) {
  FallbackResult out;
  out.paused.assign(n_req, 0);
  std::vector<int> keep(n_req);
  for (int r = 0; r < n_req; ++r) keep[r] = r;
  for (;;) {
    std::vector<int64_t> bk(keep.size());
    for (size_t i = 0; i < keep.size(); ++i) bk[i] = b[keep[i]];
    SearchResult sr = plan_search((int)keep.size(), L, bk.data(), gpu_blocks, slots, bandwidth, comp, max_evals, stagger);
    out.res.evals += sr.evals;
    if (sr.t < std::numeric_limits<double>::infinity()) {
      out.res.t = sr.t;
      out.res.exhaustive = sr.exhaustive;
      out.res.x.assign((size_t)n_req * L, 1);
      for (size_t i = 0; i < keep.size(); ++i)
        std::copy(sr.x.begin() + i * L, sr.x.begin() + (i + 1) * L, out.res.x.begin() + (size_t)keep[i] * L);
      return out;
    }
    // infeasible even with everything offloaded: pick the victim
    size_t v = 0;
    for (size_t i = 1; i < keep.size(); ++i)
      if (b[keep[i]] + deposited[keep[i]] >= b[keep[v]] + deposited[keep[v]]) v = i;
    out.paused[keep[v]] = 1;
    ++out.n_paused;
    keep.erase(keep.begin() + v);
  }
}

}  // namespace orbit
