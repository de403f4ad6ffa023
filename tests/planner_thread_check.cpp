// Thread-sanitizer driver for the background planner: many submissions racing with polls, then
// destruction with a job in flight.  Built and run by test_host_sanitizers.py (host code only).
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_2601_10729_amd/csrc/orbit_async_planner.hpp"

using namespace orbit;

int main() {
  const int L = 16;
  std::vector<double> comp(L, 1.0);
  int64_t collected = 0, last_ticket = 0;
  {
    AsyncPlanner p;
    for (int it = 0; it < 200; ++it) {
      PlanJob j;
      j.n_req = 3;
      j.L = L;
      j.slots = 1 + it % 2;
      j.blocks = {4 + it % 5, 9, 2 + it % 3};
      j.gpu_blocks = 15 * L * (it % 4 + 1) / 4;
      j.max_evals = 2000;
      j.bandwidth = 2.0;
      j.comp = comp;
      const int64_t t = p.submit(std::move(j));
      if (t <= last_ticket) { std::printf("tickets must grow\n"); return 1; }
      last_ticket = t;
      PlanDone d;
      if (p.poll(it % 7 == 0, d)) {
        if (d.ticket > t || d.n_req != 3) { std::printf("bad result\n"); return 1; }
        ++collected;
      }
    }
    PlanDone d;
    if (p.poll(true, d)) {
      if (d.ticket != last_ticket) { std::printf("waiting must deliver the newest job\n"); return 1; }
      ++collected;
    }
    PlanJob j;
    j.n_req = 5;
    j.L = 32;
    j.blocks = {7, 14, 21, 28, 35};
    j.gpu_blocks = 2000;
    j.max_evals = 200000;
    j.bandwidth = 2.0;
    j.comp.assign(32, 1.0);
    p.submit(std::move(j));  // destroyed while this one runs
  }
  std::printf("planner threads ok, %lld plans collected\n", (long long)collected);
  return collected > 0 ? 0 : 1;
}
