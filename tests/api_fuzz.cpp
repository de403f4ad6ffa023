// Randomised driver of the C ABI in ORBIT_FLAG_HOST_ONLY mode (no GPU call is made): plan
// switches, pauses, drops, steps and per-layer calls in legal and illegal orders.  Built with the
// host half of the library under AddressSanitizer + UndefinedBehaviorSanitizer by
// test_host_sanitizers.py.  Checks: only documented error codes come back, a failed call changes
// no length, lengths follow a model kept here, Eq. (1) holds after every successful plan.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <vector>

#include "../include/orbit.h"

#define CHECK(x)                                                                   \
  do {                                                                             \
    if (!(x)) {                                                                    \
      std::printf("CHECK failed at line %d: %s (last error: %s)\n", __LINE__, #x, orbit_last_error(ctx)); \
      return 1;                                                                    \
    }                                                                              \
  } while (0)

int main(int argc, char **argv) {
  const unsigned seed = argc > 1 ? (unsigned)std::atoi(argv[1]) : 1u;
  const int rounds = argc > 2 ? std::atoi(argv[2]) : 400;
  std::mt19937 rng(seed);
  auto rnd = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
  const int L = rnd(1, 5), window = rnd(1, 6), max_req = 6;
  const int64_t page = 2 * 8 * 16 * 128 * 2;
  orbit_config cfg{};
  cfg.n_layers = L;
  cfg.n_q_heads = 32;
  cfg.n_kv_heads = 8;
  cfg.head_dim = 128;
  cfg.page_tokens = 16;
  cfg.max_requests = max_req;
  cfg.max_tokens_per_request = 2048;
  cfg.prefetch_slots = rnd(1, 3);
  cfg.chunk_tokens = 32 * rnd(1, 16);
  cfg.decode_window = window;
  cfg.flags = ORBIT_FLAG_HOST_ONLY | (rnd(0, 2) == 0 ? ORBIT_FLAG_ZERO_COPY : 0);
  cfg.hbm_arena_bytes = 3000 * page;
  cfg.host_arena_bytes = 12000 * page;
  orbit_ctx *ctx = nullptr;
  CHECK(orbit_create(&cfg, &ctx) == ORBIT_OK);

  std::vector<int64_t> order;           // active ids in plan order
  std::map<int64_t, int> len, paused;   // id -> stored tokens (all layers equal between steps)
  std::map<int64_t, int> cap;           // id -> tokens that fit the blocks reserved by the current plan
  int64_t next_id = 1;
  int n_steps = 0, n_plans = 0;
  auto room = [&]() {  // a step is legal while every request still has a reserved slot for one more token
    for (int64_t id : order)
      if (len[id] >= cap[id]) return false;
    return true;
  };
  auto reserve = [&]() {
    cap.clear();
    for (int64_t id : order) cap[id] = (len[id] + window + 15) / 16 * 16;
  };
  const int bpr = (L + 7) / 8;

  auto lengths_match = [&]() -> bool {
    for (int64_t id : order)
      for (int l = 0; l < L; ++l) {
        int32_t n = -1, tier = -1;
        if (orbit_get_pages(ctx, id, l, &tier, nullptr, &n, nullptr, 0) < 0 || n != len[id] || tier < 0 || tier > 2) return false;
      }
    return true;
  };

  for (int it = 0; it < rounds; ++it) {
    const int op = order.empty() ? 0 : rnd(0, 9);
    if (op <= 1) {  // new plan
      std::vector<int64_t> ids;
      for (int64_t id : order)
        if (rnd(0, 4) != 0) ids.push_back(id);
      for (auto &kv : paused)
        if (rnd(0, 1) && (int)ids.size() < max_req) ids.push_back(kv.first);
      std::vector<int64_t> fresh;
      while ((int)ids.size() < max_req && (rnd(0, 1) || ids.empty())) {
        ids.push_back(next_id);
        fresh.push_back(next_id++);
      }
      std::vector<int32_t> n;
      for (int64_t id : ids) {
        if (len.count(id)) n.push_back(len[id]);
        else if (paused.count(id)) n.push_back(paused[id]);
        else n.push_back(rnd(0, 900));
      }
      std::vector<uint8_t> bm(ids.size() * bpr);
      for (auto &b : bm) b = (uint8_t)rnd(0, 255);
      int64_t out4[4];
      CHECK(orbit_plan_check((int)ids.size(), L, 16, n.data(), bm.data(), (cfg.flags & ORBIT_FLAG_ZERO_COPY) ? 0 : cfg.prefetch_slots,
                             window, out4) == ORBIT_OK);
      const int64_t budget = std::max<int64_t>(0, out4[2] + rnd(-30, 100));
      const int rc = orbit_plan_load(ctx, (int)ids.size(), ids.data(), n.data(), bm.data(), budget * page);
      if (rc != ORBIT_OK) {
        CHECK(rc == ORBIT_E_CAPACITY || rc == ORBIT_E_HOST_CAPACITY);
        CHECK(budget < out4[2] || budget > 3000 || rc == ORBIT_E_HOST_CAPACITY);
        CHECK(lengths_match());
      } else {
        for (int64_t id : order) {
          bool kept = false;
          for (int64_t k : ids) kept |= k == id;
          if (!kept) len.erase(id);
        }
        for (size_t i = 0; i < ids.size(); ++i) {
          paused.erase(ids[i]);
          len[ids[i]] = n[i];
        }
        order = ids;
        reserve();
        ++n_plans;
        orbit_plan_info info;
        CHECK(orbit_get_plan_info(ctx, &info) == ORBIT_OK);
        CHECK(info.resident_blocks + info.staging_blocks <= info.budget_blocks && info.n_requests == (int)ids.size());
        CHECK(info.in_place_blocks >= 0 && info.in_place_blocks <= info.moved_to_host_blocks);
        CHECK(info.deferred_to_host_blocks >= 0 &&
              info.deferred_to_host_blocks <= info.moved_to_host_blocks + info.evicted_blocks);
        CHECK(lengths_match());
      }
    } else if (op <= 4) {  // whole step
      const int rc = orbit_step(ctx, nullptr, nullptr, nullptr, nullptr, nullptr);
      if (room()) {
        CHECK(rc == ORBIT_OK);
        for (int64_t id : order) ++len[id];
        ++n_steps;
      } else {
        CHECK(rc == ORBIT_E_STATE);
      }
      CHECK(lengths_match());
    } else if (op <= 6) {  // the same through the per-layer calls, prefetches at random points
      if (!room()) {
        CHECK(orbit_kv_append_batch(ctx, rnd(0, L - 1), nullptr, nullptr) == ORBIT_E_STATE);
        CHECK(lengths_match());
        continue;
      }
      for (int l = 0; l < L; ++l) {
        if (rnd(0, 1)) {
          const int rc = orbit_kv_prefetch(ctx, rnd(l, L - 1));
          CHECK(rc == ORBIT_OK || rc == ORBIT_E_STATE);  // E_STATE: range still needed by a prefetched layer
        }
        if (rnd(0, 2) == 0) {  // append and attention in one call; refused (nothing changed) if its staging range is taken
          const int rc = orbit_decode_layer(ctx, l, nullptr, nullptr, nullptr, nullptr, nullptr);
          CHECK(rc == ORBIT_OK || rc == ORBIT_E_STATE);
          if (rc == ORBIT_OK) continue;
        }
        if (rnd(0, 1)) {
          CHECK(orbit_kv_append_batch(ctx, l, nullptr, nullptr) == ORBIT_OK);
        } else {
          int dummy = 0;  // host-only mode never reads k and v; any non-NULL pointer passes the check
          for (int64_t id : order) CHECK(orbit_kv_append(ctx, id, l, &dummy, &dummy) == ORBIT_OK);
        }
        const int rc = orbit_decode_attention(ctx, l, nullptr, nullptr, nullptr);
        // E_STATE: a later layer was prefetched into the range this layer needs and has not been attended
        CHECK(rc == ORBIT_OK || rc == ORBIT_E_STATE);
      }
      for (int64_t id : order) ++len[id];
      ++n_steps;
      CHECK(lengths_match());
      // leave no prefetched layer unattended: attend every layer once more, in order, until none blocks
      for (int pass = 0; pass < L + 1; ++pass)
        for (int l = 0; l < L; ++l) (void)orbit_decode_attention(ctx, l, nullptr, nullptr, nullptr);
    } else if (op == 7 && order.size() > 1) {
      const int64_t id = order[rnd(0, (int)order.size() - 1)];
      const int rc = orbit_request_pause(ctx, id);
      if (rc == ORBIT_OK) {
        paused[id] = len[id];
        len.erase(id);
        for (size_t i = 0; i < order.size(); ++i)
          if (order[i] == id) { order.erase(order.begin() + i); break; }
        reserve();
      } else {
        CHECK(rc == ORBIT_E_STATE || rc == ORBIT_E_CAPACITY || rc == ORBIT_E_HOST_CAPACITY);
      }
      CHECK(lengths_match());
    } else if (op == 8 && !paused.empty()) {
      const int64_t id = paused.begin()->first;
      CHECK(orbit_request_drop(ctx, id) == ORBIT_OK);
      paused.erase(id);
      CHECK(orbit_request_drop(ctx, id) == ORBIT_E_NOT_FOUND);
    } else {  // calls that must fail cleanly
      CHECK(orbit_kv_prefetch(ctx, L) == ORBIT_E_INVAL);
      CHECK(orbit_decode_attention(ctx, -1, nullptr, nullptr, nullptr) == ORBIT_E_INVAL);
      int dummy = 0;
      CHECK(orbit_kv_append(ctx, 987654321, 0, &dummy, &dummy) == ORBIT_E_NOT_FOUND);
      CHECK(orbit_request_pause(ctx, 987654321) == ORBIT_E_NOT_FOUND);
      CHECK(orbit_decode_attention_static(ctx, 0, &dummy, &dummy, nullptr) < 0);   // a host-only context has no scratch
      {  // SLO replay on a random run: the deposit never adds violations, counts stay within the run
        double steps[24];
        const int ns = rnd(0, 24);
        for (int i = 0; i < ns; ++i) steps[i] = rnd(0, 50) / 10.0;
        orbit_slo_report rep;
        CHECK(orbit_slo_replay(steps, ns, 0.1 * rnd(1, 40), rnd(0, 1), &rep) == ORBIT_OK);
        CHECK(rep.tokens == ns && rep.visible_violations <= rep.backend_violations && rep.backend_violations <= ns);
        CHECK(rep.max_deposit >= 0 && rep.max_deposit <= ns);
        CHECK(orbit_slo_replay(steps, ns, 0.0, 0, &rep) == ORBIT_E_INVAL);
        CHECK(orbit_slo_replay(nullptr, 3, 1.0, 0, &rep) == ORBIT_E_INVAL);
      }
      CHECK(lengths_match());
    }
  }
  CHECK(orbit_destroy(ctx) == ORBIT_OK);
  std::printf("api fuzz ok: %d plans, %d steps\n", n_plans, n_steps);
  return n_plans > 2 ? 0 : 1;
}
