// Randomised exercise of the HIP-free host logic (block tables, allocators, delta migration,
// pause / resume, work list, planner, deposit) meant to be built with
//   g++ -std=c++17 -O1 -g -fsanitize=address,undefined
// Every step re-checks the layout invariants; any violation aborts with a message.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>

#include "../paper_2601_10729_amd/csrc/orbit_deposit.hpp"
#include "../paper_2601_10729_amd/csrc/orbit_host.hpp"
#include "../paper_2601_10729_amd/csrc/orbit_planner.hpp"

using namespace orbit;

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "invariant failed: %s (line %d)\n", #cond, __LINE__); \
      std::abort();                                                        \
    }                                                                      \
  } while (0)

static void check_layout(const HostState &hs) {
  std::set<int32_t> seen, in_place;
  std::vector<std::pair<int64_t, int64_t>> runs;
  auto visit = [&](const Req &q, bool active) {
    for (int l = 0; l < hs.sh.L; ++l) {
      const LayerKV &lk = q.layers[l];
      CHECK(lk.tier == 0 || lk.tier == 1);
      if (lk.tier == 1) {
        for (int32_t p : lk.pages) {
          CHECK(p >= 0 && p < hs.arena_pages && hs.hbm.used[p]);
          CHECK(seen.insert(p).second);
          CHECK(p < hs.info.staging_first_page);
        }
        if (active) CHECK((int)lk.pages.size() == q.reserved);
      } else {
        CHECK(lk.host_page0 >= 0 && lk.host_page0 + lk.host_cap <= hs.host_pages);
        CHECK(lk.host_cap >= ceil_div(lk.len, hs.sh.P));
        runs.push_back({lk.host_page0, lk.host_page0 + lk.host_cap});
        if (active && !lk.dual_pages.empty()) {  // still read in place: the table row lists pages nobody owns any more
          const int32_t *row = &hs.h_table[((size_t)(&q - hs.reqs.data()) * hs.sh.L + l) * hs.sh.cap_pages];
          CHECK((int64_t)lk.dual_pages.size() >= ceil_div(lk.len, hs.sh.P));
          for (size_t i = 0; i < lk.dual_pages.size(); ++i) {
            CHECK(row[i] == lk.dual_pages[i] && row[i] >= 0 && row[i] < hs.info.staging_first_page);
            CHECK(!hs.hbm.used[row[i]] && in_place.insert(row[i]).second);
          }
        } else if (active && hs.sh.zero_copy) {
          CHECK(lk.stage_page0 < 0 && hs.info.staging_blocks == 0 && hs.blocks.empty());
          const int32_t *row = &hs.h_table[((size_t)(&q - hs.reqs.data()) * hs.sh.L + l) * hs.sh.cap_pages];
          for (int i = 0; i < q.reserved; ++i) CHECK(~row[i] == lk.host_page0 + i);   // in-place host page ids
        } else if (active) {
          CHECK(lk.stage_page0 >= hs.info.staging_first_page);
          CHECK(lk.stage_page0 + q.reserved <= hs.info.staging_first_page + hs.info.staging_blocks);
        }
      }
    }
  };
  for (auto &q : hs.reqs) visit(q, true);
  for (auto &q : hs.paused) visit(q, false);
  int64_t used = 0;
  for (uint8_t u : hs.hbm.used) used += u;
  CHECK(used == (int64_t)seen.size());
  std::sort(runs.begin(), runs.end());
  for (size_t i = 1; i < runs.size(); ++i) CHECK(runs[i - 1].second <= runs[i].first);
  int64_t run_pages = 0;
  for (auto &r : runs) run_pages += r.second - r.first;
  CHECK(run_pages + hs.host.total_free() == hs.host_pages);
  CHECK(hs.info.resident_blocks + hs.info.staging_blocks <= hs.info.budget_blocks);
}

// The deferred copies that no plan load has waited for yet, each with the block it carries.  A plan load that says it
// need not wait for them (needs_lazy_wait == false, or a layer it does not name in wait_layer) must leave them alone: an HBM page one of them reads stays with
// its block or with nobody and outside the staging region, a host page one of them writes stays with its block or
// with nobody, and none of the copies the plan load runs at once writes either kind of page or reads such a host page.
struct PendingCopy {
  int64_t src, dst, id;
  int layer;
};

static void check_pending(const HostState &hs, const std::vector<std::vector<PageOp>> &phases,
                          std::vector<PendingCopy> &pending) {
  if (hs.needs_lazy_wait) {  // the layers it waits for (a layer's copies have one event) are settled
    std::vector<PendingCopy> rest;
    for (auto &pc : pending)
      if (!hs.wait_layer[pc.layer]) rest.push_back(pc);
    pending.swap(rest);
  }
  std::vector<int> src_at((size_t)hs.arena_pages, -1), dst_at((size_t)hs.host_pages, -1);
  for (size_t i = 0; i < pending.size(); ++i) {
    src_at[pending[i].src] = (int)i;
    dst_at[pending[i].dst] = (int)i;
    CHECK(pending[i].src < hs.info.staging_first_page);
  }
  for (auto &ph : phases)
    for (auto &op : ph) {
      if (op.kind == OP_HOST_TO_HBM || op.kind == OP_HBM_TO_HBM) CHECK(src_at[op.dst] < 0);
      if (op.kind == OP_HBM_TO_HOST || op.kind == OP_HOST_TO_HOST) CHECK(dst_at[op.dst] < 0);
      if (op.kind == OP_HOST_TO_HBM || op.kind == OP_HOST_TO_HOST) CHECK(dst_at[op.src] < 0);
    }
  auto visit = [&](const Req &q) {
    for (int l = 0; l < hs.sh.L; ++l) {
      const LayerKV &lk = q.layers[l];
      if (lk.tier == 1)
        for (int32_t p : lk.pages)
          if (src_at[p] >= 0) CHECK(pending[src_at[p]].id == q.id && pending[src_at[p]].layer == l);
      if (lk.tier == 0)
        for (int64_t p = lk.host_page0; p < lk.host_page0 + lk.host_cap; ++p)
          if (dst_at[p] >= 0) CHECK(pending[dst_at[p]].id == q.id && pending[dst_at[p]].layer == l);
    }
  };
  for (auto &q : hs.reqs) visit(q);
  for (auto &q : hs.paused) visit(q);
  // this plan load's own deferred copies join the list, under the block whose host run they fill
  for (auto &op : hs.deferred) {
    CHECK(op.kind == OP_HBM_TO_HOST && dst_at[op.dst] < 0);
    PendingCopy pc{op.src, op.dst, -1, -1};
    auto owner = [&](const Req &q) {
      for (int l = 0; l < hs.sh.L; ++l) {
        const LayerKV &lk = q.layers[l];
        if (lk.tier == 0 && op.dst >= lk.host_page0 && op.dst < lk.host_page0 + lk.host_cap) { pc.id = q.id; pc.layer = l; }
      }
    };
    for (auto &q : hs.reqs) owner(q);
    for (auto &q : hs.paused) owner(q);
    CHECK(pc.id >= 0);
    pending.push_back(pc);
  }
}

// Where every block's tokens are: a tag (request, layer, block index) per HBM page and per host page, moved by the
// copies a plan load asks for (the deferred ones after the others, as late as they may run), set where a step writes
// a token and where a new request's KV is filled in.  Whatever an active or paused block would be read from must
// carry the block's own tags; a block read in place must carry them in both of its homes.
struct Tag {
  int64_t id = -1;
  int l = -1, i = -1;
  bool is(int64_t id_, int l_, int i_) const { return id == id_ && l == l_ && i == i_; }
};

struct ContentModel {
  std::vector<Tag> hbm, host;
  std::set<int64_t> known;
  void run(const PageOp &op) {
    const Tag t = (op.kind == OP_HBM_TO_HOST || op.kind == OP_HBM_TO_HBM) ? hbm[op.src] : host[op.src];
    ((op.kind == OP_HOST_TO_HBM || op.kind == OP_HBM_TO_HBM) ? hbm[op.dst] : host[op.dst]) = t;
  }
  void after_plan(const HostState &hs, const std::vector<std::vector<PageOp>> &phases) {
    for (auto &ph : phases)
      for (auto &op : ph) run(op);
    for (auto &op : hs.deferred) run(op);
    for (auto &q : hs.reqs)
      if (known.insert(q.id).second)  // a new request: the caller fills its KV in
        for (int l = 0; l < hs.sh.L; ++l)
          for (int i = 0; i < (int)ceil_div(q.layers[l].len, hs.sh.P); ++i) write(q, l, i);
  }
  void write(const Req &q, int l, int i) {
    const LayerKV &lk = q.layers[l];
    const Tag t{q.id, l, i};
    if (lk.tier == 1) hbm[lk.pages[i]] = t;
    else host[lk.host_page0 + i] = t;
    if (!lk.dual_pages.empty()) {
      CHECK(i < (int)lk.dual_pages.size());
      hbm[lk.dual_pages[i]] = t;
    }
  }
  void check(const HostState &hs) const {
    auto visit = [&](const Req &q) {
      for (int l = 0; l < hs.sh.L; ++l) {
        const LayerKV &lk = q.layers[l];
        for (int i = 0; i < (int)ceil_div(lk.len, hs.sh.P); ++i) {
          if (lk.tier == 1) CHECK(hbm[lk.pages[i]].is(q.id, l, i));
          else CHECK(host[lk.host_page0 + i].is(q.id, l, i));
          if (!lk.dual_pages.empty()) CHECK(hbm[lk.dual_pages[i]].is(q.id, l, i));
        }
      }
    };
    for (auto &q : hs.reqs) visit(q);
    for (auto &q : hs.paused) visit(q);
  }
};

int main(int argc, char **argv) {
  const unsigned seed = argc > 1 ? (unsigned)std::atoi(argv[1]) : 1u;
  const int rounds = argc > 2 ? std::atoi(argv[2]) : 300;
  std::mt19937 rng(seed);
  auto rnd = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
  Shape sh;
  sh.L = rnd(1, 6);
  sh.Hq = 32;
  sh.Hkv = 8;
  sh.G = 4;
  sh.D = 128;
  sh.P = 16;
  sh.max_req = 8;
  sh.max_tokens = 4096;
  sh.page_bytes = 65536;
  sh.cap_pages = 256;
  sh.chunk_tokens = 64 * rnd(1, 8);
  sh.window = rnd(0, 40);
  sh.slots = rnd(1, 3);
  sh.zero_copy = rnd(0, 3) == 0;
  HostState hs;
  const int arena_pages = rnd(0, 2) ? 3000 : rnd(600, 3000), host_pages = rnd(0, 2) ? 3000 : rnd(400, 3000);  // sometimes tight
  hs.init(sh, arena_pages, host_pages);
  std::vector<int64_t> known_ids;
  std::vector<int32_t> known_len;
  int ok = 0, rejected = 0, not_waited = 0;
  std::vector<PendingCopy> pending;
  ContentModel content;
  content.hbm.resize(arena_pages);
  content.host.resize(host_pages);
  int kept_in_place = 0;
  for (int it = 0; it < rounds; ++it) {
    const int action = rnd(0, 9);
    std::vector<std::vector<PageOp>> phases;
    if (action <= 5 || !hs.has_plan) {  // new plan: keep some, add some, resume some
      std::vector<int64_t> ids;
      std::vector<int32_t> lens;
      for (auto &q : hs.reqs)
        if (rnd(0, 3)) { ids.push_back(q.id); lens.push_back(q.layers[0].len); }
      for (auto &q : hs.paused)
        if (rnd(0, 2) == 0 && (int)ids.size() < sh.max_req) { ids.push_back(q.id); lens.push_back(q.layers[0].len); }
      while ((int)ids.size() < sh.max_req && rnd(0, 2) == 0) {
        ids.push_back(1000 + it * 10 + (int64_t)ids.size());
        lens.push_back(rnd(0, 1500));
      }
      const int n = (int)ids.size(), bpr = (sh.L + 7) / 8;
      std::vector<uint8_t> bm((size_t)n * bpr);
      for (auto &b : bm) b = (uint8_t)rng();
      const int64_t budget = (int64_t)rnd(200, 3200) * sh.page_bytes;
      int rc = hs.plan_load(n, ids.data(), lens.data(), bm.data(), budget, phases);
      rc == 0 ? ++ok : ++rejected;
      for (auto &ph : phases)
        for (auto &op : ph) CHECK(op.src >= 0 && op.dst >= 0);
      if (rc == 0) {
        not_waited += !pending.empty() && !hs.needs_lazy_wait;
        check_pending(hs, phases, pending);
        content.after_plan(hs, phases);
        kept_in_place += hs.info.still_in_place_blocks > 0;
      }
    } else if (action <= 7 && !hs.reqs.empty()) {  // pause one
      int rc = hs.pause(hs.reqs[rnd(0, (int)hs.reqs.size() - 1)].id, phases);
      rc == 0 ? ++ok : ++rejected;
      if (rc == 0) {
        not_waited += !pending.empty() && !hs.needs_lazy_wait;
        check_pending(hs, phases, pending);
        content.after_plan(hs, phases);
        kept_in_place += hs.info.still_in_place_blocks > 0;
      }
    } else if (action == 8 && !hs.paused.empty()) {
      CHECK(hs.drop_paused(hs.paused[rnd(0, (int)hs.paused.size() - 1)].id) == 0);
    } else if (!hs.reqs.empty()) {  // append one token everywhere when the window allows it
      bool room = true;
      for (auto &q : hs.reqs) room &= q.layers[0].len / sh.P < q.reserved;
      if (room) {
        // what the step path does for blocks still read in place: hand a layer over when a block would outgrow the
        // pages it has left (and, here, now and then as if its copies had landed)
        std::vector<int> flipped;
        for (int l = 0; l < sh.L && hs.has_plan; ++l) {
          bool must = rnd(0, 3) == 0;
          for (auto &q : hs.reqs) {
            const LayerKV &lk = q.layers[l];
            must |= !lk.dual_pages.empty() && ceil_div((int64_t)lk.len + 1, sh.P) > (int64_t)lk.dual_pages.size();
          }
          if (must && hs.dual_in_layer[l]) hs.flip_layer(l, flipped);
        }
        for (auto &q : hs.reqs)
          for (int l = 0; l < sh.L; ++l) {
            content.write(q, l, q.layers[l].len / sh.P);
            q.layers[l].len += 1;
          }
      }
    }
    if (hs.has_plan) {
      check_layout(hs);
      content.check(hs);
      std::vector<int32_t> items;
      bool all_nonempty = !hs.reqs.empty();
      for (auto &q : hs.reqs) all_nonempty &= q.layers[0].len > 0;
      if (all_nonempty) {
        CHECK(hs.build_work_items(0, items) == 0);
        CHECK((int64_t)items.size() / 4 <= hs.max_segments());
        std::vector<int64_t> covered(hs.reqs.size(), 0);
        for (size_t i = 0; i < items.size(); i += 4) {
          CHECK(items[i] >= 0 && items[i] < (int)hs.reqs.size());
          CHECK(items[i + 1] == covered[items[i]] && items[i + 1] % 32 == 0 && items[i + 2] >= 1);
          CHECK(items[i + 2] == sh.chunk_tokens);
          CHECK(items[i + 3] >= 0 && items[i + 3] < hs.work_workers && hs.work_order[items[i + 3]] == (int)(i / 4));
          covered[items[i]] += std::min<int64_t>(items[i + 2], hs.reqs[items[i]].layers[0].len - items[i + 1]);
        }
        for (size_t r = 0; r < hs.reqs.size(); ++r) CHECK(covered[r] == hs.reqs[r].layers[0].len);
      }
    }
  }
  // planner and deposit under the sanitizers
  std::vector<int64_t> b = {30, 70, 110};
  std::vector<double> comp(8, 1.0);
  SearchResult sr = plan_search(3, 8, b.data(), 1200, 2, 5.0, comp.data(), 5000);
  CHECK(sr.t >= 8.0 && sr.x.size() == 24);
  Deposit d;
  d.slo = 1.0;
  double t = 0;
  int32_t tok;
  double when;
  for (int i = 0; i < 200; ++i) {
    t += (rng() % 300) / 100.0;
    d.push(i, t);
    while (d.pop_due(t, &tok, &when)) CHECK(when <= t);
  }
  std::printf("host fuzz ok: seed %u, %d plan changes accepted, %d rejected, %d ran beside earlier deferred copies, %d kept blocks read in place\n",
              seed, ok, rejected, not_waited, kept_in_place);
  return 0;
}
