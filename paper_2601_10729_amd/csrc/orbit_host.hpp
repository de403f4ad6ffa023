// Host-side state of liborbit: block tables, allocators, Eq. (1), the staging-region schedule
// and the split-K work list.  Pure integer logic, no HIP calls: it is also what runs under
// ORBIT_FLAG_HOST_ONLY.
//
// Paper anchors: block counts b_r and the 16-token growth rule (Section 2.3); placement matrix
// x[r,l], Eq. (1) and the prefetch buffer B_buf (Section 3.3.1, "GPU Capacity Bound"); delta
// migration and the contiguous staging range (Section 3.2, "KV Manager"); one arena indexed by
// a (request x layer) table (Section 4).
#pragma once

#include <algorithm>
#include <cstdint>
#include <map>
#include <string>
#include <unordered_map>
#include <utility>
#include <vector>

#include "../../include/orbit.h"

namespace orbit {

struct Shape {
  int L = 0, Hq = 0, Hkv = 0, D = 0, P = 0, G = 0;
  int max_req = 0;
  int64_t max_tokens = 0;
  int64_t page_bytes = 0;
  int cap_pages = 0;    // page-table row length (even)
  int chunk_tokens = 0; // tokens per attention work segment; 0 = chosen per launch
  int window = 0;       // decode window (tokens)
  int slots = 1;        // staging region = slots * B_buf
  bool zero_copy = false;  // offloaded blocks are read in place: no staging region at all
};

enum PageOpKind { OP_HBM_TO_HOST = 0, OP_HOST_TO_HBM = 1, OP_HBM_TO_HBM = 2, OP_HOST_TO_HOST = 3 };
struct PageOp {
  int kind;
  int64_t src, dst;  // page index in the HBM arena or in the host arena, by kind
};
// One (request, layer) block that leaves HBM in a plan load (phase `phase`): its first n pages are copied to
// the host run starting at host_run.
struct DemoteGroup {
  int phase, layer;
  size_t n;
  int req;                         // index in the new batch, or -1 for a paused request's eviction
  int64_t host_run;
  std::vector<int32_t> old_pages;  // the block list it had in HBM (used and reserved pages)
};

struct LayerKV {
  uint8_t tier = 1;            // 1 = HBM, 0 = host
  int32_t len = 0;             // tokens stored
  std::vector<int32_t> pages;  // arena page ids (tier 1), `reserved` of them
  int64_t host_page0 = -1;     // first page of the host run (tier 0)
  int32_t host_cap = 0;        // pages in the host run
  int32_t stage_page0 = -1;    // first staging page (tier 0)
  // Non-empty while a block that the last plan load demoted is still on its way to the host: the HBM
  // pages it had (no longer owned, but untouched until a later plan load hands them out) are read in place.
  std::vector<int32_t> dual_pages;
};

struct Req {
  int64_t id = 0;
  int32_t reserved = 0;  // blocks per layer under the current plan: ceil((ctx_len + window) / P)
  std::vector<LayerKV> layers;
};

// Lowest-free-page allocator over the HBM arena.
struct HbmAlloc {
  std::vector<uint8_t> used;
  int64_t cursor = 0;
  int32_t alloc_below(int64_t limit) {
    if (limit > (int64_t)used.size()) limit = (int64_t)used.size();
    while (cursor < limit && used[cursor]) ++cursor;
    if (cursor >= limit) return -1;
    used[cursor] = 1;
    return (int32_t)cursor++;
  }
  void release(int64_t p) {
    used[p] = 0;
    if (p < cursor) cursor = p;
  }
};

// First-fit allocator of contiguous page runs in the pinned host arena.
struct RunAlloc {
  std::map<int64_t, int64_t> free_;  // start -> length
  void reset(int64_t n) {
    free_.clear();
    if (n > 0) free_[0] = n;
  }
  int64_t alloc(int64_t n) {
    if (n <= 0) return 0;
    for (auto it = free_.begin(); it != free_.end(); ++it) {
      if (it->second >= n) {
        int64_t s = it->first, len = it->second;
        free_.erase(it);
        if (len > n) free_[s + n] = len - n;
        return s;
      }
    }
    return -1;
  }
  void release(int64_t s, int64_t n) {
    if (n <= 0) return;
    auto nx = free_.lower_bound(s);
    if (nx != free_.end() && s + n == nx->first) {
      n += nx->second;
      nx = free_.erase(nx);
    }
    if (nx != free_.begin()) {
      auto pv = std::prev(nx);
      if (pv->first + pv->second == s) {
        pv->second += n;
        return;
      }
    }
    free_[s] = n;
  }
  // Grows the run [s, s+n) in place to `m` pages if the pages right behind it are free.
  bool extend(int64_t s, int64_t n, int64_t m) {
    auto it = free_.find(s + n);
    if (m <= n) return true;
    if (it == free_.end() || it->second < m - n) return false;
    const int64_t len = it->second;
    free_.erase(it);
    if (len > m - n) free_[s + m] = len - (m - n);
    return true;
  }
  int64_t total_free() const {
    int64_t t = 0;
    for (auto &kv : free_) t += kv.second;
    return t;
  }
};

struct CopyItem {
  int layer, req;
  int32_t stage_page0, reserved;
};
struct StageBlock {
  int layer;
  int32_t p0, n;  // absolute arena page range [p0, p0+n)
  std::vector<CopyItem> copies;
};
struct LiveBlock {
  int layer;
  int32_t p0, p1;
  bool consumed;
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Eq. (1) pieces for a placement.  x is row-major [n_req][L] of 0/1.
struct Eq1 {
  int64_t resident = 0, buffer = 0, host = 0;
};
inline Eq1 eq1_eval(int n_req, int L, const std::vector<int64_t> &b, const std::vector<uint8_t> &x) {
  Eq1 e;
  for (int l = 0; l < L; ++l) {
    int64_t off = 0;
    for (int r = 0; r < n_req; ++r) {
      if (x[(size_t)r * L + l]) e.resident += b[r];
      else off += b[r];
    }
    e.host += off;
    e.buffer = std::max(e.buffer, off);
  }
  return e;
}

inline bool bitmap_get(const uint8_t *bm, int L, int r, int l) {
  return (bm[(size_t)r * ((L + 7) / 8) + l / 8] >> (l % 8)) & 1;
}

class HostState {
 public:
  Shape sh;
  int64_t arena_pages = 0, host_pages = 0;
  std::vector<Req> reqs;    // plan order
  std::vector<Req> paused;  // out of the batch; their HBM blocks are reclaimable (removable cache)
  int64_t last_budget_bytes = 0;
  HbmAlloc hbm;
  RunAlloc host;
  bool has_plan = false;
  orbit_plan_info info{};

  std::vector<StageBlock> blocks;   // one per layer that has offloaded requests, in layer order
  std::vector<int> block_of_layer;  // index into blocks or -1
  std::vector<LiveBlock> live;      // staging ranges currently holding (or receiving) a layer

  // host mirror of the device page table (lengths live in the requests and travel with every launch)
  std::vector<int32_t> h_table;  // [max_req][L][cap_pages]

  // Deferred demotions of the last plan load (Section 4: plan changes are applied without stopping the
  // decode loop).  An HBM -> host copy whose source pages the new plan does not need at once (they lie
  // below the staging region and no allocation of this plan load took them) is taken out of `phases` and
  // listed here, grouped by layer: it may run beside the following steps, and only a later use of that
  // layer's host blocks, or a later plan load that touches its pages (lazy_src_mark_), has to wait for it.
  //
  // A deferred block of an active request stays readable where it was (LayerKV::dual_pages): attention reads
  // those pages, the step's new token goes there and into the host run, and the layer is not prefetched for that
  // request, until the copy has landed and `flip_layer` hands the block over to the staging schedule.  So that
  // the new token never meets a copy in flight, the last used page of such a block is copied at once (it stays
  // in `phases`) and only the pages before it are deferred.  In the zero-copy mode the hand-over switches the
  // row to the host pages instead of a staging range.
  std::vector<PageOp> deferred;          // sorted by layer
  std::vector<size_t> deferred_end;      // [L] end offset of layer l's ops in `deferred`
  std::vector<uint8_t> reuse_mark_;      // [arena_pages] scratch of the classification
  std::vector<int32_t> dual_in_layer;    // [L] blocks of the layer that are read in place
  // Deferred copies of earlier plan loads may still be running when the next one comes.  It has to wait for them
  // only if it touches what they touch: it hands out an HBM page one of them still reads (to a block, or to the
  // staging region), or a host page one of them still writes (as part of a new or grown host run), or it reads
  // such a host page.  The marks hold the pages of every deferred copy that no plan load has waited for yet; a
  // wait is for the copies of whole layers (one event each), and takes those layers' marks away.
  std::vector<uint8_t> lazy_src_mark_, lazy_dst_mark_;  // [arena_pages], [host_pages]: 0, or 1 + the layer of the copy
  int64_t lazy_src_top_ = 0;             // one past the highest marked HBM page
  bool lazy_marks_any_ = false;
  bool needs_lazy_wait = false;          // finding of the last successful plan_load: any layer's copies ...
  std::vector<uint8_t> wait_layer;       // ... and which layers' [L]
  static_assert(ORBIT_MAX_LAYERS < 255, "a page mark holds layer + 1 in a byte");
  // [L] after the last plan load: the layer has an active host block that is not read in place and whose host run
  // a deferred copy not yet waited for may still be writing (whoever reads it must wait for the layer's copies even
  // while other blocks of the layer are read in place)
  std::vector<uint8_t> plain_pending;

  std::string err;

  void init(const Shape &s, int64_t arena_pages_, int64_t host_pages_) {
    sh = s;
    arena_pages = arena_pages_;
    host_pages = host_pages_;
    hbm.used.assign((size_t)arena_pages, 0);
    hbm.cursor = 0;
    host.reset(host_pages);
    h_table.assign((size_t)sh.max_req * sh.L * sh.cap_pages, 0);
    block_of_layer.assign(sh.L, -1);
    deferred_end.assign(sh.L, 0);
    dual_in_layer.assign(sh.L, 0);
    lazy_src_mark_.assign((size_t)arena_pages, 0);
    lazy_dst_mark_.assign((size_t)host_pages, 0);
    plain_pending.assign(sh.L, 0);
    wait_layer.assign(sh.L, 0);
  }

  // Every deferred copy has landed (the caller has seen it on the device): nothing is left to collide with.
  void forget_deferred() {
    if (!lazy_marks_any_) return;
    std::fill(lazy_src_mark_.begin(), lazy_src_mark_.end(), 0);
    std::fill(lazy_dst_mark_.begin(), lazy_dst_mark_.end(), 0);
    lazy_marks_any_ = false;
    lazy_src_top_ = 0;
  }

  int find(int64_t id) const {
    for (size_t i = 0; i < reqs.size(); ++i)
      if (reqs[i].id == id) return (int)i;
    return -1;
  }
  int find_paused(int64_t id) const {
    for (size_t i = 0; i < paused.size(); ++i)
      if (paused[i].id == id) return (int)i;
    return -1;
  }
  int32_t *table_row(int r, int l) { return &h_table[((size_t)r * sh.L + l) * sh.cap_pages]; }

  // ------------------------------------------------------------------------------ plan load
  // On success fills `phases` with the page copies to run, in order (one blit per phase), and
  // commits the new state.  On failure nothing is changed.
  // `pause_id` (or -1): an active request that leaves the batch but keeps its blocks (Pause-Resume,
  // Section 3.4; removable cache, Section 4).  Paused requests not listed in `ids` stay paused;
  // listing one resumes it.  Their HBM blocks are evicted to the host only when this plan needs
  // the space, one layer at a time.
  int plan_load(int32_t n_req, const int64_t *ids, const int32_t *ctx_len, const uint8_t *bitmap,
                int64_t budget_bytes, std::vector<std::vector<PageOp>> &phases, int64_t pause_id = -1,
                bool do_pause = false) {
    // A host run gets a few pages more than the request has reserved, so that the next plan load, which reserves
    // for a longer context, need not move the run (a copy of the whole block within the host arena, and a wait for
    // whatever is still being written into it); if the arena has no room for that, the plan is laid out without.
    int rc = plan_load_once(n_req, ids, ctx_len, bitmap, budget_bytes, phases, pause_id, do_pause, true);
    if (rc == ORBIT_E_HOST_CAPACITY) rc = plan_load_once(n_req, ids, ctx_len, bitmap, budget_bytes, phases, pause_id, do_pause, false);
    return rc;
  }

  int plan_load_once(int32_t n_req, const int64_t *ids, const int32_t *ctx_len, const uint8_t *bitmap,
                     int64_t budget_bytes, std::vector<std::vector<PageOp>> &phases, int64_t pause_id, bool do_pause,
                     bool host_slack) {
    phases.clear();
    auto host_room = [&](int64_t blocks) { return blocks + (host_slack ? std::max<int64_t>(1, blocks >> 5) : 0); };
    if (n_req < 0 || n_req > sh.max_req) return fail(ORBIT_E_INVAL, "n_req out of range");
    if (n_req > 0 && (!ids || !ctx_len || !bitmap)) return fail(ORBIT_E_INVAL, "null argument");
    if (budget_bytes < 0) return fail(ORBIT_E_INVAL, "negative budget");
    const int L = sh.L, P = sh.P;
    std::vector<int64_t> rb(n_req);
    std::vector<uint8_t> x((size_t)n_req * L);
    std::unordered_map<int64_t, int> seen;
    for (int r = 0; r < n_req; ++r) {
      if (!seen.emplace(ids[r], r).second) return fail(ORBIT_E_INVAL, "duplicate request id");
      if (ctx_len[r] < 0 || (int64_t)ctx_len[r] + sh.window > sh.max_tokens)
        return fail(ORBIT_E_INVAL, "ctx_len (+ decode window) exceeds max_tokens_per_request");
      rb[r] = ceil_div((int64_t)ctx_len[r] + sh.window, P);
      for (int l = 0; l < L; ++l) x[(size_t)r * L + l] = bitmap_get(bitmap, L, r, l);
      int o = find(ids[r]);
      int po = o < 0 ? find_paused(ids[r]) : -1;
      const Req *known = o >= 0 ? &reqs[o] : (po >= 0 ? &paused[po] : nullptr);
      if (known)
        for (int l = 0; l < L; ++l)
          if (known->layers[l].len != ctx_len[r])
            return fail(ORBIT_E_STATE, "ctx_len differs from the stored length of a known request");
      if (do_pause && ids[r] == pause_id) return fail(ORBIT_E_INVAL, "request both listed and paused");
    }
    // Eq. (1)
    Eq1 e = eq1_eval(n_req, L, rb, x);
    const int64_t staging = sh.zero_copy ? 0 : (int64_t)sh.slots * e.buffer;
    const int64_t b_gpu = std::min<int64_t>(budget_bytes / sh.page_bytes, arena_pages);
    if (e.resident + staging > b_gpu)
      return fail(ORBIT_E_CAPACITY, "Eq.(1) violated: resident " + std::to_string(e.resident) + " + staging " +
                                        std::to_string(staging) + " blocks > budget " + std::to_string(b_gpu));
    if (e.host > host_pages) return fail(ORBIT_E_HOST_CAPACITY, "host arena smaller than the offloaded blocks");
    const int64_t ring_first = b_gpu - staging;

    // work on copies; commit at the end
    HbmAlloc A = hbm;
    RunAlloc H = host;
    std::vector<Req> old = reqs;
    // A block that the last plan load sent to the host, that is still read in place and that this plan wants in
    // HBM again takes its pages back: they hold all of its tokens (a step's new token went there too), so nothing
    // is copied.  Its host run is given up; the copy that may still be writing into it runs ahead of whatever
    // this or a later plan load puts there.
    int64_t reclaimed = 0;
    for (int r = 0; r < n_req; ++r) {
      const int o = find(ids[r]);
      if (o < 0) continue;
      for (int l = 0; l < L; ++l) {
        LayerKV &lk = old[o].layers[l];
        if (lk.dual_pages.empty() || !x[(size_t)r * L + l]) continue;
        lk.pages = std::move(lk.dual_pages);
        lk.dual_pages.clear();
        while ((int64_t)lk.pages.size() > rb[r]) lk.pages.pop_back();
        for (int32_t pg : lk.pages) A.used[pg] = 1;
        H.release(lk.host_page0, lk.host_cap);
        lk.tier = 1;
        lk.host_page0 = -1;
        lk.host_cap = 0;
        lk.stage_page0 = -1;
        reclaimed += ceil_div(lk.len, P);
      }
    }
    // A block that is still read in place and stays offloaded goes on being read in place if this plan load leaves
    // its pages alone: they are held back like the pages the plan load vacates, and what became of them is seen at
    // the end.  Blocks of requests that leave the batch become plain host blocks: a step waits for their layer's
    // copies before it reads the host run.
    struct StillInPlace { int r, l; int64_t host_page0; };
    std::vector<StillInPlace> still;
    std::vector<int64_t> held, held_marked;
    {
      std::vector<uint8_t> stays(old.size(), 0);
      for (int r = 0; r < n_req; ++r) {
        const int o = find(ids[r]);
        if (o < 0) continue;
        stays[o] = 1;
        for (int l = 0; l < L; ++l) {
          const LayerKV &lk = old[o].layers[l];
          if (lk.dual_pages.empty()) continue;
          still.push_back({r, l, lk.host_page0});
          for (int32_t pg : lk.dual_pages) {
            A.used[pg] = 1;
            held.push_back(pg);
          }
        }
      }
      for (size_t o = 0; o < old.size(); ++o)
        if (!stays[o])
          for (auto &lk : old[o].layers) lk.dual_pages.clear();
      // Free pages that a deferred copy not yet waited for may still read are held back too (handing one out costs
      // that wait), but go before the others when pages run short.
      if (lazy_marks_any_)
        for (int64_t pg = 0; pg < lazy_src_top_; ++pg)
          if (lazy_src_mark_[pg] && !A.used[pg]) {
            A.used[pg] = 1;
            held_marked.push_back(pg);
          }
    }
    std::vector<Req> oldp = paused;
    std::vector<Req> np;  // paused after this call
    std::vector<Req> nw(n_req);
    std::vector<int> old_of(n_req, -1), oldp_of(n_req, -1);
    std::vector<uint8_t> kept(old.size(), 0), resumed(oldp.size(), 0);
    int64_t to_host = 0, to_hbm = 0, reloc = 0, evicted = 0;

    for (int r = 0; r < n_req; ++r) {
      int o = find(ids[r]);
      old_of[r] = o;
      if (o >= 0) kept[o] = 1;
      else if ((oldp_of[r] = find_paused(ids[r])) >= 0) resumed[oldp_of[r]] = 1;
    }
    for (size_t o = 0; o < oldp.size(); ++o)
      if (!resumed[o]) np.push_back(std::move(oldp[o]));
    // (a) requests that leave the batch: paused ones keep their blocks (trimmed to what is used),
    //     dropped ones free everything
    for (size_t o = 0; o < old.size(); ++o) {
      if (kept[o]) continue;
      if (do_pause && old[o].id == pause_id) {
        Req q = std::move(old[o]);
        for (auto &lk : q.layers) {
          const size_t used = (size_t)ceil_div(lk.len, P);
          while (lk.pages.size() > used) { A.release(lk.pages.back()); lk.pages.pop_back(); }
          lk.stage_page0 = -1;
        }
        q.reserved = (int32_t)ceil_div(q.layers[0].len, P);
        np.push_back(std::move(q));
        continue;
      }
      for (auto &lk : old[o].layers) {
        for (int32_t p : lk.pages) A.release(p);
        if (lk.tier == 0) H.release(lk.host_page0, lk.host_cap);
      }
    }
    for (int r = 0; r < n_req; ++r) {
      if (old_of[r] >= 0) nw[r] = std::move(old[old_of[r]]);
      else if (oldp_of[r] >= 0) nw[r] = std::move(oldp[oldp_of[r]]);
      else {
        nw[r].id = ids[r];
        nw[r].layers.assign(L, LayerKV());
        for (auto &lk : nw[r].layers) { lk.len = ctx_len[r]; lk.tier = 2; /* unallocated */ }
      }
      nw[r].reserved = (int32_t)rb[r];
    }
    std::vector<int64_t> free_hbm;
    std::vector<std::pair<int64_t, int64_t>> free_host;
    std::vector<DemoteGroup> groups;       // blocks leaving HBM (evictions and demotions)
    std::vector<std::pair<int64_t, int64_t>> new_host;  // host page ranges this plan load hands out (start, pages)
    std::vector<int32_t> taken;            // HBM pages this plan load allocated
    // Pages that evictions and demotions vacate are handed out again only when nothing else is free: a block
    // whose old pages stay untouched can leave HBM beside the following steps and be read in place meanwhile.
    auto end_phase = [&](bool hold = false) {
      for (int64_t p : free_hbm) {
        if (hold) held.push_back(p);
        else A.release(p);
      }
      for (auto &pr : free_host) H.release(pr.first, pr.second);
      free_hbm.clear();
      free_host.clear();
    };
    auto take_page = [&]() -> int32_t {
      int32_t p = A.alloc_below(ring_first);
      for (auto *pool : {&held_marked, &held}) {
        if (p >= 0 || pool->empty()) continue;
        for (int64_t h : *pool) A.release(h);
        pool->clear();
        p = A.alloc_below(ring_first);
      }
      return p;
    };
    // (a2) removable cache: paused blocks are evicted only where this plan needs the room — every
    //      paused layer with a page inside the new staging region, then, while the active resident
    //      blocks do not fit below it, the highest resident layer of the paused request that holds
    //      the most HBM blocks.
    phases.emplace_back();
    {
      auto resident_pages = [&](const Req &q) {
        int64_t n = 0;
        for (auto &lk : q.layers) if (lk.tier == 1) n += (int64_t)lk.pages.size();
        return n;
      };
      auto evict = [&](LayerKV &lk, int layer) -> int {
        const int64_t used = (int64_t)lk.pages.size();
        int64_t run = H.alloc(used);
        if (run < 0) return ORBIT_E_HOST_CAPACITY;
        new_host.push_back({run, used});
        for (int32_t p : lk.pages) free_hbm.push_back(p);
        groups.push_back({(int)phases.size() - 1, layer, (size_t)used, -1, run, std::move(lk.pages)});
        evicted += used;
        lk.pages.clear();
        lk.tier = 0;
        lk.host_page0 = run;
        lk.host_cap = (int32_t)used;
        return ORBIT_OK;
      };
      for (auto &q : np)
        for (int l = 0; l < L; ++l) {
          LayerKV &lk = q.layers[l];
          if (lk.tier != 1) continue;
          bool inside = false;
          for (int32_t pg : lk.pages) inside |= pg >= ring_first;
          if (inside && evict(lk, l)) return fail(ORBIT_E_HOST_CAPACITY, "host arena full (evicting a paused request)");
        }
      for (;;) {
        int64_t held = 0;
        int victim = -1;
        int64_t most = 0;
        for (size_t i = 0; i < np.size(); ++i) {
          int64_t n = resident_pages(np[i]);
          held += n;
          if (n > most) { most = n; victim = (int)i; }
        }
        if (e.resident + held <= ring_first || victim < 0) break;
        for (int l = L - 1; l >= 0; --l)
          if (np[victim].layers[l].tier == 1 && !np[victim].layers[l].pages.empty()) {
            if (evict(np[victim].layers[l], l)) return fail(ORBIT_E_HOST_CAPACITY, "host arena full (evicting a paused request)");
            break;
          }
      }
    }
    end_phase(true);
    // (b) demotions HBM -> host
    phases.emplace_back();
    for (int r = 0; r < n_req; ++r)
      for (int l = 0; l < L; ++l) {
        LayerKV &lk = nw[r].layers[l];
        if (lk.tier != 1 || x[(size_t)r * L + l]) continue;
        const int64_t room = host_room(rb[r]);
        int64_t run = H.alloc(room);
        if (run < 0) return fail(ORBIT_E_HOST_CAPACITY, "host arena full or fragmented (demotion)");
        new_host.push_back({run, room});
        int64_t used = ceil_div(lk.len, P);
        to_host += used;
        for (int32_t p : lk.pages) free_hbm.push_back(p);
        groups.push_back({(int)phases.size() - 1, l, (size_t)used, r, run, std::move(lk.pages)});
        lk.pages.clear();
        lk.tier = 0;
        lk.host_page0 = run;
        lk.host_cap = (int32_t)room;
      }
    end_phase(true);
    // (c) host runs that must grow
    phases.emplace_back();
    for (int r = 0; r < n_req; ++r)
      for (int l = 0; l < L; ++l) {
        LayerKV &lk = nw[r].layers[l];
        if (lk.tier != 0 || x[(size_t)r * L + l] || lk.host_cap >= rb[r]) continue;
        const int64_t room = host_room(rb[r]);
        const int64_t grown = H.extend(lk.host_page0, lk.host_cap, room) ? room
                              : H.extend(lk.host_page0, lk.host_cap, rb[r]) ? rb[r] : 0;
        if (grown) {  // room right behind the run: no copy
          new_host.push_back({lk.host_page0 + lk.host_cap, grown - lk.host_cap});
          lk.host_cap = (int32_t)grown;
          continue;
        }
        int64_t run = H.alloc(room);
        if (run < 0) return fail(ORBIT_E_HOST_CAPACITY, "host arena full or fragmented (growth)");
        new_host.push_back({run, room});
        int64_t used = ceil_div(lk.len, P);
        for (int64_t i = 0; i < used; ++i) phases.back().push_back({OP_HOST_TO_HOST, lk.host_page0 + i, run + i});
        free_host.push_back({lk.host_page0, lk.host_cap});
        lk.host_page0 = run;
        lk.host_cap = (int32_t)room;
      }
    end_phase();
    // (d) resident blocks sitting at or above the new staging region move below it
    phases.emplace_back();
    for (int r = 0; r < n_req; ++r)
      for (int l = 0; l < L; ++l) {
        LayerKV &lk = nw[r].layers[l];
        if (lk.tier != 1 || !x[(size_t)r * L + l]) continue;
        int64_t used = ceil_div(lk.len, P);
        for (size_t i = 0; i < lk.pages.size(); ++i) {
          if (lk.pages[i] < ring_first) continue;
          int32_t np = take_page();
          if (np < 0) return fail(ORBIT_E_CAPACITY, "internal: no page below the staging region");
          taken.push_back(np);
          if ((int64_t)i < used) {
            phases.back().push_back({OP_HBM_TO_HBM, lk.pages[i], np});
            ++reloc;
          }
          free_hbm.push_back(lk.pages[i]);
          lk.pages[i] = np;
        }
      }
    end_phase();
    // (e) growth of resident lists, promotions host -> HBM, new resident requests
    phases.emplace_back();
    {
      size_t n_promote = 0, n_take = 0;
      for (int r = 0; r < n_req; ++r)
        for (int l = 0; l < L; ++l) {
          const LayerKV &lk = nw[r].layers[l];
          if (!x[(size_t)r * L + l]) continue;
          if (lk.tier == 0) n_promote += (size_t)ceil_div(lk.len, P);
          n_take += (size_t)rb[r] - (lk.tier == 1 ? std::min<size_t>(lk.pages.size(), (size_t)rb[r]) : 0);
        }
      phases.back().reserve(n_promote);
      taken.reserve(taken.size() + n_take);
    }
    for (int r = 0; r < n_req; ++r)
      for (int l = 0; l < L; ++l) {
        LayerKV &lk = nw[r].layers[l];
        if (!x[(size_t)r * L + l]) continue;
        int64_t used = ceil_div(lk.len, P);
        bool promote = (lk.tier == 0);
        if (lk.tier != 1) lk.pages.clear();
        lk.pages.reserve((size_t)rb[r]);
        while ((int64_t)lk.pages.size() < rb[r]) {
          int32_t np = take_page();
          if (np < 0) return fail(ORBIT_E_CAPACITY, "internal: resident allocation failed");
          taken.push_back(np);
          lk.pages.push_back(np);
        }
        if (promote) {
          for (int64_t i = 0; i < used; ++i) phases.back().push_back({OP_HOST_TO_HBM, lk.host_page0 + i, lk.pages[i]});
          to_hbm += used;
          free_host.push_back({lk.host_page0, lk.host_cap});
          lk.host_page0 = -1;
          lk.host_cap = 0;
        }
        lk.tier = 1;
        lk.stage_page0 = -1;
      }
    end_phase();
    // (f) new offloaded requests
    for (int r = 0; r < n_req; ++r)
      for (int l = 0; l < L; ++l) {
        LayerKV &lk = nw[r].layers[l];
        if (lk.tier != 2) continue;
        const int64_t room = host_room(rb[r]);
        int64_t run = H.alloc(room);
        if (run < 0) return fail(ORBIT_E_HOST_CAPACITY, "host arena full or fragmented (new request)");
        new_host.push_back({run, room});
        lk.tier = 0;
        lk.host_page0 = run;
        lk.host_cap = (int32_t)room;
      }

    for (auto *pool : {&held_marked, &held}) {
      for (int64_t h : *pool) A.release(h);
      pool->clear();
    }

    // staging schedule: each layer's offloaded requests occupy one contiguous range; ranges are
    // laid out round-robin over the staging region; inside a range, smallest request first.
    std::vector<StageBlock> nb;
    std::vector<int> bol(L, -1);
    int64_t cursor = 0;
    for (int l = 0; l < L && !sh.zero_copy; ++l) {
      std::vector<int> off;
      int64_t n = 0;
      for (int r = 0; r < n_req; ++r)
        if (!x[(size_t)r * L + l]) { off.push_back(r); n += rb[r]; }
      if (off.empty()) continue;
      std::stable_sort(off.begin(), off.end(), [&](int a, int b) { return rb[a] < rb[b]; });
      if (cursor + n > staging) cursor = 0;
      StageBlock sb;
      sb.layer = l;
      sb.p0 = (int32_t)(ring_first + cursor);
      sb.n = (int32_t)n;
      int64_t at = sb.p0;
      for (int r : off) {
        sb.copies.push_back({l, r, (int32_t)at, (int32_t)rb[r]});
        nw[r].layers[l].stage_page0 = (int32_t)at;
        at += rb[r];
      }
      cursor += n;
      bol[l] = (int)nb.size();
      nb.push_back(std::move(sb));
    }

    // The copies of the blocks that leave HBM are written out only now, when it is known which of them may run
    // lazily: every source page below the staging region and not handed out again by this plan load.  Those go
    // to `deferred`, grouped by layer (for a block that stays readable in place: all but the copy of its last
    // used page); the others to the phase of their group, in group order.
    std::vector<PageOp> lazy;
    std::vector<size_t> lazy_end(L, 0);
    std::vector<int32_t> dual_count(L, 0);
    int64_t n_deferred = 0, n_in_place = 0, n_still = 0;
    if (!groups.empty() || !still.empty()) {
      reuse_mark_.assign((size_t)arena_pages, 0);
      for (int32_t pg : taken) reuse_mark_[pg] = 1;
    }
    auto untouched = [&](int64_t pg) { return pg < ring_first && !reuse_mark_[pg]; };
    // The staging region grows downwards as the requests' reservations grow (a page per request and staging range
    // every 16 tokens): a copy is deferred only if its source lies a little below the region, so that the next plan
    // loads with the same placement need not wait for it.
    const int64_t defer_below = ring_first - (sh.zero_copy ? 0 : (int64_t)sh.slots * n_req);
    for (const StillInPlace &c : still) {  // its used pages untouched, its host run where it was: read in place on
      LayerKV &lk = nw[c.r].layers[c.l];
      size_t keep = 0;
      while (keep < lk.dual_pages.size() && untouched(lk.dual_pages[keep])) ++keep;
      if (lk.tier == 0 && lk.host_page0 == c.host_page0 && (int64_t)keep >= std::max<int64_t>(ceil_div(lk.len, P), 1)) {
        lk.dual_pages.resize(keep);
        ++dual_count[c.l];
        n_still += ceil_div(lk.len, P);
      } else {
        lk.dual_pages.clear();
      }
    }
    if (!groups.empty()) {
      std::vector<size_t> n_lazy(groups.size(), 0);  // the first n_lazy copies of the group are deferred
      std::vector<size_t> per_layer(L, 0), urgent(phases.size(), 0);
      for (size_t gi = 0; gi < groups.size(); ++gi) {
        DemoteGroup &g = groups[gi];
        const bool in_place = g.req >= 0;
        bool ok = g.n > (in_place ? 1u : 0u);
        for (size_t i = 0; i < g.n && ok; ++i) ok = untouched(g.old_pages[i]) && g.old_pages[i] < defer_below;
        if (ok) {
          n_lazy[gi] = in_place ? g.n - 1 : g.n;
          per_layer[g.layer] += n_lazy[gi];
          if (in_place) {  // the used pages, and as many of the reserved ones behind them as are still untouched
            size_t keep = g.n;
            while (keep < g.old_pages.size() && untouched(g.old_pages[keep])) ++keep;
            LayerKV &lk = nw[g.req].layers[g.layer];
            lk.dual_pages.assign(g.old_pages.begin(), g.old_pages.begin() + keep);
            ++dual_count[g.layer];
            n_in_place += (int64_t)g.n;
          }
        }
        urgent[g.phase] += g.n - n_lazy[gi];
        n_deferred += (int64_t)n_lazy[gi];
      }
      size_t at = 0;
      std::vector<size_t> cursor(L, 0);
      for (int l = 0; l < L; ++l) {
        cursor[l] = at;
        at += per_layer[l];
        lazy_end[l] = at;
      }
      lazy.resize(at);
      for (size_t ph = 0; ph < phases.size(); ++ph)
        if (urgent[ph]) phases[ph].reserve(phases[ph].size() + urgent[ph]);
      for (size_t gi = 0; gi < groups.size(); ++gi) {
        const DemoteGroup &g = groups[gi];
        for (size_t i = 0; i < g.n; ++i) {
          const PageOp op{OP_HBM_TO_HOST, g.old_pages[i], g.host_run + (int64_t)i};
          if (i < n_lazy[gi]) lazy[cursor[g.layer]++] = op;
          else phases[g.phase].push_back(op);
        }
      }
    }

    // Which of the copies that earlier plan loads deferred must be waited for?  (see lazy_src_mark_; a mark names
    // the layer whose copies touch the page, and the copies of a layer have one event)
    std::vector<uint8_t> wait(L, 0);
    bool wait_lazy = false;
    if (lazy_marks_any_) {
      auto hit = [&](uint8_t mark) {
        if (mark) wait[mark - 1] = 1, wait_lazy = true;
      };
      for (int64_t pg = ring_first; pg < lazy_src_top_; ++pg) hit(lazy_src_mark_[pg]);
      for (int32_t pg : taken) hit(lazy_src_mark_[pg]);
      for (auto &run : new_host)
        for (int64_t pg = run.first; pg < run.first + run.second; ++pg) hit(lazy_dst_mark_[pg]);
      for (auto &ph : phases)
        for (const PageOp &op : ph)
          if (op.kind == OP_HOST_TO_HBM || op.kind == OP_HOST_TO_HOST) hit(lazy_dst_mark_[op.src]);
    }

    // commit
    needs_lazy_wait = wait_lazy;
    wait_layer = wait;
    if (wait_lazy) {  // what has been waited for is forgotten
      bool any = false;
      for (auto *marks : {&lazy_src_mark_, &lazy_dst_mark_})
        for (uint8_t &mk : *marks) {
          if (mk && wait[mk - 1]) mk = 0;
          any |= mk != 0;
        }
      lazy_marks_any_ = any;
      if (!any) lazy_src_top_ = 0;
    }
    std::fill(plain_pending.begin(), plain_pending.end(), 0);
    if (lazy_marks_any_)
      for (int r = 0; r < n_req; ++r)
        for (int l = 0; l < L; ++l) {
          const LayerKV &lk = nw[r].layers[l];
          if (lk.tier != 0 || !lk.dual_pages.empty() || plain_pending[l]) continue;
          for (int64_t pg = lk.host_page0; pg < lk.host_page0 + lk.host_cap && !plain_pending[l]; ++pg)
            plain_pending[l] = lazy_dst_mark_[pg];
        }
    for (int l = 0; l < L; ++l)
      for (size_t i = l ? lazy_end[l - 1] : 0; i < lazy_end[l]; ++i) {
        const PageOp &op = lazy[i];
        lazy_src_top_ = std::max(lazy_src_top_, op.src + 1);
        lazy_src_mark_[op.src] = lazy_dst_mark_[op.dst] = (uint8_t)(l + 1);
        lazy_marks_any_ = true;
      }
    deferred = std::move(lazy);
    deferred_end = std::move(lazy_end);
    info.deferred_to_host_blocks = n_deferred;
    info.in_place_blocks = n_in_place;
    info.still_in_place_blocks = n_still;
    info.reclaimed_blocks = reclaimed;
    info.waited_for_deferred = wait_lazy;  // (with a device behind it, the caller may still find a reason to wait)
    dual_in_layer = std::move(dual_count);
    hbm = std::move(A);
    host = std::move(H);
    reqs = std::move(nw);
    paused = std::move(np);
    last_budget_bytes = budget_bytes;
    blocks = std::move(nb);
    block_of_layer = std::move(bol);
    live.clear();
    has_plan = true;
    info.page_bytes = sh.page_bytes;
    info.budget_blocks = b_gpu;
    info.resident_blocks = e.resident;
    info.buffer_blocks = e.buffer;
    info.staging_first_page = ring_first;
    info.staging_blocks = staging;
    info.host_blocks = e.host;
    info.moved_to_host_blocks = to_host;
    info.moved_to_hbm_blocks = to_hbm;
    info.relocated_blocks = reloc;
    info.evicted_blocks = evicted;
    info.paused_requests = (int32_t)paused.size();
    info.paused_resident_blocks = 0;
    for (auto &q : paused)
      for (auto &lk : q.layers)
        if (lk.tier == 1) info.paused_resident_blocks += (int64_t)lk.pages.size();
    info.n_requests = n_req;
    info.chunk_tokens = sh.chunk_tokens;
    rebuild_tables();
    return ORBIT_OK;
  }

  // Re-installs the current placement for the batch without `id`, which becomes paused.
  int pause(int64_t id, std::vector<std::vector<PageOp>> &phases) {
    const int o = find(id);
    if (o < 0) return fail(find_paused(id) >= 0 ? ORBIT_E_STATE : ORBIT_E_NOT_FOUND,
                           find_paused(id) >= 0 ? "request is already paused" : "unknown request id");
    for (int l = 1; l < sh.L; ++l)
      if (reqs[o].layers[l].len != reqs[o].layers[0].len)
        return fail(ORBIT_E_STATE, "request is in the middle of a step (layer lengths differ)");
    std::vector<int64_t> ids;
    std::vector<int32_t> n;
    std::vector<uint8_t> bm;
    const int bpr = (sh.L + 7) / 8;
    for (size_t r = 0; r < reqs.size(); ++r) {
      if ((int)r == o) continue;
      ids.push_back(reqs[r].id);
      n.push_back(reqs[r].layers[0].len);
      for (int l = 1; l < sh.L; ++l)
        if (reqs[r].layers[l].len != n.back())
          return fail(ORBIT_E_STATE, "a request is in the middle of a step (layer lengths differ)");
      size_t at = bm.size();
      bm.resize(at + bpr, 0);
      for (int l = 0; l < sh.L; ++l)
        if (reqs[r].layers[l].tier == 1) bm[at + l / 8] |= (uint8_t)(1u << (l % 8));
    }
    return plan_load((int32_t)ids.size(), ids.data(), n.data(), bm.data(), last_budget_bytes, phases, id, true);
  }

  int drop_paused(int64_t id) {
    const int po = find_paused(id);
    if (po < 0) return fail(find(id) >= 0 ? ORBIT_E_STATE : ORBIT_E_NOT_FOUND,
                            find(id) >= 0 ? "request is active; pause it or leave it out of the next plan" : "unknown request id");
    for (auto &lk : paused[po].layers) {
      for (int32_t p : lk.pages) hbm.release(p);
      if (lk.tier == 0) host.release(lk.host_page0, lk.host_cap);
    }
    paused.erase(paused.begin() + po);
    info.paused_requests = (int32_t)paused.size();
    info.paused_resident_blocks = 0;
    for (auto &q : paused)
      for (auto &lk : q.layers)
        if (lk.tier == 1) info.paused_resident_blocks += (int64_t)lk.pages.size();
    return ORBIT_OK;
  }

  // The blocks of `layer` that were read in place become ordinary host blocks (their copies have landed, or
  // whoever reads them next waits): `flipped` receives the request indices whose table row changed.
  void flip_layer(int layer, std::vector<int> &flipped) {
    flipped.clear();
    for (size_t r = 0; r < reqs.size(); ++r) {
      LayerKV &lk = reqs[r].layers[layer];
      if (lk.dual_pages.empty()) continue;
      lk.dual_pages.clear();
      rebuild_row((int)r, layer);
      flipped.push_back((int)r);
    }
    dual_in_layer[layer] = 0;
  }

  void rebuild_tables() {
    for (size_t r = 0; r < reqs.size(); ++r)
      for (int l = 0; l < sh.L; ++l) rebuild_row((int)r, l);
  }

  void rebuild_row(int r, int l) {
    const LayerKV &lk = reqs[r].layers[l];
    int32_t *row = table_row(r, l);
    for (int i = 0; i < sh.cap_pages; ++i) row[i] = 0;
    if (!lk.dual_pages.empty())
      for (size_t i = 0; i < lk.dual_pages.size(); ++i) row[i] = lk.dual_pages[i];
    else if (lk.tier == 1)
      for (size_t i = 0; i < lk.pages.size(); ++i) row[i] = lk.pages[i];
    else if (sh.zero_copy)  // host page p is written as ~p: the kernel reads it in place
      for (int i = 0; i < reqs[r].reserved; ++i) row[i] = ~(int32_t)(lk.host_page0 + i);
    else
      for (int i = 0; i < reqs[r].reserved; ++i) row[i] = lk.stage_page0 + i;
  }

  // ------------------------------------------------------------------------------ work list
  // Every request's tokens are cut into chunks of C tokens; a chunk is one segment {request index, first
  // token, C, position in the launch order}, served by Hkv workgroups (one per kv head).  C is
  // chunk_tokens if the caller fixed it; otherwise it is chosen per launch from the lengths alone (so
  // results do not depend on the placement): the largest power of two in [128, 4096] that still gives
  // every compute unit a workgroup.  Large chunks keep a unit streaming for longer between the bubbles
  // at the start and end of a workgroup (4096 instead of 1024: 1.4-4.5 % on 1.4-10 GB launches); a small
  // launch is cut finely enough to occupy the machine (one request of 8K tokens: 256-token chunks, 13 us
  // instead of 18 us).  When no request is longer than 512 tokens, or every request fits one chunk of at most
  // 4096 tokens and that alone fills half of the units, requests are not cut and the combine launch is not needed.
  // Launch order: longest segment first (only the ragged last chunks differ), so that the last round of
  // a launch is filled with the shortest ones; padded with -1 to a multiple of 8.  A request's segments
  // are consecutive (work_seg_base[r], work_n_parts[r]); segment s of kv head g owns partial slot s * Hkv + g.
  int n_cu = 256;                                  // compute units a launch can occupy
  int work_chunk = 0;                              // C of the list in hand
  int work_workers = 0;                            // entries of work_order
  std::vector<int32_t> work_order;                 // [work_workers] segment index or -1
  std::vector<int32_t> work_seg_base, work_n_parts;  // per request
  std::vector<std::pair<int32_t, int32_t>> work_sort_;  // kept to reuse its storage

  static constexpr int kMinChunk = 128, kMaxAutoChunk = 4096, kUncutTokens = 512;

  int64_t max_segments() const {
    if (sh.chunk_tokens > 0) return (int64_t)sh.max_req * ceil_div(sh.max_tokens, sh.chunk_tokens);
    // C < 4096 is only chosen when 2C would leave units idle: fewer than 2 * n_cu / Hkv segments then
    return (int64_t)sh.max_req * ceil_div(sh.max_tokens, kMaxAutoChunk) + 2 * std::max(1, n_cu / sh.Hkv) + sh.max_req;
  }

  // The chunk size for the current lengths of `layer`.
  int choose_chunk(int layer) const {
    if (sh.chunk_tokens > 0) return sh.chunk_tokens;
    const int R = (int)reqs.size(), H = sh.Hkv;
    int64_t longest = 1;
    for (int r = 0; r < R; ++r) longest = std::max<int64_t>(longest, reqs[r].layers[layer].len);
    // requests of up to 512 tokens are never cut (merging their parts would cost more than it saves); longer
    // ones are left whole when whole requests already fill half of the machine
    if (longest <= kUncutTokens || (longest <= kMaxAutoChunk && (int64_t)R * H * 2 >= n_cu)) {
      int c = kMinChunk;
      while (c < longest) c *= 2;
      return c;
    }
    int c = kMaxAutoChunk;
    for (; c > kMinChunk; c /= 2) {
      int64_t segs = 0;
      for (int r = 0; r < R; ++r) segs += ceil_div(reqs[r].layers[layer].len, c);
      if (segs * H >= n_cu) break;
    }
    return c;
  }

  int build_work_items(int layer, std::vector<int32_t> &segs) {
    segs.clear();
    const int R = (int)reqs.size();
    for (int r = 0; r < R; ++r)
      if (reqs[r].layers[layer].len < 1) return fail(ORBIT_E_INVAL, "a request holds no token in this layer");
    const int C = work_chunk = choose_chunk(layer);
    work_seg_base.assign(R, 0);
    work_n_parts.assign(R, 0);
    work_sort_.clear();
    for (int r = 0; r < R; ++r) {
      const int64_t n = reqs[r].layers[layer].len;
      work_seg_base[r] = (int32_t)(segs.size() / 4);
      work_n_parts[r] = (int32_t)ceil_div(n, C);
      for (int64_t t = 0; t < n; t += C) {
        work_sort_.push_back({(int32_t)std::min<int64_t>(C, n - t), (int32_t)(segs.size() / 4)});
        segs.push_back(r);
        segs.push_back((int32_t)t);
        segs.push_back(C);
        segs.push_back(0);
      }
    }
    const int nseg = (int)(segs.size() / 4);
    if (nseg > max_segments()) return fail(ORBIT_E_CAPACITY, "work list larger than the buffers sized at creation");
    // (length descending, index ascending) is a total order: std::sort works in place, no temporary buffer
    std::sort(work_sort_.begin(), work_sort_.end(), [](const std::pair<int32_t, int32_t> &a, const std::pair<int32_t, int32_t> &b) {
      return a.first != b.first ? a.first > b.first : a.second < b.second;
    });
    work_workers = (nseg + 7) & ~7;
    work_order.assign(work_workers, -1);
    for (int i = 0; i < nseg; ++i) {
      work_order[i] = work_sort_[i].second;
      segs[4 * (size_t)work_sort_[i].second + 3] = i;
    }
    return ORBIT_OK;
  }

  int fail(int code, const std::string &msg) {
    err = msg;
    return code;
  }
};

}  // namespace orbit
