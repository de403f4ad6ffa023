// C ABI of liborbit (see include/orbit.h): ties the host state (orbit_host.hpp) to the gfx950
// kernels (orbit_kernels.hip) and to the two caller streams.  There is no CPU fallback: without
// a GPU every call that needs one returns ORBIT_E_HIP (ORBIT_FLAG_HOST_ONLY contexts run the
// integer host logic only and never produce attention output).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/orbit.h"
#include "orbit_host.hpp"
#include "orbit_kernels.h"
#include "orbit_planner.hpp"
#include "orbit_deposit.hpp"
#include "orbit_async_planner.hpp"

using namespace orbit;

namespace {
std::string g_create_error;
constexpr int kItemBufs = 2;  // pinned staging buffers of the work list
// Width of the kernel that carries the deferred copies of a plan switch.  Nobody waits for these copies before a
// plan load that needs their pages: the blocks are read in place meanwhile, so a narrow kernel (about 20 GB/s) is the better one: it
// leaves the compute units and the host->device direction of the link to the steps (measured behind an 11.5 GB
// demotion, steps 1-3 after the switch: 66 / 64 / 109 ms with 8 workgroups, 80 / 115 / 184 ms with 32,
// 120 / 154 / 203 ms with 128, 209 / 203 / 203 ms with 512; a steady step takes 203 ms).
constexpr int kDeferredCopyWorkgroups = 8;
static_assert(kMaxRequests == ORBIT_MAX_REQUESTS, "per-request launch arguments are sized by ORBIT_MAX_REQUESTS");
}  // namespace

// Split-K scratch of orbit_decode_attention_static: one array per GPU, in the library's own image, so
// that the entry point never allocates.  The symbol below is only a host-side handle; the address the
// kernels use is resolved once per device with hipGetSymbolAddress and kept in g_static_scratch.
constexpr size_t kStaticScratchBytes = (size_t)ORBIT_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
constexpr int kMaxDevices = 64;
void *g_static_scratch[kMaxDevices];  // per device ordinal; filled under g_static_scratch_mu
std::mutex g_static_scratch_mu;

// Device address of `scratch` on the current device (resolved on first use, then cached).
hipError_t static_scratch_for_current_device(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_scratch_mu);
  if (!g_static_scratch[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_static_scratch[dev] = ptr;
  }
  *out = g_static_scratch[dev];
  return hipSuccess;
}
}  // namespace

struct orbit_deposit {
  Deposit d;
};

struct orbit_planner {
  AsyncPlanner a;
  PlanDone held;      // a collected result that did not fit the caller's buffer yet
  bool has_held = false;
};

struct orbit_ctx {
  orbit_config cfg{};
  HostState hs;
  bool host_only = false;
  hipStream_t cs = nullptr, xs = nullptr;  // compute, copy (caller-owned)
  hipStream_t ds = nullptr;                // library-owned: deferred HBM -> host copies of a plan switch
  uint8_t *arena = nullptr;
  uint8_t *host_dev = nullptr;  // device-visible address of the pinned host arena
  int32_t *d_table = nullptr, *d_items = nullptr;
  float *d_pacc = nullptr, *d_pml = nullptr;
  BlitOp *d_ops = nullptr;            // device list of page copies of the last plan switch
  BlitOp *h_ops_pinned = nullptr;     // its pinned staging copy
  size_t d_ops_cap = 0;
  int32_t *h_tab_pinned = nullptr;                           // pinned snapshot the table upload reads
  hipEvent_t ev_ops = nullptr, ev_tab = nullptr;             // last use of the staging copies
  hipEvent_t ev_tab_rows = nullptr;                          // last single-row upload from the pinned table mirror
  hipEvent_t ev_plan_c = nullptr, ev_plan_x = nullptr;       // stream ordering of a plan switch
  hipEvent_t ev_ops_up = nullptr, ev_lazy_all = nullptr;     // op list uploaded; every deferred copy of the last switch done
  std::vector<hipEvent_t> ev_lazy;                           // per layer: that layer's deferred copies done
  std::vector<uint8_t> lazy_x, lazy_c;                       // per layer: copy / compute stream has yet to wait for ev_lazy[l]
  // A plan load that runs beside the deferred copies of earlier ones and defers copies of its own in a layer keeps
  // that layer's older event here: the blocks those older copies carry are plain host blocks by now, and whoever
  // reads them waits for this one, whatever the newer copies (whose blocks are read in place) are doing.
  std::vector<hipEvent_t> ev_lazy_prev;
  std::vector<uint8_t> prev_x, prev_c;                       // per layer: copy / compute stream has yet to wait for ev_lazy_prev[l]
  std::vector<uint8_t> settle_full;  // per layer: a plain host block's copies are among those ev_lazy[l] stands for
  bool lazy_outstanding = false;
  BlitOp *d_lazy[2] = {nullptr, nullptr};   // op lists of deferred copies: two, because the copies of one switch may
  size_t d_lazy_cap[2] = {0, 0};            // still be running when the next switch enqueues its own
  hipEvent_t ev_lazy_buf[2] = {nullptr, nullptr};  // the kernels that read d_lazy[i] are done
  int lazy_buf = 0;
  int32_t *h_items_pinned[kItemBufs] = {};
  hipEvent_t ev_items[kItemBufs] = {};
  int items_buf = 0;
  int64_t seg_cap = 0;                // most segments a work list can have
  int64_t slots = 0;                  // seg_cap * Hkv split-K partial slots
  std::vector<hipEvent_t> ev_ready, ev_done;
  hipEvent_t ev_tmp = nullptr;
  std::vector<hipEvent_t> t_wait0, t_wait1, t_attn0, t_attn1, t_comb1, t_copy0, t_copy1;
  hipEvent_t t_step0 = nullptr, t_step1 = nullptr;
  std::vector<uint8_t> host_dirty;    // per layer: host pages written since the last ordering point
  std::vector<uint8_t> copy_timed;    // per layer: t_copy0/1 recorded in this step
  std::vector<int64_t> copy_bytes;    // per layer, last prefetch
  std::vector<int32_t> items_key;     // chunk counts and chunk size the uploaded work list was built for
  std::vector<int32_t> items_key_tmp, items_tmp;  // scratch of ensure_work_items, kept for their storage
  std::vector<int> flipped_tmp;       // scratch of flip_in_place_blocks
  uint8_t *static_scratch = nullptr;  // this device's copy of the library's static split-K scratch
  int64_t n_segs = 0;
  bool items_valid = false;
  float scale_log2 = 0.f;
  AttnParams attn_args{};               // launch arguments, kept here because of their size
  CombineParams comb_args{};
  bool timing = false;
  std::string err;
};

namespace {

int set_err(orbit_ctx *c, int code, const std::string &msg) {
  c->err = msg;
  return code;
}
int hip_fail(orbit_ctx *c, hipError_t e, const char *what) {
  c->err = std::string(what) + ": " + hipGetErrorString(e);
  return ORBIT_E_HIP;
}
#define HIPCHECK(c, x)                                  \
  do {                                                  \
    hipError_t e_ = (x);                                \
    if (e_ != hipSuccess) return hip_fail((c), e_, #x); \
  } while (0)

int make_events(orbit_ctx *c, std::vector<hipEvent_t> &v, int n, bool timing) {
  v.assign(n, nullptr);
  for (int i = 0; i < n; ++i)
    HIPCHECK(c, hipEventCreateWithFlags(&v[i], timing ? hipEventDefault : hipEventDisableTiming));
  return ORBIT_OK;
}
void drop_events(std::vector<hipEvent_t> &v) {
  for (auto e : v)
    if (e) (void)hipEventDestroy(e);
  v.clear();
}

LiveBlock *find_live(orbit_ctx *c, int layer) {
  for (auto &lb : c->hs.live)
    if (lb.layer == layer) return &lb;
  return nullptr;
}

// A layer's host blocks may still be on their way out of HBM (deferred copies of the last plan switch):
// whoever is about to read or write them waits, stream-side, once per stream.
int wait_deferred(orbit_ctx *c, int layer, bool on_copy_stream) {
  if (c->host_only) return ORBIT_OK;
  std::vector<uint8_t> &flag = on_copy_stream ? c->lazy_x : c->lazy_c;
  if (!flag[layer]) return ORBIT_OK;
  HIPCHECK(c, hipStreamWaitEvent(on_copy_stream ? c->xs : c->cs, c->ev_lazy[layer], 0));
  flag[layer] = 0;
  (on_copy_stream ? c->prev_x : c->prev_c)[layer] = 0;  // the copies run in order: the newer event covers the older
  return ORBIT_OK;
}

// The same for the copies that plan loads before the last one deferred: their blocks are never read in place any more.
int wait_deferred_older(orbit_ctx *c, int layer, bool on_copy_stream) {
  if (c->host_only) return ORBIT_OK;
  std::vector<uint8_t> &flag = on_copy_stream ? c->prev_x : c->prev_c;
  if (!flag[layer]) return ORBIT_OK;
  HIPCHECK(c, hipStreamWaitEvent(on_copy_stream ? c->xs : c->cs, c->ev_lazy_prev[layer], 0));
  flag[layer] = 0;
  return ORBIT_OK;
}

// In front of a read of the layer's plain host blocks (those not read in place).  While blocks of the layer are still
// read in place, the layer's newest copies are theirs and only the older ones matter, unless a plan load found a
// plain block whose copies belong to the newest as well (settle_full).
int settle_host_blocks(orbit_ctx *c, int layer, bool on_copy_stream) {
  if (c->host_only) return ORBIT_OK;
  bool any = false;  // (a layer whose blocks are all resident, or all read in place, has nothing to wait for)
  for (const Req &q : c->hs.reqs) any |= q.layers[layer].tier == 0 && q.layers[layer].dual_pages.empty();
  if (!any) return ORBIT_OK;
  return c->hs.dual_in_layer[layer] && !c->settle_full[layer] ? wait_deferred_older(c, layer, on_copy_stream)
                                                               : wait_deferred(c, layer, on_copy_stream);
}

// Blocks of `layer` that the last plan load demoted and that are still read where they were in HBM: once the
// layer's deferred copies have landed (asked of the event, not waited for) they become ordinary host blocks,
// i.e. their page-table rows point into the staging region from here on (row uploads on the compute stream,
// behind every launch enqueued so far) and the caller prefetches them.  force: do it now and make the compute
// stream wait for the copies; also taken when a block's next token would not fit the pages it still has.
// grow: tokens the caller is about to add to every request of the layer before attending (1 in front of a step's
// length bump, 0 behind it).
int flip_in_place_blocks(orbit_ctx *c, int layer, bool force, int grow = 1) {
  HostState &hs = c->hs;
  if (!hs.dual_in_layer[layer]) return ORBIT_OK;
  const Shape &sh = hs.sh;
  for (const Req &q : hs.reqs) {
    const LayerKV &lk = q.layers[layer];
    if (!lk.dual_pages.empty() && ceil_div((int64_t)lk.len + grow, sh.P) > (int64_t)lk.dual_pages.size()) force = true;
  }
  if (!force && !c->host_only) {
    const hipError_t e = hipEventQuery(c->ev_lazy[layer]);
    if (e == hipErrorNotReady) {
      (void)hipGetLastError();  // "not ready" is an answer, not an error a later launch check should find
      return ORBIT_OK;
    }
    if (e != hipSuccess) return hip_fail(c, e, "hipEventQuery(ev_lazy)");
  }
  if (!c->host_only) {
    if (int rc = wait_deferred(c, layer, false)) return rc;
    // the last whole-table upload no longer reads the pinned mirror (a row is rewritten at most once between two
    // of those, so row uploads need not wait for each other)
    HIPCHECK(c, hipEventSynchronize(c->ev_tab));
  }
  hs.flip_layer(layer, c->flipped_tmp);
  if (!c->host_only) {
    for (int r : c->flipped_tmp) {
      const size_t off = ((size_t)r * sh.L + layer) * sh.cap_pages;
      std::memcpy(c->h_tab_pinned + off, hs.h_table.data() + off, (size_t)sh.cap_pages * sizeof(int32_t));
      HIPCHECK(c, hipMemcpyAsync(c->d_table + off, c->h_tab_pinned + off, (size_t)sh.cap_pages * sizeof(int32_t),
                                 hipMemcpyHostToDevice, c->cs));
    }
    HIPCHECK(c, hipEventRecord(c->ev_tab_rows, c->cs));
  }
  return ORBIT_OK;
}

// 0 = issued (or nothing to do), 1 = blocked by a prefetched layer not yet attended, <0 = error
int prefetch_impl(orbit_ctx *c, int layer) {
  HostState &hs = c->hs;
  const int b = hs.block_of_layer[layer];
  if (b < 0) return 0;
  LiveBlock *mine = find_live(c, layer);
  if (mine && !mine->consumed) return 0;
  const StageBlock &blk = hs.blocks[b];
  const int32_t p0 = blk.p0, p1 = blk.p0 + blk.n;
  for (auto &lb : hs.live)
    if (lb.p0 < p1 && p0 < lb.p1 && !lb.consumed) return 1;
  for (size_t i = 0; i < hs.live.size();) {
    LiveBlock &lb = hs.live[i];
    if (lb.p0 < p1 && p0 < lb.p1) {
      if (!c->host_only) HIPCHECK(c, hipStreamWaitEvent(c->xs, c->ev_done[lb.layer], 0));
      hs.live.erase(hs.live.begin() + i);
    } else {
      ++i;
    }
  }
  if (c->host_dirty[layer]) {
    if (!c->host_only) {
      HIPCHECK(c, hipEventRecord(c->ev_tmp, c->cs));
      HIPCHECK(c, hipStreamWaitEvent(c->xs, c->ev_tmp, 0));
    }
    c->host_dirty[layer] = 0;
  }
  if (int rc = flip_in_place_blocks(c, layer, false)) return rc;
  if (int rc = settle_host_blocks(c, layer, true)) return rc;  // they are read below
  if (c->timing && !c->host_only) HIPCHECK(c, hipEventRecord(c->t_copy0[layer], c->xs));
  int64_t bytes = 0;
  for (const CopyItem &ci : blk.copies) {
    const LayerKV &lk = hs.reqs[ci.req].layers[layer];
    const int64_t used = ceil_div(lk.len, hs.sh.P);
    if (used == 0 || !lk.dual_pages.empty()) continue;  // a block read in place needs no staging copy
    const int64_t nbytes = used * hs.sh.page_bytes;
    bytes += nbytes;
    if (!c->host_only)
      HIPCHECK(c, hipMemcpyAsync(c->arena + (int64_t)ci.stage_page0 * hs.sh.page_bytes,
                                 (const uint8_t *)c->cfg.host_arena + lk.host_page0 * hs.sh.page_bytes, (size_t)nbytes,
                                 hipMemcpyHostToDevice, c->xs));
  }
  c->copy_bytes[layer] = bytes;
  if (!c->host_only) {
    if (c->timing) {
      HIPCHECK(c, hipEventRecord(c->t_copy1[layer], c->xs));
      c->copy_timed[layer] = 1;
    }
    HIPCHECK(c, hipEventRecord(c->ev_ready[layer], c->xs));
  }
  hs.live.push_back({layer, p0, p1, false});
  return 0;
}

// The work list is a function of the chunk size chosen for the current lengths and of each request's chunk
// count; it is rebuilt (and uploaded again, stream-ordered on the compute stream) when those change.
int ensure_work_items(orbit_ctx *c, int layer) {
  HostState &hs = c->hs;
  const int nreq = (int)hs.reqs.size();
  std::vector<int32_t> &key = c->items_key_tmp;
  key.resize(nreq + 1);
  for (int r = 0; r < nreq; ++r)
    if (hs.reqs[r].layers[layer].len < 1) return set_err(c, ORBIT_E_INVAL, "a request holds no token in this layer");
  const int chunk = hs.choose_chunk(layer);
  key[nreq] = chunk;
  for (int r = 0; r < nreq; ++r) key[r] = (int32_t)ceil_div(hs.reqs[r].layers[layer].len, chunk);
  if (c->items_valid && key == c->items_key) return ORBIT_OK;
  std::vector<int32_t> &segs = c->items_tmp;
  int rc = hs.build_work_items(layer, segs);
  if (rc) return set_err(c, rc, hs.err);
  c->n_segs = (int64_t)segs.size() / 4;
  if (!c->host_only) {
    const int b = c->items_buf = (c->items_buf + 1) % kItemBufs;
    HIPCHECK(c, hipEventSynchronize(c->ev_items[b]));  // last upload from this buffer is long done
    int32_t *dst = c->h_items_pinned[b];
    for (int w = 0; w < hs.work_workers; ++w) {  // launch order; the kernel finds a segment with one load
      const int s = hs.work_order[w];
      if (s < 0) {
        dst[4 * w] = -1;
        dst[4 * w + 1] = dst[4 * w + 2] = dst[4 * w + 3] = 0;
      } else {
        dst[4 * w] = segs[4 * (size_t)s];
        dst[4 * w + 1] = segs[4 * (size_t)s + 1];
        dst[4 * w + 2] = segs[4 * (size_t)s + 2];
        dst[4 * w + 3] = s;
      }
    }
    HIPCHECK(c, hipMemcpyAsync(c->d_items, dst, (size_t)hs.work_workers * 4 * sizeof(int32_t), hipMemcpyHostToDevice, c->cs));
    HIPCHECK(c, hipEventRecord(c->ev_items[b], c->cs));
  }
  c->items_key = key;  // same capacity after the first call: no allocation
  c->items_valid = true;
  return ORBIT_OK;
}

// Waits for the layer's staging data (prefetching it first if nobody did), then attention + combine.
// k_new / v_new non-null: the lengths already count a token whose rows are still in those buffers; the
// kernel attends to it and stores it (append fused into the launch).
// use_static: the split-K partials live in the library's static scratch instead of the context's
// own buffers (orbit_decode_attention_static); checked against its size before anything is enqueued.
int attention_impl(orbit_ctx *c, int layer, const void *q, void *out, float *out_f32, bool wait_done_already,
                   const uint16_t *k_new = nullptr, const uint16_t *v_new = nullptr, bool use_static = false) {
  HostState &hs = c->hs;
  const Shape &sh = hs.sh;
  const int nreq = (int)hs.reqs.size();
  int rc = ensure_work_items(c, layer);
  if (rc) return rc;
  auto up256 = [](size_t n) { return (n + 255) & ~(size_t)255; };
  const size_t part_slots = (size_t)c->n_segs * sh.Hkv;
  const size_t pacc_bytes = up256(part_slots * sh.G * 128 * sizeof(float)), pml_bytes = up256(part_slots * 32 * sizeof(float));
  if (use_static) {
    if (c->host_only || !c->static_scratch) return set_err(c, ORBIT_E_STATE, "no static scratch on this context");
    if (pacc_bytes + pml_bytes > kStaticScratchBytes)
      return set_err(c, ORBIT_E_CAPACITY, "orbit_decode_attention_static: this batch needs " +
                                              std::to_string(pacc_bytes + pml_bytes) +
                                              " bytes of split-K scratch, the static buffer holds " +
                                              std::to_string(kStaticScratchBytes));
  }
  const bool staged = hs.block_of_layer[layer] >= 0;
  if (staged && !wait_done_already) {
    LiveBlock *lb = find_live(c, layer);
    if (!lb || lb->consumed) {
      rc = prefetch_impl(c, layer);
      if (rc == 1) return set_err(c, ORBIT_E_STATE, "staging range still needed by a prefetched layer not yet attended");
      if (rc) return rc;
      lb = find_live(c, layer);
    }
    if (!c->host_only) HIPCHECK(c, hipStreamWaitEvent(c->cs, c->ev_ready[layer], 0));
    lb->consumed = true;
  }
  // a block whose copy to the host may be in flight is read in place, and the append's write into its host run
  // cannot meet a copy (its last page was copied at once).  The staged mode hands such blocks over in the layer's
  // prefetch; the zero-copy mode, which has none, here: the lengths already count the token of a fused append
  if (sh.zero_copy && (rc = flip_in_place_blocks(c, layer, false, 0))) return rc;
  if (sh.zero_copy && (rc = settle_host_blocks(c, layer, false))) return rc;  // host blocks are read where they are
  if (!c->host_only) {
    if (c->timing) HIPCHECK(c, hipEventRecord(c->t_attn0[layer], c->cs));
    AttnParams &ap = c->attn_args;  // the per-request part is rewritten below; the rest is cheap to refill
    ap.arena = c->arena;
    ap.host = c->host_dev;
    ap.table = c->d_table;
    ap.work = c->d_items;
    ap.q = (const uint16_t *)q;
    if (use_static) {
      // every call on this GPU shares the array and inherits whatever the last one left; nothing in it has
      // to start at zero: the attention launch writes every partial that the combine launch reads
      ap.pacc = reinterpret_cast<float *>(c->static_scratch);
      ap.pml = reinterpret_cast<float *>(c->static_scratch + pacc_bytes);
    } else {
      ap.pacc = c->d_pacc;
      ap.pml = c->d_pml;
    }
    ap.out = (uint16_t *)out;
    ap.out_f32 = out_f32;
    ap.k_new = k_new;
    ap.v_new = v_new;
    ap.page_bytes = sh.page_bytes;
    ap.L = sh.L;
    ap.layer = layer;
    ap.cap_pages = sh.cap_pages;
    ap.Hq = sh.Hq;
    ap.Hkv = sh.Hkv;
    ap.G = sh.G;
    ap.n_workers = hs.work_workers;
    ap.scale_log2 = c->scale_log2;
    for (int r = 0; r < nreq; ++r) {
      const LayerKV &lk = hs.reqs[r].layers[layer];
      ap.req[r].n_tok = lk.len;
      // a staged block, and one still read in place, has a second home: its host run
      ap.req[r].host_page0 = (k_new && lk.tier == 0 && (!sh.zero_copy || !lk.dual_pages.empty())) ? (int32_t)lk.host_page0 : -1;
      ap.req[r].n_parts = hs.work_n_parts[r];
    }
    HIPCHECK(c, launch_attention(ap, c->cs));
    if (c->timing) HIPCHECK(c, hipEventRecord(c->t_attn1[layer], c->cs));
    bool multi = false;
    for (int r = 0; r < nreq; ++r) multi |= hs.work_n_parts[r] > 1;
    if (multi) {  // requests of a single segment were finished by the attention launch
      CombineParams &cp = c->comb_args;
      cp.pacc = ap.pacc;
      cp.pml = ap.pml;
      cp.out = ap.out;
      cp.out_f32 = out_f32;
      cp.Hq = sh.Hq;
      cp.Hkv = sh.Hkv;
      cp.G = sh.G;
      cp.n_req = nreq;
      for (int r = 0; r < nreq; ++r) {
        cp.seg_base[r] = hs.work_seg_base[r];
        cp.n_parts[r] = hs.work_n_parts[r];
      }
      HIPCHECK(c, launch_combine(cp, c->cs));
    }
    if (c->timing) HIPCHECK(c, hipEventRecord(c->t_comb1[layer], c->cs));
    if (staged && (c->cfg.flags & ORBIT_FLAG_POISON_STAGING)) {  // nobody may read this range again before it is refilled
      const StageBlock &blk = hs.blocks[hs.block_of_layer[layer]];
      HIPCHECK(c, launch_poison(c->arena + (int64_t)blk.p0 * sh.page_bytes, (int64_t)blk.n * sh.page_bytes, c->cs));
    }
    if (staged) HIPCHECK(c, hipEventRecord(c->ev_done[layer], c->cs));
  }
  return ORBIT_OK;
}

int check_layer(orbit_ctx *c, int layer) {
  if (!c) return ORBIT_E_INVAL;
  if (!c->hs.has_plan) return set_err(c, ORBIT_E_STATE, "no plan installed");
  if (layer < 0 || layer >= c->hs.sh.L) return set_err(c, ORBIT_E_INVAL, "layer out of range");
  return ORBIT_OK;
}

// GPU side of a plan switch, without any host-side stream synchronisation: the copy stream first
// waits for everything already enqueued on the compute stream, then runs the page migrations
// (one blit per phase, in order); the compute stream waits for them and then receives the new
// page table (lengths travel with every launch).  The pinned staging copies are reused only after their last transfer.
// Before a plan load: if the deferred copies of earlier ones have all landed, the new one has nothing to look out for.
int retire_deferred(orbit_ctx *c) {
  if (c->host_only || !c->lazy_outstanding) return ORBIT_OK;
  const hipError_t e = hipEventQuery(c->ev_lazy_all);
  if (e == hipErrorNotReady) {
    (void)hipGetLastError();
    return ORBIT_OK;
  }
  if (e != hipSuccess) return hip_fail(c, e, "hipEventQuery(ev_lazy_all)");
  std::fill(c->lazy_x.begin(), c->lazy_x.end(), 0);
  std::fill(c->lazy_c.begin(), c->lazy_c.end(), 0);
  std::fill(c->prev_x.begin(), c->prev_x.end(), 0);
  std::fill(c->prev_c.begin(), c->prev_c.end(), 0);
  std::fill(c->settle_full.begin(), c->settle_full.end(), 0);
  c->lazy_outstanding = false;
  c->hs.forget_deferred();
  return ORBIT_OK;
}

int apply_plan_gpu(orbit_ctx *c, const std::vector<std::vector<PageOp>> &phases) {
  if (c->host_only) return ORBIT_OK;
  const HostState &hs = c->hs;
  const Shape &sh = hs.sh;
  HIPCHECK(c, hipEventRecord(c->ev_plan_c, c->cs));
  HIPCHECK(c, hipStreamWaitEvent(c->xs, c->ev_plan_c, 0));
  // Deferred copies of earlier switches may still be running.  This switch waits for those of a layer only if it
  // touches a page they touch (HostState::wait_layer), and for all of them if it needs the op-list buffer their
  // kernels still read.
  const int lb = c->lazy_buf ^ 1;
  bool wait_lazy = false, waited_some = false;
  if (c->lazy_outstanding && hs.needs_lazy_wait)
    for (int l = 0; l < sh.L; ++l) {  // the copy stream waits for the layers this plan load collides with; the
      if (!hs.wait_layer[l]) continue;  // compute stream waits for the copy stream below
      HIPCHECK(c, hipStreamWaitEvent(c->xs, c->ev_lazy[l], 0));
      c->lazy_x[l] = c->lazy_c[l] = c->prev_x[l] = c->prev_c[l] = 0;
      waited_some = true;
    }
  if (c->lazy_outstanding && !hs.deferred.empty()) {
    const hipError_t e = hipEventQuery(c->ev_lazy_buf[lb]);
    if (e == hipErrorNotReady) {
      (void)hipGetLastError();
      wait_lazy = true;
    } else if (e != hipSuccess) {
      return hip_fail(c, e, "hipEventQuery(ev_lazy_buf)");
    }
  }
  c->hs.info.waited_for_deferred = wait_lazy || waited_some;
  if (wait_lazy) {
    HIPCHECK(c, hipStreamWaitEvent(c->xs, c->ev_lazy_all, 0));
    std::fill(c->lazy_x.begin(), c->lazy_x.end(), 0);
    std::fill(c->lazy_c.begin(), c->lazy_c.end(), 0);  // the compute stream waits for this switch below
    std::fill(c->prev_x.begin(), c->prev_x.end(), 0);
    std::fill(c->prev_c.begin(), c->prev_c.end(), 0);
    c->lazy_outstanding = false;
  }
  // Plain host blocks that earlier deferred copies may still be writing (HostState::plain_pending, nothing after a
  // wait): where the layer keeps blocks read in place, a reader of the plain ones must not skip the layer's event.
  // (A layer that gets copies of this plan load moves that event to ev_lazy_prev below instead.)
  for (int l = 0; l < sh.L; ++l)
    c->settle_full[l] = (c->lazy_x[l] || c->lazy_c[l]) && hs.plain_pending[l] && hs.dual_in_layer[l] &&
                        hs.deferred_end[l] == (l ? hs.deferred_end[l - 1] : 0);
  size_t urgent = 0;
  for (auto &ph : phases) urgent += ph.size();
  const size_t total = urgent + hs.deferred.size();
  if (total > 0) {
    HIPCHECK(c, hipEventSynchronize(c->ev_ops));
    if (total > c->d_ops_cap) {
      const size_t cap = std::max(total, 2 * c->d_ops_cap);
      if (c->d_ops) HIPCHECK(c, hipFree(c->d_ops));
      if (c->h_ops_pinned) HIPCHECK(c, hipHostFree(c->h_ops_pinned));
      c->d_ops = nullptr;
      c->h_ops_pinned = nullptr;
      c->d_ops_cap = 0;
      HIPCHECK(c, hipMalloc((void **)&c->d_ops, cap * sizeof(BlitOp)));
      HIPCHECK(c, hipHostMalloc((void **)&c->h_ops_pinned, cap * sizeof(BlitOp), hipHostMallocDefault));
      c->d_ops_cap = cap;
    }
    const int64_t pb = sh.page_bytes;
    auto hbm = [&](int64_t p) { return (uint64_t)(uintptr_t)(c->arena + p * pb); };
    auto hst = [&](int64_t p) { return (uint64_t)(uintptr_t)(c->host_dev + p * pb); };
    auto to_blit = [&](const PageOp &op) {
      BlitOp b{};
      switch (op.kind) {
        case OP_HBM_TO_HOST: b.src = hbm(op.src); b.dst = hst(op.dst); break;
        case OP_HOST_TO_HBM: b.src = hst(op.src); b.dst = hbm(op.dst); break;
        case OP_HBM_TO_HBM: b.src = hbm(op.src); b.dst = hbm(op.dst); break;
        default: b.src = hst(op.src); b.dst = hst(op.dst); break;
      }
      return b;
    };
    size_t n = 0;
    for (auto &ph : phases)
      for (const PageOp &op : ph) c->h_ops_pinned[n++] = to_blit(op);
    for (const PageOp &op : hs.deferred) c->h_ops_pinned[n++] = to_blit(op);
    if (urgent) HIPCHECK(c, hipMemcpyAsync(c->d_ops, c->h_ops_pinned, urgent * sizeof(BlitOp), hipMemcpyHostToDevice, c->xs));
    if (!hs.deferred.empty()) {
      if (hs.deferred.size() > c->d_lazy_cap[lb]) {
        HIPCHECK(c, hipEventSynchronize(c->ev_lazy_buf[lb]));  // the kernels that read the old buffer
        if (c->d_lazy[lb]) HIPCHECK(c, hipFree(c->d_lazy[lb]));
        c->d_lazy[lb] = nullptr;
        c->d_lazy_cap[lb] = 0;
        const size_t cap = hs.deferred.size() + hs.deferred.size() / 4;
        HIPCHECK(c, hipMalloc((void **)&c->d_lazy[lb], cap * sizeof(BlitOp)));
        c->d_lazy_cap[lb] = cap;
      }
      HIPCHECK(c, hipMemcpyAsync(c->d_lazy[lb], c->h_ops_pinned + urgent, hs.deferred.size() * sizeof(BlitOp),
                                 hipMemcpyHostToDevice, c->xs));
    }
    HIPCHECK(c, hipEventRecord(c->ev_ops_up, c->xs));
    size_t at = 0;
    for (auto &ph : phases) {
      if (ph.empty()) continue;
      HIPCHECK(c, launch_blit(c->d_ops + at, (int64_t)ph.size(), pb, c->xs));  // phases run in stream order
      at += ph.size();
    }
    HIPCHECK(c, hipEventRecord(c->ev_ops, c->xs));
    if (!hs.deferred.empty()) {
      // the deferred copies start behind everything enqueued so far on both caller streams and then run on the
      // library's own stream, beside the next steps: the link carries them in the direction the prefetches leave free
      HIPCHECK(c, hipStreamWaitEvent(c->ds, c->ev_ops_up, 0));
      size_t lo = 0;
      for (int l = 0; l < sh.L; ++l) {
        const size_t hi = hs.deferred_end[l];
        if (hi > lo) {
          HIPCHECK(c, launch_blit_narrow(c->d_lazy[lb] + lo, (int64_t)(hi - lo), pb, kDeferredCopyWorkgroups, c->ds));
          if ((c->lazy_x[l] || c->lazy_c[l]) && hs.plain_pending[l]) {  // copies of an earlier plan load, into a block
            // that is no longer read in place, that a stream has not waited for yet
            std::swap(c->ev_lazy[l], c->ev_lazy_prev[l]);
            c->prev_x[l] |= c->lazy_x[l];
            c->prev_c[l] |= c->lazy_c[l];
          }
          HIPCHECK(c, hipEventRecord(c->ev_lazy[l], c->ds));
          c->lazy_x[l] = c->lazy_c[l] = 1;
        }
        lo = hi;
      }
      HIPCHECK(c, hipEventRecord(c->ev_lazy_all, c->ds));
      HIPCHECK(c, hipEventRecord(c->ev_lazy_buf[lb], c->ds));
      c->lazy_buf = lb;
      c->lazy_outstanding = true;
    }
  }
  HIPCHECK(c, hipEventRecord(c->ev_plan_x, c->xs));
  HIPCHECK(c, hipStreamWaitEvent(c->cs, c->ev_plan_x, 0));
  const size_t n_req = hs.reqs.size();
  if (n_req > 0) {
    const size_t nt = n_req * sh.L * sh.cap_pages;
    HIPCHECK(c, hipEventSynchronize(c->ev_tab));
    HIPCHECK(c, hipEventSynchronize(c->ev_tab_rows));
    std::memcpy(c->h_tab_pinned, hs.h_table.data(), nt * sizeof(int32_t));
    HIPCHECK(c, hipMemcpyAsync(c->d_table, c->h_tab_pinned, nt * sizeof(int32_t), hipMemcpyHostToDevice, c->cs));
    HIPCHECK(c, hipEventRecord(c->ev_tab, c->cs));
  }
  return ORBIT_OK;
}

}  // namespace

extern "C" {

const char *orbit_last_error(orbit_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int orbit_plan_check(int32_t n_req, int32_t n_layers, int32_t page_tokens, const int32_t *ctx_len,
                     const uint8_t *placement_bitmap, int32_t prefetch_slots, int32_t decode_window, int64_t *out4) try {
  if (n_req < 0 || n_layers < 1 || page_tokens < 1 || prefetch_slots < 0 || decode_window < 0 || !out4) return ORBIT_E_INVAL;
  if (n_req > 0 && (!ctx_len || !placement_bitmap)) return ORBIT_E_INVAL;
  std::vector<int64_t> b(n_req);
  std::vector<uint8_t> x((size_t)n_req * n_layers);
  for (int r = 0; r < n_req; ++r) {
    if (ctx_len[r] < 0) return ORBIT_E_INVAL;
    b[r] = ceil_div((int64_t)ctx_len[r] + decode_window, page_tokens);
    for (int l = 0; l < n_layers; ++l) x[(size_t)r * n_layers + l] = bitmap_get(placement_bitmap, n_layers, r, l);
  }
  Eq1 e = eq1_eval(n_req, n_layers, b, x);
  out4[0] = e.resident;
  out4[1] = e.buffer;
  out4[2] = e.resident + (int64_t)prefetch_slots * e.buffer;
  out4[3] = e.host;
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

int orbit_deposit_create(double slo_interval, orbit_deposit **out) try {
  if (!out || !(slo_interval > 0.0)) return ORBIT_E_INVAL;
  *out = new orbit_deposit();
  (*out)->d.slo = slo_interval;
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}
int orbit_deposit_destroy(orbit_deposit *d) {
  if (!d) return ORBIT_E_INVAL;
  delete d;
  return ORBIT_OK;
}
int orbit_deposit_push(orbit_deposit *d, int32_t token, double now) try {
  if (!d) return ORBIT_E_INVAL;
  if (d->d.finished) return ORBIT_E_STATE;
  if (!d->d.gen.empty() && now < d->d.gen.back()) return ORBIT_E_INVAL;
  d->d.push(token, now);
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}
int orbit_deposit_finish(orbit_deposit *d, double now) try {
  if (!d) return ORBIT_E_INVAL;
  d->d.finished = true;
  d->d.finish_time = now;
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}
int64_t orbit_deposit_release(orbit_deposit *d, double now, int32_t *tokens_out, double *times_out, int64_t cap) try {
  if (!d || cap < 0 || (cap > 0 && (!tokens_out || !times_out))) return ORBIT_E_INVAL;
  int64_t n = 0;
  while (n < cap && d->d.pop_due(now, tokens_out + n, times_out + n)) ++n;
  return n;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}
int orbit_deposit_stats(orbit_deposit *d, int64_t *out4) try {
  if (!d || !out4) return ORBIT_E_INVAL;
  out4[0] = (int64_t)d->d.tok.size();
  out4[1] = d->d.delivered;
  out4[2] = d->d.visible_violations;
  out4[3] = d->d.max_size;
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}
int orbit_slo_replay(const double *step_latency, int64_t n_steps, double slo_interval, int32_t finish_at_end,
                     orbit_slo_report *out) try {
  if (!out || n_steps < 0 || (n_steps > 0 && !step_latency) || !(slo_interval > 0.0)) return ORBIT_E_INVAL;
  for (int64_t k = 0; k < n_steps; ++k)
    if (!(step_latency[k] >= 0.0)) return ORBIT_E_INVAL;
  const SloReport r = slo_replay(step_latency, n_steps, slo_interval, finish_at_end != 0);
  out->tokens = r.tokens;
  out->backend_violations = r.backend_violations;
  out->visible_violations = r.visible_violations;
  out->max_deposit = r.max_deposit;
  out->tpot = r.tpot;
  out->max_visible_gap = r.max_visible_gap;
  out->tpot_violated = r.tpot_violated ? 1 : 0;
  out->reserved_ = 0;
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

int orbit_profile_mismatch(double predicted, double observed, double fraction) {
  return profile_mismatch(predicted, observed, fraction) ? 1 : 0;
}
int orbit_profile_ewma(double *profile, const double *observed, int64_t n, double weight) try {
  if (n < 0 || (n > 0 && (!profile || !observed)) || !(weight >= 0.0 && weight <= 1.0)) return ORBIT_E_INVAL;
  profile_ewma(profile, observed, n, weight);
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

int orbit_distance_options(int32_t n_layers, int32_t *counts_out, int32_t cap) try {
  if (n_layers < 1 || n_layers > ORBIT_MAX_LAYERS) return ORBIT_E_INVAL;
  std::vector<int> v = distance_counts(n_layers);
  if (counts_out)
    for (int i = 0; i < (int)v.size() && i < cap; ++i) counts_out[i] = v[i];
  return (int)v.size();
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

int orbit_distance_pattern(int32_t n_layers, int32_t offload_count, uint8_t *row_out) try {
  if (n_layers < 1 || n_layers > ORBIT_MAX_LAYERS || offload_count < 0 || offload_count > n_layers || !row_out)
    return ORBIT_E_INVAL;
  std::vector<uint8_t> x(n_layers);
  if (!distance_pattern(n_layers, offload_count, x.data())) return ORBIT_E_INVAL;  // not a floor(L/k)
  for (int i = 0; i < (n_layers + 7) / 8; ++i) row_out[i] = 0;
  for (int l = 0; l < n_layers; ++l)
    if (x[l]) row_out[l / 8] |= (uint8_t)(1u << (l % 8));
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

static bool planner_args_ok(int32_t n_req, int32_t n_layers, const int64_t *blocks, double bw, const double *comp) {
  if (n_req < 0 || n_req > ORBIT_MAX_REQUESTS || n_layers < 1 || n_layers > ORBIT_MAX_LAYERS || !comp) return false;
  if (!(bw > 0.0) || (n_req > 0 && !blocks)) return false;
  for (int r = 0; r < n_req; ++r)
    if (blocks[r] < 0) return false;
  for (int l = 0; l < n_layers; ++l)
    if (!(comp[l] >= 0.0)) return false;
  return true;
}

int orbit_model_latency(int32_t n_req, int32_t n_layers, const int64_t *blocks, const uint8_t *placement_bitmap,
                        double blocks_per_time, const double *comp, double *stall_out, double *t_batch) try {
  if (!planner_args_ok(n_req, n_layers, blocks, blocks_per_time, comp) || !t_batch) return ORBIT_E_INVAL;
  if (n_req > 0 && !placement_bitmap) return ORBIT_E_INVAL;
  std::vector<uint8_t> x((size_t)n_req * n_layers);
  for (int r = 0; r < n_req; ++r)
    for (int l = 0; l < n_layers; ++l) x[(size_t)r * n_layers + l] = bitmap_get(placement_bitmap, n_layers, r, l);
  *t_batch = simulate_prefetch(n_req, n_layers, x.data(), blocks, blocks_per_time, comp, stall_out);
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

static int plan_search_entry(bool stagger, int32_t n_req, int32_t n_layers, const int64_t *blocks, int64_t gpu_blocks, int32_t prefetch_slots,
                      double blocks_per_time, const double *comp, int64_t max_evals, uint8_t *bitmap_out,
                      double *t_batch, int64_t *evals_out) {
  if (!planner_args_ok(n_req, n_layers, blocks, blocks_per_time, comp) || prefetch_slots < 1 || gpu_blocks < 0 ||
      max_evals < 1 || !t_batch || (n_req > 0 && !bitmap_out))
    return ORBIT_E_INVAL;
  SearchResult res = plan_search(n_req, n_layers, blocks, gpu_blocks, prefetch_slots, blocks_per_time, comp, max_evals, stagger);
  if (evals_out) *evals_out = res.evals;
  if (!(res.t < std::numeric_limits<double>::infinity())) return ORBIT_E_CAPACITY;
  *t_batch = res.t;
  const int bpr = (n_layers + 7) / 8;
  for (int i = 0; i < n_req * bpr; ++i) bitmap_out[i] = 0;
  for (int r = 0; r < n_req; ++r)
    for (int l = 0; l < n_layers; ++l)
      if (res.x[(size_t)r * n_layers + l]) bitmap_out[r * bpr + l / 8] |= (uint8_t)(1u << (l % 8));
  return ORBIT_OK;
}

int orbit_plan_search(int32_t n_req, int32_t n_layers, const int64_t *blocks, int64_t gpu_blocks, int32_t prefetch_slots,
                      double blocks_per_time, const double *comp, int64_t max_evals, uint8_t *bitmap_out,
                      double *t_batch, int64_t *evals_out) try {
  return plan_search_entry(false, n_req, n_layers, blocks, gpu_blocks, prefetch_slots, blocks_per_time, comp, max_evals,
                           bitmap_out, t_batch, evals_out);
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

int orbit_plan_search_staggered(int32_t n_req, int32_t n_layers, const int64_t *blocks, int64_t gpu_blocks,
                                int32_t prefetch_slots, double blocks_per_time, const double *comp, int64_t max_evals,
                                uint8_t *bitmap_out, double *t_batch, int64_t *evals_out) try {
  return plan_search_entry(true, n_req, n_layers, blocks, gpu_blocks, prefetch_slots, blocks_per_time, comp, max_evals,
                           bitmap_out, t_batch, evals_out);
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

int orbit_plan_search_or_pause(int32_t n_req, int32_t n_layers, const int64_t *blocks, const int64_t *deposited_tokens,
                               int64_t gpu_blocks, int32_t prefetch_slots, double blocks_per_time, const double *comp,
                               int64_t max_evals, int32_t flags, uint8_t *bitmap_out, uint8_t *paused_out, double *t_batch) try {
  if (!planner_args_ok(n_req, n_layers, blocks, blocks_per_time, comp) || prefetch_slots < 1 || gpu_blocks < 0 ||
      max_evals < 1 || !t_batch || (flags & ~ORBIT_SEARCH_STAGGER) || (n_req > 0 && (!bitmap_out || !paused_out || !deposited_tokens)))
    return ORBIT_E_INVAL;
  for (int r = 0; r < n_req; ++r)
    if (deposited_tokens[r] < 0) return ORBIT_E_INVAL;
  FallbackResult fr = plan_search_or_pause(n_req, n_layers, blocks, deposited_tokens, gpu_blocks, prefetch_slots,
                                           blocks_per_time, comp, max_evals, (flags & ORBIT_SEARCH_STAGGER) != 0);
  *t_batch = fr.res.t;
  const int bpr = (n_layers + 7) / 8;
  for (int i = 0; i < n_req * bpr; ++i) bitmap_out[i] = 0;
  for (int r = 0; r < n_req; ++r) {
    paused_out[r] = fr.paused[r];
    for (int l = 0; l < n_layers; ++l)
      if (fr.res.x[(size_t)r * n_layers + l]) bitmap_out[r * bpr + l / 8] |= (uint8_t)(1u << (l % 8));
  }
  return fr.n_paused;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

int orbit_planner_create(orbit_planner **out) try {
  if (!out) return ORBIT_E_INVAL;
  *out = new orbit_planner();
  return ORBIT_OK;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}
int orbit_planner_destroy(orbit_planner *p) {
  if (!p) return ORBIT_E_INVAL;
  delete p;
  return ORBIT_OK;
}
int64_t orbit_planner_submit(orbit_planner *p, int32_t n_req, int32_t n_layers, const int64_t *blocks, int64_t gpu_blocks,
                             int32_t prefetch_slots, double blocks_per_time, const double *comp, int64_t max_evals,
                             int32_t flags) try {
  if (!p || !planner_args_ok(n_req, n_layers, blocks, blocks_per_time, comp) || prefetch_slots < 1 || gpu_blocks < 0 ||
      max_evals < 1 || (flags & ~ORBIT_SEARCH_STAGGER))
    return ORBIT_E_INVAL;
  PlanJob j;
  j.n_req = n_req;
  j.L = n_layers;
  j.slots = prefetch_slots;
  j.gpu_blocks = gpu_blocks;
  j.max_evals = max_evals;
  j.bandwidth = blocks_per_time;
  j.stagger = (flags & ORBIT_SEARCH_STAGGER) != 0;
  j.blocks.assign(blocks, blocks + n_req);
  j.comp.assign(comp, comp + n_layers);
  return p->a.submit(std::move(j));
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}
int orbit_planner_poll(orbit_planner *p, int32_t wait, int64_t *ticket_out, uint8_t *bitmap_out, int64_t bitmap_cap,
                       double *t_batch, int64_t *evals_out) try {
  if (!p) return ORBIT_E_INVAL;
  PlanDone fresh;
  if (p->a.poll(wait != 0, fresh)) {  // a newer result supersedes one the caller could not take
    p->held = std::move(fresh);
    p->has_held = true;
  }
  if (!p->has_held) return 0;
  const PlanDone &d = p->held;
  if (ticket_out) *ticket_out = d.ticket;
  if (evals_out) *evals_out = d.res.evals;
  if (!(d.res.t < std::numeric_limits<double>::infinity())) {
    p->has_held = false;
    return ORBIT_E_CAPACITY;
  }
  const int bpr = (d.L + 7) / 8;
  if ((int64_t)d.n_req * bpr > bitmap_cap || (d.n_req > 0 && !bitmap_out)) return ORBIT_E_INVAL;
  if (t_batch) *t_batch = d.res.t;
  for (int i = 0; i < d.n_req * bpr; ++i) bitmap_out[i] = 0;
  for (int r = 0; r < d.n_req; ++r)
    for (int l = 0; l < d.L; ++l)
      if (d.res.x[(size_t)r * d.L + l]) bitmap_out[r * bpr + l / 8] |= (uint8_t)(1u << (l % 8));
  p->has_held = false;
  return 1;
} catch (const std::exception &) {
  return ORBIT_E_NOMEM;
}

int orbit_create(const orbit_config *cfg, orbit_ctx **out) try {
  auto bad = [&](const char *m) {
    g_create_error = m;
    return ORBIT_E_INVAL;
  };
  if (!cfg || !out) return bad("null argument");
  *out = nullptr;
  if (cfg->n_layers < 1 || cfg->n_layers > ORBIT_MAX_LAYERS) return bad("n_layers out of range");
  if (cfg->head_dim != 128) return bad("head_dim must be 128");
  if (cfg->page_tokens != 16) return bad("page_tokens must be 16");
  if (cfg->n_kv_heads < 1 || cfg->n_q_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads) return bad("bad head counts");
  if (cfg->n_q_heads / cfg->n_kv_heads > 16) return bad("more than 16 query heads per kv head");
  if (cfg->n_kv_heads > 128) return bad("more than 128 kv heads");
  if (cfg->max_requests < 1 || cfg->max_requests > ORBIT_MAX_REQUESTS) return bad("max_requests out of range");
  if (cfg->max_tokens_per_request < 1 || cfg->max_tokens_per_request > (1 << 24)) return bad("max_tokens_per_request out of range");
  if (cfg->prefetch_slots < 1 || cfg->prefetch_slots > 16) return bad("prefetch_slots out of range");
  if (cfg->decode_window < 0) return bad("negative decode_window");
  const int ch = cfg->chunk_tokens;
  if (ch != 0 && (ch < 32 || ch % 32 || ch > 65536)) return bad("chunk_tokens must be 0 or a multiple of 32");
  const bool host_only = (cfg->flags & ORBIT_FLAG_HOST_ONLY) != 0;
  const bool zero_copy = (cfg->flags & ORBIT_FLAG_ZERO_COPY) != 0;
  if (cfg->flags & ~(ORBIT_FLAG_HOST_ONLY | ORBIT_FLAG_ZERO_COPY | ORBIT_FLAG_POISON_STAGING)) return bad("unknown flag");
  if (cfg->hbm_arena_bytes < 0 || cfg->host_arena_bytes < 0) return bad("negative arena size");
  if (!host_only) {
    if (!cfg->hbm_arena || ((uintptr_t)cfg->hbm_arena & 255)) return bad("hbm_arena must be a 256-byte aligned device pointer");
    if (cfg->host_arena_bytes > 0 && !cfg->host_arena) return bad("host_arena is NULL");
    if (cfg->compute_stream == cfg->copy_stream) return bad("compute_stream and copy_stream must differ");
  }

  std::unique_ptr<orbit_ctx> c(new orbit_ctx());
  c->cfg = *cfg;
  c->host_only = host_only;
  Shape sh;
  sh.L = cfg->n_layers;
  sh.Hq = cfg->n_q_heads;
  sh.Hkv = cfg->n_kv_heads;
  sh.G = sh.Hq / sh.Hkv;
  sh.D = 128;
  sh.P = 16;
  sh.max_req = cfg->max_requests;
  sh.max_tokens = cfg->max_tokens_per_request;
  sh.page_bytes = (int64_t)2 * sh.Hkv * sh.P * sh.D * 2;
  sh.cap_pages = (int)((ceil_div(sh.max_tokens, sh.P) + 1) & ~(int64_t)1);
  sh.chunk_tokens = ch;
  sh.window = cfg->decode_window;
  sh.slots = cfg->prefetch_slots;
  sh.zero_copy = zero_copy;
  const int64_t arena_pages = cfg->hbm_arena_bytes / sh.page_bytes;
  if (arena_pages > 0x7FFFFFF0) return bad("hbm arena has too many pages");
  if (cfg->host_arena_bytes / sh.page_bytes > 0x7FFFFFF0) return bad("host arena has too many pages");
  if (ch && (int64_t)sh.max_req * ceil_div(sh.max_tokens, ch) * sh.Hkv > 0x7FFFFFF0 / 2)
    return bad("max_requests x max_tokens_per_request / chunk_tokens x n_kv_heads exceeds 2^30 work items");
  if ((int64_t)sh.max_req * sh.L * sh.cap_pages > ((int64_t)1 << 34))
    return bad("page table (max_requests x n_layers x blocks per request) would exceed 2^34 entries");
  c->hs.init(sh, arena_pages, cfg->host_arena_bytes / sh.page_bytes);
  c->host_dirty.assign(sh.L, 0);
  c->lazy_x.assign(sh.L, 0);
  c->lazy_c.assign(sh.L, 0);
  c->prev_x.assign(sh.L, 0);
  c->prev_c.assign(sh.L, 0);
  c->settle_full.assign(sh.L, 0);
  c->hs.live.reserve(sh.L + 1);
  c->items_key_tmp.reserve(sh.max_req + 1);
  c->flipped_tmp.reserve(sh.max_req);
  c->items_key.reserve(sh.max_req + 1);
  c->copy_timed.assign(sh.L, 0);
  c->copy_bytes.assign(sh.L, 0);
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)sh.D);
  c->scale_log2 = (float)((double)scale * 1.4426950408889634);
  if (!host_only) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      c->hs.n_cu = cus;
  }
  c->seg_cap = c->hs.max_segments();
  c->slots = c->seg_cap * sh.Hkv;
  const size_t items_words = (size_t)(c->seg_cap + 8) * 4;
  if (!host_only) {  // storage of the work-list builder, so that attention calls do not touch the heap
    c->items_tmp.reserve((size_t)c->seg_cap * 4);
    c->hs.work_order.reserve((size_t)c->seg_cap + 8);
    c->hs.work_sort_.reserve((size_t)c->seg_cap);
    c->hs.work_seg_base.reserve(sh.max_req);
    c->hs.work_n_parts.reserve(sh.max_req);
  }

  if (!host_only) {
    orbit_ctx *p = c.get();
    auto hipbad = [&](hipError_t e, const char *what) {  // releases what was created so far
      g_create_error = std::string(what) + ": " + hipGetErrorString(e);
      orbit_destroy(c.release());
      return ORBIT_E_HIP;
    };
#define CREATE_CHECK(x)                                \
  do {                                                 \
    hipError_t e_ = (x);                               \
    if (e_ != hipSuccess) return hipbad(e_, #x);       \
  } while (0)
    p->cs = (hipStream_t)cfg->compute_stream;
    p->xs = (hipStream_t)cfg->copy_stream;
    p->arena = (uint8_t *)cfg->hbm_arena;
    if (cfg->host_arena_bytes > 0) {
      void *dp = nullptr;
      CREATE_CHECK(hipHostGetDevicePointer(&dp, cfg->host_arena, 0));
      p->host_dev = (uint8_t *)dp;
    }
    {
      void *sp = nullptr;
      CREATE_CHECK(static_scratch_for_current_device(&sp));
      p->static_scratch = (uint8_t *)sp;
    }
    CREATE_CHECK(hipMalloc((void **)&p->d_table, c->hs.h_table.size() * sizeof(int32_t)));
    CREATE_CHECK(hipMalloc((void **)&p->d_items, items_words * sizeof(int32_t)));
    CREATE_CHECK(hipMalloc((void **)&p->d_pacc, (size_t)c->slots * sh.G * 128 * sizeof(float)));
    CREATE_CHECK(hipMalloc((void **)&p->d_pml, (size_t)c->slots * 32 * sizeof(float)));
    CREATE_CHECK(hipMemset(p->d_table, 0, c->hs.h_table.size() * sizeof(int32_t)));
    for (int b = 0; b < kItemBufs; ++b) {
      CREATE_CHECK(hipHostMalloc((void **)&p->h_items_pinned[b], items_words * sizeof(int32_t), hipHostMallocDefault));
      CREATE_CHECK(hipEventCreateWithFlags(&p->ev_items[b], hipEventDisableTiming));
    }
    CREATE_CHECK(hipHostMalloc((void **)&p->h_tab_pinned, c->hs.h_table.size() * sizeof(int32_t), hipHostMallocDefault));
    CREATE_CHECK(hipEventCreateWithFlags(&p->ev_ops, hipEventDisableTiming));
    CREATE_CHECK(hipEventCreateWithFlags(&p->ev_tab, hipEventDisableTiming));
    CREATE_CHECK(hipEventCreateWithFlags(&p->ev_tab_rows, hipEventDisableTiming));
    CREATE_CHECK(hipEventCreateWithFlags(&p->ev_plan_c, hipEventDisableTiming));
    CREATE_CHECK(hipEventCreateWithFlags(&p->ev_plan_x, hipEventDisableTiming));
    CREATE_CHECK(hipEventCreateWithFlags(&p->ev_tmp, hipEventDisableTiming));
    CREATE_CHECK(hipEventCreateWithFlags(&p->ev_ops_up, hipEventDisableTiming));
    CREATE_CHECK(hipEventCreateWithFlags(&p->ev_lazy_all, hipEventDisableTiming));
    for (int b = 0; b < 2; ++b) CREATE_CHECK(hipEventCreateWithFlags(&p->ev_lazy_buf[b], hipEventDisableTiming));
    CREATE_CHECK(hipStreamCreateWithFlags(&p->ds, hipStreamNonBlocking));  // default priority, as the caller's streams
    CREATE_CHECK(hipEventCreate(&p->t_step0));
    CREATE_CHECK(hipEventCreate(&p->t_step1));
#undef CREATE_CHECK
    int rc = 0;
    if ((rc = make_events(p, p->ev_ready, sh.L, false)) || (rc = make_events(p, p->ev_done, sh.L, false)) ||
        (rc = make_events(p, p->ev_lazy, sh.L, false)) || (rc = make_events(p, p->ev_lazy_prev, sh.L, false)) ||
        (rc = make_events(p, p->t_wait0, sh.L, true)) || (rc = make_events(p, p->t_wait1, sh.L, true)) ||
        (rc = make_events(p, p->t_attn0, sh.L, true)) || (rc = make_events(p, p->t_attn1, sh.L, true)) ||
        (rc = make_events(p, p->t_comb1, sh.L, true)) || (rc = make_events(p, p->t_copy0, sh.L, true)) ||
        (rc = make_events(p, p->t_copy1, sh.L, true))) {
      g_create_error = p->err;
      orbit_destroy(c.release());
      return rc;
    }
  }
  *out = c.release();
  return ORBIT_OK;
} catch (const std::exception &e) {
  g_create_error = std::string("host allocation failed: ") + e.what();
  return ORBIT_E_NOMEM;
}

int orbit_destroy(orbit_ctx *c) {
  if (!c) return ORBIT_E_INVAL;
  if (!c->host_only) {
    if (c->cs || c->xs) {
      (void)hipStreamSynchronize(c->cs);
      (void)hipStreamSynchronize(c->xs);
    }
    if (c->ds) {
      (void)hipStreamSynchronize(c->ds);
      (void)hipStreamDestroy(c->ds);
    }
    (void)hipFree(c->d_table);
    (void)hipFree(c->d_items);
    (void)hipFree(c->d_pacc);
    (void)hipFree(c->d_pml);
    (void)hipFree(c->d_ops);
    for (int b = 0; b < 2; ++b) {
      (void)hipFree(c->d_lazy[b]);
      if (c->ev_lazy_buf[b]) (void)hipEventDestroy(c->ev_lazy_buf[b]);
    }
    if (c->h_ops_pinned) (void)hipHostFree(c->h_ops_pinned);
    if (c->h_tab_pinned) (void)hipHostFree(c->h_tab_pinned);
    for (hipEvent_t e : {c->ev_ops, c->ev_tab, c->ev_tab_rows, c->ev_plan_c, c->ev_plan_x, c->ev_ops_up, c->ev_lazy_all})
      if (e) (void)hipEventDestroy(e);
    for (int b = 0; b < kItemBufs; ++b) {
      if (c->h_items_pinned[b]) (void)hipHostFree(c->h_items_pinned[b]);
      if (c->ev_items[b]) (void)hipEventDestroy(c->ev_items[b]);
    }
    if (c->ev_tmp) (void)hipEventDestroy(c->ev_tmp);
    if (c->t_step0) (void)hipEventDestroy(c->t_step0);
    if (c->t_step1) (void)hipEventDestroy(c->t_step1);
    drop_events(c->ev_ready);
    drop_events(c->ev_done);
    drop_events(c->ev_lazy);
    drop_events(c->ev_lazy_prev);
    drop_events(c->t_wait0);
    drop_events(c->t_wait1);
    drop_events(c->t_attn0);
    drop_events(c->t_attn1);
    drop_events(c->t_comb1);
    drop_events(c->t_copy0);
    drop_events(c->t_copy1);
  }
  delete c;
  return ORBIT_OK;
}

int orbit_plan_load(orbit_ctx *c, int32_t n_req, const int64_t *req_ids, const int32_t *ctx_len,
                    const uint8_t *placement_bitmap, int64_t hbm_budget_bytes) try {
  if (!c) return ORBIT_E_INVAL;
  for (auto &lb : c->hs.live)
    if (!lb.consumed) return set_err(c, ORBIT_E_STATE, "a prefetched layer was never attended; finish it before a new plan");
  std::vector<std::vector<PageOp>> phases;
  if (int rr = retire_deferred(c)) return rr;
  int rc = c->hs.plan_load(n_req, req_ids, ctx_len, placement_bitmap, hbm_budget_bytes, phases);
  if (rc) return set_err(c, rc, c->hs.err);
  c->items_valid = false;
  std::fill(c->host_dirty.begin(), c->host_dirty.end(), 0);
  return apply_plan_gpu(c, phases);
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_request_pause(orbit_ctx *c, int64_t req_id) try {
  if (!c) return ORBIT_E_INVAL;
  if (!c->hs.has_plan) return set_err(c, ORBIT_E_STATE, "no plan installed");
  for (auto &lb : c->hs.live)
    if (!lb.consumed) return set_err(c, ORBIT_E_STATE, "a prefetched layer was never attended; finish it before pausing");
  std::vector<std::vector<PageOp>> phases;
  if (int rr = retire_deferred(c)) return rr;
  int rc = c->hs.pause(req_id, phases);
  if (rc) return set_err(c, rc, c->hs.err);
  c->items_valid = false;
  std::fill(c->host_dirty.begin(), c->host_dirty.end(), 0);
  return apply_plan_gpu(c, phases);
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_request_drop(orbit_ctx *c, int64_t req_id) try {
  if (!c) return ORBIT_E_INVAL;
  int rc = c->hs.drop_paused(req_id);
  return rc ? set_err(c, rc, c->hs.err) : ORBIT_OK;
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_get_plan_info(orbit_ctx *c, orbit_plan_info *out) try {
  if (!c || !out) return ORBIT_E_INVAL;
  if (!c->hs.has_plan) return set_err(c, ORBIT_E_STATE, "no plan installed");
  *out = c->hs.info;
  return ORBIT_OK;
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

static int fill_or_read(orbit_ctx *c, bool write, int64_t req_id, int32_t layer, int64_t first, int64_t n, void *k, void *v) {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  const int r = c->hs.find(req_id);
  if (r < 0) return set_err(c, ORBIT_E_NOT_FOUND, "unknown request id");
  LayerKV &lk = c->hs.reqs[r].layers[layer];
  if (first < 0 || n < 0 || first + n > lk.len) return set_err(c, ORBIT_E_INVAL, "token range outside the stored length");
  if (n == 0) return ORBIT_OK;
  if (!k || !v) return set_err(c, ORBIT_E_INVAL, "null argument");
  if (!lk.dual_pages.empty() && (rc = flip_in_place_blocks(c, layer, true))) return rc;  // the host copy itself is wanted
  if (write && lk.tier == 0) {
    LiveBlock *lb = find_live(c, layer);
    if (lb && !lb->consumed) return set_err(c, ORBIT_E_STATE, "layer is prefetched; attend it before rewriting its host blocks");
    c->host_dirty[layer] = 1;
  }
  if (c->host_only) return ORBIT_OK;
  if (lk.tier == 0 && (rc = wait_deferred(c, layer, false))) return rc;
  const Shape &sh = c->hs.sh;
  FillParams fp{};
  fp.arena = c->arena;
  if (lk.tier == 1) fp.row = c->d_table + ((int64_t)r * sh.L + layer) * sh.cap_pages;
  else fp.host_run = c->host_dev + lk.host_page0 * sh.page_bytes;
  fp.k = (uint16_t *)k;
  fp.v = (uint16_t *)v;
  fp.page_bytes = sh.page_bytes;
  fp.first_token = first;
  fp.n_tokens = n;
  fp.Hkv = sh.Hkv;
  HIPCHECK(c, write ? launch_fill(fp, c->cs) : launch_gather(fp, c->cs));
  return ORBIT_OK;
}

int orbit_kv_fill(orbit_ctx *c, int64_t req_id, int32_t layer, int64_t first_token, int64_t n_tokens, const void *k,
                  const void *v) try {
  return fill_or_read(c, true, req_id, layer, first_token, n_tokens, (void *)k, (void *)v);
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_kv_read(orbit_ctx *c, int64_t req_id, int32_t layer, int64_t first_token, int64_t n_tokens, void *k_out,
                  void *v_out) try {
  return fill_or_read(c, false, req_id, layer, first_token, n_tokens, k_out, v_out);
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

// Bookkeeping of one appended token; returns the kernel item.
static int append_item(orbit_ctx *c, int r, int layer, AppendItem &item) {
  HostState &hs = c->hs;
  LayerKV &lk = hs.reqs[r].layers[layer];
  const int64_t pi = lk.len / hs.sh.P;
  if (pi >= hs.reqs[r].reserved)
    return set_err(c, ORBIT_E_STATE, "decode window used up: the request needs a block the plan did not reserve");
  item.tok = lk.len;
  if (lk.tier == 1) {
    item.page = lk.pages[pi];
    item.host_page = 0;
  } else {
    LiveBlock *lb = find_live(c, layer);
    item.page = (lb && !lb->consumed) ? (int32_t)(lk.stage_page0 + pi) : -1;  // live staging copy gets the token too
    item.host_page = c->host_only ? 1 : (uint64_t)(uintptr_t)(c->host_dev + (lk.host_page0 + pi) * hs.sh.page_bytes);
  }
  lk.len += 1;
  return ORBIT_OK;
}

// An append into a layer whose prefetch is in flight also writes the staging copy: the compute
// stream must first see that copy landed, or the transfer could overwrite the new token.
static int wait_for_live_copy(orbit_ctx *c, int layer) {
  if (int rc = flip_in_place_blocks(c, layer, true)) return rc;  // this path writes host blocks and staging copies only
  if (int rc = wait_deferred(c, layer, false)) return rc;  // the append may write into a host block
  LiveBlock *lb = find_live(c, layer);
  if (lb && !lb->consumed && !c->host_only) HIPCHECK(c, hipStreamWaitEvent(c->cs, c->ev_ready[layer], 0));
  return ORBIT_OK;
}

// One token for every request of the plan, in plan order: k, v device [n_req][Hkv][D].
// mark_dirty: remember that host pages of this layer were written on the compute stream, so that the
// layer's next prefetch orders itself behind them.  orbit_step does not need the mark: there a
// staging range is refilled only after the layer that read it last has finished, and that layer
// was enqueued on the compute stream after this append.
static int append_layer(orbit_ctx *c, int l, const uint16_t *k, const uint16_t *v, bool mark_dirty) {
  HostState &hs = c->hs;
  const Shape &sh = hs.sh;
  const int nreq = (int)hs.reqs.size();
  int rc;
  for (int r0 = 0; r0 < nreq; r0 += kAppendBatch) {
    AppendParams ap{};
    const int n = std::min(kAppendBatch, nreq - r0);
    for (int i = 0; i < n; ++i) {
      if ((rc = append_item(c, r0 + i, l, ap.items[i]))) return rc;
      if (mark_dirty && hs.reqs[r0 + i].layers[l].tier == 0) c->host_dirty[l] = 1;
    }
    if (c->host_only) continue;
    ap.arena = c->arena;
    ap.k = k + (int64_t)r0 * sh.Hkv * sh.D;  // non-NULL here: host-only contexts left the loop above
    ap.v = v + (int64_t)r0 * sh.Hkv * sh.D;
    ap.page_bytes = sh.page_bytes;
    ap.Hkv = sh.Hkv;
    ap.n = n;
    HIPCHECK(c, launch_append(ap, c->cs));
  }
  return ORBIT_OK;
}

int orbit_kv_append_batch(orbit_ctx *c, int32_t layer, const void *k, const void *v) try {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  if (!c->host_only && (!k || !v)) return set_err(c, ORBIT_E_INVAL, "null argument");
  for (const Req &q : c->hs.reqs)  // all or nothing: checked before any length moves
    if (q.layers[layer].len / c->hs.sh.P >= q.reserved)
      return set_err(c, ORBIT_E_STATE, "decode window used up: a request needs a block the plan did not reserve");
  if ((rc = wait_for_live_copy(c, layer))) return rc;
  return append_layer(c, layer, (const uint16_t *)k, (const uint16_t *)v, true);
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_kv_append(orbit_ctx *c, int64_t req_id, int32_t layer, const void *k, const void *v) try {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  if (!k || !v) return set_err(c, ORBIT_E_INVAL, "null argument");
  const int r = c->hs.find(req_id);
  if (r < 0) return set_err(c, ORBIT_E_NOT_FOUND, "unknown request id");
  if ((rc = wait_for_live_copy(c, layer))) return rc;
  AppendParams ap{};
  if ((rc = append_item(c, r, layer, ap.items[0]))) return rc;
  if (c->hs.reqs[r].layers[layer].tier == 0) c->host_dirty[layer] = 1;
  if (c->host_only) return ORBIT_OK;
  const Shape &sh = c->hs.sh;
  ap.arena = c->arena;
  ap.k = (const uint16_t *)k;
  ap.v = (const uint16_t *)v;
  ap.page_bytes = sh.page_bytes;
  ap.Hkv = sh.Hkv;
  ap.n = 1;
  HIPCHECK(c, launch_append(ap, c->cs));
  return ORBIT_OK;
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_kv_prefetch(orbit_ctx *c, int32_t layer) try {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  rc = prefetch_impl(c, layer);
  if (rc == 1) return set_err(c, ORBIT_E_STATE, "staging range still needed by a prefetched layer not yet attended");
  return rc;
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_decode_attention(orbit_ctx *c, int32_t layer, const void *q, void *out, float *out_f32) try {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  if (c->hs.reqs.empty()) return set_err(c, ORBIT_E_STATE, "the plan has no request");
  if (!c->host_only && (!q || !out)) return set_err(c, ORBIT_E_INVAL, "null argument");
  c->timing = false;
  return attention_impl(c, layer, q, out, out_f32, false);
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_decode_layer(orbit_ctx *c, int32_t layer, const void *q, const void *k_new, const void *v_new, void *out,
                       float *out_f32) try {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  HostState &hs = c->hs;
  if (hs.reqs.empty()) return set_err(c, ORBIT_E_STATE, "the plan has no request");
  if (!c->host_only && (!q || !k_new || !v_new || !out)) return set_err(c, ORBIT_E_INVAL, "null argument");
  for (const Req &rq : hs.reqs)  // all or nothing: checked before any length moves
    if (rq.layers[layer].len / hs.sh.P >= rq.reserved)
      return set_err(c, ORBIT_E_STATE, "decode window used up: a request needs a block the plan did not reserve");
  c->timing = false;
  const bool staged = hs.block_of_layer[layer] >= 0;
  if (staged) {  // the layer's copies are issued over the lengths before the new token, which the launch itself adds
    LiveBlock *lb = find_live(c, layer);
    if (!lb || lb->consumed) {
      rc = prefetch_impl(c, layer);
      if (rc == 1) return set_err(c, ORBIT_E_STATE, "staging range still needed by a prefetched layer not yet attended");
      if (rc) return rc;
    }
    if (!c->host_only) HIPCHECK(c, hipStreamWaitEvent(c->cs, c->ev_ready[layer], 0));
  }
  for (Req &rq : hs.reqs) rq.layers[layer].len += 1;
  if (staged) find_live(c, layer)->consumed = true;
  return attention_impl(c, layer, q, out, out_f32, true, (const uint16_t *)k_new, (const uint16_t *)v_new);
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_decode_attention_static(orbit_ctx *c, int32_t layer, const void *q, void *out, float *out_f32) try {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  if (c->hs.reqs.empty()) return set_err(c, ORBIT_E_STATE, "the plan has no request");
  if (c->host_only) return set_err(c, ORBIT_E_STATE, "host-only context");
  if (!q || !out) return set_err(c, ORBIT_E_INVAL, "null argument");
  c->timing = false;
  return attention_impl(c, layer, q, out, out_f32, false, nullptr, nullptr, true);
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int orbit_step(orbit_ctx *c, const void *q, const void *k_new, const void *v_new, void *out, orbit_step_stats *stats) try {
  if (!c) return ORBIT_E_INVAL;
  HostState &hs = c->hs;
  if (!hs.has_plan || hs.reqs.empty()) return set_err(c, ORBIT_E_STATE, "no plan (or an empty one) installed");
  if (!c->host_only && (!q || !k_new || !v_new || !out)) return set_err(c, ORBIT_E_INVAL, "null argument");
  const Shape &sh = hs.sh;
  const int nreq = (int)hs.reqs.size();
  for (int r = 0; r < nreq; ++r)
    for (int l = 0; l < sh.L; ++l)
      if (hs.reqs[r].layers[l].len / sh.P >= hs.reqs[r].reserved)
        return set_err(c, ORBIT_E_STATE, "decode window used up: load a new plan before this step");
  for (auto &lb : hs.live)
    if (!lb.consumed) return set_err(c, ORBIT_E_STATE, "a prefetched layer was never attended; finish it before orbit_step");
  c->timing = stats != nullptr && !c->host_only;
  std::fill(c->copy_timed.begin(), c->copy_timed.end(), 0);
  std::fill(c->copy_bytes.begin(), c->copy_bytes.end(), 0);

  size_t next_pf = 0;
  auto pump = [&]() -> int {
    while (next_pf < hs.blocks.size()) {
      int rc = prefetch_impl(c, hs.blocks[next_pf].layer);
      if (rc == 1) break;
      if (rc) return rc;
      ++next_pf;
    }
    return ORBIT_OK;
  };
  int rc = pump();
  if (rc) return rc;
  if (c->timing) HIPCHECK(c, hipEventRecord(c->t_step0, c->cs));
  int64_t hbm_bytes = 0;
  const int64_t tok_bytes = sh.page_bytes / sh.P;
  const int64_t q_stride = (int64_t)nreq * sh.Hq * sh.D, kv_stride = (int64_t)nreq * sh.Hkv * sh.D;
  for (int l = 0; l < sh.L; ++l) {
    const int b = hs.block_of_layer[l];
    if (b >= 0) {
      LiveBlock *lb = find_live(c, l);
      if (!lb || lb->consumed) {
        if ((rc = pump())) return rc;
        lb = find_live(c, l);
        if (!lb || lb->consumed) return set_err(c, ORBIT_E_STATE, "internal: staging schedule cannot make progress");
      }
      if (!c->host_only) {
        if (c->timing) HIPCHECK(c, hipEventRecord(c->t_wait0[l], c->cs));
        HIPCHECK(c, hipStreamWaitEvent(c->cs, c->ev_ready[l], 0));
        if (c->timing) HIPCHECK(c, hipEventRecord(c->t_wait1[l], c->cs));
      }
    }
    // a3: this layer's new token of every request joins the cache inside the attention launch (the
    // workgroup that owns its position takes the row from k_new / v_new, attends to it and stores it: into the
    // resident page, or into the live staging copy and the host run); here only the lengths move
    for (int r = 0; r < nreq; ++r) {
      LayerKV &lk = hs.reqs[r].layers[l];
      lk.len += 1;
      if (lk.tier == 1 || !lk.dual_pages.empty()) hbm_bytes += (int64_t)lk.len * tok_bytes;
      else if (sh.zero_copy) c->copy_bytes[l] += ceil_div(lk.len, sh.P) * sh.page_bytes;  // read over the link by the kernel
    }
    if (b >= 0) find_live(c, l)->consumed = true;
    rc = attention_impl(c, l, q ? (const uint16_t *)q + l * q_stride : nullptr, out ? (uint16_t *)out + l * q_stride : nullptr,
                        nullptr, true, k_new ? (const uint16_t *)k_new + l * kv_stride : nullptr,
                        v_new ? (const uint16_t *)v_new + l * kv_stride : nullptr);
    if (rc) return rc;
    if (b >= 0 && (rc = pump())) return rc;
  }
  if (stats) {
    std::memset(stats, 0, sizeof(*stats));
    stats->hbm_kv_bytes = hbm_bytes;
    stats->hbm_blocks_budget = hs.info.budget_blocks;
    stats->hbm_blocks_reserved = hs.info.resident_blocks + hs.info.staging_blocks;
    for (int l = 0; l < sh.L; ++l) {
      stats->link_bytes[l] = c->copy_bytes[l];
      stats->link_kv_bytes += c->copy_bytes[l];
    }
    if (c->timing) {
      HIPCHECK(c, hipEventRecord(c->t_step1, c->cs));
      HIPCHECK(c, hipEventSynchronize(c->t_step1));
      HIPCHECK(c, hipStreamSynchronize(c->xs));
      HIPCHECK(c, hipEventElapsedTime(&stats->step_ms, c->t_step0, c->t_step1));
      for (int l = 0; l < sh.L; ++l) {
        HIPCHECK(c, hipEventElapsedTime(&stats->attn_ms[l], c->t_attn0[l], c->t_attn1[l]));
        HIPCHECK(c, hipEventElapsedTime(&stats->combine_ms[l], c->t_attn1[l], c->t_comb1[l]));
        stats->attn_ms_total += stats->attn_ms[l];
        if (hs.block_of_layer[l] >= 0) {
          HIPCHECK(c, hipEventElapsedTime(&stats->stall_ms[l], c->t_wait0[l], c->t_wait1[l]));
          stats->stall_ms_total += stats->stall_ms[l];
          if (c->copy_timed[l]) {
            HIPCHECK(c, hipEventElapsedTime(&stats->copy_ms[l], c->t_copy0[l], c->t_copy1[l]));
            stats->copy_ms_total += stats->copy_ms[l];
          }
        }
      }
    }
  }
  c->timing = false;
  return ORBIT_OK;
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int64_t orbit_get_pages(orbit_ctx *c, int64_t req_id, int32_t layer, int32_t *tier, int64_t *host_first_page,
                        int32_t *length, int32_t *pages_out, int64_t cap) try {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  const int r = c->hs.find(req_id);
  const int pr = r < 0 ? c->hs.find_paused(req_id) : -1;
  if (r < 0 && pr < 0) return set_err(c, ORBIT_E_NOT_FOUND, "unknown request id");
  const Req &q = r >= 0 ? c->hs.reqs[r] : c->hs.paused[pr];
  const LayerKV &lk = q.layers[layer];
  const bool in_place = !lk.dual_pages.empty();
  if (tier) *tier = in_place ? 2 : lk.tier;
  if (host_first_page) *host_first_page = lk.tier == 0 ? lk.host_page0 : -1;
  if (length) *length = lk.len;
  const int64_t n = in_place ? (int64_t)lk.dual_pages.size()
                             : (lk.tier == 1 ? (int64_t)lk.pages.size() : (r >= 0 ? q.reserved : lk.host_cap));
  if (pages_out)
    for (int64_t i = 0; i < n && i < cap; ++i)
      pages_out[i] = in_place ? lk.dual_pages[i]
                              : (lk.tier == 1 ? lk.pages[i] : (r >= 0 && lk.stage_page0 >= 0 ? lk.stage_page0 + (int32_t)i : -1));
  return n;
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int64_t orbit_get_work_items(orbit_ctx *c, int32_t layer, int32_t *items_out, int64_t cap) try {
  int rc = check_layer(c, layer);
  if (rc) return rc;
  std::vector<int32_t> items;
  rc = c->hs.build_work_items(layer, items);
  c->items_valid = false;  // the builder's per-request state now describes this list, not the uploaded one
  if (rc) return set_err(c, rc, c->hs.err);
  const int64_t n = (int64_t)items.size() / 4;
  if (items_out)
    for (int64_t i = 0; i < n && i < cap; ++i) {
      const int64_t len = c->hs.reqs[items[4 * i]].layers[layer].len;
      items_out[4 * i] = items[4 * i];
      items_out[4 * i + 1] = items[4 * i + 1];
      items_out[4 * i + 2] = (int32_t)std::min<int64_t>(items[4 * i + 2], len - items[4 * i + 1]);  // the last chunk is ragged
      items_out[4 * i + 3] = items[4 * i + 3];
    }
  return n;
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

int64_t orbit_get_copy_schedule(orbit_ctx *c, int32_t *rows_out, int64_t cap) try {
  if (!c) return ORBIT_E_INVAL;
  if (!c->hs.has_plan) return set_err(c, ORBIT_E_STATE, "no plan installed");
  int64_t n = 0;
  for (const StageBlock &b : c->hs.blocks)
    for (const CopyItem &ci : b.copies) {
      if (rows_out && n < cap) {
        int32_t *row = rows_out + n * 5;
        row[0] = ci.layer;
        row[1] = ci.req;
        row[2] = ci.stage_page0;
        row[3] = ci.reserved;
        row[4] = b.p0 - (int32_t)c->hs.info.staging_first_page;
      }
      ++n;
    }
  return n;
} catch (const std::exception &e) {  // nothing may unwind through the C ABI
  return c ? set_err(c, ORBIT_E_NOMEM, std::string("host allocation failed: ") + e.what()) : ORBIT_E_NOMEM;
}

}  // extern "C"
