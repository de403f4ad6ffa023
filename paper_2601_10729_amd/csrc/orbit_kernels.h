// Launch wrappers of the gfx950 kernels (defined in orbit_kernels.hip).  Plain C++; every
// function only enqueues work on the given stream and returns the HIP status.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace orbit {

constexpr int kAppendBatch = 64;  // requests per append launch (items travel as kernel arguments)

constexpr int kMaxRequests = 256;  // = ORBIT_MAX_REQUESTS: per-request launch arguments travel by value

struct AttnReq {
  int32_t n_tok;            // tokens attended for this request in this layer (the appended one included)
  int32_t host_page0;       // append mode: first page of the (request, layer) run in the host arena that must
                            // receive the new token besides the page attention reads, or -1
  int32_t n_parts;          // segments this request's tokens were cut into
};

struct AttnParams {
  uint8_t *arena;           // device, page 0 of the HBM arena
  uint8_t *host;            // device-visible page 0 of the pinned host arena, or NULL
  const int32_t *table;     // device [max_req][L][cap_pages] page ids; a negative id i names host page ~i
  const int32_t *work;      // device [n_workers][4]: the segments in launch order, {request, first token (multiple
                            // of 32), tokens, segment index}; request -1 = padding
  const uint16_t *q;        // device [n_req][Hq][128] bf16
  float *pacc;              // device [n_segs * Hkv][G][128] un-normalised partial outputs; slot = segment * Hkv + kv head
  float *pml;               // device [n_segs * Hkv][2][16] partial (max, sum) in log2 units
  uint16_t *out;            // device [n_req][Hq][128] bf16: written here only for requests of a single segment
  float *out_f32;           // optional device [n_req][Hq][128] fp32
  const uint16_t *k_new;    // append mode: device [n_req][Hkv][128] bf16 rows of the token at position n_tok-1; else NULL
  const uint16_t *v_new;
  int64_t page_bytes;
  int32_t L, layer, cap_pages, Hq, Hkv, G;
  int32_t n_workers;        // multiple of 8; the grid is n_workers * Hkv workgroups
  float scale_log2;         // softmax scale * log2(e)
  AttnReq req[kMaxRequests];
};

struct CombineParams {
  const float *pacc;
  const float *pml;
  uint16_t *out;            // device [n_req][Hq][128] bf16
  float *out_f32;           // optional
  int32_t Hq, Hkv, G, n_req;
  int32_t seg_base[kMaxRequests];  // first segment of each request
  int32_t n_parts[kMaxRequests];   // its number of segments; requests of a single segment are skipped
};

struct AppendItem {
  int32_t tok;              // position the new token takes (= length before the append)
  int32_t page;             // arena page id to write (resident page or live staging page), or -1
  uint64_t host_page;       // device-visible address of the host page to write, or 0
};

struct AppendParams {
  uint8_t *arena;
  const uint16_t *k;        // device [.. n][Hkv][128] bf16, row i belongs to request r0 + i
  const uint16_t *v;
  int64_t page_bytes;
  int32_t Hkv, n;
  AppendItem items[kAppendBatch];
};

struct FillParams {
  uint8_t *arena;           // HBM arena (resident destination) ...
  const int32_t *row;       // ... through this device page-table row, or
  uint8_t *host_run;        // device-visible address of the host run's first page (row == NULL)
  uint16_t *k;              // token-major [n_tokens][Hkv][128] bf16 (source of fill, dest of read)
  uint16_t *v;
  int64_t page_bytes, first_token, n_tokens;
  int32_t Hkv;
};

struct BlitOp {
  uint64_t src, dst;        // device-visible addresses of one page each
};

hipError_t launch_attention(const AttnParams &p, hipStream_t s);
hipError_t launch_combine(const CombineParams &p, hipStream_t s);
hipError_t launch_append(const AppendParams &p, hipStream_t s);
hipError_t launch_fill(const FillParams &p, hipStream_t s);
hipError_t launch_gather(const FillParams &p, hipStream_t s);
hipError_t launch_blit(const BlitOp *ops_dev, int64_t n_ops, int64_t page_bytes, hipStream_t s);
hipError_t launch_poison(uint8_t *p, int64_t bytes, hipStream_t s);
hipError_t launch_blit_narrow(const BlitOp *ops_dev, int64_t n_ops, int64_t page_bytes, int workgroups, hipStream_t s);

}  // namespace orbit
