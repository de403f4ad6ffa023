/*
 * CPU oracle for batched GQA decode attention over a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP library is
 * checked against; the product never calls it.  It shares no code with the HIP path.
 *
 * What it computes (the paper only describes decode attention in prose, Section 2.1 and the
 * caption of Figure 1: one query token per request attends over that request's cached keys and
 * values; with grouped-query attention several query heads share one KV head).  The textbook
 * definition is written out, in float64, as two explicit passes:
 *
 *     s_t = scale * sum_d q[h][d] * k_t[g][d]           g = h / (Hq / Hkv)
 *     w_t = exp(s_t - max_t s_t) / sum_t exp(s_t - max_t s_t)
 *     o[h][:] = sum_t w_t * v_t[g][:]
 *
 * over exactly the ctx_len stored tokens (slots past ctx_len in the last block are excluded,
 * not zero-scored).  K and V are bf16 and are widened exactly; nothing is blocked, fused or
 * reordered.
 *
 * Paged layout (the KV cache is kept in fixed blocks of 16 tokens per layer, Section 2.3; the
 * per-layer caches are flattened into one arena addressed by a (request x layer) table,
 * Section 4).  One block ("page") holds, for every KV head, a K tile then a V tile, bf16:
 *
 *     page   = [K tile of head 0] ... [K tile of head Hkv-1] [V tile of head 0] ... [V tile Hkv-1]
 *     K tile : element (tok, dim) at  (dim/8)*(P*8) + tok*8 + dim%8
 *     V tile : element (tok, dim) at  ((((dim/32)*(P/4) + tok/4)*16 + dim%16)*2 + (dim/16)%2)*4 + tok%4
 *
 * with P tokens per page and D dims per head (D % 32 == 0, P % 4 == 0).  The paper's figure
 * of its own flattened layout is not available; this in-page order is this project's choice
 * and is restated here from its written definition, not from the library's source.
 *
 * Pinned by tests/test_oracle_pins.py (closed forms, invariants, dense long-double brute
 * force).
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline double bf16_to_f64(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static inline int64_t k_offset(int g, int tok, int dim, int P, int D) {
  return (int64_t)g * P * D + (int64_t)(dim / 8) * (P * 8) + (int64_t)tok * 8 + dim % 8;
}

static inline int64_t v_offset(int g, int tok, int dim, int P, int D, int Hkv) {
  int64_t in_tile = ((((int64_t)(dim / 32) * (P / 4) + tok / 4) * 16 + dim % 16) * 2 + (dim / 16) % 2) * 4 + tok % 4;
  return (int64_t)Hkv * P * D + (int64_t)g * P * D + in_tile;
}

static int shape_ok(int Hq, int Hkv, int D, int P) {
  return Hq > 0 && Hkv > 0 && Hq % Hkv == 0 && D > 0 && D % 32 == 0 && P > 0 && P % 4 == 0;
}

/* Write tokens [tok0, tok0+ntok) of one (request, layer), given token-major
 * k, v = [ntok][Hkv][D] bf16, into the arena through that request's page list. */
int oracle_pack_tokens(uint16_t *arena, int64_t arena_pages, const int32_t *pages, int64_t n_pages,
                       int Hkv, int D, int P, int64_t tok0, int64_t ntok,
                       const uint16_t *k, const uint16_t *v) {
  if (!shape_ok(Hkv, Hkv, D, P) || tok0 < 0 || ntok < 0) return -1;
  const int64_t page_elems = 2LL * Hkv * P * D;
  for (int64_t i = 0; i < ntok; ++i) {
    int64_t t = tok0 + i;
    if (t / P >= n_pages) return -2;
    int32_t pg = pages[t / P];
    if (pg < 0 || pg >= arena_pages) return -3;
    uint16_t *base = arena + (int64_t)pg * page_elems;
    for (int g = 0; g < Hkv; ++g)
      for (int d = 0; d < D; ++d) {
        base[k_offset(g, (int)(t % P), d, P, D)] = k[(i * Hkv + g) * D + d];
        base[v_offset(g, (int)(t % P), d, P, D, Hkv)] = v[(i * Hkv + g) * D + d];
      }
  }
  return 0;
}

/* The inverse gather: tokens [tok0, tok0+ntok) back to token-major k, v. */
int oracle_unpack_tokens(const uint16_t *arena, int64_t arena_pages, const int32_t *pages,
                         int64_t n_pages, int Hkv, int D, int P, int64_t tok0, int64_t ntok,
                         uint16_t *k, uint16_t *v) {
  if (!shape_ok(Hkv, Hkv, D, P) || tok0 < 0 || ntok < 0) return -1;
  const int64_t page_elems = 2LL * Hkv * P * D;
  for (int64_t i = 0; i < ntok; ++i) {
    int64_t t = tok0 + i;
    if (t / P >= n_pages) return -2;
    int32_t pg = pages[t / P];
    if (pg < 0 || pg >= arena_pages) return -3;
    const uint16_t *base = arena + (int64_t)pg * page_elems;
    for (int g = 0; g < Hkv; ++g)
      for (int d = 0; d < D; ++d) {
        k[(i * Hkv + g) * D + d] = base[k_offset(g, (int)(t % P), d, P, D)];
        v[(i * Hkv + g) * D + d] = base[v_offset(g, (int)(t % P), d, P, D, Hkv)];
      }
  }
  return 0;
}

/* Attention of ONE (request, query head).  weights (may be NULL) receives w_t, t < n. */
static int attend_one(const uint16_t *arena, int64_t arena_pages, const int32_t *pages, int64_t n,
                      int h, int Hq, int Hkv, int D, int P, const uint16_t *q_row, double scale,
                      double *out_row, double *weights) {
  const int g = h / (Hq / Hkv);
  const int64_t page_elems = 2LL * Hkv * P * D;
  double *s = weights ? weights : (double *)malloc((size_t)n * sizeof(double));
  if (!s) return -4;
  double mx = -INFINITY;
  for (int64_t t = 0; t < n; ++t) {
    int32_t pg = pages[t / P];
    if (pg < 0 || pg >= arena_pages) { if (!weights) free(s); return -3; }
    const uint16_t *base = arena + (int64_t)pg * page_elems;
    double dot = 0.0;
    for (int d = 0; d < D; ++d)
      dot += bf16_to_f64(q_row[d]) * bf16_to_f64(base[k_offset(g, (int)(t % P), d, P, D)]);
    s[t] = scale * dot;
    if (s[t] > mx) mx = s[t];
  }
  double z = 0.0;
  for (int64_t t = 0; t < n; ++t) { s[t] = exp(s[t] - mx); z += s[t]; }
  for (int64_t t = 0; t < n; ++t) s[t] /= z;
  for (int d = 0; d < D; ++d) out_row[d] = 0.0;
  for (int64_t t = 0; t < n; ++t) {
    const uint16_t *base = arena + (int64_t)pages[t / P] * page_elems;
    for (int d = 0; d < D; ++d)
      out_row[d] += s[t] * bf16_to_f64(base[v_offset(g, (int)(t % P), d, P, D, Hkv)]);
  }
  if (!weights) free(s);
  return 0;
}

/* One layer, all requests.  page_table: [n_req][table_stride] page ids; q: [n_req][Hq][D] bf16;
 * out: [n_req][Hq][D] float64.  scale <= 0 selects 1/sqrt(D).  Returns 0, or <0 on bad input
 * (ctx_len < 1 is an error: softmax over nothing is undefined). */
int oracle_decode_attention(const uint16_t *arena, int64_t arena_pages, int n_req, int Hq, int Hkv,
                            int D, int P, const int32_t *page_table, int64_t table_stride,
                            const int32_t *ctx_len, const uint16_t *q, double scale, double *out) {
  if (!shape_ok(Hq, Hkv, D, P) || n_req < 0) return -1;
  if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
  for (int r = 0; r < n_req; ++r)
    if (ctx_len[r] < 1 || ((int64_t)ctx_len[r] + P - 1) / P > table_stride) return -2;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
  for (int r = 0; r < n_req; ++r)
    for (int h = 0; h < Hq; ++h) {
      int e = attend_one(arena, arena_pages, page_table + (int64_t)r * table_stride, ctx_len[r], h, Hq,
                         Hkv, D, P, q + ((int64_t)r * Hq + h) * D, scale,
                         out + ((int64_t)r * Hq + h) * D, NULL);
      if (e) {
#pragma omp atomic write
        err = e;
      }
    }
  return err;
}

/* Softmax weights and output of a single (request, head); weights has room for n doubles. */
int oracle_attention_weights(const uint16_t *arena, int64_t arena_pages, const int32_t *pages, int64_t n,
                             int h, int Hq, int Hkv, int D, int P, const uint16_t *q_row, double scale,
                             double *out_row, double *weights) {
  if (!shape_ok(Hq, Hkv, D, P) || n < 1 || h < 0 || h >= Hq || !weights) return -1;
  if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
  return attend_one(arena, arena_pages, pages, n, h, Hq, Hkv, D, P, q_row, scale, out_row, weights);
}

/* Limits the OpenMP team used by oracle_decode_attention (n >= 1); no effect without OpenMP. */
void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n >= 1) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}
