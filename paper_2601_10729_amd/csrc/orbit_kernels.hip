// gfx950 (CDNA4, MI355X) kernels of liborbit.
//
//  attention : split-K GQA decode attention over paged K/V, one workgroup (4 wavefronts of 64)
//              per (request, kv head, chunk).  The in-page tile order is chosen so that every
//              16-byte per-lane global load lands directly in MFMA operand order:
//                 S^T[tok][head] = K[tok][dim] . Q^T[dim][head]      v_mfma_f32_16x16x32_bf16
//                 O^T[dim][head] = V^T[dim][tok] . P^T[tok][head]    v_mfma_f32_16x16x32_bf16
//              The query-head group (G <= 16) is the N dimension, padded with zero columns.
//              Online softmax in base 2, fp32, reduced across lanes with wavefront shuffles; the
//              four wavefronts of a workgroup are merged through LDS in a fixed order.  A
//              (request, kv head) that fits one chunk is normalised and written out at once.  In
//              append mode the workgroup that owns the position of the new token takes its K/V row
//              from the caller's buffers, attends to it and writes it into the page(s).
//  combine   : merges the chunks of a (request, query head) in fixed order and normalises.  It is a
//              launch of its own on purpose: a kernel boundary is the cheapest way to make one
//              workgroup's partial visible to another on a chip whose 8 XCDs each have their own L2
//              (merging inside the attention launch needs a device-scope release, i.e. an L2
//              write-back, per workgroup: measured 319 us per layer against 224 us).
//  append    : scatters one new token per request into its page (HBM and/or mapped host page).
//  fill/gather/blit : bulk token-major <-> page conversion and whole-page copies.
//
// Decode attention itself is only described in prose by the paper (Section 2.1); the block
// size of 16 tokens is Section 2.3, the single arena addressed by a (request x layer) table is
// Section 4, new KV of an offloaded layer going straight to the host is Section 3.2.
#include "orbit_kernels.h"

namespace orbit {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kD = 128;         // head dim
constexpr int kP = 16;          // tokens per page
constexpr int kTileBytes = kP * kD * 2;  // one K or V tile of one head: 4 KiB
constexpr int kWaves = 4;

struct Tile {  // two pages of one kv head as they sit in registers: 64 VGPRs
  u32x4_t k0[4], v0[4], k1[4], v1[4];
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t bf16_rne_bits(float f) {  // finite, non-NaN inputs only
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __builtin_bit_cast(float, b << 16); }

__device__ __forceinline__ float xor_max(float v, int mask) { return fmaxf(v, __shfl_xor(v, mask, 64)); }

// K/V is read exactly once per launch: nontemporal loads keep it from displacing anything in the caches.
__device__ __forceinline__ u32x4_t load16(const uint8_t *p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
}

// Page ids are wave-uniform (scalar).  A negative id i names page ~i of the mapped host arena: the
// zero-copy mode reads offloaded blocks over the host link instead of from a staging copy.
__device__ __forceinline__ uint8_t *page_ptr(const AttnParams &p, int id) {
  return id >= 0 ? p.arena + (int64_t)id * p.page_bytes : p.host + (int64_t)(~id) * p.page_bytes;
}

__device__ __forceinline__ void load_page(u32x4_t (&k)[4], u32x4_t (&v)[4], const uint8_t *ktile, const uint8_t *vtile,
                                          uint32_t lane_off) {
  // wave-uniform tile addresses + a 32-bit per-lane offset: scalar-base global loads, 1 KiB per instruction
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) k[kk] = load16(ktile + (lane_off + kk * 1024u));
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) v[kk] = load16(vtile + (lane_off + kk * 1024u));
}

__device__ __forceinline__ void zero_page(u32x4_t (&k)[4], u32x4_t (&v)[4]) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    k[kk] = u32x4_t{0, 0, 0, 0};
    v[kk] = u32x4_t{0, 0, 0, 0};
  }
}

// The last token of a request (position n-1) is attended to as a tile of its own, with the token in
// slot 0 and every other slot masked, in both modes, so that a step which appends inside the launch
// and an append followed by a separate attention launch do the same arithmetic.
// APPEND: the row comes from the caller's k_new / v_new and is also stored into slot `s` of the page
// at `ktile` / `vtile` and, if `mirror_k` is not null, of the host page that backs a staged block.
// Otherwise it is gathered from slot `s` of the page.
// Register order (see the page layout): lane l holds of K token l%16, dims (4kk + l/16)*8 .. +8;
// of V tokens 4(l/16) + i%4 in 16-bit element i, dims 32kk + 16(i/4) + l%16.
template <bool APPEND>
__device__ __forceinline__ void last_token_tile(Tile &T, int s, int lane, const uint16_t *krow, const uint16_t *vrow,
                                                uint8_t *ktile, uint8_t *vtile, uint8_t *mirror_k, uint8_t *mirror_v) {
  zero_page(T.k0, T.v0);
  zero_page(T.k1, T.v1);
  if ((lane & 15) == 0) {  // K of slot 0: lanes 0, 16, 32, 48
    const int src = (16 * (lane >> 4) + s) * 16;  // where slot s of the same dims sits in each KiB of the page
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (APPEND) {
        const u32x4_t w = *reinterpret_cast<const u32x4_t *>(krow + (4 * kk + (lane >> 4)) * 8);
        T.k0[kk] = w;
        *reinterpret_cast<u32x4_t *>(ktile + kk * 1024 + src) = w;
        if (mirror_k) *reinterpret_cast<u32x4_t *>(mirror_k + kk * 1024 + src) = w;
      } else {
        T.k0[kk] = *reinterpret_cast<const u32x4_t *>(ktile + kk * 1024 + src);
      }
    }
  }
  if (lane < 16) {  // V of slot 0: element 0 (dims 32kk + lane) and element 4 (dims 32kk + 16 + lane)
    const int src = (16 * (s >> 2) + lane) * 16 + 2 * (s & 3);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint16_t lo, hi;
      if (APPEND) {
        lo = vrow[32 * kk + lane];
        hi = vrow[32 * kk + 16 + lane];
        *reinterpret_cast<uint16_t *>(vtile + kk * 1024 + src) = lo;
        *reinterpret_cast<uint16_t *>(vtile + kk * 1024 + src + 8) = hi;
        if (mirror_v) {
          *reinterpret_cast<uint16_t *>(mirror_v + kk * 1024 + src) = lo;
          *reinterpret_cast<uint16_t *>(mirror_v + kk * 1024 + src + 8) = hi;
        }
      } else {
        lo = *reinterpret_cast<const uint16_t *>(vtile + kk * 1024 + src);
        hi = *reinterpret_cast<const uint16_t *>(vtile + kk * 1024 + src + 8);
      }
      T.v0[kk][0] = lo;
      T.v0[kk][2] = hi;
    }
  }
}

// One 32-token tile in two phases.  `valid` = tokens of the tile that exist (1..32); MASK = false
// promises valid == 32.
// Phase 1: scores S^T = K.Q^T, online-softmax update of (m, l); returns the bf16 weights in
// B-operand order and the factor alpha by which the running accumulator must shrink.
template <bool MASK>
__device__ __forceinline__ bf16x8_t tile_scores(const Tile &T, const bf16x8_t (&q)[4], float &m, float &l,
                                                float scale_log2, int valid, int j, float &alpha) {
  f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, T.k0[kk]), q[kk], s0, 0, 0, 0);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, T.k1[kk]), q[kk], s1, 0, 0, 0);
  // lane (j, n) now holds, for query head n, tokens 4j..4j+3 of page 0 (s0) and of page 1 (s1)
  float x[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[i] = s0[i] * scale_log2;
    x[4 + i] = s1[i] * scale_log2;
  }
  if (MASK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int t = 4 * j + i;
      if (t >= valid) x[i] = -INFINITY;
      if (t + kP >= valid) x[4 + i] = -INFINITY;
    }
  }
  float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
  mx = xor_max(mx, 16);
  mx = xor_max(mx, 32);
  const float mn = fmaxf(m, mx);  // finite: token 0 of the tile always exists
  alpha = fast_exp2(m - mn);
  uint32_t pb[8];
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pb[i] = bf16_rne_bits(fast_exp2(x[i] - mn));
    psum += bf16_bits_to_f32(pb[i]);  // normaliser uses the rounded weights that multiply V
  }
  l = l * alpha + psum;
  m = mn;
  u32x4_t pw = {pb[0] | (pb[1] << 16), pb[2] | (pb[3] << 16), pb[4] | (pb[5] << 16), pb[6] | (pb[7] << 16)};
  return __builtin_bit_cast(bf16x8_t, pw);
}

// Phase 2: O^T = alpha O^T + V^T.P^T.
template <bool MASK>
__device__ __forceinline__ void tile_pv(Tile &T, const bf16x8_t pB, float alpha, f32x4_t (&acc)[8], int valid, int j) {
  if (MASK) {
    // a slot past the stored length may hold anything (even Inf/NaN bits): clear it so that
    // weight 0 times garbage cannot poison the accumulator
    uint32_t mk0[2], mk1[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int t = 4 * j + 2 * h;
      mk0[h] = (t < valid ? 0x0000FFFFu : 0u) | (t + 1 < valid ? 0xFFFF0000u : 0u);
      mk1[h] = (t + kP < valid ? 0x0000FFFFu : 0u) | (t + 1 + kP < valid ? 0xFFFF0000u : 0u);
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      T.v0[kk] = T.v0[kk] & u32x4_t{mk0[0], mk0[1], mk0[0], mk0[1]};
      T.v1[kk] = T.v1[kk] & u32x4_t{mk1[0], mk1[1], mk1[0], mk1[1]};
    }
  }
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) {
    acc[nb] *= alpha;
    const int e = nb & 1;
    u32x4_t a = {T.v0[nb >> 1][2 * e], T.v0[nb >> 1][2 * e + 1], T.v1[nb >> 1][2 * e], T.v1[nb >> 1][2 * e + 1]};
    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), pB, acc[nb], 0, 0, 0);
  }
}

template <bool MASK>
__device__ __forceinline__ void process_tile(Tile &T, const bf16x8_t (&q)[4], f32x4_t (&acc)[8], float &m, float &l,
                                             float scale_log2, int valid, int j) {
  float alpha;
  const bf16x8_t pB = tile_scores<MASK>(T, q, m, l, scale_log2, valid, j, alpha);
  tile_pv<MASK>(T, pB, alpha, acc, valid, j);
}

// One workgroup per (segment, kv head), in the launch order the host chose.  Two register tiles per
// wave: the next tile's loads are in flight while the current one is processed (about 16 KiB per wave,
// 64 KiB per CU, outstanding at all times); 1 workgroup per CU slot.
// APPEND: n_tok counts a token whose K/V row is still in k_new/v_new (see last_token_tile).
template <bool APPEND>
__global__ __launch_bounds__(256, 1) void attention_kernel(const AttnParams p) {
  extern __shared__ float smem[];  // [3][G][128] accumulators of waves 1..3, then [4][2][16] (m, l)
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j = lane >> 4, nn = lane & 15;
  const uint32_t lane_off = (uint32_t)lane * 16u;
  const int G = p.G;
  const int64_t v_off = (int64_t)p.Hkv * kTileBytes;

  // workgroup b runs on XCD b mod 8: the Hkv heads of a segment, which share its pages, sit 8 workgroups apart
  const int b = blockIdx.x, jj = b >> 3;
  const int g = jj % p.Hkv;
  const int32_t *it = p.work + (int64_t)((jj / p.Hkv) * 8 + (b & 7)) * 4;
  const int r = it[0], tok0 = it[1], seg = it[3];
  if (r < 0) return;  // padding of the launch order to a multiple of 8
  const int64_t head_off = (int64_t)g * kTileBytes;
  const int n = p.req[r].n_tok;
  const bool single = p.req[r].n_parts == 1;
  const int span = min(it[2], n - tok0);
  // the request's last token is handled after the paged tiles (see last_token_tile)
  const bool has_last = tok0 + span == n;
  const int ntok = span - (has_last ? 1 : 0);  // >= 0
  const int ntiles = (ntok + 2 * kP - 1) / (2 * kP);
  const int32_t *row = p.table + ((int64_t)r * p.L + p.layer) * p.cap_pages + tok0 / kP;

  bf16x8_t q[4];
  {
    const uint16_t *qrow = p.q + ((int64_t)r * p.Hq + g * G + (nn < G ? nn : 0)) * kD;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4_t w = *reinterpret_cast<const u32x4_t *>(qrow + (4 * kk + j) * 8);
      if (nn >= G) w = u32x4_t{0, 0, 0, 0};
      q[kk] = __builtin_bit_cast(bf16x8_t, w);
    }
  }

  f32x4_t acc[8];
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;

  auto load_tile = [&](Tile &T, int t) {
    const int valid = ntok - 2 * kP * t;
    const int p0 = __builtin_amdgcn_readfirstlane(row[2 * t]);
    const uint8_t *t0 = page_ptr(p, p0) + head_off;
    load_page(T.k0, T.v0, t0, t0 + v_off, lane_off);
    if (valid > kP) {
      const int p1 = __builtin_amdgcn_readfirstlane(row[2 * t + 1]);
      const uint8_t *t1 = page_ptr(p, p1) + head_off;
      load_page(T.k1, T.v1, t1, t1 + v_off, lane_off);
    } else {
      zero_page(T.k1, T.v1);
    }
  };
  auto run_tile = [&](Tile &T, int t) {
    const int valid = ntok - 2 * kP * t;
    if (valid >= 2 * kP) process_tile<false>(T, q, acc, m, l, p.scale_log2, 2 * kP, j);
    else process_tile<true>(T, q, acc, m, l, p.scale_log2, valid, j);
  };

  {
    Tile A, B;
    int t = wave;
    if (t < ntiles) load_tile(A, t);
    while (t < ntiles) {
      int tn = t + kWaves;
      if (tn < ntiles) load_tile(B, tn);
      run_tile(A, t);
      t = tn;
      if (t >= ntiles) break;
      tn = t + kWaves;
      if (tn < ntiles) load_tile(A, tn);
      run_tile(B, t);
      t = tn;
    }
  }
  if (has_last && wave == ntiles % kWaves) {  // the wave next in the rotation
    Tile T;
    const int pi = ntok >> 4, slot = ntok & 15;  // the token sits right behind the paged ones
    const int pid = __builtin_amdgcn_readfirstlane(row[pi]);
    uint8_t *kt = page_ptr(p, pid) + head_off;
    uint8_t *mk = nullptr;
    const uint16_t *krow = nullptr, *vrow = nullptr;
    if (APPEND) {
      const int hp = p.req[r].host_page0;
      if (hp >= 0) mk = p.host + ((int64_t)hp + tok0 / kP + pi) * p.page_bytes + head_off;
      krow = p.k_new + ((int64_t)r * p.Hkv + g) * kD;
      vrow = p.v_new + ((int64_t)r * p.Hkv + g) * kD;
    }
    last_token_tile<APPEND>(T, slot, lane, krow, vrow, kt, kt + v_off, mk, mk ? mk + v_off : nullptr);
    process_tile<true>(T, q, acc, m, l, p.scale_log2, 1, j);
  }

  // l holds this lane's share of the normaliser; fold the four token groups of each head
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);

  float *sm_acc = smem;                      // [3][G][128]
  float *sm_ml = smem + 3 * G * kD;          // [4][2][16]
  if (j == 0) {
    sm_ml[wave * 32 + nn] = m;
    sm_ml[wave * 32 + 16 + nn] = l;
  }
  if (wave > 0 && nn < G) {
    float *dst = sm_acc + ((wave - 1) * G + nn) * kD + 4 * j;
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) *reinterpret_cast<f32x4_t *>(dst + 16 * nb) = acc[nb];
  }
  __syncthreads();
  if (wave == 0 && nn < G) {
    float mw[kWaves], lw[kWaves];
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      mw[w] = sm_ml[w * 32 + nn];
      lw[w] = sm_ml[w * 32 + 16 + nn];
    }
    const float M = fmaxf(fmaxf(mw[0], mw[1]), fmaxf(mw[2], mw[3]));  // finite: some wave had a tile
    float f[kWaves];
#pragma unroll
    for (int w = 0; w < kWaves; ++w) f[w] = fast_exp2(mw[w] - M);
    float lt = lw[0] * f[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) lt += lw[w] * f[w];
    if (single) {  // the only segment of this (request, kv head): normalise and write the output
      const float inv = 1.0f / lt;
      const int64_t o = ((int64_t)r * p.Hq + g * G + nn) * kD + 4 * j;
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) {
        f32x4_t v = acc[nb] * f[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w)
          v += *reinterpret_cast<const f32x4_t *>(sm_acc + ((w - 1) * G + nn) * kD + 4 * j + 16 * nb) * f[w];
        v *= inv;
        *reinterpret_cast<u32x2_t *>(p.out + o + 16 * nb) =
            u32x2_t{bf16_rne_bits(v[0]) | (bf16_rne_bits(v[1]) << 16), bf16_rne_bits(v[2]) | (bf16_rne_bits(v[3]) << 16)};
        if (p.out_f32) *reinterpret_cast<f32x4_t *>(p.out_f32 + o + 16 * nb) = v;
      }
    } else {
      const int64_t pslot = (int64_t)seg * p.Hkv + g;
      float *out = p.pacc + (pslot * G + nn) * kD + 4 * j;
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) {
        f32x4_t o = acc[nb] * f[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w)
          o += *reinterpret_cast<const f32x4_t *>(sm_acc + ((w - 1) * G + nn) * kD + 4 * j + 16 * nb) * f[w];
        *reinterpret_cast<f32x4_t *>(out + 16 * nb) = o;
      }
      if (j == 0) {
        p.pml[pslot * 32 + nn] = M;
        p.pml[pslot * 32 + 16 + nn] = lt;
      }
    }
  }
}

// One workgroup of 4 waves per (request, query head) with more than one segment; lane handles dims
// 2*lane, 2*lane+1; wave w takes segments w, w+4, ... of the request; the four partial sums are added in
// wave order.
__global__ __launch_bounds__(256) void combine_kernel(const CombineParams p) {
  __shared__ float sm[kWaves][kD + 1];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = blockIdx.x / p.Hq, h = blockIdx.x % p.Hq;
  const int g = h / p.G, nn = h % p.G;
  const int nc = p.n_parts[r];
  if (nc == 1) return;  // written by the attention launch itself
  const int64_t base = p.seg_base[r];
  auto slot = [&](int c) { return (base + c) * p.Hkv + g; };

  float M = -INFINITY;
  for (int c = lane; c < nc; c += 64) M = fmaxf(M, p.pml[slot(c) * 32 + nn]);
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) M = xor_max(M, s);

  float o0 = 0.f, o1 = 0.f, lsum = 0.f;
  for (int c = wave; c < nc; c += kWaves) {
    const int64_t s = slot(c);
    const float f = fast_exp2(p.pml[s * 32 + nn] - M);
    lsum += p.pml[s * 32 + 16 + nn] * f;
    const float2 a = *reinterpret_cast<const float2 *>(p.pacc + (s * p.G + nn) * kD + 2 * lane);
    o0 += a.x * f;
    o1 += a.y * f;
  }
  sm[wave][2 * lane] = o0;
  sm[wave][2 * lane + 1] = o1;
  if (lane == 0) sm[wave][kD] = lsum;
  __syncthreads();
  if (wave == 0) {
    float t0 = sm[0][2 * lane], t1 = sm[0][2 * lane + 1], lt = sm[0][kD];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      t0 += sm[w][2 * lane];
      t1 += sm[w][2 * lane + 1];
      lt += sm[w][kD];
    }
    const float inv = 1.0f / lt;
    t0 *= inv;
    t1 *= inv;
    const int64_t o = ((int64_t)r * p.Hq + h) * kD + 2 * lane;
    *reinterpret_cast<uint32_t *>(p.out + o) = bf16_rne_bits(t0) | (bf16_rne_bits(t1) << 16);
    if (p.out_f32) *reinterpret_cast<float2 *>(p.out_f32 + o) = float2{t0, t1};
  }
}

__device__ __forceinline__ int v_elem_offset(int tok, int dim) {
  return ((((dim >> 5) * (kP / 4) + (tok >> 2)) * 16 + (dim & 15)) * 2 + ((dim >> 4) & 1)) * 4 + (tok & 3);
}

__global__ __launch_bounds__(256) void append_kernel(const AppendParams p) {
  const AppendItem item = p.items[blockIdx.x];
  const int slot = item.tok % kP;
  const uint16_t *ksrc = p.k + (int64_t)blockIdx.x * p.Hkv * kD;
  const uint16_t *vsrc = p.v + (int64_t)blockIdx.x * p.Hkv * kD;
  uint8_t *dests[2] = {item.page >= 0 ? p.arena + (int64_t)item.page * p.page_bytes : nullptr,
                       reinterpret_cast<uint8_t *>(item.host_page)};
  for (int d = 0; d < 2; ++d) {
    uint8_t *base = dests[d];
    if (!base) continue;
    for (int i = threadIdx.x; i < p.Hkv * 16; i += blockDim.x) {
      const int g = i >> 4, c = i & 15;
      const u32x4_t w = *reinterpret_cast<const u32x4_t *>(ksrc + g * kD + c * 8);
      *reinterpret_cast<u32x4_t *>(base + (int64_t)g * kTileBytes + (c * kP + slot) * 16) = w;
    }
    uint16_t *vt = reinterpret_cast<uint16_t *>(base + (int64_t)p.Hkv * kTileBytes);
    for (int i = threadIdx.x; i < p.Hkv * kD; i += blockDim.x) {
      const int g = i / kD, dim = i % kD;
      vt[g * (kTileBytes / 2) + v_elem_offset(slot, dim)] = vsrc[i];
    }
  }
}

__device__ __forceinline__ uint8_t *fill_page_base(const FillParams &p, int64_t page_index) {
  return p.row ? p.arena + (int64_t)p.row[page_index] * p.page_bytes : p.host_run + page_index * p.page_bytes;
}

// grid (pages touched, Hkv); token-major -> page tiles.
__global__ __launch_bounds__(256) void fill_kernel(const FillParams p) {
  const int64_t pi = p.first_token / kP + blockIdx.x;
  const int g = blockIdx.y;
  uint8_t *base = fill_page_base(p, pi);
  const int64_t lo = p.first_token, hi = p.first_token + p.n_tokens;
  const int tid = threadIdx.x;
  {  // K: thread (c, t) moves one 16-byte chunk
    const int c = tid >> 4, t = tid & 15;
    const int64_t tok = pi * kP + t;
    if (tok >= lo && tok < hi) {
      const u32x4_t w = *reinterpret_cast<const u32x4_t *>(p.k + ((tok - lo) * p.Hkv + g) * kD + c * 8);
      *reinterpret_cast<u32x4_t *>(base + (int64_t)g * kTileBytes + (c * kP + t) * 16) = w;
    }
  }
  {  // V: thread owns the 16-byte chunk (nbp, j, m) = 2 dims x 4 tokens
    const int nbp = tid >> 6, jq = (tid >> 4) & 3, mm = tid & 15;
    uint16_t *dst = reinterpret_cast<uint16_t *>(base + (int64_t)(p.Hkv + g) * kTileBytes) + tid * 8;
    const int64_t t0 = pi * kP + 4 * jq;
    uint16_t w[8];
    bool all = t0 >= lo && t0 + 3 < hi;
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int64_t tok = t0 + i;
        const bool in = tok >= lo && tok < hi;
        w[e * 4 + i] = in ? p.v[((tok - lo) * p.Hkv + g) * kD + (2 * nbp + e) * 16 + mm] : (uint16_t)0;
      }
    if (all) {
      u32x4_t pk = {w[0] | ((uint32_t)w[1] << 16), w[2] | ((uint32_t)w[3] << 16), w[4] | ((uint32_t)w[5] << 16),
                    w[6] | ((uint32_t)w[7] << 16)};
      *reinterpret_cast<u32x4_t *>(dst) = pk;
    } else {
#pragma unroll
      for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int64_t tok = t0 + i;
          if (tok >= lo && tok < hi) dst[e * 4 + i] = w[e * 4 + i];
        }
    }
  }
}

// grid (pages touched, Hkv); page tiles -> token-major.
__global__ __launch_bounds__(256) void gather_kernel(const FillParams p) {
  const int64_t pi = p.first_token / kP + blockIdx.x;
  const int g = blockIdx.y;
  const uint8_t *base = fill_page_base(p, pi);
  const int64_t lo = p.first_token, hi = p.first_token + p.n_tokens;
  const int tid = threadIdx.x;
  {
    const int c = tid >> 4, t = tid & 15;
    const int64_t tok = pi * kP + t;
    if (tok >= lo && tok < hi) {
      const u32x4_t w = *reinterpret_cast<const u32x4_t *>(base + (int64_t)g * kTileBytes + (c * kP + t) * 16);
      *reinterpret_cast<u32x4_t *>(p.k + ((tok - lo) * p.Hkv + g) * kD + c * 8) = w;
    }
  }
  {
    const int nbp = tid >> 6, jq = (tid >> 4) & 3, mm = tid & 15;
    const uint16_t *src = reinterpret_cast<const uint16_t *>(base + (int64_t)(p.Hkv + g) * kTileBytes) + tid * 8;
    const int64_t t0 = pi * kP + 4 * jq;
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int64_t tok = t0 + i;
        if (tok >= lo && tok < hi) p.v[((tok - lo) * p.Hkv + g) * kD + (2 * nbp + e) * 16 + mm] = src[e * 4 + i];
      }
  }
}

__global__ __launch_bounds__(256) void blit_kernel(const BlitOp *ops, int64_t units_per_page) {
  const BlitOp op = ops[blockIdx.x];
  const u32x4_t *s = reinterpret_cast<const u32x4_t *>(op.src);
  u32x4_t *d = reinterpret_cast<u32x4_t *>(op.dst);
  for (int64_t i = (int64_t)blockIdx.y * blockDim.x + threadIdx.x; i < units_per_page;
       i += (int64_t)gridDim.y * blockDim.x)
    d[i] = s[i];
}

// Debugging aid (ORBIT_FLAG_POISON_STAGING): a consumed staging range is filled with quiet-NaN bf16 patterns.
__global__ __launch_bounds__(256) void poison_kernel(u32x4_t *p, int64_t n_units) {
  const u32x4_t nan4 = {0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u};
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_units; i += (int64_t)gridDim.x * blockDim.x) p[i] = nan4;
}

// The same copies with a small, fixed number of workgroups that walk the list: for copies that run
// beside the decode steps.  A link-bound copy needs few bytes in flight, and workgroups parked on the
// link must not fill the wavefront slots the attention launches need.
__global__ __launch_bounds__(256) void blit_narrow_kernel(const BlitOp *ops, int64_t n_ops, int64_t units_per_page) {
  for (int64_t o = blockIdx.x; o < n_ops; o += gridDim.x) {
    const BlitOp op = ops[o];
    const u32x4_t *s = reinterpret_cast<const u32x4_t *>(op.src);
    u32x4_t *d = reinterpret_cast<u32x4_t *>(op.dst);
    for (int64_t i = threadIdx.x; i < units_per_page; i += blockDim.x) d[i] = s[i];
  }
}

// ------------------------------------------------------------------------------------ launches

hipError_t launch_attention(const AttnParams &p, hipStream_t s) {
  if (p.n_workers <= 0) return hipSuccess;
  const size_t lds = (size_t)(3 * p.G * kD + kWaves * 32) * sizeof(float);
  const dim3 grid((unsigned)(p.n_workers * p.Hkv)), block(256);
  if (p.k_new) hipLaunchKernelGGL(attention_kernel<true>, grid, block, lds, s, p);
  else hipLaunchKernelGGL(attention_kernel<false>, grid, block, lds, s, p);
  return hipGetLastError();
}

hipError_t launch_combine(const CombineParams &p, hipStream_t s) {
  if (p.n_req <= 0) return hipSuccess;
  hipLaunchKernelGGL(combine_kernel, dim3((unsigned)(p.n_req * p.Hq)), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_append(const AppendParams &p, hipStream_t s) {
  if (p.n <= 0) return hipSuccess;
  hipLaunchKernelGGL(append_kernel, dim3((unsigned)p.n), dim3(256), 0, s, p);
  return hipGetLastError();
}

static dim3 fill_grid(const FillParams &p) {
  const int64_t first = p.first_token / kP, last = (p.first_token + p.n_tokens - 1) / kP;
  return dim3((unsigned)(last - first + 1), (unsigned)p.Hkv);
}

hipError_t launch_fill(const FillParams &p, hipStream_t s) {
  if (p.n_tokens <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_kernel, fill_grid(p), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_gather(const FillParams &p, hipStream_t s) {
  if (p.n_tokens <= 0) return hipSuccess;
  hipLaunchKernelGGL(gather_kernel, fill_grid(p), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_blit(const BlitOp *ops_dev, int64_t n_ops, int64_t page_bytes, hipStream_t s) {
  if (n_ops <= 0) return hipSuccess;
  const int64_t units = page_bytes / 16;
  const unsigned split = (unsigned)std::max<int64_t>(1, std::min<int64_t>(8, units / 1024));
  hipLaunchKernelGGL(blit_kernel, dim3((unsigned)n_ops, split), dim3(256), 0, s, ops_dev, units);
  return hipGetLastError();
}

hipError_t launch_poison(uint8_t *p, int64_t bytes, hipStream_t s) {
  if (bytes <= 0) return hipSuccess;
  hipLaunchKernelGGL(poison_kernel, dim3(1024), dim3(256), 0, s, reinterpret_cast<u32x4_t *>(p), bytes / 16);
  return hipGetLastError();
}

hipError_t launch_blit_narrow(const BlitOp *ops_dev, int64_t n_ops, int64_t page_bytes, int workgroups, hipStream_t s) {
  if (n_ops <= 0) return hipSuccess;
  const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>(workgroups, n_ops));
  hipLaunchKernelGGL(blit_narrow_kernel, dim3(grid), dim3(256), 0, s, ops_dev, n_ops, page_bytes / 16);
  return hipGetLastError();
}

}  // namespace orbit
