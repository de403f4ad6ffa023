// Load-only streaming probe (test-side evidence, not part of the library): what HBM read rate does
// MI355X deliver for the address pattern of the attention kernel, and for its alternatives?
//
// Every variant reads the same 1.476 GB (22528 blocks of 64 KiB, the size of one attention launch of
// the 8B-shaped batch-16 workload) with workgroups of 4 wavefronts, 16 KiB register tiles (two blocks' K and V
// tile of one head, the attention kernel's tile), 16-byte loads, no arithmetic beyond an XOR that keeps the
// loads alive.  A block is 8 heads x 4 KiB of K followed by 8 heads x 4 KiB of V.
//   kernel-pattern       a workgroup owns one KV head of a 64-block chunk (1024 tokens), its four wavefronts take
//                        the chunk's tiles in turn; the 8 heads of a chunk run on one XCD (workgroup i runs on
//                        XCD i mod 8); two tiles per wavefront in flight, nontemporal loads
//   kernel-pattern-4096  the same with 256-block chunks (4096 tokens, 704 workgroups): what attention_kernel
//                        issues at this launch size
//   heads-scattered      kernel-pattern, the 8 heads of a chunk on 8 different XCDs
//   plain-loads          kernel-pattern with ordinary instead of nontemporal loads
//   whole-blocks         a workgroup reads 8 whole consecutive blocks (the same 512 KiB per workgroup)
//   depth-3              kernel-pattern-4096 with three tiles per wavefront in flight
//   head-pair            two heads per workgroup, two wavefronts per head, 128-block chunks (2 MiB per workgroup)
//   head-quad            four heads per workgroup, a wavefront per head, 64-block chunks (2 MiB per workgroup): the
//                        workgroup reads 16 KiB of adjacent K tiles and 16 KiB of adjacent V tiles of every block
//   head-quad-256        the same with 16-block chunks (512 KiB per workgroup, 2816 workgroups)
//   head-quad-depth-3    head-quad with three tiles in flight
//   kv-adjacent          kernel-pattern-4096 on a page layout that puts a head's K and V tile side by side (8 KiB
//                        contiguous per head and block)
// Prints one line per variant: "<name> <microseconds> <GB/s>" (best of 8 launches).  Every variant's farthest
// address is checked on the host against the allocation before anything is launched.
#include <hip/hip_runtime.h>

#include <cstdio>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr long kBlock = 64 * 1024;  // one (request, layer) block
constexpr long kBlocks = 22528;     // 352 chunks of 64 blocks

struct Tile {
  u32x4 r[16];
};

struct Variant {
  const char *name;
  int whole;         // 1: whole-blocks (each workgroup reads 8 consecutive blocks front to back)
  int chunk_blocks;  // blocks per chunk
  int hpw;           // heads per workgroup: 1, 2 or 4 (4 / hpw wavefronts share a head)
  int scatter;       // 1: the heads of a chunk on different XCDs
  int nt;            // nontemporal loads
  int depth;         // tiles in flight per wavefront: 2 or 3
  int kv_adjacent;   // page layout with K and V of a head adjacent
};

template <bool NT>
__device__ __forceinline__ u32x4 ld(const unsigned char *p) {
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return *reinterpret_cast<const u32x4 *>(p);
}

template <bool NT>
__global__ __launch_bounds__(256, 1) void read_kernel(const unsigned char *__restrict__ base, const Variant v, unsigned *sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x;
  const int groups = 8 / v.hpw, wph = 4 / v.hpw;  // head groups of a chunk, wavefronts per head
  int sub, chunk;
  if (v.scatter) {
    sub = i % groups;
    chunk = i / groups;
  } else {  // spans of 8 chunks x `groups` head groups, group-major inside a span: all groups of chunk k have i mod 8 == k
    sub = (i >> 3) % groups;
    chunk = (i / (8 * groups)) * 8 + (i & 7);
  }
  const int g = sub * v.hpw + wave / wph;
  const int t0 = v.whole ? wave : wave % wph, tstep = v.whole ? 4 : wph;
  const int ntiles = v.whole ? 32 : v.chunk_blocks / 2;
  u32x4 acc = {0, 0, 0, 0};
  auto load = [&](Tile &T, int t) {  // tile t = blocks 2t, 2t+1 of the chunk, or 16 KiB of the run (whole-blocks)
    if (v.whole) {
      const unsigned char *p = base + ((long)i * 8) * kBlock + (long)t * 16384 + lane * 16;
#pragma unroll
      for (int k = 0; k < 16; ++k) T.r[k] = ld<NT>(p + k * 1024);
      return;
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const unsigned char *blk = base + ((long)chunk * v.chunk_blocks + 2 * t + b) * kBlock + lane * 16;
      const long k_at = v.kv_adjacent ? g * 8192L : g * 4096L, v_at = v.kv_adjacent ? g * 8192L + 4096 : 32768 + g * 4096L;
#pragma unroll
      for (int k = 0; k < 4; ++k) T.r[8 * b + k] = ld<NT>(blk + k_at + k * 1024);
#pragma unroll
      for (int k = 0; k < 4; ++k) T.r[8 * b + 4 + k] = ld<NT>(blk + v_at + k * 1024);
    }
  };
  auto use = [&](Tile &T) {
#pragma unroll
    for (int k = 0; k < 16; ++k) acc ^= T.r[k];
  };
  int t = t0;
  if (v.depth == 3) {
    Tile A, B, C;
    if (t < ntiles) load(A, t);
    if (t + tstep < ntiles) load(B, t + tstep);
    while (t < ntiles) {
      if (t + 2 * tstep < ntiles) load(C, t + 2 * tstep);
      use(A);
      t += tstep;
      if (t >= ntiles) break;
      if (t + 2 * tstep < ntiles) load(A, t + 2 * tstep);
      use(B);
      t += tstep;
      if (t >= ntiles) break;
      if (t + 2 * tstep < ntiles) load(B, t + 2 * tstep);
      use(C);
      t += tstep;
    }
  } else {
    Tile A, B;
    if (t < ntiles) load(A, t);
    while (t < ntiles) {
      if (t + tstep < ntiles) load(B, t + tstep);
      use(A);
      t += tstep;
      if (t >= ntiles) break;
      if (t + tstep < ntiles) load(A, t + tstep);
      use(B);
      t += tstep;
    }
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = 1;  // never true for the fill pattern: keeps the loads
}

int main() {
  const size_t bytes = (size_t)kBlocks * kBlock;
  const Variant vs[] = {
      {"kernel-pattern", 0, 64, 1, 0, 1, 2, 0},   {"heads-scattered", 0, 64, 1, 1, 1, 2, 0},
      {"plain-loads", 0, 64, 1, 0, 0, 2, 0},      {"whole-blocks", 1, 64, 1, 0, 1, 2, 0},
      {"kernel-pattern-4096", 0, 256, 1, 0, 1, 2, 0}, {"depth-3", 0, 256, 1, 0, 1, 3, 0},
      {"head-pair", 0, 128, 2, 0, 1, 2, 0},       {"head-quad", 0, 64, 4, 0, 1, 2, 0},
      {"head-quad-256", 0, 16, 4, 0, 1, 2, 0},    {"head-quad-depth-3", 0, 64, 4, 0, 1, 3, 0},
      {"kv-adjacent", 0, 256, 1, 0, 1, 2, 1}};
  // host-side bounds: a variant's chunks must tile the allocation exactly, in whole spans of 8 chunks
  for (const Variant &v : vs) {
    const long chunks = kBlocks / v.chunk_blocks;
    const bool ok = v.whole ? (kBlocks % 8 == 0)
                            : (kBlocks % v.chunk_blocks == 0 && chunks % 8 == 0 && v.chunk_blocks % 2 == 0 && 8 % v.hpw == 0);
    // the farthest byte: last block, last head, V tile, last KiB, last lane
    const long far = (kBlocks - 1) * kBlock + 7 * 8192L + 4096 + 3 * 1024 + 63 * 16 + 16;
    if (!ok || far > (long)bytes) {
      std::printf("probe variant %s does not fit the allocation\n", v.name);
      return 2;
    }
  }
  void *p = nullptr;
  unsigned *sink = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess || hipMalloc((void **)&sink, 4) != hipSuccess) return 1;
  if (hipMemset(p, 1, bytes) != hipSuccess || hipMemset(sink, 0, 4) != hipSuccess) return 1;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
  for (const Variant &v : vs) {
    const int grid = v.whole ? (int)(kBlocks / 8) : (int)(kBlocks / v.chunk_blocks) * (8 / v.hpw);
    float best = 1e30f;
    for (int rep = 0; rep < 10; ++rep) {
      (void)hipEventRecord(e0, nullptr);
      if (v.nt) hipLaunchKernelGGL(read_kernel<true>, dim3(grid), dim3(256), 0, nullptr, (const unsigned char *)p, v, sink);
      else hipLaunchKernelGGL(read_kernel<false>, dim3(grid), dim3(256), 0, nullptr, (const unsigned char *)p, v, sink);
      (void)hipEventRecord(e1, nullptr);
      if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) {
        std::printf("launch failed\n");
        return 3;
      }
      float ms = 0.f;
      (void)hipEventElapsedTime(&ms, e0, e1);
      if (rep >= 2 && ms < best) best = ms;
    }
    std::printf("%s %.1f %.0f\n", v.name, best * 1e3, (double)bytes / best / 1e6);
  }
  (void)hipFree(p);
  (void)hipFree(sink);
  return 0;
}
