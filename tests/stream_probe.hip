// Load-only streaming probe (test-side evidence, not part of the library): what HBM read rate does
// MI355X deliver for the address pattern of the attention kernel, and for its alternatives?
//
// Every variant reads the same 1.476 GB (22528 blocks of 64 KiB, the size of one attention launch of
// the 8B-shaped batch-16 workload) with 2816 workgroups of 4 wavefronts, two 16 KiB register tiles per
// wavefront in flight, 16-byte loads, no arithmetic beyond an XOR that keeps the loads alive:
//   kernel-pattern   a workgroup owns one KV head of a 64-block chunk (1024 tokens) and reads that head's
//                    4 KiB K tile and 4 KiB V tile of every block; the 8 heads of a chunk run on one XCD
//                    (workgroup i runs on XCD i mod 8)
//   kernel-pattern-4096  the same with 256-block chunks (4096 tokens, 704 workgroups) - what
//                    attention_kernel issues at this launch size
//   heads-scattered  the same reads, the 8 heads of a chunk on 8 different XCDs
//   plain-loads      kernel-pattern with ordinary instead of nontemporal loads
//   whole-blocks     a workgroup reads 8 whole consecutive blocks (the same 512 KiB per workgroup)
// Prints one line per variant: "<name> <microseconds> <GB/s>".  All addresses are checked on the host
// against the allocation before anything is launched.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr long kBlock = 64 * 1024;       // one (request, layer) block: 8 heads x (4 KiB K + 4 KiB V)
constexpr int kHeads = 8;
constexpr int kChunkBlocks = 64;         // 1024 tokens
constexpr int kChunks = 352;             // 2816 workgroups / 8 heads
constexpr long kBlocks = (long)kChunks * kChunkBlocks;
constexpr int kWorkgroups = kChunks * kHeads;

struct Tile {
  u32x4 r[16];
};

template <bool NT>
__device__ __forceinline__ u32x4 ld(const unsigned char *p) {
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return *reinterpret_cast<const u32x4 *>(p);
}

// mode 0: kernel pattern, 1: heads scattered over XCDs, 2: whole blocks
template <bool NT>
__global__ __launch_bounds__(256, 1) void read_kernel(const unsigned char *__restrict__ base, int mode, int chunk_blocks,
                                                      unsigned *sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x;
  int g, chunk;
  if (mode == 1) {
    g = i & 7;
    chunk = i >> 3;
  } else {  // spans of 8 chunks x 8 heads, head-major inside a span: the heads of chunk k all have i mod 8 == k
    g = (i >> 3) & 7;
    chunk = (i >> 6) * 8 + (i & 7);
  }
  u32x4 acc = {0, 0, 0, 0};
  auto load = [&](Tile &T, int t) {  // tile t = blocks 2t, 2t+1 of the chunk (mode 0/1) or 16 KiB of the run (mode 2)
    if (mode == 2) {
      const unsigned char *p = base + ((long)i * 8) * kBlock + (long)t * 16384 + lane * 16;
#pragma unroll
      for (int k = 0; k < 16; ++k) T.r[k] = ld<NT>(p + k * 1024);
    } else {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const unsigned char *blk = base + ((long)chunk * chunk_blocks + 2 * t + b) * kBlock + g * 4096 + lane * 16;
#pragma unroll
        for (int k = 0; k < 4; ++k) T.r[8 * b + k] = ld<NT>(blk + k * 1024);              // K tile
#pragma unroll
        for (int k = 0; k < 4; ++k) T.r[8 * b + 4 + k] = ld<NT>(blk + 32768 + k * 1024);  // V tile
      }
    }
  };
  auto use = [&](Tile &T) {
#pragma unroll
    for (int k = 0; k < 16; ++k) acc ^= T.r[k];
  };
  const int ntiles = mode == 2 ? 32 : chunk_blocks / 2;
  Tile A, B;
  int t = wave;
  load(A, t);
  while (t < ntiles) {
    int tn = t + 4;
    if (tn < ntiles) load(B, tn);
    use(A);
    t = tn;
    if (t >= ntiles) break;
    tn = t + 4;
    if (tn < ntiles) load(A, tn);
    use(B);
    t = tn;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = 1;  // never true for the fill pattern: keeps the loads
}

int main() {
  const size_t bytes = (size_t)kBlocks * kBlock;
  // host-side bounds: the farthest byte any variant touches
  const long far_pattern = ((long)(kChunks - 1) * kChunkBlocks + 63) * kBlock + 7 * 4096 + 32768 + 3 * 1024 + 63 * 16 + 16;
  const long far_blocks = ((long)(kWorkgroups - 1) * 8) * kBlock + 31L * 16384 + 15 * 1024 + 63 * 16 + 16;
  const long far_big = ((long)(kChunks / 4 - 1) * (4 * kChunkBlocks) + 4 * kChunkBlocks - 1) * kBlock + 7 * 4096 + 32768 + 3 * 1024 + 63 * 16 + 16;
  static_assert(kChunks % 32 == 0, "the 4096-token variant needs whole spans of 8 chunks");
  if (far_pattern > (long)bytes || far_blocks > (long)bytes || far_big > (long)bytes) {
    std::printf("probe addresses out of bounds\n");
    return 2;
  }
  void *p = nullptr;
  unsigned *sink = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess || hipMalloc((void **)&sink, 4) != hipSuccess) return 1;
  if (hipMemset(p, 1, bytes) != hipSuccess || hipMemset(sink, 0, 4) != hipSuccess) return 1;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
  const char *names[5] = {"kernel-pattern", "heads-scattered", "plain-loads", "whole-blocks", "kernel-pattern-4096"};
  for (int v = 0; v < 5; ++v) {
    const int mode = v == 1 ? 1 : (v == 3 ? 2 : 0);
    const int chunk_blocks = v == 4 ? 4 * kChunkBlocks : kChunkBlocks;
    const int grid = v == 4 ? kWorkgroups / 4 : kWorkgroups;
    float best = 1e30f;
    for (int rep = 0; rep < 8; ++rep) {
      (void)hipEventRecord(e0, nullptr);
      if (v == 2) hipLaunchKernelGGL(read_kernel<false>, dim3(grid), dim3(256), 0, nullptr, (const unsigned char *)p, mode, chunk_blocks, sink);
      else hipLaunchKernelGGL(read_kernel<true>, dim3(grid), dim3(256), 0, nullptr, (const unsigned char *)p, mode, chunk_blocks, sink);
      (void)hipEventRecord(e1, nullptr);
      if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) {
        std::printf("launch failed\n");
        return 3;
      }
      float ms = 0.f;
      (void)hipEventElapsedTime(&ms, e0, e1);
      if (rep >= 2 && ms < best) best = ms;
    }
    std::printf("%s %.1f %.0f\n", names[v], best * 1e3, (double)bytes / best / 1e6);
  }
  (void)hipFree(p);
  (void)hipFree(sink);
  return 0;
}
