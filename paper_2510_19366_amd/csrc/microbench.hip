// Machine-peak microbenchmarks behind moe_prism_microbench (measurement only, no part of the
// layer): what the matrix cores, the LDS, the global->LDS copy path and HBM deliver on this
// chip in loops shaped like the grouped-FFN kernels', so that a kernel's utilisation can be
// quoted against a measured ceiling as well as against the datasheet.
//
// Every test also reports the shader clock it ran at: s_memtime counts shader clocks,
// s_memrealtime a constant 100 MHz, so their ratio over the kernel is the average clock.
#include "../../include/moe_prism.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

namespace mpub {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__device__ __forceinline__ uint64_t shader_clock() { return __builtin_readcyclecounter(); }
__device__ __forceinline__ uint64_t real_clock() { return __builtin_amdgcn_s_memrealtime(); }

struct Clk {  // written by workgroup 0, lane 0
  unsigned long long shader, real;
};

// ------------------------------------------------------------------ matrix cores, operands in registers
// NACC independent 32x32 accumulators per wave, operands loaded once from `data` (so the
// caller chooses constant or random bf16 bit patterns).
template <int NACC>
__global__ __launch_bounds__(256) void mfma_reg_kernel(const uint4* __restrict__ data, float* out,
                                                       int iters, Clk* clk) {
  const uint4 qa = data[threadIdx.x], qb = data[256 + threadIdx.x];
  const bf16x8 a = __builtin_bit_cast(bf16x8, qa), b = __builtin_bit_cast(bf16x8, qb);
  f32x16 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.0f;
  const uint64_t c0 = shader_clock(), r0 = real_clock();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  const uint64_t c1 = shader_clock(), r1 = real_clock();
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[i][j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) *clk = Clk{c1 - c0, r1 - r0};
}

// The rank-1 fp32 form the router-logits kernel issues (one binary32 FMA per output and
// instruction): NACC independent chains of 32 x 64 outputs per wave.
typedef __attribute__((__vector_size__(32 * sizeof(float)))) float f32x32;
template <int NACC>
__global__ __launch_bounds__(256) void mfma_f32_rank1_kernel(const uint4* __restrict__ data, float* out,
                                                            int iters, Clk* clk) {
  const uint4 q = data[threadIdx.x];
  const float a = __uint_as_float(q.x << 16), b = __uint_as_float(q.y << 16);  // bf16 bits widened
  f32x32 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int j = 0; j < 32; ++j) acc[i][j] = 0.0f;
  const uint64_t c0 = shader_clock(), r0 = real_clock();
  for (int it = 0; it < iters; ++it) {
    static_assert(NACC == 2, "two chains: A block 0 and A block 1");
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x1f32(a, b, acc[0], 1, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x1f32(a, b, acc[1], 1, 1, 0);
  }
  const uint64_t c1 = shader_clock(), r1 = real_clock();
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int j = 0; j < 32; ++j) s += acc[i][j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) *clk = Clk{c1 - c0, r1 - r0};
}

// The same with a different pair of operand registers for every k step (32 pairs, as the
// logits kernel has them after reading a slab from LDS).
__global__ __launch_bounds__(256) void mfma_f32_rank1_many_operands_kernel(const uint4* __restrict__ data,
                                                                          float* out, int iters, Clk* clk) {
  float fa[32], fb[32];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint4 q = data[(threadIdx.x + 37 * i) & 4095], r = data[(threadIdx.x + 53 * i + 11) & 4095];
    fa[4 * i] = __uint_as_float(q.x << 16); fa[4 * i + 1] = __uint_as_float(q.y << 16);
    fa[4 * i + 2] = __uint_as_float(q.z << 16); fa[4 * i + 3] = __uint_as_float(q.w << 16);
    fb[4 * i] = __uint_as_float(r.x << 16); fb[4 * i + 1] = __uint_as_float(r.y << 16);
    fb[4 * i + 2] = __uint_as_float(r.z << 16); fb[4 * i + 3] = __uint_as_float(r.w << 16);
  }
  f32x32 acc0, acc1;
#pragma unroll
  for (int j = 0; j < 32; ++j) acc0[j] = acc1[j] = 0.0f;
  const uint64_t c0 = shader_clock(), r0 = real_clock();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x1f32(fa[i], fb[i], acc0, 1, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x1f32(fa[i], fb[i], acc1, 1, 1, 0);
    }
  }
  const uint64_t c1 = shader_clock(), r1 = real_clock();
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < 32; ++j) s += acc0[j] + acc1[j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) *clk = Clk{c1 - c0, r1 - r0};
}

// ------------------------------------------------------------------ matrix cores fed from LDS
// A workgroup of WAVES waves multiplies a resident LDS tile again and again: rows of 32
// K-elements (64 bytes, 4 chunks of 16 bytes, XOR-swizzled like the FFN kernels' ring
// stages), wave tile (MB x 32) slot rows by (NB x 32) weight rows, waves laid out WM x WN.
// No global traffic inside the loop: this is the ceiling of the LDS -> MFMA part alone.
__device__ __forceinline__ int swz32(int r, int c) { return r * 32 + ((c ^ ((r >> 2) & 3)) << 3); }

template <int MB, int NB, int WM, int WN, int OCC>
__global__ __launch_bounds__(WM* WN * 64) __attribute__((amdgpu_waves_per_eu(OCC, OCC))) void mfma_lds_kernel(const uint4* __restrict__ data,
                                                              float* out, int iters, Clk* clk) {
  constexpr int A_ROWS = WM * MB * 32, B_ROWS = WN * NB * 32, STAGES = 2;
  extern __shared__ __align__(16) uint16_t sm[];
  constexpr int WORDS = STAGES * (A_ROWS + B_ROWS) * 4;  // uint4 per tile
  for (int i = threadIdx.x; i < WORDS; i += WM * WN * 64)
    reinterpret_cast<uint4*>(sm)[i] = data[i & 4095];
  __syncthreads();
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int wm = wv / WN, wn = wv % WN;
  f32x16 acc[MB][NB];
#pragma unroll
  for (int m = 0; m < MB; ++m)
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[m][n][j] = 0.0f;
  const uint64_t c0 = shader_clock(), r0 = real_clock();
  for (int it = 0; it < iters; ++it) {
    const uint16_t* sa = sm + (it & 1) * (A_ROWS + B_ROWS) * 32;
    const uint16_t* sb = sa + A_ROWS * 32;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int c = ks * 2 + (lane >> 5);
      bf16x8 fa[MB], fb[NB];
#pragma unroll
      for (int m = 0; m < MB; ++m)
        fa[m] = *reinterpret_cast<const bf16x8*>(sa + swz32((wm * MB + m) * 32 + (lane & 31), c));
#pragma unroll
      for (int n = 0; n < NB; ++n)
        fb[n] = *reinterpret_cast<const bf16x8*>(sb + swz32((wn * NB + n) * 32 + (lane & 31), c));
#pragma unroll
      for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int n = 0; n < NB; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[n], fa[m], acc[m][n], 0, 0, 0);
    }
  }
  const uint64_t c1 = shader_clock(), r1 = real_clock();
  float s = 0.0f;
#pragma unroll
  for (int m = 0; m < MB; ++m)
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) s += acc[m][n][j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) *clk = Clk{c1 - c0, r1 - r0};
}

// ------------------------------------------------------------------ LDS read bandwidth
// 16-byte reads in the fragment pattern (32 rows x one chunk index per half wave), NR
// fragments per wave and iteration, conflict-free by the swizzle.
template <int NT, int NR>
__global__ __launch_bounds__(NT) void lds_read_kernel(float* out, int iters, Clk* clk) {
  extern __shared__ __align__(16) uint16_t sm[];
  for (int i = threadIdx.x; i < 512 * 32; i += NT) sm[i] = (uint16_t)i;
  __syncthreads();
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  uint4 acc = make_uint4(0, 0, 0, 0);
  const uint64_t c0 = shader_clock(), r0 = real_clock();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const int row = (((wv * NR + r + it) * 32) + (lane & 31)) & 511;  // moves every iteration
      const int c = ((it & 1) << 1) + (lane >> 5);
      const uint4 v = *reinterpret_cast<const uint4*>(sm + swz32(row, c));
      acc.x ^= v.x;
      acc.y ^= v.y;
      acc.z ^= v.z;
      acc.w ^= v.w;
    }
  }
  const uint64_t c1 = shader_clock(), r1 = real_clock();
  out[blockIdx.x * NT + threadIdx.x] = (float)(acc.x ^ acc.y ^ acc.z ^ acc.w);
  if (blockIdx.x == 0 && threadIdx.x == 0) *clk = Clk{c1 - c0, r1 - r0};
}

// ------------------------------------------------------------------ global -> LDS and global -> register streams
__device__ __forceinline__ void dma16(const void* g, uint32_t lds) {
  uint32_t keep;  // m0 is reserved by the compiler: put its value back after the copy
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 1\n\tglobal_load_lds_dwordx4 %1, off\n\t"
               "s_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(g), "s"(lds)
               : "memory");
}
// the same copy with a cache-policy modifier: 1 = sc0, 2 = sc1, 3 = sc0 sc1, 4 = nt
template <int policy>
__device__ __forceinline__ void dma16_policy(const void* g, uint32_t lds) {
  uint32_t keep;
#define MPUB_DMA(MOD)                                                                                   \
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 1\n\tglobal_load_lds_dwordx4 %1, off" MOD "\n\t" \
               "s_mov_b32 m0, %0"                                                                       \
               : "=&s"(keep)                                                                            \
               : "v"(g), "s"(lds)                                                                       \
               : "memory")
  if constexpr (policy == 1) MPUB_DMA(" sc0");
  else if constexpr (policy == 2) MPUB_DMA(" sc1");
  else if constexpr (policy == 3) MPUB_DMA(" sc0 sc1");
  else MPUB_DMA(" nt");
#undef MPUB_DMA
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Every wave streams 16-row x 64-byte pieces (4 lanes per row: the operand-tile copy
// pattern) of rows `row_stride` bytes apart out of a region of `footprint` bytes, DEPTH
// copies in flight.  TO_LDS: global_load_lds_dwordx4; else 16-byte loads into registers.
// layout 0: 4 adjacent lanes share a row (coalesced 64-byte runs); layout 1: every lane
// its own row, 32 rows x two 16-byte halves (the MFMA operand layout read straight from memory);
// layout 2: like 0, but a wave steps 128 bytes along the row, so only the first 64 bytes of
// every 128-byte line are ever requested (what a K stage of 32 bf16 elements asks of the
// caches when the other half of the line is needed a stage later).
template <int DEPTH, int NW, bool TO_LDS, int POLICY = 0>
__global__ __launch_bounds__(NW * 64) void stream_kernel(const char* __restrict__ src,
                                                         size_t footprint, int iters,
                                                         size_t row_stride, int layout, float* out,
                                                         Clk* clk) {
  extern __shared__ __align__(16) char smc[];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smc +
                  wv * (DEPTH + 1) * 1024;
  base = __builtin_amdgcn_readfirstlane(base);
  // a wave walks whole row blocks (rows x row_stride bytes) and then moves on by the number
  // of waves in the grid, so the grid streams through the entire footprint
  const size_t wave_id = (size_t)blockIdx.x * NW + wv, n_waves = (size_t)gridDim.x * NW;
  const int rows = layout == 1 ? 32 : 16;
  const size_t blk_bytes = rows * row_stride, n_blk = footprint / blk_bytes;
  const size_t lane_off = layout != 1 ? (size_t)(lane >> 2) * row_stride + (lane & 3) * 16
                                      : (size_t)(lane & 31) * row_stride + (lane >> 5) * 16;
  const size_t kstep = layout == 0 ? 64 : (layout == 1 ? 32 : 128);
  size_t k = 0, blk = wave_id % n_blk;
  const char* p = src + blk * blk_bytes + lane_off;
  auto advance = [&]() {
    k += kstep;
    if (k >= row_stride) {
      k = 0;
      blk = (blk + n_waves) % n_blk;
      p = src + blk * blk_bytes + lane_off;
    }
  };
  uint4 acc = make_uint4(0, 0, 0, 0);
  const uint64_t c0 = shader_clock(), r0 = real_clock();
  if (TO_LDS) {
    for (int it = 0; it < iters; ++it) {
      if constexpr (POLICY == 0) dma16(p + k, base + (it % (DEPTH + 1)) * 1024);
      else dma16_policy<POLICY>(p + k, base + (it % (DEPTH + 1)) * 1024);
      advance();
      wait_vm<DEPTH>();
    }
    wait_vm<0>();
  } else {
    for (int it = 0; it < iters; it += DEPTH) {
      uint4 v[DEPTH];
#pragma unroll
      for (int u = 0; u < DEPTH; ++u) {
        v[u] = *reinterpret_cast<const uint4*>(p + k);
        advance();
      }
#pragma unroll
      for (int u = 0; u < DEPTH; ++u) {
        acc.x ^= v[u].x;
        acc.y ^= v[u].y;
        acc.z ^= v[u].z;
        acc.w ^= v[u].w;
      }
    }
  }
  const uint64_t c1 = shader_clock(), r1 = real_clock();
  __syncthreads();
  out[blockIdx.x * NW * 64 + threadIdx.x] =
      (float)(acc.x ^ acc.y ^ acc.z ^ acc.w) + (TO_LDS ? (float)smc[threadIdx.x * 4] : 0.0f);
  if (blockIdx.x == 0 && threadIdx.x == 0) *clk = Clk{c1 - c0, r1 - r0};
}

// ------------------------------------------------------------------ completion latencies
// One wave per workgroup: cycles from issuing (mode 0) a 16-byte-per-lane store to rows 4 KiB
// apart, (mode 1) a global->LDS copy of the same shape, (mode 2) the store followed by the
// copy, until s_waitcnt vmcnt(0) returns.  vmcnt retires in issue order, so mode 2 shows how
// long a copy issued behind a store is held back by that store's acknowledgement.  Averaged
// over `iters` rounds, each on fresh addresses; reported in shader cycles.
__global__ __launch_bounds__(64) void latency_kernel(char* __restrict__ buf, size_t span, int iters,
                                                     int mode, float* out, Clk* clk) {
  extern __shared__ __align__(16) char smc[];
  const int lane = threadIdx.x;
  const uint32_t lds = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smc);
  uint64_t total = 0;
  const uint64_t r0 = real_clock(), c00 = shader_clock();
  for (int it = 0; it < iters; ++it) {
    const size_t blk = ((size_t)blockIdx.x * iters + it) * (64 * 4096) % span;
    char* st = buf + blk + (size_t)(lane >> 1) * 4096 + (lane & 1) * 16;            // 32 rows x 32 bytes
    const char* ld = buf + span + blk + (size_t)(lane >> 2) * 4096 + (lane & 3) * 16;  // 16 rows x 64 bytes
    const uint4 v = make_uint4(lane, it, 2, 3);
    wait_vm<0>();
    const uint64_t c0 = shader_clock();
    if (mode != 1) *reinterpret_cast<uint4*>(st) = v;
    if (mode != 0) dma16(ld, lds);
    wait_vm<0>();
    total += shader_clock() - c0;
  }
  const uint64_t c1 = shader_clock(), r1 = real_clock();
  if (lane == 0) out[blockIdx.x] = (float)total / iters;
  if (blockIdx.x == 0 && lane == 0) *clk = Clk{c1 - c00, r1 - r0};
}

// ------------------------------------------------------------------ HBM streaming copy
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src,
                                                   uint4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += 4 * stride) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * stride < n) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * stride < n) dst[i + u * stride] = v[u];
  }
}

// read-only and write-only HBM streams (every thread 16 bytes per step, grid-strided)
__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ src, size_t n, float* out) {
  const size_t stride = (size_t)gridDim.x * 256;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += 4 * stride) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = i + u * stride < n ? src[i + u * stride] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      acc.x ^= v[u].x;
      acc.y ^= v[u].y;
      acc.z ^= v[u].z;
      acc.w ^= v[u].w;
    }
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1.0f;  // keeps the loads alive
}
__global__ __launch_bounds__(256) void write_kernel(uint4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  const uint4 v = make_uint4(threadIdx.x, 1, 2, 3);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = v;
}

// The fused FFN kernel's output pattern: a workgroup of 8 waves owns 256 consecutive rows of
// `row_bytes` each and walks along them in steps of `seg` bytes per row (a wave: 32 rows,
// 8 or more lanes per row segment), so consecutive stores of a wave are row_bytes apart; after
// row_bytes / seg steps it moves on to its next 256 rows.
__global__ __launch_bounds__(512) void write_tiles_kernel(char* __restrict__ dst, size_t n_rows,
                                                          int row_bytes, int seg) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int lanes_per_row = seg / 16, rows_per_store = 64 / lanes_per_row;
  const uint4 v = make_uint4(threadIdx.x, 1, 2, 3);
  for (size_t tile = blockIdx.x; tile * 256 + 256 <= n_rows; tile += gridDim.x) {
    char* base = dst + (tile * 256 + wv * 32) * (size_t)row_bytes;
    for (int s = 0; s < row_bytes / seg; ++s)
      for (int r0 = 0; r0 < 32; r0 += rows_per_store) {
        const int r = r0 + lane / lanes_per_row;
        *reinterpret_cast<uint4*>(base + (size_t)r * row_bytes + (size_t)s * seg + (lane % lanes_per_row) * 16) = v;
      }
  }
}

struct Bufs {
  char* big = nullptr;  // 3 GiB source region, 1 GiB destination behind it
  float* out = nullptr;
  uint4* data[2] = {nullptr, nullptr};  // 64 KiB of operand bits: [0] small integers, [1] random
  Clk* clk = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
};
constexpr size_t SRC_BYTES = (size_t)3 << 30, DST_BYTES = (size_t)1 << 30;

static bool setup(Bufs& b) {
  if (hipMalloc(&b.big, SRC_BYTES + DST_BYTES) != hipSuccess) return false;
  if (hipMemset(b.big, 1, SRC_BYTES + DST_BYTES) != hipSuccess) return false;
  if (hipMalloc(&b.out, 64 << 20) != hipSuccess) return false;
  if (hipMalloc(&b.clk, sizeof(Clk)) != hipSuccess) return false;
  // operand bits: bf16 small integers 0..3, and pseudo-random bf16 in roughly N(0,1)
  // (sum of four uniforms from a 64-bit LCG; measurement data, not the method's RNG)
  std::vector<uint16_t> h(32768);
  for (int v = 0; v < 2; ++v) {
    uint64_t s = 0x9E3779B97F4A7C15ull;
    for (size_t i = 0; i < h.size(); ++i) {
      float f;
      if (v == 0) {
        f = (float)(i & 3);
      } else {
        float u = 0.0f;
        for (int q = 0; q < 4; ++q) {
          s = s * 6364136223846793005ull + 1442695040888963407ull;
          u += (float)((s >> 40) & 0xFFFF) / 65536.0f;
        }
        f = (u - 2.0f) * 1.7320508f;
      }
      uint32_t bits;
      __builtin_memcpy(&bits, &f, 4);
      h[i] = (uint16_t)((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16);
    }
    if (hipMalloc(&b.data[v], 65536) != hipSuccess) return false;
    if (hipMemcpy(b.data[v], h.data(), 65536, hipMemcpyHostToDevice) != hipSuccess) return false;
  }
  return hipEventCreate(&b.e0) == hipSuccess && hipEventCreate(&b.e1) == hipSuccess;
}
static void teardown(Bufs& b) {
  (void)hipDeviceSynchronize();
  if (b.big) (void)hipFree(b.big);
  if (b.out) (void)hipFree(b.out);
  if (b.clk) (void)hipFree(b.clk);
  for (int v = 0; v < 2; ++v)
    if (b.data[v]) (void)hipFree(b.data[v]);
  if (b.e0) (void)hipEventDestroy(b.e0);
  if (b.e1) (void)hipEventDestroy(b.e1);
}

// runs `launch` once untimed and `reps` times timed; ms = average, mhz = shader clock of the last run
template <class F>
static bool timed(Bufs& b, int reps, F launch, double* ms, double* mhz) {
  launch();
  if (hipDeviceSynchronize() != hipSuccess) return false;
  (void)hipEventRecord(b.e0, nullptr);
  for (int i = 0; i < reps; ++i) launch();
  (void)hipEventRecord(b.e1, nullptr);
  if (hipEventSynchronize(b.e1) != hipSuccess || hipGetLastError() != hipSuccess) return false;
  float t = 0.0f;
  (void)hipEventElapsedTime(&t, b.e0, b.e1);
  *ms = t / reps;
  Clk c{0, 0};
  (void)hipMemcpy(&c, b.clk, sizeof(c), hipMemcpyDeviceToHost);
  *mhz = c.real ? 100.0 * (double)c.shader / (double)c.real : 0.0;
  return true;
}

template <int MB, int NB, int WM, int WN, int per_cu>
static bool run_lds_mfma(Bufs& b, int ncu, int variant, double* tflops, double* mhz) {
  constexpr size_t lds = 2ull * (WM * MB * 32 + WN * NB * 32) * 64;
  auto kern = mfma_lds_kernel<MB, NB, WM, WN, per_cu * WM * WN / 4>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    return false;
  const int iters = 4000, grid = ncu * per_cu;
  double ms = 0;
  if (!timed(b, 3, [&] { kern<<<grid, WM * WN * 64, lds>>>(b.data[variant], b.out, iters, b.clk); },
             &ms, mhz))
    return false;
  *tflops = 2.0 * 32 * 32 * 32 * MB * NB * WM * WN * (double)iters * grid / (ms * 1e-3) / 1e12;
  return true;
}

template <int DEPTH, int NW, bool TO_LDS, int POLICY = 0>
static bool run_stream(Bufs& b, int ncu, size_t footprint, int layout, double* tbs, double* mhz) {
  auto kern = stream_kernel<DEPTH, NW, TO_LDS, POLICY>;
  const size_t lds = (size_t)NW * (DEPTH + 1) * 1024;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    return false;
  const int iters = 4096;
  double ms = 0;
  if (!timed(b, 3, [&] { kern<<<ncu, NW * 64, lds>>>(b.big, footprint, iters, 4096, layout, b.out, b.clk); },
             &ms, mhz))
    return false;
  *tbs = (double)ncu * NW * iters * 1024 / (ms * 1e-3) / 1e12;
  return true;
}

}  // namespace mpub

using namespace mpub;

extern "C" int moe_prism_microbench(int32_t max_results, moe_prism_microbench_result* results,
                                    int32_t* n_results) {
  if (results == nullptr || n_results == nullptr || max_results < 0) return MOE_PRISM_ERR_INVALID_ARG;
  *n_results = 0;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
    return MOE_PRISM_ERR_LAUNCH;
  const int ncu = prop.multiProcessorCount;
  Bufs b;
  if (!setup(b)) {
    teardown(b);
    return MOE_PRISM_ERR_LAUNCH;
  }
  bool ok = true;
  auto put = [&](const char* name, double value, const char* unit, double mhz) {
    if (*n_results >= max_results) return;
    moe_prism_microbench_result& r = results[*n_results];
    __builtin_strncpy(r.name, name, sizeof(r.name) - 1);
    r.name[sizeof(r.name) - 1] = 0;
    __builtin_strncpy(r.unit, unit, sizeof(r.unit) - 1);
    r.unit[sizeof(r.unit) - 1] = 0;
    r.value = value;
    r.shader_mhz = mhz;
    ++*n_results;
  };
  double v = 0, mhz = 0, ms = 0;
  const char* dname[2] = {"const", "random"};
  char nm[64];

  // 1. register-resident MFMA
  for (int var = 0; var < 2 && ok; ++var) {
    const int iters = 20000, grid = ncu;  // one wave per SIMD
    ok = timed(b, 3, [&] { mfma_reg_kernel<4><<<grid, 256>>>(b.data[var], b.out, iters, b.clk); }, &ms, &mhz);
    v = 2.0 * 32 * 32 * 16 * 4 * (double)iters * grid * 4 / (ms * 1e-3) / 1e12;
    __builtin_snprintf(nm, sizeof(nm), "mfma_32x32x16_bf16_registers_%s_1wave_per_simd", dname[var]);
    put(nm, v, "TFLOP/s", mhz);
    if (!ok) break;
    ok = timed(b, 3, [&] { mfma_reg_kernel<4><<<2 * grid, 256>>>(b.data[var], b.out, iters, b.clk); }, &ms, &mhz);
    v = 2.0 * 32 * 32 * 16 * 4 * (double)iters * grid * 8 / (ms * 1e-3) / 1e12;
    __builtin_snprintf(nm, sizeof(nm), "mfma_32x32x16_bf16_registers_%s_2waves_per_simd", dname[var]);
    put(nm, v, "TFLOP/s", mhz);
  }
  // 1b. the rank-1 fp32 form of the logits kernel: two chains per wave, two waves per SIMD
  for (int var = 0; var < 2 && ok; ++var) {
    const int iters = 20000, grid = 2 * ncu;
    ok = timed(b, 3, [&] { mfma_f32_rank1_kernel<2><<<grid, 256>>>(b.data[var], b.out, iters, b.clk); }, &ms, &mhz);
    v = 2.0 * 32 * 64 * 2 * (double)iters * grid * 4 / (ms * 1e-3) / 1e12;
    __builtin_snprintf(nm, sizeof(nm), "mfma_32x32x1_2b_f32_registers_%s_2waves_per_simd", dname[var]);
    put(nm, v, "TFLOP/s", mhz);
  }
  // long run (about 2 ms) and a run as short as the logits kernel at 16K tokens x 512 sub-experts
  for (int var = 0; var < 4 && ok; ++var) {
    const int iters = var < 2 ? 640 : 64, grid = 2 * ncu;
    ok = timed(b, 3, [&] { mfma_f32_rank1_many_operands_kernel<<<grid, 256>>>(b.data[var & 1], b.out, iters, b.clk); }, &ms, &mhz);
    v = 2.0 * 32 * 64 * 64 * (double)iters * grid * 4 / (ms * 1e-3) / 1e12;
    __builtin_snprintf(nm, sizeof(nm), "mfma_32x32x1_2b_f32_32_operand_pairs_%s_2waves_per_simd%s", dname[var & 1],
                       var < 2 ? "" : "_0.2ms_run");
    put(nm, v, "TFLOP/s", mhz);
  }
  // 2. LDS-fed MFMA, wave tiles of the FFN kernels and larger ones
  for (int var = 0; var < 2 && ok; ++var) {
#define LDS_MFMA(MB, NB, WM, WN, PER_CU, LABEL)                                     \
  if (ok) {                                                                        \
    ok = run_lds_mfma<MB, NB, WM, WN, PER_CU>(b, ncu, var, &v, &mhz);               \
    __builtin_snprintf(nm, sizeof(nm), "mfma_lds_fed_%s_%s", LABEL, dname[var]);    \
    put(nm, v, "TFLOP/s", mhz);                                                    \
  }
    LDS_MFMA(2, 3, 4, 2, 1, "wave64x96_8waves")
    LDS_MFMA(2, 4, 4, 2, 1, "wave64x128_8waves")
    LDS_MFMA(4, 3, 1, 4, 1, "wave128x96_4waves")
    LDS_MFMA(4, 3, 1, 4, 2, "wave128x96_2x4waves")
    LDS_MFMA(4, 2, 1, 4, 2, "wave128x64_2x4waves")
    LDS_MFMA(4, 4, 2, 2, 1, "wave128x128_4waves")
    LDS_MFMA(1, 12, 8, 1, 1, "wave32x384_8waves")
#undef LDS_MFMA
  }
  // 3. LDS read bandwidth
  if (ok) {
    const int iters = 20000;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(lds_read_kernel<512, 8>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
    ok = timed(b, 3, [&] { lds_read_kernel<512, 8><<<ncu, 512, 32768>>>(b.out, iters, b.clk); }, &ms, &mhz);
    v = 1024.0 * 8 * 8 * iters * ncu / (ms * 1e-3) / 1e12;
    put("lds_read_b128_8waves", v, "TB/s", mhz);
    if (mhz > 0) put("lds_read_b128_8waves_per_cu", v * 1e12 / ncu / (mhz * 1e6), "B/clk/CU", mhz);
  }
  if (ok) {
    const int iters = 20000;
    ok = timed(b, 3, [&] { lds_read_kernel<256, 8><<<ncu, 256, 32768>>>(b.out, iters, b.clk); }, &ms, &mhz);
    v = 1024.0 * 8 * 4 * iters * ncu / (ms * 1e-3) / 1e12;
    put("lds_read_b128_4waves", v, "TB/s", mhz);
    if (mhz > 0) put("lds_read_b128_4waves_per_cu", v * 1e12 / ncu / (mhz * 1e6), "B/clk/CU", mhz);
  }
  // 4. operand streams from L2 / last-level cache / HBM
  const size_t fps[3] = {(size_t)2 << 20, (size_t)128 << 20, SRC_BYTES};
  const char* fpn[3] = {"l2_2MiB", "llc_128MiB", "hbm_3GiB"};
  for (int f = 0; f < 3 && ok; ++f) {
    ok = run_stream<16, 8, true>(b, ncu, fps[f], 0, &v, &mhz);
    __builtin_snprintf(nm, sizeof(nm), "global_to_lds_dwordx4_%s", fpn[f]);
    put(nm, v, "TB/s", mhz);
    if (!ok) break;
    ok = run_stream<16, 8, true>(b, ncu, fps[f], 2, &v, &mhz);
    __builtin_snprintf(nm, sizeof(nm), "global_to_lds_dwordx4_first_half_of_each_line_%s", fpn[f]);
    put(nm, v, "TB/s", mhz);
    if (!ok) break;
    const char* pol[5] = {"", "sc0", "sc1", "sc0_sc1", "nt"};
    for (int q = 1; q <= 4 && ok && f == 0; ++q) {  // cache-policy modifiers, L2-resident footprint
      if (q == 1) ok = run_stream<16, 8, true, 1>(b, ncu, fps[f], 2, &v, &mhz);
      if (q == 2) ok = run_stream<16, 8, true, 2>(b, ncu, fps[f], 2, &v, &mhz);
      if (q == 3) ok = run_stream<16, 8, true, 3>(b, ncu, fps[f], 2, &v, &mhz);
      if (q == 4) ok = run_stream<16, 8, true, 4>(b, ncu, fps[f], 2, &v, &mhz);
      __builtin_snprintf(nm, sizeof(nm), "global_to_lds_dwordx4_first_half_of_each_line_%s_%s", pol[q], fpn[f]);
      put(nm, v, "TB/s", mhz);
    }
    if (!ok) break;
    ok = run_stream<8, 8, false>(b, ncu, fps[f], 0, &v, &mhz);
    __builtin_snprintf(nm, sizeof(nm), "global_to_regs_dwordx4_rows_of_4_lanes_%s", fpn[f]);
    put(nm, v, "TB/s", mhz);
    if (!ok) break;
    ok = run_stream<8, 8, false>(b, ncu, fps[f], 1, &v, &mhz);
    __builtin_snprintf(nm, sizeof(nm), "global_to_regs_dwordx4_row_per_lane_%s", fpn[f]);
    put(nm, v, "TB/s", mhz);
    if (!ok) break;
    ok = run_stream<8, 4, false>(b, ncu, fps[f], 1, &v, &mhz);
    __builtin_snprintf(nm, sizeof(nm), "global_to_regs_dwordx4_row_per_lane_4waves_%s", fpn[f]);
    put(nm, v, "TB/s", mhz);
  }
  // 4b. completion latency of a store, a copy, and a copy behind a store: one wave alone on the
  // chip, and one wave on every CU at once
  for (int load = 0; load < 2 && ok; ++load) {
    const char* mname[3] = {"store_16B_rows_ack", "global_to_lds_copy", "copy_issued_behind_store"};
    for (int mode = 0; mode < 3 && ok; ++mode) {
      const int grid = load ? ncu : 1, iters = 2000;
      ok = timed(b, 1, [&] { latency_kernel<<<grid, 64, 1024>>>(b.big, (size_t)1 << 30, iters, mode, b.out, b.clk); }, &ms, &mhz);
      std::vector<float> h(grid);
      (void)hipMemcpy(h.data(), b.out, grid * sizeof(float), hipMemcpyDeviceToHost);
      double sum = 0;
      for (float f : h) sum += f;
      __builtin_snprintf(nm, sizeof(nm), "latency_%s_%s", mname[mode], load ? "all_cus" : "one_wave");
      put(nm, sum / grid, "cycles", mhz);
    }
  }
  // 5. HBM streaming copy, 1 GiB
  if (ok) {
    const size_t n = DST_BYTES / 16;
    ok = timed(b, 5, [&] {
      copy_kernel<<<ncu * 8, 256>>>(reinterpret_cast<const uint4*>(b.big),
                                    reinterpret_cast<uint4*>(b.big + SRC_BYTES), n);
    }, &ms, &mhz);
    put("hbm_copy_1GiB_read_plus_write", 2.0 * DST_BYTES / (ms * 1e-3) / 1e12, "TB/s", 0.0);
  }
  if (ok) {
    const size_t n = SRC_BYTES / 16;
    ok = timed(b, 5, [&] { read_kernel<<<ncu * 8, 256>>>(reinterpret_cast<const uint4*>(b.big), n, b.out); }, &ms, &mhz);
    put("hbm_read_3GiB", (double)SRC_BYTES / (ms * 1e-3) / 1e12, "TB/s", 0.0);
  }
  if (ok) {
    const size_t n = DST_BYTES / 16;
    ok = timed(b, 5, [&] { write_kernel<<<ncu * 8, 256>>>(reinterpret_cast<uint4*>(b.big + SRC_BYTES), n); }, &ms, &mhz);
    put("hbm_write_1GiB", (double)DST_BYTES / (ms * 1e-3) / 1e12, "TB/s", 0.0);
  }
  for (int seg = 64; seg <= 1024 && ok; seg *= 2) {
    const size_t rows = DST_BYTES / 4096;
    ok = timed(b, 5, [&] { write_tiles_kernel<<<ncu, 512>>>(b.big + SRC_BYTES, rows, 4096, seg); }, &ms, &mhz);
    __builtin_snprintf(nm, sizeof(nm), "hbm_write_1GiB_tiles_256rows_x_%dB_per_step", seg);
    put(nm, (double)DST_BYTES / (ms * 1e-3) / 1e12, "TB/s", 0.0);
  }
  teardown(b);
  return ok ? MOE_PRISM_OK : MOE_PRISM_ERR_LAUNCH;
}
