// Grouped SwiGLU FFN over ragged per-sub-expert groups (Sec. 3.2.1, Eq. 1-3).
//
// The slot list is cut into m-tiles of FFN_BM rows that never straddle a
// group (ffn_tiles_kernel, on the device, from group_offset), and persistent
// workgroups walk (m-tile, n-tile) work items round-robin.  Two GEMMs:
//   gate-up : h[p, c] = SiLU(x[t_p,:] . Wg[g,c,:]) * (x[t_p,:] . Wu[g,c,:])
//   down    : y[p, q] = sum_c h[p,c] * Wd[g,q,c]
// bf16: 128x128 output tiles on v_mfma_f32_32x32x16_bf16, operands staged
// through XOR-swizzled LDS, fp32 accumulation.  fp32: plain FMA tiles.
#include "kernels.h"

namespace mp {

// ---------------------------------------------------------------- m-tile table
constexpr int TILES_THREADS = 1024;
__global__ __launch_bounds__(TILES_THREADS) void ffn_tiles_kernel(const int32_t* __restrict__ off,
                                                                  MTile* __restrict__ tiles,
                                                                  int32_t* __restrict__ hdr, int E,
                                                                  int max_tiles, int n_rows) {
  __shared__ int32_t wave_tot[TILES_THREADS / 64];
  __shared__ int32_t carry;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int g0 = 0; g0 < E; g0 += TILES_THREADS) {
    int g = g0 + tid;
    int lo = 0, n = 0;
    if (g < E) {  // offsets that do not describe a slot list of n_rows rows yield no tiles
      lo = off[g];
      n = off[g + 1] - lo;
      if (lo < 0 || n < 0 || lo > n_rows || n > n_rows - lo) n = 0;
    }
    int nt = (n + FFN_BM - 1) / FFN_BM;
    int incl = nt;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
      int o = __shfl_up(incl, m, 64);
      if (lane >= m) incl += o;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    int wbase = 0;
    for (int i = 0; i < wv; ++i) wbase += wave_tot[i];
    int first = carry + wbase + incl - nt;
    for (int i = 0; i < nt; ++i) {
      MTile t;
      t.g = g;
      t.row0 = lo + i * FFN_BM;
      t.rows = min(FFN_BM, n - i * FFN_BM);
      t.pad = 0;
      if (first + i < max_tiles) tiles[first + i] = t;
    }
    __syncthreads();
    if (tid == TILES_THREADS - 1) carry = first + nt;
    __syncthreads();
  }
  if (tid == 0) hdr[HDR_MTILES] = min(carry, max_tiles);
}

hipError_t launch_ffn_tiles(const int32_t* off, MTile* tiles, int32_t* hdr, int E, int max_tiles,
                            int n_rows, hipStream_t s) {
  ffn_tiles_kernel<<<1, TILES_THREADS, 0, s>>>(off, tiles, hdr, E, max_tiles, n_rows);
  return hipGetLastError();
}

// ---------------------------------------------------------------- bf16 MFMA tile core
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BK = 64;                      // bf16 elements of K per LDS slab (128 bytes per row)
constexpr int TILE = 128;                   // output tile is TILE x TILE
constexpr int SLAB = TILE * BK;             // bf16 elements of one operand slab

struct __align__(16) Smem {  // 64 KiB: two workgroups fit in a CU's 160 KiB LDS
  uint16_t a[2][SLAB];
  uint16_t b[2][SLAB];
};

// 16-byte chunk c (0..7) of row r lives at chunk position c ^ (r & 7): rows that
// are 1..7 apart never collide on the same LDS banks for the MFMA fragment reads.
__device__ __forceinline__ int swz(int r, int c) { return r * BK + ((c ^ (r & 7)) << 3); }

// acc[mi][ni] (+)= A[128 x K] * B[128 x K]^T for this wave's 64 x 64 quadrant.
// a_base + a_row(r) + k and b_base + b_row(r) + k address K-contiguous bf16 rows
// (r = 0..127 inside the tile).  K is padded with zeros up to a multiple of BK.
// Ends with a barrier, so the caller may start the next tile right away.
template <class ARow, class BRow>
__device__ __forceinline__ void mfma_tile(const uint16_t* __restrict__ a_base,
                                          const uint16_t* __restrict__ b_base, int K, Smem& sm,
                                          f32x16 (&acc)[2][2], ARow a_row, BRow b_row) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  const int lc = tid & 7, lr = tid >> 3;  // loader: chunk lc of rows lr + 32*i

  const uint16_t* ap[4];
  const uint16_t* bp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ap[i] = a_base + a_row(lr + 32 * i) + lc * 8;
    bp[i] = b_base + b_row(lr + 32 * i) + lc * 8;
  }
  uint4 ra[4], rb[4];
  auto gload = [&](int k0) {
    bool in = k0 + lc * 8 < K;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ra[i] = in ? *reinterpret_cast<const uint4*>(ap[i] + k0) : make_uint4(0, 0, 0, 0);
      rb[i] = in ? *reinterpret_cast<const uint4*>(bp[i] + k0) : make_uint4(0, 0, 0, 0);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int r = lr + 32 * i;
      *reinterpret_cast<uint4*>(&sm.a[buf][swz(r, lc)]) = ra[i];
      *reinterpret_cast<uint4*>(&sm.b[buf][swz(r, lc)]) = rb[i];
    }
  };

  const int nslab = (K + BK - 1) / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    if (s + 1 < nslab) gload((s + 1) * BK);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int c = ks * 2 + (lane >> 5);
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        int ra_ = wm * 64 + i * 32 + (lane & 31);
        int rb_ = wn * 64 + i * 32 + (lane & 31);
        fa[i] = *reinterpret_cast<const bf16x8*>(&sm.a[buf][swz(ra_, c)]);
        fb[i] = *reinterpret_cast<const bf16x8*>(&sm.b[buf][swz(rb_, c)]);
      }
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] =
              __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
    }
    if (s + 1 < nslab) sstore(buf ^ 1);
    __syncthreads();
  }
}

// Row / column of accumulator element v of lane `lane` inside a 32 x 32 MFMA block.
__device__ __forceinline__ int acc_row(int lane, int v) {
  return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

__device__ __forceinline__ float silu_mul(float a, float u) {
  return __fdividef(a, 1.0f + __expf(-a)) * u;
}

// gate-up.  B rows of a tile are laid out so that each wave's 64-column quadrant
// holds 32 gate neurons (ni = 0) and the 32 matching up neurons (ni = 1).
constexpr int GU_BN = 64;  // neurons per n-tile
__global__ __launch_bounds__(256) void ffn_gate_up_bf16_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_gu,
    const int32_t* __restrict__ sorted_pair, const MTile* __restrict__ tiles,
    const int32_t* __restrict__ hdr, uint16_t* __restrict__ h, int d, int Is, int k_max, int T) {
  __shared__ Smem sm;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  const int NT = (Is + GU_BN - 1) / GU_BN;
  const int total = hdr[HDR_MTILES] * NT;
  for (int item = blockIdx.x; item < total; item += gridDim.x) {
    const MTile tl = tiles[item / NT];
    const int n0 = (item % NT) * GU_BN;
    auto a_row = [&](int r) {
      int tok = sorted_pair[tl.row0 + min(r, tl.rows - 1)] / k_max;
      return (long long)min(max(tok, 0), T - 1) * d;
    };
    auto b_row = [&](int r) {
      int q = r >> 6, ni = (r >> 5) & 1, j = r & 31;
      int neuron = min(n0 + q * 32 + j, Is - 1);
      return ((long long)tl.g * 2 * Is + (ni ? Is + neuron : neuron)) * d;
    };
    f32x16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
    mfma_tile(x, w_gu, d, sm, acc, a_row, b_row);
    const int col = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int row = wm * 64 + mi * 32 + acc_row(lane, v);
        if (row < tl.rows && col < Is)
          h[(size_t)(tl.row0 + row) * Is + col] = f32_to_bf16(silu_mul(acc[mi][0][v], acc[mi][1][v]));
      }
  }
}

__global__ __launch_bounds__(256) void ffn_down_bf16_kernel(
    const uint16_t* __restrict__ h, const uint16_t* __restrict__ w_dn,
    const MTile* __restrict__ tiles, const int32_t* __restrict__ hdr, uint16_t* __restrict__ y,
    int d, int Is) {
  __shared__ Smem sm;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  const int NT = (d + TILE - 1) / TILE;
  const int total = hdr[HDR_MTILES] * NT;
  for (int item = blockIdx.x; item < total; item += gridDim.x) {
    const MTile tl = tiles[item / NT];
    const int n0 = (item % NT) * TILE;
    auto a_row = [&](int r) { return (long long)(tl.row0 + min(r, tl.rows - 1)) * Is; };
    auto b_row = [&](int r) { return ((long long)tl.g * d + min(n0 + r, d - 1)) * Is; };
    f32x16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
    mfma_tile(h, w_dn, Is, sm, acc, a_row, b_row);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        int col = n0 + wn * 64 + ni * 32 + (lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int row = wm * 64 + mi * 32 + acc_row(lane, v);
          if (row < tl.rows && col < d)
            y[(size_t)(tl.row0 + row) * d + col] = f32_to_bf16(acc[mi][ni][v]);
        }
      }
  }
}

// ---------------------------------------------------------------- fp32 tiles (small reference-quality path)
// 128 x 128 output tile, 256 threads, 8 x 8 outputs per thread, K slabs of 16.
constexpr int FK = 16;
struct SmemF {
  float a[FK][TILE + 4];
  float b[FK][TILE + 4];
  long long a_off[TILE];
  long long b_off[TILE];
};

__device__ __forceinline__ void f32_tile(const float* __restrict__ a_base,
                                         const float* __restrict__ b_base, int K, SmemF& sm,
                                         float (&acc)[8][8]) {
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int lr = tid >> 1, lk = (tid & 1) * 8;  // loader: 8 floats of row lr
  for (int k0 = 0; k0 < K; k0 += FK) {
    float va[8], vb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      bool in = k0 + lk + e < K;
      va[e] = in ? a_base[sm.a_off[lr] + k0 + lk + e] : 0.0f;
      vb[e] = in ? b_base[sm.b_off[lr] + k0 + lk + e] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sm.a[lk + e][lr] = va[e];
      sm.b[lk + e][lr] = vb[e];
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < FK; ++kk) {
      float a[8], b[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        a[i] = sm.a[kk][(i >> 2) * 64 + ty * 4 + (i & 3)];
        b[i] = sm.b[kk][(i >> 2) * 64 + tx * 4 + (i & 3)];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
  }
  __syncthreads();
}

// B columns 0..63 of a tile are gate neurons n0.., columns 64..127 the matching up neurons.
__global__ __launch_bounds__(256) void ffn_gate_up_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ w_gu,
    const int32_t* __restrict__ sorted_pair, const MTile* __restrict__ tiles,
    const int32_t* __restrict__ hdr, float* __restrict__ h, int d, int Is, int k_max, int T) {
  __shared__ SmemF sm;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int NT = (Is + 63) / 64;
  const int total = hdr[HDR_MTILES] * NT;
  for (int item = blockIdx.x; item < total; item += gridDim.x) {
    const MTile tl = tiles[item / NT];
    const int n0 = (item % NT) * 64;
    if (tid < TILE) {
      int r = min(tid, tl.rows - 1);
      sm.a_off[tid] = (long long)min(max(sorted_pair[tl.row0 + r] / k_max, 0), T - 1) * d;
      int neuron = min(n0 + (tid & 63), Is - 1);
      sm.b_off[tid] = ((long long)tl.g * 2 * Is + (tid >= 64 ? Is + neuron : neuron)) * d;
    }
    __syncthreads();
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = 0.0f;
    f32_tile(x, w_gu, d, sm, acc);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int row = (i >> 2) * 64 + ty * 4 + (i & 3);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int col = n0 + tx * 4 + j;
        if (row < tl.rows && col < Is) {
          float a = acc[i][j], u = acc[i][j + 4];
          h[(size_t)(tl.row0 + row) * Is + col] = a / (1.0f + expf(-a)) * u;
        }
      }
    }
  }
}

__global__ __launch_bounds__(256) void ffn_down_f32_kernel(const float* __restrict__ h,
                                                           const float* __restrict__ w_dn,
                                                           const MTile* __restrict__ tiles,
                                                           const int32_t* __restrict__ hdr,
                                                           float* __restrict__ y, int d, int Is) {
  __shared__ SmemF sm;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int NT = (d + TILE - 1) / TILE;
  const int total = hdr[HDR_MTILES] * NT;
  for (int item = blockIdx.x; item < total; item += gridDim.x) {
    const MTile tl = tiles[item / NT];
    const int n0 = (item % NT) * TILE;
    if (tid < TILE) {
      int r = min(tid, tl.rows - 1);
      sm.a_off[tid] = (long long)(tl.row0 + r) * Is;
      sm.b_off[tid] = ((long long)tl.g * d + min(n0 + tid, d - 1)) * Is;
    }
    __syncthreads();
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = 0.0f;
    f32_tile(h, w_dn, Is, sm, acc);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int row = (i >> 2) * 64 + ty * 4 + (i & 3);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        int col = n0 + (j >> 2) * 64 + tx * 4 + (j & 3);
        if (row < tl.rows && col < d) y[(size_t)(tl.row0 + row) * d + col] = acc[i][j];
      }
    }
  }
}

// ---------------------------------------------------------------- launchers
static int persistent_grid(int max_items, int per_cu) {
  int g = num_cus() * per_cu;
  if (g > max_items) g = max_items;
  return g < 1 ? 1 : g;
}

hipError_t launch_ffn_gate_up(int dtype, const void* x, const void* w_gu, const int32_t* sorted_pair,
                              const MTile* tiles, const int32_t* hdr, void* h, int T, int d, int Is,
                              int k_max, int max_mtiles, hipStream_t s) {
  if (max_mtiles <= 0) return hipSuccess;
  long items = (long)max_mtiles * cdiv(Is, 64);
  if (dtype == 0) {
    int grid = persistent_grid((int)min(items, 1L << 30), 2);
    ffn_gate_up_f32_kernel<<<grid, 256, 0, s>>>((const float*)x, (const float*)w_gu, sorted_pair,
                                                tiles, hdr, (float*)h, d, Is, k_max, T);
  } else {
    int grid = persistent_grid((int)min(items, 1L << 30), 2);
    ffn_gate_up_bf16_kernel<<<grid, 256, 0, s>>>((const uint16_t*)x, (const uint16_t*)w_gu,
                                                 sorted_pair, tiles, hdr, (uint16_t*)h, d, Is, k_max,
                                                 T);
  }
  return hipGetLastError();
}

hipError_t launch_ffn_down(int dtype, const void* h, const void* w_dn, const MTile* tiles,
                           const int32_t* hdr, void* y, int d, int Is, int max_mtiles,
                           hipStream_t s) {
  if (max_mtiles <= 0) return hipSuccess;
  long items = (long)max_mtiles * cdiv(d, TILE);
  int grid = persistent_grid((int)min(items, 1L << 30), 2);
  if (dtype == 0)
    ffn_down_f32_kernel<<<grid, 256, 0, s>>>((const float*)h, (const float*)w_dn, tiles, hdr,
                                             (float*)y, d, Is);
  else
    ffn_down_bf16_kernel<<<grid, 256, 0, s>>>((const uint16_t*)h, (const uint16_t*)w_dn, tiles, hdr,
                                              (uint16_t*)y, d, Is);
  return hipGetLastError();
}

}  // namespace mp
