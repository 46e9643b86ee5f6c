// Grouped SwiGLU FFN over ragged per-sub-expert groups (Sec. 3.2.1, Eq. 1-3).
//
// The slot list is cut into m-tiles of FFN_BM rows that never straddle a
// group (ffn_tiles_kernel, on the device, from group_offset), and persistent
// workgroups walk (m-tile, n-tile) work items round-robin.  Two GEMMs:
//   gate-up : h[p, c] = SiLU(x[t_p,:] . Wg[g,c,:]) * (x[t_p,:] . Wu[g,c,:])
//   down    : y[p, q] = sum_c h[p,c] * Wd[g,q,c]
// This file: the m-tile table and the fp32 path (plain FMA tiles, reference
// quality, small shapes).  The bf16 MFMA kernels are in ffn_bf16.hip.
#include "ffn_common.h"

namespace mp {

// ---------------------------------------------------------------- m-tile table
constexpr int TILES_THREADS = 1024;

// block-wide exclusive scan of one int per thread; returns the thread's prefix, *total the sum
__device__ __forceinline__ int block_scan(int v, int32_t* wave_tot, int* total) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int incl = v;
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    int o = __shfl_up(incl, m, 64);
    if (lane >= m) incl += o;
  }
  __syncthreads();  // wave_tot may still be read from the previous call
  if (lane == 63) wave_tot[wv] = incl;
  __syncthreads();
  int wbase = 0, tot = 0;
  for (int i = 0; i < TILES_THREADS / 64; ++i) {
    if (i < wv) wbase += wave_tot[i];
    tot += wave_tot[i];
  }
  *total = tot;
  return wbase + incl - v;
}

// tiles[]: the m-tiles in group order (a group's tiles are contiguous)
__global__ __launch_bounds__(TILES_THREADS) void ffn_tiles_kernel(const int32_t* __restrict__ off,
                                                                  MTile* __restrict__ tiles,
                                                                  int32_t* __restrict__ hdr, int E,
                                                                  int max_tiles, int n_rows) {
  __shared__ int32_t wave_tot[TILES_THREADS / 64];
  const int tid = threadIdx.x;
  int carry = 0;  // tiles of the groups before this round (the same in every thread)
  for (int g0 = 0; g0 < E; g0 += TILES_THREADS) {
    int g = g0 + tid;
    int lo = 0, n = 0;
    if (g < E) {  // offsets that do not describe a slot list of n_rows rows yield no tiles
      lo = off[g];
      n = off[g + 1] - lo;
      if (lo < 0 || n < 0 || lo > n_rows || n > n_rows - lo) n = 0;
    }
    const int nt = (n + FFN_BM - 1) / FFN_BM;
    int round_total = 0;
    const int first = carry + block_scan(nt, wave_tot, &round_total);
    for (int i = 0; i < nt; ++i) {
      MTile t;
      t.g = g;
      t.row0 = lo + i * FFN_BM;
      t.rows = min(FFN_BM, n - i * FFN_BM);
      t.first = first;
      t.count = min(nt, max_tiles - first);  // never points past the table
      t.pad[0] = t.pad[1] = t.pad[2] = 0;
      if (first + i < max_tiles) tiles[first + i] = t;
    }
    carry += round_total;
  }
  const int n_tiles = min(carry, max_tiles);
  if (tid == 0) {
    hdr[HDR_MTILES] = n_tiles;
    hdr[HDR_DYN_GATE_UP] = 0;
    hdr[HDR_DYN_DOWN] = 0;
    for (int i = 0; i < N_XCD; ++i) hdr[HDR_DYN_FUSED + i] = 0;
    // more tiles than the table holds: only possible when a caller hands offsets that do not
    // belong to this shape's pair capacity; never silent
    if (carry > max_tiles) atomicOr(&hdr[HDR_FLAGS], 2);
  }
}

hipError_t launch_ffn_tiles(const int32_t* off, MTile* tiles, int32_t* hdr, int E, int max_tiles,
                            int n_rows, hipStream_t s) {
  ffn_tiles_kernel<<<1, TILES_THREADS, 0, s>>>(off, tiles, hdr, E, max_tiles, n_rows);
  return hipGetLastError();
}

// ---------------------------------------------------------------- fp32 tiles (small reference-quality path)
// 128 x 128 output tile, 256 threads, 8 x 8 outputs per thread, K slabs of 16.  An m-tile
// of the table (FFN_BM = 256 rows) is processed as two 128-row halves.
constexpr int FK = 16;
constexpr int TILE = 128;
constexpr int HALVES = FFN_BM / TILE;
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
  const int total = hdr[HDR_MTILES] * NT * HALVES;
  const ItemRange ir = xcd_items(total);
  for (int item = ir.begin; item < ir.end; item += ir.step) {
    MTile tl = tiles[item / (NT * HALVES)];
    const int half = (item / NT) % HALVES;
    tl.row0 += half * TILE;
    tl.rows = min(TILE, tl.rows - half * TILE);
    if (tl.rows <= 0) continue;  // uniform over the workgroup
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
  const int total = hdr[HDR_MTILES] * NT * HALVES;
  const ItemRange ir = xcd_items(total);
  for (int item = ir.begin; item < ir.end; item += ir.step) {
    MTile tl = tiles[item / (NT * HALVES)];
    const int half = (item / NT) % HALVES;
    tl.row0 += half * TILE;
    tl.rows = min(TILE, tl.rows - half * TILE);
    if (tl.rows <= 0) continue;  // uniform over the workgroup
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
hipError_t launch_ffn_gate_up(int dtype, const void* x, const void* w_gu, const int32_t* sorted_pair,
                              const MTile* tiles, int32_t* hdr, void* h, int T, int d, int Is,
                              int k_max, int max_mtiles, hipStream_t s) {
  if (max_mtiles <= 0) return hipSuccess;
  if (dtype != 0)
    return launch_gate_up_bf16((const uint16_t*)x, (const uint16_t*)w_gu, sorted_pair, tiles, hdr,
                               (uint16_t*)h, T, d, Is, k_max, max_mtiles, s);
  long items = (long)max_mtiles * HALVES * cdiv(Is, 64);
  ffn_gate_up_f32_kernel<<<persistent_grid(items, 2), 256, 0, s>>>(
      (const float*)x, (const float*)w_gu, sorted_pair, tiles, hdr, (float*)h, d, Is, k_max, T);
  return hipGetLastError();
}

hipError_t launch_ffn_down(int dtype, const void* h, const void* w_dn, const MTile* tiles,
                           int32_t* hdr, void* y, int d, int Is, int max_mtiles,
                           hipStream_t s) {
  if (max_mtiles <= 0) return hipSuccess;
  if (dtype != 0)
    return launch_down_bf16((const uint16_t*)h, (const uint16_t*)w_dn, tiles, hdr, (uint16_t*)y, d,
                            Is, max_mtiles, s);
  long items = (long)max_mtiles * HALVES * cdiv(d, TILE);
  ffn_down_f32_kernel<<<persistent_grid(items, 2), 256, 0, s>>>(
      (const float*)h, (const float*)w_dn, tiles, hdr, (float*)y, d, Is);
  return hipGetLastError();
}

}  // namespace mp
