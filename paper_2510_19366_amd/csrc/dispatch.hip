// Dispatch stage: group the token-sub-expert pairs (Sec. 2.1) by sub-expert
// with a stable counting sort that needs no global sort and no order-dependent
// atomics.
//
// Tokens are cut into chunks of 64*W tokens.  Inside a chunk, for every
// sub-expert g a bit mask over the chunk's tokens records who picked g (LDS
// atomic OR: commutative, so the result does not depend on timing).  The
// chunk's count for g is the mask's popcount, and the rank of token t among the
// chunk's pickers of g is the popcount of the mask bits below t.  A second
// kernel turns the per-chunk counts into per-chunk bases and the groups' totals,
// and the placing kernel derives the group offsets from the totals.
// Because a token picks a sub-expert at most once, "token ascending" fixes the
// order inside a group completely.
#include "kernels.h"

namespace mp {

int dispatch_chunk_words(int E, int T) {
  int cap = 8192 / (E > 0 ? E : 1);  // E * W * 8 bytes of LDS <= 64 KiB
  if (cap > 4) cap = 4;
  if (cap < 1) cap = 1;
  int w = T / (64 * 256);  // aim at >= 256 chunks (one per CU) before growing the chunks
  if (w > cap) w = cap;
  if (w < 1) w = 1;
  return w;
}

typedef unsigned long long u64;

__device__ __forceinline__ void build_masks(const int32_t* __restrict__ ids, u64* masks, int t0,
                                            int ntok, int E, int W, int k_max) {
  for (int i = threadIdx.x; i < E * W; i += blockDim.x) masks[i] = 0ull;
  __syncthreads();
  const int n = ntok * k_max;
  const int32_t* base = ids + (size_t)t0 * k_max;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    int g = base[i];
    if (g >= 0 && g < E) {
      int tl = i / k_max;
      atomicOr(&masks[g * W + (tl >> 6)], 1ull << (tl & 63));
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void dispatch_count_kernel(const int32_t* __restrict__ ids,
                                                             int32_t* __restrict__ chunk_cnt, int T,
                                                             int E, int W, int k_max) {
  extern __shared__ u64 masks[];
  const int c = blockIdx.x, t0 = c * 64 * W;
  const int ntok = min(64 * W, T - t0);
  build_masks(ids, masks, t0, ntok, E, W, k_max);
  for (int g = threadIdx.x; g < E; g += blockDim.x) {
    int n = 0;
    for (int w = 0; w < W; ++w) n += __popcll(masks[g * W + w]);
    chunk_cnt[(size_t)c * E + g] = n;
  }
}

// chunk_cnt[c,g] -> exclusive prefix over chunks (in place) and cnt[g].  The chain over chunks
// is independent per group and moves n_chunks * E * 8 bytes, too much for one CU: a workgroup
// takes SCAN_GROUPS consecutive groups and cuts the chunk range into SCAN_PARTS pieces that run
// side by side (a thread sums its piece, the pieces' sums meet in LDS, a second walk over the
// piece writes the running prefixes).  The prefix over groups (off[]) is left to the place
// kernel, where every workgroup recomputes it in LDS from cnt[].
constexpr int SCAN_GROUPS = 16, SCAN_PARTS = 16, SCAN_THREADS = SCAN_GROUPS * SCAN_PARTS;
__global__ __launch_bounds__(SCAN_THREADS) void dispatch_scan_kernel(int32_t* __restrict__ chunk_cnt,
                                                                     int32_t* __restrict__ cnt,
                                                                     int n_chunks, int E) {
  __shared__ int32_t part_tot[SCAN_PARTS][SCAN_GROUPS];
  const int gq = threadIdx.x % SCAN_GROUPS, part = threadIdx.x / SCAN_GROUPS;
  const int g = blockIdx.x * SCAN_GROUPS + gq;
  const bool in = g < E;
  const int cp = (n_chunks + SCAN_PARTS - 1) / SCAN_PARTS;
  const int c_lo = min(part * cp, n_chunks), c_hi = min(c_lo + cp, n_chunks);
  int sum = 0;
  if (in) {
    constexpr int U = 16;
    int c = c_lo;
    for (; c + U <= c_hi; c += U) {
      int v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = chunk_cnt[(size_t)(c + u) * E + g];
#pragma unroll
      for (int u = 0; u < U; ++u) sum += v[u];
    }
    for (; c < c_hi; ++c) sum += chunk_cnt[(size_t)c * E + g];
  }
  part_tot[part][gq] = sum;
  __syncthreads();
  int run = 0, total = 0;
#pragma unroll
  for (int p = 0; p < SCAN_PARTS; ++p) {
    const int s = part_tot[p][gq];
    run += p < part ? s : 0;
    total += s;
  }
  if (!in) return;
  if (part == 0) cnt[g] = total;
  constexpr int U = 8;
  int c = c_lo;
  for (; c + U <= c_hi; c += U) {
    int v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = chunk_cnt[(size_t)(c + u) * E + g];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      chunk_cnt[(size_t)(c + u) * E + g] = run;
      run += v[u];
    }
  }
  for (; c < c_hi; ++c) {
    const int v = chunk_cnt[(size_t)c * E + g];
    chunk_cnt[(size_t)c * E + g] = run;
    run += v;
  }
}

// Exclusive prefixes over the groups by one workgroup of 256 threads, into LDS: off_lds[0..E]
// of the row counts cnt[g] (off_lds[E] = P) and first_lds[0..E] of the m-tile counts
// ceil(cnt[g] / FFN_BM) (first_lds[E] = number of m-tiles).  A thread sums a run of consecutive
// groups, the 256 partial sums are scanned with shuffles, the run is walked again.
__device__ __forceinline__ void group_offsets(const int32_t* __restrict__ cnt, int32_t* off_lds,
                                              int32_t* first_lds, int32_t (*wave_tot)[2], int E) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int per = (E + 255) / 256, lo = min(tid * per, E), hi = min(lo + per, E);
  int mine = 0, mine_t = 0;
  for (int g = lo; g < hi; ++g) {
    const int n = cnt[g];
    mine += n;
    mine_t += (n + FFN_BM - 1) / FFN_BM;
  }
  int incl = mine, incl_t = mine_t;
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const int o = __shfl_up(incl, m, 64), ot = __shfl_up(incl_t, m, 64);
    if (lane >= m) {
      incl += o;
      incl_t += ot;
    }
  }
  if (lane == 63) {
    wave_tot[wv][0] = incl;
    wave_tot[wv][1] = incl_t;
  }
  __syncthreads();
  int run = incl - mine, run_t = incl_t - mine_t;
  for (int i = 0; i < wv; ++i) {
    run += wave_tot[i][0];
    run_t += wave_tot[i][1];
  }
  for (int g = lo; g < hi; ++g) {
    const int n = cnt[g];
    off_lds[g] = run;
    first_lds[g] = run_t;
    run += n;
    run_t += (n + FFN_BM - 1) / FFN_BM;
  }
  if (tid == 255) {  // lo == hi == E for the threads past the last group
    off_lds[E] = run;
    first_lds[E] = run_t;
  }
  __syncthreads();
}

// Workgroup c places the pairs of chunk c.  Every workgroup derives the group offsets from
// cnt[] (E additions); workgroup 0 also writes them out: off[0..E] and the pair count.
// With tiles != nullptr the kernel also builds the grouped FFN's m-tile table (the table
// ffn_tiles_kernel builds from off[]): workgroup c writes the tiles of groups c, c + grid, ...
// and workgroup 0 the table's header words.
__global__ __launch_bounds__(256) void dispatch_place_kernel(
    const int32_t* __restrict__ ids, const int32_t* __restrict__ chunk_base,
    const int32_t* __restrict__ cnt, int32_t* __restrict__ off, int32_t* __restrict__ hdr,
    int32_t* __restrict__ sorted_pair, int32_t* __restrict__ slot_of_pair,
    MTile* __restrict__ tiles, int max_tiles, int T, int E, int W, int k_max) {
  extern __shared__ u64 masks[];  // E * W masks, then E + 1 offsets, then E + 1 first-tile indices
  __shared__ int32_t wave_tot[4][2];
  int32_t* off_lds = reinterpret_cast<int32_t*>(masks + (size_t)E * W);
  int32_t* first_lds = off_lds + E + 1;
  const int c = blockIdx.x, t0 = c * 64 * W;
  const int ntok = max(min(64 * W, T - t0), 0);
  group_offsets(cnt, off_lds, first_lds, wave_tot, E);
  const int P = off_lds[E];
  if (c == 0) {
    for (int g = threadIdx.x; g <= E; g += blockDim.x) off[g] = off_lds[g];
    if (threadIdx.x == 0) {
      hdr[HDR_PAIRS] = P;
      if (tiles != nullptr) {
        hdr[HDR_MTILES] = min(first_lds[E], max_tiles);
        hdr[HDR_DYN_GATE_UP] = 0;
        hdr[HDR_DYN_DOWN] = 0;
        for (int i = 0; i < 8; ++i) hdr[HDR_DYN_FUSED + i] = 0;
        if (first_lds[E] > max_tiles) atomicOr(&hdr[HDR_FLAGS], 2);  // cannot happen: P <= T * k_max
      }
    }
  }
  if (tiles != nullptr) {
    for (int g = c; g < E; g += gridDim.x) {
      const int lo = off_lds[g], n = off_lds[g + 1] - lo, first = first_lds[g];
      const int nt = first_lds[g + 1] - first;
      for (int i = threadIdx.x; i < nt; i += blockDim.x) {
        MTile t;
        t.g = g;
        t.row0 = lo + i * FFN_BM;
        t.rows = min(FFN_BM, n - i * FFN_BM);
        t.first = first;
        t.count = min(nt, max_tiles - first);
        t.pad[0] = t.pad[1] = t.pad[2] = 0;
        if (first + i < max_tiles) tiles[first + i] = t;
      }
    }
  }
  build_masks(ids, masks, t0, ntok, E, W, k_max);
  const int n = ntok * k_max;
  const size_t pair0 = (size_t)t0 * k_max;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    int g = ids[pair0 + i];
    int slot = -1;
    if (g >= 0 && g < E) {
      int tl = i / k_max, wq = tl >> 6;
      int rank = __popcll(masks[g * W + wq] & ((1ull << (tl & 63)) - 1ull));
      for (int w = 0; w < wq; ++w) rank += __popcll(masks[g * W + w]);
      slot = off_lds[g] + chunk_base[(size_t)c * E + g] + rank;
      sorted_pair[slot] = (int32_t)(pair0 + i);
    }
    slot_of_pair[pair0 + i] = slot;
    if ((long)(pair0 + i) >= (long)P) sorted_pair[pair0 + i] = -1;  // tail beyond the P valid slots
  }
}

hipError_t launch_dispatch_count(const int32_t* ids, int32_t* chunk_cnt, int T, int E, int k_max,
                                 hipStream_t s) {
  if (T == 0) return hipSuccess;
  int W = dispatch_chunk_words(E, T);
  int nch = cdiv(T, 64 * W);
  dispatch_count_kernel<<<nch, 256, (size_t)E * W * 8, s>>>(ids, chunk_cnt, T, E, W, k_max);
  return hipGetLastError();
}

hipError_t launch_dispatch_scan(int32_t* chunk_cnt, int32_t* cnt, int T, int E, hipStream_t s) {
  int W = dispatch_chunk_words(E, T);
  int nch = cdiv(T, 64 * W);
  dispatch_scan_kernel<<<cdiv(E, SCAN_GROUPS), SCAN_THREADS, 0, s>>>(chunk_cnt, cnt, nch, E);
  return hipGetLastError();
}

hipError_t launch_dispatch_place(const int32_t* ids, const int32_t* chunk_base, const int32_t* cnt,
                                 int32_t* off, int32_t* hdr, int32_t* sorted_pair,
                                 int32_t* slot_of_pair, MTile* tiles, int max_tiles, int T, int E,
                                 int k_max, hipStream_t s) {
  int W = dispatch_chunk_words(E, T);
  int nch = cdiv(T, 64 * W);
  if (nch < 1) nch = 1;  // T == 0: one workgroup still writes the (all-zero) offsets
  const size_t lds = (size_t)E * W * 8 + 2 * ((size_t)E + 1) * 4;
  // up to 96 KiB + 8 bytes (E = 4096, W = 2): beyond the default limit for dynamic LDS, so the
  // limit is raised once per device (no other runtime call on the launch path afterwards)
  static bool raised[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
  if (dev < 0 || !raised[dev]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(dispatch_place_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024);
    if (e != hipSuccess) return e;
    if (dev >= 0) raised[dev] = true;
  }
  dispatch_place_kernel<<<nch, 256, lds, s>>>(ids, chunk_base, cnt, off, hdr, sorted_pair,
                                              slot_of_pair, tiles, max_tiles, T, E, W, k_max);
  return hipGetLastError();
}

}  // namespace mp
