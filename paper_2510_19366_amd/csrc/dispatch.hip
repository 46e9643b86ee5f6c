// Dispatch stage: group the token-sub-expert pairs (Sec. 2.1) by sub-expert
// with a stable counting sort that needs no global sort and no order-dependent
// atomics.
//
// Tokens are cut into chunks of 64*W tokens.  Inside a chunk, for every
// sub-expert g a bit mask over the chunk's tokens records who picked g (LDS
// atomic OR: commutative, so the result does not depend on timing).  The
// chunk's count for g is the mask's popcount, and the rank of token t among the
// chunk's pickers of g is the popcount of the mask bits below t.  A single
// block turns the per-chunk counts into per-chunk bases and group offsets.
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

// One block.  chunk_cnt[c,g] -> exclusive prefix over chunks (in place), cnt[g],
// off[g] (exclusive prefix over g), off[E] = P.
constexpr int SCAN_THREADS = 1024;
__global__ __launch_bounds__(SCAN_THREADS) void dispatch_scan_kernel(int32_t* __restrict__ chunk_cnt,
                                                                     int32_t* __restrict__ cnt,
                                                                     int32_t* __restrict__ off,
                                                                     int32_t* __restrict__ hdr,
                                                                     int n_chunks, int E) {
  __shared__ int32_t wave_tot[SCAN_THREADS / 64];
  __shared__ int32_t carry;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int g0 = 0; g0 < E; g0 += SCAN_THREADS) {
    int g = g0 + tid;
    int run = 0;
    if (g < E) {
      constexpr int U = 8;  // loads in flight per thread: the chain over chunks is latency bound
      int c = 0;
      for (; c + U <= n_chunks; c += U) {
        int v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = chunk_cnt[(size_t)(c + u) * E + g];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          chunk_cnt[(size_t)(c + u) * E + g] = run;
          run += v[u];
        }
      }
      for (; c < n_chunks; ++c) {
        int v = chunk_cnt[(size_t)c * E + g];
        chunk_cnt[(size_t)c * E + g] = run;
        run += v;
      }
      cnt[g] = run;
    }
    // block-wide exclusive scan of `run`
    int incl = run;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
      int o = __shfl_up(incl, m, 64);
      if (lane >= m) incl += o;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    int wbase = 0;
    for (int i = 0; i < wv; ++i) wbase += wave_tot[i];
    int excl = carry + wbase + incl - run;
    if (g < E) off[g] = excl;
    __syncthreads();
    if (tid == SCAN_THREADS - 1) carry = excl + run;
    __syncthreads();
  }
  if (tid == 0) {
    off[E] = carry;
    hdr[HDR_PAIRS] = carry;
  }
}

__global__ __launch_bounds__(256) void dispatch_place_kernel(
    const int32_t* __restrict__ ids, const int32_t* __restrict__ chunk_base,
    const int32_t* __restrict__ off, int32_t* __restrict__ sorted_pair,
    int32_t* __restrict__ slot_of_pair, int T, int E, int W, int k_max) {
  extern __shared__ u64 masks[];
  const int c = blockIdx.x, t0 = c * 64 * W;
  const int ntok = min(64 * W, T - t0);
  build_masks(ids, masks, t0, ntok, E, W, k_max);
  const int n = ntok * k_max;
  const int P = off[E];
  const size_t pair0 = (size_t)t0 * k_max;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    int g = ids[pair0 + i];
    int slot = -1;
    if (g >= 0 && g < E) {
      int tl = i / k_max, wq = tl >> 6;
      int rank = __popcll(masks[g * W + wq] & ((1ull << (tl & 63)) - 1ull));
      for (int w = 0; w < wq; ++w) rank += __popcll(masks[g * W + w]);
      slot = off[g] + chunk_base[(size_t)c * E + g] + rank;
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

hipError_t launch_dispatch_scan(int32_t* chunk_cnt, int32_t* cnt, int32_t* off, int32_t* hdr, int T,
                                int E, hipStream_t s) {
  int W = dispatch_chunk_words(E, T);
  int nch = cdiv(T, 64 * W);
  dispatch_scan_kernel<<<1, SCAN_THREADS, 0, s>>>(chunk_cnt, cnt, off, hdr, nch, E);
  return hipGetLastError();
}

hipError_t launch_dispatch_place(const int32_t* ids, const int32_t* chunk_base, const int32_t* off,
                                 int32_t* sorted_pair, int32_t* slot_of_pair, int T, int E,
                                 int k_max, hipStream_t s) {
  if (T == 0) return hipSuccess;
  int W = dispatch_chunk_words(E, T);
  int nch = cdiv(T, 64 * W);
  dispatch_place_kernel<<<nch, 256, (size_t)E * W * 8, s>>>(ids, chunk_base, off, sorted_pair,
                                                             slot_of_pair, T, E, W, k_max);
  return hipGetLastError();
}

}  // namespace mp
