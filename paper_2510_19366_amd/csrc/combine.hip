// Combine stage (Sec. 3.2.2): out[t,:] = sum_{j<k_t} w[t,j] * y[slot(t,j),:].
// One workgroup per token, 16-byte column vectors per thread, picks visited in
// ascending j (two batches of four row loads alternate in flight) with fp32 accumulation and a
// single final rounding.  No atomics:
// every output element has exactly one writer, so the result is reproducible.
#include "kernels.h"

namespace mp {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// 16 bytes of a row: the raw bits (a non-temporal load: y is read exactly once, and keeping it
// out of the way of everything else in L2 measured 8 % faster than a plain load), their fp32
// values, and the rounding back.
template <int DT> struct Vec;
template <> struct Vec<0> {
  static constexpr int N = 4;
  static __device__ __forceinline__ u32x4_t load(const void* base, size_t elem) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(static_cast<const float*>(base) + elem));
  }
  static __device__ __forceinline__ void widen(u32x4_t a, float (&v)[8]) {
    v[0] = __uint_as_float(a.x); v[1] = __uint_as_float(a.y);
    v[2] = __uint_as_float(a.z); v[3] = __uint_as_float(a.w);
  }
  static __device__ __forceinline__ void store(void* base, size_t elem, const float (&v)[8]) {
    *reinterpret_cast<float4*>(static_cast<float*>(base) + elem) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Vec<1> {
  static constexpr int N = 8;
  static __device__ __forceinline__ u32x4_t load(const void* base, size_t elem) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(static_cast<const uint16_t*>(base) + elem));
  }
  static __device__ __forceinline__ void widen(u32x4_t a, float (&v)[8]) {
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(void* base, size_t elem, const float (&v)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<uint4*>(static_cast<uint16_t*>(base) + elem) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// The token's slots and weights are fetched once into LDS (one element per thread), padded to
// a whole number of batches with slot-less picks, so the row loop below never waits for an
// index before it can issue its row loads.
constexpr int CB_RU = 4;        // rows per batch
constexpr int CB_CHUNK = 1024;  // = the largest k_max the library accepts (a multiple of CB_RU)

template <int DT>
__global__ __launch_bounds__(256) void combine_kernel(const void* __restrict__ y,
                                                      const int32_t* __restrict__ slot_of_pair,
                                                      const float* __restrict__ w,
                                                      const int32_t* __restrict__ k_tok,
                                                      void* __restrict__ out, int d, int k_max,
                                                      int n_rows) {
  constexpr int N = Vec<DT>::N, RU = CB_RU;
  __shared__ int32_t s_slot[CB_CHUNK];
  __shared__ float s_w[CB_CHUNK];
  const int t = blockIdx.x;
  // The slots and weights of all k_max picks are requested together with the token's budget
  // (one memory latency instead of two in a row); picks beyond the budget are masked afterwards.
  int kt = k_tok[t];
  const int kp = (k_max + RU - 1) / RU * RU;  // <= CB_CHUNK
  for (int j = threadIdx.x; j < kp; j += 256) {
    const bool in = j < k_max;
    const int sl = in ? slot_of_pair[(size_t)t * k_max + j] : -1;
    const float wj = in ? w[(size_t)t * k_max + j] : 0.0f;
    const int ktc = kt < 0 ? 0 : (kt > k_max ? k_max : kt);
    const bool ok = j < ktc && sl >= 0 && sl < n_rows;  // a pick without a slot contributes nothing:
    s_slot[j] = ok ? sl : -1;                           // its row is not even read (y may hold anything there)
    s_w[j] = ok ? wj : 0.0f;
  }
  kt = kt < 0 ? 0 : (kt > k_max ? k_max : kt);
  const int ktp = (kt + RU - 1) / RU * RU;
  __syncthreads();
  for (int col = threadIdx.x * N; col < d; col += 256 * N) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    // Two batches of RU rows alternate: the loads of one are in flight while the other is
    // added, still in ascending j.
    auto issue = [&](int j0, u32x4_t (&r)[RU]) {
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int sl = s_slot[j0 + u];  // the same for every thread: a uniform branch
        r[u] = u32x4_t{0u, 0u, 0u, 0u};
        if (sl >= 0) r[u] = Vec<DT>::load(y, (size_t)sl * d + col);
      }
    };
    auto consume = [&](int j0, const u32x4_t (&r)[RU]) {
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const float wj = s_w[j0 + u];
        float v[8];
        Vec<DT>::widen(r[u], v);
#pragma unroll
        for (int e = 0; e < N; ++e) acc[e] = fmaf(wj, v[e], acc[e]);
      }
    };
    u32x4_t ra[RU], rb[RU];
    if (ktp > 0) issue(0, ra);
    for (int j = 0; j < ktp; j += 2 * RU) {
      const bool second = j + RU < ktp;
      if (second) issue(j + RU, rb);
      consume(j, ra);
      if (second) {
        if (j + 2 * RU < ktp) issue(j + 2 * RU, ra);
        consume(j + RU, rb);
      }
    }
    Vec<DT>::store(out, (size_t)t * d + col, acc);
  }
}

hipError_t launch_combine(int dtype, const void* y, const int32_t* slot_of_pair, const float* w,
                          const int32_t* k_tok, void* out, int T, int d, int k_max, hipStream_t s) {
  if (T == 0) return hipSuccess;
  if (dtype == 0)
    combine_kernel<0><<<T, 256, 0, s>>>(y, slot_of_pair, w, k_tok, out, d, k_max, T * k_max);
  else
    combine_kernel<1><<<T, 256, 0, s>>>(y, slot_of_pair, w, k_tok, out, d, k_max, T * k_max);
  return hipGetLastError();
}

}  // namespace mp
