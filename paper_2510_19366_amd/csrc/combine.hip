// Combine stage (Sec. 3.2.2): out[t,:] = sum_{j<k_t} w[t,j] * y[slot(t,j),:].
// One workgroup per token, 16-byte column vectors per thread, picks visited in
// ascending j (four row loads in flight) with fp32 accumulation and a single final rounding.  No atomics:
// every output element has exactly one writer, so the result is reproducible.
#include "kernels.h"

namespace mp {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int DT> struct Vec;  // 16 bytes of a row
template <> struct Vec<0> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const void* base, size_t elem, float (&v)[8]) {
    const f32x4_t a = __builtin_nontemporal_load(
        reinterpret_cast<const f32x4_t*>(static_cast<const float*>(base) + elem));
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  }
  static __device__ __forceinline__ void store(void* base, size_t elem, const float (&v)[8]) {
    *reinterpret_cast<float4*>(static_cast<float*>(base) + elem) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Vec<1> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const void* base, size_t elem, float (&v)[8]) {
    // y is read exactly once: a non-temporal load keeps it from displacing anything in L2
    // (measured 8 % faster than a plain load)
    const u32x4_t a = __builtin_nontemporal_load(
        reinterpret_cast<const u32x4_t*>(static_cast<const uint16_t*>(base) + elem));
    uint32_t w[4] = {a.x, a.y, a.z, a.w};
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

// The token's slots and weights are fetched once into LDS (one element per thread), so the
// row loop below never waits for an index before it can issue its row loads.
constexpr int CB_CHUNK = 1024;  // = the largest k_max the library accepts

template <int DT>
__global__ __launch_bounds__(256) void combine_kernel(const void* __restrict__ y,
                                                      const int32_t* __restrict__ slot_of_pair,
                                                      const float* __restrict__ w,
                                                      const int32_t* __restrict__ k_tok,
                                                      void* __restrict__ out, int d, int k_max,
                                                      int n_rows) {
  constexpr int N = Vec<DT>::N;
  constexpr int RU = 4;  // rows fetched before any is consumed (4 measured best; 8 and 16 slower)
  __shared__ int32_t s_slot[CB_CHUNK];
  __shared__ float s_w[CB_CHUNK];
  const int t = blockIdx.x;
  int kt = k_tok[t];
  kt = kt < 0 ? 0 : (kt > k_max ? k_max : kt);
  for (int j = threadIdx.x; j < kt; j += 256) {
    const int sl = slot_of_pair[(size_t)t * k_max + j];
    const bool ok = sl >= 0 && sl < n_rows;  // a pick without a slot contributes nothing:
    s_slot[j] = ok ? sl : -1;                // its row is not even read (y may hold anything there)
    s_w[j] = ok ? w[(size_t)t * k_max + j] : 0.0f;
  }
  __syncthreads();
  for (int col = threadIdx.x * N; col < d; col += 256 * N) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int j = 0;
    for (; j + RU <= kt; j += RU) {  // RU rows in flight, still added in ascending j
      float v[RU][8];
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int sl = s_slot[j + u];  // the same for every thread: a uniform branch
        if (sl >= 0) {
          Vec<DT>::load(y, (size_t)sl * d + col, v[u]);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[u][e] = 0.0f;
        }
      }
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const float wj = s_w[j + u];
#pragma unroll
        for (int e = 0; e < N; ++e) acc[e] = fmaf(wj, v[u][e], acc[e]);
      }
    }
    for (; j < kt; ++j) {
      float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      const float wj = s_w[j];
      const int sl = s_slot[j];
      if (sl >= 0) Vec<DT>::load(y, (size_t)sl * d + col, v);
#pragma unroll
      for (int e = 0; e < N; ++e) acc[e] = fmaf(wj, v[e], acc[e]);
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
