// Route stage (Sec. 3.2.2, expanded linear gate): router logits with a fixed
// summation order, then per-token top-k_t and softmax weights.
#include "kernels.h"

namespace mp {

// ---------------------------------------------------------------- expand_k
// Sec. 3.3.1: a token inherits its request's budget.
__global__ void expand_k_kernel(int R, const int32_t* __restrict__ req_k,
                                const int32_t* __restrict__ req_off, int32_t* __restrict__ k_tok) {
  int r = blockIdx.x;
  if (r >= R) return;
  int lo = req_off[r], hi = req_off[r + 1], k = req_k[r];
  for (int t = lo + threadIdx.x; t < hi; t += blockDim.x) k_tok[t] = k;
}

hipError_t launch_expand_k(int R, int T, const int32_t* req_k, const int32_t* req_off,
                           int32_t* k_tok, hipStream_t s) {
  (void)T;
  if (R > 0) expand_k_kernel<<<R, 256, 0, s>>>(R, req_k, req_off, k_tok);
  return hipGetLastError();
}

// ---------------------------------------------------------------- logits on the matrix cores
// Every logit is ONE chain of d binary32 fused multiply-adds over the hidden index in
// ascending order, then the fp32 bias add: the fixed summation order is what makes the
// routing reproducible bit for bit.  The rank-1 fp32 MFMA forms add ONE k term per
// instruction, D = a * b + D with one rounding per output (checked on the device against
// fmaf chains of 4096 terms, subnormal sums included: bit-identical), so issuing one per k in
// ascending order computes exactly that chain, at twice the rate of unpacked v_fma_f32.  No
// split-K, no reordering.
//
// Large problems: v_mfma_f32_32x32x1_2b_f32.
//
// Workgroup tile 128 tokens x 128 sub-experts, 4 waves as 2 x 2, wave tile 64 x 64: lane l
// feeds token row l and sub-expert row l of the wave tile; with the A-block broadcast
// (cbsz = 1) instruction `ab` multiplies token block ab (32 rows) by both 32-column blocks.
// Operands are staged per K slab of 64 bytes per row in LDS rows of 80 bytes (the 16 bytes
// of padding make the per-lane row reads conflict-free).
typedef __attribute__((__vector_size__(32 * sizeof(float)))) float f32x32;
constexpr int LM_ROWB = 80;  // LDS bytes per row: 64 of data + 16 of padding

template <typename InT>
__device__ __forceinline__ float lm_elem(const uint4 (&q)[4], int i);
template <>
__device__ __forceinline__ float lm_elem<float>(const uint4 (&q)[4], int i) {
  const uint32_t w[4] = {q[i >> 2].x, q[i >> 2].y, q[i >> 2].z, q[i >> 2].w};
  return __uint_as_float(w[i & 3]);
}
template <>
__device__ __forceinline__ float lm_elem<uint16_t>(const uint4 (&q)[4], int i) {
  const uint32_t w[4] = {q[i >> 3].x, q[i >> 3].y, q[i >> 3].z, q[i >> 3].w};
  const uint32_t v = w[(i >> 1) & 3];
  return __uint_as_float((i & 1) ? (v & 0xffff0000u) : (v << 16));
}

template <typename InT>
__global__ __launch_bounds__(256) void logits_mfma_kernel(const InT* __restrict__ x,
                                                          const InT* __restrict__ w,
                                                          const float* __restrict__ bias,
                                                          float* __restrict__ logits,
                                                          int32_t* __restrict__ hdr, int T, int d,
                                                          int E) {
  constexpr int KB = 64 / sizeof(InT);  // K elements per slab: 32 bf16 or 16 fp32
  __shared__ __align__(16) unsigned char sm[2][256 * LM_ROWB];  // rows 0..127 tokens, 128..255 sub-experts
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) hdr[HDR_FLAGS] = 0;
  const int m0 = blockIdx.y * 128, n0 = blockIdx.x * 128;

  // loader: 16-byte chunk lc of rows lr + 64 i
  const int lc = tid & 3, lr = tid >> 2;
  auto row_src = [&](int row) {
    const InT* base = row < 128 ? x + (size_t)min(m0 + row, T - 1) * d
                                : w + (size_t)min(n0 + row - 128, E - 1) * d;
    return reinterpret_cast<const unsigned char*>(base) + lc * 16;
  };
  const unsigned char* src0 = row_src(lr);
  const unsigned char* src1 = row_src(lr + 64);
  const unsigned char* src2 = row_src(lr + 128);
  const unsigned char* src3 = row_src(lr + 192);
  uint4 pre0, pre1, pre2, pre3;  // named registers: an indexed array here ends up in scratch memory
#define LM_GLOAD(k0_)                                                                   \
  do {                                                                                  \
    const size_t o_ = (size_t)(k0_) * sizeof(InT);                                      \
    pre0 = *reinterpret_cast<const uint4*>(src0 + o_);                                  \
    pre1 = *reinterpret_cast<const uint4*>(src1 + o_);                                  \
    pre2 = *reinterpret_cast<const uint4*>(src2 + o_);                                  \
    pre3 = *reinterpret_cast<const uint4*>(src3 + o_);                                  \
  } while (0)
#define LM_SSTORE(buf_)                                                                 \
  do {                                                                                  \
    unsigned char* b_ = &sm[buf_][lr * LM_ROWB + lc * 16];                              \
    *reinterpret_cast<uint4*>(b_) = pre0;                                               \
    *reinterpret_cast<uint4*>(b_ + 64 * LM_ROWB) = pre1;                                \
    *reinterpret_cast<uint4*>(b_ + 128 * LM_ROWB) = pre2;                               \
    *reinterpret_cast<uint4*>(b_ + 192 * LM_ROWB) = pre3;                               \
  } while (0)

  f32x32 acc0, acc1;
#pragma unroll
  for (int v = 0; v < 32; ++v) {
    acc0[v] = 0.0f;
    acc1[v] = 0.0f;
  }
  const int a_off = (wm * 64 + lane) * LM_ROWB, b_off = (128 + wn * 64 + lane) * LM_ROWB;

  LM_GLOAD(0);
  LM_SSTORE(0);
  __syncthreads();
  int buf = 0;
  for (int k0 = 0; k0 < d; k0 += KB) {  // d % 64 == 0, so d % KB == 0
    const bool more = k0 + KB < d;
    if (more) LM_GLOAD(k0 + KB);
    uint4 qa[4], qb[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      qa[c] = *reinterpret_cast<const uint4*>(&sm[buf][a_off + c * 16]);
      qb[c] = *reinterpret_cast<const uint4*>(&sm[buf][b_off + c * 16]);
    }
#pragma unroll
    for (int i = 0; i < KB; ++i) {  // ascending k: one fused multiply-add per logit and step
      const float a = lm_elem<InT>(qa, i), b = lm_elem<InT>(qb, i);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x1f32(a, b, acc0, 1, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x1f32(a, b, acc1, 1, 1, 0);
    }
    if (more) LM_SSTORE(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // accumulator v of lane l: column block j = v / 16, row 8 ((v % 16) / 4) + 4 (l / 32) + v % 4
  // of the 32-row token block, column l % 32
#pragma unroll
  for (int ab = 0; ab < 2; ++ab) {
#pragma unroll
    for (int v = 0; v < 32; ++v) {
      const int vv = v & 15;
      const int row = m0 + wm * 64 + ab * 32 + 8 * (vv >> 2) + 4 * (lane >> 5) + (vv & 3);
      const int col = n0 + wn * 64 + (v >> 4) * 32 + (lane & 31);
      if (row < T && col < E) {
        float r = ab == 0 ? acc0[v] : acc1[v];
        if (bias != nullptr) r = r + bias[col];
        logits[(size_t)row * E + col] = r;
      }
    }
  }
#undef LM_GLOAD
#undef LM_SSTORE
}

// Small problems (few 128 x 128 tiles): the per-logit chain of d dependent FMAs is what takes
// the time, so the tile per wave is made as small as the matrix cores allow.
// v_mfma_f32_4x4x1_16b_f32 performs 16 independent 4 x 4 rank-1 updates in 2 passes (8 cycles):
// block b takes its 4 A values from lanes 4b..4b+3 and its 4 B values from the same lanes, and
// lane 4b + j holds column j of block b, rows 0..3 in its 4 accumulator registers.  Again one
// binary32 FMA per logit and k.  With block b = (p, q) multiplying tokens 4p..4p+3 by
// sub-experts 4q..4q+3 (lane 4b + i feeds token 4p + i and sub-expert 4q + i) one instruction
// covers 16 tokens x 16 sub-experts.  A dependent chain of these instructions issues only
// every 44 to 64 cycles, so where the problem has enough work a wave keeps four chains going:
// NSUB x NSUB such sub-tiles per wave (NSUB = 2: 32 x 32 per wave, 64 x 64 per workgroup of
// 2 x 2 waves; NSUB = 1: 16 x 16 and 32 x 32, four times as many waves for the smallest
// problems).
// Operands are widened to fp32 once, when a slab of 32 k is stored to LDS (rows of 128 bytes
// + 16 of padding: conflict-free 16-byte reads), so the inner loop is LDS reads and MFMAs only.
// Global loads run PF slabs ahead in registers; LDS holds two slabs; one barrier per slab.
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
constexpr int L4_ROWB = 144, L4_KB = 32;

template <typename InT, int NSUB>
__global__ __launch_bounds__(256) void logits_mfma4_kernel(const InT* __restrict__ x,
                                                           const InT* __restrict__ w,
                                                           const float* __restrict__ bias,
                                                           float* __restrict__ logits,
                                                           int32_t* __restrict__ hdr, int T, int d,
                                                           int E) {
  constexpr int ROW_GB = L4_KB * sizeof(InT);      // global bytes per row and slab: 64 or 128
  constexpr int CPR = ROW_GB / 16;                  // 16-byte chunks per row: 4 or 8
  constexpr int BT = 32 * NSUB;                     // tokens (and sub-experts) per workgroup
  constexpr int L4_ROWS = 2 * BT;                   // LDS rows: BT tokens, then BT sub-experts
  constexpr int CH = L4_ROWS * CPR / 256;           // chunks per thread and slab: 1, 2 or 4
  constexpr int PF = CH >= 4 ? 4 : 8;               // slabs in flight
  __shared__ __align__(16) unsigned char sm[2][L4_ROWS * L4_ROWB];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wy = wv >> 1, wx = wv & 1;
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) hdr[HDR_FLAGS] = 0;
  const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;

  // loader: chunk id c = tid + 256 j -> row c / CPR, 16-byte piece c % CPR
  const unsigned char* src[CH];
  int dst[CH];
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int c = tid + 256 * j, row = c / CPR, pc = c % CPR;
    const InT* base = row < BT ? x + (size_t)min(m0 + row, T - 1) * d
                               : w + (size_t)min(n0 + row - BT, E - 1) * d;
    src[j] = reinterpret_cast<const unsigned char*>(base) + pc * 16;
    dst[j] = row * L4_ROWB + pc * (sizeof(InT) == 2 ? 32 : 16);
  }
  auto sstore = [&](int buf, int j, uint4 v) {  // widen to fp32 (exact) and store
    unsigned char* o = &sm[buf][dst[j]];
    if (sizeof(InT) == 2) {
      const uint4 lo = {v.x << 16, v.x & 0xffff0000u, v.y << 16, v.y & 0xffff0000u};
      const uint4 hi = {v.z << 16, v.z & 0xffff0000u, v.w << 16, v.w & 0xffff0000u};
      *reinterpret_cast<uint4*>(o) = lo;
      *reinterpret_cast<uint4*>(o + 16) = hi;
    } else {
      *reinterpret_cast<uint4*>(o) = v;
    }
  };

  const int blk = lane >> 2, li = lane & 3, p = blk >> 2, q = blk & 3;
  const int a_off = (wy * 16 * NSUB + 4 * p + li) * L4_ROWB;
  const int b_off = (BT + wx * 16 * NSUB + 4 * q + li) * L4_ROWB;

  const int ns = d / L4_KB;  // d % 64 == 0
  uint4 pre[PF][CH];
#pragma unroll
  for (int i = 0; i < PF; ++i)
#pragma unroll
    for (int j = 0; j < CH; ++j)
      pre[i][j] = *reinterpret_cast<const uint4*>(src[j] + (size_t)(i < ns ? i : 0) * ROW_GB);
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    sstore(0, j, pre[0][j]);
    pre[0][j] = *reinterpret_cast<const uint4*>(src[j] + (size_t)(PF < ns ? PF : 0) * ROW_GB);
  }
  __syncthreads();

  f32x4_t acc[NSUB][NSUB];
#pragma unroll
  for (int ia = 0; ia < NSUB; ++ia)
#pragma unroll
    for (int ib = 0; ib < NSUB; ++ib) acc[ia][ib] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

  for (int s0 = 0; s0 < ns; s0 += PF) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {  // slab s0 + i; s0 is a multiple of PF: ring slot and parity are static
      const int sl = s0 + i;
      if (sl < ns) {
        const int nx = (i + 1) % PF, par = i & 1;
        if (sl + 1 < ns) {
#pragma unroll
          for (int j = 0; j < CH; ++j) {
            sstore(par ^ 1, j, pre[nx][j]);
            pre[nx][j] = *reinterpret_cast<const uint4*>(
                src[j] + (size_t)(sl + 1 + PF < ns ? sl + 1 + PF : 0) * ROW_GB);
          }
        }
        const unsigned char* sa = &sm[par][a_off];
        const unsigned char* sb = &sm[par][b_off];
#pragma unroll
        for (int g = 0; g < L4_KB / 4; ++g) {  // 4 k per 16-byte read, ascending k
          f32x4_t fa[NSUB], fb[NSUB];
#pragma unroll
          for (int h = 0; h < NSUB; ++h) {
            fa[h] = *reinterpret_cast<const f32x4_t*>(sa + h * 16 * L4_ROWB + g * 16);
            fb[h] = *reinterpret_cast<const f32x4_t*>(sb + h * 16 * L4_ROWB + g * 16);
          }
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int ia = 0; ia < NSUB; ++ia)
#pragma unroll
              for (int ib = 0; ib < NSUB; ++ib)
                acc[ia][ib] = __builtin_amdgcn_mfma_f32_4x4x1f32(fa[ia][kk], fb[ib][kk], acc[ia][ib], 0, 0, 0);
        }
        // barrier that waits for this wave's LDS traffic only: __syncthreads() would also wait
        // for the global loads just issued and expose their latency in every slab
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
    }
  }

#pragma unroll
  for (int ia = 0; ia < NSUB; ++ia)
#pragma unroll
    for (int ib = 0; ib < NSUB; ++ib) {
      const int col = n0 + wx * 16 * NSUB + ib * 16 + 4 * q + li;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = m0 + wy * 16 * NSUB + ia * 16 + 4 * p + v;
        if (row < T && col < E) {
          float r = acc[ia][ib][v];
          if (bias != nullptr) r = r + bias[col];
          logits[(size_t)row * E + col] = r;
        }
      }
    }
}

__global__ void clear_flags_kernel(int32_t* hdr) { hdr[HDR_FLAGS] = 0; }

// 128 x 128 tiles when they fill the chip; else the small-tile kernel, with four chains per
// wave when that still gives every SIMD a wave.
template <typename InT>
static void launch_logits_t(const InT* x, const InT* w, const float* bias, float* logits,
                            int32_t* hdr, int T, int d, int E, hipStream_t s) {
  const long cus = num_cus();
  if ((long)cdiv(E, 128) * cdiv(T, 128) >= cus + cus / 2)
    logits_mfma_kernel<InT><<<dim3(cdiv(E, 128), cdiv(T, 128)), 256, 0, s>>>(x, w, bias, logits, hdr,
                                                                             T, d, E);
  else if ((long)cdiv(E, 64) * cdiv(T, 64) >= cus)
    logits_mfma4_kernel<InT, 2><<<dim3(cdiv(E, 64), cdiv(T, 64)), 256, 0, s>>>(x, w, bias, logits,
                                                                               hdr, T, d, E);
  else
    logits_mfma4_kernel<InT, 1><<<dim3(cdiv(E, 32), cdiv(T, 32)), 256, 0, s>>>(x, w, bias, logits,
                                                                               hdr, T, d, E);
}

hipError_t launch_logits(int dtype, const void* x, const void* w, const float* bias, float* logits,
                         int32_t* hdr, int T, int d, int E, hipStream_t s) {
  if (T == 0) {
    clear_flags_kernel<<<1, 1, 0, s>>>(hdr);
    return hipGetLastError();
  }
  if (dtype == 0)
    launch_logits_t((const float*)x, (const float*)w, bias, logits, hdr, T, d, E, s);
  else
    launch_logits_t((const uint16_t*)x, (const uint16_t*)w, bias, logits, hdr, T, d, E, s);
  return hipGetLastError();
}

// ---------------------------------------------------------------- top-k_t + weights
// One wavefront per token.  Lane l holds logits g = i*64 + l.  Pick j is the
// wave-wide arg-max over the logits not yet taken, by (logit desc, id asc),
// reduced with cross-lane shuffles; no sort and no global traffic besides the
// logits row and the outputs.
// Wave-wide reductions that leave the result in every lane: four DPP steps inside each row
// of 16 lanes (lane ^ 1, lane ^ 2, mirror inside 8, mirror inside 16), then the four row
// results are read with v_readlane and combined.  No LDS traffic, unlike shuffles.
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
  return __builtin_amdgcn_mov_dpp(v, CTRL, 0xf, 0xf, true);
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;

__device__ __forceinline__ float wave_max_f(float v) {
  v = fmaxf(v, __int_as_float(dpp_i<DPP_XOR1>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_i<DPP_XOR2>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_i<DPP_HALF_MIRROR>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_i<DPP_MIRROR>(__float_as_int(v))));
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ __forceinline__ int wave_min_i(int v) {
  v = min(v, dpp_i<DPP_XOR1>(v));
  v = min(v, dpp_i<DPP_XOR2>(v));
  v = min(v, dpp_i<DPP_HALF_MIRROR>(v));
  v = min(v, dpp_i<DPP_MIRROR>(v));
  const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
  const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
  return min(min(r0, r1), min(r2, r3));
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
  return x;
}

constexpr int TOPK_WAVES = 4;

// The picks run on integer keys: key(f) = bits ^ ((bits >> 31) & 0x7fffffff) orders like f for
// every non-NaN binary32 once -0.0 has been replaced by +0.0 (the two compare equal, and equal
// logits go to the lower id), integer max/min fuse with the cross-lane moves, and INT_MIN, which
// is the key of no logit (-inf maps to 0x807fffff), marks "taken or absent" without a mask.
__device__ __forceinline__ int topk_key(float f) {
  int b = __float_as_int(f);
  b = b == (int)0x80000000 ? 0 : b;  // -0.0 -> +0.0
  return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float topk_unkey(int k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }
__device__ __forceinline__ int wave_max_i(int v) {
  v = max(v, dpp_i<DPP_XOR1>(v));
  v = max(v, dpp_i<DPP_XOR2>(v));
  v = max(v, dpp_i<DPP_HALF_MIRROR>(v));
  v = max(v, dpp_i<DPP_MIRROR>(v));
  const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
  const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
  return max(max(r0, r1), max(r2, r3));
}

template <int ELEMS>
__global__ __launch_bounds__(64 * TOPK_WAVES) void topk_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ k_tok, int32_t* __restrict__ ids,
    float* __restrict__ wout, int32_t* __restrict__ hdr, int T, int E, int k_max, int renorm,
    float scale) {
  extern __shared__ float smem[];  // per wave: the k_max picked logits, then their k_max ids
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int t = blockIdx.x * TOPK_WAVES + wv;
  if (t >= T) return;
  float* se = smem + (size_t)wv * 2 * k_max;
  int* sid = reinterpret_cast<int*>(se + k_max);

  int kt = k_tok != nullptr ? k_tok[t] : k_max;  // null: every token takes k_max
  if (kt < 0 || kt > k_max) {
    if (lane == 0) atomicOr(&hdr[HDR_FLAGS], 1);
    kt = kt < 0 ? 0 : k_max;
  }

  const float NEG_INF = -__builtin_inff();
  constexpr int GONE = (int)0x80000000;  // key of an element that is taken or beyond E
  float v[ELEMS];
  const float* row = logits + (size_t)t * E;
#pragma unroll
  for (int i = 0; i < ELEMS; ++i) {
    int g = i * 64 + lane;
    v[i] = g < E ? row[g] : NEG_INF;
  }
  // full-softmax denominator (only needed when weights are not renormalised)
  float lmax = NEG_INF;
#pragma unroll
  for (int i = 0; i < ELEMS; ++i) lmax = fmaxf(lmax, v[i]);
  const float mx = wave_max_f(lmax);
  float denom = 0.0f;
  if (!renorm) {
#pragma unroll
    for (int i = 0; i < ELEMS; ++i)
      if (i * 64 + lane < E) denom += expf(v[i] - mx);
    denom = wave_sum(denom);
  }

  // Pick j: the wave-wide maximum of the lanes' best free keys, and among the lanes that hold
  // it the smallest sub-expert id (equal logits, +0.0 == -0.0 included, go to the lower id).
  // g = 64 i + lane, so inside a lane the lower element index is the lower id and the winner's
  // lane is g & 63.  Only that lane retires its element and rescans.
  int key[ELEMS];
#pragma unroll
  for (int i = 0; i < ELEMS; ++i) key[i] = i * 64 + lane < E ? topk_key(v[i]) : GONE;
  const int NONE = 0x7fffffff;
  int bk, bg;  // this lane's best free key and its id
  auto rescan = [&]() {
    bk = GONE;
#pragma unroll
    for (int i = 0; i < ELEMS; ++i) bk = max(bk, key[i]);
    int bi = 0;
#pragma unroll
    for (int i = ELEMS - 1; i >= 0; --i) bi = key[i] == bk ? i : bi;  // descending: the lowest index stays
    bg = bk == GONE ? NONE : bi * 64 + lane;
  };
  rescan();
  for (int j = 0; j < kt; ++j) {
    const int top = wave_max_i(bk);  // > GONE: k_t <= k_max <= E, a free element is left
    const unsigned long long holders = __ballot(bk == top);
    int g;
    if (__popcll(holders) == 1)  // the usual case: one lane holds the maximum
      g = __builtin_amdgcn_readlane(bg, __ffsll((long long)holders) - 1);
    else
      g = wave_min_i(bk == top ? bg : NONE);
    if (lane == 0) {
      se[j] = topk_unkey(top);  // exponentials are taken for all picks at once after the loop
      sid[j] = g;
    }
    if ((g & 63) == lane) {
      const int gi = g >> 6;
#pragma unroll
      for (int i = 0; i < ELEMS; ++i) key[i] = i == gi ? GONE : key[i];
      rescan();
    }
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): LDS writes of lane 0 are done
  float dsel = 0.0f;
  for (int j = lane; j < kt; j += 64) dsel += expf(se[j] - mx);
  if (renorm) denom = wave_sum(dsel);
  for (int j = lane; j < k_max; j += 64) {
    bool on = j < kt;
    ids[(size_t)t * k_max + j] = on ? sid[j] : -1;
    wout[(size_t)t * k_max + j] = on ? scale * expf(se[j] - mx) / denom : 0.0f;
  }
}

hipError_t launch_topk(const float* logits, const int32_t* k_tok, int32_t* ids, float* w,
                       int32_t* hdr, int T, int E, int k_max, int renorm, float scale,
                       hipStream_t s) {
  if (T == 0) return hipSuccess;
  dim3 grid(cdiv(T, TOPK_WAVES)), block(64 * TOPK_WAVES);
  size_t sh = (size_t)TOPK_WAVES * 2 * k_max * sizeof(float);
  int elems = cdiv(E, 64);
#define MP_TOPK(N)                                                                              \
  topk_kernel<N><<<grid, block, sh, s>>>(logits, k_tok, ids, w, hdr, T, E, k_max, renorm, scale)
  if (elems <= 1) MP_TOPK(1);
  else if (elems <= 2) MP_TOPK(2);
  else if (elems <= 4) MP_TOPK(4);
  else if (elems <= 8) MP_TOPK(8);
  else if (elems <= 16) MP_TOPK(16);
  else if (elems <= 32) MP_TOPK(32);
  else MP_TOPK(64);
#undef MP_TOPK
  return hipGetLastError();
}

// ---------------------------------------------------------------- proxy gate: per-expert top-kappa
// Sec. 3.2.2, training-free proxy gating.  One thread per (token, expert rank j).  For the expert
// the original router ranked j, the S sub-experts are scored by the mean absolute activation of
// their r gate neurons (act: row slot(t, j) of the proxy activations, sub-expert n at columns
// n r .. n r + r - 1, summed in ascending column order in fp32), and the best kappa[k_t][j] are
// taken, score descending, equal scores to the smaller index.  Selected sub-experts are
// appended in rank order with the expert's weight: rank j writes at the sum of the ranks'
// allocations before it, the last rank also pads the tail.
template <typename ActT>
__device__ __forceinline__ float act_abs(const ActT* p);
template <>
__device__ __forceinline__ float act_abs<float>(const float* p) { return fabsf(*p); }
template <>
__device__ __forceinline__ float act_abs<uint16_t>(const uint16_t* p) { return fabsf(bf16_to_f32(*p)); }

template <typename ActT>
__global__ __launch_bounds__(256) void proxy_select_kernel(
    const ActT* __restrict__ act, int act_ld, const int32_t* __restrict__ ids0,
    const float* __restrict__ w0, const int32_t* __restrict__ slot0,
    const int32_t* __restrict__ k_tok, const int32_t* __restrict__ kappa, int32_t* __restrict__ ids,
    float* __restrict__ w, int32_t* __restrict__ hdr, int T, int S, int r, int m, int k_max) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= T * m) return;
  const int t = idx / m, j = idx % m;
  const int k_cap = min(k_max, m * S);
  int kt = k_tok[t];
  if (kt < 0 || kt > k_cap) {
    if (j == 0) atomicOr(&hdr[HDR_FLAGS], 1);
    kt = kt < 0 ? 0 : k_cap;
  }
  const int32_t* kap_row = kappa + (size_t)kt * m;
  auto alloc = [&](int jj) {
    const int e = ids0[(size_t)t * m + jj], slot = slot0[(size_t)t * m + jj];
    int kap = kap_row[jj];
    kap = kap < 0 ? 0 : (kap > S ? S : kap);
    return (e < 0 || slot < 0) ? 0 : kap;
  };
  int pos = 0;
  for (int jj = 0; jj < j; ++jj) pos += alloc(jj);
  const int kap = alloc(j);
  int32_t* o = ids + (size_t)t * k_max;
  float* ow = w + (size_t)t * k_max;
  if (kap > 0) {
    const int e = ids0[idx];
    const ActT* a = act + (size_t)slot0[idx] * act_ld;
    const float inv_r = 1.0f / (float)r;
    float sc[PROXY_MAX_SUB];
#pragma unroll
    for (int n = 0; n < PROXY_MAX_SUB; ++n) {
      float sum = 0.0f;
      if (n < S)
        for (int c = 0; c < r; ++c) sum += act_abs<ActT>(a + n * r + c);
      sc[n] = n < S ? sum * inv_r : -1.0f;  // scores are >= 0: -1 marks taken or absent
    }
    const float wj = w0[idx];
    for (int i = 0; i < kap && pos < k_max; ++i) {
      int best = 0;
#pragma unroll
      for (int n = 1; n < PROXY_MAX_SUB; ++n)
        if (sc[n] > sc[best]) best = n;
#pragma unroll
      for (int n = 0; n < PROXY_MAX_SUB; ++n)
        if (n == best) sc[n] = -1.0f;
      o[pos] = e * S + best;
      ow[pos] = wj;
      ++pos;
    }
  }
  if (j == m - 1)
    for (; pos < k_max; ++pos) {
      o[pos] = -1;
      ow[pos] = 0.0f;
    }
}

hipError_t launch_proxy_select(int dtype, const void* act, int act_ld, const int32_t* ids0,
                               const float* w0, const int32_t* slot0, const int32_t* k_tok,
                               const int32_t* kappa, int32_t* ids, float* w, int32_t* hdr, int T,
                               int S, int r, int m, int k_max, hipStream_t s) {
  if (T == 0) return hipSuccess;
  if (dtype == 0)
    proxy_select_kernel<float><<<cdiv(T * m, 256), 256, 0, s>>>((const float*)act, act_ld, ids0, w0, slot0,
                                                           k_tok, kappa, ids, w, hdr, T, S, r, m, k_max);
  else
    proxy_select_kernel<uint16_t><<<cdiv(T * m, 256), 256, 0, s>>>((const uint16_t*)act, act_ld, ids0, w0,
                                                              slot0, k_tok, kappa, ids, w, hdr, T, S, r,
                                                              m, k_max);
  return hipGetLastError();
}

}  // namespace mp
