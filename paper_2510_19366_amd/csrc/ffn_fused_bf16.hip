// bf16 grouped SwiGLU FFN (Sec. 3.2.1, Eq. 1-3) for narrow sub-experts, fused: gate-up,
// SwiGLU and the down projection of an m-tile run in one workgroup and the activations
// h never leave the registers.
//
//   y[p, :] = ( SiLU(x[t_p,:] Wg[g]^T) * (x[t_p,:] Wu[g]^T) ) Wd[g]^T        p in group g
//
// Split: a persistent workgroup (8 wavefronts, one per CU) owns an m-tile of 256 slot rows of
// one group; wave w owns rows 32w .. 32w+31 and ALL 2*Is gate/up rows and all d output
// columns.  With v_mfma_f32_32x32x16_bf16 and the weight rows as first operand, a lane ends
// phase 1 with gate and up of 8 consecutive neurons of one slot row (the weight rows of a
// 32-row block are fed in a permuted order: 16 neurons' gate rows and the same neurons' up
// rows).  After SiLU(g)*u those 8 values, packed to bf16, are exactly the second-operand
// fragment of one K step of the down GEMM for the same 32 slot rows: phase 2 takes h from
// registers, no LDS round trip, no barrier between the phases, and neither h nor a second
// pass over the tile table touches HBM.
//
// Operands travel global -> LDS directly (global_load_lds_dwordx4).  Weights: a ring of 4
// slots of Is*128 bytes shared by the waves (phase 1: 2*Is rows x 32 K-elements; phase 2:
// 64 output columns x Is K-elements; both fill a slot exactly), published by one s_barrier
// per stage.  Slot rows of x: a ring of 3 slots of 2 KiB PRIVATE to each wave (a wave copies
// the rows it multiplies itself), so x needs no barrier.  Two stages are in flight while one
// is multiplied.  vmcnt retires in issue order, so "everything but the operations this wave
// issued in the previous iteration has landed" is one s_waitcnt with that count.
#include "ffn_common.h"

namespace mp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace fused {

constexpr int NT = 512;   // threads: 8 waves
constexpr int BM = FFN_BM;
constexpr int NSW = 4;    // weight ring slots
constexpr int NSX = 3;    // x ring slots (per wave)
constexpr int X_WAVE = 32 * 64;        // bytes of one wave's x stage: 32 rows x 32 K-elements
constexpr int X_SLOT = 8 * X_WAVE;

template <int IS>
struct Cfg {
  static_assert(IS % 64 == 0 && IS >= 64 && IS <= 192, "fused path: Is in {64, 128, 192}");
  static constexpr int NBLK = IS / 16;     // 32-row weight blocks of phase 1 = K steps of phase 2
  static constexpr int WPW = IS / 64;      // copy instructions per wave and weight stage
  static constexpr int W_SLOT = IS * 128;  // bytes
  static constexpr int CPR = IS / 8;       // 16-byte chunks per weight row in phase 2
  static constexpr int ROW2 = IS * 2;      // bytes per weight row in phase 2
  static constexpr int OFF_X = NSW * W_SLOT;
  static constexpr int OFF_PAIR = OFF_X + NSX * X_SLOT;
  static constexpr int LDS_BYTES = OFF_PAIR + 2 * BM * 4;
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per CU");
};

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// one wave-wide copy global -> LDS: lane i's 16 (4) bytes at base + voff land at lds + 16 i (4 i).
// m0 is reserved by the compiler, so its value is put back.
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t lds) {
  uint32_t keep;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 1\n\t"
      "global_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
      : "=&s"(keep)
      : "v"(voff), "s"(base), "s"(lds)
      : "memory");
}
__device__ __forceinline__ void dma4(const void* base, uint32_t voff, uint32_t lds) {
  uint32_t keep;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 1\n\t"
      "global_load_lds_dword %1, %2\n\ts_mov_b32 m0, %0"
      : "=&s"(keep)
      : "v"(voff), "s"(base), "s"(lds)
      : "memory");
}
// 16-byte store at base + voff + IMM, counted by hand like the copies (the compiler neither
// merges nor splits it).  A store of more than 8 bytes reads its data registers for a few
// cycles after issue and the compiler's hazard handling does not look inside an asm block:
// the s_nop keeps the next VALU write away from them.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <int IMM>
__device__ __forceinline__ void store16(void* base, uint32_t voff, u32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3\n\ts_nop 1" ::"v"(voff), "v"(v), "s"(base), "n"(IMM)
               : "memory");
}
// until at most n of this wave's vector memory operations are pending (n is wave-uniform)
__device__ __forceinline__ void wait_pending(int n) {
#define MP_W(N) \
  case N:       \
    asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); \
    break;
  switch (n) {
    MP_W(0) MP_W(1) MP_W(2) MP_W(3) MP_W(4) MP_W(5) MP_W(6) MP_W(7) MP_W(8) MP_W(9) MP_W(10)
    MP_W(11) MP_W(12)
    default:
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
#undef MP_W
}
__device__ __forceinline__ void barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ float silu_mul(float a, float u) {
  return __fdividef(a, 1.0f + __expf(-a)) * u;
}

// weight-row permutations (MFMA row i = 8a + 4hi + b of a 32-row block):
// phase 1: block row 16*(a>>1) + 8hi + 4(a&1) + b, block rows 0..15 = gate rows of 16 neurons,
// 16..31 = their up rows: accumulators 0..7 of a lane = gate of neurons 8hi..8hi+7, 8..15 = up
__device__ __forceinline__ int wrow_gu(int i) {
  const int a = i >> 3, hi = (i >> 2) & 1, b = i & 3;
  return 16 * (a >> 1) + 8 * hi + 4 * (a & 1) + b;
}
// phase 2: block row 16hi + 4a + b: a lane's 16 accumulators = output columns 16hi .. 16hi+15
__device__ __forceinline__ int wrow_dn(int i) {
  const int a = i >> 3, hi = (i >> 2) & 1, b = i & 3;
  return 16 * hi + 4 * a + b;
}
// LDS swizzles (16-byte chunk c of row r sits at chunk position c ^ f(r)); 16 lanes read 16
// rows at one chunk index, f spreads them over all banks.
// 64-byte rows (phase 1, both operands): rows of equal r & 3 share banks
__device__ __forceinline__ int f1(int r) { return (r >> 2) & 3; }
// Is*2-byte rows (phase 2): 384- and 128-byte rows alternate between two bank halves (8 rows of
// equal parity must differ), 256-byte rows all start in bank 0 (16 rows must differ); the 16
// rows read together are {0..7, 16..23} + const
template <int IS>
__device__ __forceinline__ int f2(int r) {
  return IS == 128 ? ((r & 7) | (((r >> 4) & 1) << 3)) : (((r >> 1) & 3) | (((r >> 4) & 1) << 2));
}

struct TileHdr {  // wave-uniform
  int g, row0, rows;
};

template <int IS>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void ffn_fused_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_gu,
    const uint16_t* __restrict__ w_dn, const int32_t* __restrict__ sorted_pair,
    const MTile* __restrict__ tiles, int32_t* __restrict__ hdr, uint16_t* __restrict__ y, int T,
    int d, int k_max) {
  using C = Cfg<IS>;
  constexpr int NBLK = C::NBLK, WPW = C::WPW;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63, wv = uni(threadIdx.x >> 6);
  const int S1 = d / 32, S2 = d / 64, ST = S1 + S2;

  const int n_tiles = hdr[HDR_MTILES];
  const ItemRange ir = xcd_items(n_tiles);
  const int n_my = ir.begin < ir.end ? (ir.end - ir.begin + ir.step - 1) / ir.step : 0;
  if (n_my == 0) return;  // uniform over the workgroup
  const int total = n_my * ST;

  const uint32_t lds0 = lds_addr(smem);
  const int32_t* pair_lds = reinterpret_cast<const int32_t*>(smem + C::OFF_PAIR);

  auto load_hdr = [&](int my_idx, TileHdr& t) {
    const MTile m = tiles[ir.begin + my_idx * ir.step];
    t.g = uni(m.g);
    t.row0 = uni(m.row0);
    t.rows = uni(m.rows);
  };

  // ---- per-lane copy offsets that never change
  // phase 1 weights: piece pc = 16 ring rows; ring row lr holds block row lr & 31 of block lr >> 5
  uint32_t voff_w1[WPW], voff_w2[WPW];
#pragma unroll
  for (int j = 0; j < WPW; ++j) {
    const int pc = wv * WPW + j;
    const int lr = pc * 16 + (lane >> 2), pos = lane & 3;
    const int rr = lr & 31, neuron = (lr >> 5) * 16 + (rr & 15);
    const int grow = (rr >> 4) ? IS + neuron : neuron;
    voff_w1[j] = (uint32_t)grow * (uint32_t)d * 2u + (uint32_t)((pos ^ f1(lr)) * 16);
    // phase 2 weights: piece = 64 consecutive 16-byte positions of a [64 x CPR] slot
    const int p = pc * 64 + lane, r2 = p / C::CPR, pos2 = p % C::CPR;
    voff_w2[j] = (uint32_t)r2 * C::ROW2 + (uint32_t)((pos2 ^ f2<IS>(r2)) * 16);
  }
  // ---- per-lane fragment read offsets (bytes inside a slot)
  const int fr = lane & 31, fh = lane >> 5;
  // phase 1: row wrow_gu(fr) (+ 32 per block), chunk 2 ks + fh
  uint32_t rd_w1[2], rd_x[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int r = wrow_gu(fr), c = 2 * ks + fh;
    rd_w1[ks] = (uint32_t)(r * 64 + ((c ^ f1(r)) * 16));
    rd_x[ks] = (uint32_t)(fr * 64 + ((c ^ f1(fr)) * 16));
  }
  const int r2rd = wrow_dn(fr);
  const uint32_t rd_w2_row = (uint32_t)r2rd * C::ROW2;
  const int f2rd = f2<IS>(r2rd);

  // x offsets of the rows this lane copies (2 pieces of 16 rows), for the current / next tile
  uint32_t xoff_cur[2], xoff_nxt[2];
  auto x_offsets = [&](int parity, uint32_t (&xo)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int lr = j * 16 + (lane >> 2), pos = lane & 3;
      int tok = pair_lds[parity * BM + wv * 32 + lr] / k_max;
      tok = min(max(tok, 0), T - 1);
      xo[j] = (uint32_t)tok * (uint32_t)d * 2u + (uint32_t)((pos ^ f1(lr)) * 16);
    }
  };
  auto fetch_pairs = [&](const TileHdr& t, int parity) -> int {  // waves 0..3, 64 rows each
    if (wv >= 4) return 0;
    const int r = max(min(wv * 64 + lane, t.rows - 1), 0);
    dma4(sorted_pair + t.row0, (uint32_t)r * 4u, lds0 + C::OFF_PAIR + (uint32_t)(parity * BM + wv * 64) * 4u);
    return 1;
  };
  // copies of weight stage s of a tile into ring slot `slot`
  auto issue_w = [&](const TileHdr& t, int s, int slot) -> int {
    const uint32_t dst = lds0 + (uint32_t)slot * C::W_SLOT + (uint32_t)(wv * WPW) * 1024u;
    if (s < S1) {
      const uint16_t* base = w_gu + (size_t)t.g * (2 * IS) * d + (size_t)s * 32;
#pragma unroll
      for (int j = 0; j < WPW; ++j) dma16(base, voff_w1[j], dst + j * 1024u);
    } else {
      const uint16_t* base = w_dn + ((size_t)t.g * d + (size_t)(s - S1) * 64) * IS;
#pragma unroll
      for (int j = 0; j < WPW; ++j) dma16(base, voff_w2[j], dst + j * 1024u);
    }
    return WPW;
  };
  // copies of this wave's rows of x stage s (phase 1 only) into its private ring slot
  auto issue_x = [&](const TileHdr& t, const uint32_t (&xo)[2], int s, int slot) -> int {
    if (s >= S1 || t.rows <= wv * 32) return 0;
    const uint32_t dst = lds0 + C::OFF_X + (uint32_t)slot * X_SLOT + (uint32_t)wv * X_WAVE;
    const uint16_t* base = x + (size_t)s * 32;
    dma16(base, xo[0], dst);
    dma16(base, xo[1], dst + 1024u);
    return 2;
  };

  // ---- prologue: tile 0's slot list, then the first stages
  TileHdr cur, nxt;
  load_hdr(0, cur);
  nxt = cur;
  if (n_my > 1) load_hdr(1, nxt);
  fetch_pairs(cur, 0);
  wait_pending(0);
  barrier();
  x_offsets(0, xoff_cur);
  xoff_nxt[0] = xoff_cur[0];
  xoff_nxt[1] = xoff_cur[1];

  // producer cursors: stage inside its tile and whether that tile is `nxt`
  int pw_s = 0, pw_next = 0, pw_slot = 0;  // next weight stage to issue
  int px_s = 0, px_next = 0, px_slot = 0;  // next x stage to issue
  int pw_q = 0, px_q = 0;                  // their global stage numbers
  auto produce_w = [&]() -> int {
    if (pw_q >= total) return 0;
    const int n = issue_w(pw_next ? nxt : cur, pw_s, pw_slot);
    ++pw_q;
    pw_slot = pw_slot + 1 == NSW ? 0 : pw_slot + 1;
    if (++pw_s == ST) {
      pw_s = 0;
      pw_next = 1;
    }
    return n;
  };
  auto produce_x = [&]() -> int {
    if (px_q >= total) return 0;
    const int n = px_next ? issue_x(nxt, xoff_nxt, px_s, px_slot) : issue_x(cur, xoff_cur, px_s, px_slot);
    ++px_q;
    px_slot = px_slot + 1 == NSX ? 0 : px_slot + 1;
    if (++px_s == ST) {
      px_s = 0;
      px_next = 1;
    }
    return n;
  };
  produce_w();  // W(0)
  produce_w();  // W(1)
  produce_x();  // x(0)
  int cnt_prev = produce_w();  // W(2)   } the group an iteration would have issued
  cnt_prev += produce_x();     // x(1)   }
  wait_pending(cnt_prev);      // W(0), W(1), x(0) have landed
  barrier();

  int tile_i = 0, c_wslot = 0, c_xslot = 0;
  // head of every iteration (stage s of the current tile): everything this wave issued before
  // the previous iteration has landed, i.e. its part of W(q+1), and x(q); the barrier
  // publishes W(q+1) and frees the slot of W(q-1); then the copies of W(q+3) and x(q+2) go out
  auto head = [&](int s) -> int {
    wait_pending(cnt_prev);
    barrier();
    int cnt = produce_w();
    cnt += produce_x();
    if (s == 1 && tile_i + 1 < n_my) cnt += fetch_pairs(nxt, (tile_i + 1) & 1);
    if (s == S1 && tile_i + 1 < n_my) x_offsets((tile_i + 1) & 1, xoff_nxt);
    return cnt;
  };

  for (; tile_i < n_my; ++tile_i) {
    const bool active = cur.rows > wv * 32;
    bf16x8 hfrag[NBLK];
    {
      // ---- phase 1: acc1[blk] += W-block(blk) x-rows^T, 32 K-elements per stage
      f32x16 acc1[NBLK];
#pragma unroll
      for (int b = 0; b < NBLK; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc1[b][v] = 0.0f;
      for (int s = 0; s < S1; ++s) {
        cnt_prev = head(s);
        if (active) {
          const unsigned char* wslot = smem + c_wslot * C::W_SLOT;
          const unsigned char* xs = smem + C::OFF_X + c_xslot * X_SLOT + wv * X_WAVE;
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 xa = *reinterpret_cast<const bf16x8*>(xs + rd_x[ks]);
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
              const bf16x8 wf = *reinterpret_cast<const bf16x8*>(wslot + rd_w1[ks] + b * 2048);
              acc1[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xa, acc1[b], 0, 0, 0);
            }
          }
        }
        c_wslot = c_wslot + 1 == NSW ? 0 : c_wslot + 1;
        c_xslot = c_xslot + 1 == NSX ? 0 : c_xslot + 1;
      }
      // ---- SwiGLU: gate/up accumulators -> the bf16 K-step fragments of phase 2
#pragma unroll
      for (int b = 0; b < NBLK; ++b) {
        const f32x16 v = acc1[b];
        const uint4 pk = make_uint4(pack_bf16x2(silu_mul(v[0], v[8]), silu_mul(v[1], v[9])),
                                    pack_bf16x2(silu_mul(v[2], v[10]), silu_mul(v[3], v[11])),
                                    pack_bf16x2(silu_mul(v[4], v[12]), silu_mul(v[5], v[13])),
                                    pack_bf16x2(silu_mul(v[6], v[14]), silu_mul(v[7], v[15])));
        hfrag[b] = __builtin_bit_cast(bf16x8, pk);
      }
    }
    // ---- phase 2: 64 output columns per stage, K = Is from the register-resident h fragments
    const int row = wv * 32 + fr;
    const uint32_t vo = (uint32_t)row * (uint32_t)d * 2u + (uint32_t)fh * 32u;
    for (int s2 = 0; s2 < S2; ++s2) {
      int cnt = head(S1 + s2);
      if (active) {
        const unsigned char* wslot = smem + c_wslot * C::W_SLOT;
        f32x16 acc2[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc2[b][v] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < NBLK; ++ks) {
          const uint32_t co = (uint32_t)(((2 * ks + fh) ^ f2rd) * 16);
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const bf16x8 wd = *reinterpret_cast<const bf16x8*>(wslot + rd_w2_row + b * 32 * C::ROW2 + co);
            acc2[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wd, hfrag[ks], acc2[b], 0, 0, 0);
          }
        }
        // lane (row fr, half fh) holds columns 64 s2 + 32 b + 16 fh + 0..15 of slot row 32 wv + fr
        if (row < cur.rows) {
          uint16_t* ybase = y + (size_t)cur.row0 * d + (size_t)s2 * 64;
          const f32x16 a0 = acc2[0], a1 = acc2[1];
          store16<0>(ybase, vo, u32x4{pack_bf16x2(a0[0], a0[1]), pack_bf16x2(a0[2], a0[3]),
                                           pack_bf16x2(a0[4], a0[5]), pack_bf16x2(a0[6], a0[7])});
          store16<16>(ybase, vo, u32x4{pack_bf16x2(a0[8], a0[9]), pack_bf16x2(a0[10], a0[11]),
                                            pack_bf16x2(a0[12], a0[13]), pack_bf16x2(a0[14], a0[15])});
          store16<64>(ybase, vo, u32x4{pack_bf16x2(a1[0], a1[1]), pack_bf16x2(a1[2], a1[3]),
                                            pack_bf16x2(a1[4], a1[5]), pack_bf16x2(a1[6], a1[7])});
          store16<80>(ybase, vo, u32x4{pack_bf16x2(a1[8], a1[9]), pack_bf16x2(a1[10], a1[11]),
                                            pack_bf16x2(a1[12], a1[13]), pack_bf16x2(a1[14], a1[15])});
        }
        cnt += 4;  // row 32 wv of an active wave is valid, so the four stores were issued
      }
      cnt_prev = cnt;
      c_wslot = c_wslot + 1 == NSW ? 0 : c_wslot + 1;
      c_xslot = c_xslot + 1 == NSX ? 0 : c_xslot + 1;  // the x ring turns with every stage
    }
    // ---- next tile
    cur = nxt;
    xoff_cur[0] = xoff_nxt[0];
    xoff_cur[1] = xoff_nxt[1];
    pw_next = 0;
    px_next = 0;
    if (tile_i + 2 < n_my) load_hdr(tile_i + 2, nxt);
  }
}

template <int IS>
static hipError_t launch_is(const uint16_t* x, const uint16_t* w_gu, const uint16_t* w_dn,
                            const int32_t* sorted_pair, const MTile* tiles, int32_t* hdr,
                            uint16_t* y, int T, int d, int k_max, int max_mtiles, hipStream_t s) {
  static bool done[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
  if (dev < 0 || !done[dev]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_fused_kernel<IS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg<IS>::LDS_BYTES);
    if (e != hipSuccess) return e;
    if (dev >= 0) done[dev] = true;
  }
  const int grid = persistent_grid(max_mtiles, 1);
  ffn_fused_kernel<IS><<<grid, NT, Cfg<IS>::LDS_BYTES, s>>>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y,
                                                            T, d, k_max);
  return hipGetLastError();
}

}  // namespace fused

// Shapes the fused kernel takes: Is in {64, 128, 192}; d a multiple of 64 with at least 8
// phase-1 stages (the next tile's slot list is fetched while the current tile runs); 32-bit
// byte offsets inside x and inside one sub-expert's weights.
bool ffn_fused_supported(int T, int d, int Is) {
  if (Is != 64 && Is != 128 && Is != 192) return false;
  if (d % 64 != 0 || d < 256) return false;
  if ((long)T * d * 2 >= (1L << 32) || (long)2 * Is * d * 2 >= (1L << 32)) return false;
  if ((long)FFN_BM * d * 2 >= (1L << 32)) return false;
  return true;
}

hipError_t launch_ffn_fused_bf16(const uint16_t* x, const uint16_t* w_gu, const uint16_t* w_dn,
                                 const int32_t* sorted_pair, const MTile* tiles, int32_t* hdr,
                                 uint16_t* y, int T, int d, int Is, int k_max, int max_mtiles,
                                 hipStream_t s) {
  if (max_mtiles <= 0) return hipSuccess;
  switch (Is) {
    case 64: return fused::launch_is<64>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y, T, d, k_max, max_mtiles, s);
    case 128: return fused::launch_is<128>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y, T, d, k_max, max_mtiles, s);
    case 192: return fused::launch_is<192>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y, T, d, k_max, max_mtiles, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mp
