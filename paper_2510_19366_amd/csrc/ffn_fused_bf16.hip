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
#include <type_traits>

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
constexpr int EPI_WAVE = 1024;         // bytes of a wave's output staging: 16 rows x 32 columns
constexpr int RUN = 32;   // consecutive tiles an XCD takes per turn
constexpr int PD = 4;     // fragment reads in flight ahead of the MFMAs

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
  static constexpr int OFF_EPI = OFF_PAIR + 2 * BM * 4;  // 1 KiB per wave: output transposition
  static constexpr int OFF_DYN = OFF_EPI + 8 * EPI_WAVE;  // two words: tile numbers drawn by wave 0
  static constexpr int LDS_BYTES = OFF_DYN + 16;
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per CU");
};

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Wave-wide copies global -> LDS: lane i's 16 (4) bytes at base + voff land at lds + 16 i (4 i).
// N copies of one group go to consecutive KiB of LDS.  m0 carries the LDS address; it is
// reserved by the compiler, so its value is put back.
template <int N>
__device__ __forceinline__ void dma16_group(const void* base, const uint32_t (&voff)[N], uint32_t lds) {
  static_assert(N >= 1 && N <= 3, "copies per group");
  uint32_t keep;
  if constexpr (N == 1) {
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(voff[0]), "s"(base), "s"(lds)
        : "memory");
  } else if constexpr (N == 2) {
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %4\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %3\n\ts_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(voff[0]), "v"(voff[1]), "s"(base), "s"(lds)
        : "memory", "scc");
  } else {
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %5\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %4\n\ts_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %2, %4\n\ts_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %3, %4\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "s"(base), "s"(lds)
        : "memory", "scc");
  }
}
__device__ __forceinline__ void dma4(const void* base, uint32_t voff, uint32_t lds) {
  uint32_t keep;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
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
// f(integral_constant<I>) for I = BEGIN .. END-1: a loop whose index can be a template argument
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(std::integral_constant<int, BEGIN>{});
    static_for<BEGIN + 1, END>(f);
  }
}
// until at most n of this wave's vector memory operations are pending (n is wave-uniform, 0..12;
// the count is an immediate of s_waitcnt, so n selects one of 13 instructions by bisection)
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
template <int LO, int HI>
__device__ __forceinline__ void wait_bisect(int n) {
  if constexpr (LO == HI) {
    wait_vm<LO>();
  } else {
    constexpr int MID = (LO + HI + 1) / 2;
    if (n >= MID)
      wait_bisect<MID, HI>(n);
    else
      wait_bisect<LO, MID - 1>(n);
  }
}
__device__ __forceinline__ void wait_pending(int n) { wait_bisect<0, 12>(n > 12 ? 0 : n); }
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

// One matrix-core step.  MATH = false is the traffic probe: the same operand reads, copies,
// barriers, waits and stores, with one cheap ALU operation in place of the multiply (the
// fragments stay live, the results mean nothing).
template <bool MATH>
__device__ __forceinline__ f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) {
  if constexpr (MATH) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  } else {
    const uint4 u = __builtin_bit_cast(uint4, a), v = __builtin_bit_cast(uint4, b);
    c[0] += __uint_as_float((u.x ^ v.x) & 0x3fffffffu);
    c[5] += __uint_as_float((u.w ^ v.y) & 0x3fffffffu);
    return c;
  }
}

template <int IS, bool MATH>
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

  // Tiles are drawn at run time, one tile ahead of the one being multiplied, in table order
  // (group-major: ragged tails, which only stream weights, stay interleaved with full tiles;
  // drawing the heavy tiles first measured slower).  The workgroups of an XCD (workgroup b runs
  // on XCD b % 8) share a cursor: the i-th tile an XCD draws is (i / RUN) * 8 RUN + xcd * RUN +
  // i % RUN, so runs of RUN consecutive tiles, which mostly belong to one group, meet in one L2.
  const int n_tiles = hdr[HDR_MTILES];
  const int xcd = blockIdx.x % N_XCD;
  int32_t* dyn_lds = reinterpret_cast<int32_t*>(smem + C::OFF_DYN);
  auto draw = [&]() {  // one lane of the workgroup
    const int i = atomicAdd(&hdr[HDR_DYN_FUSED + xcd], 1);
    return (i / RUN) * (RUN * N_XCD) + xcd * RUN + (i % RUN);
  };
  if (threadIdx.x == 0) {
    dyn_lds[0] = draw();
    dyn_lds[1] = draw();
  }
  __syncthreads();
  const int k0 = uni(dyn_lds[0]), k1 = uni(dyn_lds[1]);
  if (k0 >= n_tiles) return;  // uniform over the workgroup
  __syncthreads();            // dyn_lds is written again below

  const uint32_t lds0 = lds_addr(smem);
  const int32_t* pair_lds = reinterpret_cast<const int32_t*>(smem + C::OFF_PAIR);

  auto load_hdr = [&](int k, TileHdr& t) {
    const MTile m = tiles[k];
    t.g = uni(m.g);
    t.row0 = uni(m.row0);
    t.rows = uni(m.rows);
  };

  // ---- per-lane copy offsets that never change
  // phase 1 weights: piece pc = 16 ring rows; ring row lr holds block row lr & 31 of block lr >> 5
  uint32_t voff_w1[WPW];
#pragma unroll
  for (int j = 0; j < WPW; ++j) {
    const int pc = wv * WPW + j;
    const int lr = pc * 16 + (lane >> 2), pos = lane & 3;
    const int rr = lr & 31, neuron = (lr >> 5) * 16 + (rr & 15);
    const int grow = (rr >> 4) ? IS + neuron : neuron;
    voff_w1[j] = (uint32_t)grow * (uint32_t)d * 2u + (uint32_t)((pos ^ f1(lr)) * 16);
  }
  // phase 2 weights: piece = 64 consecutive 16-byte positions of a [64 x CPR] slot; computed
  // when needed (registers are scarcest in phase 1, which does not use these)
  auto voff_w2 = [&](int j) {
    const int p = (wv * WPW + j) * 64 + lane, r2 = p / C::CPR, pos2 = p % C::CPR;
    return (uint32_t)r2 * C::ROW2 + (uint32_t)((pos2 ^ f2<IS>(r2)) * 16);
  };
  // A copy of the lane id that the optimiser cannot see through: per-lane constants of one
  // phase are derived from it at the start of that phase, so they do not occupy registers
  // during the other (phase 1 runs at the register limit).
  auto opaque_lane = [&]() {
    int l = lane;
    asm volatile("" : "+v"(l));
    return l;
  };

  // x offsets of the rows this lane copies (2 pieces of 16 rows) from a tile's slot list in LDS
  auto x_offsets = [&](int parity, uint32_t (&xo)[2]) {
    const int l = opaque_lane();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int lr = j * 16 + (l >> 2), pos = l & 3;
      int tok = pair_lds[parity * BM + wv * 32 + lr] / k_max;
      tok = min(max(tok, 0), T - 1);
      xo[j] = (uint32_t)tok * (uint32_t)d * 2u + (uint32_t)((pos ^ f1(lr)) * 16);
    }
  };
  auto fetch_pairs = [&](const TileHdr& t, int parity) -> int {  // waves 0..3, 64 rows each
    if (wv >= 4) return 0;
    const int r = max(min(wv * 64 + opaque_lane(), t.rows - 1), 0);
    dma4(sorted_pair + t.row0, (uint32_t)r * 4u, lds0 + C::OFF_PAIR + (uint32_t)(parity * BM + wv * 64) * 4u);
    return 1;
  };

  // ---- prologue: tile 0's slot list
  TileHdr cur, nxt;
  load_hdr(k0, cur);
  nxt = cur;
  bool has_next = k1 < n_tiles;
  if (has_next) load_hdr(k1, nxt);
  int k_after = n_tiles;  // the tile after `nxt` (>= n_tiles: none)
  int par = 0;            // which half of the slot-list buffer holds the current tile's entries
  fetch_pairs(cur, 0);
  wait_vm<0>();
  barrier();

  // ---- producers.  Each keeps a running global pointer and LDS address and counts the stages
  // left in its phase; they run ahead of the multiplying code across phase and tile borders
  // (the next tile's header `nxt` is known a whole tile ahead).
  // weights: stage q + 3
  const uint16_t* pw_ptr = w_gu + (size_t)cur.g * (2 * IS) * d;
  int pw_g = cur.g, pw_phase = 0, pw_cnt = S1;
  bool pw_on = true;  // false once the last tile's last stage has been issued
  const uint32_t pw_dst0 = lds0 + (uint32_t)(wv * WPW) * 1024u;
  uint32_t pw_dst = pw_dst0;
  auto produce_w = [&]() -> int {
    if (!pw_on) return 0;
    if (pw_phase) {
      uint32_t vo[WPW];
#pragma unroll
      for (int j = 0; j < WPW; ++j) vo[j] = voff_w2(j);
      dma16_group<WPW>(pw_ptr, vo, pw_dst);
      pw_ptr += 64 * IS;
    } else {
      dma16_group<WPW>(pw_ptr, voff_w1, pw_dst);
      pw_ptr += 32;
    }
    pw_dst = pw_dst + C::W_SLOT == pw_dst0 + NSW * C::W_SLOT ? pw_dst0 : pw_dst + C::W_SLOT;
    if (--pw_cnt == 0) {
      if (pw_phase == 0) {  // on to the down weights of the same group
        pw_phase = 1;
        pw_cnt = S2;
        pw_ptr = w_dn + (size_t)pw_g * d * IS;
      } else if (has_next) {  // on to the next tile
        pw_phase = 0;
        pw_cnt = S1;
        pw_g = nxt.g;
        pw_ptr = w_gu + (size_t)pw_g * (2 * IS) * d;
      } else {
        pw_on = false;
      }
    }
    return WPW;
  };
  // x: stage q + 2, phase-1 stages only, and only for a wave that has rows in the tile.  The
  // cursor leaves a tile only while the multiplying code is in that tile's phase 2, which is
  // where the next tile's offsets `xo_next` live.
  uint32_t xoff[2];
  x_offsets(0, xoff);
  const uint16_t* px_ptr = x;
  int px_s = 0;
  bool px_on = true;
  bool px_act = cur.rows > wv * 32;
  const uint32_t px_dst0 = lds0 + C::OFF_X + (uint32_t)wv * X_WAVE;
  uint32_t px_dst = px_dst0;
  auto produce_x = [&](const uint32_t* xo_next) -> int {
    if (!px_on) return 0;
    int n = 0;
    if (px_s < S1 && px_act) {
      dma16_group<2>(px_ptr, xoff, px_dst);
      n = 2;
    }
    px_ptr += 32;
    px_dst = px_dst + X_SLOT == px_dst0 + NSX * X_SLOT ? px_dst0 : px_dst + X_SLOT;
    if (++px_s == ST && xo_next != nullptr) {
      if (has_next) {  // on to the next tile
        px_s = 0;
        px_ptr = x;
        px_act = nxt.rows > wv * 32;
        xoff[0] = xo_next[0];
        xoff[1] = xo_next[1];
      } else {
        px_on = false;
      }
    }
    return n;
  };
  // Stage numbering: q counts the stages this workgroup walks.  Per iteration q a wave
  //   (a) multiplies stage q (W(q) was published by the barrier of iteration q - 1, x(q) is its own),
  //   (b) passes barrier(q): every wave has finished reading W(q-1), and W(q+1) is published,
  //   (c) issues its copies of x(q+2) and W(q+3) (into the slots of x(q-1), W(q-1)),
  //   (d) waits until everything it issued before (c) has landed, except the output stores of
  //       the previous iteration: that is x(q+1) and its part of W(q+2) (issued in iteration
  //       q - 1).  From here on the x fragments of stage q + 1 may be read.
  // (b) and (c) sit between MFMAs of (a) so that their scalar work hides behind them; (d) closes
  // the iteration.
  produce_w();  // W(0)
  produce_w();  // W(1)
  produce_x(nullptr);  // x(0)
  {
    int c0 = produce_x(nullptr);  // x(1)  } what iteration -1 would have issued
    c0 += produce_w();            // W(2)  }
    wait_pending(c0);             // W(0), W(1), x(0) have landed
  }
  barrier();

  // wave 0 draws the tile after `nxt` early in a tile (its wait for the returned number drains
  // that wave's copies once per tile); every wave picks the number up two barriers later
  auto sched_hook = [&](int s) {
    if (s == 0 && has_next && threadIdx.x == 0) dyn_lds[0] = draw();
    if (s == 2 && has_next) k_after = uni(dyn_lds[0]);
  };
  uint32_t c_w = 0, c_x = 0;  // byte offsets of the ring slots of stage q
  int n_allow = 0;  // operations that may still be pending at (d): last iteration's output stores + (c)
  auto step_d = [&]() {
    wait_pending(n_allow);
    n_allow = 0;
  };
  auto next_w = [&](uint32_t c) { return c + C::W_SLOT == NSW * C::W_SLOT ? 0u : c + C::W_SLOT; };
  auto next_x = [&](uint32_t c) { return c + X_SLOT == NSX * X_SLOT ? 0u : c + X_SLOT; };
  constexpr int STEPS = 2 * NBLK;          // MFMAs per wave and stage, both phases
  constexpr int B_STEP = 1;                // (b), (c) after this step
  // (d) after the last step: the copies get the longest possible flight (two iterations; measured
  // 4-6 % faster than waiting earlier and reading the next stage's x fragments inside the stream);
  // only the x fragments of stage q + 1 depend on (d), the weight fragments of stage q + 1 are
  // already published and are read during the last PD steps
  constexpr int WT_STEP = STEPS - 1;
  static_assert(WT_STEP > B_STEP, "order of the in-stage hooks");

  for (;;) {
    if (cur.rows <= wv * 32) {
      // a wave whose 32 rows lie beyond the tile's rows only takes part in the copies and barriers
      uint32_t xo_next[2] = {xoff[0], xoff[1]};
      for (int s = 0; s < ST; ++s) {
        barrier();
        n_allow += produce_x(xo_next);
        n_allow += produce_w();
        sched_hook(s);
        if (s == 1 && has_next) n_allow += fetch_pairs(nxt, par ^ 1);
        if (s == S1 && has_next) x_offsets(par ^ 1, xo_next);
        step_d();
        c_w = next_w(c_w);
        c_x = next_x(c_x);
      }
    } else {
      bf16x8 hfrag[NBLK];
      {
        // ---- phase 1: acc1[blk] += W-block(blk) x-rows^T, 32 K-elements (2 K steps) per stage.
        // The fragment of step i + PD is read right after the MFMA of step i is issued (the
        // scheduling barriers keep that order), and the stream of reads runs on into the next
        // stage (after the last stage of the phase it reads a slot whose values are not used).
        const int l = opaque_lane(), fr = l & 31, fh = l >> 5;
        // fragment read offsets: row wrow_gu(fr) (+ 32 per block), chunk 2 ks + fh
        uint32_t rd_w1[2], rd_x[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const int r = wrow_gu(fr), c = 2 * ks + fh;
          rd_w1[ks] = (uint32_t)(r * 64 + ((c ^ f1(r)) * 16));
          rd_x[ks] = (uint32_t)(C::OFF_X + wv * X_WAVE + fr * 64 + ((c ^ f1(fr)) * 16));
        }
        auto rd_w1f = [&](uint32_t slot, int step) {
          return *reinterpret_cast<const bf16x8*>(smem + slot + rd_w1[step / NBLK] + (step % NBLK) * 2048);
        };
        auto rd_xf = [&](uint32_t slot, int ks) {
          return *reinterpret_cast<const bf16x8*>(smem + slot + rd_x[ks]);
        };
        f32x16 acc1[NBLK];
#pragma unroll
        for (int b = 0; b < NBLK; ++b)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc1[b][v] = 0.0f;
        bf16x8 xa[2], wf[PD];
        xa[0] = rd_xf(c_x, 0);
#pragma unroll
        for (int i = 0; i < PD; ++i) wf[i] = rd_w1f(c_w, i);
        xa[1] = rd_xf(c_x, 1);
        for (int s = 0; s < S1; ++s) {
          const uint32_t nw = next_w(c_w), nx = next_x(c_x);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < STEPS; ++i) {
            acc1[i % NBLK] = mma<MATH>(wf[i % PD], xa[i / NBLK], acc1[i % NBLK]);
            wf[i % PD] = i + PD < STEPS ? rd_w1f(c_w, i + PD) : rd_w1f(nw, i + PD - STEPS);
            __builtin_amdgcn_sched_barrier(0);
            if (i == B_STEP) {
              barrier();
              n_allow += produce_x(nullptr);  // stays inside this tile's stages
              n_allow += produce_w();
              sched_hook(s);
              if (s == 1 && has_next) n_allow += fetch_pairs(nxt, par ^ 1);
              __builtin_amdgcn_sched_barrier(0);
            }
            if (i == WT_STEP) {
              step_d();
              __builtin_amdgcn_sched_barrier(0);
            }
          }
          xa[0] = rd_xf(nx, 0);
          xa[1] = rd_xf(nx, 1);
          c_w = nw;
          c_x = nx;
        }
        // ---- SwiGLU: gate/up accumulators -> the bf16 K-step fragments of phase 2, block by
        // block (16 accumulator registers become 4), before anything of phase 2 is read
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
          const f32x16 v = acc1[b];
          const uint4 pk = make_uint4(pack_bf16x2(silu_mul(v[0], v[8]), silu_mul(v[1], v[9])),
                                      pack_bf16x2(silu_mul(v[2], v[10]), silu_mul(v[3], v[11])),
                                      pack_bf16x2(silu_mul(v[4], v[12]), silu_mul(v[5], v[13])),
                                      pack_bf16x2(silu_mul(v[6], v[14]), silu_mul(v[7], v[15])));
          hfrag[b] = __builtin_bit_cast(bf16x8, pk);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // ---- phase 2: 64 output columns per stage (2 blocks of 32), K = Is (NBLK K steps) from
      // the register-resident h fragments; step i = K step i >> 1 of block i & 1
      const int l = opaque_lane(), fr = l & 31, fh = l >> 5;
      const int r2rd = wrow_dn(fr), f2rd = f2<IS>(r2rd);
      const uint32_t rd_w2_row = (uint32_t)r2rd * C::ROW2;
      auto rd_w2f = [&](uint32_t slot, int step) {
        const uint32_t co = (uint32_t)(((2 * (step >> 1) + fh) ^ f2rd) * 16);
        return *reinterpret_cast<const bf16x8*>(smem + slot + rd_w2_row + (step & 1) * 32 * C::ROW2 + co);
      };
      // Output staging: a lane ends a stage with 16 consecutive columns of ONE slot row per
      // block, and neighbouring lanes hold different rows, 2*d bytes apart; stored like that
      // every lane's 16 bytes are a memory access of their own (measured: 64 accesses per
      // instruction, and the stores alone keep the address unit busy for a quarter of the
      // kernel).  So 16 rows x 32 columns at a time go through 1 KiB of wave-private LDS and are
      // stored with 4 adjacent lanes covering 64 contiguous bytes of a row.
      // Staging rows are 64 bytes (4 chunks of 16); chunk c of row r sits at position
      // c ^ ((r >> 2) & 3), which makes both the 16-lane writes (16 rows, one chunk index) and the
      // linear reads (4 rows x 4 positions) hit all 64 banks once.
      unsigned char* epi = smem + C::OFF_EPI + wv * EPI_WAVE;
      const int er = fr & 15, es = (er >> 2) & 3;
      const uint32_t epi_wr0 = (uint32_t)(er * 64 + ((2 * fh) ^ es) * 16);
      const uint32_t epi_wr1 = (uint32_t)(er * 64 + ((2 * fh + 1) ^ es) * 16);
      const uint32_t epi_rd = (uint32_t)l * 16u;  // row l >> 2 of the 16, position l & 3
      const int srow = wv * 32 + (l >> 2);        // + 16 for the second half of the wave's rows
      const int echunk = (l & 3) ^ ((l >> 4) & 3);  // the chunk that sits at this lane's position
      const uint32_t vo = (uint32_t)srow * (uint32_t)d * 2u + (uint32_t)echunk * 16u;
      const uint32_t vo16 = vo + 16u * (uint32_t)d * 2u;
      uint16_t* ybase = y + (size_t)cur.row0 * d;
      uint32_t xo_next[2] = {xoff[0], xoff[1]};
      bf16x8 wd[PD];
#pragma unroll
      for (int i = 0; i < PD; ++i) wd[i] = rd_w2f(c_w, i);
      for (int s2 = 0; s2 < S2; ++s2) {
        const uint32_t nw = next_w(c_w);
        f32x16 acc2[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc2[b][v] = 0.0f;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
          acc2[i & 1] = mma<MATH>(wd[i % PD], hfrag[i >> 1], acc2[i & 1]);
          wd[i % PD] = i + PD < STEPS ? rd_w2f(c_w, i + PD) : rd_w2f(nw, i + PD - STEPS);
          __builtin_amdgcn_sched_barrier(0);
          if (i == B_STEP) {
            barrier();
            n_allow += produce_x(xo_next);
            n_allow += produce_w();
            if (s2 == 0 && has_next) x_offsets(par ^ 1, xo_next);
            __builtin_amdgcn_sched_barrier(0);
          }
          if (i == WT_STEP) {
            step_d();
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // lane (row fr, half fh) holds columns 64 s2 + 32 b + 16 fh + 0..15 of slot row 32 wv + fr
        static_for<0, 4>([&](auto Q) {
          constexpr int b = decltype(Q)::value >> 1, hf = decltype(Q)::value & 1;
          const f32x16 a = acc2[b];
          if ((fr >> 4) == hf) {
            *reinterpret_cast<uint4*>(epi + epi_wr0) = make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]),
                                                                 pack_bf16x2(a[4], a[5]), pack_bf16x2(a[6], a[7]));
            *reinterpret_cast<uint4*>(epi + epi_wr1) = make_uint4(pack_bf16x2(a[8], a[9]), pack_bf16x2(a[10], a[11]),
                                                                 pack_bf16x2(a[12], a[13]), pack_bf16x2(a[14], a[15]));
          }
          const uint4 q = *reinterpret_cast<const uint4*>(epi + epi_rd);
          if (srow + 16 * hf < cur.rows) store16<b * 64>(ybase, hf ? vo16 : vo, u32x4{q.x, q.y, q.z, q.w});
        });
        // Stores that were certainly issued (a lower bound keeps the wait at (d) safe): row 32 wv
        // of this wave is valid, rows 32 wv + 16.. only if the tile has that many.  They may
        // stay pending through the next iteration's (d).
        n_allow = cur.rows > wv * 32 + 16 ? 4 : 2;
        ybase += 64;
        c_w = nw;
        c_x = next_x(c_x);  // the x ring turns with every stage
      }
    }
    // ---- next tile
    if (!has_next) break;
    cur = nxt;
    par ^= 1;
    has_next = k_after < n_tiles;
    if (has_next) load_hdr(k_after, nxt);
    k_after = n_tiles;
  }
}

template <int IS, bool MATH>
static hipError_t launch_is(const uint16_t* x, const uint16_t* w_gu, const uint16_t* w_dn,
                            const int32_t* sorted_pair, const MTile* tiles, int32_t* hdr,
                            uint16_t* y, int T, int d, int k_max, int max_mtiles, hipStream_t s) {
  static bool done[64] = {};  // per instantiation (IS, MATH)
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
  if (dev < 0 || !done[dev]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_fused_kernel<IS, MATH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg<IS>::LDS_BYTES);
    if (e != hipSuccess) return e;
    if (dev >= 0) done[dev] = true;
  }
  const int grid = persistent_grid(max_mtiles, 1);
  ffn_fused_kernel<IS, MATH><<<grid, NT, Cfg<IS>::LDS_BYTES, s>>>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y,
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

template <bool MATH>
static hipError_t launch_fused(const uint16_t* x, const uint16_t* w_gu, const uint16_t* w_dn,
                               const int32_t* sorted_pair, const MTile* tiles, int32_t* hdr,
                               uint16_t* y, int T, int d, int Is, int k_max, int max_mtiles,
                               hipStream_t s) {
  if (max_mtiles <= 0) return hipSuccess;
  switch (Is) {
    case 64: return fused::launch_is<64, MATH>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y, T, d, k_max, max_mtiles, s);
    case 128: return fused::launch_is<128, MATH>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y, T, d, k_max, max_mtiles, s);
    case 192: return fused::launch_is<192, MATH>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y, T, d, k_max, max_mtiles, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_ffn_fused_bf16(const uint16_t* x, const uint16_t* w_gu, const uint16_t* w_dn,
                                 const int32_t* sorted_pair, const MTile* tiles, int32_t* hdr,
                                 uint16_t* y, int T, int d, int Is, int k_max, int max_mtiles,
                                 hipStream_t s) {
  return launch_fused<true>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y, T, d, Is, k_max, max_mtiles, s);
}

// The kernel's memory operations alone (see mma<false>): what y holds afterwards means nothing.
hipError_t launch_ffn_fused_traffic_bf16(const uint16_t* x, const uint16_t* w_gu,
                                         const uint16_t* w_dn, const int32_t* sorted_pair,
                                         const MTile* tiles, int32_t* hdr, uint16_t* y, int T,
                                         int d, int Is, int k_max, int max_mtiles, hipStream_t s) {
  return launch_fused<false>(x, w_gu, w_dn, sorted_pair, tiles, hdr, y, T, d, Is, k_max, max_mtiles, s);
}

}  // namespace mp
