// bf16 grouped SwiGLU FFN on MFMA (Sec. 3.2.1, Eq. 1-3): the two grouped GEMMs
//   gate-up : h[p, c] = SiLU(x[t_p,:] . Wg[g,c,:]) * (x[t_p,:] . Wu[g,c,:])
//   down    : y[p, q] = sum_c h[p,c] * Wd[g,q,c]
// over ragged groups, as persistent workgroups that walk (m-tile, n-tile) items.
//
// Tile: 256 slot rows x BN weight rows (BN = 256 or 192), 8 wavefronts (4 along the slot
// rows x 2 along the weight rows), one workgroup per CU.  Per K step of 16 a wave multiplies
// 2 slot blocks by BN/64 weight blocks of 32 rows with v_mfma_f32_32x32x16_bf16 (measured at
// twice the rate of the 16x16x32 form on this chip).  The weight block is the MFMA's first
// operand and its rows are fed in a permuted order, so that a lane ends up with 8 or 16
// consecutive output columns of one slot row and stores them as 16-byte words.
// Drivers, all with operand slabs going global -> LDS directly (global_load_lds_dwordx4),
// explicit s_waitcnt vmcnt counts and rings that run across item boundaries:
//   run_items_k64 (K % 64 == 0): stages of 64 K-elements = whole 128-byte cache lines per row
//     and copy, ring of 2 stages, one s_barrier per stage, all waves in one instruction stream
//     with the fragment reads pipelined through the MFMAs;
//   run_items_dma (other K): ring of 4-5 stages of 32 K-elements; for long K the two wave
//     groups alternate between multiplying and preparing the next stage;
//   run_items (K too short for a ring): 64-wide slabs through registers into a double-buffered,
//     XOR-swizzled LDS tile, one slab ahead of the MFMAs.
// Narrow sub-experts (Is in {64, 128, 192}) take the fused kernel in ffn_fused_bf16.hip
// instead; these two kernels serve every other shape.
#include <cstdlib>
#include <type_traits>

#include "ffn_common.h"

namespace mp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = FFN_BM;   // 256 slot rows per tile
constexpr int BK = 64;       // bf16 elements of K per slab: 128 bytes per row
constexpr int NT_ = 512;     // threads per workgroup
constexpr int A_LD = BM * 8 / NT_;  // 16-byte loads per thread and slab for the slot rows (4)

// 16-byte chunk c (0..7) of row r is stored at chunk position c ^ f(r).  A fragment
// read is served 16 lanes at a time (16 rows at one chunk index) from 64 banks: even
// rows fall into one half of the banks, odd rows into the other, so f must differ
// over the 8 rows of equal parity that one such group reads.
//   SWZ_SEQ: the group reads 16 consecutive rows            -> f = (r >> 1) & 7
//   SWZ_SPLIT: it reads rows {0..7, 16..23} or {8..15, 24..31} of a 32-row block
//                                                           -> f = ((r >> 1) & 3) | ((r >> 4) & 1) << 2
constexpr int SWZ_SEQ = 0, SWZ_SPLIT = 1;
template <int MODE>
__device__ __forceinline__ int swz(int r, int c) {
  const int f = MODE == SWZ_SEQ ? ((r >> 1) & 7) : (((r >> 1) & 3) | (((r >> 4) & 1) << 2));
  return r * BK + ((c ^ f) << 3);
}

template <int BN>
struct Tile {
  static constexpr int B_LD = BN * 8 / NT_;       // 16-byte loads per thread and slab (4 or 3)
  static constexpr int NB = BN / 2 / 32;          // 32-row weight blocks per wave (4 or 3)
  static constexpr int A_ELEMS = BM * BK, B_ELEMS = BN * BK;
  static constexpr size_t LDS_BYTES = 2 * (size_t)(A_ELEMS + B_ELEMS) * 2;
};

template <int BN, int WSWZ>
struct Pipe {
  using TL = Tile<BN>;
  uint16_t* smem_;  // [2][A_ELEMS] slot-row slabs, then [2][B_ELEMS] weight-row slabs
  uint4 ra[A_LD], rb[TL::B_LD];
  int lc, lr;  // this thread copies chunk lc of rows lr + 64*i

  __device__ __forceinline__ void init(uint16_t* smem) {
    smem_ = smem;
    lc = threadIdx.x & 7;
    lr = threadIdx.x >> 3;
  }
  // global -> registers: slab starting at element k0 of the item's rows; K is the row
  // length.  Row addresses are recomputed from the item (a few integer operations per load)
  // instead of being kept in registers, which the accumulators need.
  template <class Op, class Item>
  __device__ __forceinline__ void gload(const Op& op, const Item& it, int k0, int K) {
    const int k = k0 + lc * 8;
    const bool in = k < K;  // K tail (K % 64 != 0) is zero-filled
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      ra[i] = in ? *reinterpret_cast<const uint4*>(op.a_row(it, lr + 64 * i, i) + k)
                 : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < TL::B_LD; ++i)
      rb[i] = in ? *reinterpret_cast<const uint4*>(op.b_row(it, lr + 64 * i) + k)
                 : make_uint4(0, 0, 0, 0);
  }
  __device__ __forceinline__ uint16_t* sa(int buf) const { return smem_ + buf * TL::A_ELEMS; }
  __device__ __forceinline__ uint16_t* sb(int buf) const {
    return smem_ + 2 * TL::A_ELEMS + buf * TL::B_ELEMS;
  }
  // registers -> LDS buffer `buf`
  __device__ __forceinline__ void sstore(int buf) {
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      *reinterpret_cast<uint4*>(sa(buf) + swz<SWZ_SEQ>(lr + 64 * i, lc)) = ra[i];
#pragma unroll
    for (int i = 0; i < TL::B_LD; ++i)
      *reinterpret_cast<uint4*>(sb(buf) + swz<WSWZ>(lr + 64 * i, lc)) = rb[i];
  }
  // one slab of MFMAs from LDS buffer `buf`.  mb_on = number of this wave's 32-row slot
  // blocks that hold at least one valid row (the others are skipped); wrow = the row of a
  // 32-row weight block this lane feeds to the MFMA (Op::wrow of lane & 31).
  __device__ __forceinline__ void compute(int buf, f32x16 (&acc)[TL::NB][2], int mb_on, int wrow) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const uint16_t* pa = sa(buf);
    const uint16_t* pb = sb(buf);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int c = ks * 2 + (lane >> 5);
      bf16x8 ft[2], fw[TL::NB];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        ft[mb] = *reinterpret_cast<const bf16x8*>(pa + swz<SWZ_SEQ>(wm * 64 + mb * 32 + (lane & 31), c));
#pragma unroll
      for (int nb = 0; nb < TL::NB; ++nb)
        fw[nb] = *reinterpret_cast<const bf16x8*>(pb + swz<WSWZ>(wn * (BN / 2) + nb * 32 + wrow, c));
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        if (mb < mb_on) {
#pragma unroll
          for (int nb = 0; nb < TL::NB; ++nb)
            acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[nb], ft[mb], acc[nb][mb], 0, 0, 0);
        }
      }
    }
  }
};

__device__ __forceinline__ float silu_mul(float a, float u) {
  return __fdividef(a, 1.0f + __expf(-a)) * u;
}
__device__ __forceinline__ uint32_t pack2(float a, float b) { return pack_bf16x2(a, b); }

// What every lane knows about a work item: group, first slot row, valid rows, first
// output column (or neuron) of the n-tile.  Wave-uniform.
struct Sc {
  int g, row0, rows, n0;
};

// Generic persistent driver.  Op supplies the per-item state (Item), the row addresses
// (a_row: slot rows, b_row: weight rows) and the epilogue.
template <int BN, class Op>
__device__ __forceinline__ void run_items(const Op& op, const MTile* __restrict__ tiles,
                                          const int32_t* __restrict__ hdr, int K, int n_tiles_n) {
  using TL = Tile<BN>;
  using Item = typename Op::Item;
  extern __shared__ __align__(16) uint16_t smem[];
  Pipe<BN, Op::WSWZ> pipe;
  pipe.init(smem);
  const int wv = threadIdx.x >> 6, wm = wv >> 1;
  const int wrow = Op::wrow(threadIdx.x & 31);
  const int total = hdr[HDR_MTILES] * n_tiles_n;
  const ItemRange ir = xcd_items(total);
  if (ir.begin >= ir.end) return;  // uniform over the workgroup
  const int nslab = (K + BK - 1) / BK;

  int item = ir.begin;
  Item cur, nxt;
  op.setup(tiles[item / n_tiles_n], item % n_tiles_n, pipe.lr, cur);
  nxt = cur;

  pipe.gload(op, cur, 0, K);
  pipe.sstore(0);
  __syncthreads();
  int buf = 0;
  for (;;) {
    const bool has_next = item + ir.step < ir.end;
    if (has_next) {
      const int ni = item + ir.step;
      op.setup(tiles[ni / n_tiles_n], ni % n_tiles_n, pipe.lr, nxt);
    }
    int mb_on = (cur.rows - wm * 64 + 31) / 32;
    mb_on = mb_on < 0 ? 0 : (mb_on > 2 ? 2 : mb_on);
    mb_on = __builtin_amdgcn_readfirstlane(mb_on);  // wave-uniform: keep the skips scalar
    f32x16 acc[TL::NB][2];
#pragma unroll
    for (int nb = 0; nb < TL::NB; ++nb)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.0f;

    for (int s = 0; s < nslab; ++s) {
      const bool last = s == nslab - 1;
      if (!last)
        pipe.gload(op, cur, (s + 1) * BK, K);
      else if (has_next)
        pipe.gload(op, nxt, 0, K);
      pipe.compute(buf, acc, mb_on, wrow);
      if (last) op.epilogue(cur, acc, mb_on, nullptr);
      if (!last || has_next) pipe.sstore(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }
    if (!has_next) break;
    item += ir.step;
    cur = nxt;
  }
}

// Tile header fields are the same for every lane: keep them in scalar registers.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// ---------------------------------------------------------------- gate-up
// A tile holds BN/2 neurons.  Each 32-row weight block is 16 neurons: rows 0..15 are their
// gate rows, rows 16..31 their up rows, so a lane's accumulators v and v + 8 are the gate
// and up value of one neuron.  MFMA row i = 8a + 4hi + b reads block row 16*(a >> 1) +
// 8hi + 4(a & 1) + b, which makes accumulators 0..7 of a lane the 8 consecutive neurons
// 8hi .. 8hi + 7.
template <int BN>
struct GateUpOp {
  static constexpr int WSWZ = SWZ_SEQ;
  const uint16_t* x;
  const uint16_t* w_gu;
  const int32_t* sorted_pair;
  uint16_t* h;
  int T, d, Is, k_max;

  static constexpr bool GATHER = true;
  struct Item : Sc {
    int tok[A_LD];  // tokens of the slot rows this thread copies
  };

  static __device__ __forceinline__ int wrow(int i) {
    const int a = i >> 3, hi = (i >> 2) & 1, b = i & 3;
    return 16 * (a >> 1) + 8 * hi + 4 * (a & 1) + b;
  }
  __device__ __forceinline__ void setup(const MTile& t, int nt, int lr, Item& it) const {
    it.g = uni(t.g);
    it.row0 = uni(t.row0);
    it.rows = uni(t.rows);
    it.n0 = uni(nt) * (BN / 2);
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
      int row = min(lr + 64 * i, it.rows - 1);
      int tok = sorted_pair[it.row0 + row] / k_max;
      it.tok[i] = min(max(tok, 0), T - 1);
    }
  }
  __device__ __forceinline__ const uint16_t* a_row(const Item& it, int, int i) const {
    return x + (size_t)it.tok[i] * d;
  }
  // DMA driver: header only; the slot list entries of the tile's rows arrive through LDS
  __device__ __forceinline__ void setup_sc(const MTile& t, int nt, Sc& sc) const {
    sc.g = uni(t.g);
    sc.row0 = uni(t.row0);
    sc.rows = uni(t.rows);
    sc.n0 = uni(nt) * (BN / 2);
  }
  __device__ __forceinline__ const int32_t* idx_src(const Sc& sc, int r) const {
    return sorted_pair + sc.row0 + min(r, sc.rows - 1);
  }
  // store instructions a wave's epilogue issues (one per row block and weight block), if
  // that is known exactly: every block of the wave inside the n-range; else 0
  static constexpr int STORES_PER_MB = Tile<BN>::NB;
  __device__ __forceinline__ int stores_issued(const Sc& sc, int mb_on, int, int wn) const {
    const bool all = sc.n0 + wn * (BN / 4) + (Tile<BN>::NB - 1) * 16 < Is;
    return all ? mb_on * STORES_PER_MB : 0;
  }
  __device__ __forceinline__ const uint16_t* a_src(const Sc&, int r, const int32_t* pair_lds) const {
    const int tok = pair_lds[r] / k_max;
    return x + (size_t)min(max(tok, 0), T - 1) * d;
  }
  // the same rows as a wave-uniform base plus a 32-bit byte offset per row (K = 64 driver)
  __device__ __forceinline__ void bases(const Sc& sc, const uint16_t*& ba, const uint16_t*& bb) const {
    ba = x;
    bb = w_gu + (size_t)sc.g * 2 * Is * d;
  }
  __device__ __forceinline__ uint32_t a_off(const Sc&, int r, const int32_t* pair_lds) const {
    const int tok = pair_lds[r] / k_max;
    return (uint32_t)min(max(tok, 0), T - 1) * (uint32_t)d * 2u;
  }
  __device__ __forceinline__ uint32_t b_off(const Sc& it, int br) const {
    const int blk = br >> 5, rr = br & 31;
    const int neuron = min(it.n0 + blk * 16 + (rr & 15), Is - 1);
    return (uint32_t)((rr >> 4) ? Is + neuron : neuron) * (uint32_t)d * 2u;
  }
  static bool offsets_fit(long T, long d, long Is) {
    return T * d * 2 < (1L << 32) && 2 * Is * d * 2 < (1L << 32);
  }
  __device__ __forceinline__ const uint16_t* b_row(const Sc& it, int br) const {
    const int blk = br >> 5, rr = br & 31;  // 32-row block of the tile, row inside it
    const int neuron = min(it.n0 + blk * 16 + (rr & 15), Is - 1);
    return w_gu + ((size_t)it.g * 2 * Is + ((rr >> 4) ? Is + neuron : neuron)) * d;
  }
  __device__ __forceinline__ void epilogue(const Sc& it, f32x16 (&acc)[Tile<BN>::NB][2],
                                           int mb_on, uint16_t*) const {
    constexpr int NB = Tile<BN>::NB;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int n0 = it.n0 + wn * (BN / 4) + 8 * (lane >> 5);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      if (mb >= mb_on) continue;
      const int row = wm * 64 + mb * 32 + (lane & 31);
      if (row >= it.rows) continue;
      uint16_t* hrow = h + (size_t)(it.row0 + row) * Is;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int col = n0 + nb * 16;
        if (col < Is) {  // Is % 32 == 0 and col % 8 == 0: all 8 neurons are inside
          const f32x16 v = acc[nb][mb];
          *reinterpret_cast<uint4*>(hrow + col) = make_uint4(
              pack2(silu_mul(v[0], v[8]), silu_mul(v[1], v[9])),
              pack2(silu_mul(v[2], v[10]), silu_mul(v[3], v[11])),
              pack2(silu_mul(v[4], v[12]), silu_mul(v[5], v[13])),
              pack2(silu_mul(v[6], v[14]), silu_mul(v[7], v[15])));
        }
      }
    }
  }
};

template <int BN>
__global__ __launch_bounds__(NT_) void gate_up_bf16_kernel(GateUpOp<BN> op,
                                                           const MTile* __restrict__ tiles,
                                                           const int32_t* __restrict__ hdr,
                                                           int n_tiles_n) {
  run_items<BN>(op, tiles, hdr, op.d, n_tiles_n);
}

// ---------------------------------------------------------------- down
// A 32-row weight block is 32 consecutive output columns.  MFMA row i = 8a + 4hi + b reads
// block row 16hi + 4a + b, so a lane's 16 accumulators are the consecutive columns
// 16hi .. 16hi + 15.
template <int BN>
struct DownOp {
  static constexpr int WSWZ = SWZ_SPLIT;
  const uint16_t* h;
  const uint16_t* w_dn;
  uint16_t* y;
  int d, Is;

  static constexpr bool GATHER = false;
  typedef Sc Item;

  static __device__ __forceinline__ int wrow(int i) {
    const int a = i >> 3, hi = (i >> 2) & 1, b = i & 3;
    return 16 * hi + 4 * a + b;
  }
  __device__ __forceinline__ void setup(const MTile& t, int nt, int, Item& it) const {
    it.g = uni(t.g);
    it.row0 = uni(t.row0);
    it.rows = uni(t.rows);
    it.n0 = uni(nt) * BN;
  }
  __device__ __forceinline__ const uint16_t* a_row(const Item& it, int r, int) const {
    return h + (size_t)(it.row0 + min(r, it.rows - 1)) * Is;
  }
  __device__ __forceinline__ void setup_sc(const MTile& t, int nt, Sc& sc) const {
    sc.g = uni(t.g);
    sc.row0 = uni(t.row0);
    sc.rows = uni(t.rows);
    sc.n0 = uni(nt) * BN;
  }
  __device__ __forceinline__ const int32_t* idx_src(const Sc&, int) const { return nullptr; }
  static constexpr int STORES_PER_MB = 2 * Tile<BN>::NB;
  // a lower bound that is one of 0, STORES_PER_MB, 2 * STORES_PER_MB
  __device__ __forceinline__ int stores_issued(const Sc& sc, int mb_on, int wm, int wn) const {
    const bool all = sc.n0 + wn * (BN / 2) + (Tile<BN>::NB - 1) * 32 < d;
    if (!all) return 0;
    // the coalescing epilogue stores 8 rows per instruction: only full 32-row blocks count
    const int full_blocks = min(max((sc.rows - wm * 64) / 32, 0), 2);
    return (BN == 256 ? full_blocks : mb_on) * STORES_PER_MB;
  }
  __device__ __forceinline__ const uint16_t* a_src(const Sc& sc, int r, const int32_t*) const {
    return h + (size_t)(sc.row0 + min(r, sc.rows - 1)) * Is;
  }
  __device__ __forceinline__ void bases(const Sc& sc, const uint16_t*& ba, const uint16_t*& bb) const {
    ba = h + (size_t)sc.row0 * Is;
    bb = w_dn + (size_t)sc.g * d * Is;
  }
  __device__ __forceinline__ uint32_t a_off(const Sc& sc, int r, const int32_t*) const {
    return (uint32_t)min(r, sc.rows - 1) * (uint32_t)Is * 2u;
  }
  __device__ __forceinline__ uint32_t b_off(const Sc& it, int br) const {
    return (uint32_t)min(it.n0 + br, d - 1) * (uint32_t)Is * 2u;
  }
  static bool offsets_fit(long, long d, long Is) { return d * Is * 2 < (1L << 32); }
  __device__ __forceinline__ const uint16_t* b_row(const Sc& it, int br) const {
    return w_dn + ((size_t)it.g * d + min(it.n0 + br, d - 1)) * Is;
  }
  // Direct form: a lane stores its 16 consecutive columns of one row (two 16-byte stores).
  __device__ __forceinline__ void epilogue_direct(const Sc& it, f32x16 (&acc)[Tile<BN>::NB][2],
                                                  int mb_on) const {
    constexpr int NB = Tile<BN>::NB;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int n0 = it.n0 + wn * (BN / 2) + 16 * (lane >> 5);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      if (mb >= mb_on) continue;
      const int row = wm * 64 + mb * 32 + (lane & 31);
      if (row >= it.rows) continue;
      uint16_t* yrow = y + (size_t)(it.row0 + row) * d;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int col = n0 + nb * 32;
        if (col < d) {  // d % 64 == 0 and col % 16 == 0: all 16 columns are inside
          const f32x16 v = acc[nb][mb];
          *reinterpret_cast<uint4*>(yrow + col) = make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]),
                                                             pack2(v[4], v[5]), pack2(v[6], v[7]));
          *reinterpret_cast<uint4*>(yrow + col + 8) = make_uint4(
              pack2(v[8], v[9]), pack2(v[10], v[11]), pack2(v[12], v[13]), pack2(v[14], v[15]));
        }
      }
    }
  }
  // Coalescing form (BN = 256, wave-private 4 KiB of LDS): 32 rows x 64 columns at a time are
  // written to LDS in the accumulator layout and read back row-major, so that every store
  // instruction writes 8 rows x 128 contiguous bytes (whole cache lines) instead of 64
  // scattered 16-byte pieces.  y is the layer's largest HBM stream.  LDS rows are 128 bytes,
  // 16-byte chunk c of row r sits at position c ^ ((r >> 1) & 7): conflict-free both ways.
  __device__ __forceinline__ void epilogue(const Sc& it, f32x16 (&acc)[Tile<BN>::NB][2], int mb_on,
                                           uint16_t* scratch) const {
    constexpr int NB = Tile<BN>::NB;
    if (BN != 256 || scratch == nullptr) {
      epilogue_direct(it, acc, mb_on);
      return;
    }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int r = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      if (mb >= mb_on) continue;
      const int valid = it.rows - (wm * 64 + mb * 32);  // rows of this block inside the tile
#pragma unroll
      for (int half = 0; half < NB / 2; ++half) {
        const int col0 = it.n0 + wn * (BN / 2) + half * 64;
        if (col0 >= d) continue;  // d % 64 == 0: a half is inside or outside as a whole
#pragma unroll
        for (int nbl = 0; nbl < 2; ++nbl) {
          const f32x16 v = acc[half * 2 + nbl][mb];
          const int c = nbl * 4 + 2 * hi, sw = (r >> 1) & 7;
          *reinterpret_cast<uint4*>(scratch + r * 64 + (((c) ^ sw) << 3)) =
              make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
          *reinterpret_cast<uint4*>(scratch + r * 64 + (((c + 1) ^ sw) << 3)) = make_uint4(
              pack2(v[8], v[9]), pack2(v[10], v[11]), pack2(v[12], v[13]), pack2(v[14], v[15]));
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int row = j * 8 + (lane >> 3), c = lane & 7;
          const uint4 q = *reinterpret_cast<const uint4*>(scratch + row * 64 + ((c ^ ((row >> 1) & 7)) << 3));
          if (row < valid)
            *reinterpret_cast<uint4*>(y + (size_t)(it.row0 + wm * 64 + mb * 32 + row) * d + col0 + c * 8) = q;
        }
      }
    }
  }
};

template <int BN>
__global__ __launch_bounds__(NT_) void down_bf16_kernel(DownOp<BN> op,
                                                        const MTile* __restrict__ tiles,
                                                        const int32_t* __restrict__ hdr,
                                                        int n_tiles_n) {
  run_items<BN>(op, tiles, hdr, op.Is, n_tiles_n);
}

// ---------------------------------------------------------------- DMA ring driver
// Same tiles and MFMA schedule, but the operand slabs travel global -> LDS directly
// (global_load_lds_dwordx4: lane i of a wave deposits its 16 bytes at LDS base + 16 i),
// through a ring of NS stages of 32 K-elements each, NS - 1 stages ahead of the MFMAs.
// Nothing passes through registers, so several stages can be in flight; the waits are
// explicit (s_waitcnt vmcnt counts this wave's outstanding copies, oldest first) and one
// s_barrier per stage both publishes the stage that landed and frees the one just used.
// The ring runs across item boundaries.  For the gate-up GEMM the slot list entries of the
// next tile (which tokens to gather) are copied into LDS the same way, one item ahead.
constexpr int SK = 32;  // K elements per stage: 64 bytes per row, 4 chunks of 16 bytes
constexpr int DYN_DIV = 8;  // 1/DYN_DIV of the work items go to the shared pool

// chunk c (0..3) of row r sits at position c ^ g(r); 16 lanes read 16 rows at one chunk
// index, rows of equal r & 3 share banks, so g must differ over them (see swz above)
template <int MODE>
__device__ __forceinline__ int swz32(int r, int c) {
  const int g = MODE == SWZ_SEQ ? ((r >> 2) & 3) : (((r >> 2) & 1) | (((r >> 4) & 1) << 1));
  return r * SK + ((c ^ g) << 3);
}
template <int MODE>
__device__ __forceinline__ int chunk_of(int r, int pos) {  // inverse: which chunk sits at pos
  const int g = MODE == SWZ_SEQ ? ((r >> 2) & 3) : (((r >> 2) & 1) | (((r >> 4) & 1) << 1));
  return pos ^ g;
}

// LDS plan: NS ring stages, then the slot-list entries of two tiles (gate-up only), then
// 4 KiB per wave of scratch for the coalescing epilogue (down only).
constexpr int EPI_WAVE_BYTES = 4096;
template <int BN, bool GATHER>
struct Ring {
  static constexpr int NS = (BN == 192 && GATHER) ? 5 : 4;  // stages in LDS
  static constexpr int D = NS - 1;              // stages in flight ahead of the MFMAs
  static constexpr int NB = BN / 2 / 32;
  static constexpr int A_ST = BM * SK, B_ST = BN * SK, STAGE = A_ST + B_ST;  // elements
  static constexpr size_t RING_BYTES = (size_t)NS * STAGE * 2;
  static constexpr size_t PAIR_BYTES = GATHER ? 2 * BM * sizeof(int32_t) : 0;
  static constexpr size_t EPI_BYTES = GATHER ? 0 : (NT_ / 64) * EPI_WAVE_BYTES;
  static constexpr size_t LDS_BYTES = RING_BYTES + PAIR_BYTES + EPI_BYTES;
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per CU");
  // 16-row copy instructions per wave and stage for the weight rows
  static __device__ __forceinline__ int nb_dma(int wv) { return BN == 256 ? 2 : (wv < 4 ? 2 : 1); }
  static __device__ __forceinline__ int b_block(int wv, int j) {
    return BN == 256 ? 2 * wv + j : (wv < 4 ? 2 * wv + j : 8 + (wv - 4));
  }
};

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// one wave-wide copy: every lane fetches 16 (4) bytes at g; lane i's data lands at lds + 16 i (4 i)
// m0 carries the LDS address of the copy.  The compiler reserves m0 and does not accept it in
// a clobber list, so the value it may be keeping there is saved and put back.
__device__ __forceinline__ void dma16(const void* g, uint32_t lds) {
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 1\n\tglobal_load_lds_dwordx4 %1, off\n\t"
               "s_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(g), "s"(lds)
               : "memory");
}
__device__ __forceinline__ void dma4(const void* g, uint32_t lds) {
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 1\n\tglobal_load_lds_dword %1, off\n\t"
               "s_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(g), "s"(lds)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_copies() {  // until at most N of this wave's copies are pending
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// wait until at most BASE + extra operations are pending; extra is 0, PER_MB or 2 * PER_MB
template <int BASE, int PER_MB>
__device__ __forceinline__ void wait_steady(int extra) {
  if (extra == 2 * PER_MB)
    wait_copies<BASE + 2 * PER_MB>();
  else if (extra == PER_MB)
    wait_copies<BASE + PER_MB>();
  else
    wait_copies<BASE>();
}

template <int BN, class Op, bool PP>
__device__ __forceinline__ void run_items_dma(const Op& op, const MTile* __restrict__ tiles,
                                              int32_t* __restrict__ hdr, int K, int n_tiles_n,
                                              int dyn_word) {
  using RG = Ring<BN, Op::GATHER>;
  constexpr int NS = RG::NS, D = RG::D, NB = RG::NB;
  extern __shared__ __align__(16) uint16_t smem[];
  int32_t* pair_lds = reinterpret_cast<int32_t*>(smem + (size_t)NS * RG::STAGE);  // [2][BM]
  const int lane = threadIdx.x & 63, wv = uni(threadIdx.x >> 6);
  uint16_t* epi_lds = RG::EPI_BYTES ? smem + (RG::RING_BYTES + RG::PAIR_BYTES) / 2 + (size_t)wv * (EPI_WAVE_BYTES / 2) : nullptr;
  const int wm = wv >> 1, wn = wv & 1;
  const int wrow = Op::wrow(lane & 31);
  // Work split: the first 1 - 1/DYN_DIV of the item list is dealt out statically (XCD-aware,
  // see xcd_items), the rest is a pool that workgroups draw from in batches once their own
  // share is done, which evens out the finishing times (m-tiles differ in their row counts).
  // The draw is an atomic with a returned value, so it sits between two pipeline runs, where
  // no copy is in flight that the wait for the returned value could serialise.  The drawn index
  // reaches the other waves through the first word of the (then idle) ring.
  int32_t* dyn_next = reinterpret_cast<int32_t*>(smem);
  const int total_items = hdr[HDR_MTILES] * n_tiles_n;
  const int n_static = total_items - total_items / DYN_DIV;
  const int nst = K / SK;  // K % 32 == 0 for every supported shape
  const int batch = nst >= 24 ? 1 : (24 + nst - 1) / nst;
  ItemRange ir = xcd_items(n_static);
  int n_my = ir.begin < ir.end ? (ir.end - ir.begin + ir.step - 1) / ir.step : 0;
  const uint32_t smem_base = lds_addr(smem);
  const uint32_t pair_base = lds_addr(pair_lds);

  // rows this lane copies: 16-row block `blk` of the tile, row blk*16 + lane/4, position lane%4
  const int sub = lane >> 2, pos = lane & 3;
  const int nbd = RG::nb_dma(wv);

  Sc cur, nxt;
  // Item -> (m-tile, n-tile).  A group's items are contiguous; inside a group they are walked
  // in chunks of C n-tiles x all of the group's m-tiles, so that the ~32 items an XCD works on
  // at a time form a block a x b of m-tiles x n-tiles with a + b small: each activation tile
  // is then fetched once for b n-tiles and each weight tile once for a m-tiles.
  auto load_sc = [&](int my_idx, Sc& sc) {
    const int item = ir.begin + my_idx * ir.step;
    const MTile t0 = tiles[item / n_tiles_n];
    const int first = uni(t0.first), cnt = uni(t0.count);
    const int L = item - first * n_tiles_n;
    int C = 32 / (cnt < 6 ? cnt : 6);
    C = C > n_tiles_n ? n_tiles_n : C;
    const int per = cnt * C;
    const int c = L / per, r = L % per;
    const int Cc = min(C, n_tiles_n - c * C);
    op.setup_sc(tiles[first + r / Cc], c * C + r % Cc, sc);
  };
  // copy the slot-list entries of an item's rows into pair_lds[parity] (waves 0..3, 64 rows each)
  auto fetch_pairs = [&](const Sc& sc, int parity) {
    if (Op::GATHER && wv < 4)
      dma4(op.idx_src(sc, wv * 64 + lane), pair_base + (uint32_t)(parity * BM + wv * 64) * 4);
  };
  const uint16_t* pa[2];
  const uint16_t* pb[2];
  auto producer_rows = [&](const Sc& sc, int parity) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int r = wv * 32 + j * 16 + sub;
      pa[j] = op.a_src(sc, r, pair_lds + parity * BM) + chunk_of<SWZ_SEQ>(r, pos) * 8;
      const int br = RG::b_block(wv, j) * 16 + sub;
      pb[j] = op.b_row(sc, br) + chunk_of<Op::WSWZ>(br, pos) * 8;
    }
  };
  auto issue_stage = [&](int slot, int k0) {
    const uint32_t sa = smem_base + (uint32_t)slot * (RG::STAGE * 2);
    const uint32_t sb = sa + RG::A_ST * 2;
#pragma unroll
    for (int j = 0; j < 2; ++j) dma16(pa[j] + k0, sa + (uint32_t)(wv * 32 + j * 16) * (SK * 2));
    dma16(pb[0] + k0, sb + (uint32_t)(RG::b_block(wv, 0) * 16) * (SK * 2));
    if (nbd == 2) dma16(pb[1] + k0, sb + (uint32_t)(RG::b_block(wv, 1) * 16) * (SK * 2));
  };

  // fragments of one K step of 16 from ring slot `slot`
  struct Frag {
    bf16x8 t[2], w[NB];
  };
  auto read_frags = [&](int slot, int ks, Frag& f) {
    const uint16_t* sa = smem + (size_t)slot * RG::STAGE;
    const uint16_t* sb = sa + RG::A_ST;
    const int c = ks * 2 + (lane >> 5);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
      f.t[mb] = *reinterpret_cast<const bf16x8*>(sa + swz32<SWZ_SEQ>(wm * 64 + mb * 32 + (lane & 31), c));
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      f.w[nb] = *reinterpret_cast<const bf16x8*>(sb + swz32<Op::WSWZ>(wn * (BN / 2) + nb * 32 + wrow, c));
  };

  for (;;) {
  if (n_my > 0) {
    const int total = n_my * nst;
    // ---- prologue of one pipeline run over n_my items
    load_sc(0, cur);
    nxt = cur;
    if (n_my > 1) load_sc(1, nxt);
    fetch_pairs(cur, 0);
    wait_copies<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");  // LDS reads below must stay below the barrier
    producer_rows(cur, 0);
    if (n_my > 1) fetch_pairs(nxt, 1);
    // producer: global stage, stage in item, item, ring slot.  It runs NS - 1 stages ahead of
    // the MFMAs: stage q is being multiplied, stage q + 1 has landed (its first fragments are
    // read early), stages q + 2 .. q + NS - 1 are in flight.
    int p = 0, p_stage = 0, p_item = 0, p_slot = 0;
    for (; p < NS - 1 && p < total; ++p) {  // nst >= NS: all inside the first item
      issue_stage(p_slot, p_stage * SK);
      ++p_stage;
      p_slot = p_slot + 1 == NS ? 0 : p_slot + 1;
    }
    if (nbd == 2) wait_copies<(NS - 2) * 4>(); else wait_copies<(NS - 2) * 3>();  // stage 0 landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    f32x16 acc[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.0f;
    int mb_on = (cur.rows - wm * 64 + 31) / 32;
    mb_on = uni(mb_on < 0 ? 0 : (mb_on > 2 ? 2 : mb_on));

    if constexpr (PP) {
      // ---- main loop.  The two wave groups (waves 0-3 and 4-7: one wave of each per SIMD) run
      // the same sequence, group 1 one phase behind group 0: while one wave of a SIMD issues the
      // MFMAs of a stage, the other does everything else (the previous tile's epilogue, waiting
      // for copies, reading fragments, issuing copies), so the matrix pipe is not left idle
      // during that work.  Phases are separated by workgroup barriers; to shift group 1 it takes
      // one extra barrier before the loop and group 0 one after it.
      //   prepare(q): wait for this wave's copies of stage q + 1 (every wave did the same for
      //               stage q one or two phases ago, with a barrier since: stage q is complete;
      //               waiting before issuing more copies also measured faster than after);
      //               read this wave's fragments of stage q into registers; issue this wave's
      //               copies of stage q + NS - 1 into the slot of stage q - 1, which both groups
      //               have finished reading (reads are complete before a wave's barrier).
      //   multiply(q): the MFMAs of stage q from registers.
      Frag f0, f1;  // the two K halves of one stage
      int c_stage = 0, c_item = 0, c_slot = 0;
      int st_credit = 0, st_count = 0;  // iterations left in which st_count stores may be pending
      bool item_done = false;
      auto finish_item = [&]() {
        op.epilogue(cur, acc, mb_on, epi_lds);
        st_count = uni(op.stores_issued(cur, mb_on, wm, wn));
        st_credit = NS - 2;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.0f;
        ++c_item;
        cur = nxt;
        mb_on = (cur.rows - wm * 64 + 31) / 32;
        mb_on = uni(mb_on < 0 ? 0 : (mb_on > 2 ? 2 : mb_on));
        if (c_item + 1 < n_my) {
          load_sc(c_item + 1, nxt);
          fetch_pairs(nxt, (c_item + 1) & 1);
        }
        item_done = false;
      };
      const int grp = wv >> 2;
      if (grp == 1) {
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
      for (int q = 0; q < total; ++q) {
        // ---- prepare(q)
        if (item_done) finish_item();
        // Stage q + 1 has landed once at most the operations issued after it are pending: the
        // copies of the NS - 3 younger stages and, for NS - 2 iterations after an epilogue, that
        // epilogue's stores (vector memory operations retire in issue order, loads and stores
        // alike; counting the stores keeps the ring from draining behind every output tile).
        if (q + 1 < total) {
          if (p - q - 2 >= NS - 3) {
            const int extra = st_credit > 0 ? st_count : 0;
            if (nbd == 2) wait_steady<(NS - 3) * 4, Op::STORES_PER_MB>(extra);
            else wait_steady<(NS - 3) * 3, Op::STORES_PER_MB>(extra);
          } else {
            wait_copies<0>();
          }
        }
        st_credit = st_credit > 0 ? st_credit - 1 : 0;
        read_frags(c_slot, 0, f0);
        read_frags(c_slot, 1, f1);
        if (p < total) {
          if (p_stage == nst) {  // the producer enters the next item
            p_stage = 0;
            ++p_item;
            producer_rows(nxt, p_item & 1);
          }
          issue_stage(p_slot, p_stage * SK);
          ++p;
          ++p_stage;
          p_slot = p_slot + 1 == NS ? 0 : p_slot + 1;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // fragments are in registers
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // ---- multiply(q).  A wave whose 64 slot rows are all beyond the tile's rows skips the
        // MFMAs (the tile takes as long as its fullest wave, so finer skipping would buy nothing).
        if (mb_on > 0) {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
              acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.w[nb], f0.t[mb], acc[nb][mb], 0, 0, 0);
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
              acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.w[nb], f1.t[mb], acc[nb][mb], 0, 0, 0);
        }
        c_slot = c_slot + 1 == NS ? 0 : c_slot + 1;
        if (++c_stage == nst) {  // the item is complete; its epilogue runs in the next prepare phase
          c_stage = 0;
          item_done = true;
        }
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
      if (item_done) finish_item();
      if (grp == 0) {
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
    } else {
      // ---- main loop, all waves in step (short K: the epilogues dominate and are better run
      // by all waves at once).  One barrier per stage publishes stage q + 1 and frees the
      // slot of stage q - 1; the first fragments of stage q + 1 are read between the MFMAs.
      Frag f0, f1;
      read_frags(0, 0, f0);
      int c_stage = 0, c_item = 0, c_slot = 0;
      int st_credit = 0, st_count = 0;  // iterations left in which st_count stores may be pending
      for (int q = 0; q < total; ++q) {
        const int n_slot = c_slot + 1 == NS ? 0 : c_slot + 1;
        // Stage q + 1 has landed once at most the operations issued after it are pending: the
        // copies of the NS - 3 younger stages and, for NS - 2 iterations after an epilogue, that
        // epilogue's stores (vector memory operations retire in issue order, loads and stores
        // alike; counting the stores keeps the ring from draining behind every output tile).
        if (p - q - 2 >= NS - 3) {
          const int extra = st_credit > 0 ? st_count : 0;
          if (nbd == 2) wait_steady<(NS - 3) * 4, Op::STORES_PER_MB>(extra);
          else wait_steady<(NS - 3) * 3, Op::STORES_PER_MB>(extra);
        } else {
          wait_copies<0>();
        }
        st_credit = st_credit > 0 ? st_credit - 1 : 0;
        __builtin_amdgcn_s_barrier();  // publishes stage q + 1, frees the slot of stage q - 1
        asm volatile("" ::: "memory");
        if (p < total) {
          if (p_stage == nst) {  // the producer enters the next item
            p_stage = 0;
            ++p_item;
            producer_rows(nxt, p_item & 1);
          }
          issue_stage(p_slot, p_stage * SK);
          ++p;
          ++p_stage;
          p_slot = p_slot + 1 == NS ? 0 : p_slot + 1;
        }
        // ---- MFMAs of stage q; the first fragments of stage q + 1 are fetched in between.
        // A wave whose 64 slot rows are all beyond the tile's rows skips the MFMAs (the tile
        // takes as long as its fullest wave, so finer skipping would buy nothing).
        read_frags(c_slot, 1, f1);
        if (mb_on > 0) {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
              acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.w[nb], f0.t[mb], acc[nb][mb], 0, 0, 0);
        }
        if (q + 1 < total) read_frags(n_slot, 0, f0);
        if (mb_on > 0) {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
              acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.w[nb], f1.t[mb], acc[nb][mb], 0, 0, 0);
        }
        c_slot = n_slot;
        if (++c_stage == nst) {  // the item is complete
          op.epilogue(cur, acc, mb_on, epi_lds);
          st_count = uni(op.stores_issued(cur, mb_on, wm, wn));
          st_credit = NS - 2;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
              for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.0f;
          c_stage = 0;
          ++c_item;
          cur = nxt;
          mb_on = (cur.rows - wm * 64 + 31) / 32;
          mb_on = uni(mb_on < 0 ? 0 : (mb_on > 2 ? 2 : mb_on));
          if (c_item + 1 < n_my) {
            load_sc(c_item + 1, nxt);
            fetch_pairs(nxt, (c_item + 1) & 1);
          }
        }
      }
    }
  }
    // ---- next batch from the pool (every copy of this run has landed, every wave is here)
    __syncthreads();
    if (threadIdx.x == 0) *dyn_next = atomicAdd(&hdr[dyn_word], batch);
    __syncthreads();
    ir.begin = n_static + uni(*dyn_next);  // read before this wave reaches the next run's first barrier
    if (ir.begin >= total_items) break;
    ir.end = min(total_items, ir.begin + batch);
    ir.step = 1;
    n_my = ir.end - ir.begin;
  }
}

template <int BN, bool PP>
__global__ __launch_bounds__(NT_) void gate_up_bf16_dma_kernel(GateUpOp<BN> op,
                                                               const MTile* __restrict__ tiles,
                                                               int32_t* __restrict__ hdr,
                                                               int n_tiles_n) {
  run_items_dma<BN, GateUpOp<BN>, PP>(op, tiles, hdr, op.d, n_tiles_n, HDR_DYN_GATE_UP);
}
template <int BN, bool PP>
__global__ __launch_bounds__(NT_) void down_bf16_dma_kernel(DownOp<BN> op,
                                                            const MTile* __restrict__ tiles,
                                                            int32_t* __restrict__ hdr,
                                                            int n_tiles_n) {
  run_items_dma<BN, DownOp<BN>, PP>(op, tiles, hdr, op.Is, n_tiles_n, HDR_DYN_DOWN);
}

// ---------------------------------------------------------------- K = 64 driver
// The caches of this chip move whole 128-byte lines: a copy that asks for 64 bytes of a row
// (a K stage of 32 elements) pulls the line from L2 into L1 all the same, and when the other
// half is wanted a stage later the line has left the 32 KiB L1 again, so the L2 -> L1 path
// carries every byte twice (measured: copies that touch only half of each line reach half the
// bandwidth at every level of the hierarchy).  With wide sub-experts that path is what the
// kernels above wait for.  This driver therefore works in stages of 64 K-elements, 128 bytes
// per row and copy: 8 lanes of a copy instruction fetch one whole line.
//   * Ring of 2 stages of (256 + BN) rows x 128 bytes (128 KiB for BN = 256).
//   * All waves run the same instruction stream; per stage a wave issues 4 K steps of 2 x NB
//     MFMAs, and the fragments of step i + 1 are read from LDS while step i is multiplied
//     (sched_barriers pin that interleaving), across stage and item borders.
//   * One s_barrier per stage, three quarters into it: by then a wave has read its last
//     fragments of stage q and has waited for its own copies of stage q + 1, so the barrier
//     both frees the slot of stage q and publishes stage q + 1; the copies of stage q + 2 go
//     out right behind it and have one whole stage of flight.
//   * Vector memory operations retire in issue order, so "my copies of stage q + 1 have landed"
//     is s_waitcnt vmcnt(n) with n = what this wave issued after them (an epilogue's stores,
//     a slot-list fetch), bounded from below.
constexpr int SK2 = 64;
template <int BN, bool GATHER>
struct Ring64 {
  static constexpr int NB = BN / 2 / 32;
  static constexpr int WB = BN / 64;  // copy instructions (8 rows x 128 bytes) per wave and stage, weight rows
  static constexpr int A_ST = BM * SK2, B_ST = BN * SK2, STAGE = A_ST + B_ST;  // elements
  static constexpr size_t RING_BYTES = 2 * (size_t)STAGE * 2;
  static constexpr size_t PAIR_BYTES = GATHER ? 2 * BM * sizeof(int32_t) : 0;
  static constexpr size_t EPI_BYTES = GATHER ? 0 : (NT_ / 64) * EPI_WAVE_BYTES;
  static constexpr size_t LDS_BYTES = RING_BYTES + PAIR_BYTES + EPI_BYTES;
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per CU");
};

// N copies of one wave: lane i's 16 bytes at base + voff[j] land at lds + 1024 j + 16 i
template <int N>
__device__ __forceinline__ void dma16_rows(const void* base, const uint32_t (&voff)[N], uint32_t lds) {
  static_assert(N == 3 || N == 4, "copies per group");
  uint32_t keep;
  if constexpr (N == 3) {
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %5\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %4\n\ts_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %2, %4\n\ts_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %3, %4\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "s"(base), "s"(lds)
        : "memory", "scc");
  } else {
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %6\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %5\n\ts_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %2, %5\n\ts_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %3, %5\n\ts_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %4, %5\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "v"(voff[3]), "s"(base), "s"(lds)
        : "memory", "scc");
  }
}
// until at most n of this wave's vector memory operations are pending (n wave-uniform; the
// count is an immediate of s_waitcnt, so n selects one instruction by bisection)
template <int LO, int HI>
__device__ __forceinline__ void wait_upto(int n) {
  if constexpr (LO == HI) {
    wait_copies<LO>();
  } else {
    constexpr int MID = (LO + HI + 1) / 2;
    if (n >= MID)
      wait_upto<MID, HI>(n);
    else
      wait_upto<LO, MID - 1>(n);
  }
}
// which 16-byte chunk of a 128-byte row sits at position pos (inverse of swz)
template <int MODE>
__device__ __forceinline__ int chunk64_of(int r, int pos) {
  const int f = MODE == SWZ_SEQ ? ((r >> 1) & 7) : (((r >> 1) & 3) | (((r >> 4) & 1) << 2));
  return pos ^ f;
}

template <int BN, class Op>
__device__ __forceinline__ void run_items_k64(const Op& op, const MTile* __restrict__ tiles,
                                              int32_t* __restrict__ hdr, int K, int n_tiles_n,
                                              int dyn_word) {
  using RG = Ring64<BN, Op::GATHER>;
  constexpr int NB = RG::NB, WB = RG::WB;
  constexpr int NM = 2 * NB;      // MFMAs per K step
  constexpr int NF = 2 + NB;      // fragments per K step
  extern __shared__ __align__(16) uint16_t smem[];
  int32_t* pair_lds = reinterpret_cast<int32_t*>(smem + 2 * (size_t)RG::STAGE);  // [2][BM]
  const int lane = threadIdx.x & 63, wv = uni(threadIdx.x >> 6);
  uint16_t* epi_lds = RG::EPI_BYTES ? smem + (RG::RING_BYTES + RG::PAIR_BYTES) / 2 + (size_t)wv * (EPI_WAVE_BYTES / 2) : nullptr;
  const int wm = wv >> 1, wn = wv & 1;
  const int wrow = Op::wrow(lane & 31);
  // work split and item order: as in run_items_dma
  int32_t* dyn_next = reinterpret_cast<int32_t*>(smem);
  const int total_items = hdr[HDR_MTILES] * n_tiles_n;
  const int n_static = total_items - total_items / DYN_DIV;
  const int nst = K / SK2;  // K % 64 == 0 on this path
  const int batch = nst >= 12 ? 1 : (12 + nst - 1) / nst;
  ItemRange ir = xcd_items(n_static);
  int n_my = ir.begin < ir.end ? (ir.end - ir.begin + ir.step - 1) / ir.step : 0;
  const uint32_t smem_base = lds_addr(smem);
  const uint32_t pair_base = lds_addr(pair_lds);
  const int sub = lane >> 3, pos = lane & 7;  // a copy covers 8 rows: row lane / 8, position lane % 8

  Sc cur, nxt;
  auto load_sc = [&](int my_idx, Sc& sc) {
    const int item = ir.begin + my_idx * ir.step;
    const MTile t0 = tiles[item / n_tiles_n];
    const int first = uni(t0.first), cnt = uni(t0.count);
    const int L = item - first * n_tiles_n;
    int C = 32 / (cnt < 6 ? cnt : 6);
    C = C > n_tiles_n ? n_tiles_n : C;
    const int per = cnt * C;
    const int c = L / per, r = L % per;
    const int Cc = min(C, n_tiles_n - c * C);
    op.setup_sc(tiles[first + r / Cc], c * C + r % Cc, sc);
  };
  auto fetch_pairs = [&](const Sc& sc, int parity) -> int {
    if (Op::GATHER && wv < 4) {
      dma4(op.idx_src(sc, wv * 64 + lane), pair_base + (uint32_t)(parity * BM + wv * 64) * 4);
      return 1;
    }
    return 0;
  };
  // producer: uniform bases that advance 64 elements per stage, byte offsets of this lane's rows
  const uint16_t* pa;
  const uint16_t* pb;
  uint32_t va[4], vb[WB];
  auto producer_rows = [&](const Sc& sc, int parity) {
    op.bases(sc, pa, pb);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = wv * 32 + j * 8 + sub;
      va[j] = op.a_off(sc, r, pair_lds + parity * BM) + (uint32_t)chunk64_of<SWZ_SEQ>(r, pos) * 16u;
    }
#pragma unroll
    for (int j = 0; j < WB; ++j) {
      const int br = (wv * WB + j) * 8 + sub;
      vb[j] = op.b_off(sc, br) + (uint32_t)chunk64_of<Op::WSWZ>(br, pos) * 16u;
    }
  };
  auto issue_stage = [&](int slot) {
    const uint32_t sa = smem_base + (uint32_t)slot * (RG::STAGE * 2);
    const uint32_t sb = sa + RG::A_ST * 2;
    dma16_rows<4>(pa, va, sa + (uint32_t)wv * 4096u);
    dma16_rows<WB>(pb, vb, sb + (uint32_t)(wv * WB) * 1024u);
    pa += SK2;
    pb += SK2;
  };

  struct Frag {
    bf16x8 t[2], w[NB];
  };
  // fragment e (0, 1: slot-row blocks; 2..: weight blocks) of K step ks of ring slot `slot`
  auto read_frag = [&](int slot, int ks, int e) -> bf16x8 {
    const uint16_t* sa = smem + (size_t)slot * RG::STAGE;
    const int c = ks * 2 + (lane >> 5);
    if (e < 2) return *reinterpret_cast<const bf16x8*>(sa + swz<SWZ_SEQ>(wm * 64 + e * 32 + (lane & 31), c));
    return *reinterpret_cast<const bf16x8*>(sa + RG::A_ST + swz<Op::WSWZ>(wn * (BN / 2) + (e - 2) * 32 + wrow, c));
  };
  auto put_frag = [&](Frag& f, int e, bf16x8 v) {
    if (e < 2) f.t[e] = v; else f.w[e - 2] = v;
  };

  for (;;) {
  if (n_my > 0) {
    const int total = n_my * nst;
    // ---- prologue of one pipeline run over n_my items
    load_sc(0, cur);
    nxt = cur;
    if (n_my > 1) load_sc(1, nxt);
    fetch_pairs(cur, 0);
    wait_copies<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    producer_rows(cur, 0);
    if (n_my > 1) fetch_pairs(nxt, 1);
    int p = 0, p_stage = 0, p_item = 0;  // producer: stages issued, stage inside its item, item
    auto produce = [&]() -> int {       // the next stage's copies, into slot p & 1
      if (p >= total) return 0;
      if (p_stage == nst) {  // the producer enters the next item
        p_stage = 0;
        ++p_item;
        producer_rows(nxt, p_item & 1);
      }
      issue_stage(p & 1);
      ++p;
      ++p_stage;
      return 4 + WB;
    };
    produce();                       // stage 0
    const int second = produce();    // stage 1 (nst >= 2)
    wait_upto<0, 8>(second);         // stage 0 and the slot-list fetch have landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    f32x16 acc[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.0f;
    int mb_on = (cur.rows - wm * 64 + 31) / 32;
    mb_on = uni(mb_on < 0 ? 0 : (mb_on > 2 ? 2 : mb_on));

    Frag f0, f1;
#pragma unroll
    for (int e = 0; e < NF; ++e) put_frag(f0, e, read_frag(0, 0, e));
    int c_stage = 0, c_item = 0;
    int n_allow = 0;  // operations issued after the copies of the stage the next wait is for
    // One K step: the MFMAs of `use`; behind MFMA i the fragment i of (slot_f, ks_f) is read into
    // `fill`.  HOOK: after the first MFMA the stage's wait, barrier and copy issue.
    auto kstep = [&](const Frag& use, Frag& fill, int slot_f, int ks_f, auto on, auto&& hook) {
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const int mb = m / NB, nb = m % NB;
        if constexpr (decltype(on)::value)
          acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(use.w[nb], use.t[mb], acc[nb][mb], 0, 0, 0);
        if (m == 0) hook();
        if (m < NF) put_frag(fill, m, read_frag(slot_f, ks_f, m));
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto nohook = [] {};
    auto stage = [&](int slot, auto on) {
      __builtin_amdgcn_sched_barrier(0);
      kstep(f0, f1, slot, 1, on, nohook);
      kstep(f1, f0, slot, 2, on, nohook);
      kstep(f0, f1, slot, 3, on, nohook);
      kstep(f1, f0, slot ^ 1, 0, on, [&] {
        // every fragment of stage q is in registers (the MFMA above needed the last ones)
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wait_upto<0, 24>(n_allow);       // this wave's copies of stage q + 1 have landed
        n_allow = 0;
        __builtin_amdgcn_s_barrier();    // frees the slot of stage q, publishes stage q + 1
        asm volatile("" ::: "memory");
        produce();                       // stage q + 2 into the slot of stage q
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    for (int q = 0; q < total; ++q) {
      // a wave whose 64 slot rows are all beyond the tile's rows multiplies nothing
      if (mb_on > 0)
        stage(q & 1, std::true_type{});
      else
        stage(q & 1, std::false_type{});
      if (++c_stage == nst) {  // the item is complete
        op.epilogue(cur, acc, mb_on, epi_lds);
        n_allow += uni(op.stores_issued(cur, mb_on, wm, wn));
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.0f;
        c_stage = 0;
        ++c_item;
        cur = nxt;
        mb_on = (cur.rows - wm * 64 + 31) / 32;
        mb_on = uni(mb_on < 0 ? 0 : (mb_on > 2 ? 2 : mb_on));
        if (c_item + 1 < n_my) {
          load_sc(c_item + 1, nxt);
          n_allow += fetch_pairs(nxt, (c_item + 1) & 1);
        }
      }
    }
  }
    // ---- next batch from the pool (every copy of this run has landed, every wave is here)
    wait_copies<0>();
    __syncthreads();
    if (threadIdx.x == 0) *dyn_next = atomicAdd(&hdr[dyn_word], batch);
    __syncthreads();
    ir.begin = n_static + uni(*dyn_next);
    if (ir.begin >= total_items) break;
    ir.end = min(total_items, ir.begin + batch);
    ir.step = 1;
    n_my = ir.end - ir.begin;
  }
}

template <int BN>
__global__ __launch_bounds__(NT_) void gate_up_bf16_k64_kernel(GateUpOp<BN> op,
                                                               const MTile* __restrict__ tiles,
                                                               int32_t* __restrict__ hdr,
                                                               int n_tiles_n) {
  run_items_k64<BN, GateUpOp<BN>>(op, tiles, hdr, op.d, n_tiles_n, HDR_DYN_GATE_UP);
}
template <int BN>
__global__ __launch_bounds__(NT_) void down_bf16_k64_kernel(DownOp<BN> op,
                                                            const MTile* __restrict__ tiles,
                                                            int32_t* __restrict__ hdr,
                                                            int n_tiles_n) {
  run_items_k64<BN, DownOp<BN>>(op, tiles, hdr, op.Is, n_tiles_n, HDR_DYN_DOWN);
}

// ---------------------------------------------------------------- launchers
// The tiles need more than the default 64 KiB of dynamic LDS (the CU has 160 KiB).  The
// attribute is set once per kernel and device, so the launch path makes no other runtime call
// (which also keeps it usable while the caller's stream is being captured into a graph,
// after one eager call).
template <auto Kern>
static hipError_t allow_lds(size_t bytes) {
  static bool done[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
  if (dev >= 0 && done[dev]) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && dev >= 0) done[dev] = true;
  return e;
}

// tile width (in units) with the least padding of n; ties go to the wider tile
static int pick_bn(int n, int wide, int narrow) {
  long pw = (long)cdiv(n, wide) * wide, pn = (long)cdiv(n, narrow) * narrow;
  return pn < pw ? narrow : wide;
}

template <auto Kern, class Op>
static hipError_t launch_persistent(const Op& op, size_t lds_bytes, int grid, const MTile* tiles,
                                    int32_t* hdr, int ntn, hipStream_t s) {
  hipError_t e = allow_lds<Kern>(lds_bytes);
  if (e != hipSuccess) return e;
  Kern<<<grid, NT_, lds_bytes, s>>>(op, tiles, hdr, ntn);
  return hipGetLastError();
}

// Items with at least this many K stages run the two-group schedule; with fewer, the epilogues
// dominate and the in-step schedule is faster (measured at K = 192: 6 stages per item).
constexpr int PP_MIN_STAGES = 12;
// The K = 64 driver needs a few stages per item (its producer runs two stages ahead and enters
// at most one new item per stage).  MOE_PRISM_FFN_K=32 forces the 32-element stages (A/B
// measurements; tests run both drivers on the same shapes).
constexpr int K64_MIN_STAGES = 4;
static bool force_k32() {
  const char* e = getenv("MOE_PRISM_FFN_K");
  return e != nullptr && e[0] == '3' && e[1] == '2' && e[2] == 0;
}

template <int BN>
static hipError_t launch_gate_up_bn(const GateUpOp<BN>& op, int max_mtiles, const MTile* tiles,
                                    int32_t* hdr, hipStream_t s) {
  using RG = Ring<BN, true>;
  const int ntn = cdiv(op.Is, BN / 2);
  const int grid = persistent_grid((long)max_mtiles * ntn, 1);
  const int nst = op.d / SK;
  // stages of 64 K-elements (whole cache lines per row): d % 64 == 0 always; at least 4 stages
  // per item, 32-bit byte offsets inside x and inside one sub-expert's weights
  if (op.d / SK2 >= K64_MIN_STAGES && GateUpOp<BN>::offsets_fit(op.T, op.d, op.Is) && !force_k32())
    return launch_persistent<gate_up_bf16_k64_kernel<BN>>(op, Ring64<BN, true>::LDS_BYTES, grid, tiles, hdr, ntn, s);
  // the ring needs the next tile's slot-list entries one item ahead, published by a barrier
  // before any wave uses them: K/32 >= 2 D stages per item
  if (nst >= 2 * RG::D && nst >= PP_MIN_STAGES)
    return launch_persistent<gate_up_bf16_dma_kernel<BN, true>>(op, RG::LDS_BYTES, grid, tiles, hdr, ntn, s);
  if (nst >= 2 * RG::D)
    return launch_persistent<gate_up_bf16_dma_kernel<BN, false>>(op, RG::LDS_BYTES, grid, tiles, hdr, ntn, s);
  return launch_persistent<gate_up_bf16_kernel<BN>>(op, Tile<BN>::LDS_BYTES, grid, tiles, hdr, ntn, s);
}

hipError_t launch_gate_up_bf16(const uint16_t* x, const uint16_t* w_gu, const int32_t* sorted_pair,
                               const MTile* tiles, int32_t* hdr, uint16_t* h, int T, int d,
                               int Is, int k_max, int max_mtiles, hipStream_t s) {
  if (pick_bn(Is, 128, 96) == 128)
    return launch_gate_up_bn(GateUpOp<256>{x, w_gu, sorted_pair, h, T, d, Is, k_max}, max_mtiles, tiles, hdr, s);
  return launch_gate_up_bn(GateUpOp<192>{x, w_gu, sorted_pair, h, T, d, Is, k_max}, max_mtiles, tiles, hdr, s);
}

template <int BN>
static hipError_t launch_down_bn(const DownOp<BN>& op, int max_mtiles, const MTile* tiles,
                                 int32_t* hdr, hipStream_t s) {
  using RG = Ring<BN, false>;
  const int ntn = cdiv(op.d, BN);
  const int grid = persistent_grid((long)max_mtiles * ntn, 1);
  const int nst = op.Is / SK;
  if (op.Is % SK2 == 0 && op.Is / SK2 >= K64_MIN_STAGES && DownOp<BN>::offsets_fit(0, op.d, op.Is) && !force_k32())
    return launch_persistent<down_bf16_k64_kernel<BN>>(op, Ring64<BN, false>::LDS_BYTES, grid, tiles, hdr, ntn, s);
  // the ring keeps D stages in flight inside one item or the next: K/32 >= NS stages per item
  if (nst >= RG::NS && nst >= PP_MIN_STAGES)
    return launch_persistent<down_bf16_dma_kernel<BN, true>>(op, RG::LDS_BYTES, grid, tiles, hdr, ntn, s);
  if (nst >= RG::NS)
    return launch_persistent<down_bf16_dma_kernel<BN, false>>(op, RG::LDS_BYTES, grid, tiles, hdr, ntn, s);
  return launch_persistent<down_bf16_kernel<BN>>(op, Tile<BN>::LDS_BYTES, grid, tiles, hdr, ntn, s);
}

hipError_t launch_down_bf16(const uint16_t* h, const uint16_t* w_dn, const MTile* tiles,
                            int32_t* hdr, uint16_t* y, int d, int Is, int max_mtiles,
                            hipStream_t s) {
  if (pick_bn(d, 256, 192) == 256)
    return launch_down_bn(DownOp<256>{h, w_dn, y, d, Is}, max_mtiles, tiles, hdr, s);
  return launch_down_bn(DownOp<192>{h, w_dn, y, d, Is}, max_mtiles, tiles, hdr, s);
}

}  // namespace mp
