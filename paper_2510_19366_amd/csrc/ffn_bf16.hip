// bf16 grouped SwiGLU FFN on MFMA (Sec. 3.2.1, Eq. 1-3): the two grouped GEMMs
//   gate-up : h[p, c] = SiLU(x[t_p,:] . Wg[g,c,:]) * (x[t_p,:] . Wu[g,c,:])
//   down    : y[p, q] = sum_c h[p,c] * Wd[g,q,c]
// over ragged groups, as persistent workgroups that walk (m-tile, n-tile) items.
//
// Tile: 256 slot rows x BN weight rows (BN = 256 or 192), K slabs of 64, 8
// wavefronts (4 along the slot rows x 2 along the weight rows), one workgroup
// per CU.  Per K step of 16 a wave multiplies 2 slot blocks by BN/64 weight
// blocks of 32 rows with v_mfma_f32_32x32x16_bf16 (measured at twice the rate
// of the 16x16x32 form on this chip).  The weight block is the MFMA's first
// operand and its rows are fed in a permuted order, so that a lane ends up
// with 8 or 16 consecutive output columns of one slot row and stores them as
// 16-byte words.  Operand slabs go global -> registers ->
// LDS (XOR-swizzled, conflict-free for the fragment reads) one slab ahead of
// the MFMAs, and the software pipeline runs across item boundaries: the first
// slab of the next item is fetched while the last slab of the current one is
// multiplied and its outputs are stored.
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
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

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
#ifndef MP_EXP_NOLOAD
      if (!last)
        pipe.gload(op, cur, (s + 1) * BK, K);
      else if (has_next)
        pipe.gload(op, nxt, 0, K);
#endif
#ifndef MP_EXP_NOMFMA
      pipe.compute(buf, acc, mb_on, wrow);
#endif
      if (last) op.epilogue(cur, acc, mb_on);
#ifndef MP_EXP_NOLOAD
      if (!last || has_next) pipe.sstore(buf ^ 1);
#endif
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

  struct Item {
    int g, row0, rows, n0;  // uniform
    int tok[A_LD];          // tokens of the slot rows this thread copies
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
  __device__ __forceinline__ const uint16_t* b_row(const Item& it, int br) const {
    const int blk = br >> 5, rr = br & 31;  // 32-row block of the tile, row inside it
    const int neuron = min(it.n0 + blk * 16 + (rr & 15), Is - 1);
    return w_gu + ((size_t)it.g * 2 * Is + ((rr >> 4) ? Is + neuron : neuron)) * d;
  }
  __device__ __forceinline__ void epilogue(const Item& it, f32x16 (&acc)[Tile<BN>::NB][2],
                                           int mb_on) const {
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

  struct Item {
    int g, row0, rows, n0;  // uniform
  };

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
  __device__ __forceinline__ const uint16_t* b_row(const Item& it, int br) const {
    return w_dn + ((size_t)it.g * d + min(it.n0 + br, d - 1)) * Is;
  }
  __device__ __forceinline__ void epilogue(const Item& it, f32x16 (&acc)[Tile<BN>::NB][2],
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
};

template <int BN>
__global__ __launch_bounds__(NT_) void down_bf16_kernel(DownOp<BN> op,
                                                        const MTile* __restrict__ tiles,
                                                        const int32_t* __restrict__ hdr,
                                                        int n_tiles_n) {
  run_items<BN>(op, tiles, hdr, op.Is, n_tiles_n);
}

// ---------------------------------------------------------------- launchers
// The tiles need more than the default 64 KiB of dynamic LDS (the CU has 160 KiB).
template <class Kern>
static hipError_t allow_lds(Kern kern, size_t bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// tile width (in units) with the least padding of n; ties go to the wider tile
static int pick_bn(int n, int wide, int narrow) {
  long pw = (long)cdiv(n, wide) * wide, pn = (long)cdiv(n, narrow) * narrow;
  return pn < pw ? narrow : wide;
}

hipError_t launch_gate_up_bf16(const uint16_t* x, const uint16_t* w_gu, const int32_t* sorted_pair,
                               const MTile* tiles, const int32_t* hdr, uint16_t* h, int T, int d,
                               int Is, int k_max, int max_mtiles, hipStream_t s) {
  hipError_t e;
  if (pick_bn(Is, 128, 96) == 128) {
    GateUpOp<256> op{x, w_gu, sorted_pair, h, T, d, Is, k_max};
    const int ntn = cdiv(Is, 128);
    if ((e = allow_lds(gate_up_bf16_kernel<256>, Tile<256>::LDS_BYTES)) != hipSuccess) return e;
    gate_up_bf16_kernel<256><<<persistent_grid((long)max_mtiles * ntn, 1), NT_,
                               Tile<256>::LDS_BYTES, s>>>(op, tiles, hdr, ntn);
  } else {
    GateUpOp<192> op{x, w_gu, sorted_pair, h, T, d, Is, k_max};
    const int ntn = cdiv(Is, 96);
    if ((e = allow_lds(gate_up_bf16_kernel<192>, Tile<192>::LDS_BYTES)) != hipSuccess) return e;
    gate_up_bf16_kernel<192><<<persistent_grid((long)max_mtiles * ntn, 1), NT_,
                               Tile<192>::LDS_BYTES, s>>>(op, tiles, hdr, ntn);
  }
  return hipGetLastError();
}

hipError_t launch_down_bf16(const uint16_t* h, const uint16_t* w_dn, const MTile* tiles,
                            const int32_t* hdr, uint16_t* y, int d, int Is, int max_mtiles,
                            hipStream_t s) {
  hipError_t e;
  if (pick_bn(d, 256, 192) == 256) {
    DownOp<256> op{h, w_dn, y, d, Is};
    const int ntn = cdiv(d, 256);
    if ((e = allow_lds(down_bf16_kernel<256>, Tile<256>::LDS_BYTES)) != hipSuccess) return e;
    down_bf16_kernel<256><<<persistent_grid((long)max_mtiles * ntn, 1), NT_, Tile<256>::LDS_BYTES,
                            s>>>(op, tiles, hdr, ntn);
  } else {
    DownOp<192> op{h, w_dn, y, d, Is};
    const int ntn = cdiv(d, 192);
    if ((e = allow_lds(down_bf16_kernel<192>, Tile<192>::LDS_BYTES)) != hipSuccess) return e;
    down_bf16_kernel<192><<<persistent_grid((long)max_mtiles * ntn, 1), NT_, Tile<192>::LDS_BYTES,
                            s>>>(op, tiles, hdr, ntn);
  }
  return hipGetLastError();
}

}  // namespace mp
