// Internal launcher interface between the C ABI (api.hip) and the kernel files.
// gfx950 only.  Every launcher enqueues on `s` and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mp {

// Workspace header: int32 words at the start of ws.
// HDR_DYN_*: cursors of the FFN kernels' work pools (cleared with the m-tile table)
// HDR_DYN_FUSED .. +7: the fused FFN kernel's per-XCD tile cursors
enum { HDR_FLAGS = 0, HDR_PAIRS = 1, HDR_MTILES = 2, HDR_DYN_GATE_UP = 3, HDR_DYN_DOWN = 4, HDR_DYN_FUSED = 8, HDR_WORDS = 64 };

constexpr int FFN_BM = 256;  // rows of one m-tile of the grouped GEMMs

struct MTile {  // one m-tile of a group: rows [row0, row0 + rows) of the slot list
  int32_t g, row0, rows;
  int32_t first;  // table index of the group's first m-tile
  int32_t count;  // m-tiles of the group
  int32_t pad[3];
};

inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

hipError_t launch_expand_k(int R, int T, const int32_t* req_k, const int32_t* req_off,
                           int32_t* k_tok, hipStream_t s);

hipError_t launch_logits(int dtype, const void* x, const void* w, const float* bias, float* logits,
                         int32_t* hdr, int T, int d, int E, hipStream_t s);
hipError_t launch_topk(const float* logits, const int32_t* k_tok, int32_t* ids, float* w,
                       int32_t* hdr, int T, int E, int k_max, int renorm, float scale,
                       hipStream_t s);

// dispatch: chunk_cnt is [n_chunks, E] scratch
int dispatch_chunk_words(int E, int T);          // 64-token words per chunk
hipError_t launch_dispatch_count(const int32_t* ids, int32_t* chunk_cnt, int T, int E, int k_max,
                                 hipStream_t s);
// proxy gate (Sec. 3.2.2): per-expert top-kappa on the gate-neuron activations
constexpr int PROXY_MAX_SUB = 16;
hipError_t launch_proxy_select(int dtype, const void* act, int act_ld, const int32_t* ids0,
                               const float* w0, const int32_t* slot0, const int32_t* k_tok,
                               const int32_t* kappa, int32_t* ids, float* w, int32_t* hdr, int T,
                               int S, int r, int m, int k_max, hipStream_t s);
hipError_t launch_dispatch_scan(int32_t* chunk_cnt, int32_t* cnt, int T, int E, hipStream_t s);
// also writes off[0..E] and hdr[HDR_PAIRS] (from cnt[]) and, with tiles != nullptr, the grouped
// FFN's m-tile table and its header words (what launch_ffn_tiles builds from off[])
struct MTile;
hipError_t launch_dispatch_place(const int32_t* ids, const int32_t* chunk_base, const int32_t* cnt,
                                 int32_t* off, int32_t* hdr, int32_t* sorted_pair,
                                 int32_t* slot_of_pair, MTile* tiles, int max_tiles, int T, int E,
                                 int k_max, hipStream_t s);

// grouped FFN
hipError_t launch_ffn_tiles(const int32_t* off, MTile* tiles, int32_t* hdr, int E, int max_tiles,
                            int n_rows, hipStream_t s);
hipError_t launch_ffn_gate_up(int dtype, const void* x, const void* w_gu, const int32_t* sorted_pair,
                              const MTile* tiles, int32_t* hdr, void* h, int T, int d, int Is,
                              int k_max, int max_mtiles, hipStream_t s);
hipError_t launch_ffn_down(int dtype, const void* h, const void* w_dn, const MTile* tiles,
                           int32_t* hdr, void* y, int d, int Is, int max_mtiles,
                           hipStream_t s);

// fused gate-up -> SwiGLU -> down for narrow sub-experts (bf16); see ffn_fused_bf16.hip
bool ffn_fused_supported(int T, int d, int Is);
hipError_t launch_ffn_fused_bf16(const uint16_t* x, const uint16_t* w_gu, const uint16_t* w_dn,
                                 const int32_t* sorted_pair, const MTile* tiles, int32_t* hdr,
                                 uint16_t* y, int T, int d, int Is, int k_max, int max_mtiles,
                                 hipStream_t s);
// the same kernel without the matrix products (measurement: its memory traffic alone)
hipError_t launch_ffn_fused_traffic_bf16(const uint16_t* x, const uint16_t* w_gu,
                                         const uint16_t* w_dn, const int32_t* sorted_pair,
                                         const MTile* tiles, int32_t* hdr, uint16_t* y, int T,
                                         int d, int Is, int k_max, int max_mtiles, hipStream_t s);

hipError_t launch_combine(int dtype, const void* y, const int32_t* slot_of_pair, const float* w,
                          const int32_t* k_tok, void* out, int T, int d, int k_max, hipStream_t s);

int num_cus();  // compute units of the current device (cached)

// bf16 helpers (bit patterns in uint16_t)
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// two fp32 -> two bf16 (round to nearest even) in one word, a in the low half: v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

}  // namespace mp
