// C ABI of the library (see include/moe_prism.h): argument checks, workspace
// layout, per-kernel event timing, and the stage / layer entry points.  All
// arithmetic is in the kernel files.
#include "../../include/moe_prism.h"

#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "kernels.h"

namespace mp {

int num_cus() {
  static int cached = 0;
  if (cached == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cached = prop.multiProcessorCount;
    if (cached <= 0) cached = 256;
  }
  return cached;
}

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Layout {
  size_t hdr, logits, chunk_cnt, tiles, h, ids, w, cnt, off, sorted_pair, slot_of_pair, y, total;
  int max_mtiles, n_chunks;
};

static int check_shape(const moe_prism_shape* s) {
  if (s == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  if (s->T < 0 || s->d <= 0 || s->n_experts <= 0 || s->n_sub <= 0 || s->inter_sub <= 0 ||
      s->k_max <= 0)
    return MOE_PRISM_ERR_INVALID_ARG;
  if (s->dtype != MOE_PRISM_F32 && s->dtype != MOE_PRISM_BF16) return MOE_PRISM_ERR_INVALID_ARG;
  if (s->renormalize != 0 && s->renormalize != 1) return MOE_PRISM_ERR_INVALID_ARG;
  long E = (long)s->n_experts * s->n_sub;
  if (s->d % 64 != 0 || s->inter_sub % 32 != 0) return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  if (E > 4096 || s->k_max > E || s->k_max > 1024) return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  if ((long)s->T * s->k_max >= (1L << 31) || (long)s->T * E >= (1L << 31))
    return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  if ((long)s->T * s->k_max * s->inter_sub >= (1L << 40)) return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  return MOE_PRISM_OK;
}

static Layout layout_of(const moe_prism_shape* s) {
  Layout L;
  const size_t T = (size_t)s->T, E = (size_t)s->n_experts * s->n_sub, km = (size_t)s->k_max;
  const size_t el = s->dtype == MOE_PRISM_F32 ? 4 : 2;
  const size_t rows = T * km;
  L.n_chunks = cdiv((long)T, 64L * dispatch_chunk_words((int)E, s->T));
  L.max_mtiles = (int)(rows / FFN_BM + E);
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o += align256(bytes);
    return at;
  };
  L.hdr = take(HDR_WORDS * 4);
  L.logits = take(T * E * 4);
  L.chunk_cnt = take((size_t)L.n_chunks * E * 4);
  L.tiles = take((size_t)L.max_mtiles * sizeof(MTile));
  L.h = take(rows * s->inter_sub * el);
  L.ids = take(rows * 4);
  L.w = take(rows * 4);
  L.cnt = take(E * 4);
  L.off = take((E + 1) * 4);
  L.sorted_pair = take(rows * 4);
  L.slot_of_pair = take(rows * 4);
  L.y = take(rows * s->d * el);
  L.total = o;
  return L;
}

// ------------------------------------------------------------ event timing
struct Rec {
  int kernel;
  hipEvent_t a, b;
};
static std::mutex g_mu;
static bool g_timing = false;
static uint32_t g_timing_mask = ~0u;  // bit k: kernel id k is timed
static std::vector<Rec> g_recs;
static std::vector<hipEvent_t> g_pool;

static hipEvent_t get_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

struct Timed {  // brackets one kernel launch with events when timing is on
  hipStream_t s;
  Rec r{};
  bool on = false;
  Timed(int kernel, hipStream_t st) : s(st) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_timing || ((g_timing_mask >> kernel) & 1u) == 0) return;
    on = true;
    r.kernel = kernel;
    r.a = get_event();
    r.b = get_event();
    (void)hipEventRecord(r.a, s);
  }
  ~Timed() {
    if (!on) return;
    (void)hipEventRecord(r.b, s);
    std::lock_guard<std::mutex> lk(g_mu);
    g_recs.push_back(r);
  }
};

#define MP_LAUNCH(KERNEL_ID, CALL)                          \
  do {                                                      \
    hipError_t e_;                                          \
    {                                                       \
      mp::Timed timed_(KERNEL_ID, st);                      \
      e_ = (CALL);                                          \
    }                                                       \
    if (e_ != hipSuccess) return MOE_PRISM_ERR_LAUNCH;      \
  } while (0)

// ------------------------------------------------------------ stages on a layout
static int do_route(const moe_prism_shape* s, const Layout& L, const void* x, const void* w_router,
                    const float* bias, const int32_t* k_tok, int32_t* ids, float* w, float* logits,
                    char* ws, hipStream_t st) {
  const int E = s->n_experts * s->n_sub;
  int32_t* hdr = reinterpret_cast<int32_t*>(ws + L.hdr);
  MP_LAUNCH(MOE_PRISM_K_LOGITS,
            launch_logits(s->dtype, x, w_router, bias, logits, hdr, s->T, s->d, E, st));
  MP_LAUNCH(MOE_PRISM_K_TOPK, launch_topk(logits, k_tok, ids, w, hdr, s->T, E, s->k_max,
                                          s->renormalize, s->routed_scale, st));
  return MOE_PRISM_OK;
}

// with_tiles: the place kernel also builds the grouped FFN's m-tile table (the layer entry
// points, where the FFN follows on the same offsets; do_ffn is then told not to rebuild it)
static int do_dispatch(const moe_prism_shape* s, const Layout& L, const int32_t* ids, int32_t* cnt,
                       int32_t* off, int32_t* sorted_pair, int32_t* slot_of_pair, char* ws,
                       hipStream_t st, bool with_tiles = false) {
  const int E = s->n_experts * s->n_sub;
  int32_t* hdr = reinterpret_cast<int32_t*>(ws + L.hdr);
  int32_t* chunk = reinterpret_cast<int32_t*>(ws + L.chunk_cnt);
  MP_LAUNCH(MOE_PRISM_K_DISPATCH_COUNT, launch_dispatch_count(ids, chunk, s->T, E, s->k_max, st));
  MP_LAUNCH(MOE_PRISM_K_DISPATCH_SCAN, launch_dispatch_scan(chunk, cnt, s->T, E, st));
  MP_LAUNCH(MOE_PRISM_K_DISPATCH_PLACE,
            launch_dispatch_place(ids, chunk, cnt, off, hdr, sorted_pair, slot_of_pair,
                                  with_tiles ? reinterpret_cast<MTile*>(ws + L.tiles) : nullptr,
                                  L.max_mtiles, s->T, E, s->k_max, st));
  return MOE_PRISM_OK;
}

// The fused gate-up/SwiGLU/down kernel serves bf16 layers with narrow sub-experts; the
// environment variable MOE_PRISM_FFN=split forces the two-kernel path (for A/B measurements
// and so that tests reach both paths on the same shapes).
static bool use_fused_ffn(const moe_prism_shape* s) {
  if (s->dtype != MOE_PRISM_BF16 || !ffn_fused_supported(s->T, s->d, s->inter_sub)) return false;
  const char* e = getenv("MOE_PRISM_FFN");
  return !(e != nullptr && strcmp(e, "split") == 0);
}

static int do_ffn(const moe_prism_shape* s, const Layout& L, const void* x, const void* w_gu,
                  const void* w_dn, const int32_t* off, const int32_t* sorted_pair, void* y,
                  char* ws, hipStream_t st, bool traffic_probe = false, bool tiles_built = false) {
  const int E = s->n_experts * s->n_sub;
  int32_t* hdr = reinterpret_cast<int32_t*>(ws + L.hdr);
  MTile* tiles = reinterpret_cast<MTile*>(ws + L.tiles);
  void* h = ws + L.h;
  if (!tiles_built)
    MP_LAUNCH(MOE_PRISM_K_FFN_TILES, launch_ffn_tiles(off, tiles, hdr, E, L.max_mtiles, s->T * s->k_max, st));
  if (s->T == 0) return MOE_PRISM_OK;
  if (traffic_probe) {
    MP_LAUNCH(MOE_PRISM_K_FFN_TRAFFIC,
              launch_ffn_fused_traffic_bf16((const uint16_t*)x, (const uint16_t*)w_gu,
                                            (const uint16_t*)w_dn, sorted_pair, tiles, hdr,
                                            (uint16_t*)y, s->T, s->d, s->inter_sub, s->k_max,
                                            L.max_mtiles, st));
    return MOE_PRISM_OK;
  }
  if (use_fused_ffn(s)) {
    MP_LAUNCH(MOE_PRISM_K_FFN_FUSED,
              launch_ffn_fused_bf16((const uint16_t*)x, (const uint16_t*)w_gu, (const uint16_t*)w_dn,
                                    sorted_pair, tiles, hdr, (uint16_t*)y, s->T, s->d, s->inter_sub,
                                    s->k_max, L.max_mtiles, st));
    return MOE_PRISM_OK;
  }
  MP_LAUNCH(MOE_PRISM_K_FFN_GATE_UP,
            launch_ffn_gate_up(s->dtype, x, w_gu, sorted_pair, tiles, hdr, h, s->T, s->d, s->inter_sub,
                               s->k_max, L.max_mtiles, st));
  MP_LAUNCH(MOE_PRISM_K_FFN_DOWN, launch_ffn_down(s->dtype, h, w_dn, tiles, hdr, y, s->d,
                                                  s->inter_sub, L.max_mtiles, st));
  return MOE_PRISM_OK;
}

// Proxy-gate route stage (Sec. 3.2.2, training-free proxy gating): the original router's
// top-m experts, a grouped gate-up pass over the gate neurons' rows, per-expert top-kappa.
// Scratch: the logits, chunk-count, tile and h regions, and the start of the y region.
struct ProxyScratch {
  int32_t *ids0, *cnt0, *off0, *sp0, *sl0;
  float* w0;
};
static ProxyScratch proxy_scratch(const moe_prism_shape* s, const Layout& L, char* ws, int m) {
  char* p = ws + L.y;
  const size_t n = align256((size_t)s->T * m * 4);
  ProxyScratch q;
  q.ids0 = reinterpret_cast<int32_t*>(p);
  q.w0 = reinterpret_cast<float*>(p + n);
  q.sp0 = reinterpret_cast<int32_t*>(p + 2 * n);
  q.sl0 = reinterpret_cast<int32_t*>(p + 3 * n);
  q.cnt0 = reinterpret_cast<int32_t*>(p + 4 * n);
  q.off0 = reinterpret_cast<int32_t*>(p + 4 * n + align256((size_t)s->n_experts * 4));
  return q;
}
static int check_proxy(const moe_prism_shape* s, int m, int r, int rows_half) {
  const long el = s->dtype == MOE_PRISM_F32 ? 4 : 2;
  if (m <= 0 || r <= 0 || rows_half <= 0) return MOE_PRISM_ERR_INVALID_ARG;
  if (m > s->n_experts || s->n_sub > PROXY_MAX_SUB || rows_half % 32 != 0 ||
      rows_half < s->n_sub * r)
    return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  // the stage's activations [T*m, rows_half] live in the h region, its tables in the y region
  if ((long)m * rows_half > (long)s->k_max * s->inter_sub) return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  // the stage's T*m pairs over N groups are cut into m-tiles in the layer's tile table
  // (T*k_max / FFN_BM + E entries): they must fit (always true for m <= k_max)
  const long table = (long)s->T * s->k_max / FFN_BM + (long)s->n_experts * s->n_sub;
  if ((long)s->T * m / FFN_BM + s->n_experts > table) return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  if (4L * align256((size_t)s->T * m * 4) + 2L * align256(((size_t)s->n_experts + 1) * 4) >
      (long)s->T * s->k_max * s->d * el)
    return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  return MOE_PRISM_OK;
}
static int do_route_proxy(const moe_prism_shape* s, const Layout& L, const void* x,
                          const void* w_router0, const float* bias0, const void* w_proxy, int m,
                          int r, int rows_half, const int32_t* kappa, const int32_t* k_tok,
                          int32_t* ids, float* w, char* ws, hipStream_t st) {
  const int N = s->n_experts;
  int32_t* hdr = reinterpret_cast<int32_t*>(ws + L.hdr);
  float* logits0 = reinterpret_cast<float*>(ws + L.logits);
  int32_t* chunk = reinterpret_cast<int32_t*>(ws + L.chunk_cnt);
  MTile* tiles = reinterpret_cast<MTile*>(ws + L.tiles);
  void* act = ws + L.h;
  const ProxyScratch q = proxy_scratch(s, L, ws, m);
  MP_LAUNCH(MOE_PRISM_K_LOGITS,
            launch_logits(s->dtype, x, w_router0, bias0, logits0, hdr, s->T, s->d, N, st));
  MP_LAUNCH(MOE_PRISM_K_TOPK, launch_topk(logits0, nullptr, q.ids0, q.w0, hdr, s->T, N, m,
                                          s->renormalize, s->routed_scale, st));
  MP_LAUNCH(MOE_PRISM_K_DISPATCH_COUNT, launch_dispatch_count(q.ids0, chunk, s->T, N, m, st));
  MP_LAUNCH(MOE_PRISM_K_DISPATCH_SCAN, launch_dispatch_scan(chunk, q.cnt0, s->T, N, st));
  MP_LAUNCH(MOE_PRISM_K_DISPATCH_PLACE,
            launch_dispatch_place(q.ids0, chunk, q.cnt0, q.off0, hdr, q.sp0, q.sl0, nullptr, 0, s->T, N,
                                  m, st));
  MP_LAUNCH(MOE_PRISM_K_FFN_TILES, launch_ffn_tiles(q.off0, tiles, hdr, N, L.max_mtiles, s->T * m, st));
  if (s->T == 0) return MOE_PRISM_OK;
  MP_LAUNCH(MOE_PRISM_K_FFN_GATE_UP,
            launch_ffn_gate_up(s->dtype, x, w_proxy, q.sp0, tiles, hdr, act, s->T, s->d, rows_half, m,
                               L.max_mtiles, st));
  MP_LAUNCH(MOE_PRISM_K_PROXY_SELECT,
            launch_proxy_select(s->dtype, act, rows_half, q.ids0, q.w0, q.sl0, k_tok, kappa, ids, w,
                                hdr, s->T, s->n_sub, r, m, s->k_max, st));
  return MOE_PRISM_OK;
}

}  // namespace mp

using namespace mp;

#define MP_CHECK_SHAPE(s)            \
  do {                               \
    int rc_ = check_shape(s);        \
    if (rc_ != MOE_PRISM_OK) return rc_; \
  } while (0)

#define MP_CHECK_WS(s, L, ws, ws_bytes)                                          \
  Layout L = layout_of(s);                                                       \
  do {                                                                           \
    if ((ws) == nullptr || ((uintptr_t)(ws) & 255) != 0) return MOE_PRISM_ERR_INVALID_ARG; \
    if ((ws_bytes) < L.total) return MOE_PRISM_ERR_WORKSPACE;                    \
  } while (0)

extern "C" {

int moe_prism_workspace_bytes(const moe_prism_shape* shape, size_t* bytes) {
  if (bytes == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  MP_CHECK_SHAPE(shape);
  *bytes = layout_of(shape).total;
  return MOE_PRISM_OK;
}

int moe_prism_layer_offsets(const moe_prism_shape* shape, size_t* offsets) {
  if (offsets == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  MP_CHECK_SHAPE(shape);
  Layout L = layout_of(shape);
  size_t v[8] = {L.ids, L.w, L.cnt, L.off, L.sorted_pair, L.slot_of_pair, L.y, L.logits};
  for (int i = 0; i < 8; ++i) offsets[i] = v[i];
  return MOE_PRISM_OK;
}

int moe_prism_expand_k(int32_t R, int32_t T_total, const int32_t* req_k, const int32_t* req_off,
                       int32_t* k_tok, void* stream) {
  if (R < 0 || T_total < 0) return MOE_PRISM_ERR_INVALID_ARG;
  if (R == 0 || T_total == 0) return MOE_PRISM_OK;
  if (req_k == nullptr || req_off == nullptr || k_tok == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (launch_expand_k(R, T_total, req_k, req_off, k_tok, st) != hipSuccess)
    return MOE_PRISM_ERR_LAUNCH;
  return MOE_PRISM_OK;
}

int moe_prism_route(const moe_prism_shape* shape, const void* x, const void* w_router,
                    const float* router_bias, const int32_t* k_tok, int32_t* topk_ids,
                    float* topk_w, float* logits_out, void* ws, size_t ws_bytes, void* stream) {
  MP_CHECK_SHAPE(shape);
  if (w_router == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->T > 0 && (x == nullptr || k_tok == nullptr || topk_ids == nullptr || topk_w == nullptr))
    return MOE_PRISM_ERR_INVALID_ARG;
  MP_CHECK_WS(shape, L, ws, ws_bytes);
  char* w8 = static_cast<char*>(ws);
  float* logits = logits_out ? logits_out : reinterpret_cast<float*>(w8 + L.logits);
  return do_route(shape, L, x, w_router, router_bias, k_tok, topk_ids, topk_w, logits, w8,
                  (hipStream_t)stream);
}

int moe_prism_dispatch(const moe_prism_shape* shape, const int32_t* topk_ids, int32_t* group_count,
                       int32_t* group_offset, int32_t* sorted_pair, int32_t* slot_of_pair,
                       void* ws, size_t ws_bytes, void* stream) {
  MP_CHECK_SHAPE(shape);
  if (group_count == nullptr || group_offset == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->T > 0 && (topk_ids == nullptr || sorted_pair == nullptr || slot_of_pair == nullptr))
    return MOE_PRISM_ERR_INVALID_ARG;
  MP_CHECK_WS(shape, L, ws, ws_bytes);
  return do_dispatch(shape, L, topk_ids, group_count, group_offset, sorted_pair, slot_of_pair,
                     static_cast<char*>(ws), (hipStream_t)stream);
}

int moe_prism_grouped_ffn(const moe_prism_shape* shape, const void* x, const void* w_gate_up,
                          const void* w_down, const int32_t* group_offset,
                          const int32_t* sorted_pair, void* y, void* ws, size_t ws_bytes,
                          void* stream) {
  MP_CHECK_SHAPE(shape);
  if (w_gate_up == nullptr || w_down == nullptr || group_offset == nullptr)
    return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->T > 0 && (x == nullptr || sorted_pair == nullptr || y == nullptr))
    return MOE_PRISM_ERR_INVALID_ARG;
  MP_CHECK_WS(shape, L, ws, ws_bytes);
  return do_ffn(shape, L, x, w_gate_up, w_down, group_offset, sorted_pair, y,
                static_cast<char*>(ws), (hipStream_t)stream);
}

int moe_prism_ffn_traffic_probe(const moe_prism_shape* shape, const void* x, const void* w_gate_up,
                                const void* w_down, const int32_t* group_offset,
                                const int32_t* sorted_pair, void* y, void* ws, size_t ws_bytes,
                                void* stream) {
  MP_CHECK_SHAPE(shape);
  if (w_gate_up == nullptr || w_down == nullptr || group_offset == nullptr)
    return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->T > 0 && (x == nullptr || sorted_pair == nullptr || y == nullptr))
    return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->dtype != MOE_PRISM_BF16 || !mp::ffn_fused_supported(shape->T, shape->d, shape->inter_sub))
    return MOE_PRISM_ERR_UNSUPPORTED_SHAPE;
  MP_CHECK_WS(shape, L, ws, ws_bytes);
  return do_ffn(shape, L, x, w_gate_up, w_down, group_offset, sorted_pair, y,
                static_cast<char*>(ws), (hipStream_t)stream, true);
}

int moe_prism_combine(const moe_prism_shape* shape, const void* y, const int32_t* slot_of_pair,
                      const float* topk_w, const int32_t* k_tok, void* out, void* stream) {
  MP_CHECK_SHAPE(shape);
  if (shape->T == 0) return MOE_PRISM_OK;
  if (y == nullptr || slot_of_pair == nullptr || topk_w == nullptr || k_tok == nullptr ||
      out == nullptr)
    return MOE_PRISM_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  MP_LAUNCH(MOE_PRISM_K_COMBINE, launch_combine(shape->dtype, y, slot_of_pair, topk_w, k_tok, out,
                                                shape->T, shape->d, shape->k_max, st));
  return MOE_PRISM_OK;
}

// Workspace of moe_prism_layer_static: one file-scope device array per GPU, held until the
// process ends.  `scratch` itself is only a host-side handle of the symbol; the device address
// is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[MOE_PRISM_STATIC_WS_BYTES];
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[64] = {};

static int static_workspace(char** ws) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MOE_PRISM_ERR_LAUNCH;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr)
      return MOE_PRISM_ERR_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *ws = static_cast<char*>(g_scratch_ptr[dev]);
  return MOE_PRISM_OK;
}

static int layer_on(const moe_prism_shape* shape, const Layout& L, const void* x,
                    const void* w_router, const float* router_bias, const int32_t* k_tok,
                    const void* w_gate_up, const void* w_down, void* out, char* w8, hipStream_t st) {
  int32_t* ids = reinterpret_cast<int32_t*>(w8 + L.ids);
  float* w = reinterpret_cast<float*>(w8 + L.w);
  int32_t* cnt = reinterpret_cast<int32_t*>(w8 + L.cnt);
  int32_t* off = reinterpret_cast<int32_t*>(w8 + L.off);
  int32_t* sp = reinterpret_cast<int32_t*>(w8 + L.sorted_pair);
  int32_t* sl = reinterpret_cast<int32_t*>(w8 + L.slot_of_pair);
  void* y = w8 + L.y;
  int rc = do_route(shape, L, x, w_router, router_bias, k_tok, ids, w,
                    reinterpret_cast<float*>(w8 + L.logits), w8, st);
  if (rc) return rc;
  rc = do_dispatch(shape, L, ids, cnt, off, sp, sl, w8, st, true);
  if (rc) return rc;
  rc = do_ffn(shape, L, x, w_gate_up, w_down, off, sp, y, w8, st, false, true);
  if (rc) return rc;
  if (shape->T == 0) return MOE_PRISM_OK;
  MP_LAUNCH(MOE_PRISM_K_COMBINE, launch_combine(shape->dtype, y, sl, w, k_tok, out, shape->T,
                                                shape->d, shape->k_max, st));
  return MOE_PRISM_OK;
}

int moe_prism_layer(const moe_prism_shape* shape, const void* x, const void* w_router,
                    const float* router_bias, const int32_t* k_tok, const void* w_gate_up,
                    const void* w_down, void* out, void* ws, size_t ws_bytes, void* stream) {
  MP_CHECK_SHAPE(shape);
  if (w_router == nullptr || w_gate_up == nullptr || w_down == nullptr)
    return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->T > 0 && (x == nullptr || k_tok == nullptr || out == nullptr))
    return MOE_PRISM_ERR_INVALID_ARG;
  MP_CHECK_WS(shape, L, ws, ws_bytes);
  return layer_on(shape, L, x, w_router, router_bias, k_tok, w_gate_up, w_down, out,
                  static_cast<char*>(ws), (hipStream_t)stream);
}

int moe_prism_layer_static(const moe_prism_shape* shape, const void* x, const void* w_router,
                           const float* router_bias, const int32_t* k_tok, const void* w_gate_up,
                           const void* w_down, void* out, void* stream) {
  MP_CHECK_SHAPE(shape);
  if (w_router == nullptr || w_gate_up == nullptr || w_down == nullptr)
    return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->T > 0 && (x == nullptr || k_tok == nullptr || out == nullptr))
    return MOE_PRISM_ERR_INVALID_ARG;
  const Layout L = layout_of(shape);
  if (L.total > (size_t)MOE_PRISM_STATIC_WS_BYTES) return MOE_PRISM_ERR_WORKSPACE;
  char* w8 = nullptr;
  int rc = static_workspace(&w8);
  if (rc) return rc;
  return layer_on(shape, L, x, w_router, router_bias, k_tok, w_gate_up, w_down, out, w8,
                  (hipStream_t)stream);
}

int moe_prism_route_proxy(const moe_prism_shape* shape, const void* x, const void* w_router0,
                          const float* router_bias0, const void* w_proxy, int32_t m, int32_t r,
                          int32_t rows_half, const int32_t* kappa, const int32_t* k_tok,
                          int32_t* topk_ids, float* topk_w, void* ws, size_t ws_bytes, void* stream) {
  MP_CHECK_SHAPE(shape);
  int rc = check_proxy(shape, m, r, rows_half);
  if (rc) return rc;
  if (w_router0 == nullptr || w_proxy == nullptr || kappa == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->T > 0 && (x == nullptr || k_tok == nullptr || topk_ids == nullptr || topk_w == nullptr))
    return MOE_PRISM_ERR_INVALID_ARG;
  MP_CHECK_WS(shape, L, ws, ws_bytes);
  return do_route_proxy(shape, L, x, w_router0, router_bias0, w_proxy, m, r, rows_half, kappa, k_tok,
                        topk_ids, topk_w, static_cast<char*>(ws), (hipStream_t)stream);
}

int moe_prism_layer_proxy(const moe_prism_shape* shape, const void* x, const void* w_router0,
                          const float* router_bias0, const void* w_proxy, int32_t m, int32_t r,
                          int32_t rows_half, const int32_t* kappa, const int32_t* k_tok,
                          const void* w_gate_up, const void* w_down, void* out, void* ws,
                          size_t ws_bytes, void* stream) {
  MP_CHECK_SHAPE(shape);
  int rc = check_proxy(shape, m, r, rows_half);
  if (rc) return rc;
  if (w_router0 == nullptr || w_proxy == nullptr || kappa == nullptr || w_gate_up == nullptr ||
      w_down == nullptr)
    return MOE_PRISM_ERR_INVALID_ARG;
  if (shape->T > 0 && (x == nullptr || k_tok == nullptr || out == nullptr))
    return MOE_PRISM_ERR_INVALID_ARG;
  MP_CHECK_WS(shape, L, ws, ws_bytes);
  char* w8 = static_cast<char*>(ws);
  hipStream_t st = (hipStream_t)stream;
  int32_t* ids = reinterpret_cast<int32_t*>(w8 + L.ids);
  float* w = reinterpret_cast<float*>(w8 + L.w);
  int32_t* cnt = reinterpret_cast<int32_t*>(w8 + L.cnt);
  int32_t* off = reinterpret_cast<int32_t*>(w8 + L.off);
  int32_t* sp = reinterpret_cast<int32_t*>(w8 + L.sorted_pair);
  int32_t* sl = reinterpret_cast<int32_t*>(w8 + L.slot_of_pair);
  void* y = w8 + L.y;
  rc = do_route_proxy(shape, L, x, w_router0, router_bias0, w_proxy, m, r, rows_half, kappa, k_tok,
                      ids, w, w8, st);
  if (rc) return rc;
  rc = do_dispatch(shape, L, ids, cnt, off, sp, sl, w8, st, true);
  if (rc) return rc;
  rc = do_ffn(shape, L, x, w_gate_up, w_down, off, sp, y, w8, st, false, true);
  if (rc) return rc;
  if (shape->T == 0) return MOE_PRISM_OK;
  MP_LAUNCH(MOE_PRISM_K_COMBINE, launch_combine(shape->dtype, y, sl, w, k_tok, out, shape->T,
                                                shape->d, shape->k_max, st));
  return MOE_PRISM_OK;
}

int moe_prism_status(const void* ws, int32_t* host_flags, int32_t* host_pairs, void* stream) {
  if (ws == nullptr) return MOE_PRISM_ERR_INVALID_ARG;
  int32_t hdr[2] = {0, 0};
  hipStream_t st = (hipStream_t)stream;
  if (hipMemcpyAsync(hdr, ws, sizeof(hdr), hipMemcpyDeviceToHost, st) != hipSuccess)
    return MOE_PRISM_ERR_LAUNCH;
  if (hipStreamSynchronize(st) != hipSuccess) return MOE_PRISM_ERR_LAUNCH;
  if (host_flags) *host_flags = hdr[HDR_FLAGS];
  if (host_pairs) *host_pairs = hdr[HDR_PAIRS];
  return MOE_PRISM_OK;
}

int moe_prism_timing_enable(int on) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_timing = on != 0;
  return MOE_PRISM_OK;
}

int moe_prism_timing_select(uint32_t kernel_mask) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_timing_mask = kernel_mask;
  return MOE_PRISM_OK;
}

int moe_prism_timing_read(float* ms, int32_t* calls) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (int i = 0; i < MOE_PRISM_N_KERNELS; ++i) {
    if (ms) ms[i] = 0.0f;
    if (calls) calls[i] = 0;
  }
  int rc = MOE_PRISM_OK;
  for (const Rec& r : g_recs) {
    float t = 0.0f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&t, r.a, r.b) != hipSuccess)
      rc = MOE_PRISM_ERR_LAUNCH;
    if (ms) ms[r.kernel] += t;
    if (calls) calls[r.kernel] += 1;
    g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_recs.clear();
  return rc;
}

const char* moe_prism_strerror(int code) {
  switch (code) {
    case MOE_PRISM_OK: return "ok";
    case MOE_PRISM_ERR_INVALID_ARG: return "invalid argument (null pointer, negative size, bad flag, unaligned workspace)";
    case MOE_PRISM_ERR_UNSUPPORTED_SHAPE: return "unsupported shape (need d % 64 == 0, inter_sub % 32 == 0, k_max <= min(E, 1024), E <= 4096, int32 index range)";
    case MOE_PRISM_ERR_WORKSPACE: return "workspace smaller than moe_prism_workspace_bytes() (or, for moe_prism_layer_static, the shape needs more than MOE_PRISM_STATIC_WS_BYTES)";
    case MOE_PRISM_ERR_LAUNCH: return "HIP runtime error while enqueuing";
    default: return "unknown error";
  }
}

}  // extern "C"
