/*
 * moe_prism.h - C ABI of the MI355X (gfx950) routed-expert forward of an MoE FFN
 * layer whose experts are split into sub-experts and whose top-k varies per token.
 *
 * Method: MoE-Prism (arXiv 2510.19366).  N experts are each cut into S
 * sub-experts along the SwiGLU intermediate dimension (Sec. 3.2.1, Eq. 1-3); one
 * linear gate scores all E = N*S sub-experts and a layer-wide top-k is taken
 * (Sec. 3.2.2, expanded linear gate); the budget k belongs to a request and each
 * of its tokens inherits it (Sec. 3.3.1).  Unlike the batch-maximum execution
 * of Sec. 3.3.1 / 3.4.2, this library resolves k per token on the device, so the
 * work is sum_t k_t token-sub-expert pairs (Sec. 2.1) and not T * max k.
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers owned by the caller unless the
 *     argument says "host".  The library never allocates, frees or synchronises
 *     (except moe_prism_status and moe_prism_timing_read, which say so).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     kernels of a call are enqueued on it, in order.
 *   - `ws` is a caller-owned device workspace of at least
 *     moe_prism_workspace_bytes() bytes, 256-byte aligned.  Its first bytes hold
 *     a status word and counters written by the kernels; the rest is scratch.
 *     Calls that share a workspace must be ordered on one stream.
 *   - Return value: MOE_PRISM_OK or a negative error.  Errors found on the host
 *     are returned before anything is launched.  Conditions visible only on the
 *     device (a budget outside [0, k_max]) are clamped and flagged in the status
 *     word (moe_prism_status).
 *   - Layouts are row-major, innermost index last.  Activations and weights are
 *     fp32 (dtype 0) or bf16 bit patterns (dtype 1); logits, routing weights and
 *     all tables are fp32 / int32 for both.
 *   - A token-sub-expert pair is named pair = t * k_max + j (j-th pick of token
 *     t).  A slot is a row of the group-major pair list.  g = e * S + s is the
 *     flat sub-expert id (expert-major).
 */
#ifndef MOE_PRISM_H
#define MOE_PRISM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported from the shared library */
#define MOE_PRISM_API __attribute__((visibility("default")))

#define MOE_PRISM_OK 0
#define MOE_PRISM_ERR_INVALID_ARG (-1)       /* null pointer, negative size, bad flag   */
#define MOE_PRISM_ERR_UNSUPPORTED_SHAPE (-2) /* see moe_prism_shape                      */
#define MOE_PRISM_ERR_WORKSPACE (-3)         /* ws_bytes < moe_prism_workspace_bytes()   */
#define MOE_PRISM_ERR_LAUNCH (-4)            /* the HIP runtime refused a launch         */

#define MOE_PRISM_F32 0
#define MOE_PRISM_BF16 1

/* status-word bits (moe_prism_status) */
#define MOE_PRISM_STATUS_K_CLAMPED 1 /* some k_tok[t] was outside [0, k_max] and was clamped */
#define MOE_PRISM_STATUS_TILES_TRUNCATED 2 /* group offsets describe more 256-row tiles than the
                                              workspace's tile table holds: rows were left out */

/*
 * Problem shape (host struct, read during the call, not retained).
 * Supported: T >= 0; d % 64 == 0, d >= 64; inter_sub % 32 == 0; 1 <= k_max <= min(E, 1024);
 * E = n_experts * n_sub <= 4096.  T * k_max and T * E must fit in int32.
 */
typedef struct {
  int32_t T;           /* tokens in this invocation                                      */
  int32_t d;           /* hidden size                                                    */
  int32_t n_experts;   /* N: original experts                                            */
  int32_t n_sub;       /* S: sub-experts per expert (the paper's N of Sec. 3.2.1)        */
  int32_t inter_sub;   /* Is = I / S: intermediate neurons per sub-expert (C/N, Eq. 3)   */
  int32_t k_max;       /* largest budget a token may carry, in sub-expert units          */
  int32_t dtype;       /* MOE_PRISM_F32 or MOE_PRISM_BF16                                */
  int32_t renormalize; /* 1: softmax over the k_t selected; 0: softmax over all E        */
  float routed_scale;  /* multiplies every routing weight: S x the model's own factor    */
                       /* (the scaling by the split count that Sec. 3.2.2 prescribes)    */
} moe_prism_shape;

/* Bytes of workspace any entry point below needs for `shape` (host only). */
MOE_PRISM_API int moe_prism_workspace_bytes(const moe_prism_shape* shape, size_t* bytes);

/*
 * Sec. 3.3.1: every token inherits the budget of its request.
 * req_k[R], req_off[R+1] (token ranges, req_off[0] = 0, non-decreasing) ->
 * k_tok[req_off[R]].  R and T_total (= req_off[R], passed by the caller because
 * req_off lives on the device) are host values.
 */
MOE_PRISM_API int moe_prism_expand_k(int32_t R, int32_t T_total, const int32_t* req_k, const int32_t* req_off,
                       int32_t* k_tok, void* stream);

/*
 * Route (Sec. 3.2.2, expanded linear gate).
 *   logits[t,g] = sum_j x[t,j] * w_router[g,j] (+ router_bias[g]), computed as one
 *   binary32 fused-multiply-add chain per logit, j ascending, then one binary32 add
 *   of the bias: the routing decision is reproducible bit for bit.
 *   topk_ids[t, 0..k_t-1] = sub-experts with the k_t largest logits, ordered by
 *   logit descending, equal logits by id ascending; entries j >= k_t are -1.
 *   topk_w[t,j] = routed_scale * softmax weight of pick j (over the picks if
 *   renormalize, else over all E); entries j >= k_t are 0.
 * x [T,d], w_router [E,d] in shape->dtype; router_bias [E] fp32 or NULL;
 * k_tok [T]; topk_ids, topk_w [T,k_max]; logits_out [T,E] fp32 or NULL (then the
 * logits live in ws).  NaN logits are not supported.
 */
MOE_PRISM_API int moe_prism_route(const moe_prism_shape* shape, const void* x, const void* w_router,
                    const float* router_bias, const int32_t* k_tok, int32_t* topk_ids,
                    float* topk_w, float* logits_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Dispatch: the pairs (Sec. 2.1) grouped by sub-expert, without a sort.
 *   group_count[g]   = number of pairs routed to g
 *   group_offset[g]  = exclusive prefix; group_offset[E] = P = number of pairs
 *   sorted_pair[p]   = pair in slot p; group-major, token-ascending inside a group
 *                      (unique, since a token picks a sub-expert at most once);
 *                      -1 for p >= P
 *   slot_of_pair[q]  = slot of pair q, -1 if topk_ids[q] < 0
 * topk_ids [T,k_max] (ids in [-1, E)); group_count [E]; group_offset [E+1];
 * sorted_pair, slot_of_pair [T*k_max].
 */
MOE_PRISM_API int moe_prism_dispatch(const moe_prism_shape* shape, const int32_t* topk_ids, int32_t* group_count,
                       int32_t* group_offset, int32_t* sorted_pair, int32_t* slot_of_pair,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * Grouped SwiGLU FFN over the ragged groups (Sec. 3.2.1, Eq. 1-3 restricted to
 * one sub-expert's neurons).  For slot p of group g holding token t:
 *   h[c]   = SiLU(x[t,:] . Wg[g,c,:]) * (x[t,:] . Wu[g,c,:]),   c < Is
 *   y[p,q] = sum_c h[c] * Wd[g,q,c]
 * w_gate_up [E, 2*Is, d]: rows 0..Is-1 are the gate rows, Is..2Is-1 the up rows of
 * sub-expert g; w_down [E, d, Is].  y [T*k_max, d] in shape->dtype, rows >= P are
 * not written.  bf16: fp32 accumulation, h rounded to bf16 once, y rounded once.
 * Kernel choice (bf16): sub-experts with Is in {64, 128, 192} (and d >= 256) run one
 * fused kernel, all other shapes a gate-up and a down kernel.  Two environment
 * variables, read at every call, exist for A/B measurements and tests:
 * MOE_PRISM_FFN=split forces the two-kernel path, MOE_PRISM_FFN_K=32 its driver
 * with 32-element K stages.  Results agree within the rounding stated above.
 */
MOE_PRISM_API int moe_prism_grouped_ffn(const moe_prism_shape* shape, const void* x, const void* w_gate_up,
                          const void* w_down, const int32_t* group_offset,
                          const int32_t* sorted_pair, void* y, void* ws, size_t ws_bytes,
                          void* stream);

/*
 * Combine (Sec. 3.2.2, gate-weighted sum of the selected sub-expert outputs):
 *   out[t,:] = sum_{j < k_t} topk_w[t,j] * y[slot_of_pair[t*k_max+j], :]
 * j ascending, fp32 accumulation, one rounding to shape->dtype; k_t = 0 gives a
 * zero row.  No atomics: the result is bitwise reproducible.
 */
MOE_PRISM_API int moe_prism_combine(const moe_prism_shape* shape, const void* y, const int32_t* slot_of_pair,
                      const float* topk_w, const int32_t* k_tok, void* out, void* stream);

/*
 * The whole path route -> dispatch -> grouped FFN -> combine on one stream with
 * no host synchronisation; all intermediates live in ws.  out [T,d].
 * Stream capture: the first call of a kernel on a device raises that kernel's
 * dynamic-LDS limit (a runtime call that must not be recorded), so call the entry
 * point once eagerly on the device before capturing it into a HIP graph; afterwards
 * a call only launches kernels, and one captured graph serves any budget mix of the
 * same shape (sizes are read from device memory).
 */
MOE_PRISM_API int moe_prism_layer(const moe_prism_shape* shape, const void* x, const void* w_router,
                    const float* router_bias, const int32_t* k_tok, const void* w_gate_up,
                    const void* w_down, void* out, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_prism_layer for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, kernels and results as moe_prism_layer, but the intermediates live in a
 * device array of MOE_PRISM_STATIC_WS_BYTES that is part of the library's code object (one
 * copy per GPU, held until the process ends).  The call allocates and frees nothing.
 * Shapes whose moe_prism_workspace_bytes() exceeds MOE_PRISM_STATIC_WS_BYTES are refused
 * with MOE_PRISM_ERR_WORKSPACE before anything is launched.  Every call on a GPU uses
 * that GPU's one array (whatever the stream), which keeps the previous call's contents;
 * the kernels reset the words that must start at zero.  Calls that overlap in time on one
 * GPU race: order them on one stream or with events.  The status word of this variant
 * cannot be read back (budgets outside [0, k_max] are still clamped).
 */
#define MOE_PRISM_STATIC_WS_BYTES (64u << 20)
MOE_PRISM_API int moe_prism_layer_static(const moe_prism_shape* shape, const void* x,
                                         const void* w_router, const float* router_bias,
                                         const int32_t* k_tok, const void* w_gate_up,
                                         const void* w_down, void* out, void* stream);

/*
 * Proxy-gate route mode (Sec. 3.2.2, "Training-Free Proxy Gating"): routing for a model
 * refactored WITHOUT training a new gate.  The original router w_router0 [N, d] (+ bias0 [N]
 * or NULL) scores the N original experts and its native top m are taken, ordered by logit,
 * with weights w_j = softmax (renormalised over the m if shape->renormalize) x routed_scale.
 * For the expert ranked j its S = shape->n_sub sub-experts are scored by the mean absolute
 * SwiGLU activation of their r gate neurons, and the best kappa[k_t][j] of them are executed
 * (score descending, equal scores to the smaller index); every selected sub-expert inherits
 * w_j, so routed_scale is the original model's (no factor S).  topk_ids / topk_w are filled
 * like moe_prism_route's (flat ids e*S + n, appended in rank order, -1 / 0 padded), so
 * moe_prism_dispatch, _grouped_ffn and _combine follow unchanged.
 *
 *   w_proxy   [N, 2*rows_half, d], activation dtype: per original expert the gate rows of its
 *             gate neurons (neuron c of sub-expert n at row n*r + c), zero rows up to
 *             rows_half, then their up rows in the same order.  rows_half % 32 == 0,
 *             rows_half >= S*r.
 *   kappa     [(m*S + 1), m] int32, device: row k is the split (kappa_1..kappa_m) of budget k,
 *             0 <= kappa_j <= S, sum k.  Entries outside [0, S] are clamped.
 *   k_tok     [T] budgets in sub-expert units, 0 <= k_t <= min(k_max, m*S); others are clamped
 *             and flagged in the status word.
 * Requirements beyond moe_prism_shape's: m <= N, S <= 16, m*rows_half <= k_max*inter_sub,
 * T*m/256 + N <= T*k_max/256 + E (the stage shares the layer's tile table)
 * (MOE_PRISM_ERR_UNSUPPORTED_SHAPE otherwise).  Scores are taken from activations in the
 * activation dtype (bf16: rounded once) and summed in fp32.  Uses the logits, tile and
 * intermediate-activation regions of ws and the start of its y region as scratch: do not call
 * it between moe_prism_grouped_ffn and moe_prism_combine of the same workspace.
 */
MOE_PRISM_API int moe_prism_route_proxy(const moe_prism_shape* shape, const void* x,
                                        const void* w_router0, const float* router_bias0,
                                        const void* w_proxy, int32_t m, int32_t r,
                                        int32_t rows_half, const int32_t* kappa,
                                        const int32_t* k_tok, int32_t* topk_ids, float* topk_w,
                                        void* ws, size_t ws_bytes, void* stream);

/* moe_prism_layer with the proxy-gate route stage above in place of moe_prism_route. */
MOE_PRISM_API int moe_prism_layer_proxy(const moe_prism_shape* shape, const void* x,
                                        const void* w_router0, const float* router_bias0,
                                        const void* w_proxy, int32_t m, int32_t r,
                                        int32_t rows_half, const int32_t* kappa,
                                        const int32_t* k_tok, const void* w_gate_up,
                                        const void* w_down, void* out, void* ws, size_t ws_bytes,
                                        void* stream);

/*
 * Where moe_prism_layer keeps its intermediates inside ws (host only): byte
 * offsets of topk_ids, topk_w, group_count, group_offset, sorted_pair,
 * slot_of_pair, y, logits, in that order, into offsets[8].
 */
MOE_PRISM_API int moe_prism_layer_offsets(const moe_prism_shape* shape, size_t* offsets);

/*
 * Offline quality-tiered batching (Sec. 3.3.2, temporal separation; Eq. 5).  HOST ONLY: all
 * pointers are host pointers, nothing touches the GPU.
 *
 * The R waiting requests (arrival time, prompt tokens n_i > 0, budget k_i >= 0 in sub-expert
 * units) are sorted by (k, arrival, index) and cut into batches of at most M tokens, filled
 * strictly in that order.  A tier's under-filled last batch (n_cur tokens at budget k) is
 * promoted to the next tier's budget k_next and merged with it when
 *     (n_cur + n_next) * T(n_cur, k) >= n_cur * T(n_cur + n_next, k_next)      (binary64)
 * where n_next is the longest prefix of the next tier that fits in M - n_cur (none: no merge),
 * else it is dispatched at k.  A request longer than M forms a batch of its own.
 *
 *   table        T(n, k) in milliseconds on a grid: n_grid[n_n], k_grid[n_k] strictly
 *                ascending, ms[n_n * n_k] row-major in n; bilinear between grid points,
 *                constant outside (e.g. as printed by compare_modes --table).
 *   order        [R] out: request indices in dispatch order.
 *   batch_start  [R + 1] out: batch b is order[batch_start[b] .. batch_start[b+1]).
 *   batch_k      [R] out: the budget batch b runs at when the whole batch runs at one budget
 *                (its largest member budget).  With per-token budgets (moe_prism_layer) every
 *                request keeps its own k and batch_k is only the planner's accounting.
 *   n_batches    out.
 * Returns MOE_PRISM_OK or MOE_PRISM_ERR_INVALID_ARG.
 */
typedef struct {
  int32_t n_n, n_k;
  const int32_t* n_grid;
  const int32_t* k_grid;
  const float* ms;
} moe_prism_time_table;

MOE_PRISM_API int moe_prism_plan_batches(int32_t R, const double* arrival, const int32_t* n_tokens,
                                         const int32_t* k_qos, int32_t M,
                                         const moe_prism_time_table* table, int32_t* order,
                                         int32_t* batch_start, int32_t* batch_k,
                                         int32_t* n_batches);

/*
 * Partition solver (Sec. 3.2.1, "Partition Optimization Solver"; objective Eq. 4).  HOST ONLY,
 * offline.  A [B, C] fp32: calibration activations of one expert (B routed tokens, C intermediate
 * neurons); group_of [C]: the sub-expert (0..S-1) of every neuron; S <= 64, C % S == 0.
 * With L[b, n] = sum of |A[b, c]| over the neurons of group n (binary64, ascending c) the
 * objective for an inner budget k_in is  sum_b (sum of the S - k_in smallest L[b, .]).
 *   _greedy     neurons by descending calibration-wide L1 norm (equal norms: ascending index),
 *               each to the group with the smallest accumulated norm that still has room
 *               (equal sums: lower group).  Writes group_of.
 *   _objective  the loss of a given equal-sized partition.
 *   _anneal     `steps` proposals; proposal s swaps neurons r0 % C and r1 % C where
 *               r_i = splitmix64(seed + 3 s + i) (skipped if both are in one group); a swap that
 *               does not raise the loss is kept, one that raises it by D with probability
 *               exp(-D / temp), u = (r2 >> 11) * 2^-53, temp = t0 (t1/t0)^(s/(steps-1)).
 *               group_of is the starting partition on entry and the result on return;
 *               *loss_out (may be NULL) is its loss.
 * Returns MOE_PRISM_OK or MOE_PRISM_ERR_INVALID_ARG (including a group_of that is not an
 * equal-sized partition).
 */
MOE_PRISM_API int moe_prism_partition_greedy(int32_t B, int32_t C, int32_t S, const float* A,
                                             int32_t* group_of);
MOE_PRISM_API int moe_prism_partition_objective(int32_t B, int32_t C, int32_t S, int32_t k_in,
                                                const float* A, const int32_t* group_of,
                                                double* loss);
MOE_PRISM_API int moe_prism_partition_anneal(int32_t B, int32_t C, int32_t S, int32_t k_in,
                                             const float* A, int32_t* group_of, int64_t steps,
                                             double t0, double t1, uint64_t seed, double* loss_out);

/* Debug: synchronises `stream`, copies the status word to *host_flags and the
 * number of pairs of the last dispatch to *host_pairs (either may be NULL). */
MOE_PRISM_API int moe_prism_status(const void* ws, int32_t* host_flags, int32_t* host_pairs, void* stream);

/*
 * Per-kernel timing with HIP events recorded on the caller's stream.  While
 * enabled, every entry point brackets each kernel it launches with events.
 * moe_prism_timing_read synchronises on the recorded events, adds the elapsed
 * milliseconds of each kernel since the last reset into ms[MOE_PRISM_N_KERNELS]
 * (host), the launch counts into calls[...] (host), and resets.
 * moe_prism_timing_select restricts the bracketing to the kernels whose bit
 * (1 << MOE_PRISM_K_*) is set in kernel_mask (default: all), e.g. to time one
 * kernel inside a throughput measurement without event records around the rest.
 */
#define MOE_PRISM_K_LOGITS 0
#define MOE_PRISM_K_TOPK 1
#define MOE_PRISM_K_DISPATCH_COUNT 2
#define MOE_PRISM_K_DISPATCH_SCAN 3
#define MOE_PRISM_K_DISPATCH_PLACE 4
#define MOE_PRISM_K_FFN_TILES 5
#define MOE_PRISM_K_FFN_GATE_UP 6
#define MOE_PRISM_K_FFN_DOWN 7
#define MOE_PRISM_K_COMBINE 8
#define MOE_PRISM_K_PROXY_SELECT 9
#define MOE_PRISM_K_FFN_FUSED 10 /* gate-up + SwiGLU + down in one kernel (narrow sub-experts) */
#define MOE_PRISM_K_FFN_TRAFFIC 11 /* moe_prism_ffn_traffic_probe */
#define MOE_PRISM_N_KERNELS 12
MOE_PRISM_API int moe_prism_timing_enable(int on);
MOE_PRISM_API int moe_prism_timing_select(uint32_t kernel_mask);
MOE_PRISM_API int moe_prism_timing_read(float* ms, int32_t* calls);

/*
 * Machine-peak microbenchmarks (measurement only; no passage of the paper): what the
 * matrix cores (operands in registers / fed from LDS, constant and random bf16 data),
 * the LDS, the global->LDS and global->register paths (L2-, last-level-cache- and
 * HBM-sized footprints) and an HBM streaming copy deliver on the current device, in
 * loops shaped like the grouped-FFN kernels'.  Allocates and frees about 4 GiB of device
 * memory of its own, runs on the null stream and synchronises.  results[max_results]
 * (host) receives one record per test, *n_results (host) their number; shader_mhz is the
 * average shader clock during the test (0 where not measured).
 */
typedef struct {
  char name[64];
  char unit[16];
  double value;
  double shader_mhz;
} moe_prism_microbench_result;
MOE_PRISM_API int moe_prism_microbench(int32_t max_results, moe_prism_microbench_result* results,
                                       int32_t* n_results);

/*
 * Traffic probe of the fused grouped-FFN kernel (measurement only; no passage of the
 * paper).  Same arguments and checks as moe_prism_grouped_ffn; launches that kernel's
 * copies, barriers, waits, operand reads and output stores over the same tile table with
 * the matrix products left out, so its duration (kernel id MOE_PRISM_K_FFN_TRAFFIC) is the
 * time the kernel's memory traffic takes by itself.  The rows of y it writes hold no
 * meaningful values.  MOE_PRISM_ERR_UNSUPPORTED_SHAPE for shapes the fused kernel does not
 * serve (moe_prism_grouped_ffn runs its two-kernel path there).
 */
MOE_PRISM_API int moe_prism_ffn_traffic_probe(const moe_prism_shape* shape, const void* x,
                                              const void* w_gate_up, const void* w_down,
                                              const int32_t* group_offset,
                                              const int32_t* sorted_pair, void* y, void* ws,
                                              size_t ws_bytes, void* stream);

MOE_PRISM_API const char* moe_prism_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* MOE_PRISM_H */
