/*
 * libzeda: forward pass of one ZEDA dynamic-MoE layer on one MI355X (gfx950).
 *
 * The layer is the one of Section 2.1 ("Zero-Expert Injection"): a router scores N normal experts
 * and Z (= N_Z) parameter-free zero experts, the top-K set is taken over all N+Z candidates, and the
 * output is Eq. 1,
 *        y~(h) = sum over the selected NORMAL experts i of  g~_i(h) * E_i(h),
 * so that slots which land on a zero expert cost nothing.  Each normal expert is a gate, an up and a
 * down projection (Appendix D, Eq. 9: 6*H*H_e FLOPs per token and expert), read here as SwiGLU:
 *        E_i(h) = W_down[i] * ( silu(W_gate[i] h) .* (W_up[i] h) ).
 *
 * Conventions common to every entry point
 *   - Experts 0..N-1 are normal, N..N+Z-1 are zero experts (their router rows are appended to the
 *     original ones).  Z = 0 is the static top-K layer.
 *   - Every pointer is a DEVICE pointer owned by the caller, 16-byte aligned, unless it says "host".
 *     The library allocates nothing, frees nothing and never synchronises: all work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and the call returns.
 *   - Matrices are dense row-major with the reduction dimension contiguous:
 *     x[T,H], w_router[N+Z,H], w_gate[N,I,H], w_up[N,I,H], w_down[N,H,I], out[T,H]
 *     (the three expert tensors may instead be in the tiled layout, see zeda_weight_layout).
 *     Their element type is desc->dtype (fp32, or bf16 with fp32 accumulation).  Indices are int32,
 *     routing weights fp32.
 *   - Inputs are never written.  Outputs are fully overwritten.
 *   - Return value: ZEDA_OK, or a negative zeda_status.  Arguments are checked before anything is enqueued, so
 *     ZEDA_EINVAL, ZEDA_EUNSUPPORTED and ZEDA_EWORKSPACE mean that nothing ran.  ZEDA_EHIP reports a failed launch or
 *     runtime query; in an entry point that enqueues several kernels the earlier ones may already be on the stream
 *     (outputs are then undefined).
 *   - Calls that share a workspace or output buffer must be ordered by the caller (same stream).
 *   - Process state: none that a caller can observe, but launch geometry (workgroups the device holds at once) and the
 *     kernels' opt-in to more than 64 KiB of LDS are looked up on the first call of each kernel variant on each device
 *     and cached per device ordinal (up to 64 devices) for the life of the process.  Those first calls make runtime
 *     queries that are not allowed during stream capture: run every entry point once, eagerly, on the device and
 *     shape class that will be captured before capturing it into a HIP graph.  The calling thread's current device
 *     must be the one that owns the pointers and the stream.
 *
 * Shape limits (ZEDA_EUNSUPPORTED otherwise): 1 <= K <= min(N+Z, 16); N+Z <= 256;
 * T*K < 2^24; bf16: H % 128 == 0 and I % 64 == 0; fp32: H % 4 == 0, I % 4 == 0, H and I <= 12288.
 */
#ifndef ZEDA_H
#define ZEDA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZEDA_OK = 0,
    ZEDA_EINVAL = -1,       /* NULL required pointer, misaligned pointer, T<0, K<1, K>N+Z, N<1, Z<0, bad enum */
    ZEDA_EUNSUPPORTED = -2, /* valid layer, outside the shape limits above; tiled weights with fp32 */
    ZEDA_EWORKSPACE = -3,   /* workspace smaller than the matching *_workspace_bytes() */
    ZEDA_EHIP = -4          /* a kernel launch failed (hipGetLastError) */
} zeda_status;

typedef enum { ZEDA_F32 = 0, ZEDA_BF16 = 1 } zeda_dtype;

/* How the routing weight g~_i of a selected expert is formed from the softmax p over all N+Z logits.
 * Section 4.3.4: the weights of the surviving normal experts are not renormalised after the zero
 * experts are removed (TOPK_NORM, the default reading: normalised over all K selected slots, zero
 * experts included, then zero slots are dropped); Eq. 7 is the renormalised ablation. */
typedef enum {
    ZEDA_GATE_SOFTMAX = 0,    /* g = p_i                                                     */
    ZEDA_GATE_TOPK_NORM = 1,  /* g = p_i / sum of p over the K selected slots (default)      */
    ZEDA_GATE_REAL_RENORM = 2 /* g = p_i / sum of p over the selected normal experts (Eq. 7) */
} zeda_gate_norm;

/* Storage of the expert weights w_gate, w_up, w_down (the router weights are always row-major).
 * ZEDA_WEIGHTS_TILED is what zeda_pack_expert_weights writes: same size, 32x32 blocks laid out so that the
 * expert GEMM fetches them with long contiguous reads; weights are static, so they are packed once when
 * they are loaded.  bf16 only. */
typedef enum { ZEDA_WEIGHTS_ROW_MAJOR = 0, ZEDA_WEIGHTS_TILED = 1 } zeda_weight_layout;

/* What a parameter-free expert returns.  ZEDA_EXPERT_ZERO is the method's zero expert (Section 2.1): nothing.
 * ZEDA_EXPERT_COPY is the copy-expert variant of Appendix B, which returns its input, so the layer output gains
 * (sum of the routing weights of the token's slots on parameter-free experts) * h.  Either way such a slot
 * schedules no expert computation. */
typedef enum { ZEDA_EXPERT_ZERO = 0, ZEDA_EXPERT_COPY = 1 } zeda_free_expert_kind;

typedef struct {
    int32_t T;         /* tokens in this call                      */
    int32_t H;         /* hidden size                              */
    int32_t I;         /* expert intermediate size (H_e)           */
    int32_t N;         /* normal experts                           */
    int32_t Z;         /* zero experts (N_Z), may be 0             */
    int32_t K;         /* slots per token                          */
    int32_t dtype;     /* zeda_dtype of x, weights, out            */
    int32_t gate_norm; /* zeda_gate_norm                           */
    int32_t weight_layout; /* zeda_weight_layout of w_gate, w_up, w_down */
    int32_t free_expert;   /* zeda_free_expert_kind of experts N..N+Z-1  */
} zeda_layer_desc;

/* Short name of a status code (host pointer to a static string). */
const char *zeda_status_string(int status);

/* Host-only size queries; 0 if the descriptor is invalid or unsupported.
 * zeda_workspace_bytes covers zeda_moe_forward and is >= the other two. */
size_t zeda_workspace_bytes(const zeda_layer_desc *desc);
size_t zeda_route_workspace_bytes(const zeda_layer_desc *desc); /* may be 0: no scratch needed for this shape */
size_t zeda_dispatch_workspace_bytes(const zeda_layer_desc *desc);
size_t zeda_expert_ffn_workspace_bytes(const zeda_layer_desc *desc);

/* Section 2.1, router over the augmented pool E' = E u Z:
 *   logit[t,e] = <x[t,:], w_router[e,:]> (+ router_bias[e]),  e in [0, N+Z);
 *   topk_ids[t,0..K) = the K largest logits of token t in descending order (fp32 compare, ties to
 *   the lower index); topk_gates[t,j] = routing weight of that slot under desc->gate_norm.
 * router_bias[N+Z] (fp32) may be NULL (the paper's router has none).  T = 0 is a no-op.
 * ws: scratch of zeda_route_workspace_bytes(desc), or NULL.  With scratch, a layer with few tokens spreads the
 * projection of a token block over several workgroups (each a slice of the hidden dimension, summed in a fixed
 * order); without it one workgroup does a block alone.  The ids are the same either way; logits may differ in
 * the last bit between the two. */
int zeda_route(const zeda_layer_desc *desc, const void *x, const void *w_router, const float *router_bias,
               int32_t *topk_ids /*[T,K]*/, float *topk_gates /*[T,K]*/, void *ws, size_t ws_bytes, void *stream);

/* Zero-slot removal and expert-sorted order (Section 2.1: zero experts contribute no computation).
 * A slot s = t*K+j is real iff topk_ids[s] < N.  The real slots are listed grouped by expert, and
 * inside an expert by ascending s:
 *   expert_offsets[e] = first row of expert e, expert_offsets[N] = R = number of real slots;
 *   sorted_slot[r] = s for r < R (entries past R are left untouched);
 *   slot_to_row[s] = r, or -1 for a zero-expert slot;  num_real[0] = R  (r_ZE = 1 - R/(T*K)).
 * ws: zeda_dispatch_workspace_bytes(desc) bytes of scratch (per-segment counts for long slot lists; short lists
 * use none of it, the pointer must be valid all the same). */
int zeda_dispatch(const zeda_layer_desc *desc, const int32_t *topk_ids, int32_t *expert_offsets /*[N+1]*/,
                  int32_t *sorted_slot /*[T*K]*/, int32_t *slot_to_row /*[T*K]*/, int32_t *num_real /*[1]*/,
                  void *ws, size_t ws_bytes, void *stream);

/* zeda_dispatch for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and results as zeda_dispatch; the
 * scratch (the per-segment counts of long slot lists) is a 256 KiB array that the library itself holds in each
 * GPU's memory from load time to the end of the process.  The call allocates and frees nothing.
 * Limit: T*K <= zeda_dispatch_noalloc_max_slots() (524288), ZEDA_EUNSUPPORTED beyond it.
 * Nothing in the scratch has to start at zero (the counts a call reads are the ones it has just written).
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams,
 * different host threads) race; order them.  The array's device address is looked up on the first call on each
 * device (a runtime query: make that first call outside stream capture); ZEDA_EHIP if the lookup fails. */
int zeda_dispatch_noalloc_max_slots(void);
int zeda_dispatch_noalloc(const zeda_layer_desc *desc, const int32_t *topk_ids, int32_t *expert_offsets /*[N+1]*/,
                          int32_t *sorted_slot /*[T*K]*/, int32_t *slot_to_row /*[T*K]*/, int32_t *num_real /*[1]*/,
                          void *stream);

/* Grouped SwiGLU expert FFN over the real slots only (Appendix D, Eq. 10: 6*H*I FLOPs per real slot):
 *   y_slot[r,:] = E_e(x[sorted_slot[r] / K, :])  for expert_offsets[e] <= r < expert_offsets[e+1].
 * Work is launched for non-empty experts only.  y_slot has room for T*K rows of H elements of
 * desc->dtype; rows past R are not written.  num_real is read on the device (no host sync).
 * ws: scratch of zeda_expert_ffn_workspace_bytes(desc) (the activations silu(G).*U). */
int zeda_expert_ffn(const zeda_layer_desc *desc, const void *x, const void *w_gate, const void *w_up,
                    const void *w_down, const int32_t *expert_offsets, const int32_t *sorted_slot,
                    const int32_t *num_real, void *y_slot /*[T*K,H]*/, void *ws, size_t ws_bytes, void *stream);

/* Eq. 1, the weighted sum back in token order, with a fixed summation order and no atomics:
 *   out[t,:] = sum over j = 0..K-1 with topk_ids[t,j] < N of topk_gates[t,j] * y_slot[slot_to_row[t*K+j], :]
 * accumulated in fp32 in ascending j.  A token with no real slot gets exact zeros.
 * With desc->free_expert == ZEDA_EXPERT_COPY (Appendix B) the term (sum over j with N <= topk_ids[t,j] < N+Z of
 * topk_gates[t,j]) * x[t,:] is added last; x[T,H] is the layer input and is only read in that mode (NULL
 * otherwise is fine). */
int zeda_combine(const zeda_layer_desc *desc, const void *y_slot, const int32_t *topk_ids, const float *topk_gates,
                 const int32_t *slot_to_row, const void *x, void *out /*[T,H]*/, void *stream);

/* The whole layer: route -> dispatch -> expert FFN -> combine, all on `stream`.
 * num_real_out[0] (device, may be NULL) receives R (0 when T = 0, which enqueues nothing else).  ws: scratch of zeda_workspace_bytes(desc); after
 * the call it holds the intermediate results at the offsets zeda_workspace_layout reports. */
int zeda_moe_forward(const zeda_layer_desc *desc, const void *x, const void *w_router, const float *router_bias,
                     const void *w_gate, const void *w_up, const void *w_down, void *out /*[T,H]*/,
                     int32_t *num_real_out, void *ws, size_t ws_bytes, void *stream);

/* Same as zeda_moe_forward, and records caller-created hipEvent_t handles around the kernels:
 * events[0] before the first kernel, events[i] after stage i in the order of zeda_stage
 * (ZEDA_NUM_STAGES + 1 events; host array of handles).  For profiling only. */
enum {
    ZEDA_STAGE_ROUTE = 0,
    ZEDA_STAGE_DISPATCH = 1,
    ZEDA_STAGE_GATEUP = 2,
    ZEDA_STAGE_DOWN = 3,
    ZEDA_STAGE_COMBINE = 4,
    ZEDA_NUM_STAGES = 5
};
int zeda_moe_forward_events(const zeda_layer_desc *desc, const void *x, const void *w_router,
                            const float *router_bias, const void *w_gate, const void *w_up, const void *w_down,
                            void *out, int32_t *num_real_out, void *ws, size_t ws_bytes, void *stream,
                            void *const *events /* host: hipEvent_t[ZEDA_NUM_STAGES + 1] */);

/* Rewrites the expert weights of a layer from row-major into ZEDA_WEIGHTS_TILED (one-time, outside the hot
 * path; the layer of Section 2.1 does not depend on how its weights are stored).  For a matrix W[F][Kd]
 * (W_gate[e], W_up[e]: F = I, Kd = H; W_down[e]: F = H, Kd = I) the output holds (F/32) x (Kd/32) blocks of
 * 2 KiB, block (rb, kb) at index kb * (F/32) + rb; a block stores rows 32rb.., columns 32kb.. as 32 rows of
 * 64 bytes whose four 16-byte pieces are permuted: piece p of row r sits at position p ^ ((r >> 2) & 3).
 * Experts follow each other as in the input.  Any of the three pairs may be NULL/NULL (skipped); in and out
 * must not overlap.  desc->dtype must be bf16 (ZEDA_EUNSUPPORTED otherwise); desc->T and weight_layout are
 * ignored. */
int zeda_pack_expert_weights(const zeda_layer_desc *desc, const void *w_gate, const void *w_up, const void *w_down,
                             void *w_gate_tiled, void *w_up_tiled, void *w_down_tiled, void *stream);

/* Batch routing statistics of Section 2.2 for one layer, the T tokens of the call being the batch B (forward
 * values only; nothing is differentiated):
 *   f[i] = fraction of tokens whose top-K set holds expert i, P[i] = mean over tokens of the routing probability
 *   of expert i (softmax over all N+Z logits - the reading taken for "mean routing probability"), i in [0, N+Z);
 *   summary[0..6] = f_E, P_E, f_Z, P_Z (sums over the normal / the zero experts), r_ZE = f_Z / K,
 *   L_A = alpha (N+Z)/K sum_i f[i] P[i] (Eq. 4),  L_GA = alpha (N + Z w)/K (f_E P_E / N + f_Z P_Z / (Z w)) (Eq. 5-6;
 *   the zero-group term is dropped at Z = 0).
 * f, P, summary: device, fp32.  w > 0 is the group weight of Eq. 5.  T >= 1.  desc->gate_norm is not used.
 * ws: scratch of zeda_routing_stats_workspace_bytes(desc).  All sums run in a fixed order. */
size_t zeda_routing_stats_workspace_bytes(const zeda_layer_desc *desc);
int zeda_routing_stats(const zeda_layer_desc *desc, const void *x, const void *w_router, const float *router_bias,
                       float alpha, float w, float *f /*[N+Z]*/, float *P /*[N+Z]*/, float *summary /*[7]*/, void *ws,
                       size_t ws_bytes, void *stream);

/* Byte offsets inside the forward workspace (host-only).  Returns ZEDA_OK or an error. */
typedef struct {
    size_t topk_ids, topk_gates, expert_offsets, sorted_slot, slot_to_row, num_real, dispatch_ws, act, y_slot, route_ws,
        total;
} zeda_ws_layout;
int zeda_workspace_layout(const zeda_layer_desc *desc, zeda_ws_layout *layout /* host */);

/* Token-level zero-expert usage (Section 4.1, "Zero Expert Activation Dynamics": different tokens have different
 * r_ZE): zero_slots[t] = number of the K slots of token t that landed on a zero expert (topk_ids[t,j] >= N), so a
 * token's r_ZE in this layer is zero_slots[t] / K.  accumulate != 0 adds the counts to what zero_slots already
 * holds instead of overwriting it: summed over the L layers of a model, zero_slots[t] / (L*K) is the token's r_ZE
 * over the model.  topk_ids: [T,K] device, as written by zeda_route (the forward workspace holds it at
 * zeda_ws_layout.topk_ids).  zero_slots: int32[T] device.  T = 0 is a no-op.  ZEDA_EINVAL on NULL / unaligned
 * pointers. */
int zeda_token_zero_slots(const zeda_layer_desc *desc, const int32_t *topk_ids, int32_t *zero_slots, int accumulate,
                          void *stream);

/* Router rows of the zero experts (Section 2.1, "router initialization"; a model-surgery step, not on the hot
 * path).  w_router[N+Z, H]: rows 0..N-1 (the post-trained router) are read and kept; rows N..N+Z-1 are written
 * as mean + std * normals[z, h], mean and (population) variance taken over the N*H original parameters.
 * normals[Z, H]: fp32 standard-normal draws supplied by the caller (device).  stats (device, may be NULL)
 * receives {mean, variance} as fp32.  desc->T is ignored.  One workgroup, deterministic. */
int zeda_init_zero_expert_rows(const zeda_layer_desc *desc, void *w_router, const float *normals, float *stats,
                               void *stream);

/* Glue of the layer-stack workload x <- x + MoE_l(RMSNorm(x)) (no attention).  Not part of the paper's layer
 * (Appendix D leaves norms and residuals out of its model); used to chain 48 layers with and without zero
 * experts.  x, out, y: [T,H] of `dtype` (zeda_dtype); arithmetic in fp32.
 *   zeda_rmsnorm:       out[t,:] = x[t,:] / sqrt(mean(x[t,:]^2) + eps) * gamma   (gamma[H] may be NULL = 1)
 *   zeda_residual_add:  x += y  (in place)
 * ZEDA_EINVAL on NULL pointers, bad dtype, T < 0, H < 1, eps < 0. */
int zeda_rmsnorm(int32_t T, int32_t H, int32_t dtype, const void *x, const void *gamma, float eps, void *out, void *stream);
int zeda_residual_add(int32_t T, int32_t H, int32_t dtype, void *x, const void *y, void *stream);

/* One pre-norm residual block of that chain in a single call: the layer of Eq. 1 (Section 2.1) applied to the
 * normalised input xn, with the weighted sum of Eq. 1 added straight into the residual stream,
 *   x_res[t,:] <- x_res[t,:] + sum_i g~_i E_i(xn[t,:])          (in place, rounded to the element type)
 *   xn_next[t,:] = RMSNorm(x_res[t,:]) * gamma_next             (of the stored row; skipped if xn_next is NULL)
 * so that the combine stage replaces zeda_combine + zeda_residual_add + the next layer's zeda_rmsnorm.  The sum
 * is added in fp32 before the one rounding, i.e. without the intermediate rounding of a separate layer output.
 * All other arguments, the workspace and the stage order are those of zeda_moe_forward.  xn, x_res, xn_next:
 * [T,H] device; xn_next may be the same buffer as xn (each row is read before it is written); x_res must be
 * distinct from both.  gamma_next[H] device or NULL (= 1).  H <= 8192 (bf16) / 4096 (fp32), else
 * ZEDA_EUNSUPPORTED.  ZEDA_EINVAL on NULL / unaligned pointers, eps < 0, or x_res aliasing xn or xn_next. */
int zeda_moe_block_forward(const zeda_layer_desc *desc, const void *xn, void *x_res, const void *w_router,
                           const float *router_bias, const void *w_gate, const void *w_up, const void *w_down,
                           const void *gamma_next, float eps, void *xn_next, int32_t *num_real_out, void *ws,
                           size_t ws_bytes, void *stream);

/* Measurement aid, not part of the layer: reads `bytes` bytes of device memory at `buf` once, every workgroup a
 * contiguous 256 KiB run with 16-byte loads - the plainest streaming read there is.  Its rate on a buffer larger than
 * the caches is what HBM delivers to a kernel that does nothing else on this machine, the yardstick beside which
 * bench.py reports the rates of the HBM-bound expert GEMMs (the published 8 TB/s is not reached by any read
 * pattern).  Nothing is written unless the XOR of all words read equals an arbitrary constant, in which case one
 * word is stored to sink (device, 4 bytes; exists so that the loads cannot be dropped).  buf 16-byte aligned,
 * bytes a multiple of 16.  ZEDA_EINVAL on NULL / unaligned arguments; bytes == 0 launches nothing. */
int zeda_stream_read_probe(const void *buf, size_t bytes, void *sink, void *stream);

/* Measurement aid, not part of the layer: `workgroups` workgroups of four waves each issue iters * 8 independent
 * 32x32x16 bf16 MFMAs (fp32 accumulators, operands held in registers, no memory traffic at all): the rate of
 * 2 * 32*32*16 * 8 * iters * 4 * workgroups FLOPs over the launch is what the matrix units deliver on this machine when
 * nothing else competes for power or issue slots - the yardstick beside which bench.py reports the compute-heavy
 * expert GEMMs.  The accumulators are summed into sink[workgroup * 256 + thread] (device, workgroups * 256 floats) so
 * that the work cannot be dropped.  ZEDA_EINVAL on NULL / unaligned sink, iters < 1, workgroups < 1. */
int zeda_mfma_probe(int workgroups, int iters, float *sink, void *stream);

/* Measurement aid, not part of the layer: both of the above in ONE kernel, to see how far a CU overlaps HBM
 * streaming with matrix work and whether that depends on which waves do what.  Workgroups of eight waves, one per
 * CU at a time (the hardware places wave w of a workgroup on SIMD w % 4); every workgroup owns 1 MiB of buf, which
 * its reading waves read once (16-byte loads, 64 KiB in flight), while each of its multiplying waves issues
 * mfmas_per_wave independent 32x32x16 bf16 MFMAs on register operands.
 *   mode & ZEDA_PROBE_READ / ZEDA_PROBE_MFMA: which of the two parts runs (at least one; the waves of a part that is
 *     switched off exit at once).
 *   mode & ZEDA_PROBE_SPLIT_SIMD clear: waves 0-3 read and waves 4-7 multiply - every SIMD holds a wave of each kind.
 *   mode & ZEDA_PROBE_SPLIT_SIMD set:   waves 3 and 7 (SIMD 3) read and the six others multiply - no SIMD holds both.
 * bytes: a multiple of 1 MiB (bytes / 1 MiB workgroups); mfmas_per_wave >= 0, rounded down to a multiple of 8.
 * sink: device, 8-byte aligned, (bytes / 1 MiB) * 512 floats followed by 8 more words: one that is only written if
 * the XOR of all words read equals an arbitrary constant, one unused, and two int64 - shader-clock cycles and ticks
 * of the constant 100 MHz counter that one wave of the workgroup in the middle of the grid counted around its own
 * work (100 * cycles / ticks = the shader clock in MHz while the kernel ran).  Timed in its three parts on the same
 * buffer, `both` = max(read, mfma) would be perfect overlap and `both` = read + mfma none at all; bench.py reports
 * the times for both placements.  ZEDA_EINVAL on NULL / unaligned pointers, bytes not a multiple of 1 MiB, a mode
 * without a part or outside 1..7, mfmas_per_wave < 0. */
enum { ZEDA_PROBE_READ = 1, ZEDA_PROBE_MFMA = 2, ZEDA_PROBE_SPLIT_SIMD = 4 };
int zeda_overlap_probe(const void *buf, size_t bytes, int mfmas_per_wave, int mode, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ZEDA_H */
