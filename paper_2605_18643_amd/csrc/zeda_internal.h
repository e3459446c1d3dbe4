// Internal declarations shared by the translation units of libzeda (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "zeda.h"

namespace zeda {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kMaxExperts = 256;  // N + Z
constexpr int kMaxK = 16;

constexpr int kMaxDevices = 64;   // launch geometry and kernel attributes are cached per device ordinal below this

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
// ordinal of the calling thread's current device, or -1 (no device, or an ordinal past kMaxDevices)
inline int current_device()
{
    int dev = 0;
    return (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) ? dev : -1;
}
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

int check_desc(const zeda_layer_desc *d);  // ZEDA_OK / ZEDA_EINVAL / ZEDA_EUNSUPPORTED
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elt_size(const zeda_layer_desc *d) { return d->dtype == ZEDA_BF16 ? 2 : 4; }

// stage launchers: arguments are already validated; each returns ZEDA_OK or ZEDA_EHIP
// partial: scratch of route_ws_bytes(d) for the split-k launch, or NULL (one kernel, no scratch)
// cnt8: route_counts_bytes(d) of scratch that receives the per-block expert counts, or NULL (bf16 only)
int launch_route(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias, int32_t *ids,
                 float *gates, float *partial, uint8_t *cnt8, hipStream_t s);
size_t route_ws_bytes(const zeda_layer_desc *d);
// Per-block expert counts of the bf16 router: cnt8 [N+Z][route_counts_ld(d)] bytes receive, per block of 16 tokens,
// the number of slots on every expert - what launch_dispatch_counts starts from.
bool route_counts_supported(const zeda_layer_desc *d);
int route_counts_ld(const zeda_layer_desc *d);
size_t route_counts_bytes(const zeda_layer_desc *d);
// expert-sorted placement that starts from those per-block counts instead of counting the ids again
bool dispatch_counts_supported(const zeda_layer_desc *d);
int launch_dispatch_counts(const zeda_layer_desc *d, const int32_t *ids, const uint8_t *cnt8, int32_t *offsets,
                           int32_t *sorted_slot, int32_t *slot_to_row, int32_t *num_real, int32_t *num_real_copy,
                           hipStream_t s);
// Section 2.2 statistics over the batch of all T tokens (f, P: [N+Z]; summary: 7 floats); ws of routing_stats_ws_bytes
int launch_routing_stats(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias, float alpha, float w,
                         float *f, float *P, float *summary, void *ws, hipStream_t s);
size_t routing_stats_ws_bytes(const zeda_layer_desc *d);
// num_real_copy (may be NULL) receives num_real as well; ws: dispatch_ws_bytes(d) of scratch
int launch_dispatch(const zeda_layer_desc *d, const int32_t *ids, int32_t *offsets, int32_t *sorted_slot,
                    int32_t *slot_to_row, int32_t *num_real, int32_t *num_real_copy, void *ws, hipStream_t s);
size_t dispatch_ws_bytes(const zeda_layer_desc *d);
// scratch held by the library itself (a file-scope device array) for zeda_dispatch_noalloc
void *dispatch_static_scratch();          // its address on the current device, NULL if the lookup fails
size_t dispatch_static_scratch_bytes();
int dispatch_static_max_slots();          // slot lists up to this length are accepted by that entry point
int launch_gateup(const zeda_layer_desc *d, const void *x, const void *wg, const void *wu, const int32_t *offsets,
                  const int32_t *sorted_slot, void *act, hipStream_t s);
int launch_down(const zeda_layer_desc *d, const void *act, const void *wd, const int32_t *offsets, void *y_slot,
                hipStream_t s);
// row-major -> tiled copy of one expert weight tensor (down: [N,H,I], else [N,I,H])
int launch_pack_weights(const zeda_layer_desc *d, const void *w, void *out, bool down, hipStream_t s);
int launch_combine(const zeda_layer_desc *d, const void *y_slot, const int32_t *ids, const float *gates,
                   const int32_t *slot_to_row, const void *x, void *out, hipStream_t s);

// combine fused with the pre-norm residual block: x_res += MoE output; xn_next (may be NULL) = RMSNorm(x_res) * gamma
bool combine_block_supported(const zeda_layer_desc *d);
int launch_combine_block(const zeda_layer_desc *d, const void *y_slot, const int32_t *ids, const float *gates,
                         const int32_t *slot_to_row, const void *x, void *x_res, const void *gamma, float eps,
                         void *xn_next, hipStream_t s);

inline int last_launch_status() { return hipGetLastError() == hipSuccess ? ZEDA_OK : ZEDA_EHIP; }

}  // namespace zeda
