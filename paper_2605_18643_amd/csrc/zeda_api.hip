// C ABI of libzeda: argument validation, workspace carving and the order of the launches.
// The layer is Eq. 1 of Section 2.1; see include/zeda.h for the meaning of every argument.
#include "zeda_internal.h"

namespace zeda {

int check_desc(const zeda_layer_desc *d)
{
    if (!d) return ZEDA_EINVAL;
    if (d->T < 0 || d->H < 1 || d->I < 1 || d->N < 1 || d->Z < 0 || d->K < 1) return ZEDA_EINVAL;
    if ((int64_t)d->K > (int64_t)d->N + d->Z) return ZEDA_EINVAL;
    if (d->dtype != ZEDA_F32 && d->dtype != ZEDA_BF16) return ZEDA_EINVAL;
    if (d->gate_norm < ZEDA_GATE_SOFTMAX || d->gate_norm > ZEDA_GATE_REAL_RENORM) return ZEDA_EINVAL;
    if (d->weight_layout != ZEDA_WEIGHTS_ROW_MAJOR && d->weight_layout != ZEDA_WEIGHTS_TILED) return ZEDA_EINVAL;
    if (d->free_expert != ZEDA_EXPERT_ZERO && d->free_expert != ZEDA_EXPERT_COPY) return ZEDA_EINVAL;
    if ((int64_t)d->N + d->Z > kMaxExperts || d->K > kMaxK) return ZEDA_EUNSUPPORTED;
    if ((int64_t)d->T * d->K >= (1 << 24)) return ZEDA_EUNSUPPORTED;
    if (d->dtype == ZEDA_BF16) {
        if (d->H % 128 != 0 || d->I % 64 != 0) return ZEDA_EUNSUPPORTED;
    } else {
        if (d->weight_layout != ZEDA_WEIGHTS_ROW_MAJOR) return ZEDA_EUNSUPPORTED;
        if (d->H % 4 != 0 || d->I % 4 != 0 || d->H > 12288 || d->I > 12288) return ZEDA_EUNSUPPORTED;
    }
    return ZEDA_OK;
}

static size_t act_bytes(const zeda_layer_desc *d)
{
    return align_up((size_t)d->T * d->K * d->I * elt_size(d), 256);
}

// The whole-layer call has the router leave per-block expert counts and places from them, where both apply.
static bool fused_counts(const zeda_layer_desc *d) { return route_counts_supported(d) && dispatch_counts_supported(d); }
static size_t fused_counts_bytes(const zeda_layer_desc *d) { return fused_counts(d) ? route_counts_bytes(d) : 0; }

static void layout_of(const zeda_layer_desc *d, zeda_ws_layout *L)
{
    const size_t S = (size_t)d->T * d->K;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes ? bytes : 1, 256); return at; };
    L->topk_ids = take(S * 4);
    L->topk_gates = take(S * 4);
    L->expert_offsets = take((size_t)(d->N + 1) * 4);
    L->sorted_slot = take(S * 4);
    L->slot_to_row = take(S * 4);
    L->num_real = take(4);
    // (the whole-layer call keeps the router's per-block counts here when it uses them instead of the counting pass)
    L->dispatch_ws = take(dispatch_ws_bytes(d) > fused_counts_bytes(d) ? dispatch_ws_bytes(d) : fused_counts_bytes(d));
    L->act = take(act_bytes(d));
    L->y_slot = take(S * d->H * elt_size(d));
    L->route_ws = take(route_ws_bytes(d));
    L->total = o;
}

// one int32 written on the stream (a kernel rather than a memset node, so that captured graphs replay it reliably)
__global__ void store_i32_kernel(int32_t *p, int32_t v) { *p = v; }

// Tail of the pre-norm residual block variant: the combine adds into x_res and writes the next layer's input.
struct BlockTail {
    void *x_res;
    const void *gamma;
    float eps;
    void *xn_next;
};

// out: the layer output, or NULL when tail is given
static int forward_impl(const zeda_layer_desc *desc, const void *x, const void *w_router, const float *router_bias,
                        const void *w_gate, const void *w_up, const void *w_down, void *out, int32_t *num_real_out,
                        void *ws, size_t ws_bytes, void *stream, void *const *events, const BlockTail *tail = nullptr)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    if (!x || !w_router || !w_gate || !w_up || !w_down || !ws) return ZEDA_EINVAL;
    if (!aligned16(x) || !aligned16(w_router) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) ||
        !aligned16(ws) || (router_bias && !aligned16(router_bias)))
        return ZEDA_EINVAL;
    if (tail) {
        if (!tail->x_res || !aligned16(tail->x_res) || !aligned16(tail->gamma) || !aligned16(tail->xn_next) ||
            !(tail->eps >= 0.f) || tail->x_res == x || tail->x_res == tail->xn_next)
            return ZEDA_EINVAL;
        if (!combine_block_supported(desc)) return ZEDA_EUNSUPPORTED;
    } else if (!out || !aligned16(out)) {
        return ZEDA_EINVAL;
    }
    zeda_ws_layout L;
    layout_of(desc, &L);
    if (ws_bytes < L.total) return ZEDA_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char *w = (char *)ws;
    int32_t *ids = (int32_t *)(w + L.topk_ids);
    float *gates = (float *)(w + L.topk_gates);
    int32_t *offsets = (int32_t *)(w + L.expert_offsets);
    int32_t *sorted_slot = (int32_t *)(w + L.sorted_slot);
    int32_t *slot_to_row = (int32_t *)(w + L.slot_to_row);
    int32_t *num_real = (int32_t *)(w + L.num_real);
    void *act = w + L.act;
    void *y_slot = w + L.y_slot;
    float *route_ws = route_ws_bytes(desc) ? (float *)(w + L.route_ws) : nullptr;

    auto mark = [&](int i) {
        if (events && hipEventRecord((hipEvent_t)events[i], s) != hipSuccess) rc = ZEDA_EHIP;
    };
    mark(0);
    if (desc->T == 0) {  // no token: nothing to route, R = 0
        if (num_real_out) {
            store_i32_kernel<<<1, 1, 0, s>>>(num_real_out, 0);
            if (last_launch_status() != ZEDA_OK) return ZEDA_EHIP;
        }
        for (int i = 1; i <= ZEDA_NUM_STAGES; ++i) mark(i);
        return rc;
    }
    if (fused_counts(desc)) {
        uint8_t *cnt8 = (uint8_t *)(w + L.dispatch_ws);
        if ((rc = launch_route(desc, x, w_router, router_bias, ids, gates, route_ws, cnt8, s)) != ZEDA_OK) return rc;
        mark(1 + ZEDA_STAGE_ROUTE);
        if ((rc = launch_dispatch_counts(desc, ids, cnt8, offsets, sorted_slot, slot_to_row, num_real, num_real_out, s)) != ZEDA_OK) return rc;
    } else {
        if ((rc = launch_route(desc, x, w_router, router_bias, ids, gates, route_ws, nullptr, s)) != ZEDA_OK) return rc;
        mark(1 + ZEDA_STAGE_ROUTE);
        if ((rc = launch_dispatch(desc, ids, offsets, sorted_slot, slot_to_row, num_real, num_real_out, w + L.dispatch_ws, s)) != ZEDA_OK) return rc;
    }
    mark(1 + ZEDA_STAGE_DISPATCH);
    if ((rc = launch_gateup(desc, x, w_gate, w_up, offsets, sorted_slot, act, s)) != ZEDA_OK) return rc;
    mark(1 + ZEDA_STAGE_GATEUP);
    if ((rc = launch_down(desc, act, w_down, offsets, y_slot, s)) != ZEDA_OK) return rc;
    mark(1 + ZEDA_STAGE_DOWN);
    rc = tail ? launch_combine_block(desc, y_slot, ids, gates, slot_to_row, x, tail->x_res, tail->gamma, tail->eps,
                                     tail->xn_next, s)
              : launch_combine(desc, y_slot, ids, gates, slot_to_row, x, out, s);
    if (rc != ZEDA_OK) return rc;
    mark(1 + ZEDA_STAGE_COMBINE);
    return rc;
}

// zeda_token_zero_slots: one thread per token walks its K ids
__global__ __launch_bounds__(256) void token_zero_slots_kernel(const int32_t *__restrict__ ids, int T, int K, int N,
                                                               int32_t *__restrict__ zero_slots, int accumulate)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    int c = 0;
    for (int j = 0; j < K; ++j) c += ids[(size_t)t * K + j] >= N;
    zero_slots[t] = accumulate ? zero_slots[t] + c : c;
}

// Plain streaming read (zeda_stream_read_probe): a workgroup reads one contiguous run of kProbeRun bytes, four
// 16-byte loads per lane in flight.
constexpr size_t kProbeRun = 256 * 1024;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *__restrict__ p, size_t n16, uint32_t *__restrict__ sink)
{
    constexpr size_t per_wg = kProbeRun / 16;
    const size_t lo = (size_t)blockIdx.x * per_wg, hi = lo + per_wg < n16 ? lo + per_wg : n16;
    u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = lo + threadIdx.x;
    for (; i + 768 < hi; i += 1024) {
        const u32x4 a = p[i], b = p[i + 256], c = p[i + 512], d = p[i + 768];
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < hi; i += 256) acc ^= p[i];
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x5eda5edau && (acc[0] + acc[1]) == 0x0badcafeu) *sink = acc[2];
}

static int launch_stream_read(const void *buf, size_t bytes, uint32_t *sink, hipStream_t s)
{
    const size_t n16 = bytes / 16, grid = (bytes + kProbeRun - 1) / kProbeRun;
    if (grid > 0x7fffffffu) return ZEDA_EUNSUPPORTED;
    stream_read_kernel<<<(unsigned)grid, 256, 0, s>>>((const u32x4 *)buf, n16, sink);
    return last_launch_status();
}

// zeda_mfma_probe: eight independent accumulator blocks per wave, the same two operand fragments every time
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *__restrict__ sink, int iters)
{
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t h = (threadIdx.x * 8u + i) * 2654435761u;  // fixed pseudo-random operands in (-1, 1)
        a[i] = (bf16_t)(((h >> 8) & 0xffff) / 32768.0f - 1.0f);
        b[i] = (bf16_t)(((h >> 16) & 0xffff) / 32768.0f - 1.0f);
    }
    f32x16 acc[8];
#pragma unroll
    for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 8; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[n][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// zeda_overlap_probe.  Waves go to the four SIMDs of a CU round-robin (wave w runs on SIMD w % 4).  SPLIT false: waves
// 0-3 stream, waves 4-7 multiply, so every SIMD holds one wave of each kind.  SPLIT true: waves 3 and 7 (SIMD 3) stream,
// the six others multiply, so no SIMD holds both kinds.  The readers keep the same number of bytes in flight per
// workgroup either way (64 KiB).  96 KiB of LDS that nobody touches hold the kernel to one workgroup per CU in every mode.
constexpr size_t kOverlapChunk = 1 << 20;
constexpr int kOverlapLds = 96 * 1024;
template <bool READ, bool MFMA, bool SPLIT>
__global__ __launch_bounds__(512) void overlap_probe_kernel(const u32x4 *__restrict__ p, int mfmas, float *__restrict__ sink,
                                                            uint32_t *__restrict__ usink)
{
    extern __shared__ unsigned char overlap_pad[];
    if (mfmas < 0) overlap_pad[threadIdx.x] = 1;  // (never: keeps the allocation)
    constexpr int RT = SPLIT ? 128 : 256;  // reading threads
    constexpr int NLD = SPLIT ? 32 : 16;   // 16-byte loads of a lane in flight
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool reader = SPLIT ? (wave & 3) == 3 : wave < 4;
    const int rtid = SPLIT ? (wave >> 2) * 64 + lane : (int)threadIdx.x;
    // one wave of each kind in the workgroup in the middle of the grid reads the cycle counter and the 100 MHz counter
    // around its work (readers report if there are readers, else the multiplying wave does)
    const bool rec = blockIdx.x == (gridDim.x >> 1) && lane == 0 && (READ ? (reader && rtid == 0) : wave == (SPLIT ? 0 : 4));
    long long c0 = 0, r0 = 0;
    if (blockIdx.x == (gridDim.x >> 1)) {
        c0 = __builtin_amdgcn_s_memtime();
        r0 = __builtin_amdgcn_s_memrealtime();
    }
    long long *clk = reinterpret_cast<long long *>(usink + 2);
    if (reader) {
        if (!READ) return;
        constexpr size_t chunk16 = kOverlapChunk / 16;
        static_assert(chunk16 % (NLD * RT) == 0, "a workgroup's loads stay inside its MiB");
        const u32x4 *q = p + (size_t)blockIdx.x * chunk16;
        u32x4 acc = {0u, 0u, 0u, 0u};
        for (size_t i = rtid; i < chunk16; i += NLD * RT) {
            u32x4 v[NLD];
#pragma unroll
            for (int u = 0; u < NLD; ++u) v[u] = q[i + u * RT];
#pragma unroll
            for (int u = 0; u < NLD; ++u) acc ^= v[u];
        }
        if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x5eda5edau && (acc[0] + acc[1]) == 0x0badcafeu) *usink = acc[2];
        if (rec) {
            clk[0] = __builtin_amdgcn_s_memtime() - c0 + (long long)(acc[0] & 0u);  // (after the loads have landed)
            clk[1] = __builtin_amdgcn_s_memrealtime() - r0;
        }
    } else {
        if (!MFMA) return;
        bf16x8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t h = (threadIdx.x * 8u + i) * 2654435761u;
            a[i] = (bf16_t)(((h >> 8) & 0xffff) / 32768.0f - 1.0f);
            b[i] = (bf16_t)(((h >> 16) & 0xffff) / 32768.0f - 1.0f);
        }
        f32x16 acc[8];
#pragma unroll
        for (int n = 0; n < 8; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
        for (int it = 0; it < mfmas / 8; ++it) {
#pragma unroll
            for (int n = 0; n < 8; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
        }
        float s = 0.f;
#pragma unroll
        for (int n = 0; n < 8; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[n][v];
        sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
        if (rec) {
            clk[0] = __builtin_amdgcn_s_memtime() - c0 + (long long)(s != s ? 1 : 0);  // (after the MFMAs have finished)
            clk[1] = __builtin_amdgcn_s_memrealtime() - r0;
        }
    }
}

template <bool READ, bool MFMA, bool SPLIT>
static int launch_overlap_probe(const u32x4 *p, size_t grid, int mfmas, float *sink, uint32_t *usink, hipStream_t s)
{
    static bool done[kMaxDevices] = {};  // per instantiation and device (idempotent)
    const int dev = current_device();
    if (dev < 0) return ZEDA_EHIP;
    if (!done[dev]) {
        if (hipFuncSetAttribute((const void *)overlap_probe_kernel<READ, MFMA, SPLIT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kOverlapLds) != hipSuccess)
            return ZEDA_EHIP;
        done[dev] = true;
    }
    overlap_probe_kernel<READ, MFMA, SPLIT><<<(unsigned)grid, 512, kOverlapLds, s>>>(p, mfmas, sink, usink);
    return last_launch_status();
}

}  // namespace zeda

using namespace zeda;

extern "C" {

const char *zeda_status_string(int status)
{
    switch (status) {
        case ZEDA_OK: return "ZEDA_OK";
        case ZEDA_EINVAL: return "ZEDA_EINVAL";
        case ZEDA_EUNSUPPORTED: return "ZEDA_EUNSUPPORTED";
        case ZEDA_EWORKSPACE: return "ZEDA_EWORKSPACE";
        case ZEDA_EHIP: return "ZEDA_EHIP";
        default: return "ZEDA_UNKNOWN";
    }
}

size_t zeda_workspace_bytes(const zeda_layer_desc *desc)
{
    if (check_desc(desc) != ZEDA_OK) return 0;
    zeda_ws_layout L;
    layout_of(desc, &L);
    return L.total;
}

size_t zeda_dispatch_workspace_bytes(const zeda_layer_desc *desc)
{
    if (check_desc(desc) != ZEDA_OK) return 0;
    return dispatch_ws_bytes(desc);
}

size_t zeda_expert_ffn_workspace_bytes(const zeda_layer_desc *desc)
{
    if (check_desc(desc) != ZEDA_OK) return 0;
    return act_bytes(desc);
}

int zeda_workspace_layout(const zeda_layer_desc *desc, zeda_ws_layout *layout)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    if (!layout) return ZEDA_EINVAL;
    layout_of(desc, layout);
    return ZEDA_OK;
}

size_t zeda_route_workspace_bytes(const zeda_layer_desc *desc)
{
    if (check_desc(desc) != ZEDA_OK) return 0;
    return route_ws_bytes(desc);
}

int zeda_route(const zeda_layer_desc *desc, const void *x, const void *w_router, const float *router_bias,
               int32_t *topk_ids, float *topk_gates, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    if (!x || !w_router || !topk_ids || !topk_gates) return ZEDA_EINVAL;
    if (!aligned16(x) || !aligned16(w_router) || !aligned16(topk_ids) || !aligned16(topk_gates) ||
        (router_bias && !aligned16(router_bias)) || (ws && !aligned16(ws)))
        return ZEDA_EINVAL;
    if (ws && ws_bytes < route_ws_bytes(desc)) return ZEDA_EWORKSPACE;
    if (desc->T == 0) return ZEDA_OK;
    float *partial = (ws && route_ws_bytes(desc)) ? (float *)ws : nullptr;
    return launch_route(desc, x, w_router, router_bias, topk_ids, topk_gates, partial, nullptr, (hipStream_t)stream);
}

int zeda_dispatch(const zeda_layer_desc *desc, const int32_t *topk_ids, int32_t *expert_offsets, int32_t *sorted_slot,
                  int32_t *slot_to_row, int32_t *num_real, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    if (!topk_ids || !expert_offsets || !sorted_slot || !slot_to_row || !num_real || !ws) return ZEDA_EINVAL;
    if (!aligned16(topk_ids) || !aligned16(expert_offsets) || !aligned16(sorted_slot) || !aligned16(slot_to_row) ||
        !aligned16(ws) || (reinterpret_cast<uintptr_t>(num_real) & 3u))
        return ZEDA_EINVAL;
    if (ws_bytes < dispatch_ws_bytes(desc)) return ZEDA_EWORKSPACE;
    return launch_dispatch(desc, topk_ids, expert_offsets, sorted_slot, slot_to_row, num_real, nullptr, ws,
                           (hipStream_t)stream);
}

int zeda_dispatch_noalloc_max_slots(void) { return dispatch_static_max_slots(); }

int zeda_dispatch_noalloc(const zeda_layer_desc *desc, const int32_t *topk_ids, int32_t *expert_offsets,
                          int32_t *sorted_slot, int32_t *slot_to_row, int32_t *num_real, void *stream)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    if (!topk_ids || !expert_offsets || !sorted_slot || !slot_to_row || !num_real) return ZEDA_EINVAL;
    if (!aligned16(topk_ids) || !aligned16(expert_offsets) || !aligned16(sorted_slot) || !aligned16(slot_to_row) ||
        (reinterpret_cast<uintptr_t>(num_real) & 3u))
        return ZEDA_EINVAL;
    // the library's own scratch is sized for the segmented form's longest list
    if ((int64_t)desc->T * desc->K > dispatch_static_max_slots()) return ZEDA_EUNSUPPORTED;
    if (dispatch_ws_bytes(desc) > dispatch_static_scratch_bytes()) return ZEDA_EUNSUPPORTED;
    void *ws = dispatch_static_scratch();
    if (!ws) return ZEDA_EHIP;
    return launch_dispatch(desc, topk_ids, expert_offsets, sorted_slot, slot_to_row, num_real, nullptr, ws,
                           (hipStream_t)stream);
}

int zeda_expert_ffn(const zeda_layer_desc *desc, const void *x, const void *w_gate, const void *w_up,
                    const void *w_down, const int32_t *expert_offsets, const int32_t *sorted_slot,
                    const int32_t *num_real, void *y_slot, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    if (!x || !w_gate || !w_up || !w_down || !expert_offsets || !sorted_slot || !num_real || !y_slot || !ws)
        return ZEDA_EINVAL;
    if (!aligned16(x) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) || !aligned16(expert_offsets) ||
        !aligned16(sorted_slot) || !aligned16(y_slot) || !aligned16(ws))
        return ZEDA_EINVAL;
    if (ws_bytes < act_bytes(desc)) return ZEDA_EWORKSPACE;
    if (desc->T == 0) return ZEDA_OK;
    // num_real equals expert_offsets[N]; the kernels read the offsets, so R never crosses to the host.
    hipStream_t s = (hipStream_t)stream;
    if ((rc = launch_gateup(desc, x, w_gate, w_up, expert_offsets, sorted_slot, ws, s)) != ZEDA_OK) return rc;
    return launch_down(desc, ws, w_down, expert_offsets, y_slot, s);
}

int zeda_combine(const zeda_layer_desc *desc, const void *y_slot, const int32_t *topk_ids, const float *topk_gates,
                 const int32_t *slot_to_row, const void *x, void *out, void *stream)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    const bool copy = desc->free_expert == ZEDA_EXPERT_COPY;
    if (!y_slot || !topk_ids || !topk_gates || !slot_to_row || !out || (copy && !x)) return ZEDA_EINVAL;
    if (!aligned16(y_slot) || !aligned16(topk_ids) || !aligned16(topk_gates) || !aligned16(slot_to_row) ||
        !aligned16(out) || (copy && !aligned16(x)))
        return ZEDA_EINVAL;
    if (desc->T == 0) return ZEDA_OK;
    return launch_combine(desc, y_slot, topk_ids, topk_gates, slot_to_row, x, out, (hipStream_t)stream);
}

int zeda_moe_forward(const zeda_layer_desc *desc, const void *x, const void *w_router, const float *router_bias,
                     const void *w_gate, const void *w_up, const void *w_down, void *out, int32_t *num_real_out,
                     void *ws, size_t ws_bytes, void *stream)
{
    return forward_impl(desc, x, w_router, router_bias, w_gate, w_up, w_down, out, num_real_out, ws, ws_bytes, stream,
                        nullptr);
}

int zeda_moe_forward_events(const zeda_layer_desc *desc, const void *x, const void *w_router,
                            const float *router_bias, const void *w_gate, const void *w_up, const void *w_down,
                            void *out, int32_t *num_real_out, void *ws, size_t ws_bytes, void *stream,
                            void *const *events)
{
    if (!events) return ZEDA_EINVAL;
    for (int i = 0; i <= ZEDA_NUM_STAGES; ++i)
        if (!events[i]) return ZEDA_EINVAL;
    return forward_impl(desc, x, w_router, router_bias, w_gate, w_up, w_down, out, num_real_out, ws, ws_bytes, stream,
                        events);
}

int zeda_moe_block_forward(const zeda_layer_desc *desc, const void *xn, void *x_res, const void *w_router,
                           const float *router_bias, const void *w_gate, const void *w_up, const void *w_down,
                           const void *gamma_next, float eps, void *xn_next, int32_t *num_real_out, void *ws,
                           size_t ws_bytes, void *stream)
{
    const BlockTail tail = {x_res, gamma_next, eps, xn_next};
    return forward_impl(desc, xn, w_router, router_bias, w_gate, w_up, w_down, nullptr, num_real_out, ws, ws_bytes,
                        stream, nullptr, &tail);
}

size_t zeda_routing_stats_workspace_bytes(const zeda_layer_desc *desc)
{
    if (check_desc(desc) != ZEDA_OK) return 0;
    return routing_stats_ws_bytes(desc);
}

int zeda_routing_stats(const zeda_layer_desc *desc, const void *x, const void *w_router, const float *router_bias,
                       float alpha, float w, float *f, float *P, float *summary, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    if (!x || !w_router || !f || !P || !summary || !ws || desc->T < 1 || !(w > 0.f)) return ZEDA_EINVAL;
    if (!aligned16(x) || !aligned16(w_router) || !aligned16(ws) || (router_bias && !aligned16(router_bias)) ||
        (reinterpret_cast<uintptr_t>(f) & 3u) || (reinterpret_cast<uintptr_t>(P) & 3u) ||
        (reinterpret_cast<uintptr_t>(summary) & 3u))
        return ZEDA_EINVAL;
    if (ws_bytes < routing_stats_ws_bytes(desc)) return ZEDA_EWORKSPACE;
    return launch_routing_stats(desc, x, w_router, router_bias, alpha, w, f, P, summary, ws, (hipStream_t)stream);
}

int zeda_pack_expert_weights(const zeda_layer_desc *desc, const void *w_gate, const void *w_up, const void *w_down,
                             void *w_gate_tiled, void *w_up_tiled, void *w_down_tiled, void *stream)
{
    if (!desc) return ZEDA_EINVAL;
    zeda_layer_desc d = *desc;
    d.T = 0;
    d.weight_layout = ZEDA_WEIGHTS_ROW_MAJOR;
    int rc = check_desc(&d);
    if (rc != ZEDA_OK) return rc;
    if (d.dtype != ZEDA_BF16) return ZEDA_EUNSUPPORTED;
    const void *in[3] = {w_gate, w_up, w_down};
    void *out[3] = {w_gate_tiled, w_up_tiled, w_down_tiled};
    const size_t bytes = (size_t)d.N * d.I * d.H * 2;
    for (int i = 0; i < 3; ++i) {
        if ((in[i] == nullptr) != (out[i] == nullptr)) return ZEDA_EINVAL;
        if (!in[i]) continue;
        if (!aligned16(in[i]) || !aligned16(out[i])) return ZEDA_EINVAL;
        const char *a = (const char *)in[i], *b = (const char *)out[i];
        if (a < b + bytes && b < a + bytes) return ZEDA_EINVAL;  // overlap
    }
    for (int i = 0; i < 3; ++i) {
        if (!in[i]) continue;
        rc = launch_pack_weights(&d, in[i], out[i], /*down=*/i == 2, (hipStream_t)stream);
        if (rc != ZEDA_OK) return rc;
    }
    return ZEDA_OK;
}

int zeda_token_zero_slots(const zeda_layer_desc *desc, const int32_t *topk_ids, int32_t *zero_slots, int accumulate,
                          void *stream)
{
    int rc = check_desc(desc);
    if (rc != ZEDA_OK) return rc;
    if (desc->T == 0) return ZEDA_OK;
    if (!topk_ids || !zero_slots || (reinterpret_cast<uintptr_t>(topk_ids) & 3u) || (reinterpret_cast<uintptr_t>(zero_slots) & 3u))
        return ZEDA_EINVAL;
    token_zero_slots_kernel<<<ceil_div(desc->T, 256), 256, 0, (hipStream_t)stream>>>(topk_ids, desc->T, desc->K, desc->N,
                                                                                    zero_slots, accumulate);
    return last_launch_status();
}

int zeda_stream_read_probe(const void *buf, size_t bytes, void *sink, void *stream)
{
    if (!buf || !sink || !aligned16(buf) || (bytes & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return ZEDA_EINVAL;
    if (bytes == 0) return ZEDA_OK;
    return launch_stream_read(buf, bytes, (uint32_t *)sink, (hipStream_t)stream);
}

int zeda_mfma_probe(int workgroups, int iters, float *sink, void *stream)
{
    if (!sink || (reinterpret_cast<uintptr_t>(sink) & 3u) || iters < 1 || workgroups < 1) return ZEDA_EINVAL;
    mfma_probe_kernel<<<(unsigned)workgroups, 256, 0, (hipStream_t)stream>>>(sink, iters);
    return last_launch_status();
}

int zeda_overlap_probe(const void *buf, size_t bytes, int mfmas_per_wave, int mode, float *sink, void *stream)
{
    const int what = mode & (ZEDA_PROBE_READ | ZEDA_PROBE_MFMA);
    if (!buf || !sink || !aligned16(buf) || (reinterpret_cast<uintptr_t>(sink) & 7u) || (bytes % kOverlapChunk) != 0 ||
        mode < 1 || mode > 7 || what == 0 || mfmas_per_wave < 0)
        return ZEDA_EINVAL;
    const size_t grid = bytes / kOverlapChunk;
    if (grid == 0) return ZEDA_OK;
    if (grid > 0x7fffffffu) return ZEDA_EUNSUPPORTED;
    uint32_t *usink = reinterpret_cast<uint32_t *>(sink + grid * 512);
    hipStream_t s = (hipStream_t)stream;
    const u32x4 *p = (const u32x4 *)buf;
    const bool split = (mode & ZEDA_PROBE_SPLIT_SIMD) != 0;
    if (what == ZEDA_PROBE_READ)
        return split ? launch_overlap_probe<true, false, true>(p, grid, mfmas_per_wave, sink, usink, s)
                     : launch_overlap_probe<true, false, false>(p, grid, mfmas_per_wave, sink, usink, s);
    if (what == ZEDA_PROBE_MFMA)
        return split ? launch_overlap_probe<false, true, true>(p, grid, mfmas_per_wave, sink, usink, s)
                     : launch_overlap_probe<false, true, false>(p, grid, mfmas_per_wave, sink, usink, s);
    return split ? launch_overlap_probe<true, true, true>(p, grid, mfmas_per_wave, sink, usink, s)
                 : launch_overlap_probe<true, true, false>(p, grid, mfmas_per_wave, sink, usink, s);
}

}  // extern "C"
