// Zero-slot removal and expert-sorted order of the real slots (Section 2.1: slots on zero experts
// contribute no computation, so they are dropped before any expert work is scheduled).
// A deterministic counting sort: ballots and prefix sums only, no atomic placement, so the order
// inside an expert is ascending slot index on every run.
//   1. count:  per block of 4096 slots an LDS histogram over the N normal experts; zero-expert
//              slots get slot_to_row = -1 here.
//   2. place:  one workgroup per normal expert.  It sums the block histograms into all expert
//              counts, scans them to its own first row (workgroup 0 also publishes expert_offsets
//              and num_real), then its 16 waves walk the slot list in contiguous segments: a first
//              pass counts matches per wave, a second pass writes each match at
//              first_row + matches before it.
#include "zeda_internal.h"

namespace zeda {

constexpr int kCountThreads = 256;
constexpr int kPlaceThreads = 1024;
constexpr int kPlaceWaves = kPlaceThreads / 64;

__global__ __launch_bounds__(kCountThreads) void dispatch_count_kernel(const int32_t *__restrict__ ids, int S, int N,
                                                                       int32_t *__restrict__ block_hist,
                                                                       int32_t *__restrict__ slot_to_row)
{
    __shared__ int hist[kMaxExperts];
    const int tid = threadIdx.x;
    for (int e = tid; e < N; e += kCountThreads) hist[e] = 0;
    __syncthreads();
    const int base = blockIdx.x * kCountSlotsPerBlock;
    // 16 slots per thread, as four 16-byte loads that are all issued before any is used
    constexpr int kVec = kCountSlotsPerBlock / kCountThreads / 4;
    int4 v[kVec];
#pragma unroll
    for (int u = 0; u < kVec; ++u) {
        const int s = base + (u * kCountThreads + tid) * 4;
        if (s + 3 < S) v[u] = *reinterpret_cast<const int4 *>(ids + s);
        else {
            v[u].x = s + 0 < S ? ids[s + 0] : -2;
            v[u].y = s + 1 < S ? ids[s + 1] : -2;
            v[u].z = s + 2 < S ? ids[s + 2] : -2;
            v[u].w = s + 3 < S ? ids[s + 3] : -2;
        }
    }
#pragma unroll
    for (int u = 0; u < kVec; ++u) {
        const int s = base + (u * kCountThreads + tid) * 4;
        const int e4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = e4[q];
            if (e >= 0 && e < N) atomicAdd(&hist[e], 1);  // integer counts: the result does not depend on order
            else if (s + q < S) slot_to_row[s + q] = -1;
        }
    }
    __syncthreads();
    for (int e = tid; e < N; e += kCountThreads) block_hist[(size_t)blockIdx.x * N + e] = hist[e];
}

__global__ __launch_bounds__(kPlaceThreads) void dispatch_place_kernel(const int32_t *__restrict__ ids, int S, int N,
                                                                       int nblocks,
                                                                       const int32_t *__restrict__ block_hist,
                                                                       int32_t *__restrict__ expert_offsets,
                                                                       int32_t *__restrict__ sorted_slot,
                                                                       int32_t *__restrict__ slot_to_row,
                                                                       int32_t *__restrict__ num_real)
{
    __shared__ int cnt[kMaxExperts + 1];
    __shared__ int wave_cnt[kPlaceWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int e = blockIdx.x;

    if (tid < N) {
        int m = 0;
        for (int b0 = 0; b0 < nblocks; b0 += 8) {
            int part[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) part[u] = b0 + u < nblocks ? block_hist[(size_t)(b0 + u) * N + tid] : 0;
#pragma unroll
            for (int u = 0; u < 8; ++u) m += part[u];
        }
        cnt[tid] = m;
    }
    __syncthreads();
    if (wave == 0) {
        // exclusive scan of cnt[0..N): lane l owns experts 4l..4l+3
        int c[4], local = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int idx = 4 * lane + q;
            c[q] = idx < N ? cnt[idx] : 0;
            local += c[q];
        }
        int incl = local;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        int run = incl - local;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int idx = 4 * lane + q;
            if (idx < N) cnt[idx] = run;
            run += c[q];
        }
        if (lane == 63) cnt[kMaxExperts] = incl;  // R
    }
    __syncthreads();
    const int first_row = cnt[e];
    if (e == 0) {
        for (int i = tid; i < N; i += kPlaceThreads) expert_offsets[i] = cnt[i];
        if (tid == 0) {
            expert_offsets[N] = cnt[kMaxExperts];
            num_real[0] = cnt[kMaxExperts];
        }
    }

    // contiguous segment of this wave, in groups of 256 slots (4 consecutive slots per lane)
    const int groups = (S + 255) / 256;
    const int gpw = (groups + kPlaceWaves - 1) / kPlaceWaves;
    // every workgroup reads the whole id list: each starts at a different segment so that they do not all
    // queue on the same L2 channel at the same time (segment seg is still placed after segments < seg)
    const int seg = (wave + e) % kPlaceWaves;
    const int g0 = seg * gpw, g1 = min(groups, g0 + gpw);
    const int4 *ids4 = reinterpret_cast<const int4 *>(ids);
    const int full4 = S / 4;  // int4 loads are in bounds below this index

    auto load4 = [&](int g) -> int4 {
        int q = g * 64 + lane;
        if (q < full4) return ids4[q];
        int4 v;
        int s = q * 4;
        v.x = s + 0 < S ? ids[s + 0] : -1;
        v.y = s + 1 < S ? ids[s + 1] : -1;
        v.z = s + 2 < S ? ids[s + 2] : -1;
        v.w = s + 3 < S ? ids[s + 3] : -1;
        return v;
    };

    // The segment is walked in batches of kBatch groups whose loads are all issued before any is used.
    // When the whole segment is one batch (the usual case) the ids stay in registers for the second pass.
    constexpr int kBatch = 8;
    const bool one_batch = gpw <= kBatch;
    int4 keep[kBatch];
    int my = 0;
    for (int gb = g0; gb < g1; gb += kBatch) {
        int4 v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) v[u] = (gb + u < g1) ? load4(gb + u) : make_int4(-1, -1, -1, -1);
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            my += __popcll(__ballot(v[u].x == e)) + __popcll(__ballot(v[u].y == e)) + __popcll(__ballot(v[u].z == e)) +
                  __popcll(__ballot(v[u].w == e));
            keep[u] = v[u];
        }
    }
    if (lane == 0) wave_cnt[seg] = my;
    __syncthreads();
    int before = first_row;
    for (int w = 0; w < seg; ++w) before += wave_cnt[w];

    for (int gb = g0; gb < g1; gb += kBatch) {
        int4 v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
            v[u] = one_batch ? keep[u] : ((gb + u < g1) ? load4(gb + u) : make_int4(-1, -1, -1, -1));
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const bool hx = v[u].x == e, hy = v[u].y == e, hz = v[u].z == e, hw = v[u].w == e;
            // matches in lower lanes of this group: ballots and bit counts, no cross-lane data movement
            const unsigned long long bx = __ballot(hx), by = __ballot(hy), bz = __ballot(hz), bw = __ballot(hw);
            const unsigned long long below = (1ull << lane) - 1ull;
            int r = before + __popcll(bx & below) + __popcll(by & below) + __popcll(bz & below) + __popcll(bw & below);
            const int group_total = __popcll(bx) + __popcll(by) + __popcll(bz) + __popcll(bw);
            const int s = ((gb + u) * 64 + lane) * 4;
            if (hx) { sorted_slot[r] = s + 0; slot_to_row[s + 0] = r; ++r; }
            if (hy) { sorted_slot[r] = s + 1; slot_to_row[s + 1] = r; ++r; }
            if (hz) { sorted_slot[r] = s + 2; slot_to_row[s + 2] = r; ++r; }
            if (hw) { sorted_slot[r] = s + 3; slot_to_row[s + 3] = r; ++r; }
            before += group_total;
        }
    }
}

int launch_dispatch(const zeda_layer_desc *d, const int32_t *ids, int32_t *offsets, int32_t *sorted_slot,
                    int32_t *slot_to_row, int32_t *num_real, int32_t *block_hist, hipStream_t s)
{
    const int S = d->T * d->K;
    const int nb = ceil_div(S, kCountSlotsPerBlock);
    if (nb > 0) {
        dispatch_count_kernel<<<nb, kCountThreads, 0, s>>>(ids, S, d->N, block_hist, slot_to_row);
        if (hipGetLastError() != hipSuccess) return ZEDA_EHIP;
    }
    dispatch_place_kernel<<<d->N, kPlaceThreads, 0, s>>>(ids, S, d->N, nb, block_hist, offsets, sorted_slot, slot_to_row,
                                                          num_real);
    return last_launch_status();
}

}  // namespace zeda
