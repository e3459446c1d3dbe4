// Zero-slot removal and expert-sorted order of the real slots (Section 2.1: slots on zero experts
// contribute no computation, so they are dropped before any expert work is scheduled).
// A deterministic counting sort in one kernel: ballots and bit counts only, no atomics, so the order
// inside an expert is ascending slot index on every run.
// One workgroup per normal expert e.  Its 16 waves walk the slot list in contiguous segments.  A first
// pass counts, per wave, the slots on expert e and the slots on experts below e; the latter, summed, is
// the expert's first row (so no histogram and no scan across workgroups is needed, and workgroup e
// publishes expert_offsets[e] itself).  A second pass writes each match at first row + matches before it.
// Slots on zero experts get slot_to_row = -1 from the workgroup whose index their 256-slot group maps to.
#include "zeda_internal.h"

namespace zeda {

constexpr int kPlaceThreads = 1024;
constexpr int kPlaceWaves = kPlaceThreads / 64;

__global__ __launch_bounds__(kPlaceThreads) void dispatch_kernel(const int32_t *__restrict__ ids, int S, int N,
                                                                 int32_t *__restrict__ expert_offsets,
                                                                 int32_t *__restrict__ sorted_slot,
                                                                 int32_t *__restrict__ slot_to_row,
                                                                 int32_t *__restrict__ num_real,
                                                                 int32_t *__restrict__ num_real_copy)
{
    __shared__ int wave_match[kPlaceWaves], wave_below[kPlaceWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int e = blockIdx.x;

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
    auto count = [&](bool p) { return __popcll(__ballot(p)); };

    // The segment is walked in batches of kBatch groups whose loads are all issued before any is used.
    // When the whole segment is one batch (the usual case) the ids stay in registers for the second pass.
    constexpr int kBatch = 8;
    const bool one_batch = gpw <= kBatch;
    int4 keep[kBatch];
    int match = 0, below = 0;
    for (int gb = g0; gb < g1; gb += kBatch) {
        int4 v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) v[u] = (gb + u < g1) ? load4(gb + u) : make_int4(-1, -1, -1, -1);
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            match += count(v[u].x == e) + count(v[u].y == e) + count(v[u].z == e) + count(v[u].w == e);
            // ids below e, as unsigned compares so that the -1 padding does not count
            below += count((unsigned)v[u].x < (unsigned)e) + count((unsigned)v[u].y < (unsigned)e) +
                     count((unsigned)v[u].z < (unsigned)e) + count((unsigned)v[u].w < (unsigned)e);
            keep[u] = v[u];
        }
    }
    if (lane == 0) {
        wave_match[seg] = match;
        wave_below[seg] = below;
    }
    __syncthreads();
    int first_row = 0, total = 0, before = 0;
#pragma unroll
    for (int w = 0; w < kPlaceWaves; ++w) {
        first_row += wave_below[w];
        total += wave_match[w];
        if (w < seg) before += wave_match[w];
    }
    before += first_row;
    if (tid == 0) {
        expert_offsets[e] = first_row;
        if (e == N - 1) {
            expert_offsets[N] = first_row + total;  // R: every real slot is on an expert <= N-1
            num_real[0] = first_row + total;
            if (num_real_copy) num_real_copy[0] = first_row + total;
        }
    }

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
            const unsigned long long lower = (1ull << lane) - 1ull;
            int r = before + __popcll(bx & lower) + __popcll(by & lower) + __popcll(bz & lower) + __popcll(bw & lower);
            const int group_total = __popcll(bx) + __popcll(by) + __popcll(bz) + __popcll(bw);
            const int s = ((gb + u) * 64 + lane) * 4;
            if (hx) { sorted_slot[r] = s + 0; slot_to_row[s + 0] = r; ++r; }
            if (hy) { sorted_slot[r] = s + 1; slot_to_row[s + 1] = r; ++r; }
            if (hz) { sorted_slot[r] = s + 2; slot_to_row[s + 2] = r; ++r; }
            if (hw) { sorted_slot[r] = s + 3; slot_to_row[s + 3] = r; ++r; }
            before += group_total;
            // zero-expert slots (and ids that are no expert at all) of the groups this workgroup is in charge of
            if ((gb + u) % N == e && gb + u < g1) {
                if ((unsigned)v[u].x >= (unsigned)N && s + 0 < S) slot_to_row[s + 0] = -1;
                if ((unsigned)v[u].y >= (unsigned)N && s + 1 < S) slot_to_row[s + 1] = -1;
                if ((unsigned)v[u].z >= (unsigned)N && s + 2 < S) slot_to_row[s + 2] = -1;
                if ((unsigned)v[u].w >= (unsigned)N && s + 3 < S) slot_to_row[s + 3] = -1;
            }
        }
    }
}

int launch_dispatch(const zeda_layer_desc *d, const int32_t *ids, int32_t *offsets, int32_t *sorted_slot,
                    int32_t *slot_to_row, int32_t *num_real, int32_t *num_real_copy, hipStream_t s)
{
    dispatch_kernel<<<d->N, kPlaceThreads, 0, s>>>(ids, d->T * d->K, d->N, offsets, sorted_slot, slot_to_row, num_real,
                                                  num_real_copy);
    return last_launch_status();
}

}  // namespace zeda
