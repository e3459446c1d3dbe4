// Zero-slot removal and expert-sorted order of the real slots (Section 2.1: slots on zero experts
// contribute no computation, so they are dropped before any expert work is scheduled).
// A deterministic counting sort in one kernel: ballots and bit counts only, no atomics, so the order
// inside an expert is ascending slot index on every run.
// One workgroup per normal expert e.  Its 16 waves walk the slot list in contiguous segments.  A first
// pass counts, per wave, the slots on expert e and the slots on experts below e; the latter, summed, is
// the expert's first row (so no histogram and no scan across workgroups is needed, and workgroup e
// publishes expert_offsets[e] itself).  A second pass writes each match at first row + matches before it.
// Slots on zero experts get slot_to_row = -1 from the workgroup whose index their 256-slot group maps to.
//
// That kernel reads the whole slot list once per expert.  From about fifty thousand slots on a second form takes
// over, linear in the number of slots: the list is cut into segments of 2048 slots; a first kernel counts, per
// segment, the slots on every expert; a second one turns the counts into the first row of every (expert, segment)
// pair and places the segment's slots.  Inside a 64-slot group a lane finds the lanes with the same expert from
// eight ballots over the bits of the id (no loop over experts), its rank among them is a bit count, and the
// running row of an expert lives in LDS per wave.  Still no atomics: in a group only the first lane of each expert
// updates that expert's counter, and waves own disjoint counters, so the order is again ascending slot index.
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

// ---------------------------------------------------------------------------------------------
// segmented form
// ---------------------------------------------------------------------------------------------
constexpr int kSegThreads = 512;
constexpr int kSegWaves = kSegThreads / 64;
constexpr int kSegGroups = 4;                                  // 64-slot groups per wave
constexpr int kSegSlots = kSegWaves * kSegGroups * 64;         // 2048
constexpr int kSegMax = 256;                                   // segments at most (the place kernel walks them all)
constexpr int kSegMinSlots = 32769;  // up to 32768 slots the one-kernel form is faster (8 us against 10.6; above, 13 us)

// lanes of the wave whose slot is on the same normal expert as this lane's (0 for a lane that is on none)
__device__ __forceinline__ unsigned long long same_expert_lanes(int id, bool real)
{
    unsigned long long m = __ballot(real);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const unsigned long long bb = __ballot((id >> b) & 1);
        m &= ((id >> b) & 1) ? bb : ~bb;
    }
    return real ? m : 0ull;
}

// s_cnt[wave][e] += number of this wave's slots on expert e, for its kSegGroups groups of 64 slots
__device__ __forceinline__ void count_wave(const int32_t *__restrict__ ids, int S, int N, int first_slot, int *cnt_w)
{
    const int lane = threadIdx.x & 63;
    for (int g = 0; g < kSegGroups; ++g) {
        const int s = first_slot + g * 64 + lane;
        const int id = s < S ? ids[s] : -1;
        const bool real = (unsigned)id < (unsigned)N;
        const unsigned long long m = same_expert_lanes(id, real);
        // the first lane of every expert present adds the group's count (distinct experts, distinct addresses)
        if (real && (m & ((1ull << lane) - 1ull)) == 0) cnt_w[id] += __popcll(m);
    }
}

__global__ __launch_bounds__(kSegThreads) void dispatch_count_kernel(const int32_t *__restrict__ ids, int S, int N,
                                                                     int32_t *__restrict__ hist /*[segments][N]*/)
{
    __shared__ int s_cnt[kSegWaves][kMaxExperts];
    const int tid = threadIdx.x, wave = tid >> 6, seg = blockIdx.x;
    for (int i = tid; i < kSegWaves * kMaxExperts; i += kSegThreads) (&s_cnt[0][0])[i] = 0;
    __syncthreads();
    count_wave(ids, S, N, seg * kSegSlots + wave * (kSegGroups * 64), s_cnt[wave]);
    __syncthreads();
    if (tid < N) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < kSegWaves; ++w) t += s_cnt[w][tid];
        hist[(size_t)seg * N + tid] = t;
    }
}

__global__ __launch_bounds__(kSegThreads) void dispatch_place_kernel(const int32_t *__restrict__ ids, int S, int N,
                                                                     const int32_t *__restrict__ hist, int segments,
                                                                     int32_t *__restrict__ expert_offsets,
                                                                     int32_t *__restrict__ sorted_slot,
                                                                     int32_t *__restrict__ slot_to_row,
                                                                     int32_t *__restrict__ num_real,
                                                                     int32_t *__restrict__ num_real_copy)
{
    __shared__ int s_cnt[kSegWaves][kMaxExperts];  // counts of this segment's waves, then their running rows
    __shared__ int s_tot[kMaxExperts];             // rows of every expert in the whole list, then its first row
    __shared__ int s_wsum[kMaxExperts / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, seg = blockIdx.x;
    for (int i = tid; i < kSegWaves * kMaxExperts; i += kSegThreads) (&s_cnt[0][0])[i] = 0;
    __syncthreads();
    const int first_slot = seg * kSegSlots + wave * (kSegGroups * 64);
    count_wave(ids, S, N, first_slot, s_cnt[wave]);

    // thread e: rows of expert e in the segments before this one, and in all of them
    int before = 0, total = 0;
    if (tid < N) {
#pragma unroll 8
        for (int g = 0; g < segments; ++g) {  // (independent loads: several in flight)
            const int c = hist[(size_t)g * N + tid];
            total += c;
            before += g < seg ? c : 0;
        }
    }
    // exclusive scan of the totals over the experts (kMaxExperts = 4 waves of 64 values)
    if (tid < kMaxExperts) {
        int incl = tid < N ? total : 0;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        if (lane == 63) s_wsum[wave] = incl;
        s_tot[tid] = incl - (tid < N ? total : 0);  // exclusive inside the wave
    }
    __syncthreads();  // (also: every wave's counts are in s_cnt)
    if (tid < kMaxExperts) {
        int add = 0;
        for (int w = 0; w < wave; ++w) add += s_wsum[w];
        const int first_row = s_tot[tid] + add;  // first row of expert tid
        if (seg == 0 && tid < N) expert_offsets[tid] = first_row;
        if (seg == 0 && tid == N - 1) {
            const int R = first_row + total;
            expert_offsets[N] = R;
            num_real[0] = R;
            if (num_real_copy) num_real_copy[0] = R;
        }
        // running row of (wave, expert): the expert's first row, the segments before, the waves before
        int row = first_row + before;
        if (tid < N) {
#pragma unroll
            for (int w = 0; w < kSegWaves; ++w) {
                const int c = s_cnt[w][tid];
                s_cnt[w][tid] = row;
                row += c;
            }
        }
    }
    __syncthreads();

    int *row_w = s_cnt[wave];
    for (int g = 0; g < kSegGroups; ++g) {
        const int s = first_slot + g * 64 + lane;
        const int id = s < S ? ids[s] : -1;
        const bool real = (unsigned)id < (unsigned)N;
        const unsigned long long m = same_expert_lanes(id, real);
        const int rank = __popcll(m & ((1ull << lane) - 1ull));
        if (real) {
            const int base = row_w[id];   // same value for all lanes of the expert: read before its first lane writes
            const int r = base + rank;
            sorted_slot[r] = s;
            slot_to_row[s] = r;
            if (rank == 0) row_w[id] = base + __popcll(m);
        } else if (s < S) {
            slot_to_row[s] = -1;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// placement from the router's per-block counts
// ---------------------------------------------------------------------------------------------
// The router kernel that holds its token rows in LDS leaves, per block of 16 tokens, the number of slots on every
// expert (one byte each, cnt8[e][block]).  With those the placement needs no counting pass over the ids and no
// second kernel: a workgroup takes 64 tokens (4 blocks, 64*K slots, one 64-slot group per wave), adds up, per
// expert, the bytes of all blocks (the expert's rows) and of the blocks before its own (the rows before its
// segment) - four threads per expert, 16 blocks per 16-byte load, v_sad_u8 adding four bytes at a time - scans
// the totals over the experts, and places its slots as the segmented form above does.
constexpr int kCntTokens = 64;     // tokens per workgroup: 4 blocks of the router
constexpr int kCntThreads = 1024;  // 16 waves: K <= 16 groups of 64 slots
constexpr int kCntMaxTokens = 16384;  // beyond this the tables every workgroup adds up get long: the forms above take over
static_assert(kCntThreads / 64 >= kMaxK && kCntThreads / kMaxExperts == 4, "one wave per 64-slot group, four threads per expert");

__global__ __launch_bounds__(kCntThreads) void dispatch_place_counts_kernel(const int32_t *__restrict__ ids, int S, int N, int K,
                                                                            const uint8_t *__restrict__ cnt8, int cnt_ld, int nblk,
                                                                            int32_t *__restrict__ expert_offsets,
                                                                            int32_t *__restrict__ sorted_slot,
                                                                            int32_t *__restrict__ slot_to_row,
                                                                            int32_t *__restrict__ num_real,
                                                                            int32_t *__restrict__ num_real_copy)
{
    __shared__ int s_cnt[kMaxK][kMaxExperts];  // slots of wave w's group on every expert, then the running rows
    __shared__ int s_tot[4][kMaxExperts], s_bef[4][kMaxExperts];
    __shared__ int s_first[kMaxExperts];
    __shared__ int s_wsum[kMaxExperts / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, seg = blockIdx.x;
    for (int i = tid; i < kMaxK * kMaxExperts; i += kCntThreads) (&s_cnt[0][0])[i] = 0;
    __syncthreads();
    // this wave's group of 64 slots
    const int s = seg * (kCntTokens * K) + wave * 64 + lane;
    const bool in_seg = wave < K && s < S;
    const int id = in_seg ? ids[s] : -1;
    const bool real = (unsigned)id < (unsigned)N;
    const unsigned long long m = same_expert_lanes(id, real);
    const int rank = __popcll(m & ((1ull << lane) - 1ull));
    if (real && rank == 0) s_cnt[wave][id] = __popcll(m);

    // thread (e, part): rows of expert e in a quarter of the blocks, and in those of them before this segment
    {
        const int e = tid & (kMaxExperts - 1), part = tid >> 8;
        int total = 0, before = 0;
        if (e < N) {
            const int words = cnt_ld / 16, per = (words + 3) / 4;  // 16-byte words of the expert's row of bytes
            const uint4 *row = reinterpret_cast<const uint4 *>(cnt8 + (size_t)e * cnt_ld);
            const int first_blk = seg * (kCntTokens / 16);
            for (int wi = part * per; wi < min(words, (part + 1) * per); ++wi) {
                const uint4 v = row[wi];
                const unsigned dw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int b0 = wi * 16 + q * 4;  // blocks b0 .. b0+3
                    unsigned x = dw[q];
                    if (b0 + 4 > nblk) x = b0 >= nblk ? 0u : (x & ((1u << (8 * (nblk - b0))) - 1u));  // bytes past the last block
                    const int c = (int)__builtin_amdgcn_sad_u8(x, 0u, 0u);
                    total += c;
                    before += b0 < first_blk ? c : 0;  // (segments start at multiples of four blocks)
                }
            }
        }
        s_tot[part][e] = total;
        s_bef[part][e] = before;
    }
    __syncthreads();
    int total = 0, before = 0;
    if (tid < kMaxExperts) {
#pragma unroll
        for (int q = 0; q < 4; ++q) { total += s_tot[q][tid]; before += s_bef[q][tid]; }
        // exclusive scan of the totals over the experts
        int incl = total;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        if (lane == 63) s_wsum[wave] = incl;
        s_first[tid] = incl - total;
    }
    __syncthreads();
    if (tid < kMaxExperts) {
        int add = 0;
        for (int w = 0; w < wave; ++w) add += s_wsum[w];
        const int first_row = s_first[tid] + add;
        if (seg == 0 && tid < N) expert_offsets[tid] = first_row;
        if (seg == 0 && tid == N - 1) {
            const int R = first_row + total;
            expert_offsets[N] = R;
            num_real[0] = R;
            if (num_real_copy) num_real_copy[0] = R;
        }
        // running row of (wave, expert): the expert's first row, the segments before, the waves before
        int row = first_row + before;
        if (tid < N) {
            for (int w = 0; w < K; ++w) {
                const int c = s_cnt[w][tid];
                s_cnt[w][tid] = row;
                row += c;
            }
        }
    }
    __syncthreads();
    if (real) {
        const int r = s_cnt[wave][id] + rank;
        sorted_slot[r] = s;
        slot_to_row[s] = r;
    } else if (in_seg) {
        slot_to_row[s] = -1;
    }
}

bool dispatch_counts_supported(const zeda_layer_desc *d) { return d->T <= kCntMaxTokens; }

int launch_dispatch_counts(const zeda_layer_desc *d, const int32_t *ids, const uint8_t *cnt8, int32_t *offsets,
                           int32_t *sorted_slot, int32_t *slot_to_row, int32_t *num_real, int32_t *num_real_copy,
                           hipStream_t s)
{
    const int S = d->T * d->K, nblk = ceil_div(d->T, 16);
    dispatch_place_counts_kernel<<<ceil_div(d->T, kCntTokens), kCntThreads, 0, s>>>(
        ids, S, d->N, d->K, cnt8, route_counts_ld(d), nblk, offsets, sorted_slot, slot_to_row, num_real, num_real_copy);
    return last_launch_status();
}

size_t dispatch_ws_bytes(const zeda_layer_desc *d)
{
    const size_t S = (size_t)d->T * d->K, segments = (S + kSegSlots - 1) / kSegSlots;
    if (S < (size_t)kSegMinSlots || segments > (size_t)kSegMax) return 256;  // the one-kernel form needs no scratch
    return align_up(segments * d->N * sizeof(int32_t), 256);
}

// Library-owned scratch of zeda_dispatch_noalloc: the per-segment counts of the segmented form at its largest
// (kSegMax segments x kMaxExperts experts).  One copy per GPU, held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the device address it returns is what kernels get.
constexpr size_t kStaticScratchBytes = (size_t)kSegMax * kMaxExperts * sizeof(int32_t);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

size_t dispatch_static_scratch_bytes() { return kStaticScratchBytes; }
int dispatch_static_max_slots() { return kSegMax * kSegSlots; }

// device address of `scratch` on the calling thread's current device (looked up once per device), or NULL
void *dispatch_static_scratch()
{
    static void *ptrs[kMaxDevices] = {};  // idempotent per device, so a race between host threads is harmless
    const int dev = current_device();
    if (dev < 0) return nullptr;
    if (!ptrs[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        ptrs[dev] = p;
    }
    return ptrs[dev];
}

int launch_dispatch(const zeda_layer_desc *d, const int32_t *ids, int32_t *offsets, int32_t *sorted_slot,
                    int32_t *slot_to_row, int32_t *num_real, int32_t *num_real_copy, void *ws, hipStream_t s)
{
    const int S = d->T * d->K, segments = (S + kSegSlots - 1) / kSegSlots;
    if (S >= kSegMinSlots && segments <= kSegMax) {
        int32_t *hist = (int32_t *)ws;
        dispatch_count_kernel<<<segments, kSegThreads, 0, s>>>(ids, S, d->N, hist);
        dispatch_place_kernel<<<segments, kSegThreads, 0, s>>>(ids, S, d->N, hist, segments, offsets, sorted_slot,
                                                               slot_to_row, num_real, num_real_copy);
        return last_launch_status();
    }
    dispatch_kernel<<<d->N, kPlaceThreads, 0, s>>>(ids, S, d->N, offsets, sorted_slot, slot_to_row, num_real,
                                                  num_real_copy);
    return last_launch_status();
}

}  // namespace zeda
