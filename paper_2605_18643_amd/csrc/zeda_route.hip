// Router of the augmented expert pool (Section 2.1): logits over N normal + Z zero experts, the
// top-K set with a deterministic lower-index tie-break, and the routing weights (Section 4.3.4 for
// the normalisation choices).  One fused kernel: projection -> LDS -> wave-level selection.
#include <limits.h>

#include "zeda_internal.h"

namespace zeda {

constexpr int kRouteTokens = 32;  // tokens per workgroup of the bf16 kernel (one MFMA column block)
constexpr int kRouteThreads = 256;

// Selection runs four tokens per wave, one per row of 16 lanes (the unit of the VALU's data-parallel-primitive
// cross-lane path), so all reductions stay inside a row and need no LDS traffic and no scalar round trips.
// row_ror rotates a value inside its row; max/min folded over rotations by 8, 4, 2, 1 leave every lane of the
// row with the row's result, and since max and min do not depend on the order all lanes agree exactly.
template <int N>
__device__ __forceinline__ int dpp_row_ror(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, 0x120 + N, 0xf, 0xf, false);
}
__device__ __forceinline__ float row_max(float v)
{
    v = fmaxf(v, __int_as_float(dpp_row_ror<8>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_row_ror<4>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_row_ror<2>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_row_ror<1>(__float_as_int(v))));
    return v;
}
__device__ __forceinline__ int row_min(int v)
{
    v = min(v, dpp_row_ror<8>(v));
    v = min(v, dpp_row_ror<4>(v));
    v = min(v, dpp_row_ror<2>(v));
    v = min(v, dpp_row_ror<1>(v));
    return v;
}
// Sum over the row in one fixed order (an inclusive scan with row_shr 1, 2, 4, 8 leaves the total in the row's
// last lane), handed to every lane of the row, so that all lanes divide by the same number.
__device__ __forceinline__ float row_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x111, 0xf, 0xf, false));  // lanes without a source add zero
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x112, 0xf, 0xf, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, false));
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 47));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
    const int r = (threadIdx.x & 63) >> 4;
    return r == 0 ? r0 : r == 1 ? r1 : r == 2 ? r2 : r3;
}

// Sum over all 64 lanes in a fixed order, returned to every lane.
__device__ __forceinline__ float wave_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x111, 0xf, 0xf, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x112, 0xf, 0xf, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, false));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, false));
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 47));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
    return (r0 + r1) + (r2 + r3);
}

// Selection and gates for the four tokens tk0..tk0+3 of the workgroup's block (whose fp32 logits are rows of
// lg in LDS), executed by one wave: token tk0 + r belongs to lane row r, and lane l of the row holds the
// candidates l, l + 16, ... (NC of them).  One round: the row maximum, then the lowest expert index among the
// candidates equal to it (ties go to the lower index), which its owner then removes.  Lane j of the row keeps
// slot j, so lanes 0..K-1 end up with the slots in descending-logit order (K <= 16).
// Returns the expert of the slot this lane keeps (lane j < K of a row: slot j of the row's token), or -1.
// probs (may be NULL): an LDS table [token][LDP] that receives, for every token of the wave, the routing
// probability of every expert (softmax over all NE logits).
template <int NC, int NP>
__device__ __forceinline__ int select_rows(const float *lg, int LD, int pstride, int np_rt, const float *__restrict__ bias, int tk0,
                                           int ntok, int t0, int T, int NE, int N, int K, int gate_norm,
                                           int32_t *__restrict__ ids, float *__restrict__ gates, float *probs = nullptr,
                                           int LDP = 0)
{
    const int lane = threadIdx.x & 63, l16 = lane & 15, tk = tk0 + (lane >> 4);
    const bool ok = tk < ntok && t0 + tk < T;
    float cand[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int e = l16 + 16 * c;
        float v = -INFINITY;
        if (ok && e < NE) {
            // the NP partial sums over slices of the hidden dimension, added in a fixed order, then the bias
            v = lg[tk * LD + e];
#pragma unroll
            for (int q = 1; q < NP; ++q) v += lg[(size_t)q * pstride + tk * LD + e];
            if (bias) v += bias[e];
        }
        cand[c] = v;
    }
    auto local_max = [&]() {
        float m = cand[0];
#pragma unroll
        for (int c = 1; c < NC; ++c) m = fmaxf(m, cand[c]);
        return m;
    };
    const float all_max = row_max(local_max());
    float all_sum = 0.f;
    if (gate_norm == ZEDA_GATE_SOFTMAX || probs) {
        float ex[NC], sacc = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            ex[c] = (ok && l16 + 16 * c < NE) ? expf(cand[c] - all_max) : 0.f;
            sacc += ex[c];
        }
        all_sum = row_sum(sacc);
        if (probs && ok) {
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (l16 + 16 * c < NE) probs[tk * LDP + l16 + 16 * c] = ex[c] / all_sum;
        }
    }
    int my_id = 0;
    float my_logit = -INFINITY;
    for (int j = 0; j < K; ++j) {
        const float m = row_max(local_max());
        int mine = INT_MAX;
#pragma unroll
        for (int c = NC - 1; c >= 0; --c)
            if (cand[c] == m) mine = l16 + 16 * c;  // descending c: the lowest index survives
        const int win = row_min(mine);
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if (win == l16 + 16 * c) cand[c] = -INFINITY;
        if (l16 == j) { my_id = win; my_logit = m; }
    }
    const bool slot = l16 < K;
    const float ex = slot ? expf(my_logit - all_max) : 0.f;
    float dn;
    if (gate_norm == ZEDA_GATE_SOFTMAX) dn = all_sum;
    else if (gate_norm == ZEDA_GATE_TOPK_NORM) dn = row_sum(ex);
    else dn = row_sum((slot && my_id < N) ? ex : 0.f);
    if (slot && ok && ids) {
        const size_t o = (size_t)(t0 + tk) * K + l16;
        ids[o] = my_id;
        gates[o] = dn > 0.f ? ex / dn : 0.f;
    }
    return (slot && ok) ? my_id : -1;
}

// All ntok tokens of a workgroup of NWAVES waves, four per wave at a time.  lg holds NP partial logit tables
// pstride floats apart.
// s_cnt (LDS, may be NULL): [ntok / 16][kMaxExperts] counters, zeroed by the caller; every selected slot adds one to
// the counter of its expert in its block of 16 tokens (the counts do not depend on the order of the additions).
// probs (LDS, may be NULL): [ntok][LDP] table that receives every token's routing probabilities.
template <int NC, int NP, int NWAVES>
__device__ __forceinline__ void select_block(const float *lg, int LD, int pstride, int np_rt, const float *__restrict__ bias, int ntok,
                                             int t0, int T, int NE, int N, int K, int gate_norm, int32_t *__restrict__ ids,
                                             float *__restrict__ gates, int *s_cnt = nullptr, float *probs = nullptr,
                                             int LDP = 0)
{
    const int wave = threadIdx.x >> 6;
    for (int tk0 = 4 * wave; tk0 < ntok; tk0 += 4 * NWAVES) {
        const int id = select_rows<NC, NP>(lg, LD, pstride, np_rt, bias, tk0, ntok, t0, T, NE, N, K, gate_norm, ids, gates, probs, LDP);
        if (s_cnt && id >= 0) atomicAdd(&s_cnt[(tk0 >> 4) * kMaxExperts + id], 1);
    }
}

// After select_block (and a barrier): what the workgroup's blocks of 16 tokens hand to the expert-sorted placement
// and to the routing statistics.  cnt8[e][cnt_ld] bytes: slots of every block on expert e; p_part[block][NE]: the
// block's sum of every expert's routing probability, added in token order.
template <int THREADS>
__device__ __forceinline__ void publish_blocks(const int *s_cnt, const float *probs, int LDP, int ntok, int t0, int T, int NE,
                                               uint8_t *__restrict__ cnt8, int cnt_ld, float *__restrict__ p_part)
{
    const int nblk = (ntok + 15) >> 4;
    for (int i = threadIdx.x; i < nblk * NE; i += THREADS) {
        const int u = i / NE, e = i - u * NE, blk = (t0 >> 4) + u;
        if (t0 + u * 16 >= T) continue;
        if (cnt8) cnt8[(size_t)e * cnt_ld + blk] = (uint8_t)s_cnt[u * kMaxExperts + e];
        if (p_part) {
            float ps = 0.f;
            const int nt = min(16, min(ntok, T - t0) - u * 16);
            for (int t = 0; t < nt; ++t) ps += probs[(u * 16 + t) * LDP + e];
            p_part[(size_t)blk * NE + e] = ps;
        }
    }
}

// bf16 router.  A workgroup owns kRouteTokens tokens and all NE experts (NB MFMA row blocks of 32; tokens
// are the MFMA columns).  x rows and router rows stream through an LDS ring (up to six slots) in 64-wide
// k chunks with global->LDS loads, 128-byte rows whose 16-byte pieces are XOR-permuted by the row index
// (applied on the global address) so that fragment reads spread over the banks; a counted s_waitcnt and
// one s_barrier per chunk order the ring.  The four waves split the four 16-wide MFMA steps of every
// chunk, so each holds a partial sum over a quarter of the hidden dimension; each stores it in an LDS table
// of its own and the selection adds the four tables in wave order (a fixed order: the logits are
// reproducible); each wave selects for 8 tokens, four at a time (one per row of 16 lanes).
// With many tokens the router rows, which every workgroup reads in full, are most of the traffic (640 KiB per
// workgroup from L2 against 128 KiB of token rows): TB = 2 gives a workgroup two token blocks (64 tokens), which
// halves that traffic per token; it is used once there are enough token blocks to fill the device without it.
// ring depth: as many slots as fit in LDS, at most six
constexpr int route_stages(int nb, int tb = 1)
{
    return 160 * 1024 / ((32 * tb + 32 * nb) * 128) < 6 ? 160 * 1024 / ((32 * tb + 32 * nb) * 128) : 6;
}

__device__ __forceinline__ int route_swz(int row, int piece) { return piece ^ ((row >> 1) & 7); }

template <int N>
__device__ __forceinline__ void route_wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int NB, int TB>
__global__ __launch_bounds__(kRouteThreads) void route_bf16_kernel(const bf16_t *__restrict__ x,
                                                                   const bf16_t *__restrict__ wr,
                                                                   const float *__restrict__ bias, int T, int H, int N,
                                                                   int NE, int K, int gate_norm,
                                                                   int32_t *__restrict__ ids, float *__restrict__ gates,
                                                                   float *__restrict__ partial, int Tpad,
                                                                   uint8_t *__restrict__ cnt8, int cnt_ld,
                                                                   float *__restrict__ p_part)
{
    constexpr int TOK = 32 * TB;                  // tokens of the workgroup
    constexpr int LD = NB * 32 + 1;
    constexpr int ROWS = TOK + 32 * NB;           // rows of one ring slot: tokens first, then router rows
    constexpr int STAGE = ROWS * 128;
    constexpr int NL = TB + NB;                   // wave load instructions (8 rows each) per chunk and wave
    constexpr int kRouteStages = route_stages(NB, TB);
    constexpr int NT = 4 / TB;                    // partial logit tables in LDS (the four waves' sums meet in them)
    static_assert(kRouteThreads == kMaxExperts, "");
    static_assert(kRouteTokens == 32 && kRouteThreads == 256 && (TB == 1 || TB == 2), "token blocks of 32, four waves");
    static_assert(NT * TOK * LD * 4 + (TOK / 16) * kMaxExperts * 4 <= kRouteStages * STAGE,
                  "the partial logit tables and the per-block expert counters reuse the ring");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    float *lg = reinterpret_cast<float *>(lds);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = blockIdx.x * TOK;
    const int col = lane & 31, half = lane >> 5;

    const bf16_t *src[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int row = (wave + 4 * i) * 8 + (lane >> 3), piece = lane & 7;
        const bf16_t *base = row < TOK ? x + (size_t)min(t0 + row, T - 1) * H : wr + (size_t)min(row - TOK, NE - 1) * H;
        src[i] = base + route_swz(row, piece) * 8;
    }
    // All workgroups read the same router rows, and rows are a power-of-two number of bytes apart, so one
    // k chunk of every row sits on a single L2 channel: workgroups walking the chunks in the same order
    // would queue on that channel.  Each starts at a different chunk instead (the sum over k does not
    // depend on the order; the order is fixed per workgroup, so results stay reproducible).
    // gridDim.y workgroups share a token block: each takes a contiguous slice of the hidden dimension
    const int nk = H / 64 / gridDim.y, k0 = blockIdx.y * nk;
    const int rot = (int)((blockIdx.x * 5u) % (unsigned)nk);
    auto issue = [&](int chunk) {
        unsigned char *slot = lds + (chunk % kRouteStages) * STAGE;
        int kc = chunk + rot;
        if (kc >= nk) kc -= nk;
#pragma unroll
        for (int i = 0; i < NL; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[i] + (size_t)(k0 + kc) * 64),
                                             (__attribute__((address_space(3))) void *)(slot + (wave + 4 * i) * 1024), 16, 0, 0);
    };

    f32x16 acc[NB][TB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int u = 0; u < TB; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][u][v] = 0.f;

#pragma unroll
    for (int c = 0; c < kRouteStages - 1; ++c)
        if (c < nk) issue(c);
    for (int it = 0; it < nk; ++it) {
        if (it + kRouteStages - 2 < nk) route_wait_vmcnt<(kRouteStages - 2) * NL>();
        else route_wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (it + kRouteStages - 1 < nk) issue(it + kRouteStages - 1);
        const unsigned char *cur = lds + (it % kRouteStages) * STAGE;
        // this wave's 16-wide step of the chunk: pieces 2*wave and 2*wave+1 of every row
        bf16x8 tb[TB];
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int trow = u * 32 + col;
            tb[u] = *reinterpret_cast<const bf16x8 *>(cur + trow * 128 + route_swz(trow, 2 * wave + half) * 16);
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int row = TOK + b * 32 + col;
            const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(cur + row * 128 + route_swz(row, 2 * wave + half) * 16);
#pragma unroll
            for (int u = 0; u < TB; ++u) acc[b][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, tb[u], acc[b][u], 0, 0, 0);
        }
    }
    __syncthreads();  // everyone is done with the ring: its memory now holds the logits

    // acc[b][u][v]: expert 32b + 8(v/4) + 4*half + v%4, token 32u + col.  The waves' partial sums (each over a
    // quarter of the hidden dimension) meet in NT tables: wave w uses table w % NT, the waves of a table take turns
    // in wave order, the first one storing and the later ones adding; the selection adds the tables in order.
    // Every order is fixed, so the logits are reproducible.
    float *mine = lg + (wave % NT) * (TOK * LD);
#pragma unroll
    for (int turn = 0; turn < 4 / NT; ++turn) {
        if (wave / NT == turn) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int u = 0; u < TB; ++u)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float *p = mine + (u * 32 + col) * LD + b * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                        *p = turn == 0 ? acc[b][u][v] : *p + acc[b][u][v];
                    }
        }
        __syncthreads();
    }
    if (partial == nullptr) {
        // cnt8, p_part (either may be NULL): per block of 16 tokens, the slots on every expert (for the expert-sorted
        // placement) and the sums of the routing probabilities (routing statistics), see publish_blocks.  The
        // probabilities of a token overwrite its row of the first logit table once the token's logits are in registers.
        int *s_cnt = reinterpret_cast<int *>(lg + NT * TOK * LD);
        if (cnt8) {
            for (int i = tid; i < (TOK / 16) * kMaxExperts; i += kRouteThreads) s_cnt[i] = 0;
            __syncthreads();
        }
        select_block<2 * NB, NT, 4>(lg, LD, TOK * LD, NT, bias, TOK, t0, T, NE, N, K, gate_norm, ids, gates,
                                    cnt8 ? s_cnt : nullptr, p_part ? lg : nullptr, LD);
        if (cnt8 || p_part) {
            __syncthreads();
            publish_blocks<kRouteThreads>(s_cnt, lg, LD, TOK, t0, T, NE, cnt8, cnt_ld, p_part);
        }
    } else {
        // split-k launch: this workgroup's sums over its slice (the tables added in order) go to
        // partial[blockIdx.y][token][expert]; route_select_kernel adds the slices in order and selects
        float *dst = partial + ((size_t)blockIdx.y * Tpad + t0) * (NB * 32);
        for (int i = tid; i < TOK * NB * 32; i += kRouteThreads) {
            const int tk = i / (NB * 32), e = i - tk * (NB * 32);
            float v = lg[tk * LD + e];
#pragma unroll
            for (int q = 1; q < NT; ++q) v += lg[q * TOK * LD + tk * LD + e];
            dst[i] = v;
        }
    }
}

// Second step of a split-k launch: 16 tokens per workgroup, four per wave, logits read from the partial tables.
constexpr int kSelectTokens = 16;
template <int NB, int NSPLIT>
__global__ __launch_bounds__(kRouteThreads) void route_select_kernel(const float *__restrict__ partial, int Tpad,
                                                                     const float *__restrict__ bias, int T, int N, int NE,
                                                                     int K, int gate_norm, int32_t *__restrict__ ids,
                                                                     float *__restrict__ gates, uint8_t *__restrict__ cnt8,
                                                                     int cnt_ld, float *__restrict__ p_part)
{
    static_assert(kSelectTokens == 16, "one block of the per-block tables per workgroup");
    constexpr int LDP = NB * 32 + 1;
    __shared__ int s_cnt[kMaxExperts];
    __shared__ float s_probs[kSelectTokens * LDP];  // (used by the statistics run only)
    const int t0 = blockIdx.x * kSelectTokens;
    if (cnt8) {
        s_cnt[threadIdx.x] = 0;  // (kRouteThreads == kMaxExperts)
        __syncthreads();
    }
    // (the number of slices is a template parameter so that all loads of a lane's candidates are issued together)
    select_block<2 * NB, NSPLIT, 4>(partial + (size_t)t0 * (NB * 32), NB * 32, Tpad * NB * 32, NSPLIT, bias, kSelectTokens,
                                    t0, T, NE, N, K, gate_norm, ids, gates, cnt8 ? s_cnt : nullptr,
                                    p_part ? s_probs : nullptr, LDP);
    if (cnt8 || p_part) {
        __syncthreads();
        publish_blocks<kRouteThreads>(s_cnt, s_probs, LDP, kSelectTokens, t0, T, NE, cnt8, cnt_ld, p_part);
    }
}

// fp32 router (plain FMA): a workgroup owns 8 tokens staged in LDS chunk by chunk; a wave walks the
// experts, its lanes stride over the hidden dimension, partial sums meet in a fixed butterfly.
constexpr int kRouteF32Tokens = 8;
constexpr int kRouteF32Chunk = 1024;

__global__ __launch_bounds__(kRouteThreads) void route_f32_kernel(const float *__restrict__ x,
                                                                  const float *__restrict__ wr,
                                                                  const float *__restrict__ bias, int T, int H, int N,
                                                                  int NE, int K, int gate_norm,
                                                                  int32_t *__restrict__ ids, float *__restrict__ gates,
                                                                  float *__restrict__ logits_out, int LDg)
{
    __shared__ float xs[kRouteF32Tokens * kRouteF32Chunk];
    __shared__ float lg[kRouteF32Tokens * (kMaxExperts + 1)];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * kRouteF32Tokens;
    constexpr int LD = kMaxExperts + 1;
    for (int i = tid; i < kRouteF32Tokens * NE; i += kRouteThreads) lg[(i / NE) * LD + (i % NE)] = 0.f;
    for (int h0 = 0; h0 < H; h0 += kRouteF32Chunk) {
        const int hc = min(kRouteF32Chunk, H - h0);
        __syncthreads();
        for (int i = tid; i < kRouteF32Tokens * hc; i += kRouteThreads) {
            int tk = i / hc, h = i - tk * hc;
            int t = min(t0 + tk, T - 1);
            xs[tk * kRouteF32Chunk + h] = x[(size_t)t * H + h0 + h];
        }
        __syncthreads();
        for (int e = wave; e < NE; e += 4) {
            float part[kRouteF32Tokens];
#pragma unroll
            for (int tk = 0; tk < kRouteF32Tokens; ++tk) part[tk] = 0.f;
            const float *w = wr + (size_t)e * H + h0;
            for (int h = lane; h < hc; h += 64) {
                float wv = w[h];
#pragma unroll
                for (int tk = 0; tk < kRouteF32Tokens; ++tk) part[tk] = fmaf(wv, xs[tk * kRouteF32Chunk + h], part[tk]);
            }
#pragma unroll
            for (int tk = 0; tk < kRouteF32Tokens; ++tk) {
                float s = wave_sum(part[tk]);
                if (lane == 0) lg[tk * LD + e] += s;
            }
        }
    }
    __syncthreads();
    if (logits_out) {  // statistics run: hand the logits (without the bias) to route_stats_kernel
        for (int i = tid; i < kRouteF32Tokens * NE; i += kRouteThreads)
            logits_out[(size_t)(t0 + i / NE) * LDg + (i % NE)] = lg[(i / NE) * LD + (i % NE)];
        return;
    }
    select_block<kMaxExperts / 16, 1, 4>(lg, LD, 0, 1, bias, kRouteF32Tokens, t0, T, NE, N, K, gate_norm, ids, gates);
}

// How many workgroups share a token block (bf16 with scratch): as many as still run in one round of workgroups
// (one per CU; a round and a half costs as much as two), never more than eight, and the hidden dimension must split
// into whole 64-wide chunks.
int route_ksplit(const zeda_layer_desc *d)
{
    if (d->dtype != ZEDA_BF16) return 1;
    const int blocks = ceil_div(d->T, kRouteTokens), chunks = d->H / 64;
    int c = 1;
    while (c < 8 && blocks * 2 * c <= 256 && chunks % (2 * c) == 0) c *= 2;
    return c;
}

size_t route_ws_bytes(const zeda_layer_desc *d)
{
    const int c = route_ksplit(d);
    if (c == 1) return 0;
    const size_t Tpad = (size_t)ceil_div(d->T, kRouteTokens) * kRouteTokens;
    return (size_t)c * Tpad * ceil_div(d->N + d->Z, 32) * 32 * sizeof(float);
}

// One kernel, no scratch, 64 tokens per workgroup: for token counts that fill the device with such blocks.
// The router kernels use more LDS than a launch gets by default: opt in once per kernel and device.
template <int NB, int TB>
static bool route_lds_opt_in(int lds_bytes)
{
    static bool done[kMaxDevices] = {};  // per instantiation and device; idempotent, so a race between host threads is harmless
    const int dev = current_device();
    if (dev < 0) return false;
    if (!done[dev]) {
        if (hipFuncSetAttribute((const void *)route_bf16_kernel<NB, TB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                lds_bytes) != hipSuccess)
            return false;
        done[dev] = true;
    }
    return true;
}

// Optional per-block outputs of a router launch (see publish_blocks); all NULL / 0 when not wanted.
struct RouteExtras {
    uint8_t *cnt8;
    int cnt_ld;
    float *p_part;
};

template <int NB>
static int launch_route_bf16_wide(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias,
                                  int32_t *ids, float *gates, const RouteExtras &ex, hipStream_t s)
{
    const int blocks = ceil_div(d->T, 64);
    constexpr int lds_bytes = route_stages(NB, 2) * (64 + 32 * NB) * 128;
    if (!route_lds_opt_in<NB, 2>(lds_bytes)) return ZEDA_EHIP;
    route_bf16_kernel<NB, 2><<<dim3(blocks, 1), kRouteThreads, lds_bytes, s>>>(
        (const bf16_t *)x, (const bf16_t *)wr, bias, d->T, d->H, d->N, d->N + d->Z, d->K, d->gate_norm, ids, gates, nullptr,
        blocks * 64, ex.cnt8, ex.cnt_ld, ex.p_part);
    return last_launch_status();
}

// More than 256 blocks of 32 tokens: a second round of 32-token workgroups would start behind the first (8500 tokens:
// 38 us); 64-token blocks run in one round and read the router rows half as often (33 us from 8193 to 16384 tokens).
constexpr int kRouteWideTokens = 8193;

template <int NB>
static int launch_route_bf16(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias, int32_t *ids,
                             float *gates, float *partial, const RouteExtras &ex, hipStream_t s)
{
    if constexpr (NB <= 6) {
        if (d->T >= kRouteWideTokens) return launch_route_bf16_wide<NB>(d, x, wr, bias, ids, gates, ex, s);
    }
    const int blocks = ceil_div(d->T, kRouteTokens), Tpad = blocks * kRouteTokens;
    const int c = partial ? route_ksplit(d) : 1;
    constexpr int lds_bytes = route_stages(NB) * (kRouteTokens + 32 * NB) * 128;
    if (!route_lds_opt_in<NB, 1>(lds_bytes)) return ZEDA_EHIP;
    route_bf16_kernel<NB, 1><<<dim3(blocks, c), kRouteThreads, lds_bytes, s>>>(
        (const bf16_t *)x, (const bf16_t *)wr, bias, d->T, d->H, d->N, d->N + d->Z, d->K, d->gate_norm, ids, gates,
        c > 1 ? partial : nullptr, Tpad, ex.cnt8, ex.cnt_ld, ex.p_part);
    if (c == 1) return last_launch_status();
    const dim3 sgrid(ceil_div(d->T, kSelectTokens));
    const int NE = d->N + d->Z;
    if (c == 2)
        route_select_kernel<NB, 2><<<sgrid, kRouteThreads, 0, s>>>(partial, Tpad, bias, d->T, d->N, NE, d->K, d->gate_norm, ids, gates, ex.cnt8, ex.cnt_ld, ex.p_part);
    else if (c == 4)
        route_select_kernel<NB, 4><<<sgrid, kRouteThreads, 0, s>>>(partial, Tpad, bias, d->T, d->N, NE, d->K, d->gate_norm, ids, gates, ex.cnt8, ex.cnt_ld, ex.p_part);
    else
        route_select_kernel<NB, 8><<<sgrid, kRouteThreads, 0, s>>>(partial, Tpad, bias, d->T, d->N, NE, d->K, d->gate_norm, ids, gates, ex.cnt8, ex.cnt_ld, ex.p_part);
    return last_launch_status();
}

static int launch_route_bf16_any(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias, int32_t *ids,
                                 float *gates, float *partial, const RouteExtras &ex, hipStream_t s)
{
    switch (ceil_div(d->N + d->Z, 32)) {
        case 1: return launch_route_bf16<1>(d, x, wr, bias, ids, gates, partial, ex, s);
        case 2: return launch_route_bf16<2>(d, x, wr, bias, ids, gates, partial, ex, s);
        case 3: return launch_route_bf16<3>(d, x, wr, bias, ids, gates, partial, ex, s);
        case 4: return launch_route_bf16<4>(d, x, wr, bias, ids, gates, partial, ex, s);
        case 5: return launch_route_bf16<5>(d, x, wr, bias, ids, gates, partial, ex, s);
        case 6: return launch_route_bf16<6>(d, x, wr, bias, ids, gates, partial, ex, s);
        case 7: return launch_route_bf16<7>(d, x, wr, bias, ids, gates, partial, ex, s);
        default: return launch_route_bf16<8>(d, x, wr, bias, ids, gates, partial, ex, s);
    }
}

int route_counts_ld(const zeda_layer_desc *d) { return (int)align_up((size_t)ceil_div(d->T, 16), 16); }
size_t route_counts_bytes(const zeda_layer_desc *d) { return align_up((size_t)(d->N + d->Z) * route_counts_ld(d), 256); }
bool route_counts_supported(const zeda_layer_desc *d) { return d->dtype == ZEDA_BF16; }

// ---------------------------------------------------------------------------------------------
// Batch routing statistics (Section 2.2, Eq. 4-6): f_i, P_i, the group sums and the forward values of the
// two auxiliary losses, over all T tokens as the batch.  bf16: the router kernels themselves leave, per block of 16
// tokens, the slots on every expert and the sums of the routing probabilities (the logits, the softmax and the
// selected set are in their registers anyway), and one final workgroup adds the blocks up in order
// (route_stats_final_kernel).  fp32: logits to scratch (route_f32_kernel), per-block sums (route_stats_kernel), the
// same final workgroup.  Every floating-point sum runs in a fixed order.
// ---------------------------------------------------------------------------------------------
constexpr int kStatsTokens = 64;  // tokens per workgroup of route_stats_kernel: four batches of four per wave

template <int NC>
__global__ __launch_bounds__(kRouteThreads) void route_stats_kernel(const float *__restrict__ logits, int nsplit, int Tpad,
                                                                    int LDg, const float *__restrict__ bias, int T, int NE,
                                                                    int K, float *__restrict__ p_part,
                                                                    int32_t *__restrict__ f_part)
{
    __shared__ float s_p[16][kMaxExperts];
    __shared__ int s_f[16][kMaxExperts];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, row = lane >> 4;
    const int t0 = blockIdx.x * kStatsTokens;
    float psum[NC];
    int fcnt[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) { psum[c] = 0.f; fcnt[c] = 0; }
    for (int batch = 0; batch < kStatsTokens / 16; ++batch) {
        const int t = t0 + batch * 16 + wave * 4 + row;
        const bool ok = t < T;
        float cand[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) cand[c] = -INFINITY;
        if (ok) {
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (l16 + 16 * c < NE) cand[c] = logits[(size_t)t * LDg + l16 + 16 * c];
            for (int q = 1; q < nsplit; ++q) {
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    if (l16 + 16 * c < NE) cand[c] += logits[((size_t)q * Tpad + t) * LDg + l16 + 16 * c];
            }
            if (bias) {
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    if (l16 + 16 * c < NE) cand[c] += bias[l16 + 16 * c];
            }
        }
        // probabilities: softmax over all N+Z logits of the token (the row)
        float m = cand[0];
#pragma unroll
        for (int c = 1; c < NC; ++c) m = fmaxf(m, cand[c]);
        m = row_max(m);
        float ex[NC], sacc = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            ex[c] = (ok && l16 + 16 * c < NE) ? expf(cand[c] - m) : 0.f;
            sacc += ex[c];
        }
        const float all = row_sum(sacc);
        if (ok) {
#pragma unroll
            for (int c = 0; c < NC; ++c) psum[c] += ex[c] / all;
        }
        // the top-K set, as in select_rows: K rounds of (row maximum, lowest index among equals)
        for (int j = 0; j < K; ++j) {
            float mm = cand[0];
#pragma unroll
            for (int c = 1; c < NC; ++c) mm = fmaxf(mm, cand[c]);
            mm = row_max(mm);
            int mine = INT_MAX;
#pragma unroll
            for (int c = NC - 1; c >= 0; --c)
                if (cand[c] == mm) mine = l16 + 16 * c;
            const int win = row_min(mine);
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (win == l16 + 16 * c) {
                    cand[c] = -INFINITY;
                    if (ok) ++fcnt[c];
                }
        }
    }
    // 16 (wave, row) partial tables -> one per workgroup, added in table order
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        s_p[wave * 4 + row][l16 + 16 * c] = psum[c];
        s_f[wave * 4 + row][l16 + 16 * c] = fcnt[c];
    }
    __syncthreads();
    if (tid < NE) {
        float ps = 0.f;
        int fs = 0;
#pragma unroll
        for (int r = 0; r < 16; ++r) { ps += s_p[r][tid]; fs += s_f[r][tid]; }
        p_part[(size_t)blockIdx.x * NE + tid] = ps;
        f_part[(size_t)blockIdx.x * NE + tid] = fs;
    }
}

// f_part: [nblocks][NE] int32 counts, or NULL: then cnt8[e][cnt_ld] holds them as bytes
__global__ __launch_bounds__(kRouteThreads) void route_stats_final_kernel(const float *__restrict__ p_part,
                                                                          const int32_t *__restrict__ f_part,
                                                                          const uint8_t *__restrict__ cnt8, int cnt_ld, int nblocks,
                                                                          int T, int N, int NE, int K, float alpha, float w,
                                                                          float *__restrict__ f, float *__restrict__ P,
                                                                          float *__restrict__ summary)
{
    __shared__ float s_f[kMaxExperts], s_P[kMaxExperts];
    const int e = threadIdx.x;
    if (e < NE) {
        float ps = 0.f;
        long long fs = 0;
        for (int b = 0; b < nblocks; ++b) {
            ps += p_part[(size_t)b * NE + e];
            fs += f_part ? f_part[(size_t)b * NE + e] : (int)cnt8[(size_t)e * cnt_ld + b];
        }
        s_P[e] = ps / (float)T;
        s_f[e] = (float)((double)fs / (double)T);
        f[e] = s_f[e];
        P[e] = s_P[e];
    }
    __syncthreads();
    if (e == 0) {
        float fE = 0.f, PE = 0.f, fZ = 0.f, PZ = 0.f, dot = 0.f;
        for (int i = 0; i < NE; ++i) {
            dot += s_f[i] * s_P[i];
            if (i < N) { fE += s_f[i]; PE += s_P[i]; } else { fZ += s_f[i]; PZ += s_P[i]; }
        }
        const int Z = NE - N;
        summary[0] = fE; summary[1] = PE; summary[2] = fZ; summary[3] = PZ;
        summary[4] = fZ / (float)K;
        summary[5] = alpha * (float)NE / (float)K * dot;                                   // Eq. 4
        summary[6] = alpha * ((float)N + (float)Z * w) / (float)K *
                     (fE * PE / (float)N + (Z > 0 ? fZ * PZ / ((float)Z * w) : 0.f));       // Eq. 5-6
    }
}

// scratch: the logit tables, then the per-block sums
static size_t stats_logits_bytes(const zeda_layer_desc *d)
{
    const size_t Tpad = (size_t)ceil_div(d->T, kRouteTokens) * kRouteTokens;
    return align_up((size_t)route_ksplit(d) * Tpad * ceil_div(d->N + d->Z, 32) * 32 * sizeof(float), 256);
}
size_t routing_stats_ws_bytes(const zeda_layer_desc *d)
{
    const size_t NE = (size_t)(d->N + d->Z);
    if (d->dtype == ZEDA_BF16)  // split-k scratch of the router, per-block counts, per-block probability sums
        return align_up(route_ws_bytes(d), 256) + route_counts_bytes(d) + align_up((size_t)ceil_div(d->T, 16) * NE * 4, 256);
    const size_t nblk = (size_t)ceil_div(d->T, kStatsTokens);
    return stats_logits_bytes(d) + align_up(nblk * NE * 4, 256) * 2;
}

int launch_routing_stats(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias, float alpha, float w,
                         float *f, float *P, float *summary, void *ws, hipStream_t s)
{
    const int NE = d->N + d->Z;
    if (d->dtype == ZEDA_BF16) {
        float *partial = route_ws_bytes(d) ? (float *)ws : nullptr;
        uint8_t *cnt8 = (uint8_t *)ws + align_up(route_ws_bytes(d), 256);
        float *p_part = (float *)(cnt8 + route_counts_bytes(d));
        const RouteExtras ex = {cnt8, route_counts_ld(d), p_part};
        const int rc = launch_route_bf16_any(d, x, wr, bias, nullptr, nullptr, partial, ex, s);
        if (rc != ZEDA_OK) return rc;
        route_stats_final_kernel<<<1, kRouteThreads, 0, s>>>(p_part, nullptr, cnt8, ex.cnt_ld, ceil_div(d->T, 16), d->T, d->N, NE,
                                                             d->K, alpha, w, f, P, summary);
        return last_launch_status();
    }
    const int NB = ceil_div(NE, 32), LDg = NB * 32;
    const int Tpad = ceil_div(d->T, kRouteTokens) * kRouteTokens, nblk = ceil_div(d->T, kStatsTokens);
    float *logits = (float *)ws;
    float *p_part = (float *)((char *)ws + stats_logits_bytes(d));
    int32_t *f_part = (int32_t *)((char *)p_part + align_up((size_t)nblk * NE * 4, 256));
    route_f32_kernel<<<ceil_div(d->T, kRouteF32Tokens), kRouteThreads, 0, s>>>(
        (const float *)x, (const float *)wr, bias, d->T, d->H, d->N, NE, d->K, d->gate_norm, nullptr, nullptr, logits, LDg);
    if (hipGetLastError() != hipSuccess) return ZEDA_EHIP;
#define ZEDA_STATS(NC) route_stats_kernel<NC><<<nblk, kRouteThreads, 0, s>>>(logits, 1, Tpad, LDg, bias, d->T, NE, d->K, p_part, f_part)
    switch (ceil_div(NE, 16)) {
        case 1: ZEDA_STATS(1); break;   case 2: ZEDA_STATS(2); break;   case 3: ZEDA_STATS(3); break;
        case 4: ZEDA_STATS(4); break;   case 5: ZEDA_STATS(5); break;   case 6: ZEDA_STATS(6); break;
        case 7: ZEDA_STATS(7); break;   case 8: ZEDA_STATS(8); break;   case 9: ZEDA_STATS(9); break;
        case 10: ZEDA_STATS(10); break; case 11: ZEDA_STATS(11); break; case 12: ZEDA_STATS(12); break;
        case 13: ZEDA_STATS(13); break; case 14: ZEDA_STATS(14); break; case 15: ZEDA_STATS(15); break;
        default: ZEDA_STATS(16); break;
    }
#undef ZEDA_STATS
    if (hipGetLastError() != hipSuccess) return ZEDA_EHIP;
    route_stats_final_kernel<<<1, kRouteThreads, 0, s>>>(p_part, f_part, nullptr, 0, nblk, d->T, d->N, NE, d->K, alpha, w, f, P,
                                                         summary);
    return last_launch_status();
}

int launch_route(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias, int32_t *ids,
                 float *gates, float *partial, uint8_t *cnt8, hipStream_t s)
{
    const int NE = d->N + d->Z;
    if (d->dtype == ZEDA_BF16) {
        const RouteExtras ex = {cnt8, cnt8 ? route_counts_ld(d) : 0, nullptr};
        return launch_route_bf16_any(d, x, wr, bias, ids, gates, partial, ex, s);
    }
    dim3 grid(ceil_div(d->T, kRouteF32Tokens));
    route_f32_kernel<<<grid, kRouteThreads, 0, s>>>((const float *)x, (const float *)wr, bias, d->T, d->H, d->N, NE, d->K,
                                                    d->gate_norm, ids, gates, nullptr, 0);
    return last_launch_status();
}

}  // namespace zeda
