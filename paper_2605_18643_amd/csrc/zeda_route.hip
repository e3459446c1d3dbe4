// Router of the augmented expert pool (Section 2.1): logits over N normal + Z zero experts, the
// top-K set with a deterministic lower-index tie-break, and the routing weights (Section 4.3.4 for
// the normalisation choices).  One fused kernel: projection -> LDS -> wave-level selection.
#include "zeda_internal.h"

namespace zeda {

constexpr int kRouteTokens = 32;  // tokens per workgroup of the bf16 kernel (one MFMA column block)
constexpr int kRouteThreads = 256;

// (value, index) butterfly: every lane ends with the maximum value, ties to the lower index.
__device__ __forceinline__ void wave_argmax(float &v, int &i)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        float ov = __shfl_xor(v, off);
        int oi = __shfl_xor(i, off);
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// Selection and gates for one token, executed by one wave.  `row` points at the token's NE fp32
// logits in LDS.  Lane c-th candidate is expert lane + 64*c.
__device__ __forceinline__ void select_token(const float *row, int NE, int N, int K, int gate_norm, int32_t *ids_out,
                                             float *gates_out)
{
    const int lane = threadIdx.x & 63;
    float cand[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        int e = lane + 64 * c;
        cand[c] = e < NE ? row[e] : -INFINITY;
    }
    float all_max = fmaxf(fmaxf(cand[0], cand[1]), fmaxf(cand[2], cand[3]));
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) all_max = fmaxf(all_max, __shfl_xor(all_max, off));
    float all_sum = 0.f;
    if (gate_norm == ZEDA_GATE_SOFTMAX) {
#pragma unroll
        for (int c = 0; c < 4; ++c) all_sum += (lane + 64 * c < NE) ? expf(cand[c] - all_max) : 0.f;
        all_sum = wave_sum(all_sum);
    }
    int my_id = 0;
    float my_logit = -INFINITY;
    for (int j = 0; j < K; ++j) {
        float bv = cand[0];
        int bi = lane;
#pragma unroll
        for (int c = 1; c < 4; ++c)
            if (cand[c] > bv) { bv = cand[c]; bi = lane + 64 * c; }
        wave_argmax(bv, bi);
        if ((bi & 63) == lane) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if ((bi >> 6) == c) cand[c] = -INFINITY;
        }
        if (lane == j) { my_id = bi; my_logit = bv; }
    }
    // lanes 0..K-1 hold the slots in descending-logit order
    const bool slot = lane < K;
    float ex = slot ? expf(my_logit - all_max) : 0.f;
    float denom;
    if (gate_norm == ZEDA_GATE_SOFTMAX) denom = all_sum;
    else if (gate_norm == ZEDA_GATE_TOPK_NORM) denom = wave_sum(ex);
    else denom = wave_sum((slot && my_id < N) ? ex : 0.f);
    if (slot) {
        ids_out[lane] = my_id;
        gates_out[lane] = denom > 0.f ? ex / denom : 0.f;
    }
}

// bf16 router.  A workgroup owns kRouteTokens tokens and all NE experts; its 4 waves split the hidden
// dimension, each accumulating NB 32x32 MFMA blocks (experts are MFMA rows, tokens MFMA columns), then
// the partial sums are added in LDS in wave order and each wave selects for 8 tokens.
// Inside every 64-wide k chunk lane half h and step s read elements 32h+8s..+8 of both operands: the
// sum over k does not depend on the order, and each lane then walks 64 contiguous bytes.
template <int NB>
__global__ __launch_bounds__(kRouteThreads) void route_bf16_kernel(const bf16_t *__restrict__ x,
                                                                   const bf16_t *__restrict__ wr,
                                                                   const float *__restrict__ bias, int T, int H, int N,
                                                                   int NE, int K, int gate_norm,
                                                                   int32_t *__restrict__ ids, float *__restrict__ gates)
{
    constexpr int LD = NB * 32 + 1;
    __shared__ float lg[kRouteTokens * LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * kRouteTokens;
    const int col = lane & 31, half = lane >> 5;
    // 64-wide k chunks are dealt to the four waves round-robin (H is a multiple of 64)
    const bf16_t *xrow = x + (size_t)min(t0 + col, T - 1) * H + half * 32;
    const bf16_t *wrow[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) wrow[b] = wr + (size_t)min(b * 32 + col, NE - 1) * H + half * 32;

    f32x16 acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

    for (int k0 = wave * 64; k0 < H; k0 += 4 * 64) {
        bf16x8 xb[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) xb[s] = *reinterpret_cast<const bf16x8 *>(xrow + k0 + s * 8);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            bf16x8 wa[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) wa[s] = *reinterpret_cast<const bf16x8 *>(wrow[b] + k0 + s * 8);
#pragma unroll
            for (int s = 0; s < 4; ++s) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[s], xb[s], acc[b], 0, 0, 0);
        }
    }

    // acc[b][v]: expert 32b + 8(v/4) + 4*half + v%4, token col.  Add the four k-quarters in wave order.
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int e = b * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                    float *p = &lg[col * LD + e];
                    *p = (w == 0) ? acc[b][v] : *p + acc[b][v];
                }
        }
        __syncthreads();
    }
    if (bias) {
        for (int i = tid; i < kRouteTokens * NE; i += kRouteThreads) {
            int tk = i / NE, e = i - tk * NE;
            lg[tk * LD + e] += bias[e];
        }
        __syncthreads();
    }
    for (int tk = wave; tk < kRouteTokens; tk += 4) {
        int t = t0 + tk;
        if (t < T) select_token(&lg[tk * LD], NE, N, K, gate_norm, ids + (size_t)t * K, gates + (size_t)t * K);
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
                                                                  int32_t *__restrict__ ids, float *__restrict__ gates)
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
    if (bias) {
        for (int i = tid; i < kRouteF32Tokens * NE; i += kRouteThreads) lg[(i / NE) * LD + (i % NE)] += bias[i % NE];
        __syncthreads();
    }
    for (int tk = wave; tk < kRouteF32Tokens; tk += 4) {
        int t = t0 + tk;
        if (t < T) select_token(&lg[tk * LD], NE, N, K, gate_norm, ids + (size_t)t * K, gates + (size_t)t * K);
    }
}

template <int NB>
static void launch_route_bf16(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias, int32_t *ids,
                              float *gates, hipStream_t s)
{
    dim3 grid(ceil_div(d->T, kRouteTokens));
    route_bf16_kernel<NB><<<grid, kRouteThreads, 0, s>>>((const bf16_t *)x, (const bf16_t *)wr, bias, d->T, d->H, d->N,
                                                         d->N + d->Z, d->K, d->gate_norm, ids, gates);
}

int launch_route(const zeda_layer_desc *d, const void *x, const void *wr, const float *bias, int32_t *ids,
                 float *gates, hipStream_t s)
{
    const int NE = d->N + d->Z;
    if (d->dtype == ZEDA_BF16) {
        switch (ceil_div(NE, 32)) {
            case 1: launch_route_bf16<1>(d, x, wr, bias, ids, gates, s); break;
            case 2: launch_route_bf16<2>(d, x, wr, bias, ids, gates, s); break;
            case 3: launch_route_bf16<3>(d, x, wr, bias, ids, gates, s); break;
            case 4: launch_route_bf16<4>(d, x, wr, bias, ids, gates, s); break;
            case 5: launch_route_bf16<5>(d, x, wr, bias, ids, gates, s); break;
            case 6: launch_route_bf16<6>(d, x, wr, bias, ids, gates, s); break;
            case 7: launch_route_bf16<7>(d, x, wr, bias, ids, gates, s); break;
            default: launch_route_bf16<8>(d, x, wr, bias, ids, gates, s); break;
        }
    } else {
        dim3 grid(ceil_div(d->T, kRouteF32Tokens));
        route_f32_kernel<<<grid, kRouteThreads, 0, s>>>((const float *)x, (const float *)wr, bias, d->T, d->H, d->N, NE,
                                                        d->K, d->gate_norm, ids, gates);
    }
    return last_launch_status();
}

}  // namespace zeda
