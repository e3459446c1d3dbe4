// Eq. 1 of Section 2.1, the weighted sum back in token order:
//   out[t,:] = sum over the token's slots on normal experts of g~ * (expert output of that slot).
// A gather by token: one workgroup per token reads at most K rows of y_slot through slot_to_row and
// accumulates in fp32 in ascending slot rank, so there are no atomics, the order of additions is
// fixed, and every load and store is a contiguous 16-byte piece per lane.  The token's real slots are
// first compacted (one ballot) so that the row loads can be issued four at a time without a branch per
// slot.  A token with no real slot stores exact zeros (its sum is empty).
// Copy-expert variant (Appendix B): a slot on a parameter-free expert contributes g~ * h instead of nothing;
// those weights are summed in ascending slot rank and the term is added after the real slots.
// Block variant (FUSE): the workgroup holds the token's whole row, so in a pre-norm residual chain it also adds
// the row to the residual stream in place and writes the RMSNorm of the new stream row, the next layer's
// input: one pass over the row instead of three kernels.
#include "zeda_internal.h"

namespace zeda {

constexpr int kCombineThreads = 256;

template <typename T> struct Vec;
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    typedef bf16x8 type;
};
template <> struct Vec<float> {
    static constexpr int N = 4;
    typedef f32x4 type;
};

// vectors of a row one thread keeps in registers between the residual add and the norm (FUSE)
constexpr int kFuseVecs = 4;

// x_res, gamma, eps, xn_next: FUSE only.  x (the layer input, COPY only) and xn_next may be the same buffer:
// a thread reads its pieces of a row before it writes them.
template <typename T, bool COPY, bool FUSE>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(const T *__restrict__ y_slot,
                                                                  const int32_t *__restrict__ ids,
                                                                  const float *__restrict__ gates,
                                                                  const int32_t *__restrict__ slot_to_row, const T *x,
                                                                  T *__restrict__ out, int H, int N, int NE, int K,
                                                                  int rows_cap, T *__restrict__ x_res,
                                                                  const T *__restrict__ gamma, float eps, T *xn_next)
{
    constexpr int VN = Vec<T>::N;
    typedef typename Vec<T>::type vec_t;
    // the token's real slots, compacted in ascending slot rank: row in y_slot and routing weight
    __shared__ int s_row[kMaxK + 4];
    __shared__ float s_g[kMaxK + 4];
    __shared__ int s_n;
    __shared__ float s_zg[kMaxK];  // COPY: routing weight of slot j if it is on a parameter-free expert, else 0
    const int t = blockIdx.x;
    if (threadIdx.x < 64) {
        const int j = threadIdx.x;
        int r = -1;
        float g = 0.f;
        if (j < K) {
            const int s = t * K + j;
            const int e = ids[s];
            r = slot_to_row[s];
            g = gates[s];
            if (COPY) s_zg[j] = (e >= N && e < NE) ? g : 0.f;
            if (!(e >= 0 && e < N && r >= 0 && r < rows_cap)) r = -1;  // a slot on a zero expert (or a bad index)
        }
        const unsigned long long real = __ballot(r >= 0);
        if (r >= 0) {
            const int pos = __popcll(real & ((1ull << j) - 1ull));
            s_row[pos] = r;
            s_g[pos] = g;
        }
        const int n = __popcll(real);
        if (j == 0) s_n = n;
        if (j < 4) {  // padding of the last group of four: any valid row, weight never used
            s_row[n + j] = 0;
            s_g[n + j] = 0.f;
        }
    }
    __syncthreads();
    const int n = s_n;
    float gz = 0.f;
    if (COPY)
        for (int j = 0; j < K; ++j) gz += s_zg[j];  // ascending slot rank, the same on every thread
    float keep[FUSE ? kFuseVecs : 1][VN];  // FUSE: the new residual row as stored, for the norm
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < (FUSE ? kFuseVecs : 1); ++c) {
        // FUSE: at most kFuseVecs vectors per thread (checked by the launcher), the loop unrolls into registers
        for (int v = threadIdx.x + c * kCombineThreads; v < H / VN; v += FUSE ? H : kCombineThreads) {
            float acc[VN];
#pragma unroll
            for (int i = 0; i < VN; ++i) acc[i] = 0.f;
            // four rows at a time, so that their loads are in flight together; a padded entry is loaded (row 0, or
            // nothing but readable memory when there are no rows at all) and left out of the sum
            for (int j0 = 0; j0 < n; j0 += 4) {
                vec_t y[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) y[q] = *reinterpret_cast<const vec_t *>(y_slot + (size_t)s_row[j0 + q] * H + (size_t)v * VN);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool use = j0 + q < n;
                    const float g = s_g[j0 + q];
#pragma unroll
                    for (int i = 0; i < VN; ++i) acc[i] = use ? fmaf(g, (float)y[q][i], acc[i]) : acc[i];
                }
            }
            if (COPY) {
                const vec_t xv = *reinterpret_cast<const vec_t *>(x + (size_t)t * H + (size_t)v * VN);
#pragma unroll
                for (int i = 0; i < VN; ++i) acc[i] = fmaf(gz, (float)xv[i], acc[i]);
            }
            vec_t o;
            if (FUSE) {
                const vec_t rv = *reinterpret_cast<const vec_t *>(x_res + (size_t)t * H + (size_t)v * VN);
#pragma unroll
                for (int i = 0; i < VN; ++i) {
                    o[i] = (T)((float)rv[i] + acc[i]);
                    keep[c][i] = (float)o[i];
                    ss = fmaf(keep[c][i], keep[c][i], ss);
                }
                *reinterpret_cast<vec_t *>(x_res + (size_t)t * H + (size_t)v * VN) = o;
            } else {
#pragma unroll
                for (int i = 0; i < VN; ++i) o[i] = (T)acc[i];
                *reinterpret_cast<vec_t *>(out + (size_t)t * H + (size_t)v * VN) = o;
            }
        }
    }
    if (FUSE && xn_next) {
        __shared__ float part[kCombineThreads / 64];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
        __syncthreads();
        const float total = (part[0] + part[1]) + (part[2] + part[3]);
        const float scale = 1.0f / sqrtf(total / (float)H + eps);
#pragma unroll
        for (int c = 0; c < kFuseVecs; ++c) {
            const int v = threadIdx.x + c * kCombineThreads;
            if (v < H / VN) {
                vec_t o;
                if (gamma) {
                    const vec_t gv = *reinterpret_cast<const vec_t *>(gamma + (size_t)v * VN);
#pragma unroll
                    for (int i = 0; i < VN; ++i) o[i] = (T)(keep[c][i] * scale * (float)gv[i]);
                } else {
#pragma unroll
                    for (int i = 0; i < VN; ++i) o[i] = (T)(keep[c][i] * scale);
                }
                *reinterpret_cast<vec_t *>(xn_next + (size_t)t * H + (size_t)v * VN) = o;
            }
        }
    }
}

template <typename T>
static void launch_combine_t(const zeda_layer_desc *d, const void *y_slot, const int32_t *ids, const float *gates,
                             const int32_t *slot_to_row, const void *x, void *out, hipStream_t s)
{
    const int S = d->T * d->K, NE = d->N + d->Z;
    if (d->free_expert == ZEDA_EXPERT_COPY)
        combine_kernel<T, true, false><<<d->T, kCombineThreads, 0, s>>>((const T *)y_slot, ids, gates, slot_to_row,
                                                                       (const T *)x, (T *)out, d->H, d->N, NE, d->K, S,
                                                                       nullptr, nullptr, 0.f, nullptr);
    else
        combine_kernel<T, false, false><<<d->T, kCombineThreads, 0, s>>>((const T *)y_slot, ids, gates, slot_to_row,
                                                                        nullptr, (T *)out, d->H, d->N, NE, d->K, S,
                                                                        nullptr, nullptr, 0.f, nullptr);
}

template <typename T>
static void launch_combine_block_t(const zeda_layer_desc *d, const void *y_slot, const int32_t *ids, const float *gates,
                                   const int32_t *slot_to_row, const void *x, void *x_res, const void *gamma, float eps,
                                   void *xn_next, hipStream_t s)
{
    const int S = d->T * d->K, NE = d->N + d->Z;
    if (d->free_expert == ZEDA_EXPERT_COPY)
        combine_kernel<T, true, true><<<d->T, kCombineThreads, 0, s>>>((const T *)y_slot, ids, gates, slot_to_row,
                                                                      (const T *)x, nullptr, d->H, d->N, NE, d->K, S,
                                                                      (T *)x_res, (const T *)gamma, eps, (T *)xn_next);
    else
        combine_kernel<T, false, true><<<d->T, kCombineThreads, 0, s>>>((const T *)y_slot, ids, gates, slot_to_row,
                                                                       nullptr, nullptr, d->H, d->N, NE, d->K, S,
                                                                       (T *)x_res, (const T *)gamma, eps, (T *)xn_next);
}

int launch_combine(const zeda_layer_desc *d, const void *y_slot, const int32_t *ids, const float *gates,
                   const int32_t *slot_to_row, const void *x, void *out, hipStream_t s)
{
    if (d->dtype == ZEDA_BF16) launch_combine_t<bf16_t>(d, y_slot, ids, gates, slot_to_row, x, out, s);
    else launch_combine_t<float>(d, y_slot, ids, gates, slot_to_row, x, out, s);
    return last_launch_status();
}

bool combine_block_supported(const zeda_layer_desc *d)
{
    const int vn = d->dtype == ZEDA_BF16 ? Vec<bf16_t>::N : Vec<float>::N;
    return d->H / vn <= kFuseVecs * kCombineThreads;
}

int launch_combine_block(const zeda_layer_desc *d, const void *y_slot, const int32_t *ids, const float *gates,
                         const int32_t *slot_to_row, const void *x, void *x_res, const void *gamma, float eps,
                         void *xn_next, hipStream_t s)
{
    if (!combine_block_supported(d)) return ZEDA_EUNSUPPORTED;
    if (d->dtype == ZEDA_BF16) launch_combine_block_t<bf16_t>(d, y_slot, ids, gates, slot_to_row, x, x_res, gamma, eps, xn_next, s);
    else launch_combine_block_t<float>(d, y_slot, ids, gates, slot_to_row, x, x_res, gamma, eps, xn_next, s);
    return last_launch_status();
}

}  // namespace zeda
