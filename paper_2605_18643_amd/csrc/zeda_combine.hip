// Eq. 1 of Section 2.1, the weighted sum back in token order:
//   out[t,:] = sum over the token's slots on normal experts of g~ * (expert output of that slot).
// A gather by token: one workgroup per token reads at most K rows of y_slot through slot_to_row and
// accumulates in fp32 in ascending slot rank, so there are no atomics, the order of additions is
// fixed, and every load and store is a contiguous 16-byte piece per lane.  A token with no real slot
// stores exact zeros (its sum is empty).
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

template <typename T>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(const T *__restrict__ y_slot,
                                                                  const int32_t *__restrict__ ids,
                                                                  const float *__restrict__ gates,
                                                                  const int32_t *__restrict__ slot_to_row,
                                                                  T *__restrict__ out, int H, int N, int K, int rows_cap)
{
    constexpr int VN = Vec<T>::N;
    typedef typename Vec<T>::type vec_t;
    const int t = blockIdx.x;
    // slot j of the token: row in y_slot, or -1 when the slot is on a zero expert (kept in registers)
    int row[kMaxK];
    float g[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
        row[j] = -1;
        g[j] = 0.f;
        if (j < K) {
            const int s = t * K + j;
            const int e = ids[s];
            const int r = slot_to_row[s];
            if (e >= 0 && e < N && r >= 0 && r < rows_cap) {
                row[j] = r;
                g[j] = gates[s];
            }
        }
    }
    for (int v = threadIdx.x; v < H / VN; v += kCombineThreads) {
        float acc[VN];
#pragma unroll
        for (int i = 0; i < VN; ++i) acc[i] = 0.f;
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) {
            if (row[j] >= 0) {
                const vec_t y = *reinterpret_cast<const vec_t *>(y_slot + (size_t)row[j] * H + (size_t)v * VN);
#pragma unroll
                for (int i = 0; i < VN; ++i) acc[i] = fmaf(g[j], (float)y[i], acc[i]);
            }
        }
        vec_t o;
#pragma unroll
        for (int i = 0; i < VN; ++i) o[i] = (T)acc[i];
        *reinterpret_cast<vec_t *>(out + (size_t)t * H + (size_t)v * VN) = o;
    }
}

int launch_combine(const zeda_layer_desc *d, const void *y_slot, const int32_t *ids, const float *gates,
                   const int32_t *slot_to_row, void *out, hipStream_t s)
{
    if (d->dtype == ZEDA_BF16)
        combine_kernel<bf16_t><<<d->T, kCombineThreads, 0, s>>>((const bf16_t *)y_slot, ids, gates, slot_to_row,
                                                               (bf16_t *)out, d->H, d->N, d->K, d->T * d->K);
    else
        combine_kernel<float><<<d->T, kCombineThreads, 0, s>>>((const float *)y_slot, ids, gates, slot_to_row,
                                                              (float *)out, d->H, d->N, d->K, d->T * d->K);
    return last_launch_status();
}

}  // namespace zeda
