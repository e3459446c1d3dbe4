// Glue kernels of the layer-stack workload (a chain of MoE layers with a pre-norm residual block around
// each, x <- x + MoE_l(RMSNorm(x)), no attention).  The paper's model of the layer leaves norms and
// residuals out (Appendix D counts matrix products only); they exist here so that a 48-layer stack can be
// run and timed with and without zero experts.  Norm arithmetic is fp32; the residual stream keeps the
// layer's element type.
#include "zeda_internal.h"

namespace zeda {

constexpr int kStackThreads = 256;

template <typename T>
__global__ __launch_bounds__(kStackThreads) void rmsnorm_kernel(const T *__restrict__ x, const T *__restrict__ gamma,
                                                                float eps, T *__restrict__ out, int H)
{
    __shared__ float part[kStackThreads / 64];
    const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const T *xr = x + (size_t)t * H;
    float ss = 0.f;
    for (int h = tid; h < H; h += kStackThreads) {
        const float v = (float)xr[h];
        ss = fmaf(v, v, ss);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if (lane == 0) part[wave] = ss;
    __syncthreads();
    const float total = (part[0] + part[1]) + (part[2] + part[3]);
    const float scale = 1.0f / sqrtf(total / (float)H + eps);
    for (int h = tid; h < H; h += kStackThreads) {
        float v = (float)xr[h] * scale;
        if (gamma) v *= (float)gamma[h];
        out[(size_t)t * H + h] = (T)v;
    }
}

template <typename T>
__global__ __launch_bounds__(kStackThreads) void residual_add_kernel(T *__restrict__ x, const T *__restrict__ y, size_t n)
{
    size_t i = blockIdx.x * (size_t)kStackThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kStackThreads;
    for (; i < n; i += stride) x[i] = (T)((float)x[i] + (float)y[i]);
}

// Router rows of the zero experts (Section 2.1, router initialisation): Gaussian with the mean and the
// variance of the N*H original router parameters; the standard-normal draws are an input.  One workgroup: the
// reduction is a fixed tree over fixed per-thread strides (fp64), so the rows are the same on every run.
constexpr int kInitThreads = 1024;
template <typename T>
__global__ __launch_bounds__(kInitThreads) void init_zero_rows_kernel(T *__restrict__ wr, const float *__restrict__ normals,
                                                                      int N, int Z, int H, float *__restrict__ stats)
{
    __shared__ double red[kInitThreads];
    __shared__ double s_mean, s_sd;
    const int tid = threadIdx.x;
    const size_t n = (size_t)N * H;
    auto block_sum = [&](double v) {
        red[tid] = v;
        __syncthreads();
        for (int o = kInitThreads / 2; o > 0; o >>= 1) {
            if (tid < o) red[tid] += red[tid + o];
            __syncthreads();
        }
        const double r = red[0];
        __syncthreads();
        return r;
    };
    double a = 0.0;
    for (size_t i = tid; i < n; i += kInitThreads) a += (double)(float)wr[i];
    const double mean = block_sum(a) / (double)n;
    double q = 0.0;
    for (size_t i = tid; i < n; i += kInitThreads) {
        const double dlt = (double)(float)wr[i] - mean;
        q += dlt * dlt;
    }
    const double var = block_sum(q) / (double)n;
    if (tid == 0) {
        s_mean = mean;
        s_sd = sqrt(var);
        if (stats) { stats[0] = (float)mean; stats[1] = (float)var; }
    }
    __syncthreads();
    const double m = s_mean, sd = s_sd;
    T *rows = wr + n;
    for (size_t i = tid; i < (size_t)Z * H; i += kInitThreads) rows[i] = (T)(float)(m + sd * (double)normals[i]);
}

}  // namespace zeda

using namespace zeda;

extern "C" {

int zeda_rmsnorm(int32_t T, int32_t H, int32_t dtype, const void *x, const void *gamma, float eps, void *out, void *stream)
{
    if (T < 0 || H < 1 || (dtype != ZEDA_F32 && dtype != ZEDA_BF16) || !x || !out || !(eps >= 0.f)) return ZEDA_EINVAL;
    if (T == 0) return ZEDA_OK;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == ZEDA_BF16)
        rmsnorm_kernel<bf16_t><<<T, kStackThreads, 0, s>>>((const bf16_t *)x, (const bf16_t *)gamma, eps, (bf16_t *)out, H);
    else
        rmsnorm_kernel<float><<<T, kStackThreads, 0, s>>>((const float *)x, (const float *)gamma, eps, (float *)out, H);
    return last_launch_status();
}

int zeda_residual_add(int32_t T, int32_t H, int32_t dtype, void *x, const void *y, void *stream)
{
    if (T < 0 || H < 1 || (dtype != ZEDA_F32 && dtype != ZEDA_BF16) || !x || !y) return ZEDA_EINVAL;
    const size_t n = (size_t)T * H;
    if (n == 0) return ZEDA_OK;
    hipStream_t s = (hipStream_t)stream;
    const int grid = (int)((n + kStackThreads * 8 - 1) / (kStackThreads * 8) < 65536 ? (n + kStackThreads * 8 - 1) / (kStackThreads * 8) : 65536);
    if (dtype == ZEDA_BF16) residual_add_kernel<bf16_t><<<grid, kStackThreads, 0, s>>>((bf16_t *)x, (const bf16_t *)y, n);
    else residual_add_kernel<float><<<grid, kStackThreads, 0, s>>>((float *)x, (const float *)y, n);
    return last_launch_status();
}

int zeda_init_zero_expert_rows(const zeda_layer_desc *desc, void *w_router, const float *normals, float *stats, void *stream)
{
    if (!desc) return ZEDA_EINVAL;
    zeda_layer_desc d = *desc;
    d.T = 0;
    int rc = check_desc(&d);
    if (rc != ZEDA_OK) return rc;
    if (!w_router || (d.Z > 0 && !normals) || !aligned16(w_router) || (reinterpret_cast<uintptr_t>(normals) & 3u) ||
        (reinterpret_cast<uintptr_t>(stats) & 3u))
        return ZEDA_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    if (d.dtype == ZEDA_BF16)
        init_zero_rows_kernel<bf16_t><<<1, kInitThreads, 0, s>>>((bf16_t *)w_router, normals, d.N, d.Z, d.H, stats);
    else
        init_zero_rows_kernel<float><<<1, kInitThreads, 0, s>>>((float *)w_router, normals, d.N, d.Z, d.H, stats);
    return last_launch_status();
}

}  // extern "C"
