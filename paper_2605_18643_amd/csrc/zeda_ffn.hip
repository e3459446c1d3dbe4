// Grouped SwiGLU expert FFN over the real slots only (Appendix D, Eq. 10: the 6*H*H_e FLOPs of the
// gate, up and down projections are spent on the (1 - r_ZE) share of slots that landed on a normal
// expert).  Two grouped GEMMs on the bf16 MFMA units with fp32 accumulation:
//   gate/up:  act[r, i]  = silu(<x[tok(r)], W_gate[e][i]>) * <x[tok(r)], W_up[e][i]>
//   down:     y_slot[r,h] = <act[r], W_down[e][h]>
// for the rows r of expert e in expert-sorted order.  Both operands have the reduction dimension
// contiguous, so every MFMA fragment is one 16-byte LDS read.  The tile kernel is in zeda_ffn_tile.h;
// this file picks the tile shapes and holds the plain fp32 path.
#include "zeda_ffn_tile.h"

namespace zeda {

// ---------------------------------------------------------------------------------------------
// fp32 path (plain FMA, for the fp32 configuration): one workgroup per sorted row.
// ---------------------------------------------------------------------------------------------
constexpr int kF32Threads = 256;

__device__ __forceinline__ int expert_of_row(const int32_t *__restrict__ offsets, int N, int r)
{
    int lo = 0, hi = N;  // largest e with offsets[e] <= r (empty experts share an offset with the next one)
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (offsets[mid] <= r) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ float wave_sum_f(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__global__ __launch_bounds__(kF32Threads) void ffn_f32_gateup_kernel(const float *__restrict__ x,
                                                                     const float *__restrict__ wg,
                                                                     const float *__restrict__ wu,
                                                                     const int32_t *__restrict__ offsets,
                                                                     const int32_t *__restrict__ sorted_slot,
                                                                     float *__restrict__ act, int N, int K, int H, int I, int T)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    float *xs = reinterpret_cast<float *>(lds);
    const int r = blockIdx.x;
    if (r >= offsets[N]) return;
    const int e = expert_of_row(offsets, N, r);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *xr = x + (size_t)min(max(sorted_slot[r] / K, 0), T - 1) * H;
    for (int h = tid; h < H; h += kF32Threads) xs[h] = xr[h];
    __syncthreads();
    for (int i = wave; i < I; i += kF32Threads / 64) {
        const float *g = wg + ((size_t)e * I + i) * H, *u = wu + ((size_t)e * I + i) * H;
        float sg = 0.f, su = 0.f;
        for (int h = lane; h < H; h += 64) {
            sg = fmaf(g[h], xs[h], sg);
            su = fmaf(u[h], xs[h], su);
        }
        sg = wave_sum_f(sg);
        su = wave_sum_f(su);
        if (lane == 0) act[(size_t)r * I + i] = sg / (1.f + expf(-sg)) * su;
    }
}

__global__ __launch_bounds__(kF32Threads) void ffn_f32_down_kernel(const float *__restrict__ act,
                                                                   const float *__restrict__ wd,
                                                                   const int32_t *__restrict__ offsets,
                                                                   float *__restrict__ y, int N, int H, int I)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    float *as = reinterpret_cast<float *>(lds);
    const int r = blockIdx.x;
    if (r >= offsets[N]) return;
    const int e = expert_of_row(offsets, N, r);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < I; i += kF32Threads) as[i] = act[(size_t)r * I + i];
    __syncthreads();
    for (int h = wave; h < H; h += kF32Threads / 64) {
        const float *w = wd + ((size_t)e * H + h) * I;
        float s = 0.f;
        for (int i = lane; i < I; i += 64) s = fmaf(w[i], as[i], s);
        s = wave_sum_f(s);
        if (lane == 0) y[(size_t)r * H + h] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
//              G FB WF NSW NST KC   (NSW, NST: depth of the weight and of the token ring)
typedef TileCfg<4, 2, 4, 2, 2, 64> CfgPrefill;  // 256 tokens x 256 weight rows, 8 waves, one workgroup per CU
typedef TileCfg<4, 2, 2, 2, 2, 64> CfgNarrow;   // 256 tokens x 128 weight rows, 4 waves: any H % 128 == 0, I % 64 == 0
typedef TileCfg<1, 2, 2, 4, 4, 32> CfgDecode;   // 64 tokens x 128 weight rows, 4 waves, two workgroups per CU
// tiled weights come in 32-wide k blocks: 32-wide chunks, four deep
typedef TileCfg<4, 2, 4, 4, 4, 32> CfgPrefillT;
typedef TileCfg<4, 2, 2, 4, 4, 32> CfgNarrowT;
// 320 tokens x 256 weight rows (token ring three deep): an expert with a few rows more than a multiple of 256 gets
// one token tile less than CfgPrefillT would give it, i.e. one pass less over its weights.  It is the second
// geometry of the adaptive kernel, which picks one of the two from the expert loads.
typedef TileCfg<5, 2, 4, 4, 3, 32> CfgPrefillT5;

// Persistent grid: as many workgroups as the device holds at once, rounded down to a multiple of 8 so that
// every XCD gets the same number (the kernel reads the count from gridDim).
template <class C, bool GATEUP, bool TILED>
static int resident_grid()
{
    static int grids[kMaxDevices] = {};  // per instantiation and device; idempotent, so a race between host threads is harmless
    const int dev = current_device();
    if (dev < 0) return 0;
    int &grid = grids[dev];
    if (grid == 0) {
        auto kern = ffn_bf16_kernel<C, GATEUP, TILED>;
        int cus = 0, per_cu = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kern, C::THREADS, C::LDS_BYTES) != hipSuccess)
            return 0;
        const int g = cus * (per_cu > 0 ? per_cu : 1) / 8 * 8;
        grid = g > 0 ? g : 8;
    }
    return grid;
}

template <class CA, class CB, bool GATEUP, bool TILED>
static int launch_adaptive_kernel(const zeda_layer_desc *d, const void *tok, const void *w0, const void *w1,
                                  const int32_t *offsets, const int32_t *sorted_slot, void *out, hipStream_t s)
{
    constexpr int kLds = CA::LDS_BYTES > CB::LDS_BYTES ? CA::LDS_BYTES : CB::LDS_BYTES;
    auto kern = ffn_bf16_adaptive_kernel<CA, CB, GATEUP, TILED>;
    static int grids[kMaxDevices] = {};  // (as in resident_grid)
    const int dev = current_device();
    if (dev < 0) return ZEDA_EHIP;
    int &grid = grids[dev];
    if (grid == 0) {
        int cus = 0, per_cu = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLds) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kern, CA::THREADS, kLds) != hipSuccess)
            return ZEDA_EHIP;
        const int g = cus * (per_cu > 0 ? per_cu : 1) / 8 * 8;
        grid = g > 0 ? g : 8;
    }
    const int Kdim = GATEUP ? d->H : d->I, Fdim = GATEUP ? d->I : d->H;
    const int n_ftiles = GATEUP ? Fdim / (CA::BF / 2) : Fdim / CA::BF;
    kern<<<grid, CA::THREADS, kLds, s>>>((const bf16_t *)tok, (const bf16_t *)w0, (const bf16_t *)w1, offsets, sorted_slot,
                                         (bf16_t *)out, d->N, d->K, Kdim, Fdim, n_ftiles, d->T);
    return last_launch_status();
}

// Whether the expert loads may sit just above a multiple of the 256-row tile, where the wide tile saves a pass over
// the weights (the adaptive kernel then decides on the device; where they cannot, the plain kernel saves the 1-2 %
// the second geometry costs the first).  The mean row count is T*K/N when every slot is real - loads then cluster
// around it - and anything below that with zero experts.
static bool rows_may_straddle_tile(const zeda_layer_desc *d)
{
    const double all_real = (double)d->T * d->K / d->N;
    // (at a thousand rows per expert and more the passes saved no longer pay for it: measured on config 4)
    if (d->Z > 0) return all_real > 256.0 && all_real < 1024.0;
    for (int k = 1; k <= 2; ++k)
        if (all_real > 240.0 * k && all_real <= 330.0 * k) return true;
    return false;
}

template <class C, bool GATEUP, bool TILED>
static int launch_tile_kernel(const zeda_layer_desc *d, const void *tok, const void *w0, const void *w1,
                              const int32_t *offsets, const int32_t *sorted_slot, void *out, hipStream_t s)
{
    const int grid = resident_grid<C, GATEUP, TILED>();
    if (grid == 0) return ZEDA_EHIP;
    const int Kdim = GATEUP ? d->H : d->I, Fdim = GATEUP ? d->I : d->H;
    const int n_ftiles = GATEUP ? Fdim / (C::BF / 2) : Fdim / C::BF;
    ffn_bf16_kernel<C, GATEUP, TILED><<<grid, C::THREADS, C::LDS_BYTES, s>>>((const bf16_t *)tok, (const bf16_t *)w0,
                                                                     (const bf16_t *)w1, offsets, sorted_slot,
                                                                     (bf16_t *)out, d->N, d->K, Kdim, Fdim, n_ftiles, d->T);
    return last_launch_status();
}

// Feature tiles must divide the output width: gate/up tiles are BF/2 columns of I, down tiles BF columns of H.
template <class C>
static bool cfg_fits(const zeda_layer_desc *d)
{
    return d->I % (C::BF / 2) == 0 && d->H % C::BF == 0;
}

template <bool GATEUP>
static int launch_bf16(const zeda_layer_desc *d, const void *tok, const void *w0, const void *w1, const int32_t *offsets,
                       const int32_t *sorted_slot, void *out, hipStream_t s)
{
    // an expert never has more rows than there are tokens: small batches take the short token tile
    const bool decode = d->T <= CfgDecode::BT && cfg_fits<CfgDecode>(d);
    if (d->weight_layout == ZEDA_WEIGHTS_TILED) {
        if (decode) return launch_tile_kernel<CfgDecode, GATEUP, true>(d, tok, w0, w1, offsets, sorted_slot, out, s);
        if (cfg_fits<CfgPrefillT>(d)) {
            if (rows_may_straddle_tile(d))
                return launch_adaptive_kernel<CfgPrefillT, CfgPrefillT5, GATEUP, true>(d, tok, w0, w1, offsets, sorted_slot, out, s);
            return launch_tile_kernel<CfgPrefillT, GATEUP, true>(d, tok, w0, w1, offsets, sorted_slot, out, s);
        }
        return launch_tile_kernel<CfgNarrowT, GATEUP, true>(d, tok, w0, w1, offsets, sorted_slot, out, s);
    }
    if (decode) return launch_tile_kernel<CfgDecode, GATEUP, false>(d, tok, w0, w1, offsets, sorted_slot, out, s);
    if (cfg_fits<CfgPrefill>(d))
        return launch_tile_kernel<CfgPrefill, GATEUP, false>(d, tok, w0, w1, offsets, sorted_slot, out, s);
    return launch_tile_kernel<CfgNarrow, GATEUP, false>(d, tok, w0, w1, offsets, sorted_slot, out, s);
}

int launch_pack_weights(const zeda_layer_desc *d, const void *w, void *out, bool down, hipStream_t s)
{
    const int F = down ? d->H : d->I, Kd = down ? d->I : d->H;
    const size_t pieces = (size_t)d->N * F * Kd / 8;
    pack_weights_kernel<<<(unsigned)((pieces + 255) / 256), 256, 0, s>>>((const bf16_t *)w, (bf16_t *)out, F, Kd, pieces);
    return last_launch_status();
}

int launch_gateup(const zeda_layer_desc *d, const void *x, const void *wg, const void *wu, const int32_t *offsets,
                  const int32_t *sorted_slot, void *act, hipStream_t s)
{
    if (d->dtype == ZEDA_BF16) return launch_bf16<true>(d, x, wg, wu, offsets, sorted_slot, act, s);
    const int S = d->T * d->K;
    ffn_f32_gateup_kernel<<<S, kF32Threads, (size_t)d->H * sizeof(float), s>>>(
        (const float *)x, (const float *)wg, (const float *)wu, offsets, sorted_slot, (float *)act, d->N, d->K, d->H, d->I,
        d->T);
    return last_launch_status();
}

int launch_down(const zeda_layer_desc *d, const void *act, const void *wd, const int32_t *offsets, void *y_slot,
                hipStream_t s)
{
    if (d->dtype == ZEDA_BF16) return launch_bf16<false>(d, act, wd, nullptr, offsets, nullptr, y_slot, s);
    const int S = d->T * d->K;
    ffn_f32_down_kernel<<<S, kF32Threads, (size_t)d->I * sizeof(float), s>>>((const float *)act, (const float *)wd, offsets,
                                                                              (float *)y_slot, d->N, d->H, d->I);
    return last_launch_status();
}

}  // namespace zeda
