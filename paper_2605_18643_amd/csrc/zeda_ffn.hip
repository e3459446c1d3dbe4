// Grouped SwiGLU expert FFN over the real slots only (Appendix D, Eq. 10: the 6*H*H_e FLOPs of the
// gate, up and down projections are spent on the (1 - r_ZE) share of slots that landed on a normal
// expert).  Two grouped GEMMs on the bf16 MFMA units with fp32 accumulation:
//   gate/up:  act[r, i]  = silu(<x[tok(r)], W_gate[e][i]>) * <x[tok(r)], W_up[e][i]>
//   down:     y_slot[r,h] = <act[r], W_down[e][h]>
// for the rows r of expert e in expert-sorted order.  Both operands have the reduction dimension
// contiguous, so every MFMA fragment is one 16-byte load.
//
// Tiling.  A workgroup owns (expert, token tile, feature tile).  Weight rows are the MFMA "A" operand
// (output rows), tokens the "B" operand (output columns): a lane then holds 4 consecutive output
// features of one token per register quad and stores them as one 8- or 16-byte word.  Both tiles are
// staged through LDS in 64-wide k chunks (128-byte rows, 16-byte pieces XOR-swizzled by the row pair
// so that the 32 rows a fragment read touches spread over all banks), double buffered, with the next
// chunk's global loads in flight while the current one is multiplied.
// There is no host-side work list: every workgroup derives its tile from expert_offsets with a wave
// scan, so the grid is sized for the worst case and surplus workgroups return at once; experts with no
// rows get no tile at all.  Workgroup ids are dealt so that each XCD (ids round-robin over the 8 XCDs)
// walks a contiguous range of tiles: the tiles of one expert share its L2.
#include "zeda_internal.h"

namespace zeda {

template <int TB_, int FB_, int WT_, int WF_>
struct TileCfg {
    static constexpr int TB = TB_, FB = FB_, WT = WT_, WF = WF_;
    static constexpr int BT = 32 * TB * WT;      // tokens per tile
    static constexpr int BF = 32 * FB * WF;      // weight rows per tile (gate and up rows both count)
    static constexpr int THREADS = 64 * WT * WF;
    static constexpr int LDS_BYTES = 2 * (BT + BF) * 128;
};

__device__ __forceinline__ int swz(int row, int piece) { return piece ^ ((row >> 1) & 7); }

// Tile lookup shared by both GEMMs.  Every wave computes the same answer.
struct TileLoc {
    int expert, row0, rows;  // first sorted row of the tile and its row count (<= BT)
};

template <int BT>
__device__ __forceinline__ bool locate_tile(const int32_t *__restrict__ offsets, int N, int tile_m, TileLoc &loc)
{
    const int lane = threadIdx.x & 63;
    int off[5];
#pragma unroll
    for (int q = 0; q < 5; ++q) off[q] = offsets[min(4 * lane + q, N)];
    int nt[4], local = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        nt[q] = (off[q + 1] - off[q] + BT - 1) / BT;
        local += nt[q];
    }
    int incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    const int total = __shfl(incl, 63);
    if (tile_m >= total) return false;
    int excl = incl - local;
    const bool mine = tile_m >= excl && tile_m < incl;
    int e = 0, mt = 0, m = 0, o0 = 0, ntile = 1;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (mine && tile_m >= excl && tile_m < excl + nt[q]) {
            e = 4 * lane + q; mt = tile_m - excl; m = off[q + 1] - off[q]; o0 = off[q]; ntile = nt[q];
        }
        excl += nt[q];
    }
    const int src = __ffsll((long long)__ballot(mine)) - 1;
    e = __shfl(e, src); mt = __shfl(mt, src); m = __shfl(m, src); o0 = __shfl(o0, src); ntile = __shfl(ntile, src);
    // balanced split of the expert's m rows into ntile tiles, each a multiple of 32 rows except the last
    const int per = (((m + ntile - 1) / ntile) + 31) & ~31;
    loc.expert = e;
    loc.row0 = o0 + mt * per;
    loc.rows = min(per, m - mt * per);
    return true;
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.f + __expf(-g)) * u; }

__device__ __forceinline__ void store4(bf16_t *p, float a, float b, float c, float d)
{
    bf16x4 v = {(bf16_t)a, (bf16_t)b, (bf16_t)c, (bf16_t)d};
    *reinterpret_cast<bf16x4 *>(p) = v;
}
__device__ __forceinline__ void store4(float *p, float a, float b, float c, float d)
{
    f32x4 v = {a, b, c, d};
    *reinterpret_cast<f32x4 *>(p) = v;
}

// GATEUP: tok = x[T,Kdim], w0 = W_gate[N,Fdim,Kdim], w1 = W_up, out = act[S,Fdim] (Fdim = I, Kdim = H).
// DOWN:   tok = act[S,Kdim], w0 = W_down[N,Fdim,Kdim], out = y_slot[S,Fdim]        (Fdim = H, Kdim = I).
template <class C, bool GATEUP, typename OutT>
__global__ __launch_bounds__(C::THREADS) void ffn_bf16_kernel(const bf16_t *__restrict__ tok,
                                                              const bf16_t *__restrict__ w0,
                                                              const bf16_t *__restrict__ w1,
                                                              const int32_t *__restrict__ offsets,
                                                              const int32_t *__restrict__ sorted_slot,
                                                              OutT *__restrict__ out, int N, int K, int Kdim, int Fdim,
                                                              int n_ftiles, int T)
{
    constexpr int TB = C::TB, FB = C::FB, WT = C::WT, WF = C::WF, BT = C::BT, BF = C::BF, THREADS = C::THREADS;
    constexpr int TCH = BT * 8 / THREADS;  // 16-byte pieces of the token tile per thread and k chunk
    constexpr int FCH = BF * 8 / THREADS;
    static_assert(BT * 8 % THREADS == 0 && BF * 8 % THREADS == 0, "tile rows must divide over the threads");
    static_assert(!GATEUP || FB % 2 == 0, "gate and up blocks come in pairs");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // XCD-aware order: ids i, i+8, i+16, ... run on the same XCD; give each XCD a contiguous tile range
    const int G = gridDim.x;
    const int L = (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8;
    const int tile_m = L / n_ftiles, ft = L - tile_m * n_ftiles;
    TileLoc loc;
    if (!locate_tile<BT>(offsets, N, tile_m, loc)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wt = wave / WF, wf = wave % WF;
    const int col = lane & 31, half = lane >> 5;

    // global source of every 16-byte piece this thread stages (fixed over the k loop)
    const bf16_t *tsrc[TCH];
    int tdst[TCH];
#pragma unroll
    for (int i = 0; i < TCH; ++i) {
        const int q = tid + THREADS * i, row = q >> 3, piece = q & 7;
        const int r = loc.row0 + min(row, loc.rows - 1);  // rows past the tile repeat its last row (never stored)
        size_t base;
        if (GATEUP) base = (size_t)min(max(sorted_slot[r] / K, 0), T - 1) * Kdim;  // clamp: a bad index must not fault
        else base = (size_t)r * Kdim;
        tsrc[i] = tok + base + swz(row, piece) * 8;
        tdst[i] = row * 128 + piece * 16;
    }
    const bf16_t *fsrc[FCH];
    int fdst[FCH];
#pragma unroll
    for (int i = 0; i < FCH; ++i) {
        const int q = tid + THREADS * i, row = q >> 3, piece = q & 7;
        const bf16_t *wbase;
        int grow;
        if (GATEUP) {
            const int blk = (row >> 5) % FB, wfr = row / (32 * FB);
            grow = ft * (BF / 2) + (wfr * (FB / 2) + (blk >> 1)) * 32 + (row & 31);
            wbase = (blk & 1) ? w1 : w0;
        } else {
            grow = ft * BF + row;
            wbase = w0;
        }
        fsrc[i] = wbase + ((size_t)loc.expert * Fdim + grow) * Kdim + swz(row, piece) * 8;
        fdst[i] = BT * 128 + row * 128 + piece * 16;
    }

    f32x16 acc[TB][FB];
#pragma unroll
    for (int a = 0; a < TB; ++a)
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // token blocks of this wave that hold at least one row of the tile
    const int tb_active = max(0, min(TB, (loc.rows - wt * 32 * TB + 31) / 32));

    bf16x8 treg[TCH], freg[FCH];
    constexpr int STAGE = (BT + BF) * 128;
    const int nk = Kdim / 64;

#pragma unroll
    for (int i = 0; i < TCH; ++i) treg[i] = *reinterpret_cast<const bf16x8 *>(tsrc[i]);
#pragma unroll
    for (int i = 0; i < FCH; ++i) freg[i] = *reinterpret_cast<const bf16x8 *>(fsrc[i]);
#pragma unroll
    for (int i = 0; i < TCH; ++i) *reinterpret_cast<bf16x8 *>(lds + tdst[i]) = treg[i];
#pragma unroll
    for (int i = 0; i < FCH; ++i) *reinterpret_cast<bf16x8 *>(lds + fdst[i]) = freg[i];
    __syncthreads();

    for (int it = 0; it < nk; ++it) {
        const unsigned char *cur = lds + (it & 1) * STAGE;
        unsigned char *nxt = lds + ((it + 1) & 1) * STAGE;
        const bool more = it + 1 < nk;
        if (more) {
            const int k1 = (it + 1) * 64;
#pragma unroll
            for (int i = 0; i < TCH; ++i) treg[i] = *reinterpret_cast<const bf16x8 *>(tsrc[i] + k1);
#pragma unroll
            for (int i = 0; i < FCH; ++i) freg[i] = *reinterpret_cast<const bf16x8 *>(fsrc[i] + k1);
        }
        if (tb_active > 0) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                bf16x8 fa[FB], tbv[TB];
#pragma unroll
                for (int b = 0; b < FB; ++b) {
                    const int row = (wf * FB + b) * 32 + col;
                    fa[b] = *reinterpret_cast<const bf16x8 *>(cur + BT * 128 + row * 128 + swz(row, 2 * s + half) * 16);
                }
#pragma unroll
                for (int a = 0; a < TB; ++a) {
                    const int row = (wt * TB + a) * 32 + col;
                    tbv[a] = *reinterpret_cast<const bf16x8 *>(cur + row * 128 + swz(row, 2 * s + half) * 16);
                }
#pragma unroll
                for (int a = 0; a < TB; ++a) {
                    if (a < tb_active) {
#pragma unroll
                        for (int b = 0; b < FB; ++b)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[b], tbv[a], acc[a][b], 0, 0, 0);
                    }
                }
            }
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < TCH; ++i) *reinterpret_cast<bf16x8 *>(nxt + tdst[i]) = treg[i];
#pragma unroll
            for (int i = 0; i < FCH; ++i) *reinterpret_cast<bf16x8 *>(nxt + fdst[i]) = freg[i];
        }
        __syncthreads();
    }

    // acc[a][b][v]: feature 8*(v/4) + 4*half + v%4 of block b, token col of block a
#pragma unroll
    for (int a = 0; a < TB; ++a) {
        const int trow = (wt * TB + a) * 32 + col;
        if (a < tb_active && trow < loc.rows) {
            OutT *orow = out + (size_t)(loc.row0 + trow) * Fdim;
            if (GATEUP) {
#pragma unroll
                for (int p = 0; p < FB / 2; ++p) {
                    const int c0 = ft * (BF / 2) + (wf * (FB / 2) + p) * 32 + 4 * half;
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const f32x16 &g = acc[a][2 * p], &u = acc[a][2 * p + 1];
                        store4(orow + c0 + 8 * vq, silu_mul(g[4 * vq], u[4 * vq]), silu_mul(g[4 * vq + 1], u[4 * vq + 1]),
                               silu_mul(g[4 * vq + 2], u[4 * vq + 2]), silu_mul(g[4 * vq + 3], u[4 * vq + 3]));
                    }
                }
            } else {
#pragma unroll
                for (int b = 0; b < FB; ++b) {
                    const int c0 = ft * BF + (wf * FB + b) * 32 + 4 * half;
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq)
                        store4(orow + c0 + 8 * vq, acc[a][b][4 * vq], acc[a][b][4 * vq + 1], acc[a][b][4 * vq + 2],
                               acc[a][b][4 * vq + 3]);
                }
            }
        }
    }
}

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
typedef TileCfg<2, 2, 2, 2> CfgPrefill;  // 128 tokens x 128 weight rows, 4 waves
typedef TileCfg<2, 2, 1, 4> CfgDec64;    // 64 tokens x 256 weight rows
typedef TileCfg<1, 2, 1, 4> CfgDec32;    // 32 tokens x 256 weight rows

template <class C>
static int grid_for(const zeda_layer_desc *d, int n_ftiles)
{
    const int64_t S = (int64_t)d->T * d->K;
    // sum over experts of ceil(m_e / BT) with m_e <= T and sum m_e <= S
    int64_t tiles_m = (int64_t)d->N * ceil_div(d->T, C::BT);
    const int64_t alt = S / C::BT + d->N;
    if (alt < tiles_m) tiles_m = alt;
    int64_t g = tiles_m * n_ftiles;
    return (int)((g + 7) / 8 * 8);
}

template <class C, bool GATEUP, typename OutT>
static int launch_tile_kernel(const zeda_layer_desc *d, const void *tok, const void *w0, const void *w1,
                              const int32_t *offsets, const int32_t *sorted_slot, void *out, hipStream_t s)
{
    auto kern = ffn_bf16_kernel<C, GATEUP, OutT>;
    static bool attr_set = false;  // per instantiation; idempotent, so a race between host threads is harmless
    if (!attr_set) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES) !=
            hipSuccess)
            return ZEDA_EHIP;
        attr_set = true;
    }
    const int Kdim = GATEUP ? d->H : d->I, Fdim = GATEUP ? d->I : d->H;
    const int n_ftiles = GATEUP ? Fdim / (C::BF / 2) : Fdim / C::BF;
    const int grid = grid_for<C>(d, n_ftiles);
    kern<<<grid, C::THREADS, C::LDS_BYTES, s>>>((const bf16_t *)tok, (const bf16_t *)w0, (const bf16_t *)w1, offsets,
                                               sorted_slot, (OutT *)out, d->N, d->K, Kdim, Fdim, n_ftiles, d->T);
    return last_launch_status();
}

// Feature tiles must divide the output width: gate/up tiles are BF/2 columns of I, down tiles BF columns of H.
template <class C>
static bool cfg_fits(const zeda_layer_desc *d)
{
    return d->I % (C::BF / 2) == 0 && d->H % C::BF == 0;
}

int launch_gateup(const zeda_layer_desc *d, const void *x, const void *wg, const void *wu, const int32_t *offsets,
                  const int32_t *sorted_slot, void *act, hipStream_t s)
{
    if (d->dtype == ZEDA_BF16) {
        if (d->T <= 32 && cfg_fits<CfgDec32>(d))
            return launch_tile_kernel<CfgDec32, true, bf16_t>(d, x, wg, wu, offsets, sorted_slot, act, s);
        if (d->T <= 64 && cfg_fits<CfgDec64>(d))
            return launch_tile_kernel<CfgDec64, true, bf16_t>(d, x, wg, wu, offsets, sorted_slot, act, s);
        return launch_tile_kernel<CfgPrefill, true, bf16_t>(d, x, wg, wu, offsets, sorted_slot, act, s);
    }
    const int S = d->T * d->K;
    ffn_f32_gateup_kernel<<<S, kF32Threads, (size_t)d->H * sizeof(float), s>>>(
        (const float *)x, (const float *)wg, (const float *)wu, offsets, sorted_slot, (float *)act, d->N, d->K, d->H, d->I, d->T);
    return last_launch_status();
}

int launch_down(const zeda_layer_desc *d, const void *act, const void *wd, const int32_t *offsets, void *y_slot,
                hipStream_t s)
{
    if (d->dtype == ZEDA_BF16) {
        if (d->T <= 32 && cfg_fits<CfgDec32>(d))
            return launch_tile_kernel<CfgDec32, false, bf16_t>(d, act, wd, nullptr, offsets, nullptr, y_slot, s);
        if (d->T <= 64 && cfg_fits<CfgDec64>(d))
            return launch_tile_kernel<CfgDec64, false, bf16_t>(d, act, wd, nullptr, offsets, nullptr, y_slot, s);
        return launch_tile_kernel<CfgPrefill, false, bf16_t>(d, act, wd, nullptr, offsets, nullptr, y_slot, s);
    }
    const int S = d->T * d->K;
    ffn_f32_down_kernel<<<S, kF32Threads, (size_t)d->I * sizeof(float), s>>>((const float *)act, (const float *)wd, offsets,
                                                                              (float *)y_slot, d->N, d->H, d->I);
    return last_launch_status();
}

}  // namespace zeda
