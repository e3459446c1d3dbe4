// Grouped bf16 GEMM tile kernel of the expert FFN (Appendix D, Eq. 10: gate, up and down projections of
// the real slots only).  See zeda_ffn.hip for how the two GEMMs use it.
//
// A workgroup owns (expert, token tile, feature tile).  Weight rows are the MFMA "A" operand (output
// rows), tokens the "B" operand (output columns): a lane then holds 4 consecutive output features of one
// token per register quad and stores them as one 8- or 16-byte word.
//
// Data movement.  Both tiles stream through an NSTAGE-deep ring in LDS in 64-wide k chunks, fetched with
// global->LDS loads (no staging registers): one wave instruction moves 64 pieces of 16 bytes to 1 KiB of
// consecutive LDS, i.e. 8 rows of 128 bytes, so lane l fetches the piece that belongs at position l of
// that KiB.  The 8 pieces of a row are XOR-permuted by the row index so that the 16 rows a fragment read
// touches per phase fall on distinct banks; the permutation is applied on the global address, which
// costs nothing.  NSTAGE-1 chunks are in flight while one is multiplied; a counted s_waitcnt and one
// s_barrier per chunk order the ring (the wait covers this thread's own loads, the barrier extends it to
// the workgroup and also guarantees that everyone has left the slot about to be refilled).
//
// With about half of the slots on zero experts an expert sees few rows and the GEMM is bound by streaming
// its weights from HBM, so the tile is shaped around that: all rows of an expert up to 64*G form one
// token tile (the expert's weights then stream exactly once), only the 64-row groups that hold rows are
// fetched and multiplied (the group count is a template parameter of the main loop, so it has no
// branches), and the two wave rows take alternate 32-row blocks so that both always have equal work.
//
// There is no host-side work list: every workgroup derives its tile from expert_offsets with a wave
// scan, so the grid is sized for the worst case and surplus workgroups return at once; experts with no
// rows get no tile at all.  Each XCD walks a contiguous eighth of the tiles that exist (see locate_tile).
#pragma once
#include "zeda_internal.h"

namespace zeda {

template <int G_, int FB_, int WF_, int NSTAGE_>
struct TileCfg {
    static constexpr int G = G_, FB = FB_, WF = WF_, NSTAGE = NSTAGE_;
    static constexpr int WT = 2;                  // wave rows: wave row wt owns token blocks wt, wt+2, ...
    static constexpr int BT = 64 * G;             // tokens per tile
    static constexpr int BF = 32 * FB * WF;       // weight rows per tile (gate and up rows both count)
    static constexpr int NW = WT * WF;            // waves
    static constexpr int THREADS = 64 * NW;
    static constexpr int STAGE = (BT + BF) * 128;  // bytes per ring slot: rows of 64 bf16
    static constexpr int LDS_BYTES = NSTAGE * STAGE;
    // wave load instructions (8 rows each) per chunk and wave when g 64-row groups are live
    static constexpr int nl(int g) { return (8 * g + BF / 8) / NW; }
    static_assert((BF / 8) % NW == 0 && 8 % NW == 0, "loads must divide evenly over the waves for every group count");
    static_assert(NSTAGE >= 2 && (NSTAGE - 1) * nl(G) <= 63, "vmcnt is a 6-bit counter");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS is 160 KiB per CU");
};

// position of logical piece p of row r inside its 128-byte LDS row (an involution in p)
__device__ __forceinline__ int swz(int row, int piece) { return piece ^ ((row >> 1) & 7); }

struct TileLoc {
    int expert, row0, rows;  // first sorted row of the tile and its row count (<= BT)
};

// Tile lookup.  Token tiles are numbered in expert order; feature tile ft of token tile m is work item
// m * n_ftiles + ft.  Workgroup ids go round-robin over the 8 XCDs, so workgroup b runs on XCD b % 8:
// each XCD is handed a contiguous eighth of the work items that really exist (their number is only known
// here, on the device), so that the feature tiles of an expert share one L2 and all XCDs get equal work
// even though the grid was sized for the worst case.  Every wave computes the same answer.
template <int BT>
__device__ __forceinline__ bool locate_tile(const int32_t *__restrict__ offsets, int N, int n_ftiles, TileLoc &loc,
                                            int &ft)
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
    const int items = __shfl(incl, 63) * n_ftiles;
    const int per_xcd = (items + 7) / 8;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int item = xcd * per_xcd + j;
    if (j >= per_xcd || item >= items) return false;
    const int tile_m = item / n_ftiles;
    ft = item - tile_m * n_ftiles;
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
    // balanced split of the expert's m rows into ntile tiles, each a multiple of 64 rows except the last
    const int per = (((m + ntile - 1) / ntile) + 63) & ~63;
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

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

#define ZEDA_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define ZEDA_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

struct TileArgs {
    const bf16_t *tok, *w0, *w1;
    const int32_t *sorted_slot;
    int K, Kdim, Fdim, T;
    int expert, row0, rows, ft;
};

// Main loop and epilogue for a tile with GA live 64-row groups (1 <= GA <= G).
template <class C, bool GATEUP, typename OutT, int GA>
__device__ __forceinline__ void tile_body(unsigned char *lds, const TileArgs &t, OutT *__restrict__ out)
{
    constexpr int FB = C::FB, WF = C::WF, BT = C::BT, BF = C::BF, NSTAGE = C::NSTAGE, NW = C::NW, STAGE = C::STAGE;
    constexpr int NL = C::nl(GA);   // load instructions per wave and chunk
    constexpr int NTI = 8 * GA;     // ... of the chunk that fetch token rows
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wt = wave / WF, wf = wave % WF;
    const int col = lane & 31, half = lane >> 5;

    // Source of the piece this lane fetches in each of the wave's NL load instructions per chunk.
    // Instruction j < NTI covers token rows 8j..8j+7 of the tile, the others weight rows 8(j-NTI)..+7.
    const bf16_t *src[NL];
    int dst[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int j = wave + NW * i;
        const int piece = lane & 7;
        if (j < NTI) {
            const int trow = j * 8 + (lane >> 3);
            const int r = t.row0 + min(trow, t.rows - 1);  // rows past the tile repeat its last row (never stored)
            size_t base;
            if (GATEUP) base = (size_t)min(max(t.sorted_slot[r] / t.K, 0), t.T - 1) * t.Kdim;  // a bad index must not fault
            else base = (size_t)r * t.Kdim;
            src[i] = t.tok + base + swz(trow, piece) * 8;
            dst[i] = j * 1024;
        } else {
            const int row = (j - NTI) * 8 + (lane >> 3);
            const bf16_t *wbase;
            int grow;
            if (GATEUP) {
                const int blk = (row >> 5) % FB, wfr = row / (32 * FB);
                grow = t.ft * (BF / 2) + (wfr * (FB / 2) + (blk >> 1)) * 32 + (row & 31);
                wbase = (blk & 1) ? t.w1 : t.w0;
            } else {
                grow = t.ft * BF + row;
                wbase = t.w0;
            }
            src[i] = wbase + ((size_t)t.expert * t.Fdim + grow) * t.Kdim + swz(row, piece) * 8;
            dst[i] = BT * 128 + (j - NTI) * 1024;
        }
    }
    auto issue = [&](int chunk) {
        unsigned char *slot = lds + (chunk % NSTAGE) * STAGE;
#pragma unroll
        for (int i = 0; i < NL; ++i)
            __builtin_amdgcn_global_load_lds(ZEDA_GLOBAL_PTR(src[i] + (size_t)chunk * 64), ZEDA_LDS_PTR(slot + dst[i]), 16, 0,
                                             0);
    };

    f32x16 acc[GA][FB];
#pragma unroll
    for (int a = 0; a < GA; ++a)
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int nk = t.Kdim / 64;
#pragma unroll
    for (int c = 0; c < NSTAGE - 1; ++c)
        if (c < nk) issue(c);

    for (int it = 0; it < nk; ++it) {
        // chunk `it` of this thread has landed once at most NSTAGE-2 later chunks are outstanding
        if (it + NSTAGE - 2 < nk) wait_vmcnt<(NSTAGE - 2) * NL>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (it + NSTAGE - 1 < nk) issue(it + NSTAGE - 1);  // refills the slot everyone left before the barrier
        const unsigned char *cur = lds + (it % NSTAGE) * STAGE;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8 fa[FB], tb[GA];
#pragma unroll
            for (int b = 0; b < FB; ++b) {
                const int row = (wf * FB + b) * 32 + col;
                fa[b] = *reinterpret_cast<const bf16x8 *>(cur + BT * 128 + row * 128 + swz(row, 2 * s + half) * 16);
            }
#pragma unroll
            for (int a = 0; a < GA; ++a) {
                const int row = (2 * a + wt) * 32 + col;
                tb[a] = *reinterpret_cast<const bf16x8 *>(cur + row * 128 + swz(row, 2 * s + half) * 16);
            }
#pragma unroll
            for (int a = 0; a < GA; ++a)
#pragma unroll
                for (int b = 0; b < FB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[b], tb[a], acc[a][b], 0, 0, 0);
        }
    }

    // acc[a][b][v]: feature 8*(v/4) + 4*half + v%4 of block b, token col of token block 2a + wt
#pragma unroll
    for (int a = 0; a < GA; ++a) {
        const int trow = (2 * a + wt) * 32 + col;
        if (trow < t.rows) {
            OutT *orow = out + (size_t)(t.row0 + trow) * t.Fdim + 4 * half;
            if (GATEUP) {
#pragma unroll
                for (int p = 0; p < FB / 2; ++p) {
                    const int c0 = t.ft * (BF / 2) + (wf * (FB / 2) + p) * 32;
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
                    const int c0 = t.ft * BF + (wf * FB + b) * 32;
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq)
                        store4(orow + c0 + 8 * vq, acc[a][b][4 * vq], acc[a][b][4 * vq + 1], acc[a][b][4 * vq + 2],
                               acc[a][b][4 * vq + 3]);
                }
            }
        }
    }
}

template <class C, bool GATEUP, typename OutT, int GA>
struct TileDispatch {
    static __device__ __forceinline__ void run(int g, unsigned char *lds, const TileArgs &t, OutT *__restrict__ out)
    {
        if (g == GA) tile_body<C, GATEUP, OutT, GA>(lds, t, out);
        else TileDispatch<C, GATEUP, OutT, GA - 1>::run(g, lds, t, out);
    }
};
template <class C, bool GATEUP, typename OutT>
struct TileDispatch<C, GATEUP, OutT, 0> {
    static __device__ __forceinline__ void run(int, unsigned char *, const TileArgs &, OutT *__restrict__) {}
};

// GATEUP: tok = x[T,Kdim], w0 = W_gate[N,Fdim,Kdim], w1 = W_up, out = act[S,Fdim] (Fdim = I, Kdim = H).
// DOWN:   tok = act[S,Kdim], w0 = W_down[N,Fdim,Kdim], out = y_slot[S,Fdim]        (Fdim = H, Kdim = I).
// Kdim is a multiple of 64; Fdim a multiple of the feature tile (BF/2 for GATEUP, BF for DOWN).
template <class C, bool GATEUP, typename OutT>
__global__ __launch_bounds__(C::THREADS) void ffn_bf16_kernel(const bf16_t *__restrict__ tok,
                                                              const bf16_t *__restrict__ w0,
                                                              const bf16_t *__restrict__ w1,
                                                              const int32_t *__restrict__ offsets,
                                                              const int32_t *__restrict__ sorted_slot,
                                                              OutT *__restrict__ out, int N, int K, int Kdim, int Fdim,
                                                              int n_ftiles, int T)
{
    static_assert(!GATEUP || C::FB % 2 == 0, "gate and up blocks come in pairs");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    TileLoc loc;
    int ft;
    if (!locate_tile<C::BT>(offsets, N, n_ftiles, loc, ft)) return;
    TileArgs t;
    t.tok = tok; t.w0 = w0; t.w1 = w1; t.sorted_slot = sorted_slot;
    t.K = K; t.Kdim = Kdim; t.Fdim = Fdim; t.T = T; t.ft = ft;
    // the tile is the same for every lane: keep it in scalar registers
    t.expert = __builtin_amdgcn_readfirstlane(loc.expert);
    t.row0 = __builtin_amdgcn_readfirstlane(loc.row0);
    t.rows = __builtin_amdgcn_readfirstlane(loc.rows);
    const int g = (t.rows + 63) >> 6;  // live 64-row groups, 1..G
    TileDispatch<C, GATEUP, OutT, C::G>::run(g, lds, t, out);
}

// worst-case number of workgroups: sum over experts of ceil(m_e / BT) with m_e <= T and sum m_e <= T*K
template <class C>
inline int ffn_grid(int T, int K, int N, int n_ftiles)
{
    const int64_t S = (int64_t)T * K;
    int64_t tiles_m = (int64_t)N * ((T + C::BT - 1) / C::BT);
    const int64_t alt = S / C::BT + N;
    if (alt < tiles_m) tiles_m = alt;
    const int64_t g = tiles_m * n_ftiles;
    return (int)((g + 7) / 8 * 8);
}

}  // namespace zeda
