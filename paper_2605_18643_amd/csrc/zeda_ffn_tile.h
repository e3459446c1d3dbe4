// Grouped bf16 GEMM tile kernel of the expert FFN (Appendix D, Eq. 10: gate, up and down projections of
// the real slots only).  See zeda_ffn.hip for how the two GEMMs use it.
//
// A work item is (expert, token tile, feature tile).  Weight rows are the MFMA "A" operand (output rows),
// tokens the "B" operand (output columns), all in 32x32 blocks with 16-wide k steps.
//
// Persistent workgroups.  The grid is one workgroup per CU slot; workgroup ids go round-robin over the 8
// XCDs, so each XCD takes a contiguous eighth of the work items that exist (their number is only known on
// the device, from expert_offsets) and its workgroups walk that eighth with a stride.  A workgroup first
// looks up its items (up to MAXQ at a time) and writes, per item, the tile location and the source row of
// every tile row to LDS; after that the main stream touches global memory only through global->LDS loads
// and the output stores.
//
// One continuous stream of chunks.  The weight tile and the token tile each move through a ring of slots in
// LDS (NSW and NST deep) in KC-wide k chunks, fetched with global->LDS loads (no staging registers): one
// wave instruction moves 64 pieces of 16 bytes to 1 KiB of consecutive LDS, so lane l fetches the piece
// that belongs at position l of that KiB.  The pieces of a row are XOR-permuted by the row index so that
// the 16 rows a fragment read touches per phase fall on distinct banks; the permutation is applied on the
// global address (or is already part of the stored layout, for tiled weights).  Half of the waves fetch
// weight rows only and the other half token rows only, so every wave's vmcnt counts one stream and the two
// rings may have different depths.  The chunks of all items of a workgroup form ONE sequence: while the
// last chunks of an item are multiplied and its result is written, the first chunks of the next item are
// already in flight, so HBM never sees the pipeline drain between tiles.  Per chunk there is one counted
// s_waitcnt (this wave's own loads of that chunk) and one s_barrier (everybody's loads have landed, and
// everybody has left the slots that are refilled next).  While all loads in flight belong to the item being
// multiplied the count is a constant of the item's shape; only an item's last chunks, during which the next
// item's first chunks are fetched, count what is in flight.  The refill is issued a few instructions at a
// time between the MFMAs that follow the barrier, so that the texture path never sees all waves issue at
// once; fragments are double-buffered in registers and read one k step ahead, and a step's MFMAs wait only
// for the fragment reads issued a whole step earlier.
//
// Only the 64-row groups of a token tile that hold rows are fetched and multiplied (their number is a
// template parameter of the tile body, so the MFMA loop has no branches), and the two wave rows take
// alternate 32-row blocks so that both always have equal work.  Results leave through a small per-wave
// LDS buffer that turns the MFMA layout (a lane owns 4 features of one token) into 64-byte row segments.
#pragma once
#include "zeda_internal.h"

namespace zeda {

template <int G_, int FB_, int WF_, int NSW_, int NST_, int KC_>
struct TileCfg {
    static constexpr int G = G_, FB = FB_, WF = WF_, NSW = NSW_, NST = NST_, KC = KC_;
    static constexpr int WT = 2;                  // wave rows: wave row wt owns token blocks wt, wt+2, ...
    static constexpr int BT = 64 * G;             // tokens per tile
    static constexpr int BF = 32 * FB * WF;       // weight rows per tile (gate and up rows both count)
    static constexpr int NW = WT * WF;            // waves
    static constexpr int NWW = NW / 2;            // waves 0..NWW-1 fetch the weight rows, the others the token rows
    static constexpr int NWT = NW - NWW;
    static constexpr int THREADS = 64 * NW;
    static constexpr int ROWB = 2 * KC;           // bytes of one row of a chunk
    static constexpr int PPR = ROWB / 16;         // 16-byte pieces per row
    static constexpr int RPI = 64 / PPR;          // rows covered by one wave load instruction
    static constexpr int KS = KC / 16;            // MFMA k steps per chunk
    static constexpr int WST = BF * ROWB, TST = BT * ROWB;  // bytes of a weight / token ring slot
    static constexpr int WRING = NSW * WST, TRING = NST * TST;
    static constexpr int NLW = BF / RPI / NWW;    // load instructions per chunk of a weight wave
    static constexpr int nlt(int g) { return 64 * g / RPI / NWT; }  // ... of a token wave with g live 64-row groups
    static constexpr int NLMAX = NLW > nlt(G) ? NLW : nlt(G);
    static constexpr int MAXQ = 8;                // items looked up at a time
    // Token tiles of an expert with m rows.  Tiles hold at most 256 rows unless the wider tile (BT > 256) saves a
    // pass over the expert's weights (just above a multiple of 256 rows), and not for experts so large that the
    // passes do not matter.
    static constexpr int SPLIT = BT < 256 ? BT : 256;
    static __host__ __device__ constexpr int tiles_of(int m)
    {
        const int narrow = (m + SPLIT - 1) / SPLIT, wide = (m + BT - 1) / BT;
        return (wide < narrow && m <= 4 * BT) ? wide : narrow;
    }
    static constexpr int TRING_OFF = WRING;
    static constexpr int TOK_OFF = WRING + TRING;            // int32 [MAXQ][BT]: source row of every tile row
    static constexpr int LOC_OFF = TOK_OFF + MAXQ * BT * 4;  // int4  [MAXQ]: expert, row0, rows, feature tile
    static constexpr int STG_OFF = LOC_OFF + MAXQ * 16;      // 2 KiB per wave: output transposition
    static constexpr int LDS_BYTES = STG_OFF + NW * 2048;
    static constexpr int WMAX = (NSW - 2) * NLW > (NST - 2) * nlt(G) ? (NSW - 2) * NLW : (NST - 2) * nlt(G);
    static_assert(KC == 32 || KC == 64, "rows of 64 or 128 bytes");
    static_assert((BF / RPI) % NWW == 0 && (64 / RPI) % NWT == 0, "loads must divide evenly over the waves of a role");
    static_assert(NSW >= 2 && NST >= 2 && (NSW - 1) * NLW <= 63 && (NST - 1) * nlt(G) <= 63, "vmcnt is a 6-bit counter");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS is 160 KiB per CU");
};

// position of logical piece p of row r inside its LDS row (an involution in p)
template <int KC>
__device__ __forceinline__ int swz(int row, int piece)
{
    return KC == 64 ? (piece ^ ((row >> 1) & 7)) : (piece ^ ((row >> 2) & 3));
}

// silu(g) * u with the hardware reciprocal (1 ulp) in place of an IEEE division: the result is rounded to bf16
// right after, and the division sequence was a quarter of the gate/up epilogue's instructions
__device__ __forceinline__ float silu_mul(float g, float u)
{
    return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u;
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// s_waitcnt vmcnt(n) for a wave-uniform n in LO..HI (the count is an immediate, so this is a decision tree)
template <int LO, int HI>
__device__ __forceinline__ void wait_vmcnt_tree(int n)
{
    if constexpr (LO == HI) {
        wait_vmcnt<LO>();
    } else {
        constexpr int MID = (LO + HI) / 2;
        if (n <= MID) wait_vmcnt_tree<LO, MID>(n);
        else wait_vmcnt_tree<MID + 1, HI>(n);
    }
}

// LDS accesses the compiler does not see as such.  It orders every LDS access it knows about behind all
// global->LDS loads in flight (s_waitcnt vmcnt(0)), which would drain the ring at every table lookup and
// output transposition; these go around it and wait on lgkmcnt themselves.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)(uintptr_t)p; }  // low half of a flat LDS address
__device__ __forceinline__ uint32_t lds_read_b32(uint32_t a)
{
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"(a) : "memory");
    return v;
}
__device__ __forceinline__ u32x4 lds_read_b128(uint32_t a)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(a) : "memory");
    return v;
}
template <int OFF>
__device__ __forceinline__ u32x4 lds_read_b128_at(uint32_t a)  // a + OFF, the constant in the instruction's offset field
{
    static_assert(OFF >= 0 && OFF < 65536, "16-bit offset field");
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(a), "n"(OFF) : "memory");
    return v;
}
__device__ __forceinline__ void lds_write_b64(uint32_t a, u32x2 v)
{
    asm volatile("ds_write_b64 %0, %1" ::"v"(a), "v"(v) : "memory");
}
// results of the reads above may be used after this
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void lds_wait(uint32_t &a) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a)::"memory"); }
__device__ __forceinline__ void lds_wait(u32x4 &a) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a)::"memory"); }
__device__ __forceinline__ void lds_wait(u32x4 &a, u32x4 &b) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b)::"memory"); }

#define ZEDA_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define ZEDA_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

// Per-lane view of expert_offsets: lane l holds experts 4l..4l+3, their tile counts and the running total.
template <class C>
struct TileScan {
    int off[5], nt[4], incl, local, tiles;
    __device__ __forceinline__ void init(const int32_t *__restrict__ offsets, int N)
    {
        const int lane = threadIdx.x & 63;
        int o[5];
#pragma unroll
        for (int q = 0; q < 5; ++q) o[q] = offsets[min(4 * lane + q, N)];
        init(o);
    }
    // from this lane's five offsets, already loaded
    __device__ __forceinline__ void init(const int (&o)[5])
    {
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int q = 0; q < 5; ++q) off[q] = o[q];
        local = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            nt[q] = C::tiles_of(off[q + 1] - off[q]);
            local += nt[q];
        }
        incl = local;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            int v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        tiles = __shfl(incl, 63);
    }
    // experts with at least one row (the same value in every lane)
    __device__ __forceinline__ int experts() const
    {
        int ne = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) ne += nt[q] > 0;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) ne += __shfl_xor(ne, o);
        return ne;
    }
    // (expert, first sorted row, rows, feature tile) of work item `item` = token tile * n_ftiles + feature tile;
    // the m rows of an expert are split evenly over its tiles, each a multiple of 64 rows except the last.
    __device__ __forceinline__ int4 locate(int item, int n_ftiles) const
    {
        const int lane = threadIdx.x & 63;
        const int tile_m = item / n_ftiles;
        const int ft = item - tile_m * n_ftiles;
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
        const int per = (((m + ntile - 1) / ntile) + 63) & ~63;
        return make_int4(e, o0 + mt * per, min(per, m - mt * per), ft);
    }
};

// WNT: fetch the weights with the non-temporal hint (see run_tiles).
template <class C, bool GATEUP, bool TILED, bool WNT = false>
struct Stream {
    static constexpr int FB = C::FB, WF = C::WF, BT = C::BT, BF = C::BF, NSW = C::NSW, NST = C::NST, NW = C::NW,
                         NWW = C::NWW, NWT = C::NWT, WST = C::WST, TST = C::TST, KC = C::KC, KS = C::KS, ROWB = C::ROWB,
                         PPR = C::PPR, RPI = C::RPI, NLMAX = C::NLMAX, NLW = C::NLW;
    static constexpr int NH = (NSW > NST ? NSW : NST) > 2 ? (NSW > NST ? NSW : NST) - 2 : 1;
    static_assert(!TILED || KC == 32, "tiled weights are stored in 32-wide k blocks");

    // kernel arguments
    const bf16_t *tok, *w0, *w1;
    bf16_t *out;
    int Kdim, Fdim, nk;
    // LDS
    unsigned char *wring, *tring, *stg;
    uint32_t wring_a, tring_a;  // LDS addresses of the two rings
    const int *s_tok;
    const int4 *s_loc;
    // thread position
    int lane, wave, wt, wf, col, half;
    int foff_w, foff_t;  // byte offset in a slot of this lane's k-step-0 fragment of weight block 0 / token block wt
    // Issue side.  A wave fetches one operand only, so that its vmcnt orders one stream: weight waves run
    // NSW-1 chunks ahead of the MFMAs, token waves NST-1 (token rows mostly come from L2 and need less lead).
    // The next chunk this wave fetches is chunk ikc of item iq, into slot islot of its ring.
    bool wrole;
    const bf16_t *src[NLMAX];
    int nq, iq, ikc, islot, inl;
    size_t koff;          // ikc chunks into the rows, in elements
    int kstep;            // elements from one chunk of this wave's operand to the next
    uint32_t dbase, doff; // LDS address of this wave's first piece in slot 0 of its ring; byte offset of slot islot
    int hist[NH];  // load instructions of this wave in each of the last chunks issued (newest last)
    // compute side: slots of the chunk being multiplied
    int cslot_w, cslot_t;

    __device__ __forceinline__ int4 read_loc(int q) const
    {
        u32x4 v = lds_read_b128(lds_addr(s_loc + q));
        lds_wait(v);
        return make_int4(__builtin_amdgcn_readfirstlane(v[0]), __builtin_amdgcn_readfirstlane(v[1]),
                         __builtin_amdgcn_readfirstlane(v[2]), __builtin_amdgcn_readfirstlane(v[3]));
    }
    __device__ __forceinline__ void setup_issue_item()
    {
        if (iq >= nq) { inl = 0; return; }
        const int4 loc = read_loc(iq);
        const int expert = loc.x, rows = loc.z, ft = loc.w;
        int ln = lane;
        asm volatile("" : "+v"(ln));  // (recomputed per item rather than kept live)
        const int piece = ln % PPR, rsub = ln / PPR;
        if (wrole) {
            inl = NLW;
#pragma unroll
            for (int i = 0; i < NLW; ++i) {
                const int jw = wave + NWW * i;  // covers rows jw*RPI.. of the weight tile
                if (TILED) {
                    // 16 rows = one half of a stored 32x32 unit, already in LDS order: lane l copies piece l
                    const int lb = jw >> 1, blk = lb % FB, wfr = lb / FB;
                    const bf16_t *wbase = (GATEUP && (blk & 1)) ? w1 : w0;
                    const int rb = GATEUP ? ft * (BF / 64) + wfr * (FB / 2) + (blk >> 1) : ft * (BF / 32) + lb;
                    src[i] = wbase + ((size_t)expert * (Kdim / 32) * (Fdim / 32) + rb) * 1024 + (jw & 1) * 512 + ln * 8;
                } else {
                    const int row = jw * RPI + rsub;
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
                    src[i] = wbase + ((size_t)expert * Fdim + grow) * Kdim + swz<KC>(row, piece) * 8;
                }
            }
        } else {
            const int g = (rows + 63) >> 6;
            inl = C::nlt(g);
            uint32_t srow[NLMAX];
#pragma unroll
            for (int i = 0; i < C::nlt(C::G); ++i)  // (entries past the live groups are read, and never used)
                srow[i] = lds_read_b32(lds_addr(s_tok + iq * BT + min(wave - NWW + NWT * i, NWT * inl - 1) * RPI + rsub));
#pragma unroll
            for (int i = 0; i < C::nlt(C::G); ++i) lds_wait(srow[i]);
#pragma unroll
            for (int i = 0; i < C::nlt(C::G); ++i) {
                const int trow = (wave - NWW + NWT * i) * RPI + rsub;
                src[i] = tok + (size_t)srow[i] * Kdim + swz<KC>(trow, piece) * 8;
            }
        }
    }
    __device__ __forceinline__ void init_issue()
    {
        wring_a = lds_addr(wring);
        tring_a = lds_addr(tring);
        kstep = (TILED && wrole) ? (Fdim / 32) * 1024 : KC;
        dbase = lds_addr(wrole ? wring + wave * 1024 : tring + (wave - NWW) * 1024);
        iq = 0; ikc = 0; islot = 0; inl = 0; koff = 0; doff = 0;
#pragma unroll
        for (int h = 0; h < NH; ++h) hist[h] = 0;
    }
    __device__ __forceinline__ void load_piece(int i)
    {
        const uint32_t dst = dbase + doff + i * ((NWW == NWT ? NWW : (wrole ? NWW : NWT)) * 1024);
        // (the cache-policy field of the instruction is an immediate, hence two instructions)
        if (WNT && wrole)
            __builtin_amdgcn_global_load_lds(ZEDA_GLOBAL_PTR(src[i] + koff),
                                             (__attribute__((address_space(3))) void *)(uintptr_t)dst, 16, 0, 2 /* nt */);
        else
            __builtin_amdgcn_global_load_lds(ZEDA_GLOBAL_PTR(src[i] + koff),
                                             (__attribute__((address_space(3))) void *)(uintptr_t)dst, 16, 0, 0);
    }
    // the issue position moves on by one chunk inside the current item
    __device__ __forceinline__ void next_chunk_same_item()
    {
        ++ikc;
        koff += kstep;
        const bool wrap = ++islot == (NSW == NST ? NSW : (wrole ? NSW : NST));
        doff = wrap ? 0 : doff + (WST == TST ? WST : (wrole ? WST : TST));
        islot = wrap ? 0 : islot;
    }
    // load instruction i of the chunk being issued (i < ni, wave-uniform)
    __device__ __forceinline__ void issue_one(int i, int ni)
    {
        if (i < ni) load_piece(i);
    }
    // the same when the chunk belongs to an item with GA live groups and the stream has not ended: the count is known
    template <int GA>
    __device__ __forceinline__ void issue_one_of(int i)
    {
        constexpr int NT = C::nlt(GA);
        if (i < NLW && i < NT) load_piece(i);
        else if (i < NLW) { if (wrole) load_piece(i); }
        else if (i < NT) { if (!wrole) load_piece(i); }
    }
    // bookkeeping after the instructions of one chunk were issued (ni of them; 0 once the stream has ended)
    __device__ __forceinline__ void issued(int ni)
    {
#pragma unroll
        for (int h = 0; h + 1 < NH; ++h) hist[h] = hist[h + 1];
        hist[NH - 1] = ni;
        if (iq < nq) {
            next_chunk_same_item();
            next_item_if_done();
        }
    }
    // past the last chunk of the item: the next chunk to fetch is the first one of the next item
    __device__ __forceinline__ void next_item_if_done()
    {
        if (ikc == nk) {
            ikc = 0;
            koff = 0;
            ++iq;
            setup_issue_item();
        }
    }
    __device__ __forceinline__ void issue_burst()
    {
        const int ni = inl;
#pragma unroll
        for (int i = 0; i < NLMAX; ++i) issue_one(i, ni);
        issued(ni);
    }
    // This wave's loads of the oldest chunk in flight have landed: all but the chunks issued after it
    // (depth - 2 of them, the newest entries of hist) may still be outstanding.
    __device__ __forceinline__ void wait_oldest()
    {
        int w = 0;
#pragma unroll
        for (int h = 0; h < NH; ++h)
            if (NH - h <= (wrole ? NSW - 2 : NST - 2)) w += hist[h];
        wait_vmcnt_tree<0, C::WMAX>(min(w, C::WMAX));
    }

    // Fragments of k step s of the chunk in `slot`: FB weight blocks of this wave column, GA token blocks of this
    // wave row.  Blocks start at multiples of 32 rows, so the piece permutation depends on `col` only and the
    // address is one per-lane term (foff, XOR 32*s) plus block offsets that are immediates.
    // The reads go around the compiler (see the LDS helpers above) so that the wait before a step's MFMAs can be a
    // counted one: it leaves the reads of the step after it, issued just before, in flight.
    template <int I, int N, int STRIDE>
    static __device__ __forceinline__ void read_blocks(uint32_t base, u32x4 *out)
    {
        if constexpr (I < N) {
            out[I] = lds_read_b128_at<I * STRIDE>(base);
            read_blocks<I + 1, N, STRIDE>(base, out);
        }
    }
    // wslot, tslot: LDS addresses of the chunk's weight and token slot
    template <int GA>
    __device__ __forceinline__ void load_frags(uint32_t wslot, uint32_t tslot, int s, u32x4 (&fa)[FB], u32x4 (&tb)[GA]) const
    {
        read_blocks<0, FB, 32 * ROWB>(wslot + (foff_w ^ (s << 5)), fa);
        read_blocks<0, GA, 64 * ROWB>(tslot + (foff_t ^ (s << 5)), tb);
    }
    // the fragments in fa, tb have landed when at most `newer` LDS reads issued after them are still in flight
    template <int NEWER, int GA>
    __device__ __forceinline__ void frags_landed(u32x4 (&fa)[FB], u32x4 (&tb)[GA]) const
    {
        asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(NEWER) : "memory");
#pragma unroll
        for (int b = 0; b < FB; ++b) asm volatile("" : "+v"(fa[b]));
#pragma unroll
        for (int a = 0; a < GA; ++a) asm volatile("" : "+v"(tb[a]));
    }

    // One chunk of an item with GA live groups: KS k steps; in the last one the next chunk is awaited, everybody
    // meets, and the slot everybody has left is refilled.  MAIN: all loads in flight are this item's (see tile_body).
    // MORE: the item has another chunk after this one (its first fragments are read here, after the meeting).
    template <int GA, bool MAIN, bool MORE>
    __device__ __forceinline__ void chunk(f32x16 (&acc)[GA][FB], u32x4 (&fa)[2][FB], u32x4 (&tb)[2][GA])
    {
        const uint32_t cur_w = wring_a + cslot_w * WST, cur_t = tring_a + cslot_t * TST;
        const int nslot_w = cslot_w + 1 == NSW ? 0 : cslot_w + 1, nslot_t = cslot_t + 1 == NST ? 0 : cslot_t + 1;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int p = s & 1;
            int ni = 0;
            if (s < KS - 1) {
                load_frags<GA>(cur_w, cur_t, s + 1, fa[p ^ 1], tb[p ^ 1]);
                frags_landed<FB + GA, GA>(fa[p], tb[p]);
            } else {
                // every fragment of this chunk is in registers: nobody needs its slot any more
                frags_landed<0, GA>(fa[p], tb[p]);
                // Wait for the next chunk, meet, refill the slot everybody has just left.  After the item's last
                // chunk the next chunk is the first one of the next item (nothing, at the end of the stream): it is
                // awaited HERE, before the epilogue, because the epilogue's stores count in vmcnt too - a wait
                // right after them would have to sit out their whole round trip.
                if (MAIN) {
                    constexpr int WW = (NSW - 2) * NLW, WT_ = (NST - 2) * C::nlt(GA);
                    if (WW == WT_) wait_vmcnt<WW>();
                    else if (wrole) wait_vmcnt<WW>();
                    else wait_vmcnt<WT_>();
                } else {
                    wait_oldest();
                }
                __builtin_amdgcn_s_barrier();
                if (MORE) load_frags<GA>(wring_a + nslot_w * WST, tring_a + nslot_t * TST, 0, fa[p ^ 1], tb[p ^ 1]);
                ni = inl;
            }
            // keep the reads of the next step ahead of this step's MFMAs
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < GA; ++a)
#pragma unroll
                for (int b = 0; b < FB; ++b) {
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[p][b]),
                                                                        __builtin_bit_cast(bf16x8, tb[p][a]), acc[a][b], 0, 0, 0);
                    if (s == KS - 1) {
                        // the refill of the slot freed by the barrier, spread over this step's MFMAs
                        constexpr int NM = GA * FB;
                        const int m = a * FB + b;
#pragma unroll
                        for (int i = 0; i < NLMAX; ++i)
                            if (i * NM / NLMAX == m) {
                                if (MAIN) issue_one_of<GA>(i);
                                else issue_one(i, ni);
                            }
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
            if (s == KS - 1) {
                if (MAIN) next_chunk_same_item();
                else issued(ni);
            }
        }
        cslot_w = nslot_w;
        cslot_t = nslot_t;
    }

    // One item with GA live 64-row groups: its nk chunks, then the epilogue.
    template <int GA>
    __device__ __forceinline__ void tile_body(int expert, int row0, int rows, int ft)
    {
        f32x16 acc[GA][FB];
#pragma unroll
        for (int a = 0; a < GA; ++a)
#pragma unroll
            for (int b = 0; b < FB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

        // On entry the item's first chunk has landed and everybody has met after waiting for it (the item before,
        // or the start of the stream, saw to that).
        u32x4 fa[2][FB], tb[2][GA];
        load_frags<GA>(wring_a + cslot_w * WST, tring_a + cslot_t * TST, 0, fa[0], tb[0]);

        // Main part: the chunks during which every load in flight belongs to this item, so that the number of loads
        // that may stay outstanding at the wait is a constant of the item's shape (an immediate).  The last chunks,
        // during which the first chunks of the next item are fetched, take the counted path.
        constexpr int NSMAX = NSW > NST ? NSW : NST;
        const int n_main = nk > NSMAX ? nk - NSMAX : 0;  // chunk kc refills with chunk kc + depth: still this item's
        int kc = 0;
        for (; kc < n_main; ++kc) chunk<GA, true, true>(acc, fa, tb);
        if (n_main > 0) {
#pragma unroll
            for (int h = 0; h < NH; ++h) hist[h] = wrole ? NLW : C::nlt(GA);
            next_item_if_done();  // (the deeper ring's last refill there was the item's last chunk)
        }
        for (; kc + 1 < nk; ++kc) chunk<GA, false, true>(acc, fa, tb);
        chunk<GA, false, false>(acc, fa, tb);

        // Epilogue.  acc[a][b][v] is feature 8*(v/4) + 4*half + v%4 of weight block b, token `col` of token
        // block 2a + wt.  Each 32x32 result block goes through this wave's LDS buffer (rows of 32 bf16, pieces
        // permuted by the row) and leaves as 16 bytes per lane, four lanes to a token row.
        constexpr int NOB = GATEUP ? FB / 2 : FB;
        int ln = lane;
        asm volatile("" : "+v"(ln));  // (keeps the address arithmetic below out of the main loop's registers)
        const int ecol = ln & 31, ehalf = ln >> 5;
        // staging buffer: token row `ecol` holds 32 features as 4 pieces of 16 bytes, piece p at position
        // p ^ ((row >> 2) & 3); a lane writes the half `ehalf` of piece vq and reads piece ln & 3 of rows ln >> 2, + 16
        const uint32_t stg_w = lds_addr(stg) + ecol * 64 + ((ecol >> 2) & 3) * 16 + ehalf * 8;
        const uint32_t stg_r = lds_addr(stg) + (ln >> 2) * 64 + ((ln & 3) ^ ((ln >> 4) & 3)) * 16;
#pragma unroll
        for (int a = 0; a < GA; ++a) {
            const int trow0 = (2 * a + wt) * 32;
            if (trow0 < rows) {
#pragma unroll
                for (int ob = 0; ob < NOB; ++ob) {
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        bf16x4 v;
                        if (GATEUP) {
                            const f32x16 &g = acc[a][2 * ob], &u = acc[a][2 * ob + 1];
#pragma unroll
                            for (int k = 0; k < 4; ++k) v[k] = (bf16_t)silu_mul(g[4 * vq + k], u[4 * vq + k]);
                        } else {
#pragma unroll
                            for (int k = 0; k < 4; ++k) v[k] = (bf16_t)acc[a][ob][4 * vq + k];
                        }
                        lds_write_b64(stg_w ^ (vq << 4), __builtin_bit_cast(u32x2, v));
                    }
                    const int c0 = GATEUP ? ft * (BF / 2) + (wf * (FB / 2) + ob) * 32 : ft * BF + (wf * FB + ob) * 32;
                    u32x4 o0 = lds_read_b128(stg_r), o1 = lds_read_b128(stg_r + 16 * 64);
                    lds_wait(o0, o1);
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const int r = 16 * i + (ln >> 2), pc = ln & 3;
                        if (trow0 + r < rows)
                            *reinterpret_cast<u32x4 *>(out + (size_t)(row0 + trow0 + r) * Fdim + c0 + pc * 8) = i ? o1 : o0;
                        // (a non-empty block after the per-lane branch: if that branch joined straight into a loop
                        // header the compiler would treat all the wave-uniform stream state as divergent)
                        asm volatile("" ::: "memory");
                    }
                }
            }
        }
    }
};

template <class S, int GA>
struct TileDispatch {
    static __device__ __forceinline__ void run(S &st, int g, int expert, int row0, int rows, int ft)
    {
        if (g == GA) st.template tile_body<GA>(expert, row0, rows, ft);
        else TileDispatch<S, GA - 1>::run(st, g, expert, row0, rows, ft);
    }
};
template <class S>
struct TileDispatch<S, 0> {
    static __device__ __forceinline__ void run(S &, int, int, int, int, int) {}
};

// GATEUP: tok = x[T,Kdim], w0 = W_gate[N,Fdim,Kdim], w1 = W_up, out = act[S,Fdim] (Fdim = I, Kdim = H).
// DOWN:   tok = act[S,Kdim], w0 = W_down[N,Fdim,Kdim], out = y_slot[S,Fdim]        (Fdim = H, Kdim = I).
// Kdim is a multiple of KC; Fdim a multiple of the feature tile (BF/2 for GATEUP, BF for DOWN).
// TILED: the weights are in the layout pack_weights_kernel writes.  The grid is a multiple of 8 workgroups.
template <class C, bool GATEUP, bool TILED, bool WNT>
__device__ __forceinline__ void run_tiles(unsigned char *lds, const TileScan<C> &scan0, const bf16_t *__restrict__ tok,
                                          const bf16_t *__restrict__ w0,
                                          const bf16_t *__restrict__ w1, const int32_t *__restrict__ offsets,
                                          const int32_t *__restrict__ sorted_slot, bf16_t *__restrict__ out, int N, int K,
                                          int Kdim, int Fdim, int n_ftiles, int T)
{
    static_assert(!GATEUP || C::FB % 2 == 0, "gate and up blocks come in pairs");
    int *s_tok = reinterpret_cast<int *>(lds + C::TOK_OFF);
    int4 *s_loc = reinterpret_cast<int4 *>(lds + C::LOC_OFF);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // the work items of this workgroup: first + i * stride below end
    const int wgs = gridDim.x >> 3, xcd = blockIdx.x & 7, wg = blockIdx.x >> 3;
    int mine, first;
    {
        const int items = scan0.tiles * n_ftiles, per_xcd = (items + 7) / 8;
        const int lo = xcd * per_xcd, hi = min(lo + per_xcd, items);
        first = lo + wg;
        mine = first < hi ? (hi - first + wgs - 1) / wgs : 0;
    }
    mine = __builtin_amdgcn_readfirstlane(mine); first = __builtin_amdgcn_readfirstlane(first);

    for (int q0 = 0; q0 < mine; q0 += C::MAXQ) {
        const int nq = min(C::MAXQ, mine - q0);
        if (q0 > 0) __syncthreads();  // everybody has left the tables and the ring of the batch before
        {
            TileScan<C> sc;
            sc.init(offsets, N);
            for (int q = wave; q < nq; q += C::NW) {
                const int4 loc = sc.locate(first + (q0 + q) * wgs, n_ftiles);
                if (lane == 0) s_loc[q] = loc;
            }
        }
        __syncthreads();
        for (int idx = tid; idx < nq * C::BT; idx += C::THREADS) {
            const int q = idx / C::BT, r = idx - q * C::BT;
            const int4 loc = s_loc[q];
            const int rr = loc.y + min(r, loc.z - 1);  // rows past the tile repeat its last row (never stored)
            s_tok[idx] = GATEUP ? min(max(sorted_slot[rr] / K, 0), T - 1) : rr;  // a bad index must not fault
        }
        __syncthreads();

        Stream<C, GATEUP, TILED, WNT> st;
        st.tok = tok; st.w0 = w0; st.w1 = w1; st.out = out;
        st.Kdim = Kdim; st.Fdim = Fdim; st.nk = Kdim / C::KC;
        st.wring = lds; st.tring = lds + C::TRING_OFF; st.stg = lds + C::STG_OFF + wave * 2048; st.s_tok = s_tok; st.s_loc = s_loc;
        st.lane = lane; st.wave = wave; st.wt = wave / C::WF; st.wf = wave % C::WF; st.col = lane & 31; st.half = lane >> 5;
        st.foff_t = (st.wt * 32 + st.col) * C::ROWB + swz<C::KC>(st.col, st.half) * 16;
        st.foff_w = (st.wf * C::FB * 32 + st.col) * C::ROWB + swz<C::KC>(st.col, st.half) * 16;
        st.wrole = wave < C::NWW;
        st.nq = nq; st.cslot_w = 0; st.cslot_t = 0;
        st.init_issue();
        st.setup_issue_item();
        for (int c = 0, n = (st.wrole ? C::NSW : C::NST) - 1; c < n; ++c) st.issue_burst();
        // all slots of this wave's ring but one are in flight: wait for the first chunk, meet, fill the last slot
        st.wait_oldest();
        __builtin_amdgcn_s_barrier();
        st.issue_burst();

        for (int q = 0; q < nq; ++q) {
            const int4 loc = st.read_loc(q);
            TileDispatch<Stream<C, GATEUP, TILED, WNT>, C::G>::run(st, (loc.z + 63) >> 6, loc.x, loc.y, loc.z, loc.w);
        }
    }
}

// Weights that are read once - every expert one token tile - and that are what the kernel waits for - few rows per
// expert - are fetched with the non-temporal hint: they then do not push the token rows, the activations and the
// results, which this and the next kernels of the layer re-read, out of the caches (whole layer at 127 rows per
// expert -4 %, at 3 rows -10 %; at 460 rows per expert the hint costs 2 % instead).  Decided once per launch from
// the expert loads; the cache-policy field of the load is an immediate, so the two cases are two instantiations.
template <class C, bool GATEUP, bool TILED>
__device__ __forceinline__ void run_tiles_auto(unsigned char *lds, const TileScan<C> &scan0, const bf16_t *__restrict__ tok,
                                               const bf16_t *__restrict__ w0, const bf16_t *__restrict__ w1,
                                               const int32_t *__restrict__ offsets, const int32_t *__restrict__ sorted_slot,
                                               bf16_t *__restrict__ out, int N, int K, int Kdim, int Fdim, int n_ftiles,
                                               int T)
{
    const int ne = scan0.experts();
    const bool stream_once = scan0.tiles * 16 <= ne * 17 && offsets[N] < 400 * ne;
    if (stream_once)
        run_tiles<C, GATEUP, TILED, true>(lds, scan0, tok, w0, w1, offsets, sorted_slot, out, N, K, Kdim, Fdim, n_ftiles, T);
    else
        run_tiles<C, GATEUP, TILED, false>(lds, scan0, tok, w0, w1, offsets, sorted_slot, out, N, K, Kdim, Fdim, n_ftiles, T);
}

template <class C, bool GATEUP, bool TILED>
__global__ __launch_bounds__(C::THREADS) void ffn_bf16_kernel(const bf16_t *__restrict__ tok,
                                                              const bf16_t *__restrict__ w0,
                                                              const bf16_t *__restrict__ w1,
                                                              const int32_t *__restrict__ offsets,
                                                              const int32_t *__restrict__ sorted_slot,
                                                              bf16_t *__restrict__ out, int N, int K, int Kdim, int Fdim,
                                                              int n_ftiles, int T)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    TileScan<C> sc;
    sc.init(offsets, N);
    run_tiles_auto<C, GATEUP, TILED>(lds, sc, tok, w0, w1, offsets, sorted_slot, out, N, K, Kdim, Fdim, n_ftiles, T);
}

// The same with two tile geometries in one kernel, chosen from the expert loads when the kernel starts: CB, whose
// token tile is wider than 256 rows, where it makes noticeably fewer passes over expert weights than CA (experts
// with a few rows more than CA's tile would otherwise stream their weights twice), else CA.  Every wave computes
// the same choice from expert_offsets.
template <class CA, class CB, bool GATEUP, bool TILED>
__global__ __launch_bounds__(CA::THREADS) void ffn_bf16_adaptive_kernel(const bf16_t *__restrict__ tok,
                                                                        const bf16_t *__restrict__ w0,
                                                                        const bf16_t *__restrict__ w1,
                                                                        const int32_t *__restrict__ offsets,
                                                                        const int32_t *__restrict__ sorted_slot,
                                                                        bf16_t *__restrict__ out, int N, int K, int Kdim,
                                                                        int Fdim, int n_ftiles, int T)
{
    static_assert(CA::THREADS == CB::THREADS && CA::BF == CB::BF, "one launch shape, one feature tiling");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    TileScan<CA> sa;
    sa.init(offsets, N);
    TileScan<CB> sb;
    sb.init(sa.off);
    if (sb.tiles * 16 <= sa.tiles * 15)  // at least one pass in sixteen saved
        run_tiles_auto<CB, GATEUP, TILED>(lds, sb, tok, w0, w1, offsets, sorted_slot, out, N, K, Kdim, Fdim, n_ftiles, T);
    else
        run_tiles_auto<CA, GATEUP, TILED>(lds, sa, tok, w0, w1, offsets, sorted_slot, out, N, K, Kdim, Fdim, n_ftiles, T);
}

// Tiled weight layout.  A matrix W[F][Kd] (F, Kd multiples of 32) is stored as (F/32) x (Kd/32) units of 2 KiB,
// unit (rb, kb) at index kb * (F/32) + rb, so that the row blocks of one k block follow each other: the
// consecutive row blocks of a feature tile are then one contiguous run of 8-16 KiB per k chunk.  A
// unit holds rows 32rb..32rb+31, columns 32kb..32kb+31 as 32 rows of 64 bytes, the four 16-byte pieces of
// row r permuted as in the LDS ring (piece p at position p ^ ((r >> 2) & 3)): it is the LDS image of that
// block, so the GEMM copies it with contiguous 1 KiB loads - which is what lets HBM stream at full rate
// (row-major weights are fetched as 64- or 128-byte pieces 2*Kd bytes apart).
// One thread per 16-byte piece of the output; `mats` matrices of F x Kd follow each other.
__global__ __launch_bounds__(256) void pack_weights_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ out, int F,
                                                           int Kd, size_t pieces)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= pieces) return;
    const int pos = idx & 3, r = (idx >> 2) & 31;
    const size_t unit = idx >> 7;
    const int kbs = Kd / 32, units_per_mat = (F / 32) * kbs;
    const size_t mat = unit / units_per_mat;
    const int u = (int)(unit - mat * units_per_mat), rbs = F / 32, kb = u / rbs, rb = u - kb * rbs;
    const int p = pos ^ ((r >> 2) & 3);
    const bf16x8 v = *reinterpret_cast<const bf16x8 *>(w + (mat * F + rb * 32 + r) * Kd + kb * 32 + p * 8);
    *reinterpret_cast<bf16x8 *>(out + idx * 8) = v;
}

}  // namespace zeda
