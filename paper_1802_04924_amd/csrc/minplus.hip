// Node elimination (Sec. 5.2, Eq. 2) as a batched min-plus matrix product with argmin:
//   out[a][b] = min_c ( A[a][c] + w[c] + B[c][b] ),  arg[a][b] = lowest c attaining the minimum.
//
// (min,+) is not a ring the matrix cores implement, so this runs on the integer VALU.  One
// workgroup (256 threads = 4 wavefronts) owns a square output tile and walks c in stages of TK
// candidates that are staged through LDS (double-buffered, one barrier per stage, the next stage's
// global loads in flight meanwhile); every thread keeps an RB x RB block of running minima in
// registers (RB = 4: 64 x 64 tiles, TK = 32, 4 wavefronts per SIMD; RB = 8: 128 x 128 tiles,
// TK = 16, 2 per SIMD).  w is folded into A while A is staged, so the inner loop is one add and
// half a three-way min per candidate.  When a launch has far fewer tiles than the chip has compute
// units, several workgroups share one tile: each walks its own contiguous part of the c range and
// publishes its (minimum, argmin) block to global scratch; the workgroup that arrives last merges
// the parts in ascending-c order with a strict '<', which keeps the lowest-index rule.
//
// Four arithmetic variants:
//   keyed   candidates are 32-bit keys (cost << tb) | (1 + position of c in its chunk); a chunk
//           is `spc` stages (TK*spc <= 2^tb - 1 consecutive c).  An unsigned min over keys
//           carries the lowest c of equal costs inside a chunk for free.  At every chunk end a
//           non-zero low field says the minimum changed in this chunk: (chunk, position) is
//           recorded and the field is cleared, so a later chunk can only win with a strictly
//           smaller cost.  Costs are re-based to start at 0 and, where that is tighter, clamped
//           just above the largest value the result can take (a clamped candidate can neither be
//           the minimum nor tie with it); they must then fit 32-tb bits.  The launcher's caller
//           guarantees that from value ranges; the kernel derives tb itself from the ranges it is
//           given (measured ones where an earlier launch of the same stream left them).
//   keyed, re-based per row   as keyed, but A + w is re-based to the minimum of its own row (over
//           the c range the workgroup walks) and clamped just above the spread of B: a candidate
//           further above its row's minimum than B's spread can never win.  Key width then depends
//           on the spread of B alone, however wide the values of A and w range (cost tables mix
//           nanosecond-scale and second-scale entries).  Costs one extra pass over the A rows.
//   plain   int32 compare/select per candidate (strict '<' in ascending c); no precondition.
//   value   the minimum only (signed three-way min, no argmin, no precondition), for callers that
//           recompute the argmin of the few cells they need afterwards, as the paper's undo pass does.
// A launch may mix products of different shapes (MIXED, 64 x 64 tiles): a prefix array of tile
// counts tells a workgroup which product its tile belongs to.
#include "lwp_kernels.h"

namespace lwp {

namespace {

constexpr int NT = kNodeThreads;

using v4i = int __attribute__((ext_vector_type(4)));
using gv4cptr = const v4i __attribute__((address_space(1)))*;
using gv4ptr = v4i __attribute__((address_space(1)))*;

__device__ __forceinline__ int wave_min_i32(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ int wave_max_i32(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o));
    return v;
}

// Which variant a product runs on when the choice is made on the device (guarded launches), from the
// measured ranges of its operands: packed keys on global offsets if their spread fits `limit`, else
// keys re-based per row if allowed and the spread of B fits them, else the plain variant.  A product
// whose sums may leave int32 is flagged by the kernels and runs on the plain variant.
__device__ __forceinline__ int auto_variant(long long loA, long long hiA, long long loW, long long hiW, long long loB,
                                            long long hiB, long long limit, bool row_ok) {
    const long long hi = hiA + hiW + hiB, lo = loA + loW + loB, hi2 = hiA + hiW, lo2 = loA + loW;
    if (hi > 2147483647ll || lo < -2147483648ll || hi2 > 2147483647ll || lo2 < -2147483648ll) return kModePlain;
    const long long a_max = hiA + hiW - (loA + loW), out_max = (hiA - loA) + (hiB - loB);
    if (min(a_max, out_max + 1) + (hiB - loB) <= limit) return kModeKeyed;
    if (row_ok && 2 * (hiB - loB) + 1 <= kKeyedMaxSpreadSmall) return kModeKeyedRow;
    return kModePlain;
}

// What one workgroup works on: the product's descriptor, its tile of that product, and -- for a tile
// shared by several workgroups -- its part of the c range.
struct TileWork {
    NodeDesc d;
    int tl;                 // tile index inside the product
    int part, kparts;       // this workgroup's part of the c range (kparts == 1: the whole range)
    uint32_t split_idx;     // index of a shared tile among the launch's shared tiles
};

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give every XCD a
// contiguous range of logical ids, and walk the tiles of a product in panels of 8 tile rows,
// column by column: 64 consecutive ids (the tiles resident on one XCD at a time) then form an
// 8 x 8 block that shares 8 row strips of A and 8 column strips of B.
// Split tiles (64 x 64 tiles only): the launch's first n_whole tiles have one workgroup each;
// every later tile is shared by kparts consecutive workgroups, each with a part of the c range.
// The shared tiles come last in dispatch order, so that the short workgroups fill the launch's
// last, partly empty round of workgroup slots.
template <int RB, bool MIXED>
__device__ __forceinline__ void decode_work(const NodeArgs& p, TileWork& w) {
    uint32_t bid = blockIdx.x;
    const uint32_t n_whole = (RB == 4 && p.kparts > 1) ? (uint32_t)p.n_whole : gridDim.x;
    w.kparts = 1; w.part = 0; w.split_idx = 0;
    if (bid < n_whole) {
        if ((n_whole & 7u) == 0u) bid = (bid & 7u) * (n_whole >> 3) + (bid >> 3);
    } else {
        uint32_t x = bid - n_whole;
        const uint32_t rest = gridDim.x - n_whole;
        if ((rest & 7u) == 0u) x = (x & 7u) * (rest >> 3) + (x >> 3);
        w.kparts = p.kparts;
        w.part = (int)(x % (uint32_t)w.kparts);
        w.split_idx = x / (uint32_t)w.kparts;
        bid = n_whole + w.split_idx;
    }
    int bi;
    if (MIXED) {
        // products of different shapes: find the one that owns this tile (uniform binary search)
        const int32_t __attribute__((address_space(1)))* tb0 = (const int32_t __attribute__((address_space(1)))*)(uintptr_t)p.tile_begin;
        int lo = 0, hi = p.batch;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((uint32_t)tb0[mid] <= bid) lo = mid; else hi = mid;
        }
        bi = lo;
        w.tl = (int)bid - tb0[lo];
    } else {
        const int tiles = p.tilesM * p.tilesN;
        bi = bid / tiles;
        w.tl = bid - bi * tiles;
    }
    NodeDesc& d = w.d;
    if (MIXED || p.descs) {
        d = p.descs[bi];
    } else {
        d = p.base;
        d.A += (int64_t)bi * p.sA; d.w += (int64_t)bi * p.sw; d.B += (int64_t)bi * p.sB;
        d.out += (int64_t)bi * p.sO;
        if (d.arg) d.arg += (int64_t)bi * p.sO;
        if (d.rngA) d.rngA += (int64_t)bi * p.sR;
        if (d.rngW) d.rngW += (int64_t)bi * p.sR;
        if (d.rngB) d.rngB += (int64_t)bi * p.sR;
    }
}

// Origin of tile `tl` of a product with tilesM x tilesN tiles: tiles are walked in panels of 8 tile
// rows, column by column (see decode_work).
__device__ __forceinline__ void tile_origin(int tl, int tilesM, int tilesN, int& tmi, int& tni) {
    constexpr int PANEL = 8;
    const int panel = tl / (PANEL * tilesN);
    const int prow0 = panel * PANEL;
    const int prows = min(PANEL, tilesM - prow0);
    const int within = tl - panel * PANEL * tilesN;
    tni = within / prows;
    tmi = prow0 + (within - tni * prows);
}

// A call that knows nothing about its values and has measured nothing: the workgroup takes {min, max}
// of what ITS tile reads -- the TM rows of A, all of w, the TN columns of B -- and puts them where the
// caller's bounds would be.  Everything derived from ranges (overflow test, variant, key width, the
// clamp) then holds for this tile: its sums are sums of these elements, and the minimum of w is
// attained at some c of the product, where A and B are within the strips' ranges.  The pass reads
// what the main loop reads again right after (from L2); it replaces a launch of its own over all of
// A, w and B.  All parts of a shared tile scan the whole strips and so agree on every parameter.
// red: 24 words of LDS, free until the first stage is stored.
struct StripRanges { int loA, hiA, loW, hiW, loB, hiB; };
// (Not inlined: the scan runs once per workgroup before anything else, and inlined into the tile
// function it took registers from the main loop.)
template <int TM>
__device__ __noinline__ StripRanges measure_strips(const int32_t* A_, const int32_t* W_, const int32_t* B_, int Ci, int Cj,
                                                   int Ck, int a0, int b0, int* red) {
    constexpr int TN = TM;
    using gcptr = const int32_t __attribute__((address_space(1)))*;
    const gcptr A = (gcptr)(uintptr_t)A_;
    const gcptr W = (gcptr)(uintptr_t)W_;
    const gcptr B = (gcptr)(uintptr_t)B_;
    const int tid = threadIdx.x;
    int loA = 0x7fffffff, hiA = (int)0x80000000, loW = loA, hiW = hiA, loB = loA, hiB = hiA;
    auto take4 = [](const v4i x, int& lo, int& hi) {
        lo = min(min(lo, x.x), min(x.y, min(x.z, x.w)));
        hi = max(max(hi, x.x), max(x.y, max(x.z, x.w)));
    };
    {   // A: NT / TM threads per row (rows past the end repeat the last one)
        constexpr int TPRM = NT / TM;
        const gcptr Arow = A + (int64_t)min(a0 + tid / TPRM, Ci - 1) * Cj;
        const int seg = tid % TPRM;
        if (((Cj & 3) == 0) && ((((uintptr_t)A_) & 15) == 0)) {
#pragma unroll 8
            for (int c = seg * 4; c < Cj; c += TPRM * 4) take4(*(gv4cptr)(Arow + c), loA, hiA);
        } else {
#pragma unroll 8
            for (int c = seg; c < Cj; c += TPRM) { const int v = Arow[c]; loA = min(loA, v); hiA = max(hiA, v); }
        }
    }
#pragma unroll 4
    for (int c = tid; c < Cj; c += NT) { const int v = W[c]; loW = min(loW, v); hiW = max(hiW, v); }
    if (((Ck & 3) == 0) && ((((uintptr_t)B_) & 15) == 0) && (b0 + TN <= Ck)) {
        constexpr int TPB = TN / 4;               // threads per row of the strip
        const gcptr Bcol = B + b0 + (tid % TPB) * 4;
#pragma unroll 8
        for (int c = tid / TPB; c < Cj; c += NT / TPB) take4(*(gv4cptr)(Bcol + (int64_t)c * Ck), loB, hiB);
    } else {
        const gcptr Bcol = B + min(b0 + tid % TN, Ck - 1);          // columns past the end repeat the last one
#pragma unroll 8
        for (int c = tid / TN; c < Cj; c += NT / TN) { const int v = Bcol[(int64_t)c * Ck]; loB = min(loB, v); hiB = max(hiB, v); }
    }
    loA = wave_min_i32(loA); hiA = wave_max_i32(hiA); loW = wave_min_i32(loW); hiW = wave_max_i32(hiW);
    loB = wave_min_i32(loB); hiB = wave_max_i32(hiB);
    if ((tid & 63) == 0) {
        int* r = red + 6 * (tid >> 6);
        r[0] = loA; r[1] = hiA; r[2] = loW; r[3] = hiW; r[4] = loB; r[5] = hiB;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NT / 64; ++q) {
        loA = min(loA, red[6 * q]); hiA = max(hiA, red[6 * q + 1]); loW = min(loW, red[6 * q + 2]);
        hiW = max(hiW, red[6 * q + 3]); loB = min(loB, red[6 * q + 4]); hiB = max(hiB, red[6 * q + 5]);
    }
    __syncthreads();                              // red is part of the first stage's buffer
    return {loA, hiA, loW, hiW, loB, hiB};
}
template <int RB, bool MIXED>
__device__ __forceinline__ void measure_own_strips(const NodeArgs& p, TileWork& work, int* red) {
    constexpr int TM = 16 * RB, TN = 16 * RB;
    NodeDesc& d = work.d;
    const int Ci = MIXED ? d.Ci : p.Ci, Cj = MIXED ? d.Cj : p.Cj, Ck = MIXED ? d.Ck : p.Ck;
    const int tilesM = MIXED ? (Ci + TM - 1) / TM : p.tilesM, tilesN = MIXED ? (Ck + TN - 1) / TN : p.tilesN;
    int tmi, tni;
    tile_origin(work.tl, tilesM, tilesN, tmi, tni);
    const StripRanges r = measure_strips<TM>(d.A, d.w, d.B, Ci, Cj, Ck, tmi * TM, tni * TN, red);
    d.loA = r.loA; d.hiA = r.hiA; d.loW = r.loW; d.hiW = r.hiW; d.loB = r.loB; d.hiB = r.hiB;
    d.rngA = nullptr; d.rngW = nullptr; d.rngB = nullptr;
}

// One workgroup's tile (or part of a shared tile).  smA / smB: the double-buffered LDS stages
// (2 * TK * 16 RB words each), smRow: 16 RB words (row-rebased keys only), smMisc: 16 words.
template <int MODE, int RB, int TK, bool MIXED, bool VERIFY>
__device__ __forceinline__ void minplus_tile(const NodeArgs& p, const TileWork& work, uint32_t* smA, uint32_t* smB,
                                             int32_t* smRow, int* smMisc) {
    static_assert(!MIXED || RB == 4, "launches of mixed shapes use 64 x 64 tiles");
    static_assert(!(MIXED && VERIFY), "promised ranges come with strided addressing");
    constexpr bool ROW = (MODE == kModeKeyedRow);  // keys re-based per output row
    constexpr bool KEYED = (MODE == kModeKeyed) || ROW;
    static_assert(!ROW || RB == 4, "row-rebased keys use 64 x 64 tiles");
    constexpr bool VALUE = (MODE == kModeValue);   // minimum only: no argmin, no keys, any int32
    constexpr bool PIPE = RB == 4;   // LDS reads issued one step ahead of the arithmetic
    constexpr int TM = 16 * RB, TN = 16 * RB;   // output tile
    constexpr int EP = TM * TK / NT;            // elements of A and of B each thread stages per stage
    constexpr int QUADS = RB / 4;
    static_assert(EP % 4 == 0 && TK % EP == 0 && TN % EP == 0 && (TN / EP) * TK == NT, "staging assignment");
    uint32_t (*As)[TK][TM] = reinterpret_cast<uint32_t (*)[TK][TM]>(smA);   // [stage][c][a]  (A transposed)
    uint32_t (*Bs)[TK][TN] = reinterpret_cast<uint32_t (*)[TK][TN]>(smB);   // [stage][c][b]
    const NodeDesc& d = work.d;
    const int tl = work.tl, part = work.part, kparts = work.kparts;
    const uint32_t split_idx = work.split_idx;
    // A workgroup that starts while older ones are in their arithmetic loops would get issue slots
    // only when those stall, and its start-up -- a chain of dependent loads with some scalar
    // arithmetic between them -- would take many times longer than on an idle compute unit.  Its
    // wavefronts therefore run at raised priority until their first stage is in LDS, and again
    // while they store their results.
    // (Raised only after the descriptor has been read: ahead of that read the priority change keeps
    // the compiler from using scalar loads for it.)
    __builtin_amdgcn_s_setprio(3);
    const int Ci = MIXED ? d.Ci : p.Ci, Cj = MIXED ? d.Cj : p.Cj, Ck = MIXED ? d.Ck : p.Ck;
    const int tilesM = MIXED ? (Ci + TM - 1) / TM : p.tilesM, tilesN = MIXED ? (Ck + TN - 1) / TN : p.tilesN;
    int tmi, tni;
    tile_origin(tl, tilesM, tilesN, tmi, tni);
    const int a0 = tmi * TM, b0 = tni * TN;

    // Pointers read from a descriptor are generic to the compiler; say that they are global memory,
    // otherwise the prefetch loads are issued as flat loads, which also count as LDS traffic and
    // would be waited for by the first LDS read of the stage they are meant to overlap.
    using gcptr = const int32_t __attribute__((address_space(1)))*;
    using gptr = int32_t __attribute__((address_space(1)))*;
    const gcptr A = (gcptr)(uintptr_t)d.A;
    const gcptr W = (gcptr)(uintptr_t)d.w;
    const gcptr B = (gcptr)(uintptr_t)d.B;
    const gptr O = (gptr)(uintptr_t)d.out;
    const gptr G = (gptr)(uintptr_t)d.arg;

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    // global -> LDS assignment: A: one row, EP consecutive c;  B: one c, EP consecutive columns
    constexpr int TPR = TK / EP;                 // threads per A row
    const int lr = tid / TPR, lseg = (tid % TPR) * EP;
    constexpr int TPB = TN / EP;                 // threads per B row
    const int br = tid / TPB, bseg = (tid % TPB) * EP;
    const int arow = min(a0 + lr, Ci - 1);       // clamped: rows past the end are never stored
    const bool vecA = ((Cj & 3) == 0) && ((((uintptr_t)A) | ((uintptr_t)W)) & 15) == 0;
    const bool vecB = ((Ck & 3) == 0) && ((((uintptr_t)B) & 15) == 0) && (b0 + TN <= Ck);
    const gcptr Arow = A + (int64_t)arow * Cj;

    // Per-thread source pointers of the staging loads; they advance by one stage per fetch.
    gcptr pA = Arow + lseg, pW = W + lseg;
    gcptr pB = B + (int64_t)br * Ck + b0 + bseg;
    int32_t ra[EP], rw[EP], rb[EP];
    auto fetch = [&](int c0) {
        if (vecA && c0 + TK <= Cj) {
#pragma unroll
            for (int v = 0; v < EP / 4; ++v) {
                const v4i x = ((gv4cptr)pA)[v];
                const v4i y = ((gv4cptr)pW)[v];
                ra[4 * v] = x.x; ra[4 * v + 1] = x.y; ra[4 * v + 2] = x.z; ra[4 * v + 3] = x.w;
                rw[4 * v] = y.x; rw[4 * v + 1] = y.y; rw[4 * v + 2] = y.z; rw[4 * v + 3] = y.w;
            }
        } else {
#pragma unroll
            for (int q = 0; q < EP; ++q) {
                const int c = min(c0 + lseg + q, Cj - 1);
                ra[q] = Arow[c]; rw[q] = W[c];
            }
        }
        if (vecB && c0 + TK <= Cj) {
#pragma unroll
            for (int v = 0; v < EP / 4; ++v) {
                const v4i y = ((gv4cptr)pB)[v];
                rb[4 * v] = y.x; rb[4 * v + 1] = y.y; rb[4 * v + 2] = y.z; rb[4 * v + 3] = y.w;
            }
        } else {
            const int c = min(c0 + br, Cj - 1);
            const gcptr Brow = B + (int64_t)c * Ck;
            // opaque per stage: otherwise the clamped column offsets are hoisted out of the stage loop
            // and sit in sixteen registers that the common (vector) path never uses
            int col0 = b0 + bseg;
            asm volatile("" : "+v"(col0));
#pragma unroll
            for (int q = 0; q < EP; ++q) rb[q] = Brow[min(col0 + q, Ck - 1)];
        }
        pA += TK; pW += TK; pB += (int64_t)TK * Ck;
    };
    // part q of a split tile walks stages [q*n_g, (q+1)*n_g); stages past the end of c see only
    // padding (never a winner)
    const int nstages = (Cj + TK - 1) / TK;
    const int n_g = (nstages + kparts - 1) / kparts;
    const int s_first = part * n_g;
    if (kparts > 1) { pA += (int64_t)s_first * TK; pW += (int64_t)s_first * TK; pB += (int64_t)s_first * TK * Ck; }
    // The first stage's loads need only the descriptor's pointers: they are issued before the value
    // ranges are read, so that the two memory round trips overlap.
    fetch(s_first * TK);

    // ---- value ranges of the operands: the caller's bounds, tightened by the measured ranges (read
    //      once: every read is a round trip to memory on the critical path of a small launch) ----
    long long loA = d.loA, hiA = d.hiA, loB = d.loB, hiB = d.hiB, loW = d.loW, hiW = d.hiW;
    if (d.rngA) { const gcptr r = (gcptr)(uintptr_t)d.rngA; loA = max(loA, (long long)r[0]); hiA = min(hiA, (long long)r[1]); }
    if (d.rngB) { const gcptr r = (gcptr)(uintptr_t)d.rngB; loB = max(loB, (long long)r[0]); hiB = min(hiB, (long long)r[1]); }
    if (d.rngW) { const gcptr r = (gcptr)(uintptr_t)d.rngW; loW = max(loW, (long long)r[0]); hiW = min(hiW, (long long)r[1]); }
    // the sums must fit int32
    if (d.flag) {
        const long long hi = hiA + hiW + hiB, lo = loA + loW + loB;
        const long long hi2 = hiA + hiW, lo2 = loA + loW;
        if ((hi > 2147483647ll || lo < -2147483648ll || hi2 > 2147483647ll || lo2 < -2147483648ll) && threadIdx.x == 0)
            atomicOr(d.flag, 1);
    }

    // ---- row-rebased keys: minimum of A + w over this workgroup's c range, per tile row ----
    int32_t* rmin = smRow;
    if (ROW) {
        int32_t mn = 0x7fffffff;
        const int c_end = min(Cj, (s_first + n_g) * TK);
        for (int c0 = s_first * TK; c0 < c_end; c0 += TK) {
            if (vecA && c0 + TK <= Cj) {
#pragma unroll
                for (int v = 0; v < EP / 4; ++v) {
                    const v4i x = ((gv4cptr)(Arow + c0 + lseg))[v];
                    const v4i y = ((gv4cptr)(W + c0 + lseg))[v];
                    mn = min(min(mn, x.x + y.x), min(x.y + y.y, min(x.z + y.z, x.w + y.w)));
                }
            } else {
#pragma unroll
                for (int q = 0; q < EP; ++q) {
                    const int c = c0 + lseg + q;
                    if (c < Cj) mn = min(mn, Arow[c] + W[c]);
                }
            }
        }
#pragma unroll
        for (int o = TPR / 2; o > 0; o >>= 1) mn = min(mn, __shfl_xor(mn, o));   // the TPR threads of a row are adjacent lanes
        if ((tid % TPR) == 0) rmin[lr] = mn;
        __syncthreads();
    }

    // ---- key parameters from value ranges (uniform, scalar) ----
    int32_t offA = 0, offB = 0;
    int tb = 0;
    uint32_t cap = 0xffffffffu;
    if (KEYED) {
        offA = (int32_t)(loA + loW);
        offB = (int32_t)loB;
        const long long a_max = hiA + hiW - (loA + loW);          // largest re-based A + w
        const long long out_max = (hiA - loA) + (hiB - loB);      // largest re-based result
        // per row: the row's minimum re-bases to 0 and pairs with a B of at most the spread of B, so
        // anything more than that spread above the row's minimum loses
        // (promised ranges need not be attained, so the bound on the result does not hold for them)
        const long long capl = ROW ? (hiB - loB) + 1 : (VERIFY ? a_max : min(a_max, out_max + 1));
        const long long spread = capl + (hiB - loB);
        cap = (uint32_t)capl;
        constexpr int TB_MIN = (TK <= 16) ? 5 : 6;               // a chunk holds at least one stage
        // A launch made on the assumption that packed keys will do: where a product's ranges do not
        // allow them, say so and leave the product alone (the caller then runs it another way).
        // Nothing has been stored and no barrier passed yet; uniform for the workgroup.
        if (!ROW && !VERIFY && p.speculative && spread > (1ll << (32 - TB_MIN)) - 2) {
            if (d.flag && threadIdx.x == 0) atomicOr(d.flag, 4);
            return;
        }
        tb = TB_MIN;
        for (int t = 17; t > TB_MIN; --t)
            if (spread <= (1ll << (32 - t)) - 2) { tb = t; break; }
        for (int t = TB_MIN; t < tb; ++t)
            if (((1 << t) - 1) / TK * TK >= Cj) { tb = t; break; }   // one chunk already covers all c
    }
    const uint32_t fmask = KEYED ? ((1u << tb) - 1u) : 0u;
    const uint32_t padA = KEYED ? ~fmask : 0x7fffffffu;   // never strictly below any running minimum
    const int spc = KEYED ? (int)(fmask / TK) : 1;        // stages per chunk: TK*spc <= 2^tb - 1

    // Keys: A side ((A + w - offA, clamped) << tb) - (offB << tb), B side (B << tb) + low field.
    // The re-basing of B rides on the A side (arithmetic is modulo 2^32 and the true sum is in
    // range); the low field, 1 + position of c inside its chunk, rides on the B side, where all
    // elements a thread stages share one c.  That makes three operations per A element (a
    // three-operand add, the clamp, shift-and-add) and one per B element (shift-and-add).
    uint32_t nboff = KEYED ? 0u - ((uint32_t)offB << tb) : 0u;
    uint32_t noffA = 0u - (uint32_t)(ROW ? rmin[lr] : offA);
    // opaque to the optimiser, which would otherwise rewrite the two fused forms below
    // (add3; shift-and-add) into subtract, add, subtract, shift
    if (ROW) {
        asm volatile("" : "+v"(nboff), "+v"(noffA));
    } else {
        noffA = __builtin_amdgcn_readfirstlane(noffA);  // uniform: a scalar register
        asm volatile("" : "+v"(nboff), "+s"(noffA));
    }
    // Promised ranges (VERIFY): every element of A and B is checked when it is staged -- the A strip
    // by the workgroups of the first tile column, the B strip by those of the first tile row, so
    // every element is checked once per pass over it and most workgroups check nothing.
    const bool chkA = VERIFY && tni == 0, chkB = VERIFY && tmi == 0;
    int32_t vloA = 0x7fffffff, vhiA = (int32_t)0x80000000, vloB = 0x7fffffff, vhiB = (int32_t)0x80000000;
    auto stash = [&](int c0, int pos0, int buf) {
        const uint32_t pos = (uint32_t)(pos0 + br + 1);
        uint32_t ka[EP], kb[EP];
        if (VERIFY) {       // the loads are clamped to valid elements, so everything seen here is data
            if (chkA) {
#pragma unroll
                for (int q = 0; q < EP; q += 2) { vloA = min(min(vloA, ra[q]), ra[q + 1]); vhiA = max(max(vhiA, ra[q]), ra[q + 1]); }
            }
            if (chkB) {
#pragma unroll
                for (int q = 0; q < EP; q += 2) { vloB = min(min(vloB, rb[q]), rb[q + 1]); vhiB = max(max(vhiB, rb[q]), rb[q + 1]); }
            }
        }
#pragma unroll
        for (int q = 0; q < EP; ++q) {
            if (KEYED) {
                ka[q] = (min((uint32_t)ra[q] + (uint32_t)rw[q] + noffA, cap) << tb) + nboff;
                kb[q] = ((uint32_t)rb[q] << tb) + pos;
            } else { ka[q] = (uint32_t)(ra[q] + rw[q]); kb[q] = (uint32_t)rb[q]; }
        }
        // value-only mode needs no padding: the clamped loads repeat the last candidate
        if (!VALUE && c0 + TK > Cj) {             // only the last stage can be ragged
            const bool cok = (c0 + br) < Cj;
#pragma unroll
            for (int q = 0; q < EP; ++q) {
                if ((c0 + lseg + q) >= Cj) ka[q] = padA;
                if (!cok) kb[q] = 0u;
            }
        }
#pragma unroll
        for (int q = 0; q < EP; ++q) As[buf][lseg + q][lr] = ka[q];
#pragma unroll
        for (int v = 0; v < EP / 4; ++v)
            *reinterpret_cast<uint4*>(&Bs[buf][br][bseg + 4 * v]) = make_uint4(kb[4 * v], kb[4 * v + 1], kb[4 * v + 2], kb[4 * v + 3]);
    };

    // running state of the RB x RB block
    uint32_t m1[RB][RB];   // keyed: running key minimum;  plain: running int32 minimum (as bits)
    uint32_t rec[RB][RB];  // keyed: c of the last change;  plain: running argmin
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int j = 0; j < RB; ++j) { m1[i][j] = padA; rec[i][j] = 0u; }

    int sic = 0;                      // stage index inside the current chunk
    int chunk_c0 = s_first * TK;      // first c of the current chunk
    stash(s_first * TK, 0, 0);
    __syncthreads();
    __builtin_amdgcn_s_setprio(0);

    for (int it = 0; it < n_g; ++it) {
        const int s = s_first + it;
        const int buf = it & 1;
        const bool more = (it + 1) < n_g;
        const bool chunk_end = (sic + 1 == spc);
        if (more) fetch((s + 1) * TK);

        // Operands of two candidates (cc, cc+1) per step.  With PIPE the reads of the next step are
        // issued before the arithmetic of the current one, so one wavefront alone hides the LDS
        // latency (launches too small to fill every SIMD with several wavefronts).
        uint32_t avp[PIPE ? 2 : 1][2][RB], bvp[PIPE ? 2 : 1][2][RB];
        auto lds_read = [&](int cc, uint32_t (&av)[2][RB], uint32_t (&bv)[2][RB]) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int h = 0; h < QUADS; ++h) {
                    const uint4 a4 = *reinterpret_cast<const uint4*>(&As[buf][cc + u][h * 64 + ty * 4]);
                    const uint4 b4 = *reinterpret_cast<const uint4*>(&Bs[buf][cc + u][h * 64 + tx * 4]);
                    av[u][4 * h] = a4.x; av[u][4 * h + 1] = a4.y; av[u][4 * h + 2] = a4.z; av[u][4 * h + 3] = a4.w;
                    bv[u][4 * h] = b4.x; bv[u][4 * h + 1] = b4.y; bv[u][4 * h + 2] = b4.z; bv[u][4 * h + 3] = b4.w;
                }
        };
        if (PIPE) lds_read(0, avp[0], bvp[0]);
#pragma unroll
        for (int cc = 0; cc < TK; cc += 2) {
            const int pb = PIPE ? ((cc >> 1) & 1) : 0;
            if (PIPE) {
                if (cc + 2 < TK) lds_read(cc + 2, avp[pb ^ 1], bvp[pb ^ 1]);
                __builtin_amdgcn_sched_barrier(0);      // the reads go out before this step's arithmetic
            } else lds_read(cc, avp[0], bvp[0]);
            uint32_t (&av)[2][RB] = avp[pb];
            uint32_t (&bv)[2][RB] = bvp[pb];
            if (KEYED) {
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int j = 0; j < RB; ++j)
                        m1[i][j] = min(min(m1[i][j], av[0][i] + bv[0][j]), av[1][i] + bv[1][j]);
            } else if (VALUE) {
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int j = 0; j < RB; ++j)
                        m1[i][j] = (uint32_t)min(min((int32_t)m1[i][j], (int32_t)(av[0][i] + bv[0][j])), (int32_t)(av[1][i] + bv[1][j]));
            } else {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const uint32_t c = (uint32_t)(s * TK + cc + u);
#pragma unroll
                    for (int i = 0; i < RB; ++i)
#pragma unroll
                        for (int j = 0; j < RB; ++j) {
                            const int32_t cand = (int32_t)(av[u][i] + bv[u][j]);
                            const bool lt = cand < (int32_t)m1[i][j];
                            m1[i][j] = lt ? (uint32_t)cand : m1[i][j];
                            rec[i][j] = lt ? c : rec[i][j];
                        }
                }
            }
            // keep the LDS reads of later iterations behind this iteration's arithmetic (otherwise a
            // whole stage of operands is loaded first and the register file overflows): the plain
            // variant's selects get sunk below the reads unless their results are pinned here
            if (MODE == kModePlain) {
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int j = 0; j < RB; j += 4)
                        asm volatile("" : "+v"(m1[i][j]), "+v"(m1[i][j + 1]), "+v"(m1[i][j + 2]), "+v"(m1[i][j + 3]),
                                          "+v"(rec[i][j]), "+v"(rec[i][j + 1]), "+v"(rec[i][j + 2]), "+v"(rec[i][j + 3]));
            } else if (VALUE) {
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int j = 0; j < RB; j += 4)
                        asm volatile("" : "+v"(m1[i][j]), "+v"(m1[i][j + 1]), "+v"(m1[i][j + 2]), "+v"(m1[i][j + 3]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        if (KEYED && (chunk_end || !more)) {
            // chunk end: a non-zero low field means the minimum changed inside this chunk
            const uint32_t base = (uint32_t)chunk_c0 - 1u;
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int j = 0; j < RB; ++j) {
                    const uint32_t f = m1[i][j] & fmask;
                    rec[i][j] = f ? (base + f) : rec[i][j];
                    m1[i][j] &= ~fmask;
                }
        }
        if (chunk_end) { sic = 0; chunk_c0 = (s + 1) * TK; } else { ++sic; }

        if (more) stash((s + 1) * TK, sic * TK, buf ^ 1);
        __syncthreads();
    }

    if (VERIFY) {
        bool bad = (chkA && (vloA < d.loA || vhiA > d.hiA)) || (chkB && (vloB < d.loB || vhiB > d.hiB));
        if (chkA && chkB && part == 0)      // one workgroup per product checks w
            for (int c = tid; c < Cj; c += NT) { const int32_t x = W[c]; bad |= (x < d.loW || x > d.hiW); }
        if (bad && d.flag) atomicOr(d.flag, 2);
    }

    // Split tile: every part publishes its (cost, argmin) block to global scratch; the part that
    // arrives last (a counter per tile) folds all parts in ascending-c order -- strict '<' lets the
    // earlier part keep ties -- and goes on to the epilogue.  The parts run on different compute
    // units, possibly different XCDs (separate L2s): the blocks are exchanged with device-scope
    // relaxed atomic stores and loads, which go through to memory, so no cache-wide write-back or
    // invalidate is needed; every wavefront waits for its stores to complete before the barrier
    // that precedes the bump of the counter.
    __builtin_amdgcn_s_setprio(3);
    bool raw = KEYED;                          // m1 still holds keys (otherwise plain costs)
    if (RB == 4 && kparts > 1) {
        constexpr int CELLS = RB * RB;
        int32_t* slab = p.scratch + ((int64_t)split_idx * kparts) * (2 * CELLS * NT);
        int32_t* mine = slab + (int64_t)part * (2 * CELLS * NT);
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                // a part whose stages all lie beyond Cj still holds the padding key: its cost field plus
                // the offsets may pass INT32_MAX, so the sum is formed in 64 bits and saturated (real
                // costs never exceed INT32_MAX, and such a part is the last, so it cannot win a tie)
                const long long base = ROW ? (long long)rmin[ty * 4 + (i & 3)] + offB : (long long)offA + offB;
                const int32_t cst = KEYED ? (int32_t)min((long long)(m1[i][j] >> tb) + base, 2147483647ll) : (int32_t)m1[i][j];
                __hip_atomic_store(&mine[(i * RB + j) * NT + tid], cst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (!VALUE) __hip_atomic_store(&mine[(CELLS + i * RB + j) * NT + tid], (int32_t)rec[i][j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        // Every wavefront waits until its own stores have completed -- they are write-through to
        // device scope, so completed means visible to every compute unit -- before the barrier
        // after which the arrival is counted.  (A workgroup-scope release is not enough: it
        // orders the stores for this compute unit only and need not wait for them.)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        int& arrived = smMisc[0];
        if (tid == 0) arrived = __hip_atomic_fetch_add(&p.counters[split_idx], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (arrived != kparts - 1) return;     // uniform for the workgroup
        if (tid == 0) __hip_atomic_store(&p.counters[split_idx], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
        // two parts at a time, all of their values in flight together (one round trip to the
        // memory side per pair); folded in ascending part order
        for (int q = 0; q < kparts; q += 2) {
            const int q1 = min(q + 1, kparts - 1);      // odd part count: the last part is read twice
            const int32_t* other0 = slab + (int64_t)q * (2 * CELLS * NT);
            const int32_t* other1 = slab + (int64_t)q1 * (2 * CELLS * NT);
            int32_t c2[2][RB][RB], r2[2][RB][RB];
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int j = 0; j < RB; ++j) {
                    c2[0][i][j] = __hip_atomic_load(&other0[(i * RB + j) * NT + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    c2[1][i][j] = __hip_atomic_load(&other1[(i * RB + j) * NT + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    r2[0][i][j] = VALUE ? 0 : __hip_atomic_load(&other0[(CELLS + i * RB + j) * NT + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    r2[1][i][j] = VALUE ? 0 : __hip_atomic_load(&other1[(CELLS + i * RB + j) * NT + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int j = 0; j < RB; ++j) {
                        // strict '<': a repeated part changes nothing
                        const bool take = (q + u == 0) || (c2[u][i][j] < (int32_t)m1[i][j]);
                        m1[i][j] = take ? (uint32_t)c2[u][i][j] : m1[i][j];
                        rec[i][j] = take ? (uint32_t)r2[u][i][j] : rec[i][j];
                    }
        }
        raw = false;
    }

    // epilogue: thread rows {h*64 + ty*4 + 0..3}, columns {h*64 + tx*4 + 0..3}, h < QUADS
    const bool vecO = ((Ck & 3) == 0) && ((((uintptr_t)O) | ((uintptr_t)G)) & 15) == 0 && (b0 + TN <= Ck);
    int vmin = 0x7fffffff, vmax = (int)0x80000000;
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        const int a = a0 + (i >> 2) * 64 + ty * 4 + (i & 3);
        if (a >= Ci) continue;
        int32_t val[RB];
#pragma unroll
        for (int j = 0; j < RB; ++j)
            val[j] = raw ? (int32_t)(m1[i][j] >> tb) + (ROW ? rmin[ty * 4 + (i & 3)] : offA) + offB : (int32_t)m1[i][j];
#pragma unroll
        for (int h = 0; h < QUADS; ++h) {
            const int b = b0 + h * 64 + tx * 4;
            const gptr orow = O + (int64_t)a * Ck + b;
            if (vecO) {
                *(gv4ptr)(orow) = v4i{val[h * 4], val[h * 4 + 1], val[h * 4 + 2], val[h * 4 + 3]};
                if (!VALUE && G) *(gv4ptr)(G + (int64_t)a * Ck + b) =
                    v4i{(int32_t)rec[i][h * 4], (int32_t)rec[i][h * 4 + 1], (int32_t)rec[i][h * 4 + 2], (int32_t)rec[i][h * 4 + 3]};
#pragma unroll
                for (int q = 0; q < 4; ++q) { vmin = min(vmin, val[h * 4 + q]); vmax = max(vmax, val[h * 4 + q]); }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (b + q < Ck) {
                        orow[q] = val[h * 4 + q];
                        if (!VALUE && G) G[(int64_t)a * Ck + b + q] = (int32_t)rec[i][h * 4 + q];
                        vmin = min(vmin, val[h * 4 + q]); vmax = max(vmax, val[h * 4 + q]);
                    }
            }
        }
    }
    // one workgroup per tile gets here (of a shared tile: the one that merged the parts); count the
    // product once, off the start-up path
    if (p.mode_count && tl == 0 && tid == 0) atomicAdd(&p.mode_count[MODE], 1);
    if (d.rngOut) {   // leave the measured range of this table for the launches that consume it
        vmin = wave_min_i32(vmin); vmax = wave_max_i32(vmax);
        int* red = smMisc + 1;
        if ((tid & 63) == 0) { red[2 * (tid >> 6)] = vmin; red[2 * (tid >> 6) + 1] = vmax; }
        __syncthreads();
        if (tid == 0) {
            for (int q = 1; q < NT / 64; ++q) { vmin = min(vmin, red[2 * q]); vmax = max(vmax, red[2 * q + 1]); }
            if (vmin <= vmax) { atomicMin(&d.rngOut[0], vmin); atomicMax(&d.rngOut[1], vmax); }
        }
    }
}

template <int MODE, int RB, int TK, bool MIXED = false, bool VERIFY = false, bool SELF = false>
__global__ __launch_bounds__(NT, RB == 4 ? 4 : (MODE == kModePlain ? 1 : 2)) void minplus_kernel(const NodeArgs p) {
    __shared__ __attribute__((aligned(16))) uint32_t smA[2 * TK * 16 * RB];
    __shared__ __attribute__((aligned(16))) uint32_t smB[2 * TK * 16 * RB];
    __shared__ int32_t smRow[MODE == kModeKeyedRow ? 16 * RB : 1];
    __shared__ int smMisc[16];
    TileWork work;
    decode_work<RB, MIXED>(p, work);
    if (SELF) measure_own_strips<RB, MIXED>(p, work, reinterpret_cast<int*>(smA));
    minplus_tile<MODE, RB, TK, MIXED, VERIFY>(p, work, smA, smB, smRow, smMisc);
}

// The variant is picked here, per product, from the measured ranges of its operands: the host
// then needs to know nothing about the tables' values and no value has to travel back to it.
// auto_limit: largest spread packed keys on global offsets may have at this tile size; auto_row:
// keys re-based per row are a candidate (64 x 64 tiles, launches large enough for their extra pass).
template <int RB, int TK, bool MIXED = false, bool SELF = false>
__global__ __launch_bounds__(NT, RB == 4 ? 4 : 2) void minplus_auto_kernel(const NodeArgs p) {
    __shared__ __attribute__((aligned(16))) uint32_t smA[2 * TK * 16 * RB];
    __shared__ __attribute__((aligned(16))) uint32_t smB[2 * TK * 16 * RB];
    __shared__ int32_t smRow[RB == 4 ? 16 * RB : 1];
    __shared__ int smMisc[16];
    TileWork work;
    decode_work<RB, MIXED>(p, work);
    if (SELF) measure_own_strips<RB, MIXED>(p, work, reinterpret_cast<int*>(smA));   // (a kernel of its own: the others stay as they are)
    using gcptr = const int32_t __attribute__((address_space(1)))*;
    const NodeDesc& d = work.d;
    long long loA = d.loA, hiA = d.hiA, loB = d.loB, hiB = d.hiB, loW = d.loW, hiW = d.hiW;
    if (d.rngA) { const gcptr r = (gcptr)(uintptr_t)d.rngA; loA = max(loA, (long long)r[0]); hiA = min(hiA, (long long)r[1]); }
    if (d.rngB) { const gcptr r = (gcptr)(uintptr_t)d.rngB; loB = max(loB, (long long)r[0]); hiB = min(hiB, (long long)r[1]); }
    if (d.rngW) { const gcptr r = (gcptr)(uintptr_t)d.rngW; loW = max(loW, (long long)r[0]); hiW = min(hiW, (long long)r[1]); }
    int want = auto_variant(loA, hiA, loW, hiW, loB, hiB, p.auto_limit, RB == 4 && p.auto_row != 0);
    want = __builtin_amdgcn_readfirstlane(want);         // the same for the whole workgroup: a scalar branch
    if (want == kModeKeyed) minplus_tile<kModeKeyed, RB, TK, MIXED, false>(p, work, smA, smB, smRow, smMisc);
    else if (RB == 4 && want == kModeKeyedRow) minplus_tile<kModeKeyedRow, 4, 32, MIXED, false>(p, work, smA, smB, smRow, smMisc);
    else minplus_tile<kModePlain, RB, TK, MIXED, false>(p, work, smA, smB, smRow, smMisc);
}

}  // namespace

hipError_t launch_minplus(const NodeArgs& args, int mode, bool small_tiles, hipStream_t stream, bool verify) {
    const int kparts = args.kparts > 1 ? args.kparts : 1;
    const bool mixed = args.tile_begin != nullptr;
    const int64_t tiles = mixed ? (int64_t)args.total_tiles : (int64_t)args.tilesM * args.tilesN * args.batch;
    const int64_t n_whole = kparts > 1 ? (int64_t)args.n_whole : tiles;
    if (tiles <= 0 || args.batch < 1 || n_whole < 0 || n_whole > tiles) return hipErrorInvalidValue;
    const int64_t n_shared = tiles - n_whole;
    const int64_t blocks = n_whole + n_shared * kparts;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (kparts > 1 && (!small_tiles || !args.scratch || !args.counters)) return hipErrorInvalidValue;
    if (kparts > 1 && (kparts > kSplitMaxParts || n_shared > kSplitMaxTiles || n_shared * kparts > kSplitMaxWorkgroups))
        return hipErrorInvalidValue;   // beyond the capacity of the split-tile buffers
    if (mixed && (!small_tiles || !args.descs)) return hipErrorInvalidValue;
    if (mode == kModeKeyedRow && !small_tiles) return hipErrorInvalidValue;
    if (verify && (mixed || args.descs || mode == kModeAuto || args.base.rngA || args.base.rngW || args.base.rngB)) return hipErrorInvalidValue;
    // tile-local measurement: the kernel that picks the variant, or the value-only kernel
    if (args.self_measure && (verify || mixed || (mode != kModeAuto && mode != kModeValue))) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(NT);
#define LWP_LAUNCH(MODE, RB, TK, MIXED, VERIFY) \
    hipLaunchKernelGGL((minplus_kernel<MODE, RB, TK, MIXED, VERIFY>), grid, block, 0, stream, args)
    if (mode == kModeValue && args.self_measure) {
        if (small_tiles) hipLaunchKernelGGL((minplus_kernel<kModeValue, 4, 32, false, false, true>), grid, block, 0, stream, args);
        else hipLaunchKernelGGL((minplus_kernel<kModeValue, 8, 16, false, false, true>), grid, block, 0, stream, args);
    } else if (mode == kModeAuto && args.self_measure) {
        if (small_tiles) hipLaunchKernelGGL((minplus_auto_kernel<4, 32, false, true>), grid, block, 0, stream, args);
        else hipLaunchKernelGGL((minplus_auto_kernel<8, 16, false, true>), grid, block, 0, stream, args);
    } else if (mode == kModeAuto) {
        if (mixed) hipLaunchKernelGGL((minplus_auto_kernel<4, 32, true>), grid, block, 0, stream, args);
        else if (small_tiles) hipLaunchKernelGGL((minplus_auto_kernel<4, 32, false>), grid, block, 0, stream, args);
        else hipLaunchKernelGGL((minplus_auto_kernel<8, 16, false>), grid, block, 0, stream, args);
    } else if (mixed) {
        if (mode == kModeKeyed) LWP_LAUNCH(kModeKeyed, 4, 32, true, false);
        else if (mode == kModeKeyedRow) LWP_LAUNCH(kModeKeyedRow, 4, 32, true, false);
        else if (mode == kModeValue) LWP_LAUNCH(kModeValue, 4, 32, true, false);
        else LWP_LAUNCH(kModePlain, 4, 32, true, false);
    } else if (verify) {
        if (small_tiles) {
            if (mode == kModeKeyed) LWP_LAUNCH(kModeKeyed, 4, 32, false, true);
            else if (mode == kModeKeyedRow) LWP_LAUNCH(kModeKeyedRow, 4, 32, false, true);
            else if (mode == kModeValue) LWP_LAUNCH(kModeValue, 4, 32, false, true);
            else LWP_LAUNCH(kModePlain, 4, 32, false, true);
        } else {
            if (mode == kModeKeyed) LWP_LAUNCH(kModeKeyed, 8, 16, false, true);
            else if (mode == kModeValue) LWP_LAUNCH(kModeValue, 8, 16, false, true);
            else LWP_LAUNCH(kModePlain, 8, 16, false, true);
        }
    } else if (small_tiles) {
        if (mode == kModeKeyed) LWP_LAUNCH(kModeKeyed, 4, 32, false, false);
        else if (mode == kModeKeyedRow) LWP_LAUNCH(kModeKeyedRow, 4, 32, false, false);
        else if (mode == kModeValue) LWP_LAUNCH(kModeValue, 4, 32, false, false);
        else LWP_LAUNCH(kModePlain, 4, 32, false, false);
    } else {
        if (mode == kModeKeyed) LWP_LAUNCH(kModeKeyed, 8, 16, false, false);
        else if (mode == kModeValue) LWP_LAUNCH(kModeValue, 8, 16, false, false);
        else LWP_LAUNCH(kModePlain, 8, 16, false, false);
    }
#undef LWP_LAUNCH
    return hipGetLastError();
}

}  // namespace lwp
