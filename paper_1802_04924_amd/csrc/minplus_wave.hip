// Node elimination (Sec. 5.2, Eq. 2) for launches too small for the tiled kernel:
//   out[a][b] = min_c ( A[a][c] + w[c] + B[c][b] ),  arg[a][b] = lowest c attaining the minimum.
//
// The tiled kernel needs thousands of 64 x 64 tiles to fill the chip; a launch with a handful of
// products of a few hundred configurations has a few dozen, and sharing a tile among workgroups
// costs a publication through memory, a counter and a merge -- a chain of round trips that takes
// longer than the arithmetic.  Here one WAVEFRONT owns an 8 x 8 (RB = 1) or 16 x 16 (RB = 2) output
// tile and walks all of c by itself: a product of 256 x 256 configurations makes 1024 independent
// wavefronts, one per SIMD of the chip, with no barrier, no counter and no merge anywhere.  The
// wavefront stages chunks of KC candidates in its own slice of LDS (A + w row-major, B as loaded);
// the loads of the next chunk are in flight while it works on the current one.  Arithmetic is the
// plain variant's: int32 compare/select in ascending c with a strict '<' (lowest index among equal
// candidates), or the minimum alone (three-way min) for callers that recompute the argmin.
// Loads are clamped to the last row / column / candidate, so a ragged chunk repeats its last
// candidate: a repeated candidate is never strictly smaller than the minimum it already entered.
#include <cstddef>

#include "lwp_kernels.h"

namespace lwp {

namespace {

constexpr int kWaveGroup = 256;            // threads per workgroup: 4 independent wavefronts
constexpr int kWaveLongChunkTiles = 4096;  // launches of at most this many 8 x 8 tiles stage 128 candidates at a time
constexpr int kWavesPerGroup = kWaveGroup / 64;

using gcptr = const int32_t __attribute__((address_space(1)))*;
using gptr = int32_t __attribute__((address_space(1)))*;

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

// The first descriptors of a launch travel in the kernel arguments: a launch of a few products then
// starts without the round trip to memory that reading its descriptor would cost every wavefront.
struct WaveArgs {
    NodeArgs a;
    int32_t n_inline;
    int32_t verify;       // the descriptors' ranges are promises to be checked
    NodeDesc inl[kWaveInlineDescs];
};

// SPLIT: the four wavefronts of a workgroup share ONE tile, each with a quarter of the candidates, and
// merge through LDS (for launches so small that a tile per wavefront would leave three SIMDs in four
// idle: a wavefront issues one instruction per four cycles however idle the rest of the chip is).
template <int RB, int KC, bool VALUE, bool SPLIT>
__global__ __launch_bounds__(kWaveGroup, 4) void minplus_wave_kernel(const WaveArgs wa) {
    const NodeArgs& p = wa.a;
    constexpr int TS = 8 * RB;             // output tile of one wavefront: TS x TS
    // KC: candidates per chunk.  128 with 8 x 8 tiles when every wavefront of the launch has a SIMD to
    // itself or nearly (fewer, longer chunks: nobody else hides the latency of its loads); 64 otherwise
    // (half the LDS and half the registers in flight, so that 7 instead of 4 wavefronts fit a SIMD and a
    // launch of up to 7168 wavefronts is resident at once instead of running in two generations).
    constexpr int AST = KC + 4;            // row stride of the A stage: 16-byte rows, banks staggered by 4
    constexpr int NL = TS * KC / 64;       // loads per lane and chunk, for A and for B
    constexpr int NLW = KC / 64;
    constexpr int RPL = 64 / TS;           // rows of B one load instruction covers
    static_assert(NL % 2 == 0 && KC % 64 == 0 && KC % 16 == 0 && 64 % TS == 0, "staging assignment");
    __shared__ __attribute__((aligned(16))) int32_t lds[kWavesPerGroup][TS * AST + KC * TS];

    constexpr int CELLS = RB * RB;         // output cells per lane
    // Where the wavefronts that share a tile leave their results for the merge: each in its own
    // stage, which it has finished with by then (a separate array would cost a 16 x 16 launch one
    // resident workgroup in four).
    static_assert(2 * 64 * CELLS + 8 <= TS * AST + KC * TS, "a wavefront's results fit its stage");
    int32_t (*merge)[TS * AST + KC * TS] = lds;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const int item = SPLIT ? (int)blockIdx.x : (int)blockIdx.x * kWavesPerGroup + wave;
    if (!SPLIT && item >= p.total_tiles) return;     // whole wavefronts leave; without SPLIT the kernel has no barrier

    // ---- which product, which tile (uniform) ----
    int bi, tl;
    if (p.tile_begin) {
        const gcptr tb0 = (gcptr)(uintptr_t)p.tile_begin;
        int lo = 0, hi = p.batch;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (tb0[mid] <= item) lo = mid; else hi = mid;
        }
        bi = lo;
        tl = item - tb0[lo];
    } else {
        const int tiles = p.tilesM * p.tilesN;
        bi = item / tiles;
        tl = item - bi * tiles;
    }
    bi = __builtin_amdgcn_readfirstlane(bi);
    tl = __builtin_amdgcn_readfirstlane(tl);
    NodeDesc d;
    if (bi < wa.n_inline) {
        // indexed straight in the kernel-argument segment (constant memory, a scalar load)
        using kaptr = const char __attribute__((address_space(4)))*;
        using kwptr = const uint32_t __attribute__((address_space(4)))*;
        const kwptr src = (kwptr)((kaptr)__builtin_amdgcn_kernarg_segment_ptr() + offsetof(WaveArgs, inl) + (size_t)bi * sizeof(NodeDesc));
        uint32_t words[sizeof(NodeDesc) / 4];
#pragma unroll
        for (int q = 0; q < (int)(sizeof(NodeDesc) / 4); ++q) words[q] = src[q];
        __builtin_memcpy(&d, words, sizeof(NodeDesc));
    } else if (p.descs) {
        d = p.descs[bi];
    } else {
        d = p.base;
        d.A += (int64_t)bi * p.sA; d.w += (int64_t)bi * p.sw; d.B += (int64_t)bi * p.sB;
        d.out += (int64_t)bi * p.sO;
        if (d.arg) d.arg += (int64_t)bi * p.sO;
        if (d.rngA) d.rngA += (int64_t)bi * p.sR;
        if (d.rngW) d.rngW += (int64_t)bi * p.sR;
        if (d.rngB) d.rngB += (int64_t)bi * p.sR;
        d.Ci = p.Ci; d.Cj = p.Cj; d.Ck = p.Ck;
    }
    const int Ci = d.Ci, Cj = d.Cj, Ck = d.Ck;
    const int tilesN = (Ck + TS - 1) / TS;
    const int tm = tl / tilesN, tn = tl - tm * tilesN;
    const int a0 = tm * TS, b0 = tn * TS;
    // this wavefront's share of the candidates: all of them, or a quarter
    int cbeg = 0, cend = Cj;
    if (SPLIT) {
        const int per = (Cj + kWavesPerGroup - 1) / kWavesPerGroup;
        cbeg = min(wave * per, Cj);
        cend = min(cbeg + per, Cj);
    }

    const gcptr A = (gcptr)(uintptr_t)d.A;
    const gcptr W = (gcptr)(uintptr_t)d.w;
    const gcptr B = (gcptr)(uintptr_t)d.B;
    const gptr O = (gptr)(uintptr_t)d.out;
    const gptr G = (gptr)(uintptr_t)d.arg;

    // ---- staging loads: A, TS rows of KC candidates (a load instruction covers 64 consecutive
    //      candidates of one row); B, KC rows of TS columns (a load instruction covers RPL rows).
    //      Every load is a uniform base (scalar registers) plus a small per-lane byte offset; both
    //      are clamped to the last candidate, so a chunk that reaches past the end of c repeats it.
    int32_t pa[NL], pb[NL], pw[NLW];
    using gbptr = const char __attribute__((address_space(1)))*;
    auto ldw = [](gcptr base, uint32_t byte_off) { return *(gcptr)((gbptr)base + byte_off); };
    gcptr arow[TS];                                          // row bases of the A strip
#pragma unroll
    for (int r = 0; r < TS; ++r) arow[r] = A + (int64_t)min(a0 + r, Ci - 1) * Cj;
    const int brow = lane / TS;                              // row of B inside a load instruction
    const uint32_t bcol4 = (uint32_t)min(b0 + (lane % TS), Ck - 1) * 4u;   // clamped column, fixed for the tile
    const uint32_t Ck4 = (uint32_t)Ck * 4u;                  // <= 2^18
    auto fetch = [&](int c0) {
        const int last = cend - 1 - c0;                      // the chunk's last valid candidate (>= 0)
        uint32_t offA[NLW], offB[NL];
#pragma unroll
        for (int j = 0; j < NLW; ++j) offA[j] = (uint32_t)min(lane, max(last - j * 64, 0)) * 4u;
#pragma unroll
        for (int i = 0; i < NL; ++i)
            offB[i] = (uint32_t)min(brow, max(last - i * RPL, 0)) * Ck4 + bcol4;   // < 8 * 2^18 + 2^18
        // Opaque from here on, so that the widening of the offsets to 64 bits sits next to the loads:
        // only then does the compiler use the "scalar base + 32-bit lane offset" addressing mode
        // instead of forming every address in a pair of vector registers.
#pragma unroll
        for (int j = 0; j < NLW; ++j) asm volatile("" : "+v"(offA[j]));
#pragma unroll
        for (int i = 0; i < NL; ++i) asm volatile("" : "+v"(offB[i]));
#pragma unroll
        for (int i = 0; i < NL; ++i) pa[i] = ldw(arow[(i * 64) / KC] + c0 + min((i * 64) % KC, last), offA[((i * 64) % KC) / 64]);
#pragma unroll
        for (int j = 0; j < NLW; ++j) pw[j] = ldw(W + c0 + min(j * 64, last), offA[j]);
        const gcptr Bc = B + (int64_t)c0 * Ck;
#pragma unroll
        for (int i = 0; i < NL; ++i) pb[i] = ldw(Bc + min(i * RPL, last) * Ck, offB[i]);   // < 128 * 2^16
    };

    // what the output's range pair holds so far (only a filter for the atomics at the end)
    int cur_min = 0x7fffffff, cur_max = (int)0x80000000;
    if (d.rngOut) { const gcptr r = (gcptr)(uintptr_t)d.rngOut; cur_min = r[0]; cur_max = r[1]; }
    // The sums must fit int32.  Judged from the values this wavefront stages -- the strip of A, the
    // strip of B and w -- with the tiled kernel's formula (max A + max w + max B, and the minima):
    // no measured ranges are needed, and the test is tighter than one over the whole tables.
    int32_t loA = 0x7fffffff, hiA = (int32_t)0x80000000, loB = 0x7fffffff, hiB = (int32_t)0x80000000,
            loW = 0x7fffffff, hiW = (int32_t)0x80000000;

    int32_t* As = lds[wave];               // [TS][AST]: A + w, row-major
    int32_t* Bs = As + TS * AST;           // [KC][TS]
    const int lx = lane & 7, ly = lane >> 3;

    int32_t best[RB][RB], arg[RB][RB];
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int j = 0; j < RB; ++j) { best[i][j] = 0x7fffffff; arg[i][j] = 0; }

    // One chunk's arithmetic on what the stage holds.  Groups of 16 candidates, read from LDS four at
    // a time, the next four before the arithmetic of the current four (a wavefront alone on its SIMD
    // has nobody else to hide the latency).  The stage always holds KC valid candidates, so reading
    // ahead never leaves it.  Within a group a cell records the position (0..15, constants that cost
    // no register) of its last strict improvement; the group's first index is added once per group.
    auto compute = [&](int c0) {
        const int kc = min(KC, cend - c0);
        int32_t av[2][RB][4], bv[2][4][RB];
        auto lds_read = [&](int cc, int32_t (&a)[RB][4], int32_t (&b)[4][RB]) {
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int4 a4 = *reinterpret_cast<const int4*>(&As[(ly * RB + i) * AST + cc]);
                a[i][0] = a4.x; a[i][1] = a4.y; a[i][2] = a4.z; a[i][3] = a4.w;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if constexpr (RB == 1) b[q][0] = Bs[(cc + q) * TS + lx];
                else {
                    const int2 b2 = *reinterpret_cast<const int2*>(&Bs[(cc + q) * TS + lx * 2]);
                    b[q][0] = b2.x; b[q][RB - 1] = b2.y;
                }
            }
        };
        int32_t rel[RB][RB];
        auto update = [&](int q0, const int32_t (&a)[RB][4], const int32_t (&b)[4][RB]) {
            if (VALUE) {
#pragma unroll
                for (int q = 0; q < 4; q += 2)
#pragma unroll
                    for (int i = 0; i < RB; ++i)
#pragma unroll
                        for (int j = 0; j < RB; ++j)
                            best[i][j] = min(min(best[i][j], (int32_t)((uint32_t)a[i][q] + (uint32_t)b[q][j])),
                                             (int32_t)((uint32_t)a[i][q + 1] + (uint32_t)b[q + 1][j]));
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int i = 0; i < RB; ++i)
#pragma unroll
                        for (int j = 0; j < RB; ++j) {
                            const int32_t cand = (int32_t)((uint32_t)a[i][q] + (uint32_t)b[q][j]);   // wraps only where overflow was flagged
                            const bool keep = cand >= best[i][j];      // strict '<' wins: ties keep the lower index
                            best[i][j] = min(best[i][j], cand);
                            rel[i][j] = keep ? rel[i][j] : q0 + q;
                        }
            }
        };
        lds_read(0, av[0], bv[0]);
        for (int cc = 0; cc < kc; cc += 16) {
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int j = 0; j < RB; ++j) rel[i][j] = 16;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // the reads of the next four candidates go out before the arithmetic of these four
                lds_read(min(cc + 4 * g + 4, KC - 4), av[(g + 1) & 1], bv[(g + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                update(4 * g, av[g & 1], bv[g & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (!VALUE) {
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int j = 0; j < RB; ++j) arg[i][j] = rel[i][j] < 16 ? c0 + cc + rel[i][j] : arg[i][j];
            }
        }
    };

    // The loads of chunk s are in flight while chunk s - 1 is worked on; then they are written to the
    // stage.  The stage is this wavefront's own and its LDS operations complete in order; the fences
    // keep the compiler from moving the writes across the reads of the chunk before.
    const int nch = (cend - cbeg + KC - 1) / KC;      // 0 for a wavefront whose share of the candidates is empty
    for (int s = 0; s <= nch; ++s) {
        if (s < nch) fetch(cbeg + s * KC);
        if (s > 0) compute(cbeg + (s - 1) * KC);
        if (s < nch) {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
            for (int i = 0; i < NL; i += 2) {
                loA = min(min(loA, pa[i]), pa[i + 1]); hiA = max(max(hiA, pa[i]), pa[i + 1]);
                loB = min(min(loB, pb[i]), pb[i + 1]); hiB = max(max(hiB, pb[i]), pb[i + 1]);
            }
#pragma unroll
            for (int j = 0; j < NLW; ++j) { loW = min(loW, pw[j]); hiW = max(hiW, pw[j]); }
#pragma unroll
            for (int i = 0; i < NL; ++i)
                As[((i * 64) / KC) * AST + (i * 64) % KC + lane] = (int32_t)((uint32_t)pa[i] + (uint32_t)pw[((i * 64) % KC) / 64]);
#pragma unroll
            for (int i = 0; i < NL; ++i) Bs[i * 64 + lane] = pb[i];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
    }

    if (SPLIT) {
        // the wavefronts' shares ascend in c: folding them in that order with a strict '<' keeps the
        // lowest index among equal candidates
        int32_t sl[6] = {loA, hiA, loW, hiW, loB, hiB};
        if (d.flag) {
            sl[0] = wave_min_i32(loA); sl[1] = wave_max_i32(hiA); sl[2] = wave_min_i32(loW);
            sl[3] = wave_max_i32(hiW); sl[4] = wave_min_i32(loB); sl[5] = wave_max_i32(hiB);
        }
        constexpr int ST = 2 * 64 * CELLS;     // where the six range words sit
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                merge[wave][(i * RB + j) * 64 + lane] = best[i][j];
                merge[wave][(CELLS + i * RB + j) * 64 + lane] = arg[i][j];
            }
        if (lane < 6) merge[wave][ST + lane] = sl[lane];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int q = 1; q < kWavesPerGroup; ++q) {
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int j = 0; j < RB; ++j) {
                    const int32_t ob = merge[q][(i * RB + j) * 64 + lane], oa = merge[q][(CELLS + i * RB + j) * 64 + lane];
                    const bool lt = ob < best[i][j];
                    best[i][j] = lt ? ob : best[i][j];
                    arg[i][j] = lt ? oa : arg[i][j];
                }
            loA = min(sl[0], merge[q][ST]); hiA = max(sl[1], merge[q][ST + 1]); loW = min(sl[2], merge[q][ST + 2]);
            hiW = max(sl[3], merge[q][ST + 3]); loB = min(sl[4], merge[q][ST + 4]); hiB = max(sl[5], merge[q][ST + 5]);
            sl[0] = loA; sl[1] = hiA; sl[2] = loW; sl[3] = hiW; sl[4] = loB; sl[5] = hiB;
        }
        loA = sl[0]; hiA = sl[1]; loW = sl[2]; hiW = sl[3]; loB = sl[4]; hiB = sl[5];     // uniform already
    }
    if (d.flag) {
        const long long xloA = wave_min_i32(loA), xhiA = wave_max_i32(hiA), xloB = wave_min_i32(loB), xhiB = wave_max_i32(hiB),
                        xloW = wave_min_i32(loW), xhiW = wave_max_i32(hiW);
        const long long hi = xhiA + xhiW + xhiB, lo = xloA + xloW + xloB, hi2 = xhiA + xhiW, lo2 = xloA + xloW;
        if ((hi > 2147483647ll || lo < -2147483648ll || hi2 > 2147483647ll || lo2 < -2147483648ll) && lane == 0)
            atomicOr(d.flag, 1);
        // promised ranges: the loads are clamped to valid elements, so everything seen here is data
        if (wa.verify && lane == 0 &&
            (xloA < d.loA || xhiA > d.hiA || xloW < d.loW || xhiW > d.hiW || xloB < d.loB || xhiB > d.hiB))
            atomicOr(d.flag, 2);
    }

    // ---- results ----
    int vmin = 0x7fffffff, vmax = (int)0x80000000;
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        const int a = a0 + ly * RB + i;
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const int b = b0 + lx * RB + j;
            if (a < Ci && b < Ck) {
                O[(int64_t)a * Ck + b] = best[i][j];
                if (!VALUE && G) G[(int64_t)a * Ck + b] = arg[i][j];
                vmin = min(vmin, best[i][j]); vmax = max(vmax, best[i][j]);
            }
        }
    }
    if (p.mode_count && tl == 0 && lane == 0) atomicAdd(&p.mode_count[VALUE ? kModeValue : kModePlain], 1);
    if (d.rngOut) {
        // measured range of this table, if a launch that consumes it asks for one.  Thousands of
        // wavefronts share the pair and atomics on one address take their turn, so the caller leaves
        // rngOut null where it can; wavefronts that do not extend the range as it stood when they
        // started do not touch it.
        vmin = wave_min_i32(vmin); vmax = wave_max_i32(vmax);
        if (lane == 0 && vmin <= vmax) {
            if (vmin < cur_min) atomicMin(&d.rngOut[0], vmin);
            if (vmax > cur_max) atomicMax(&d.rngOut[1], vmax);
        }
    }
}

}  // namespace

hipError_t launch_minplus_wave(const NodeArgs& args, const NodeDesc* h_descs, int mode, int rb, hipStream_t stream,
                               bool verify) {
    if ((mode != kModePlain && mode != kModeValue) || (rb != 1 && rb != 2)) return hipErrorInvalidValue;
    if (args.batch < 1 || args.total_tiles < 1 || args.kparts > 1) return hipErrorInvalidValue;
    if (!args.tile_begin) {
        // one shape: total_tiles must be what the shape implies at this tile size
        const int ts = 8 * rb;
        const int64_t tm = (args.Ci + ts - 1) / ts, tn = (args.Ck + ts - 1) / ts;
        if (args.Ci < 1 || args.Cj < 1 || args.Ck < 1 || args.tilesM != tm || args.tilesN != tn ||
            (int64_t)args.total_tiles != tm * tn * args.batch)
            return hipErrorInvalidValue;
    } else if (!args.descs) {
        return hipErrorInvalidValue;
    }
    const unsigned blocks = (unsigned)(((int64_t)args.total_tiles + kWavesPerGroup - 1) / kWavesPerGroup);
    dim3 grid(blocks), block(kWaveGroup);
    WaveArgs wa{};
    wa.a = args;
    wa.verify = verify ? 1 : 0;
    if (h_descs && args.descs) {
        wa.n_inline = args.batch < kWaveInlineDescs ? args.batch : kWaveInlineDescs;
        for (int q = 0; q < wa.n_inline; ++q) wa.inl[q] = h_descs[q];
    }
    // up to kWaveSplitTiles tiles (kWaveSplitTiles16 of the larger size): four wavefronts share a tile (a workgroup per tile);
    // 8 x 8 tiles: up to kWaveLongChunkTiles a wavefront each with long chunks; beyond, short chunks
    const bool split = args.total_tiles <= (rb == 2 ? kWaveSplitTiles16 : kWaveSplitTiles);
    const bool long_chunks = rb == 1 && !split && args.total_tiles <= kWaveLongChunkTiles;
    if (split) grid = dim3((unsigned)args.total_tiles);
#define LWP_WAVE(RB, KC, SPLIT) \
    do { \
        if (mode == kModeValue) hipLaunchKernelGGL((minplus_wave_kernel<RB, KC, true, SPLIT>), grid, block, 0, stream, wa); \
        else hipLaunchKernelGGL((minplus_wave_kernel<RB, KC, false, SPLIT>), grid, block, 0, stream, wa); \
    } while (0)
    if (split && rb == 2) LWP_WAVE(2, 64, true);
    else if (split) LWP_WAVE(1, 64, true);
    else if (long_chunks) LWP_WAVE(1, 128, false);
    else if (rb == 1) LWP_WAVE(1, 64, false);
    else LWP_WAVE(2, 64, false);
#undef LWP_WAVE
    return hipGetLastError();
}

}  // namespace lwp
