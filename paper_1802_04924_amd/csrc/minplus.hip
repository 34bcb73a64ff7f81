// Node elimination (Sec. 5.2, Eq. 2) as a batched min-plus matrix product with argmin:
//   out[a][b] = min_c ( A[a][c] + w[c] + B[c][b] ),  arg[a][b] = lowest c attaining the minimum.
//
// (min,+) is not a ring the matrix cores implement, so this runs on the integer VALU.  One
// workgroup (256 threads = 4 wavefronts) owns a 128 x 128 output tile and walks c in stages of
// 16 that are staged through LDS (double-buffered, one barrier per stage); every thread keeps an
// 8 x 8 block of running minima in registers.  w is folded into A while A is staged, so the inner
// loop is one add and half a three-way min per candidate.
//
// Two arithmetic variants:
//   keyed   candidates are 32-bit keys (cost << tb) | (1 + position of c in its chunk); a chunk
//           is `spc` stages (16*spc <= 2^tb - 1 consecutive c).  An unsigned min over keys
//           carries the lowest c of equal costs inside a chunk for free.  At every chunk end a
//           non-zero low field says the minimum changed in this chunk: (chunk, position) is
//           recorded and the field is cleared, so a later chunk can only win with a strictly
//           smaller cost.  Needs re-based costs that fit 32-tb bits; the host checks that from
//           value ranges.
//   plain   int32 compare/select per candidate (strict '<' in ascending c); no precondition.
#include "lwp_kernels.h"

namespace lwp {

namespace {

constexpr int TM = kTileM, TN = kTileN, TK = kTileK, NT = kNodeThreads;

template <bool KEYED>
__global__ __launch_bounds__(NT, KEYED ? 2 : 1) void minplus_kernel(const NodeArgs p) {
    __shared__ __attribute__((aligned(16))) uint32_t As[2][TK][TM];   // [stage][c][a]  (A transposed)
    __shared__ __attribute__((aligned(16))) uint32_t Bs[2][TK][TN];   // [stage][c][b]

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give every XCD a
    // contiguous range of logical ids, and walk the tiles of a product in panels of 8 tile rows,
    // column by column: 64 consecutive ids (the tiles resident on one XCD at a time) then form an
    // 8 x 8 block that shares 8 row strips of A and 8 column strips of B.
    uint32_t bid = blockIdx.x;
    const uint32_t total = gridDim.x;
    if ((total & 7u) == 0u) bid = (bid & 7u) * (total >> 3) + (bid >> 3);
    const int tiles = p.tilesM * p.tilesN;
    const int bi = bid / tiles;
    const int tl = bid - bi * tiles;
    constexpr int PANEL = 8;
    const int panel = tl / (PANEL * p.tilesN);
    const int prow0 = panel * PANEL;
    const int prows = min(PANEL, p.tilesM - prow0);
    const int within = tl - panel * PANEL * p.tilesN;
    const int tni = within / prows;
    const int tmi = prow0 + (within - tni * prows);
    const int a0 = tmi * TM, b0 = tni * TN;
    const int Ci = p.Ci, Cj = p.Cj, Ck = p.Ck;

    const int32_t* __restrict__ A;
    const int32_t* __restrict__ W;
    const int32_t* __restrict__ B;
    int32_t* __restrict__ O;
    int32_t* __restrict__ G;
    int32_t offA, offB, tb;
    if (p.descs) {
        const NodeDesc d = p.descs[bi];
        A = d.A; W = d.w; B = d.B; O = d.out; G = d.arg; offA = d.offA; offB = d.offB; tb = d.tb;
    } else {
        A = p.base.A + (int64_t)bi * p.sA; W = p.base.w + (int64_t)bi * p.sw; B = p.base.B + (int64_t)bi * p.sB;
        O = p.base.out + (int64_t)bi * p.sO; G = p.base.arg ? p.base.arg + (int64_t)bi * p.sO : nullptr;
        offA = p.base.offA; offB = p.base.offB; tb = p.base.tb;
    }
    const uint32_t fmask = KEYED ? ((1u << tb) - 1u) : 0u;
    const uint32_t padA = KEYED ? ~fmask : 0x7fffffffu;   // never strictly below any running minimum
    const int spc = KEYED ? (int)(fmask >> 4) : 1;        // stages per chunk: 16*spc <= 2^tb - 1

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    // global -> LDS assignment: A: one row, 8 consecutive c;  B: one c, 8 consecutive columns
    const int lr = tid >> 1, lseg = (tid & 1) * 8;
    const int br = tid >> 4, bseg = (tid & 15) * 8;
    const int arow = min(a0 + lr, Ci - 1);                   // clamped: rows past the end are never stored
    const bool vecA = ((Cj & 3) == 0) && ((((uintptr_t)A) | ((uintptr_t)W)) & 15) == 0;
    const bool vecB = ((Ck & 3) == 0) && ((((uintptr_t)B) & 15) == 0) && (b0 + TN <= Ck);
    const int32_t* __restrict__ Arow = A + (int64_t)arow * Cj;

    int32_t ra[8], rw[8], rb[8];
    auto fetch = [&](int c0) {
        if (vecA && c0 + TK <= Cj) {
            const int4* pa = reinterpret_cast<const int4*>(Arow + c0 + lseg);
            const int4* pw = reinterpret_cast<const int4*>(W + c0 + lseg);
            int4 x0 = pa[0], x1 = pa[1], w0 = pw[0], w1 = pw[1];
            ra[0] = x0.x; ra[1] = x0.y; ra[2] = x0.z; ra[3] = x0.w; ra[4] = x1.x; ra[5] = x1.y; ra[6] = x1.z; ra[7] = x1.w;
            rw[0] = w0.x; rw[1] = w0.y; rw[2] = w0.z; rw[3] = w0.w; rw[4] = w1.x; rw[5] = w1.y; rw[6] = w1.z; rw[7] = w1.w;
        } else {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int c = min(c0 + lseg + q, Cj - 1);
                ra[q] = Arow[c]; rw[q] = W[c];
            }
        }
        if (vecB && c0 + TK <= Cj) {
            const int4* pb = reinterpret_cast<const int4*>(B + (int64_t)(c0 + br) * Ck + b0 + bseg);
            int4 y0 = pb[0], y1 = pb[1];
            rb[0] = y0.x; rb[1] = y0.y; rb[2] = y0.z; rb[3] = y0.w; rb[4] = y1.x; rb[5] = y1.y; rb[6] = y1.z; rb[7] = y1.w;
        } else {
            const int c = min(c0 + br, Cj - 1);
#pragma unroll
            for (int q = 0; q < 8; ++q) rb[q] = B[(int64_t)c * Ck + min(b0 + bseg + q, Ck - 1)];
        }
    };
    // pos0 = position of c0 inside its chunk (keyed): the key's low field is 1 + position
    auto stash = [&](int c0, int pos0, int buf) {
        uint32_t kb[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int c = c0 + lseg + q;
            uint32_t ka;
            if (KEYED) ka = ((uint32_t)(ra[q] + rw[q] - offA) << tb) | (uint32_t)(pos0 + lseg + q + 1);
            else ka = (uint32_t)(ra[q] + rw[q]);
            As[buf][lseg + q][lr] = (c < Cj) ? ka : padA;
        }
        const bool cok = (c0 + br) < Cj;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            uint32_t v = KEYED ? ((uint32_t)(rb[q] - offB) << tb) : (uint32_t)rb[q];
            kb[q] = cok ? v : 0u;
        }
        *reinterpret_cast<uint4*>(&Bs[buf][br][bseg]) = make_uint4(kb[0], kb[1], kb[2], kb[3]);
        *reinterpret_cast<uint4*>(&Bs[buf][br][bseg + 4]) = make_uint4(kb[4], kb[5], kb[6], kb[7]);
    };

    // running state of the 8 x 8 block
    uint32_t m1[8][8];   // keyed: running key minimum;  plain: running int32 minimum (as bits)
    uint32_t rec[8][8];  // keyed: c of the last change;  plain: running argmin
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) { m1[i][j] = padA; rec[i][j] = 0u; }

    const int nstages = (Cj + TK - 1) / TK;
    int sic = 0;        // stage index inside the current chunk
    int chunk_c0 = 0;   // first c of the current chunk

    fetch(0);
    stash(0, 0, 0);
    __syncthreads();

    for (int s = 0; s < nstages; ++s) {
        const int buf = s & 1;
        const bool more = (s + 1) < nstages;
        const bool chunk_end = (sic + 1 == spc);
        if (more) fetch((s + 1) * TK);

#pragma unroll
        for (int cc = 0; cc < TK; cc += 2) {
            uint32_t av[2][8], bv[2][8];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint4 al = *reinterpret_cast<const uint4*>(&As[buf][cc + u][ty * 4]);
                const uint4 ah = *reinterpret_cast<const uint4*>(&As[buf][cc + u][64 + ty * 4]);
                const uint4 bl = *reinterpret_cast<const uint4*>(&Bs[buf][cc + u][tx * 4]);
                const uint4 bh = *reinterpret_cast<const uint4*>(&Bs[buf][cc + u][64 + tx * 4]);
                av[u][0] = al.x; av[u][1] = al.y; av[u][2] = al.z; av[u][3] = al.w;
                av[u][4] = ah.x; av[u][5] = ah.y; av[u][6] = ah.z; av[u][7] = ah.w;
                bv[u][0] = bl.x; bv[u][1] = bl.y; bv[u][2] = bl.z; bv[u][3] = bl.w;
                bv[u][4] = bh.x; bv[u][5] = bh.y; bv[u][6] = bh.z; bv[u][7] = bh.w;
            }
            if (KEYED) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        m1[i][j] = min(min(m1[i][j], av[0][i] + bv[0][j]), av[1][i] + bv[1][j]);
            } else {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const uint32_t c = (uint32_t)(s * TK + cc + u);
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const int32_t cand = (int32_t)(av[u][i] + bv[u][j]);
                            const bool lt = cand < (int32_t)m1[i][j];
                            m1[i][j] = lt ? (uint32_t)cand : m1[i][j];
                            rec[i][j] = lt ? c : rec[i][j];
                        }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        if (KEYED && (chunk_end || !more)) {
            // chunk end: a non-zero low field means the minimum changed inside this chunk
            const uint32_t base = (uint32_t)chunk_c0 - 1u;
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t f = m1[i][j] & fmask;
                    rec[i][j] = f ? (base + f) : rec[i][j];
                    m1[i][j] &= ~fmask;
                }
        }
        if (chunk_end) { sic = 0; chunk_c0 = (s + 1) * TK; } else { ++sic; }

        if (more) stash((s + 1) * TK, sic * TK, buf ^ 1);
        __syncthreads();
    }

    // epilogue: rows {ty*4..+3, 64+ty*4..+3}, columns {tx*4..+3, 64+tx*4..+3}
    const bool vecO = ((Ck & 3) == 0) && ((((uintptr_t)O) | ((uintptr_t)G)) & 15) == 0 && (b0 + TN <= Ck);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int a = a0 + (i >> 2) * 64 + ty * 4 + (i & 3);
        if (a >= Ci) continue;
        int32_t val[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            val[j] = KEYED ? (int32_t)(m1[i][j] >> tb) + offA + offB : (int32_t)m1[i][j];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int b = b0 + h * 64 + tx * 4;
            int32_t* orow = O + (int64_t)a * Ck + b;
            if (vecO) {
                *reinterpret_cast<int4*>(orow) = make_int4(val[h * 4], val[h * 4 + 1], val[h * 4 + 2], val[h * 4 + 3]);
                if (G) *reinterpret_cast<int4*>(G + (int64_t)a * Ck + b) =
                    make_int4((int32_t)rec[i][h * 4], (int32_t)rec[i][h * 4 + 1], (int32_t)rec[i][h * 4 + 2], (int32_t)rec[i][h * 4 + 3]);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (b + q < Ck) {
                        orow[q] = val[h * 4 + q];
                        if (G) G[(int64_t)a * Ck + b + q] = (int32_t)rec[i][h * 4 + q];
                    }
            }
        }
    }
}

}  // namespace

hipError_t launch_minplus(const NodeArgs& args, bool keyed, hipStream_t stream) {
    const int64_t blocks = (int64_t)args.tilesM * args.tilesN * args.batch;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(NT);
    if (keyed) hipLaunchKernelGGL(minplus_kernel<true>, grid, block, 0, stream, args);
    else hipLaunchKernelGGL(minplus_kernel<false>, grid, block, 0, stream, args);
    return hipGetLastError();
}

}  // namespace lwp
