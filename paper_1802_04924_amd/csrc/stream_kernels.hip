// The memory-streaming and latency-bound parts of the search: edge elimination (Eq. 3), value
// ranges of the input tables, the residual-graph minimum (Alg. 1, enumeration of the final graph
// with K <= 2 per component) and the undo pass (Alg. 1, last loop).  All of these move each
// table element once; they are bound by HBM bandwidth or by dependent-load latency, not by ALUs.
#include <algorithm>
#include <cstddef>
#include <cstring>

#include "lwp_kernels.h"

namespace lwp {

namespace {

constexpr int kThreads = 256;

// Pointers read out of descriptors are generic to the compiler; these casts say "global memory"
// so that plain global loads/stores are emitted instead of flat ones.
using gi32c = const int32_t __attribute__((address_space(1)))*;
using gi32 = int32_t __attribute__((address_space(1)))*;
using v4i = int __attribute__((ext_vector_type(4)));
using gv4c = const v4i __attribute__((address_space(1)))*;
using gv4 = v4i __attribute__((address_space(1)))*;

__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ int wave_max(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long u = __shfl_xor(v, o);
        v = u < v ? u : v;
    }
    return v;
}

// ---- Eq. 3 -----------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void edge_sum_desc_kernel(const EdgeDesc* __restrict__ descs,
                                                                 const int32_t* const* __restrict__ srcs) {
    const EdgeDesc d = descs[blockIdx.y];
    const int64_t cells = d.cells;
    const int32_t* const* sp = srcs + d.first_src;
    const int n = d.n_src;
    bool vec = ((cells & 3) == 0) && ((((uintptr_t)d.out) & 15) == 0);
    for (int q = 0; q < n; ++q) vec = vec && ((((uintptr_t)sp[q]) & 15) == 0);
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t t0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    int lo = 0x7fffffff, hi = (int)0x80000000;
    bool bad = false;
    const gi32 out = (gi32)(uintptr_t)d.out;
    if (vec) {
        const int64_t n4 = cells >> 2;
        for (int64_t x = t0; x < n4; x += stride) {
            v4i acc = ((gv4c)(uintptr_t)sp[0])[x];
            for (int q = 1; q < n; ++q) {
                const v4i v = ((gv4c)(uintptr_t)sp[q])[x];
                // signed overflow of a + v: operands agree in sign, the sum does not
                const v4i sum = acc + v;
                const v4i ov = (acc ^ sum) & (v ^ sum);
                bad |= (ov.x | ov.y | ov.z | ov.w) < 0;
                acc = sum;
            }
            ((gv4)out)[x] = acc;
            lo = min(min(lo, acc.x), min(acc.y, min(acc.z, acc.w)));
            hi = max(max(hi, acc.x), max(acc.y, max(acc.z, acc.w)));
        }
    } else {
        for (int64_t x = t0; x < cells; x += stride) {
            int32_t acc = ((gi32c)(uintptr_t)sp[0])[x];
            for (int q = 1; q < n; ++q) {
                const int32_t v = ((gi32c)(uintptr_t)sp[q])[x];
                const int32_t sum = (int32_t)((uint32_t)acc + (uint32_t)v);
                bad |= ((acc ^ sum) & (v ^ sum)) < 0;
                acc = sum;
            }
            out[x] = acc;
            lo = min(lo, acc); hi = max(hi, acc);
        }
    }
    if (bad && d.flag) atomicOr(d.flag, 1);
    if (d.rngOut) {
        __shared__ int red[2 * (kThreads / 64)];
        lo = wave_min(lo); hi = wave_max(hi);
        if ((threadIdx.x & 63) == 0) { red[2 * (threadIdx.x >> 6)] = lo; red[2 * (threadIdx.x >> 6) + 1] = hi; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int q = 1; q < kThreads / 64; ++q) { lo = min(lo, red[2 * q]); hi = max(hi, red[2 * q + 1]); }
            if (lo <= hi) { atomicMin(&d.rngOut[0], lo); atomicMax(&d.rngOut[1], hi); }
        }
    }
}

__global__ __launch_bounds__(kThreads) void edge_sum_pair_kernel(const int32_t* e1, const int32_t* e2,
                                                                 int32_t* out, int64_t cells, int32_t* flag) {
    const bool vec = ((cells & 3) == 0) && (((((uintptr_t)e1) | ((uintptr_t)e2) | ((uintptr_t)out)) & 15) == 0);
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t t0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    bool bad = false;
    if (vec) {
        const int64_t n4 = cells >> 2;
        for (int64_t x = t0; x < n4; x += stride) {
            const v4i a = ((gv4c)(uintptr_t)e1)[x];
            const v4i b = ((gv4c)(uintptr_t)e2)[x];
            const v4i sum = a + b;
            const v4i ov = (a ^ sum) & (b ^ sum);     // operands agree in sign, the sum does not
            bad |= (ov.x | ov.y | ov.z | ov.w) < 0;
            ((gv4)(uintptr_t)out)[x] = sum;
        }
    } else {
        for (int64_t x = t0; x < cells; x += stride) {
            const int32_t a = e1[x], b = e2[x];
            const int32_t sum = (int32_t)((uint32_t)a + (uint32_t)b);
            bad |= ((a ^ sum) & (b ^ sum)) < 0;
            out[x] = sum;
        }
    }
    if (bad && flag) atomicOr(flag, 1);
}

// ---- value ranges ------------------------------------------------------------------------------
__global__ void init_workspace_kernel(int32_t* stats, int32_t n_tables, int32_t* flag, unsigned long long* keys,
                                      int32_t n_keys) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n_tables) { stats[2 * t] = 0x7fffffff; stats[2 * t + 1] = (int32_t)0x80000000; }
    if (keys && t < n_keys) keys[t] = ~0ull;
    if (flag && t == 0) *flag = 0;
}

__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t value) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) p[t] = value;
}

__global__ void copy_block_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n16; t += stride) dst[t] = src[t];
}

constexpr int kRangeLoads = 8;      // 16-byte loads a thread keeps in flight
// Table y is elements [y*cells, (y+1)*cells), or [off[y], off[y+1]) if off is given; row blockIdx.y of the
// grid measures table y = y0 + blockIdx.y, or which[y0 + blockIdx.y] if a list of tables is given.
__global__ __launch_bounds__(kThreads) void ranges_kernel(const int32_t* __restrict__ tables, int64_t cells,
                                                          const int64_t* __restrict__ off,
                                                          int32_t* __restrict__ stats, int32_t y0,
                                                          const int32_t* __restrict__ which) {
    __shared__ int smin[kThreads / 64], smax[kThreads / 64];
    const int y = which ? which[y0 + blockIdx.y] : y0 + (int)blockIdx.y;
    const int32_t* T = tables + (off ? off[y] : (int64_t)y * cells);
    if (off) cells = off[y + 1] - off[y];
    int lo = 0x7fffffff, hi = (int32_t)0x80000000;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t t0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (((cells & 3) == 0) && ((((uintptr_t)T) & 15) == 0)) {
        const int64_t n4 = cells >> 2;
        const gv4c T4 = (gv4c)(uintptr_t)T;
        for (int64_t x = t0; x < n4; x += kRangeLoads * stride) {       // independent loads in flight
            v4i v[kRangeLoads];
#pragma unroll
            for (int q = 0; q < kRangeLoads; ++q) {
                const int64_t y = x + q * stride;
                v[q] = T4[y < n4 ? y : x];                     // past the end: repeat an element already counted
            }
#pragma unroll
            for (int q = 0; q < kRangeLoads; ++q) {
                lo = min(min(lo, v[q].x), min(v[q].y, min(v[q].z, v[q].w)));
                hi = max(max(hi, v[q].x), max(v[q].y, max(v[q].z, v[q].w)));
            }
        }
    } else {
        for (int64_t x = t0; x < cells; x += stride) { const int v = T[x]; lo = min(lo, v); hi = max(hi, v); }
    }
    lo = wave_min(lo); hi = wave_max(hi);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { smin[wave] = lo; smax[wave] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int q = 1; q < kThreads / 64; ++q) { lo = min(lo, smin[q]); hi = max(hi, smax[q]); }
        atomicMin(&stats[2 * y], lo);
        atomicMax(&stats[2 * y + 1], hi);
    }
}

// First launch of a search.  Blocks [0, n_nodes): w[v] = tc[v] + ts[v] and {min, max} of the row
// into stats pair w_pair0 + v (written directly: one block owns a row); a sum that leaves int32 is
// reported as the impossible pair {INT32_MAX, INT32_MIN}.  Further blocks: every other stats pair
// becomes {INT32_MAX, INT32_MIN} (ready for atomic min/max), every key all ones.
__global__ __launch_bounds__(kThreads) void prepare_search_kernel(const int32_t* __restrict__ tc,
                                                                  const int32_t* __restrict__ ts,
                                                                  int32_t* __restrict__ w, int32_t n_nodes, int32_t C,
                                                                  const int64_t* __restrict__ node_off,
                                                                  int32_t* __restrict__ stats, int32_t n_pairs,
                                                                  int32_t w_pair0, unsigned long long* __restrict__ keys,
                                                                  int32_t n_keys, int32_t* __restrict__ flag,
                                                                  const uint4* __restrict__ up_src, uint4* __restrict__ up_dst,
                                                                  int32_t up_n16) {
    if ((int)blockIdx.x >= n_nodes) {
        const int t = ((int)blockIdx.x - n_nodes) * kThreads + threadIdx.x;
        if (t == 0 && flag) *flag = 0;
        if (t < n_pairs && (t < w_pair0 || t >= w_pair0 + n_nodes)) { stats[2 * t] = 0x7fffffff; stats[2 * t + 1] = (int32_t)0x80000000; }
        if (t < n_keys) keys[t] = ~0ull;
        // the search's descriptors, from the pinned host mirror into device memory (small blocks only)
        const int stride = ((int)gridDim.x - n_nodes) * kThreads;
        for (int i = t; i < up_n16; i += stride) up_dst[i] = up_src[i];
        return;
    }
    __shared__ int smin[kThreads / 64], smax[kThreads / 64], sbad[kThreads / 64];
    const int64_t row = node_off ? node_off[blockIdx.x] : (int64_t)blockIdx.x * C;
    if (node_off) C = (int32_t)(node_off[blockIdx.x + 1] - row);
    int bad = 0;
    int lo = 0x7fffffff, hi = (int32_t)0x80000000;
    for (int x = threadIdx.x; x < C; x += kThreads) {
        const int64_t s = (int64_t)tc[row + x] + (int64_t)ts[row + x];
        bad |= (s != (int64_t)(int32_t)s);
        w[row + x] = (int32_t)s;
        lo = min(lo, (int32_t)s); hi = max(hi, (int32_t)s);
    }
    lo = wave_min(lo); hi = wave_max(hi); bad = wave_max(bad);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { smin[wave] = lo; smax[wave] = hi; sbad[wave] = bad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int q = 1; q < kThreads / 64; ++q) { lo = min(lo, smin[q]); hi = max(hi, smax[q]); bad |= sbad[q]; }
        stats[2 * (w_pair0 + (int)blockIdx.x)] = bad ? 0x7fffffff : lo;
        stats[2 * (w_pair0 + (int)blockIdx.x) + 1] = bad ? (int32_t)0x80000000 : hi;
    }
}

// ---- residual graph ----------------------------------------------------------------------------
// A component minimum is kept as one 64-bit key: (cost with flipped sign bit) << 32 | flat index,
// so an unsigned 64-bit min orders by cost first and by the lowest flat index among equal costs.
__device__ __forceinline__ unsigned long long make_key(int32_t cost, uint32_t idx) {
    return ((unsigned long long)((uint32_t)cost ^ 0x80000000u) << 32) | idx;
}

__device__ __forceinline__ void block_min_to(unsigned long long v, unsigned long long* dst) {
    __shared__ unsigned long long sm[kThreads / 64];
    v = wave_min_u64(v);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int q = 1; q < kThreads / 64; ++q) v = sm[q] < v ? sm[q] : v;
        if (v != ~0ull) atomicMin(dst, v);
    }
}

// min over (a,b) of w_i[a] + T[a][b] + w_k[b]; grid.y = component
__global__ __launch_bounds__(kThreads) void pair_min_kernel(const PairDesc* __restrict__ pairs,
                                                            unsigned long long* __restrict__ keys,
                                                            int32_t* __restrict__ flag) {
    const PairDesc d = pairs[blockIdx.y];
    const gi32c wi = (gi32c)(uintptr_t)d.wi;
    const gi32c wk = (gi32c)(uintptr_t)d.wk;
    const int Ci = d.Ci, Ck = d.Ck;
    unsigned long long best = ~0ull;
    bool bad = false;
    for (int a = blockIdx.x; a < Ci; a += gridDim.x) {
        const int32_t wa = wi[a];
        const gi32c Trow = (gi32c)(uintptr_t)d.T + (int64_t)a * Ck;
        for (int b = threadIdx.x; b < Ck; b += kThreads) {
            const long long s64 = (long long)wa + Trow[b] + wk[b];
            const int32_t s = (int32_t)s64;
            bad |= (s64 != (long long)s);
            const unsigned long long k = make_key(s, (uint32_t)a * (uint32_t)Ck + (uint32_t)b);
            best = k < best ? k : best;
        }
    }
    if (bad && flag) atomicOr(flag, 1);
    block_min_to(best, &keys[blockIdx.y]);
}

// min over a of w[a]; grid.y = isolated node
__global__ __launch_bounds__(kThreads) void single_min_kernel(const SingleDesc* __restrict__ singles,
                                                              unsigned long long* __restrict__ keys) {
    const gi32c wl = (gi32c)(uintptr_t)singles[blockIdx.y].w;
    const int C = singles[blockIdx.y].C;
    unsigned long long best = ~0ull;
    for (int x = blockIdx.x * kThreads + threadIdx.x; x < C; x += gridDim.x * kThreads) {
        const unsigned long long k = make_key(wl[x], (uint32_t)x);
        best = k < best ? k : best;
    }
    block_min_to(best, &keys[blockIdx.y]);
}

// Enumeration of a residual component (Alg. 1: the final graph's strategies are enumerated).  One
// thread per assignment of the first K-1 nodes (a "prefix", which fixes every term but those of the
// last node); the last node's configurations are an inner loop.  Consecutive threads differ in the
// later digits, so most of a wavefront reads the same table rows.
// The flat (mixed-radix) index ascends lexicographically (lowest node id most significant), so the
// 64-bit (cost, index) minimum is the lexicographically lowest optimum.
__global__ __launch_bounds__(kThreads) void component_min_kernel(const CompDesc* __restrict__ comp,
                                                                 unsigned long long n_prefix,
                                                                 unsigned long long* __restrict__ key,
                                                                 int32_t* __restrict__ flag) {
    __shared__ CompDesc d;
    // edges sorted out once: those between earlier nodes, and those that touch the last node
    __shared__ int n_inner, n_touch;
    __shared__ int8_t inner[kCompMaxEdges], touch[kCompMaxEdges];
    for (int x = threadIdx.x; x < (int)(sizeof(CompDesc) / 4); x += kThreads)
        reinterpret_cast<int32_t*>(&d)[x] = reinterpret_cast<const int32_t*>(comp)[x];
    __syncthreads();
    const int K = d.K, last = K - 1;
    if (threadIdx.x == 0) {
        int ni = 0, nt = 0;
        for (int x = 0; x < d.n_edges; ++x) {
            if (d.src_pos[x] == last || d.dst_pos[x] == last) touch[nt++] = (int8_t)x; else inner[ni++] = (int8_t)x;
        }
        n_inner = ni; n_touch = nt;
    }
    __syncthreads();
    const int ni = n_inner, nt = n_touch;
    const gi32c wl = (gi32c)(uintptr_t)d.w[last];
    const int C = d.Cn[last];
    unsigned long long best = ~0ull;
    bool bad = false;
    const unsigned long long stride = (unsigned long long)gridDim.x * kThreads;
    for (unsigned long long p = (unsigned long long)blockIdx.x * kThreads + threadIdx.x; p < n_prefix; p += stride) {
        int digit[kCompMaxNodes];
        unsigned long long r = p;
        for (int q = last - 1; q >= 0; --q) { digit[q] = (int)(r % (unsigned)d.Cn[q]); r /= (unsigned)d.Cn[q]; }
        long long base = 0;
        for (int q = 0; q < last; ++q) base += ((gi32c)(uintptr_t)d.w[q])[digit[q]];
        for (int z = 0; z < ni; ++z) {
            const int x = inner[z];
            base += ((gi32c)(uintptr_t)d.tab[x])[(int64_t)digit[d.src_pos[x]] * d.Cn[d.dst_pos[x]] + digit[d.dst_pos[x]]];
        }
        // an edge that touches the last node contributes T[first + c * step]
        constexpr int kFast = 4;
        gi32c tp[kFast];
        int64_t ts[kFast];
        for (int z = 0; z < kFast; ++z) {
            const int x = touch[z < nt ? z : 0];
            const bool out_edge = d.src_pos[x] == last;      // the last node is the edge's source
            tp[z] = (gi32c)(uintptr_t)d.tab[x] + (out_edge ? (int64_t)digit[d.dst_pos[x]] : (int64_t)digit[d.src_pos[x]] * C);
            ts[z] = out_edge ? d.Cn[d.dst_pos[x]] : 1;
        }
        for (int c = 0; c < C; ++c) {
            long long t = base + wl[c];
#pragma unroll
            for (int z = 0; z < kFast; ++z)
                if (z < nt) t += tp[z][c * ts[z]];
            for (int z = kFast; z < nt; ++z) {
                const int x = touch[z];
                const gi32c T = (gi32c)(uintptr_t)d.tab[x];
                t += (d.src_pos[x] == last) ? T[(int64_t)c * d.Cn[d.dst_pos[x]] + digit[d.dst_pos[x]]]
                                            : T[(int64_t)digit[d.src_pos[x]] * C + c];
            }
            bad |= (t != (long long)(int32_t)t);
            const unsigned long long k = make_key((int32_t)t, (uint32_t)(p * (unsigned)C + (unsigned)c));
            best = k < best ? k : best;
        }
    }
    if (bad && flag) atomicOr(flag, 1);
    block_min_to(best, key);
}

// ---- undo (Alg. 1: S^(i) = S^(i+1) + c_j, c_j the stored argmin of Eq. 2 at (c_i, c_k)) ---------
// One workgroup of 1024 threads: the recomputing form keeps 16 wavefronts busy per round.
constexpr int kUndoThreads = 1024;
constexpr int kUndoLdsNodes = 4096;
__device__ __forceinline__ void back_substitute_body(
    const PairDesc* __restrict__ pairs, int32_t n_pairs, const SingleDesc* __restrict__ singles, int32_t n_singles,
    const CompDesc* __restrict__ comps, int32_t n_comps,
    const unsigned long long* __restrict__ keys, const UndoDesc* __restrict__ undo, int32_t n_undo,
    int32_t n_nodes, const int32_t* __restrict__ flag, const int32_t* __restrict__ wstats,
    int32_t* __restrict__ result, int32_t* __restrict__ host_result, int32_t* S) {
    // S: where the strategy is built up, n_nodes words: result + 2 itself, or memory that is quicker to
    // reach for this workgroup (LDS), copied to result + 2 at the end
    __shared__ long long ssum[kUndoThreads / 64];
    // A log of up to one entry per thread is fetched here, all entries at once and before anything
    // waits: a round of the walk below then costs one trip to memory (the argmin table) instead of
    // three dependent ones (where the round starts, whether argmin tables were stored, the entry).
    __shared__ int first_of[kUndoThreads];     // entry -> first entry of its round; sign bit: no stored argmin
    const bool log_in_registers = n_undo <= kUndoThreads;
    UndoDesc mine{};
    if (log_in_registers && (int)threadIdx.x < n_undo) {
        mine = undo[threadIdx.x];
        first_of[threadIdx.x] = mine.first | (mine.arg ? 0 : (int)0x80000000);
    }
    long long cost = 0;
    for (int t = threadIdx.x; t < n_pairs + n_singles + n_comps; t += kUndoThreads) {
        const unsigned long long k = keys[t];
        uint32_t flat = (uint32_t)k;
        cost += (long long)(int32_t)((uint32_t)(k >> 32) ^ 0x80000000u);
        if (t < n_pairs) {
            const uint32_t Ck = (uint32_t)pairs[t].Ck;
            S[pairs[t].src] = (int32_t)(flat / Ck); S[pairs[t].dst] = (int32_t)(flat % Ck);
        } else if (t < n_pairs + n_singles) S[singles[t - n_pairs].node] = (int32_t)flat;
        else {
            const CompDesc* cd = comps + (t - n_pairs - n_singles);
            for (int q = cd->K - 1; q >= 0; --q) { S[cd->node[q]] = (int32_t)(flat % (uint32_t)cd->Cn[q]); flat /= (uint32_t)cd->Cn[q]; }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cost += __shfl_xor(cost, o);
    if ((threadIdx.x & 63) == 0) ssum[threadIdx.x >> 6] = cost;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long tot = 0;
        for (int q = 0; q < kUndoThreads / 64; ++q) tot += ssum[q];
        result[0] = (int32_t)(tot & 0xffffffffll);
        result[1] = (int32_t)(tot >> 32);
    }
    // An elimination that a speculative launch skipped left its tables unwritten: argmin entries
    // would then be arbitrary numbers, not configurations, so nothing is looked up through them.
    // (The flag is final: every launch that can set it has completed before this kernel starts.)
    if (flag && (*flag & 4)) {
        if (threadIdx.x == 0) {
            result[2 + n_nodes] = *flag;
            if (host_result) host_result[2 + n_nodes] = *flag;
        }
        return;
    }
    // walk the rounds backwards; node eliminations of one round never depend on each other
    int hi = n_undo;
    while (hi > 0) {
        const int word = log_in_registers ? first_of[hi - 1] : undo[hi - 1].first;     // (ssum's barrier covers first_of)
        const int lo = word & 0x7fffffff;
        const bool stored = log_in_registers ? word >= 0 : undo[lo].arg != nullptr;
        if (stored && log_in_registers) {
            const int t = threadIdx.x;
            if (t >= lo && t < hi) S[mine.j] = ((gi32c)(uintptr_t)mine.arg)[(int64_t)S[mine.i] * mine.Ck + S[mine.k]];
        } else if (stored) {
            for (int t = lo + threadIdx.x; t < hi; t += kUndoThreads) {
                const UndoDesc u = undo[t];
                S[u.j] = ((gi32c)(uintptr_t)u.arg)[(int64_t)S[u.i] * u.Ck + S[u.k]];
            }
        } else {
            // no stored argmin: c_j = lowest c minimising A[S_i][c] + w[c] + B[c][S_k] (the paper's
            // own undo step); one wavefront per elimination
            for (int t = lo + (threadIdx.x >> 6); t < hi; t += kUndoThreads / 64) {
                const UndoDesc u = undo[t];
                const gi32c Arow = (gi32c)(uintptr_t)u.A + (int64_t)S[u.i] * u.Cj;
                const gi32c Bcol = (gi32c)(uintptr_t)u.B + S[u.k];
                const gi32c wj = (gi32c)(uintptr_t)u.w;
                unsigned long long best = ~0ull;
                for (int c = threadIdx.x & 63; c < u.Cj; c += 64) {
                    const unsigned long long k = make_key(Arow[c] + wj[c] + Bcol[(int64_t)c * u.Ck], (uint32_t)c);
                    best = k < best ? k : best;
                }
                best = wave_min_u64(best);
                if ((threadIdx.x & 63) == 0) S[u.j] = (int32_t)(uint32_t)best;
            }
        }
        __syncthreads();
        hi = lo;
    }
    if (S != result + 2)
        for (int t = threadIdx.x; t < n_nodes; t += kUndoThreads) result[2 + t] = S[t];
    // a row of t_c + t_s that left int32 was recorded as the impossible range {INT32_MAX, INT32_MIN}
    __shared__ int wbad;
    if (threadIdx.x == 0) wbad = 0;
    __syncthreads();
    if (wstats)
        for (int v = threadIdx.x; v < n_nodes; v += kUndoThreads)
            if (wstats[2 * v] > wstats[2 * v + 1]) wbad = 1;
    __syncthreads();
    if (threadIdx.x == 0) result[2 + n_nodes] = (flag ? *flag : 0) | wbad;
    // the result goes straight to the caller's pinned host buffer (posted writes over the host
    // link, complete when the kernel is): one dependent copy fewer at the end of every search
    // The last word is the one a host that polls the buffer waits for: one thread stores it with
    // system-scope release semantics after a barrier behind everybody's stores (a release is
    // cumulative over the barrier; one wavefront pays for it instead of sixteen fencing each).
    if (host_result) {
        __syncthreads();
        for (int t = threadIdx.x; t < 2 + n_nodes; t += kUndoThreads) host_result[t] = result[t];
        __syncthreads();
        if (threadIdx.x == 0)
            __hip_atomic_store(&host_result[2 + n_nodes], result[2 + n_nodes], __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

__global__ __launch_bounds__(kUndoThreads) void back_substitute_kernel(
    const PairDesc* __restrict__ pairs, int32_t n_pairs, const SingleDesc* __restrict__ singles, int32_t n_singles,
    const CompDesc* __restrict__ comps, int32_t n_comps,
    const unsigned long long* __restrict__ keys, const UndoDesc* __restrict__ undo, int32_t n_undo,
    int32_t n_nodes, const int32_t* __restrict__ flag, const int32_t* __restrict__ wstats,
    int32_t* __restrict__ result, int32_t* __restrict__ host_result) {
    // the strategy is built up in LDS when it fits (the walk reads two entries of it per elimination)
    __shared__ int32_t s_lds[kUndoLdsNodes];
    back_substitute_body(pairs, n_pairs, singles, n_singles, comps, n_comps, keys, undo, n_undo, n_nodes, flag, wstats, result,
                         host_result, n_nodes <= kUndoLdsNodes ? s_lds : result + 2);
}

// ---- a whole small search in one workgroup ------------------------------------------------------
// Alg. 1 from the sum t_c + t_s to the strategy, for searches so small (the paper's own sizes: a
// handful of devices, tens of configurations per layer) that the launches of the general path --
// a dozen dependent kernels of a few microseconds each -- cost far more than the arithmetic.  One
// workgroup of 1024 threads walks the same descriptors the general path uses: per round the edge
// sums (Eq. 3) and the node eliminations (Eq. 2, one output cell per thread, candidates in ascending
// c with a strict '<'), then the residual minima and the undo pass.  A workgroup barrier separates
// the phases: all tables involved were written by this workgroup through its own compute unit.
// Overflow is found exactly (a sum that really leaves int32): 64-bit sums, or the carries of the
// 32-bit additions in the node eliminations.
__device__ __forceinline__ unsigned long long block_min_u64(unsigned long long v, unsigned long long* sm) {
    v = wave_min_u64(v);
    __syncthreads();                                  // sm may still be read from the previous call
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long r = sm[0];
    for (int q = 1; q < kUndoThreads / 64; ++q) r = sm[q] < r ? sm[q] : r;
    return r;
}

struct TinyLaunch {
    TinyArgs a;
    alignas(16) unsigned char block[kTinyInlineBytes];
};
static_assert(sizeof(TinyLaunch) <= 4096, "kernel arguments");

constexpr int kTinyPrefix = 256;          // products whose cells are dealt to the threads together
constexpr uint32_t kTinyBias = 0x80000000u;
// Every table of the search (the rows of t_c + t_s, the caller's t_x, the intermediate tables: at most
// kTinyLdsWords words together, which the host checks) has a copy in LDS, at the table's offset in
// (w | t_x | intermediates): operands are read from LDS only, results go to LDS and to global memory
// (the residual and undo phases, and nothing else, read them there).  A round is then bound by the
// compute unit's instruction rate rather than by chains of memory round trips.
// LDS holds v ^ 2^31 (the value plus 2^31 as an unsigned number): the sum of three such words is
// a + w + b + 3 * 2^31, so the two carries of its 32-bit additions tell exactly whether a + w + b
// fits int32 (it does iff exactly one of them carries), the low word is the biased sum, and unsigned
// order on it is the order of the sums -- seven vector instructions per candidate (two additions,
// compare, minimum, select, two for addresses; the carries land in scalar registers) instead of the
// sixteen of 64-bit sums and compares.
__global__ __launch_bounds__(kUndoThreads) void tiny_search_kernel(const TinyLaunch t) {
    __shared__ unsigned long long smin[kUndoThreads / 64];
    __shared__ uint32_t stage[kTinyLdsWords];
    __shared__ int cell_begin[kTinyPrefix + 1];
    __shared__ int prod_a[kTinyPrefix], prod_w[kTinyPrefix], prod_b[kTinyPrefix], prod_o[kTinyPrefix];
    __shared__ int prod_cj[kTinyPrefix], prod_ck[kTinyPrefix];
    __shared__ int32_t* prod_out[kTinyPrefix];
    __shared__ int32_t* prod_arg[kTinyPrefix];
    const int tid = threadIdx.x;
    bool bad = false;
    TinyArgs a = t.a;
    if (a.inline_block) {
        // the descriptors are in the kernel-argument segment: turn the offsets into pointers
        using kaptr = const char __attribute__((address_space(4)))*;
        const char* blk = (const char*)((kaptr)__builtin_amdgcn_kernarg_segment_ptr() + offsetof(TinyLaunch, block));
        a.rounds = (const TinyRound*)(blk + (uintptr_t)a.rounds);
        a.nodes = (const NodeDesc*)(blk + (uintptr_t)a.nodes);
        a.edges = (const EdgeDesc*)(blk + (uintptr_t)a.edges);
        a.srcs = (const int32_t* const*)(blk + (uintptr_t)a.srcs);
        a.pairs = (const PairDesc*)(blk + (uintptr_t)a.pairs);
        a.singles = (const SingleDesc*)(blk + (uintptr_t)a.singles);
        a.comps = (const CompDesc*)(blk + (uintptr_t)a.comps);
        a.undo = (const UndoDesc*)(blk + (uintptr_t)a.undo);
    }
    if (a.up_n16) {
        // the descriptor block did not fit the kernel arguments: it is copied from the host's pinned
        // mirror to where the pointers above point, by this workgroup, before anything reads it
        const uint4* src = reinterpret_cast<const uint4*>(a.up_src);
        uint4* dst = reinterpret_cast<uint4*>(a.up_dst);
#pragma unroll 4
        for (int x = tid; x < a.up_n16; x += kUndoThreads) dst[x] = src[x];
        __syncthreads();
    }
    const int n_w = (int)a.n_w, n_tx = (int)a.n_tx;
    // LDS word of a table that starts at p
    auto lds_word = [&](const int32_t* p) -> int {
        int64_t o = ((intptr_t)p - (intptr_t)a.w) >> 2;
        if (o >= 0 && o < a.n_w) return (int)o;
        o = ((intptr_t)p - (intptr_t)a.tx) >> 2;
        if (o >= 0 && o < a.n_tx) return n_w + (int)o;
        return n_w + n_tx + (int)(((intptr_t)p - (intptr_t)a.slots) >> 2);
    };
    if (tid == 0) *a.flag = 0;
    for (int64_t x = tid; x < a.n_w; x += kUndoThreads) {
        const long long s = (long long)a.tc[x] + (long long)a.ts[x];
        bad |= (s != (long long)(int32_t)s);
        a.w[x] = (int32_t)s;
        stage[x] = (uint32_t)(int32_t)s ^ kTinyBias;
    }
#pragma unroll 8
    for (int x = tid; x < n_tx; x += kUndoThreads) stage[n_w + x] = (uint32_t)a.tx[x] ^ kTinyBias;
    __syncthreads();
    for (int r = 0; r < a.n_rounds; ++r) {
        const TinyRound rd = a.rounds[r];
        for (int g = rd.g0; g < rd.g1; ++g) {                      // Eq. 3, k-way
            const EdgeDesc d = a.edges[g];
            const int32_t* const* sp = a.srcs + d.first_src;
            const int oo = lds_word(d.out);                        // may be the first source: a cell is
            for (int x = tid; x < (int)d.cells; x += kUndoThreads) {   // read and written by one thread
                long long acc = 0;
                for (int q = 0; q < d.n_src; ++q) acc += (long long)(int32_t)(stage[lds_word(sp[q]) + x] ^ kTinyBias);
                bad |= (acc != (long long)(int32_t)acc);
                d.out[x] = (int32_t)acc;
                stage[oo + x] = (uint32_t)(int32_t)acc ^ kTinyBias;
            }
        }
        if (rd.g1 > rd.g0) __syncthreads();
        // Eq. 2.  The cells of all products of the round are dealt to the threads together (the host
        // numbered them; the numbers, in LDS, tell a thread which product its cell belongs to):
        // product after product would cost the workgroup one chain of dependent loads per product
        // instead of one per round.
        for (int q0 = rd.n0; q0 < rd.n1; q0 += kTinyPrefix) {
            const int n_prod = min(kTinyPrefix, rd.n1 - q0);
            if (q0 > rd.n0) __syncthreads();                       // the arrays below are in use until here
            if (tid < n_prod) {
                const NodeDesc d = a.nodes[q0 + tid];
                const int first = a.nodes[q0].cell_begin;
                cell_begin[tid] = d.cell_begin - first;
                if (tid == n_prod - 1) cell_begin[n_prod] = d.cell_begin - first + d.Ci * d.Ck;
                prod_a[tid] = lds_word(d.A); prod_w[tid] = lds_word(d.w); prod_b[tid] = lds_word(d.B);
                prod_o[tid] = lds_word(d.out);
                prod_cj[tid] = d.Cj; prod_ck[tid] = d.Ck; prod_out[tid] = d.out; prod_arg[tid] = d.arg;
            }
            __syncthreads();
            const int total = cell_begin[n_prod];
            for (int x = tid; x < total; x += kUndoThreads) {
                int lo = 0, hi = n_prod;
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (cell_begin[mid] <= x) lo = mid; else hi = mid;
                }
                const int cell = x - cell_begin[lo];
                const int Cj = prod_cj[lo], Ck = prod_ck[lo];
                const int ra = cell / Ck, cb = cell - ra * Ck;
                const uint32_t* As = stage + prod_a[lo] + ra * Cj;
                const uint32_t* Ws = stage + prod_w[lo];
                const uint32_t* Bs = stage + prod_b[lo] + cb;
                uint32_t best = ~0u;        // no candidate is above it, and the lowest c wins ties
                int arg = 0;
                auto candidate = [&](uint32_t av, uint32_t wv, uint32_t bv, int c) {
                    uint32_t s1, v;
                    const bool c1 = __builtin_add_overflow(av, wv, &s1);
                    const bool c2 = __builtin_add_overflow(s1, bv, &v);
                    bad |= (c1 == c2);
                    if (v < best) { best = v; arg = c; }
                };
                // the LDS reads of eight (then four) candidates are issued before the first is used
                int c = 0;
                for (; c + 8 <= Cj; c += 8) {
                    uint32_t av[8], wv[8], bv[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) { av[u] = As[c + u]; wv[u] = Ws[c + u]; bv[u] = Bs[(c + u) * Ck]; }
#pragma unroll
                    for (int u = 0; u < 8; ++u) candidate(av[u], wv[u], bv[u], c + u);
                }
                if (c + 4 <= Cj) {
                    uint32_t av[4], wv[4], bv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) { av[u] = As[c + u]; wv[u] = Ws[c + u]; bv[u] = Bs[(c + u) * Ck]; }
#pragma unroll
                    for (int u = 0; u < 4; ++u) candidate(av[u], wv[u], bv[u], c + u);
                    c += 4;
                }
                for (; c < Cj; ++c) candidate(As[c], Ws[c], Bs[c * Ck], c);
                prod_out[lo][cell] = (int32_t)(best ^ kTinyBias);
                stage[prod_o[lo] + cell] = best;
                if (prod_arg[lo]) prod_arg[lo][cell] = arg;
            }
        }
        __syncthreads();
    }
    // residual graph: a 64-bit (cost, flat index) minimum per component
    for (int p = 0; p < a.n_pairs; ++p) {
        const PairDesc d = a.pairs[p];
        unsigned long long best = ~0ull;
        for (int x = tid; x < d.Ci * d.Ck; x += kUndoThreads) {
            const int ra = x / d.Ck, cb = x - ra * d.Ck;
            const long long s = (long long)d.wi[ra] + d.T[x] + d.wk[cb];
            bad |= (s != (long long)(int32_t)s);
            const unsigned long long k = make_key((int32_t)s, (uint32_t)x);
            best = k < best ? k : best;
        }
        best = block_min_u64(best, smin);
        if (tid == 0) a.keys[p] = best;
    }
    for (int q = 0; q < a.n_singles; ++q) {
        const SingleDesc d = a.singles[q];
        unsigned long long best = ~0ull;
        for (int x = tid; x < d.C; x += kUndoThreads) {
            const unsigned long long k = make_key(d.w[x], (uint32_t)x);
            best = k < best ? k : best;
        }
        best = block_min_u64(best, smin);
        if (tid == 0) a.keys[a.n_pairs + q] = best;
    }
    for (int q = 0; q < a.n_comps; ++q) {
        const CompDesc* cd = a.comps + q;
        const int K = cd->K;
        unsigned long long total = 1;
        for (int z = 0; z < K; ++z) total *= (unsigned)cd->Cn[z];
        unsigned long long best = ~0ull;
        for (unsigned long long f = tid; f < total; f += kUndoThreads) {
            int digit[kCompMaxNodes];
            unsigned long long rem = f;
            for (int z = K - 1; z >= 0; --z) { digit[z] = (int)(rem % (unsigned)cd->Cn[z]); rem /= (unsigned)cd->Cn[z]; }
            long long t = 0;
            for (int z = 0; z < K; ++z) t += cd->w[z][digit[z]];
            for (int e = 0; e < cd->n_edges; ++e)
                t += cd->tab[e][(int64_t)digit[cd->src_pos[e]] * cd->Cn[cd->dst_pos[e]] + digit[cd->dst_pos[e]]];
            bad |= (t != (long long)(int32_t)t);
            const unsigned long long k = make_key((int32_t)t, (uint32_t)f);
            best = k < best ? k : best;
        }
        best = block_min_u64(best, smin);
        if (tid == 0) a.keys[a.n_pairs + a.n_singles + q] = best;
    }
    if (bad) atomicOr(a.flag, 1);
    __syncthreads();
    // the tables in LDS have done their service: the strategy is built up there
    back_substitute_body(a.pairs, a.n_pairs, a.singles, a.n_singles, a.comps, a.n_comps, a.keys, a.undo, a.n_undo, a.n_nodes,
                         a.flag, nullptr, a.result, a.host_result, reinterpret_cast<int32_t*>(stage));
}

// ---- VALU issue-rate probe ----------------------------------------------------------------------
// Register-only chains of the inner loop's two instructions (32-bit add, three-way unsigned min) on
// 32 independent accumulators per thread: measures the int32 VALU rate the chip sustains, against
// which the min-plus kernel's rate is read.  Per loop iteration and thread: 64 adds (all 8 x 8 sums
// of two operand sets) + 32 min3 -- the arithmetic of 64 cell updates.  As compiled the loop also
// holds 7 register moves (the operand updates reuse 8 of the sums); the hardware counters show that
// they cost no issue slot -- an iteration takes 96 x 4 cycles per wavefront, not 103 x 4 -- so they
// are not counted as work.
constexpr int kProbeInstrPerIter = 64 + 32;
constexpr int kProbeUpdatesPerIter = 64;
__global__ __launch_bounds__(kThreads) void alu_probe_kernel(uint32_t* __restrict__ out, int iters, uint32_t seed) {
    uint32_t m[32], a[8], b[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) { a[q] = seed + threadIdx.x * 7u + q; b[q] = seed * 3u + blockIdx.x + 11u * q; }
#pragma unroll
    for (int j = 0; j < 32; ++j) m[j] = 0xffffffffu;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int p0 = 2 * j, p1 = 2 * j + 1;            // two of the 64 (a, b) pairs
            m[j] = min(min(m[j], a[p0 & 7] + b[p0 >> 3]), a[p1 & 7] + b[p1 >> 3]);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) a[q] += b[q];
#pragma unroll
        for (int j = 0; j < 32; j += 4) asm volatile("" : "+v"(m[j]), "+v"(m[j + 1]), "+v"(m[j + 2]), "+v"(m[j + 3]));
    }
    uint32_t r = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) r ^= m[j];
    if (r == 0x12345u) out[0] = r;        // never true in practice; keeps the chains alive
}

inline unsigned blocks_for(int64_t work_items, int64_t per_thread, unsigned cap) {
    int64_t b = (work_items + (int64_t)kThreads * per_thread - 1) / ((int64_t)kThreads * per_thread);
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

}  // namespace

hipError_t launch_edge_sum_desc(const EdgeDesc* d_descs, const int32_t* const* d_src_ptrs, int32_t n_desc,
                                int64_t max_cells, hipStream_t stream) {
    for (int32_t t0 = 0; t0 < n_desc; t0 += 65535) {
        const int32_t n = (n_desc - t0) < 65535 ? (n_desc - t0) : 65535;
        dim3 grid(blocks_for(max_cells, 16, 2048), (unsigned)n);
        hipLaunchKernelGGL(edge_sum_desc_kernel, grid, dim3(kThreads), 0, stream, d_descs + t0, d_src_ptrs);
    }
    return hipGetLastError();
}

hipError_t launch_edge_sum_pair(const int32_t* e1, const int32_t* e2, int32_t* out, int64_t cells, int32_t* flag,
                                hipStream_t stream) {
    dim3 grid(blocks_for(cells, 16, 8192));
    hipLaunchKernelGGL(edge_sum_pair_kernel, grid, dim3(kThreads), 0, stream, e1, e2, out, cells, flag);
    return hipGetLastError();
}

hipError_t launch_init_workspace(int32_t* d_stats, int32_t n_tables, int32_t* d_flag, unsigned long long* d_keys,
                                 int32_t n_keys, hipStream_t stream) {
    const int n = n_tables > n_keys ? n_tables : n_keys;
    hipLaunchKernelGGL(init_workspace_kernel, dim3((n + 256) / 256), dim3(256), 0, stream, d_stats, n_tables, d_flag,
                       d_keys, n_keys);
    return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* d_p, int64_t n, int32_t value, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, d_p, n, value);
    return hipGetLastError();
}

hipError_t launch_copy_block(const void* src, void* dst, size_t bytes, hipStream_t stream) {
    if (bytes == 0) return hipSuccess;
    if (bytes % 16 || ((uintptr_t)src | (uintptr_t)dst) % 16) return hipErrorInvalidValue;
    const int64_t n16 = (int64_t)(bytes / 16);
    const unsigned blocks = (unsigned)std::min<int64_t>((n16 + 255) / 256, 1024);
    hipLaunchKernelGGL(copy_block_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const uint4*>(src),
                       static_cast<uint4*>(dst), n16);
    return hipGetLastError();
}

hipError_t launch_ranges(const int32_t* d_tables, int32_t n_tables, int64_t cells, int32_t* d_stats,
                         hipStream_t stream, const int32_t* d_which) {
    if (n_tables <= 0) return hipSuccess;
    unsigned cap = n_tables >= 64 ? 64u : (n_tables >= 8 ? 512u : 4096u);
    for (int32_t t0 = 0; t0 < n_tables; t0 += 65535) {
        const int32_t n = (n_tables - t0) < 65535 ? (n_tables - t0) : 65535;
        dim3 grid(blocks_for(cells, 4 * kRangeLoads, cap), (unsigned)n);
        hipLaunchKernelGGL(ranges_kernel, grid, dim3(kThreads), 0, stream, d_tables, cells, (const int64_t*)nullptr, d_stats, t0,
                           d_which);
    }
    return hipGetLastError();
}

hipError_t launch_ranges_var(const int32_t* d_tables, const int64_t* d_off, int32_t n_tables, int64_t max_cells,
                             int32_t* d_stats, hipStream_t stream, const int32_t* d_which) {
    if (n_tables <= 0) return hipSuccess;
    unsigned cap = n_tables >= 64 ? 64u : (n_tables >= 8 ? 512u : 4096u);
    for (int32_t t0 = 0; t0 < n_tables; t0 += 65535) {
        const int32_t n = (n_tables - t0) < 65535 ? (n_tables - t0) : 65535;
        dim3 grid(blocks_for(max_cells, 4 * kRangeLoads, cap), (unsigned)n);
        hipLaunchKernelGGL(ranges_kernel, grid, dim3(kThreads), 0, stream, d_tables, (int64_t)0, d_off, d_stats, t0, d_which);
    }
    return hipGetLastError();
}

hipError_t launch_prepare_search(const int32_t* tc, const int32_t* ts, int32_t* w, int32_t n_nodes, int32_t C,
                                 const int64_t* d_node_off, int32_t* d_stats, int32_t n_pairs, int32_t w_pair0,
                                 unsigned long long* d_keys, int32_t n_keys, int32_t* d_flag, hipStream_t stream,
                                 const void* up_src, void* up_dst, size_t up_bytes) {
    if (up_bytes % 16 || ((uintptr_t)up_src | (uintptr_t)up_dst) % 16 || up_bytes > ((size_t)1 << 24)) return hipErrorInvalidValue;
    int n_init = (n_pairs > n_keys ? n_pairs : n_keys) + 1;
    if ((int)(up_bytes / 16) > n_init) n_init = (int)(up_bytes / 16);
    dim3 grid((unsigned)(n_nodes + (n_init + kThreads - 1) / kThreads));
    hipLaunchKernelGGL(prepare_search_kernel, grid, dim3(kThreads), 0, stream, tc, ts, w, n_nodes, C, d_node_off, d_stats,
                       n_pairs, w_pair0, d_keys, n_keys, d_flag, static_cast<const uint4*>(up_src), static_cast<uint4*>(up_dst),
                       (int32_t)(up_bytes / 16));
    return hipGetLastError();
}

hipError_t launch_pair_min(const PairDesc* d_pairs, int32_t n_pairs, int32_t max_rows,
                           unsigned long long* d_keys, int32_t* d_flag, hipStream_t stream) {
    for (int32_t t0 = 0; t0 < n_pairs; t0 += 65535) {
        const int32_t n = (n_pairs - t0) < 65535 ? (n_pairs - t0) : 65535;
        const unsigned rows = (unsigned)max_rows < 2048u ? (unsigned)(max_rows < 1 ? 1 : max_rows) : 2048u;
        dim3 grid(rows, (unsigned)n);
        hipLaunchKernelGGL(pair_min_kernel, grid, dim3(kThreads), 0, stream, d_pairs + t0, d_keys + t0, d_flag);
    }
    return hipGetLastError();
}

hipError_t launch_single_min(const SingleDesc* d_singles, int32_t n_singles, int32_t max_c,
                             unsigned long long* d_keys, hipStream_t stream) {
    for (int32_t t0 = 0; t0 < n_singles; t0 += 65535) {
        const int32_t n = (n_singles - t0) < 65535 ? (n_singles - t0) : 65535;
        dim3 grid(blocks_for(max_c, 4, 64), (unsigned)n);
        hipLaunchKernelGGL(single_min_kernel, grid, dim3(kThreads), 0, stream, d_singles + t0, d_keys + t0);
    }
    return hipGetLastError();
}

hipError_t launch_component_min(const CompDesc* d_comp, unsigned long long n_prefix,
                                unsigned long long* d_key, int32_t* d_flag, hipStream_t stream) {
    unsigned long long blocks = (n_prefix + kThreads - 1) / kThreads;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(component_min_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, d_comp, n_prefix, d_key, d_flag);
    return hipGetLastError();
}

hipError_t launch_tiny_search(const TinyArgs& args, const void* d_block, const void* h_block, size_t block_bytes,
                              hipStream_t stream) {
    if (args.n_w < 0 || args.n_tx < 0 || args.n_slots < 0 || args.n_w + args.n_tx + args.n_slots > (int64_t)kTinyLdsWords)
        return hipErrorInvalidValue;     // the kernel's LDS copy of the tables has that many words
    TinyLaunch t;            // (the launch copies the arguments)
    t.a = args;
    t.a.inline_block = 0;
    t.a.up_src = nullptr; t.a.up_dst = nullptr; t.a.up_n16 = 0;
    if (h_block && d_block && tiny_block_fits_arguments(block_bytes)) {
        std::memcpy(t.block, h_block, block_bytes);
        auto off = [&](const void* p) { return (uintptr_t)((const char*)p - (const char*)d_block); };
        t.a.rounds = (const TinyRound*)off(args.rounds);
        t.a.nodes = (const NodeDesc*)off(args.nodes);
        t.a.edges = (const EdgeDesc*)off(args.edges);
        t.a.srcs = (const int32_t* const*)off(args.srcs);
        t.a.pairs = (const PairDesc*)off(args.pairs);
        t.a.singles = (const SingleDesc*)off(args.singles);
        t.a.comps = (const CompDesc*)off(args.comps);
        t.a.undo = (const UndoDesc*)off(args.undo);
        t.a.inline_block = 1;
    } else if (h_block && d_block && tiny_block_copied_by_kernel(block_bytes)) {
        t.a.up_src = h_block; t.a.up_dst = const_cast<void*>(d_block); t.a.up_n16 = (int32_t)(block_bytes / 16);
    }
    hipLaunchKernelGGL(tiny_search_kernel, dim3(1), dim3(kUndoThreads), 0, stream, t);
    return hipGetLastError();
}

hipError_t launch_alu_probe(uint32_t* d_out, int blocks, int iters, hipStream_t stream) {
    hipLaunchKernelGGL(alu_probe_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, d_out, iters, 12345u);
    return hipGetLastError();
}
int alu_probe_instr_per_iter() { return kProbeInstrPerIter; }
int alu_probe_updates_per_iter() { return kProbeUpdatesPerIter; }

hipError_t launch_back_substitute(const PairDesc* d_pairs, int32_t n_pairs, const SingleDesc* d_singles,
                                  int32_t n_singles, const CompDesc* d_comps, int32_t n_comps,
                                  const unsigned long long* d_keys,
                                  const UndoDesc* d_undo, int32_t n_undo, int32_t n_nodes,
                                  const int32_t* d_flag, const int32_t* d_wstats, int32_t* d_result,
                                  int32_t* h_result, hipStream_t stream) {
    hipLaunchKernelGGL(back_substitute_kernel, dim3(1), dim3(kUndoThreads), 0, stream, d_pairs, n_pairs, d_singles,
                       n_singles, d_comps, n_comps, d_keys, d_undo, n_undo, n_nodes, d_flag, d_wstats, d_result, h_result);
    return hipGetLastError();
}

}  // namespace lwp
