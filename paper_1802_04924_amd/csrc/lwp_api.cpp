// C ABI of the strategy search: argument validation, value-range analysis, buffer planning and
// the launch sequence of Alg. 1 (eliminate -> solve the residual graph -> undo).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <tuple>
#include <vector>

#include "lwp.h"
#include "lwp_internal.h"
#include "lwp_kernels.h"
#include "lwp_plan.h"

using namespace lwp;

struct lwp_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;
    char* ws = nullptr;        // device workspace
    size_t ws_bytes = 0;
    char* pin = nullptr;       // pinned host staging (descriptor upload, small read-backs)
    size_t pin_bytes = 0;
    int32_t* split = nullptr;  // scratch + per-tile counters of split tiles (see minplus.hip)
    bool profiling = false;
    struct Timed { hipEvent_t a, b; int kind; int64_t work; bool keyed; };
    std::vector<Timed> timed;
    lwp_profile prof{};
};

namespace {

constexpr int64_t kI32Max = 2147483647LL, kI32Min = -2147483648LL;
constexpr int kMaxConfigs = 65536;

lwp_status fail(lwp_ctx* ctx, lwp_status s, const std::string& why) {
    if (ctx) ctx->err = why;
    return s;
}

#define LWP_HIP(ctx, call)                                                                     \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail(ctx, e_ == hipErrorOutOfMemory ? LWP_E_NOMEM : LWP_E_HIP,              \
                        std::string(#call) + ": " + hipGetErrorString(e_));                    \
    } while (0)

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

lwp_status ensure_workspace(lwp_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->ws_bytes) return LWP_OK;
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->ws) { LWP_HIP(ctx, hipFree(ctx->ws)); ctx->ws = nullptr; ctx->ws_bytes = 0; }
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, LWP_E_NOMEM, "device workspace of " + std::to_string(bytes) + " bytes: " + hipGetErrorString(e));
    }
    ctx->ws = static_cast<char*>(p);
    ctx->ws_bytes = bytes;
    return LWP_OK;
}

lwp_status ensure_pinned(lwp_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->pin_bytes) return LWP_OK;
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->pin) { LWP_HIP(ctx, hipHostFree(ctx->pin)); ctx->pin = nullptr; ctx->pin_bytes = 0; }
    void* p = nullptr;
    bytes = align_up(bytes, 1 << 16);
    hipError_t e = hipHostMalloc(&p, bytes, hipHostMallocDefault);
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(ctx, LWP_E_NOMEM, std::string("pinned host buffer: ") + hipGetErrorString(e)); }
    ctx->pin = static_cast<char*>(p);
    ctx->pin_bytes = bytes;
    return LWP_OK;
}

struct Range { int64_t lo, hi; };
bool fits(int64_t v) { return v >= kI32Min && v <= kI32Max; }

// Spread the packed-key arithmetic must represent for one product (see minplus.hip): re-based
// A + w, clamped just above the largest possible result where that is tighter, plus re-based B.
int64_t keyed_spread(Range rA, Range rw, Range rB) {
    const int64_t a_max = rA.hi + rw.hi - (rA.lo + rw.lo);
    const int64_t out_max = (rA.hi - rA.lo) + (rB.hi - rB.lo);
    return std::min(a_max, out_max + 1) + (rB.hi - rB.lo);
}

// Tile choice.  Measured on MI355X the 64 x 64 variant (4 waves per SIMD, 32-deep stages) matches or
// beats the 128 x 128 variant except for very large batches of short products (Cj < 512), where
// its four times as many workgroup start-ups show; it also quantises a launch four times finer.
int64_t large_tiles(int32_t Ci, int32_t Ck, int64_t batch) {
    return (int64_t)((Ci + kTileLarge - 1) / kTileLarge) * ((Ck + kTileLarge - 1) / kTileLarge) * batch;
}
bool want_small_tiles(int32_t Ci, int32_t Cj, int32_t Ck, int64_t batch) {
    return large_tiles(Ci, Ck, batch) < 2048 || Cj >= 512;
}

// Split tiles: a launch with few 64 x 64 tiles lets several workgroups share a tile, each with a
// part of the c range of at least two stages of 32 candidates.
// Measured: splitting pays while tiles x parts stays around 1024 workgroups (4 per compute unit).
int choose_kparts(int64_t tiles, int32_t Cj, bool small_tiles) {
    if (!small_tiles || tiles > kSplitMaxTiles) return 1;
    const int64_t nstages = (Cj + 31) / 32;
    int64_t k = std::min<int64_t>({kSplitMaxParts, kSplitMaxWorkgroups / tiles, nstages / 2});
    return k < 2 ? 1 : (int)k;
}

lwp_status ensure_split_buffers(lwp_ctx* ctx) {
    if (ctx->split) return LWP_OK;
    const size_t ints = (size_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart + kSplitMaxTiles;
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, ints * sizeof(int32_t));
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(ctx, LWP_E_NOMEM, std::string("split-tile scratch: ") + hipGetErrorString(e)); }
    ctx->split = static_cast<int32_t*>(p);
    // the counters start at zero and every launch leaves them at zero
    LWP_HIP(ctx, hipMemsetAsync(ctx->split + (size_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart, 0,
                                kSplitMaxTiles * sizeof(int32_t), ctx->stream));
    return LWP_OK;
}

void set_split(lwp_ctx* ctx, NodeArgs& a, int kparts) {
    a.kparts = kparts;
    a.scratch = kparts > 1 ? ctx->split : nullptr;
    a.counters = kparts > 1 ? ctx->split + (size_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart : nullptr;
}

// Timing of one launch when profiling is on.
struct ScopedTimer {
    lwp_ctx* ctx; size_t idx = (size_t)-1;
    ScopedTimer(lwp_ctx* c, int kind, int64_t work, bool keyed) : ctx(c) {
        if (!c->profiling) return;
        lwp_ctx::Timed t{nullptr, nullptr, kind, work, keyed};
        if (hipEventCreate(&t.a) != hipSuccess || hipEventCreate(&t.b) != hipSuccess) return;
        hipEventRecord(t.a, c->stream);
        c->timed.push_back(t);
        idx = c->timed.size() - 1;
    }
    ~ScopedTimer() { if (idx != (size_t)-1) hipEventRecord(ctx->timed[idx].b, ctx->stream); }
};

lwp_status drain_profile(lwp_ctx* ctx) {
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (auto& t : ctx->timed) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.a, t.b) == hipSuccess) {
            if (t.kind == 0) {
                ctx->prof.node_launches++; ctx->prof.node_cell_updates += t.work; ctx->prof.node_ms += ms;
                if (t.keyed) ctx->prof.keyed_launches++;
            } else {
                ctx->prof.edge_launches++; ctx->prof.edge_cells += t.work; ctx->prof.edge_ms += ms;
            }
        }
        hipEventDestroy(t.a); hipEventDestroy(t.b);
    }
    ctx->timed.clear();
    return LWP_OK;
}

lwp_status check_ctx(lwp_ctx* ctx) {
    if (!ctx) return LWP_E_INVAL;
    ctx->err.clear();
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail(ctx, LWP_E_HIP, std::string("hipSetDevice: ") + hipGetErrorString(e));
    return LWP_OK;
}

// ---- buffer planning of a whole search ---------------------------------------------------------
// Node l has Cn[l] configurations (Sec. 3: every layer has its own configuration set), so the
// table of an edge (i, j) is Cn[i] x Cn[j] and tables differ in size.  Tables produced by
// eliminations live in an arena; a region is released once the step that consumed it has been
// enqueued (launches of one stream run in order) and reused by later tables of the same size.
struct TableRef {
    bool is_slot;        // false: element offset into the caller's concatenated t_x; true: into the arena
    int64_t off;
    int32_t rows, cols;
    int64_t cells() const { return (int64_t)rows * cols; }
};

struct EdgeGroup { int32_t keep; std::vector<int32_t> others; int32_t round; };

struct Layout {
    std::vector<EdgeGroup> groups;            // edge eliminations grouped per (round, kept edge)
    std::vector<TableRef> node_A, node_B, node_out;   // per node step (in plan order)
    std::vector<int64_t> node_arg_off;        // element offset of the step's argmin table
    std::vector<std::vector<TableRef>> group_src;
    std::vector<TableRef> group_out;
    std::vector<TableRef> final_table;        // per residual pair
    std::vector<std::vector<TableRef>> comp_tables;   // per enumerated component, per edge
    std::vector<int64_t> node_off, tx_off;    // element offsets of w rows / input tables (+ total)
    int64_t slot_elems = 0, arg_elems = 0;
    bool uniform = true;                      // every node has the same number of configurations
};

constexpr int64_t kArenaAlign = 64;           // elements: regions start on 256-byte boundaries

// keep_inputs: tables consumed by node eliminations stay alive (the undo pass re-reads them).
Layout plan_buffers(const Plan& plan, int32_t n_nodes, int32_t n_edges, const int32_t* edges, const int32_t* Cn,
                    bool keep_inputs) {
    Layout L;
    L.node_off.resize((size_t)n_nodes + 1);
    L.tx_off.resize((size_t)n_edges + 1);
    L.node_off[0] = 0;
    for (int32_t v = 0; v < n_nodes; ++v) {
        L.node_off[v + 1] = L.node_off[v] + Cn[v];
        if (Cn[v] != Cn[0]) L.uniform = false;
    }
    std::vector<TableRef> cur(n_edges);
    L.tx_off[0] = 0;
    for (int32_t e = 0; e < n_edges; ++e) {
        cur[e] = {false, L.tx_off[e], Cn[edges[2 * e]], Cn[edges[2 * e + 1]]};
        L.tx_off[e + 1] = L.tx_off[e] + cur[e].cells();
    }
    std::map<int64_t, std::vector<int64_t>> free_regions;    // by size in elements
    auto take = [&](int32_t rows, int32_t cols) {
        const int64_t cells = (int64_t)rows * cols;
        auto& fl = free_regions[cells];
        int64_t off;
        if (!fl.empty()) { off = fl.back(); fl.pop_back(); }
        else { off = L.slot_elems; L.slot_elems += (cells + kArenaAlign - 1) / kArenaAlign * kArenaAlign; }
        return TableRef{true, off, rows, cols};
    };
    auto give_back = [&](const std::vector<TableRef>& rs) { for (auto& r : rs) free_regions[r.cells()].push_back(r.off); };
    size_t t = 0;
    const size_t n = plan.steps.size();
    while (t < n) {
        const int32_t round = plan.steps[t].round;
        // E-phase of this round
        std::vector<TableRef> release;
        while (t < n && plan.steps[t].round == round && plan.steps[t].kind == 1) {
            EdgeGroup g{plan.steps[t].e1, {}, round};
            while (t < n && plan.steps[t].round == round && plan.steps[t].kind == 1 && plan.steps[t].e1 == g.keep) {
                g.others.push_back(plan.steps[t].e2);
                ++t;
            }
            std::vector<TableRef> src{cur[g.keep]};
            for (int32_t o : g.others) { src.push_back(cur[o]); if (cur[o].is_slot) release.push_back(cur[o]); }
            const TableRef out = cur[g.keep].is_slot ? cur[g.keep] : take(cur[g.keep].rows, cur[g.keep].cols);   // in place when possible
            cur[g.keep] = out;
            L.groups.push_back(g); L.group_src.push_back(src); L.group_out.push_back(out);
        }
        give_back(release);
        release.clear();
        // N-phase of this round
        while (t < n && plan.steps[t].round == round && plan.steps[t].kind == 0) {
            const lwp_step& st = plan.steps[t];
            const TableRef A = cur[st.e1], B = cur[st.e2];
            L.node_A.push_back(A); L.node_B.push_back(B);
            if (!keep_inputs && A.is_slot) release.push_back(A);
            if (!keep_inputs && B.is_slot) release.push_back(B);
            const TableRef out = take(A.rows, B.cols);
            L.node_out.push_back(out);
            L.node_arg_off.push_back(L.arg_elems);
            L.arg_elems += (out.cells() + kArenaAlign - 1) / kArenaAlign * kArenaAlign;
            cur[st.e1] = out;
            ++t;
        }
        give_back(release);
    }
    for (auto& p : plan.pairs) L.final_table.push_back(cur[p.edge]);
    for (auto& c : plan.comps) {
        std::vector<TableRef> tabs;
        for (int32_t e : c.edges) tabs.push_back(cur[e]);
        L.comp_tables.push_back(tabs);
    }
    return L;
}

// Device workspace of one search.  The descriptor block is mirrored in pinned host memory and
// uploaded with a single copy; `head` = {overflow flag, pad, [min,max] per table} is read back with
// a single copy.  Tables with a range: input edges, w of every node, output of every node
// elimination, output of every edge-sum group.
struct WsLayout {
    size_t w, head, keys, result, args, slots, total;
    size_t desc, desc_bytes;                                   // descriptor block
    size_t offs, offs_bytes;                                   // row / table offsets, at the start of the block
    size_t node_desc, edge_desc, src_ptrs, pair_desc, singles, undo, comps, tile_begin;   // offsets inside the block
    int32_t n_ranges;
};

WsLayout layout_workspace(const Plan& plan, const Layout& L, int32_t n_nodes, int32_t n_edges, bool stored_argmin) {
    WsLayout o{};
    size_t off = 0;
    auto put = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
    size_t n_src = 0;
    for (auto& g : L.group_src) n_src += g.size();
    o.n_ranges = n_edges + n_nodes + plan.n_node_steps + (int32_t)L.groups.size();
    o.w = put((size_t)L.node_off[n_nodes] * sizeof(int32_t));
    o.head = put((2 + 2 * (size_t)o.n_ranges) * sizeof(int32_t));
    o.keys = put(std::max<size_t>(1, plan.pairs.size() + plan.singles.size() + plan.comps.size()) * sizeof(unsigned long long));
    o.result = put((3 + (size_t)n_nodes) * sizeof(int32_t));
    o.offs_bytes = L.uniform ? 0 : ((size_t)n_nodes + 1 + (size_t)n_edges + 1) * sizeof(int64_t);
    {
        size_t b = 0;
        auto sub = [&](size_t bytes) { size_t at = b; b = align_up(b + bytes, 16); return at; };
        o.offs = sub(o.offs_bytes);      // first, so that it can be uploaded ahead of the rest
        o.node_desc = sub((size_t)plan.n_node_steps * sizeof(NodeDesc));
        o.edge_desc = sub(L.groups.size() * sizeof(EdgeDesc));
        o.src_ptrs = sub(n_src * sizeof(void*));
        o.pair_desc = sub(plan.pairs.size() * sizeof(PairDesc));
        o.singles = sub(plan.singles.size() * sizeof(SingleDesc));
        o.undo = sub((size_t)plan.n_node_steps * sizeof(UndoDesc));
        o.comps = sub(plan.comps.size() * sizeof(CompDesc));
        o.tile_begin = sub((2 * (size_t)plan.n_node_steps + 2) * sizeof(int32_t));   // launches of mixed shapes
        o.desc_bytes = std::max<size_t>(b, 16);
    }
    o.desc = put(o.desc_bytes);
    o.args = put(stored_argmin ? (size_t)L.arg_elems * sizeof(int32_t) : 0);
    o.slots = put((size_t)L.slot_elems * sizeof(int32_t));
    o.total = off;
    return o;
}

// A residual component is enumerated outright; its flat strategy index must fit 32 bits.
bool components_enumerable(const Plan& plan, const int32_t* Cn) {
    for (auto& c : plan.comps) {
        unsigned long long n = 1;
        for (int32_t v : c.nodes) {
            n *= (unsigned long long)Cn[v];
            if (n > (1ull << 32)) return false;
        }
    }
    return true;
}

bool counts_valid(int32_t n_nodes, const int32_t* Cn) {
    if (!Cn) return false;
    for (int32_t v = 0; v < n_nodes; ++v)
        if (Cn[v] < 1 || Cn[v] > kMaxConfigs) return false;
    return true;
}

}  // namespace

namespace lwp {
hipStream_t ctx_stream(lwp_ctx* ctx) { return ctx->stream; }
lwp_status ctx_enter(lwp_ctx* ctx) { return check_ctx(ctx); }
lwp_status ctx_fail(lwp_ctx* ctx, lwp_status s, const char* why) { return fail(ctx, s, why); }
}  // namespace lwp

// ================================================================================================
extern "C" {

const char* lwp_status_string(lwp_status s) {
    switch (s) {
        case LWP_OK: return "ok";
        case LWP_E_INVAL: return "invalid argument";
        case LWP_E_GRAPH: return "invalid graph";
        case LWP_E_NOT_REDUCIBLE: return "graph not reducible";
        case LWP_E_OVERFLOW: return "int32 overflow possible";
        case LWP_E_NOMEM: return "out of memory";
        case LWP_E_HIP: return "HIP error";
    }
    return "unknown status";
}

lwp_status lwp_create(lwp_ctx** out, int device, void* hip_stream) {
    if (!out) return LWP_E_INVAL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return LWP_E_HIP;
    if (hipSetDevice(device) != hipSuccess) return LWP_E_HIP;
    lwp_ctx* c = new (std::nothrow) lwp_ctx();
    if (!c) return LWP_E_NOMEM;
    c->device = device;
    c->stream = static_cast<hipStream_t>(hip_stream);
    *out = c;
    return LWP_OK;
}

void lwp_destroy(lwp_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& t : ctx->timed) { hipEventDestroy(t.a); hipEventDestroy(t.b); }
    if (ctx->ws) (void)hipFree(ctx->ws);
    if (ctx->pin) (void)hipHostFree(ctx->pin);
    if (ctx->split) (void)hipFree(ctx->split);
    delete ctx;
}

const char* lwp_last_error(const lwp_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

lwp_status lwp_synchronize(lwp_ctx* ctx) {
    if (lwp_status s = check_ctx(ctx)) return s;
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return LWP_OK;
}

lwp_status lwp_profile_enable(lwp_ctx* ctx, int32_t on) {
    if (lwp_status s = check_ctx(ctx)) return s;
    ctx->profiling = on != 0;
    return LWP_OK;
}

lwp_status lwp_profile_reset(lwp_ctx* ctx) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (lwp_status s = drain_profile(ctx)) return s;
    ctx->prof = lwp_profile{};
    return LWP_OK;
}

lwp_status lwp_profile_read(lwp_ctx* ctx, lwp_profile* out) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (!out) return fail(ctx, LWP_E_INVAL, "null output");
    if (lwp_status s = drain_profile(ctx)) return s;
    *out = ctx->prof;
    return LWP_OK;
}

// ---- Eq. 2 -------------------------------------------------------------------------------------
lwp_status lwp_eliminate_node(lwp_ctx* ctx, int32_t batch, int32_t Ci, int32_t Cj, int32_t Ck,
                              const int32_t* d_A, const int32_t* d_w, const int32_t* d_B,
                              int32_t* d_out, int32_t* d_argmin) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (batch < 1 || Ci < 1 || Cj < 1 || Ck < 1) return fail(ctx, LWP_E_INVAL, "sizes must be positive");
    if (Cj > kMaxConfigs) return fail(ctx, LWP_E_INVAL, "Cj exceeds 65536");
    if (!d_A || !d_w || !d_B || !d_out) return fail(ctx, LWP_E_INVAL, "null table pointer");
    if (((uintptr_t)d_A | (uintptr_t)d_w | (uintptr_t)d_B | (uintptr_t)d_out | (uintptr_t)d_argmin) & 3)
        return fail(ctx, LWP_E_INVAL, "table pointer not 4-byte aligned");
    const bool prefer_small = want_small_tiles(Ci, Cj, Ck, batch);
    if ((int64_t)((Ci + kTileSmall - 1) / kTileSmall) * ((Ck + kTileSmall - 1) / kTileSmall) * batch > 0x7fffffffLL)
        return fail(ctx, LWP_E_INVAL, "too many output tiles");

    // value ranges of A, w, B over the whole batch
    if (lwp_status s = ensure_workspace(ctx, 4096)) return s;
    if (lwp_status s = ensure_pinned(ctx, 4096)) return s;
    int32_t* d_stats = reinterpret_cast<int32_t*>(ctx->ws);
    LWP_HIP(ctx, launch_init_workspace(d_stats, 3, nullptr, nullptr, 0, ctx->stream));
    LWP_HIP(ctx, launch_ranges(d_A, 1, (int64_t)batch * Ci * Cj, d_stats, ctx->stream));
    LWP_HIP(ctx, launch_ranges(d_w, 1, (int64_t)batch * Cj, d_stats + 2, ctx->stream));
    LWP_HIP(ctx, launch_ranges(d_B, 1, (int64_t)batch * Cj * Ck, d_stats + 4, ctx->stream));
    int32_t* st = reinterpret_cast<int32_t*>(ctx->pin);
    LWP_HIP(ctx, hipMemcpyAsync(st, d_stats, 6 * sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const Range rA{st[0], st[1]}, rw{st[2], st[3]}, rB{st[4], st[5]};
    if (!fits(rA.lo + rw.lo + rB.lo) || !fits(rA.hi + rw.hi + rB.hi) || !fits(rA.lo + rw.lo) || !fits(rA.hi + rw.hi))
        return fail(ctx, LWP_E_OVERFLOW, "A + w + B may leave int32");

    NodeArgs a{};
    a.descs = nullptr;
    a.base.A = d_A; a.base.w = d_w; a.base.B = d_B; a.base.out = d_out; a.base.arg = d_argmin;
    a.base.loA = (int32_t)rA.lo; a.base.hiA = (int32_t)rA.hi; a.base.loW = (int32_t)rw.lo; a.base.hiW = (int32_t)rw.hi;
    a.base.loB = (int32_t)rB.lo; a.base.hiB = (int32_t)rB.hi;
    const int64_t spread = keyed_spread(rA, rw, rB);
    // one more key bit on large tiles, worth it only if they still fill the chip; without an argmin
    // output the value-only variant runs, which has no range condition at all
    const bool value_only = (d_argmin == nullptr);
    const bool keyed = !value_only && (spread <= kKeyedMaxSpreadSmall ||
                       (spread <= kKeyedMaxSpreadLarge && (!prefer_small || large_tiles(Ci, Ck, batch) >= 512)));
    const bool small = prefer_small && (value_only || spread <= kKeyedMaxSpreadSmall || !keyed);
    const int tile = small ? kTileSmall : kTileLarge;
    const int64_t tilesM = (Ci + tile - 1) / tile, tilesN = (Ck + tile - 1) / tile;
    a.sA = (int64_t)Ci * Cj; a.sw = Cj; a.sB = (int64_t)Cj * Ck; a.sO = (int64_t)Ci * Ck;
    a.Ci = Ci; a.Cj = Cj; a.Ck = Ck; a.batch = batch;
    a.tilesM = (int32_t)tilesM; a.tilesN = (int32_t)tilesN;
    {
        ScopedTimer tm(ctx, 0, (int64_t)batch * Ci * Cj * Ck, keyed);
        const int kparts = choose_kparts(tilesM * tilesN * batch, Cj, small);
        if (kparts > 1) { if (lwp_status s = ensure_split_buffers(ctx)) return s; }
        set_split(ctx, a, kparts);
        LWP_HIP(ctx, launch_minplus(a, value_only ? kModeValue : (keyed ? kModeKeyed : kModePlain), small, ctx->stream));
    }
    return LWP_OK;
}

// ---- Eq. 3 -------------------------------------------------------------------------------------
lwp_status lwp_eliminate_edge(lwp_ctx* ctx, int32_t batch, int32_t Ci, int32_t Cj,
                              const int32_t* d_e1, const int32_t* d_e2, int32_t* d_out) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (batch < 1 || Ci < 1 || Cj < 1) return fail(ctx, LWP_E_INVAL, "sizes must be positive");
    if (!d_e1 || !d_e2 || !d_out) return fail(ctx, LWP_E_INVAL, "null table pointer");
    if (((uintptr_t)d_e1 | (uintptr_t)d_e2 | (uintptr_t)d_out) & 3)
        return fail(ctx, LWP_E_INVAL, "table pointer not 4-byte aligned");
    const int64_t cells = (int64_t)batch * Ci * Cj;
    ScopedTimer tm(ctx, 1, cells, false);
    LWP_HIP(ctx, launch_edge_sum_pair(d_e1, d_e2, d_out, cells, ctx->stream));
    return LWP_OK;
}

// ---- Alg. 1 ------------------------------------------------------------------------------------
lwp_status lwp_plan_graph(int32_t n_nodes, int32_t n_edges, const int32_t* edges, int32_t schedule,
                          lwp_step* steps, int32_t* n_steps, int32_t* n_rounds, int32_t* n_residual_nodes) {
    Plan plan;
    std::string err;
    lwp_status s = make_plan(n_nodes, n_edges, edges, schedule, plan, err);
    if (n_steps) *n_steps = (int32_t)plan.steps.size();
    if (n_rounds) *n_rounds = plan.n_rounds;
    if (s != LWP_OK) return s;
    if (steps && !plan.steps.empty()) std::memcpy(steps, plan.steps.data(), plan.steps.size() * sizeof(lwp_step));
    if (n_residual_nodes) {
        size_t k = 2 * plan.pairs.size() + plan.singles.size();
        for (auto& c : plan.comps) k += c.nodes.size();
        *n_residual_nodes = (int32_t)k;
    }
    return LWP_OK;
}

size_t lwp_search_workspace_bytes(int32_t n_nodes, int32_t n_edges, const int32_t* edges, int32_t C,
                                  int32_t schedule) {
    return lwp_search_workspace_bytes_ex(n_nodes, n_edges, edges, C, schedule, LWP_UNDO_STORED);
}

size_t lwp_search_workspace_bytes_ex(int32_t n_nodes, int32_t n_edges, const int32_t* edges, int32_t C,
                                     int32_t schedule, int32_t undo) {
    if (n_nodes < 1) return 0;
    const std::vector<int32_t> Cn((size_t)n_nodes, C);
    return lwp_search_workspace_bytes_ragged(n_nodes, n_edges, edges, Cn.data(), schedule, undo);
}

size_t lwp_search_workspace_bytes_ragged(int32_t n_nodes, int32_t n_edges, const int32_t* edges,
                                         const int32_t* C_node, int32_t schedule, int32_t undo) {
    if (n_nodes < 1 || !counts_valid(n_nodes, C_node) || (undo != LWP_UNDO_STORED && undo != LWP_UNDO_RECOMPUTE)) return 0;
    Plan plan;
    std::string err;
    if (make_plan(n_nodes, n_edges, edges, schedule, plan, err) != LWP_OK) return 0;
    if (!components_enumerable(plan, C_node)) return 0;
    Layout L = plan_buffers(plan, n_nodes, n_edges, edges, C_node, undo == LWP_UNDO_RECOMPUTE);
    return layout_workspace(plan, L, n_nodes, n_edges, undo == LWP_UNDO_STORED).total;
}

lwp_status lwp_search_graph(lwp_ctx* ctx, int32_t n_nodes, int32_t n_edges, const int32_t* edges,
                            int32_t C, const int32_t* d_tc, const int32_t* d_ts, const int32_t* d_tx,
                            int32_t schedule, int32_t* out_cost, int32_t* out_strategy) {
    return lwp_search_graph_ex(ctx, n_nodes, n_edges, edges, C, d_tc, d_ts, d_tx, schedule, LWP_UNDO_STORED, out_cost,
                               out_strategy);
}

lwp_status lwp_search_graph_ex(lwp_ctx* ctx, int32_t n_nodes, int32_t n_edges, const int32_t* edges,
                               int32_t C, const int32_t* d_tc, const int32_t* d_ts, const int32_t* d_tx,
                               int32_t schedule, int32_t undo, int32_t* out_cost, int32_t* out_strategy) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (C < 1 || C > kMaxConfigs) return fail(ctx, LWP_E_INVAL, "C must be in [1, 65536]");
    if (n_nodes < 1) return fail(ctx, LWP_E_GRAPH, "n_nodes must be >= 1");
    const std::vector<int32_t> Cn((size_t)n_nodes, C);
    return lwp_search_graph_ragged(ctx, n_nodes, n_edges, edges, Cn.data(), d_tc, d_ts, d_tx, schedule, undo, out_cost,
                                   out_strategy);
}

lwp_status lwp_search_graph_ragged(lwp_ctx* ctx, int32_t n_nodes, int32_t n_edges, const int32_t* edges,
                                   const int32_t* Cn, const int32_t* d_tc, const int32_t* d_ts,
                                   const int32_t* d_tx, int32_t schedule, int32_t undo, int32_t* out_cost,
                                   int32_t* out_strategy) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (undo != LWP_UNDO_STORED && undo != LWP_UNDO_RECOMPUTE) return fail(ctx, LWP_E_INVAL, "unknown undo mode");
    const bool stored = (undo == LWP_UNDO_STORED);
    if (n_nodes < 1) return fail(ctx, LWP_E_GRAPH, "n_nodes must be >= 1");
    if (!counts_valid(n_nodes, Cn)) return fail(ctx, LWP_E_INVAL, "every configuration count must be in [1, 65536]");
    if (!d_tc || !d_ts || (n_edges > 0 && !d_tx) || !out_cost || !out_strategy)
        return fail(ctx, LWP_E_INVAL, "null pointer");
    if (((uintptr_t)d_tc | (uintptr_t)d_ts | (uintptr_t)d_tx) & 3)
        return fail(ctx, LWP_E_INVAL, "table pointer not 4-byte aligned");
    Plan plan;
    {
        std::string err;
        lwp_status s = make_plan(n_nodes, n_edges, edges, schedule, plan, err);
        if (s != LWP_OK) return fail(ctx, s, err);
    }
    if (!components_enumerable(plan, Cn))
        return fail(ctx, LWP_E_NOT_REDUCIBLE, "a residual component has more than 2^32 strategies to enumerate");
    const Layout L = plan_buffers(plan, n_nodes, n_edges, edges, Cn, !stored);
    const WsLayout W = layout_workspace(plan, L, n_nodes, n_edges, stored);
    if (lwp_status s = ensure_workspace(ctx, W.total)) return s;
    const size_t head_in_bytes = (2 + 2 * (size_t)(n_edges + n_nodes)) * sizeof(int32_t);
    const size_t pin_head = 0, pin_desc = align_up(head_in_bytes, 256), pin_result = pin_desc + align_up(W.desc_bytes, 256);
    if (lwp_status s = ensure_pinned(ctx, pin_result + (3 + (size_t)n_nodes) * sizeof(int32_t))) return s;
    char* ws = ctx->ws;
    hipStream_t st = ctx->stream;
    int32_t* d_w = reinterpret_cast<int32_t*>(ws + W.w);
    int32_t* d_head = reinterpret_cast<int32_t*>(ws + W.head);
    int32_t* d_stats = d_head + 2;
    int32_t* d_args = reinterpret_cast<int32_t*>(ws + W.args);
    int32_t* d_slots = reinterpret_cast<int32_t*>(ws + W.slots);
    unsigned long long* d_keys = reinterpret_cast<unsigned long long*>(ws + W.keys);
    int32_t* d_result = reinterpret_cast<int32_t*>(ws + W.result);
    const int32_t n_comp = (int32_t)(plan.pairs.size() + plan.singles.size() + plan.comps.size());
    auto table_ptr = [&](const TableRef& r) -> const int32_t* { return (r.is_slot ? d_slots : d_tx) + r.off; };
    auto slot_ptr = [&](const TableRef& r) -> int32_t* { return d_slots + r.off; };
    auto w_ptr = [&](int32_t v) -> const int32_t* { return d_w + L.node_off[v]; };
    // index of the range pair of: input edge e | w of node v | output of node step | output of group
    const int32_t rng_w0 = n_edges, rng_node0 = n_edges + n_nodes, rng_group0 = rng_node0 + plan.n_node_steps;

    // 1. w = t_c + t_s with its ranges, and the range of every input table
    int32_t* d_flag = d_head;      // set by any kernel that finds a sum outside int32
    char* hb = ctx->pin + pin_desc;
    char* db = ws + W.desc;
    if (!L.uniform) {              // rows and tables of different sizes: the kernels need their offsets
        int64_t* h_offs = reinterpret_cast<int64_t*>(hb + W.offs);
        std::memcpy(h_offs, L.node_off.data(), ((size_t)n_nodes + 1) * sizeof(int64_t));
        std::memcpy(h_offs + n_nodes + 1, L.tx_off.data(), ((size_t)n_edges + 1) * sizeof(int64_t));
    }
    auto measure_inputs = [&]() -> lwp_status {
        if (L.uniform) {
            LWP_HIP(ctx, launch_prepare_search(d_tc, d_ts, d_w, n_nodes, Cn[0], nullptr, d_stats, W.n_ranges, rng_w0, d_keys, n_comp, d_flag, st));
            LWP_HIP(ctx, launch_ranges(d_tx, n_edges, (int64_t)Cn[0] * Cn[0], d_stats, st));
        } else {
            const int64_t* d_offs = reinterpret_cast<const int64_t*>(db + W.offs);
            int64_t max_cells = 1;
            for (int32_t e = 0; e < n_edges; ++e) max_cells = std::max(max_cells, L.tx_off[e + 1] - L.tx_off[e]);
            LWP_HIP(ctx, launch_prepare_search(d_tc, d_ts, d_w, n_nodes, 0, d_offs, d_stats, W.n_ranges, rng_w0, d_keys, n_comp, d_flag, st));
            LWP_HIP(ctx, launch_ranges_var(d_tx, d_offs + n_nodes + 1, n_edges, max_cells, d_stats, st));
        }
        return LWP_OK;
    };
    // Stored argmin tables need a kernel variant chosen from value ranges, so the ranges of the inputs
    // are read back (the one mid-search synchronisation) before the descriptors are written.  With
    // recomputed undo every elimination is value-only (no range condition) and overflow is judged on
    // the device from measured ranges: nothing is read back, the host assumes full int32 ranges,
    // writes the descriptors first and uploads them together with the offsets in one copy.
    int32_t* h_head = reinterpret_cast<int32_t*>(ctx->pin + pin_head);
    int32_t* stats = h_head + 2;
    if (stored) {
        if (!L.uniform) LWP_HIP(ctx, hipMemcpyAsync(db + W.offs, hb + W.offs, W.offs_bytes, hipMemcpyHostToDevice, st));
        if (lwp_status s = measure_inputs()) return s;
        LWP_HIP(ctx, hipMemcpyAsync(h_head, d_head, head_in_bytes, hipMemcpyDeviceToHost, st));
        LWP_HIP(ctx, hipStreamSynchronize(st));
        for (int32_t v = 0; v < n_nodes; ++v)
            if (stats[2 * (rng_w0 + v)] > stats[2 * (rng_w0 + v) + 1]) return fail(ctx, LWP_E_OVERFLOW, "t_c + t_s leaves int32");
    } else {
        for (int32_t t2 = 0; t2 < n_edges + n_nodes; ++t2) { stats[2 * t2] = (int32_t)kI32Min; stats[2 * t2 + 1] = (int32_t)kI32Max; }
    }

    // 2. propagate ranges through the plan: every sum any kernel forms must fit int32.  Descriptors
    //    are written straight into the pinned mirror of the device block.
    NodeDesc* nd = reinterpret_cast<NodeDesc*>(hb + W.node_desc);
    EdgeDesc* ed = reinterpret_cast<EdgeDesc*>(hb + W.edge_desc);
    const int32_t** src_ptrs = reinterpret_cast<const int32_t**>(hb + W.src_ptrs);
    PairDesc* pd = reinterpret_cast<PairDesc*>(hb + W.pair_desc);
    SingleDesc* sd = reinterpret_cast<SingleDesc*>(hb + W.singles);
    UndoDesc* ud = reinterpret_cast<UndoDesc*>(hb + W.undo);
    CompDesc* cd = reinterpret_cast<CompDesc*>(hb + W.comps);
    int32_t* tbeg = reinterpret_cast<int32_t*>(hb + W.tile_begin);
    size_t n_tbeg = 0;
    const NodeDesc* d_nd = reinterpret_cast<const NodeDesc*>(db + W.node_desc);
    const EdgeDesc* d_ed = reinterpret_cast<const EdgeDesc*>(db + W.edge_desc);
    const int32_t* const* d_src = reinterpret_cast<const int32_t* const*>(db + W.src_ptrs);
    const PairDesc* d_pd = reinterpret_cast<const PairDesc*>(db + W.pair_desc);
    const SingleDesc* d_sd = reinterpret_cast<const SingleDesc*>(db + W.singles);
    const UndoDesc* d_ud = reinterpret_cast<const UndoDesc*>(db + W.undo);
    const CompDesc* d_cd = reinterpret_cast<const CompDesc*>(db + W.comps);
    const int32_t* d_tbeg = reinterpret_cast<const int32_t*>(db + W.tile_begin);

    std::vector<Range> er(n_edges), wr(n_nodes);
    std::vector<int32_t> erng(n_edges);          // range-pair index of the edge's current table
    for (int32_t e = 0; e < n_edges; ++e) { er[e] = {stats[2 * e], stats[2 * e + 1]}; erng[e] = e; }
    for (int32_t v = 0; v < n_nodes; ++v) wr[v] = {stats[2 * (rng_w0 + v)], stats[2 * (rng_w0 + v) + 1]};
    // Node eliminations of one round are independent; those of equal kernel variant share a
    // launch if they agree in shape (Ci, Cj, Ck) or run on 64 x 64 tiles (a launch of mixed shapes),
    // so the descriptors of a round are ordered by (variant, shape).
    struct NodeWork { NodeDesc d; int64_t spread; int32_t Ci, Cj, Ck; int variant; };
    struct NodeLaunch {
        size_t first, count; int32_t Ci, Cj, Ck; int variant;
        int64_t tile_begin;      // index into the tile_begin block for mixed shapes, else -1
        int32_t total_tiles, split_Cj; int64_t updates;   // split_Cj: the Cj that decides how tiles are split
    };
    struct RoundWork { size_t g0, g1; int64_t edge_cells, edge_max_cells; std::vector<NodeLaunch> launches; };
    std::vector<RoundWork> rounds;
    // The propagated bounds are worst cases and grow along a chain although the minima do not.
    // Where they cannot prove that a step stays inside int32 the step is not refused: it runs on a
    // variant without range conditions and every kernel checks the tables' measured ranges (or
    // the sums themselves) on the device; the flag they set is read back with the result.
    auto sat = [](Range r) { return Range{std::max(r.lo, kI32Min), std::min(r.hi, kI32Max)}; };
    {
        size_t ni = 0, gi = 0, nsrc = 0, t = 0;
        const size_t n = plan.steps.size();
        std::vector<NodeWork> work;
        std::vector<size_t> order;
        while (t < n) {
            const int32_t round = plan.steps[t].round;
            RoundWork rw_{gi, gi, 0, 1, {}};
            while (t < n && plan.steps[t].round == round && plan.steps[t].kind == 1) {
                // one group = all steps adding into the same kept edge
                const auto& g = L.groups[gi];
                Range r = er[g.keep];
                for (int32_t o : g.others) r = {r.lo + er[o].lo, r.hi + er[o].hi};
                er[g.keep] = sat(r);
                erng[g.keep] = rng_group0 + (int32_t)gi;
                ed[gi].out = slot_ptr(L.group_out[gi]);
                ed[gi].rngOut = d_stats + 2 * (int64_t)erng[g.keep];
                ed[gi].flag = d_flag;
                ed[gi].cells = L.group_out[gi].cells();
                ed[gi].first_src = (int32_t)nsrc;
                ed[gi].n_src = (int32_t)L.group_src[gi].size();
                for (auto& r2 : L.group_src[gi]) src_ptrs[nsrc++] = table_ptr(r2);
                rw_.edge_cells += ed[gi].cells;
                rw_.edge_max_cells = std::max(rw_.edge_max_cells, ed[gi].cells);
                t += g.others.size();
                ++gi;
            }
            rw_.g1 = gi;
            const size_t n0 = ni;
            work.clear();
            while (t < n && plan.steps[t].round == round && plan.steps[t].kind == 0) {
                const lwp_step& s = plan.steps[t];
                const Range rA = er[s.e1], rw = wr[s.j], rB = er[s.e2];
                const bool proven = fits(rA.lo + rw.lo) && fits(rA.hi + rw.hi) && fits(rA.lo + rw.lo + rB.lo) && fits(rA.hi + rw.hi + rB.hi);
                const TableRef &tA = L.node_A[ni], &tB = L.node_B[ni], &tO = L.node_out[ni];
                NodeWork nw{};
                NodeDesc& d = nw.d;
                d.flag = d_flag;
                d.A = table_ptr(tA); d.w = w_ptr(s.j); d.B = table_ptr(tB);
                d.out = slot_ptr(tO);
                d.arg = stored ? d_args + L.node_arg_off[ni] : nullptr;
                d.loA = (int32_t)rA.lo; d.hiA = (int32_t)rA.hi; d.loW = (int32_t)rw.lo; d.hiW = (int32_t)rw.hi;
                d.loB = (int32_t)rB.lo; d.hiB = (int32_t)rB.hi;
                d.rngA = d_stats + 2 * (int64_t)erng[s.e1];
                d.rngB = d_stats + 2 * (int64_t)erng[s.e2];
                d.rngW = d_stats + 2 * (int64_t)(rng_w0 + s.j);
                d.rngOut = d_stats + 2 * (int64_t)(rng_node0 + (int32_t)ni);
                nw.spread = proven ? keyed_spread(rA, rw, rB) : (int64_t)1 << 62;   // unproven: no packed keys
                nw.Ci = tA.rows; nw.Cj = tA.cols; nw.Ck = tB.cols;
                d.Ci = nw.Ci; d.Cj = nw.Cj; d.Ck = nw.Ck;
                work.push_back(nw);
                ud[ni] = {d.arg, d.A, d.w, d.B, s.j, s.i, s.k, s.round, nw.Cj, nw.Ck, (int32_t)n0, 0};
                // any fixed c bounds the minimum from above; take the c with the smallest w
                er[s.e1] = sat({rA.lo + rw.lo + rB.lo, rA.hi + rw.lo + rB.hi});
                erng[s.e1] = rng_node0 + (int32_t)ni;
                ++ni; ++t;
            }
            // kernel variant per product: packed keys on the preferred tile size if the spread
            // allows, else packed keys on 128 x 128 tiles (one more bit), else the plain variant;
            // 0 keyed small, 1 keyed large, 2 plain small, 3 plain large, 4 value small, 5 value large
            auto shape_of = [](const NodeWork& a) { return std::make_tuple(a.Ci, a.Cj, a.Ck); };
            std::map<std::tuple<int32_t, int32_t, int32_t>, int64_t> shape_count;
            for (const NodeWork& x : work) ++shape_count[shape_of(x)];
            for (NodeWork& x : work) {
                const int64_t same = shape_count[shape_of(x)];
                const bool prefer_small = want_small_tiles(x.Ci, x.Cj, x.Ck, same);
                const bool large_fills_chip = large_tiles(x.Ci, x.Ck, same) >= 512;
                if (!stored) x.variant = prefer_small ? 4 : 5;     // value-only: no range condition
                else if (x.spread <= (prefer_small ? kKeyedMaxSpreadSmall : kKeyedMaxSpreadLarge)) x.variant = prefer_small ? 0 : 1;
                else if (x.spread <= kKeyedMaxSpreadLarge && large_fills_chip) x.variant = 1;
                else x.variant = prefer_small ? 2 : 3;
            }
            order.resize(work.size());
            for (size_t q = 0; q < order.size(); ++q) order[q] = q;
            std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) {
                return std::make_pair(work[a].variant, shape_of(work[a])) < std::make_pair(work[b].variant, shape_of(work[b]));
            });
            for (size_t a = 0; a < order.size();) {
                const int v = work[order[a]].variant;
                size_t b = a;
                while (b < order.size() && work[order[b]].variant == v) ++b;
                const bool small = (v == 0 || v == 2 || v == 4);
                const bool one_shape = shape_of(work[order[a]]) == shape_of(work[order[b - 1]]);
                if (small && !one_shape) {
                    // one launch over all shapes: product q owns tiles [tile_begin[q], tile_begin[q+1])
                    NodeLaunch nl{n0 + a, b - a, 0, 0, 0, v, (int64_t)n_tbeg, 0, 0, 0};
                    int64_t tiles = 0;
                    for (size_t q = a; q < b; ++q) {
                        NodeWork& x = work[order[q]];
                        tbeg[n_tbeg++] = (int32_t)tiles;
                        tiles += (int64_t)((x.Ci + kTileSmall - 1) / kTileSmall) * ((x.Ck + kTileSmall - 1) / kTileSmall);
                        nl.split_Cj = std::max(nl.split_Cj, x.Cj);
                        nl.updates += (int64_t)x.Ci * x.Cj * x.Ck;
                    }
                    tbeg[n_tbeg++] = (int32_t)tiles;
                    if (tiles > INT32_MAX) return fail(ctx, LWP_E_INVAL, "too many tiles in one round");
                    nl.total_tiles = (int32_t)tiles;
                    rw_.launches.push_back(nl);
                } else {
                    for (size_t q = a; q < b;) {
                        size_t e = q;
                        while (e < b && shape_of(work[order[e]]) == shape_of(work[order[q]])) ++e;
                        const NodeWork& x = work[order[q]];
                        rw_.launches.push_back({n0 + q, e - q, x.Ci, x.Cj, x.Ck, v, -1, 0, x.Cj,
                                                (int64_t)(e - q) * x.Ci * x.Cj * x.Ck});
                        q = e;
                    }
                }
                a = b;
            }
            for (size_t q = 0; q < order.size(); ++q) nd[n0 + q] = work[order[q]].d;
            rounds.push_back(std::move(rw_));
        }
    }
    int32_t pair_max_rows = 1, single_max_c = 1;
    for (size_t q = 0; q < plan.pairs.size(); ++q) {
        const auto& pr = plan.pairs[q];
        pd[q] = {table_ptr(L.final_table[q]), w_ptr(pr.src), w_ptr(pr.dst), pr.src, pr.dst, Cn[pr.src], Cn[pr.dst]};
        pair_max_rows = std::max(pair_max_rows, Cn[pr.src]);
    }
    for (size_t q = 0; q < plan.singles.size(); ++q) {
        const int32_t v = plan.singles[q];
        sd[q] = {w_ptr(v), v, Cn[v]};
        single_max_c = std::max(single_max_c, Cn[v]);
    }
    std::vector<unsigned long long> comp_prefix(plan.comps.size());
    for (size_t q = 0; q < plan.comps.size(); ++q) {
        const auto& c = plan.comps[q];
        CompDesc d{};
        d.K = (int32_t)c.nodes.size(); d.n_edges = (int32_t)c.edges.size();
        unsigned long long prefix = 1;
        for (int x = 0; x < d.K; ++x) {
            d.node[x] = c.nodes[x]; d.Cn[x] = Cn[c.nodes[x]]; d.w[x] = w_ptr(c.nodes[x]);
            if (x + 1 < d.K) prefix *= (unsigned long long)d.Cn[x];
        }
        comp_prefix[q] = prefix;
        for (int x = 0; x < d.n_edges; ++x) {
            d.tab[x] = table_ptr(L.comp_tables[q][x]);
            d.src_pos[x] = (int8_t)(std::find(c.nodes.begin(), c.nodes.end(), c.esrc[x]) - c.nodes.begin());
            d.dst_pos[x] = (int8_t)(std::find(c.nodes.begin(), c.nodes.end(), c.edst[x]) - c.nodes.begin());
        }
        cd[q] = d;
    }

    // 3. descriptors to the device: one copy
    LWP_HIP(ctx, hipMemcpyAsync(db, hb, W.desc_bytes, hipMemcpyHostToDevice, st));
    if (!stored) { if (lwp_status s = measure_inputs()) return s; }

    // 4. eliminations, round by round
    for (const RoundWork& r : rounds) {
        if (r.g1 > r.g0) {
            ScopedTimer tm(ctx, 1, r.edge_cells, false);
            LWP_HIP(ctx, launch_edge_sum_desc(d_ed + r.g0, d_src, (int32_t)(r.g1 - r.g0), r.edge_max_cells, st));
        }
        for (const NodeLaunch& nl : r.launches) {
            const int v = nl.variant;
            const bool keyed = v < 2, small = (v == 0 || v == 2 || v == 4);
            const int mode = v >= 4 ? kModeValue : (keyed ? kModeKeyed : kModePlain);
            const int tile = small ? kTileSmall : kTileLarge;
            NodeArgs na{};
            na.descs = d_nd + nl.first;
            na.Ci = nl.Ci; na.Cj = nl.Cj; na.Ck = nl.Ck; na.batch = (int32_t)nl.count;
            na.tilesM = (nl.Ci + tile - 1) / tile;
            na.tilesN = (nl.Ck + tile - 1) / tile;
            const bool mixed = nl.tile_begin >= 0;
            if (mixed) { na.tile_begin = d_tbeg + nl.tile_begin; na.total_tiles = nl.total_tiles; }
            ScopedTimer tm(ctx, 0, nl.updates, keyed);
            // a launch of mixed shapes splits by its longest product: every product divides its own
            // stages among the parts, and parts beyond a short product's stages see only padding
            const int kparts = choose_kparts(mixed ? nl.total_tiles : (int64_t)na.tilesM * na.tilesN * na.batch, nl.split_Cj, small);
            if (kparts > 1) { if (lwp_status s2 = ensure_split_buffers(ctx)) return s2; }
            set_split(ctx, na, kparts);
            LWP_HIP(ctx, launch_minplus(na, mode, small, st));
        }
    }

    // 5. residual graph, undo, results
    LWP_HIP(ctx, launch_pair_min(d_pd, (int32_t)plan.pairs.size(), pair_max_rows, d_keys, d_flag, st));
    LWP_HIP(ctx, launch_single_min(d_sd, (int32_t)plan.singles.size(), single_max_c, d_keys + plan.pairs.size(), st));
    for (size_t q = 0; q < plan.comps.size(); ++q)
        LWP_HIP(ctx, launch_component_min(d_cd + q, comp_prefix[q],
                                          d_keys + plan.pairs.size() + plan.singles.size() + q, d_flag, st));
    LWP_HIP(ctx, launch_back_substitute(d_pd, (int32_t)plan.pairs.size(), d_sd, (int32_t)plan.singles.size(),
                                        d_cd, (int32_t)plan.comps.size(), d_keys, d_ud, plan.n_node_steps, n_nodes,
                                        d_flag, d_stats + 2 * (int64_t)rng_w0, d_result, st));
    int32_t* result = reinterpret_cast<int32_t*>(ctx->pin + pin_result);
    LWP_HIP(ctx, hipMemcpyAsync(result, d_result, (3 + (size_t)n_nodes) * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    LWP_HIP(ctx, hipStreamSynchronize(st));
    if (result[2 + n_nodes]) return fail(ctx, LWP_E_OVERFLOW, "a sum may leave int32 (found on the device from the tables' actual ranges)");
    const int64_t total = (int64_t)(((uint64_t)(uint32_t)result[1] << 32) | (uint32_t)result[0]);
    if (!fits(total)) return fail(ctx, LWP_E_OVERFLOW, "the total cost leaves int32");
    *out_cost = (int32_t)total;
    std::memcpy(out_strategy, result + 2, (size_t)n_nodes * sizeof(int32_t));
    return LWP_OK;
}

}  // extern "C"
