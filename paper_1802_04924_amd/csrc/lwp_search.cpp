// Alg. 1 behind the C ABI: buffer planning, value-range analysis, descriptors and the launch
// sequence of a whole search (eliminate -> solve the residual graph -> undo).
#include <atomic>
#include <chrono>
#include <cstring>
#include <map>
#include <new>
#include <tuple>

#include "lwp_context.h"
#include "lwp_plan.h"

using namespace lwp;

namespace {

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

// kernel variants of a node-elimination launch: arithmetic picked on the device (stored argmin
// tables) or value-only (recomputed undo), on 64 x 64 or 128 x 128 tiles
// (tile size = variant & 1; the arithmetic = variant / 2)
enum { kVarAutoSmall = 0, kVarAutoLarge = 1, kVarValueSmall = 2, kVarValueLarge = 3,
       kVarKeyedSmall = 4, kVarKeyedLarge = 5, kVarPlainSmall = 6, kVarPlainLarge = 7 };
// How a search with stored argmin tables picks the arithmetic of its node eliminations:
//   kArithPlain  compare/select everywhere: for searches so small that launches are bound by latency;
//   kArithKeyed  packed keys on global offsets everywhere, launched speculatively: the fastest
//                kernel, and the right one unless a table's values range widely; a product whose
//                measured ranges do not allow the keys is skipped and flagged, and the search runs again with
//   kArithAuto   the kernel that picks keys, keys re-based per row or compare/select per product.
enum { kArithAuto = 0, kArithValue = 1, kArithKeyed = 2, kArithPlain = 3 };

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
    L.node_A.reserve(plan.n_node_steps); L.node_B.reserve(plan.n_node_steps); L.node_out.reserve(plan.n_node_steps);
    L.node_arg_off.reserve(plan.n_node_steps);
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
    std::vector<TableRef> release;
    while (t < n) {
        const int32_t round = plan.steps[t].round;
        // E-phase of this round
        release.clear();
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
            L.groups.push_back(std::move(g)); L.group_src.push_back(std::move(src)); L.group_out.push_back(out);
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
    size_t node_desc, edge_desc, src_ptrs, pair_desc, singles, undo, comps, tile_begin, tiny_rounds, range_list;   // offsets inside the block
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
        o.tiny_rounds = sub(((size_t)plan.n_rounds + 1) * sizeof(TinyRound));         // a small search in one launch
        o.range_list = sub((size_t)n_edges * sizeof(int32_t));                         // input tables whose value range is measured
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


// One search: what the host decides (plan, buffers, descriptors, launches) and the order in which
// it is put on the stream.  The device workspace and the pinned mirror are handed in by the caller.
class Search {
public:
    Search(lwp_ctx* ctx, int32_t n_nodes, int32_t n_edges, const int32_t* edges, const int32_t* Cn,
           const int32_t* d_tc, const int32_t* d_ts, const int32_t* d_tx, int32_t schedule, bool stored)
        : ctx_(ctx), n_nodes_(n_nodes), n_edges_(n_edges), edges_(edges), Cn_(Cn), d_tc_(d_tc), d_ts_(d_ts),
          d_tx_(d_tx), schedule_(schedule), stored_(stored), stream_(ctx ? ctx->stream : nullptr) {}

    // Validates the graph, fixes the schedule and lays out the buffers (host only).
    lwp_status plan();
    size_t workspace_bytes() const { return W_.total; }
    size_t pinned_bytes() const { return pin_result_ + (3 + (size_t)n_nodes_) * sizeof(int32_t); }
    void bind(char* ws, char* pin);

    // Nothing the host decides depends on the tables' values: with stored argmin tables the
    // elimination kernel picks its arithmetic variant per product on the device, from the ranges the
    // producing launches measured; with recomputed undo every elimination is value-only; overflow is
    // judged on the device in both.  So the descriptors are written first, uploaded with one copy,
    // and everything is enqueued without a read-back; the one synchronisation is at the end.
    lwp_status run(int32_t* out_cost, int32_t* out_strategy);

    // The pieces of run() for a caller that prepares once and runs many times.
    lwp_status prepare_replay();                 // descriptors for any int32 input, uploaded; synchronises
    lwp_status enqueue_all();                    // everything between the tables and the result copy
    lwp_status finish(int32_t* out_cost, int32_t* out_strategy) const;   // after the result has arrived
    void mark_result_pending() { h_result_[2 + n_nodes_] = kResultPending; }   // before enqueue_all
    lwp_status wait_for_result();                // until the undo kernel's last word has arrived
    static constexpr int32_t kResultPending = 0x40000000;   // no status word has this bit

private:
    lwp_status enqueue_tiny();                   // the whole search as one launch of one workgroup
    lwp_status upload_offsets();                 // per-node counts only: row / table offsets, ahead of the descriptors
    lwp_status measure_inputs();                 // w = t_c + t_s, ranges of w and of every input table
    lwp_status write_descriptors(int arith);     // descriptors, launch list; arith: see kArith*
    lwp_status attempt(int arith, bool replay_prepare);
    lwp_status upload_descriptors();
    lwp_status enqueue_eliminations();
    lwp_status enqueue_residual_and_undo();
    lwp_status enqueue_result_copy();

    const int32_t* table_ptr(const TableRef& r) const { return (r.is_slot ? d_slots_ : d_tx_) + r.off; }
    int32_t* slot_ptr(const TableRef& r) const { return d_slots_ + r.off; }
    const int32_t* w_ptr(int32_t v) const { return d_w_ + L_.node_off[v]; }

    struct NodeLaunch {
        size_t first, count; int32_t Ci, Cj, Ck; int variant;
        int64_t tile_begin;      // index into the tile_begin block for mixed shapes, else -1
        int32_t total_tiles, split_Cj; int64_t updates;   // split_Cj: the Cj that decides how tiles are split
        int wave_rb;             // 0: the tiled kernel; 1 / 2: a wavefront per 8 x 8 / 16 x 16 tile (tile counts in that unit)
    };
    struct RoundWork { size_t g0, g1; int64_t edge_cells, edge_max_cells; std::vector<NodeLaunch> launches; };

    lwp_ctx* ctx_;
    int32_t n_nodes_, n_edges_;
    const int32_t* edges_;
    const int32_t* Cn_;
    const int32_t *d_tc_, *d_ts_, *d_tx_;
    int32_t schedule_;
    bool stored_;
    hipStream_t stream_;

    Plan plan_;
    Layout L_;
    WsLayout W_{};
    size_t pin_desc_ = 0, pin_result_ = 0;
    int32_t n_comp_ = 0, rng_w0_ = 0, rng_node0_ = 0, rng_group0_ = 0;
    // device
    char* ws_ = nullptr;
    int32_t *d_w_ = nullptr, *d_head_ = nullptr, *d_stats_ = nullptr, *d_flag_ = nullptr, *d_args_ = nullptr,
            *d_slots_ = nullptr, *d_result_ = nullptr;
    unsigned long long* d_keys_ = nullptr;
    char* db_ = nullptr;         // descriptor block on the device
    // pinned host
    char* hb_ = nullptr;         // mirror of the descriptor block
    int32_t* h_result_ = nullptr;
    // launches
    std::vector<RoundWork> rounds_;
    std::vector<unsigned long long> comp_prefix_;
    int32_t pair_max_rows_ = 1, single_max_c_ = 1;
    // A search whose whole work is a few hundred thousand simple operations on tables that fit LDS
    // together (the paper's own sizes: a handful of devices, tens of configurations per layer) runs
    // in one launch of one workgroup: the dozen dependent launches of the general path would cost
    // several times its arithmetic.
    bool tiny_ = false;
    bool block_on_device_ = false;   // the descriptor block has been uploaded and is not rewritten (a replayed plan)
    bool any_tiled_ = true;      // some round of node eliminations runs on the tiled kernel
    // Input tables that are an operand of a node elimination as they are.  Only these need a measured
    // value range: a table that is first summed into another (Eq. 3) is covered by the range of the sum.
    std::vector<int32_t> direct_tables_;
    bool upload_with_prepare_ = false;   // measure_inputs() also copies the descriptor block to the device
    static constexpr size_t kUploadWithPrepare = (size_t)1 << 20;
    // Node eliminations of a round with little work run on the kernel that gives each wavefront a small
    // tile of its own (see kWaveMaxUpdates).
    bool round_on_wave_kernel(int64_t updates) const {
        return (!ctx_ || ctx_->wave_kernel) && updates <= kWaveMaxUpdates;
    }
};

lwp_status Search::plan() {
    {
        std::string err;
        lwp_status s = make_plan(n_nodes_, n_edges_, edges_, schedule_, plan_, err);
        if (s != LWP_OK) return fail(ctx_, s, err);
    }
    if (!components_enumerable(plan_, Cn_))
        return fail(ctx_, LWP_E_NOT_REDUCIBLE, "a residual component has more than 2^32 strategies to enumerate");
    L_ = plan_buffers(plan_, n_nodes_, n_edges_, edges_, Cn_, !stored_);
    W_ = layout_workspace(plan_, L_, n_nodes_, n_edges_, stored_);
    pin_desc_ = 0;
    pin_result_ = pin_desc_ + align_up(W_.desc_bytes, 256);
    n_comp_ = (int32_t)(plan_.pairs.size() + plan_.singles.size() + plan_.comps.size());
    {
        // Operations one workgroup would have to do.  Measured on chains of 6 to 400 nodes with 8 to 64
        // configurations: with the tables in LDS one compute unit does about 14 500 operations per
        // microsecond and spends 2.5 us per round, the general path 4.5 us per round and 8 us more at
        // the start; the two are level where operations = 116 000 + 29 000 x rounds.
        constexpr double kTinyWorkBase = 116000.0, kTinyWorkPerRound = 29000.0, kTinyEnumeration = 65536.0;
        const double kTinyWork = kTinyWorkBase + kTinyWorkPerRound * plan_.n_rounds;
        double work = (double)L_.node_off[n_nodes_];
        for (size_t q = 0; q < L_.node_A.size(); ++q) work += (double)L_.node_A[q].rows * L_.node_A[q].cols * L_.node_B[q].cols;
        for (size_t g = 0; g < L_.groups.size(); ++g) work += (double)L_.group_out[g].cells() * L_.group_src[g].size();
        for (auto& t : L_.final_table) work += (double)t.cells();
        bool small_enumerations = true;
        for (auto& c : plan_.comps) {
            double n = 1;
            for (int32_t v : c.nodes) n *= Cn_[v];
            small_enumerations = small_enumerations && n <= kTinyEnumeration;
            work += n * (double)(c.nodes.size() + c.edges.size());
        }
        const int64_t table_words = L_.node_off[n_nodes_] + L_.tx_off[n_edges_] + L_.slot_elems;
        tiny_ = small_enumerations && work <= kTinyWork && table_words <= kTinyLdsWords && (!ctx_ || ctx_->single_launch);
    }
    // the measuring pass over the input tables serves the tiled kernel only
    any_tiled_ = false;
    direct_tables_.clear();
    {
        size_t q = 0, t = 0;
        const size_t n = plan_.steps.size();
        std::vector<char> direct((size_t)n_edges_, 0);
        while (t < n) {
            const int32_t round = plan_.steps[t].round;
            int64_t updates = 0;
            const size_t q_first = q;
            for (; t < n && plan_.steps[t].round == round; ++t)
                if (plan_.steps[t].kind == 0) {
                    updates += (int64_t)L_.node_A[q].rows * L_.node_A[q].cols * L_.node_B[q].cols;
                    ++q;
                }
            if (q > q_first && !round_on_wave_kernel(updates)) {
                any_tiled_ = true;
                // its operands that are still the caller's tables (these start at the table offsets)
                for (size_t x = q_first; x < q; ++x)
                    for (const TableRef* r : {&L_.node_A[x], &L_.node_B[x]})
                        if (!r->is_slot) {
                            const auto it = std::lower_bound(L_.tx_off.begin(), L_.tx_off.end() - 1, r->off);
                            direct[(size_t)(it - L_.tx_off.begin())] = 1;
                        }
            }
        }
        for (int32_t e = 0; e < n_edges_; ++e)
            if (direct[(size_t)e]) direct_tables_.push_back(e);
    }
    // index of the range pair of: input edge e | w of node v | output of node step | output of group
    rng_w0_ = n_edges_;
    rng_node0_ = n_edges_ + n_nodes_;
    rng_group0_ = rng_node0_ + plan_.n_node_steps;
    return LWP_OK;
}

void Search::bind(char* ws, char* pin) {
    ws_ = ws;
    d_w_ = reinterpret_cast<int32_t*>(ws + W_.w);
    d_head_ = reinterpret_cast<int32_t*>(ws + W_.head);
    d_flag_ = d_head_;           // set by any kernel that finds a sum outside int32
    d_stats_ = d_head_ + 2;
    d_args_ = reinterpret_cast<int32_t*>(ws + W_.args);
    d_slots_ = reinterpret_cast<int32_t*>(ws + W_.slots);
    d_keys_ = reinterpret_cast<unsigned long long*>(ws + W_.keys);
    d_result_ = reinterpret_cast<int32_t*>(ws + W_.result);
    db_ = ws + W_.desc;
    hb_ = pin + pin_desc_;
    h_result_ = reinterpret_cast<int32_t*>(pin + pin_result_);
    if (!L_.uniform) {           // rows and tables of different sizes: the kernels need their offsets
        int64_t* h_offs = reinterpret_cast<int64_t*>(hb_ + W_.offs);
        std::memcpy(h_offs, L_.node_off.data(), ((size_t)n_nodes_ + 1) * sizeof(int64_t));
        std::memcpy(h_offs + n_nodes_ + 1, L_.tx_off.data(), ((size_t)n_edges_ + 1) * sizeof(int64_t));
    }
}

lwp_status Search::run(int32_t* out_cost, int32_t* out_strategy) {
    if (tiny_) {
        if (lwp_status s = write_descriptors(stored_ ? kArithPlain : kArithValue)) return s;
        // a block that fits the kernel arguments travels there, a larger one the kernel fetches itself
        if (!tiny_block_fits_arguments(W_.desc_bytes) && !tiny_block_copied_by_kernel(W_.desc_bytes)) {
            if (lwp_status s = upload_descriptors()) return s;
        }
        mark_result_pending();
        if (lwp_status s = enqueue_tiny()) return s;
        if (lwp_status s = wait_for_result()) return s;
        return finish(out_cost, out_strategy);
    }
    int64_t updates = 0;
    for (size_t q = 0; q < L_.node_A.size(); ++q) updates += (int64_t)L_.node_A[q].rows * L_.node_A[q].cols * L_.node_B[q].cols;
    // Below this size launches are bound by latency, not arithmetic, and the kernel with the least
    // start-up work wins (measured: AlexNet- and VGG-16-shaped searches with 256 configurations).
    constexpr int64_t kKeysPayFrom = (int64_t)1 << 29;
    int arith = !stored_ ? kArithValue : (updates < kKeysPayFrom ? kArithPlain : (ctx_->keys_failed ? kArithAuto : kArithKeyed));
    for (;;) {
        // the measuring pass needs no descriptor (only, with per-node counts, the offsets, which go
        // ahead): it runs on the device while the host writes the descriptors
        mark_result_pending();
        if (lwp_status s = upload_offsets()) return s;
        // A descriptor block of up to a megabyte is written first (microseconds: 4 for the 120-node
        // Inception-shaped graph) and copied from the pinned mirror by the first launch: a copy of its
        // own goes through the DMA engine from a few kilobytes on and holds the stream up for 15 us.
        // A larger block is written while the measuring pass runs and uploaded by such a copy.
        upload_with_prepare_ = W_.desc_bytes <= kUploadWithPrepare && W_.desc_bytes % 16 == 0;
        if (upload_with_prepare_) {
            if (lwp_status s = write_descriptors(arith)) return s;
            const lwp_status s = measure_inputs();
            upload_with_prepare_ = false;
            if (s) return s;
        } else {
            if (lwp_status s = measure_inputs()) return s;
            if (lwp_status s = write_descriptors(arith)) return s;
            if (lwp_status s = upload_descriptors()) return s;
        }
        if (lwp_status s = enqueue_eliminations()) return s;
        if (lwp_status s = enqueue_residual_and_undo()) return s;
        if (lwp_status s = enqueue_result_copy()) return s;
        if (lwp_status s = wait_for_result()) return s;
        if (arith == kArithKeyed && (h_result_[2 + n_nodes_] & 4)) {
            // some table's values range too widely for packed keys on global offsets: once more with
            // the kernel that picks per product; later searches of this context start there
            ctx_->keys_failed = true;
            arith = kArithAuto;
            continue;
        }
        return finish(out_cost, out_strategy);
    }
}

lwp_status Search::prepare_replay() {
    if (lwp_status s = write_descriptors(stored_ ? kArithAuto : kArithValue)) return s;
    if (lwp_status s = upload_descriptors()) return s;
    LWP_HIP(ctx_, hipStreamSynchronize(stream_));
    block_on_device_ = true;
    return LWP_OK;
}

lwp_status Search::enqueue_all() {
    if (tiny_) return enqueue_tiny();
    if (lwp_status s = measure_inputs()) return s;
    if (lwp_status s = enqueue_eliminations()) return s;
    if (lwp_status s = enqueue_residual_and_undo()) return s;
    return enqueue_result_copy();
}

lwp_status Search::enqueue_tiny() {
    TinyArgs a{};
    a.tc = d_tc_; a.ts = d_ts_; a.w = d_w_; a.n_w = L_.node_off[n_nodes_];
    a.tx = d_tx_; a.n_tx = L_.tx_off[n_edges_]; a.slots = d_slots_; a.n_slots = L_.slot_elems;
    a.rounds = reinterpret_cast<const TinyRound*>(db_ + W_.tiny_rounds);
    a.n_rounds = (int32_t)rounds_.size();
    a.nodes = reinterpret_cast<const NodeDesc*>(db_ + W_.node_desc);
    a.edges = reinterpret_cast<const EdgeDesc*>(db_ + W_.edge_desc);
    a.srcs = reinterpret_cast<const int32_t* const*>(db_ + W_.src_ptrs);
    a.pairs = reinterpret_cast<const PairDesc*>(db_ + W_.pair_desc);
    a.singles = reinterpret_cast<const SingleDesc*>(db_ + W_.singles);
    a.comps = reinterpret_cast<const CompDesc*>(db_ + W_.comps);
    a.n_pairs = (int32_t)plan_.pairs.size(); a.n_singles = (int32_t)plan_.singles.size(); a.n_comps = (int32_t)plan_.comps.size();
    a.keys = d_keys_;
    a.undo = reinterpret_cast<const UndoDesc*>(db_ + W_.undo);
    a.n_undo = plan_.n_node_steps; a.n_nodes = n_nodes_;
    a.flag = d_flag_; a.result = d_result_; a.host_result = h_result_;
    // (a block that is on the device already and does not fit the kernel arguments is read where it is)
    const bool read_in_place = block_on_device_ && !tiny_block_fits_arguments(W_.desc_bytes);
    LWP_HIP(ctx_, launch_tiny_search(a, db_, read_in_place ? nullptr : hb_, W_.desc_bytes, stream_));
    return LWP_OK;
}

lwp_status Search::upload_offsets() {
    if (L_.uniform) return LWP_OK;
    LWP_HIP(ctx_, hipMemcpyAsync(db_ + W_.offs, hb_ + W_.offs, W_.offs_bytes, hipMemcpyHostToDevice, stream_));
    return LWP_OK;
}

lwp_status Search::measure_inputs() {
    hipStream_t st = stream_;
    // a small descriptor block (already written then) rides along with the first launch
    const size_t up_skip = align_up(W_.offs_bytes, 16);
    const void* up_src = upload_with_prepare_ ? hb_ + up_skip : nullptr;
    void* up_dst = upload_with_prepare_ ? db_ + up_skip : nullptr;
    const size_t up_bytes = upload_with_prepare_ ? W_.desc_bytes - up_skip : 0;
    // Which input tables are measured: those the tiled kernel will read as they are, if the list of them
    // (part of the descriptor block) is on the device by the time the measuring kernel runs; else all.
    const bool listed = upload_with_prepare_ || block_on_device_;
    const int32_t* d_which = listed ? reinterpret_cast<const int32_t*>(db_ + W_.range_list) : nullptr;
    const int32_t n_listed = listed ? (int32_t)direct_tables_.size() : n_edges_;
    if (L_.uniform) {
        LWP_HIP(ctx_, launch_prepare_search(d_tc_, d_ts_, d_w_, n_nodes_, Cn_[0], nullptr, d_stats_, W_.n_ranges, rng_w0_,
                                            d_keys_, n_comp_, d_flag_, st, up_src, up_dst, up_bytes));
        if (any_tiled_) LWP_HIP(ctx_, launch_ranges(d_tx_, n_listed, (int64_t)Cn_[0] * Cn_[0], d_stats_, st, d_which));
    } else {
        const int64_t* d_offs = reinterpret_cast<const int64_t*>(db_ + W_.offs);
        int64_t max_cells = 1;
        for (int32_t e = 0; e < n_edges_; ++e) max_cells = std::max(max_cells, L_.tx_off[e + 1] - L_.tx_off[e]);
        LWP_HIP(ctx_, launch_prepare_search(d_tc_, d_ts_, d_w_, n_nodes_, 0, d_offs, d_stats_, W_.n_ranges, rng_w0_,
                                            d_keys_, n_comp_, d_flag_, st, up_src, up_dst, up_bytes));
        if (any_tiled_) LWP_HIP(ctx_, launch_ranges_var(d_tx_, d_offs + n_nodes_ + 1, n_listed, max_cells, d_stats_, st, d_which));
    }
    return LWP_OK;
}

// Writes the descriptors straight into the pinned mirror of the device block and fixes the launch
// list.  The descriptors promise nothing about the values (full int32 ranges): every kernel reads
// the ranges its producers measured (rngA / rngB / rngW) and tests on the device what it needs --
// key widths, and that no sum leaves int32; the flag those tests set comes back with the result.
lwp_status Search::write_descriptors(int arith) {
    const Plan& plan = plan_;
    const Layout& L = L_;
    const bool stored = stored_;
    NodeDesc* nd = reinterpret_cast<NodeDesc*>(hb_ + W_.node_desc);
    EdgeDesc* ed = reinterpret_cast<EdgeDesc*>(hb_ + W_.edge_desc);
    const int32_t** src_ptrs = reinterpret_cast<const int32_t**>(hb_ + W_.src_ptrs);
    PairDesc* pd = reinterpret_cast<PairDesc*>(hb_ + W_.pair_desc);
    SingleDesc* sd = reinterpret_cast<SingleDesc*>(hb_ + W_.singles);
    UndoDesc* ud = reinterpret_cast<UndoDesc*>(hb_ + W_.undo);
    CompDesc* cd = reinterpret_cast<CompDesc*>(hb_ + W_.comps);
    int32_t* tbeg = reinterpret_cast<int32_t*>(hb_ + W_.tile_begin);
    size_t n_tbeg = 0;
    if (!direct_tables_.empty())
        std::memcpy(hb_ + W_.range_list, direct_tables_.data(), direct_tables_.size() * sizeof(int32_t));
    rounds_.clear();

    std::vector<int32_t> erng(n_edges_);          // range-pair index of the edge's current table
    for (int32_t e = 0; e < n_edges_; ++e) erng[e] = e;
    // Node eliminations of one round are independent; those of equal kernel variant share a
    // launch if they agree in shape (Ci, Cj, Ck) or run on 64 x 64 tiles (a launch of mixed shapes),
    // so the descriptors of a round are ordered by (variant, shape).
    struct NodeWork { NodeDesc d; int32_t Ci, Cj, Ck; int variant; int32_t rngA, rngB; };
    // A table made by the wavefront-per-tile kernel gets its range measured only if a launch of the
    // tiled kernel consumes it (the descriptor of the producer is patched then).
    std::vector<int64_t> unmeasured(W_.n_ranges, -1);      // range pair -> descriptor of its producer
    // positions of a round's products among its output cells (single-workgroup search)
    auto number_round = [&](size_t first, size_t last) {
        constexpr int64_t cap = int64_t(1) << 30;
        int64_t cells = 0;
        for (size_t q = first; q < last; ++q) {
            NodeDesc& d = nd[q];
            d.cell_begin = (int32_t)std::min(cells, cap);
            cells += (int64_t)d.Ci * d.Ck;
        }
    };
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
            erng[g.keep] = rng_group0_ + (int32_t)gi;
            ed[gi].out = slot_ptr(L.group_out[gi]);
            ed[gi].rngOut = d_stats_ + 2 * (int64_t)erng[g.keep];
            ed[gi].flag = d_flag_;
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
            const TableRef &tA = L.node_A[ni], &tB = L.node_B[ni], &tO = L.node_out[ni];
            NodeWork nw{};
            NodeDesc& d = nw.d;
            d.flag = d_flag_;
            d.A = table_ptr(tA); d.w = w_ptr(s.j); d.B = table_ptr(tB);
            d.out = slot_ptr(tO);
            d.arg = stored ? d_args_ + L.node_arg_off[ni] : nullptr;
            d.loA = d.loW = d.loB = (int32_t)kI32Min;
            d.hiA = d.hiW = d.hiB = (int32_t)kI32Max;
            d.rngA = d_stats_ + 2 * (int64_t)erng[s.e1];
            d.rngB = d_stats_ + 2 * (int64_t)erng[s.e2];
            d.rngW = d_stats_ + 2 * (int64_t)(rng_w0_ + s.j);
            d.rngOut = d_stats_ + 2 * (int64_t)(rng_node0_ + (int32_t)ni);
            nw.Ci = tA.rows; nw.Cj = tA.cols; nw.Ck = tB.cols;
            nw.rngA = erng[s.e1]; nw.rngB = erng[s.e2];
            d.Ci = nw.Ci; d.Cj = nw.Cj; d.Ck = nw.Ck;
            work.push_back(nw);
            ud[ni] = {d.arg, d.A, d.w, d.B, s.j, s.i, s.k, s.round, nw.Cj, nw.Ck, (int32_t)n0, 0};
            erng[s.e1] = rng_node0_ + (int32_t)ni;
            ++ni; ++t;
        }
        // kernel variant per product: the search's arithmetic, and the tile size from the number of
        // tiles the products of that shape make
        auto shape_of = [](const NodeWork& a) { return std::make_tuple(a.Ci, a.Cj, a.Ck); };
        // (with one count for all nodes every product has the same shape: no table needed)
        std::map<std::tuple<int32_t, int32_t, int32_t>, int64_t> shape_count;
        if (!L.uniform) for (const NodeWork& x : work) ++shape_count[shape_of(x)];
        const size_t n_shapes = L.uniform ? (work.empty() ? 0 : 1) : shape_count.size();
        for (NodeWork& x : work) {
            const bool prefer_small = want_small_tiles(x.Ci, x.Cj, x.Ck, L.uniform ? (int64_t)work.size() : shape_count[shape_of(x)]);
            x.variant = 2 * arith + (prefer_small ? 0 : 1);
        }
        // A round with little work runs as one launch of the kernel that gives every wavefront a tile
        // of its own: with so few 64 x 64 tiles the tiled kernel's launch would be mostly latency.
        int64_t round_updates = 0;
        for (const NodeWork& x : work) round_updates += (int64_t)x.Ci * x.Cj * x.Ck;
        if (!work.empty() && round_on_wave_kernel(round_updates)) {
            int64_t t16 = 0;
            for (const NodeWork& x : work) t16 += (int64_t)((x.Ci + 15) / 16) * ((x.Ck + 15) / 16);
            int64_t round_cells = 0;
            for (const NodeWork& x : work) round_cells += (int64_t)x.Ci * x.Ck;
            const int rb = wave_tile_rb(t16, round_updates / round_cells);
            const int ts = 8 * rb;
            const bool one_shape = n_shapes == 1;
            NodeLaunch nl{n0, work.size(), work[0].Ci, work[0].Cj, work[0].Ck, 2 * (stored ? kArithPlain : kArithValue), -1, 0, 0, round_updates, rb};
            int64_t tiles = 0;
            if (!one_shape) nl.tile_begin = (int64_t)n_tbeg;
            for (const NodeWork& x : work) {
                if (!one_shape) tbeg[n_tbeg++] = (int32_t)tiles;
                tiles += (int64_t)((x.Ci + ts - 1) / ts) * ((x.Ck + ts - 1) / ts);
            }
            if (!one_shape) tbeg[n_tbeg++] = (int32_t)tiles;
            nl.total_tiles = (int32_t)tiles;       // a tile holds at least one cell: <= 2^27
            rw_.launches.push_back(nl);
            for (size_t q = 0; q < work.size(); ++q) {
                nd[n0 + q] = work[q].d;
                nd[n0 + q].rngOut = nullptr;
                unmeasured[rng_node0_ + (int32_t)(n0 + q)] = (int64_t)(n0 + q);
            }
            number_round(n0, ni);
            reinterpret_cast<TinyRound*>(hb_ + W_.tiny_rounds)[rounds_.size()] = {(int32_t)rw_.g0, (int32_t)rw_.g1, (int32_t)n0, (int32_t)ni};
            rounds_.push_back(std::move(rw_));
            continue;
        }
        for (const NodeWork& x : work)
            for (int32_t r : {x.rngA, x.rngB})
                if (unmeasured[r] >= 0) { nd[unmeasured[r]].rngOut = d_stats_ + 2 * (int64_t)r; unmeasured[r] = -1; }
        order.resize(work.size());
        for (size_t q = 0; q < order.size(); ++q) order[q] = q;
        std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) {
            return std::make_pair(work[a].variant, shape_of(work[a])) < std::make_pair(work[b].variant, shape_of(work[b]));
        });
        for (size_t a = 0; a < order.size();) {
            const int v = work[order[a]].variant;
            size_t b = a;
            while (b < order.size() && work[order[b]].variant == v) ++b;
            const bool small = (v & 1) == 0;
            const bool one_shape = shape_of(work[order[a]]) == shape_of(work[order[b - 1]]);
            if (small && !one_shape) {
                // one launch over all shapes: product q owns tiles [tile_begin[q], tile_begin[q+1])
                NodeLaunch nl{n0 + a, b - a, 0, 0, 0, v, (int64_t)n_tbeg, 0, 0, 0, 0};
                int64_t tiles = 0;
                for (size_t q = a; q < b; ++q) {
                    NodeWork& x = work[order[q]];
                    tbeg[n_tbeg++] = (int32_t)tiles;
                    tiles += (int64_t)((x.Ci + kTileSmall - 1) / kTileSmall) * ((x.Ck + kTileSmall - 1) / kTileSmall);
                    nl.split_Cj = std::max(nl.split_Cj, x.Cj);
                    nl.updates += (int64_t)x.Ci * x.Cj * x.Ck;
                }
                tbeg[n_tbeg++] = (int32_t)tiles;
                if (tiles > INT32_MAX) return fail(ctx_, LWP_E_INVAL, "too many tiles in one round");
                nl.total_tiles = (int32_t)tiles;
                rw_.launches.push_back(nl);
            } else {
                for (size_t q = a; q < b;) {
                    size_t e = q;
                    while (e < b && shape_of(work[order[e]]) == shape_of(work[order[q]])) ++e;
                    const NodeWork& x = work[order[q]];
                    rw_.launches.push_back({n0 + q, e - q, x.Ci, x.Cj, x.Ck, v, -1, 0, x.Cj,
                                            (int64_t)(e - q) * x.Ci * x.Cj * x.Ck, 0});
                    q = e;
                }
            }
            a = b;
        }
        for (size_t q = 0; q < order.size(); ++q) nd[n0 + q] = work[order[q]].d;
        number_round(n0, ni);
        reinterpret_cast<TinyRound*>(hb_ + W_.tiny_rounds)[rounds_.size()] = {(int32_t)rw_.g0, (int32_t)rw_.g1, (int32_t)n0, (int32_t)ni};
        rounds_.push_back(std::move(rw_));
    }

    pair_max_rows_ = 1; single_max_c_ = 1;
    for (size_t q = 0; q < plan.pairs.size(); ++q) {
        const auto& pr = plan.pairs[q];
        pd[q] = {table_ptr(L.final_table[q]), w_ptr(pr.src), w_ptr(pr.dst), pr.src, pr.dst, Cn_[pr.src], Cn_[pr.dst]};
        pair_max_rows_ = std::max(pair_max_rows_, Cn_[pr.src]);
    }
    for (size_t q = 0; q < plan.singles.size(); ++q) {
        const int32_t v = plan.singles[q];
        sd[q] = {w_ptr(v), v, Cn_[v]};
        single_max_c_ = std::max(single_max_c_, Cn_[v]);
    }
    comp_prefix_.assign(plan.comps.size(), 1);
    for (size_t q = 0; q < plan.comps.size(); ++q) {
        const auto& c = plan.comps[q];
        CompDesc d{};
        d.K = (int32_t)c.nodes.size(); d.n_edges = (int32_t)c.edges.size();
        unsigned long long prefix = 1;
        for (int x = 0; x < d.K; ++x) {
            d.node[x] = c.nodes[x]; d.Cn[x] = Cn_[c.nodes[x]]; d.w[x] = w_ptr(c.nodes[x]);
            if (x + 1 < d.K) prefix *= (unsigned long long)d.Cn[x];
        }
        comp_prefix_[q] = prefix;
        for (int x = 0; x < d.n_edges; ++x) {
            d.tab[x] = table_ptr(L.comp_tables[q][x]);
            d.src_pos[x] = (int8_t)(std::find(c.nodes.begin(), c.nodes.end(), c.esrc[x]) - c.nodes.begin());
            d.dst_pos[x] = (int8_t)(std::find(c.nodes.begin(), c.nodes.end(), c.edst[x]) - c.nodes.begin());
        }
        cd[q] = d;
    }
    return LWP_OK;
}

lwp_status Search::upload_descriptors() {
    if (W_.desc_bytes <= kUploadWithPrepare && W_.desc_bytes % 16 == 0)
        LWP_HIP(ctx_, launch_copy_block(hb_, db_, W_.desc_bytes, stream_));
    else
        LWP_HIP(ctx_, hipMemcpyAsync(db_, hb_, W_.desc_bytes, hipMemcpyHostToDevice, stream_));
    return LWP_OK;
}

lwp_status Search::enqueue_eliminations() {
    hipStream_t st = stream_;
    const NodeDesc* d_nd = reinterpret_cast<const NodeDesc*>(db_ + W_.node_desc);
    const EdgeDesc* d_ed = reinterpret_cast<const EdgeDesc*>(db_ + W_.edge_desc);
    const int32_t* const* d_src = reinterpret_cast<const int32_t* const*>(db_ + W_.src_ptrs);
    const int32_t* d_tbeg = reinterpret_cast<const int32_t*>(db_ + W_.tile_begin);
    for (const RoundWork& r : rounds_) {
        if (r.g1 > r.g0) {
            ScopedTimer tm(ctx_, 1, r.edge_cells, false);
            LWP_HIP(ctx_, launch_edge_sum_desc(d_ed + r.g0, d_src, (int32_t)(r.g1 - r.g0), r.edge_max_cells, st));
        }
        for (const NodeLaunch& nl : r.launches) {
            const int v = nl.variant;
            const bool small = (v & 1) == 0;
            const int arith = v / 2;
            const int mode = arith == kArithAuto ? kModeAuto : (arith == kArithValue ? kModeValue : (arith == kArithKeyed ? kModeKeyed : kModePlain));
            const int tile = small ? kTileSmall : kTileLarge;
            NodeArgs na{};
            na.descs = d_nd + nl.first;
            na.Ci = nl.Ci; na.Cj = nl.Cj; na.Ck = nl.Ck; na.batch = (int32_t)nl.count;
            na.tilesM = (nl.Ci + tile - 1) / tile;
            na.tilesN = (nl.Ck + tile - 1) / tile;
            const bool mixed = nl.tile_begin >= 0;
            if (mixed) { na.tile_begin = d_tbeg + nl.tile_begin; na.total_tiles = nl.total_tiles; }
            if (nl.wave_rb) {
                const int ts = 8 * nl.wave_rb;
                na.tilesM = (nl.Ci + ts - 1) / ts;
                na.tilesN = (nl.Ck + ts - 1) / ts;
                na.total_tiles = nl.total_tiles;
                na.mode_count = ctx_->dstate ? ctx_->dstate + 1 : nullptr;
                ScopedTimer tm(ctx_, 0, nl.updates, false);
                const NodeDesc* h_nd = reinterpret_cast<const NodeDesc*>(hb_ + W_.node_desc) + nl.first;
                LWP_HIP(ctx_, launch_minplus_wave(na, h_nd, arith == kArithValue ? kModeValue : kModePlain, nl.wave_rb, st));
                continue;
            }
            if (mode == kModeAuto) {
                na.auto_limit = small ? kKeyedMaxSpreadSmall : kKeyedMaxSpreadLarge;
                // a launch of mixed shapes is judged by its products' common size class
                na.auto_row = keyed_row_pays(mixed ? 1 : nl.Ci, mixed ? 1 : nl.Cj, mixed ? 1 : nl.Ck, mixed ? nl.updates : (int64_t)nl.count) ? 1 : 0;
            }
            na.speculative = arith == kArithKeyed ? 1 : 0;
            na.mode_count = ctx_->dstate ? ctx_->dstate + 1 : nullptr;
            ScopedTimer tm(ctx_, 0, nl.updates, arith == kArithKeyed);
            // a launch of mixed shapes splits by its longest product: every product divides its own
            // stages among the parts, and parts beyond a short product's stages see only padding
            const Split split = choose_split(mixed ? nl.total_tiles : (int64_t)na.tilesM * na.tilesN * na.batch, nl.split_Cj, small);
            if (split.kparts > 1) { if (lwp_status s2 = ensure_split_buffers(ctx_)) return s2; }
            set_split(ctx_, na, split);
            LWP_HIP(ctx_, launch_minplus(na, mode, small, st));
        }
    }
    return LWP_OK;
}

lwp_status Search::enqueue_residual_and_undo() {
    hipStream_t st = stream_;
    const PairDesc* d_pd = reinterpret_cast<const PairDesc*>(db_ + W_.pair_desc);
    const SingleDesc* d_sd = reinterpret_cast<const SingleDesc*>(db_ + W_.singles);
    const UndoDesc* d_ud = reinterpret_cast<const UndoDesc*>(db_ + W_.undo);
    const CompDesc* d_cd = reinterpret_cast<const CompDesc*>(db_ + W_.comps);
    const size_t np = plan_.pairs.size(), ns = plan_.singles.size(), nc = plan_.comps.size();
    LWP_HIP(ctx_, launch_pair_min(d_pd, (int32_t)np, pair_max_rows_, d_keys_, d_flag_, st));
    LWP_HIP(ctx_, launch_single_min(d_sd, (int32_t)ns, single_max_c_, d_keys_ + np, st));
    for (size_t q = 0; q < nc; ++q)
        LWP_HIP(ctx_, launch_component_min(d_cd + q, comp_prefix_[q], d_keys_ + np + ns + q, d_flag_, st));
    LWP_HIP(ctx_, launch_back_substitute(d_pd, (int32_t)np, d_sd, (int32_t)ns, d_cd, (int32_t)nc, d_keys_, d_ud,
                                         plan_.n_node_steps, n_nodes_, d_flag_, d_stats_ + 2 * (int64_t)rng_w0_, d_result_,
                                         h_result_, st));
    return LWP_OK;
}

lwp_status Search::enqueue_result_copy() {
    return LWP_OK;       // the undo kernel writes the result into the pinned host buffer itself
}

// Waits for the result: the undo kernel writes it into the pinned buffer, the status word last, so the
// host polls that word (a wake-up through the runtime's stream wait costs several microseconds more);
// after a while without it the ordinary wait takes over.
lwp_status Search::wait_for_result() {
    volatile int32_t* word = h_result_ + 2 + n_nodes_;
    const auto t0 = std::chrono::steady_clock::now();
    for (int spins = 0; *word == kResultPending; ++spins) {
        if ((spins & 255) == 255 && std::chrono::steady_clock::now() - t0 > std::chrono::microseconds(300)) {
            LWP_HIP(ctx_, hipStreamSynchronize(stream_));
            break;
        }
    }
    std::atomic_thread_fence(std::memory_order_acquire);
    return LWP_OK;
}

lwp_status Search::finish(int32_t* out_cost, int32_t* out_strategy) const {
    if (h_result_[2 + n_nodes_] & 3) return fail(ctx_, LWP_E_OVERFLOW, "a sum may leave int32 (found on the device from the tables' actual ranges)");
    // the total is formed in 64 bits on the device
    const int64_t total = (int64_t)(((uint64_t)(uint32_t)h_result_[1] << 32) | (uint32_t)h_result_[0]);
    if (!fits(total)) return fail(ctx_, LWP_E_OVERFLOW, "the total cost leaves int32");
    *out_cost = (int32_t)total;
    std::memcpy(out_strategy, h_result_ + 2, (size_t)n_nodes_ * sizeof(int32_t));
    return LWP_OK;
}

}  // namespace

// A search whose host-side work (schedule, buffers, descriptors) was done once.  It owns its
// workspace and pinned buffers; a run only re-enqueues the launch sequence.
struct lwp_search_plan {
    lwp_ctx* ctx = nullptr;
    std::vector<int32_t> edges, Cn;
    Search* search = nullptr;
    char* ws = nullptr;
    char* pin = nullptr;
};

// ================================================================================================
extern "C" {

void lwp_search_plan_destroy(lwp_search_plan* plan) {
    if (!plan) return;
    if (plan->ctx) { (void)hipSetDevice(plan->ctx->device); (void)hipStreamSynchronize(plan->ctx->stream); }
    if (plan->ws) (void)hipFree(plan->ws);
    if (plan->pin) (void)hipHostFree(plan->pin);
    delete plan->search;
    delete plan;
}

lwp_status lwp_search_plan_create(lwp_ctx* ctx, int32_t n_nodes, int32_t n_edges, const int32_t* edges,
                                  const int32_t* C_node, const int32_t* d_tc, const int32_t* d_ts,
                                  const int32_t* d_tx, int32_t schedule, lwp_search_plan** out) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (!out) return fail(ctx, LWP_E_INVAL, "null output");
    *out = nullptr;
    if (n_nodes < 1) return fail(ctx, LWP_E_GRAPH, "n_nodes must be >= 1");
    if (n_edges < 0 || (n_edges > 0 && !edges)) return fail(ctx, LWP_E_GRAPH, "edge list missing");
    if (!counts_valid(n_nodes, C_node)) return fail(ctx, LWP_E_INVAL, "every configuration count must be in [1, 65536]");
    if (!d_tc || !d_ts || (n_edges > 0 && !d_tx)) return fail(ctx, LWP_E_INVAL, "null pointer");
    if (((uintptr_t)d_tc | (uintptr_t)d_ts | (uintptr_t)d_tx) & 3)
        return fail(ctx, LWP_E_INVAL, "table pointer not 4-byte aligned");
    lwp_search_plan* plan = new (std::nothrow) lwp_search_plan();
    if (!plan) return fail(ctx, LWP_E_NOMEM, "plan object");
    plan->ctx = ctx;
    auto bail = [&](lwp_status s) { const std::string why = ctx->err; lwp_search_plan_destroy(plan); ctx->err = why; return s; };
    plan->edges.assign(edges, edges + 2 * (size_t)n_edges);
    plan->Cn.assign(C_node, C_node + n_nodes);
    plan->search = new (std::nothrow) Search(ctx, n_nodes, n_edges, plan->edges.data(), plan->Cn.data(), d_tc, d_ts, d_tx,
                                             schedule, /*stored=*/false);
    if (!plan->search) return bail(fail(ctx, LWP_E_NOMEM, "plan object"));
    Search& search = *plan->search;
    if (lwp_status s = search.plan()) return bail(s);
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, std::max<size_t>(search.workspace_bytes(), 256));
    if (e != hipSuccess) { (void)hipGetLastError(); return bail(fail(ctx, LWP_E_NOMEM, std::string("plan workspace: ") + hipGetErrorString(e))); }
    plan->ws = static_cast<char*>(p);
    e = hipHostMalloc(&p, search.pinned_bytes(), hipHostMallocDefault);
    if (e != hipSuccess) { (void)hipGetLastError(); return bail(fail(ctx, LWP_E_NOMEM, std::string("plan pinned buffer: ") + hipGetErrorString(e))); }
    plan->pin = static_cast<char*>(p);
    if (lwp_status s = ensure_split_buffers(ctx)) return bail(s);
    if (lwp_status s = ensure_state(ctx)) return bail(s);
    search.bind(plan->ws, plan->pin);
    if (lwp_status s = search.prepare_replay()) return bail(s);
    *out = plan;
    return LWP_OK;
}

lwp_status lwp_search_plan_run(lwp_search_plan* plan, int32_t* out_cost, int32_t* out_strategy) {
    if (!plan) return LWP_E_INVAL;
    lwp_ctx* ctx = plan->ctx;
    if (lwp_status s = check_ctx(ctx)) return s;
    if (!out_cost || !out_strategy) return fail(ctx, LWP_E_INVAL, "null pointer");
    plan->search->mark_result_pending();
    if (lwp_status s = plan->search->enqueue_all()) return s;
    if (lwp_status s = plan->search->wait_for_result()) return s;
    return plan->search->finish(out_cost, out_strategy);
}

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
    Search search(nullptr, n_nodes, n_edges, edges, C_node, nullptr, nullptr, nullptr, schedule, undo == LWP_UNDO_STORED);
    return search.plan() == LWP_OK ? search.workspace_bytes() : 0;
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
    if (n_nodes < 1) return fail(ctx, LWP_E_GRAPH, "n_nodes must be >= 1");
    if (!counts_valid(n_nodes, Cn)) return fail(ctx, LWP_E_INVAL, "every configuration count must be in [1, 65536]");
    if (!d_tc || !d_ts || (n_edges > 0 && !d_tx) || !out_cost || !out_strategy)
        return fail(ctx, LWP_E_INVAL, "null pointer");
    if (((uintptr_t)d_tc | (uintptr_t)d_ts | (uintptr_t)d_tx) & 3)
        return fail(ctx, LWP_E_INVAL, "table pointer not 4-byte aligned");
    Search search(ctx, n_nodes, n_edges, edges, Cn, d_tc, d_ts, d_tx, schedule, undo == LWP_UNDO_STORED);
    if (lwp_status s = search.plan()) return s;
    if (lwp_status s = ensure_workspace(ctx, search.workspace_bytes())) return s;
    if (lwp_status s = ensure_pinned(ctx, search.pinned_bytes())) return s;
    if (lwp_status s = ensure_state(ctx)) return s;
    search.bind(ctx->ws, ctx->pin);
    return search.run(out_cost, out_strategy);
}

}  // extern "C"
