// Single eliminations behind the C ABI: Eq. 2 (lwp_eliminate_node, lwp_eliminate_node_bounded) and
// Eq. 3 (lwp_eliminate_edge).  All three only enqueue; what their kernels find on the device (a sum
// that may leave int32, a value outside promised ranges) is reported by lwp_synchronize.
#include <mutex>

#include "lwp_context.h"

using namespace lwp;

namespace {

// Device memory one node elimination needs beyond its operands.
struct NodeScratch {
    int32_t* stats;       // measured ranges: [3][batch][2] = {min, max} of A, w, B per product
    int32_t* split;       // split-tile scratch (kSplitMaxWorkgroups parts) or null: tiles are not split
    int32_t* counters;    // split-tile arrival counters (kSplitMaxTiles, zero between launches)
    int32_t* flag;        // error bits (see lwp_ctx::dstate)
    int32_t* mode_count;  // optional: products per kernel variant
};

struct NodeCall {
    int32_t batch, Ci, Cj, Ck;
    const int32_t *A, *w, *B;
    int32_t *out, *arg;
};

void fill_common(NodeArgs& a, const NodeCall& c, const NodeScratch& sc, bool small) {
    const int tile = small ? kTileSmall : kTileLarge;
    a.descs = nullptr;
    a.base.A = c.A; a.base.w = c.w; a.base.B = c.B; a.base.out = c.out; a.base.arg = c.arg;
    a.base.flag = sc.flag;
    a.sA = (int64_t)c.Ci * c.Cj; a.sw = c.Cj; a.sB = (int64_t)c.Cj * c.Ck; a.sO = (int64_t)c.Ci * c.Ck;
    a.Ci = c.Ci; a.Cj = c.Cj; a.Ck = c.Ck; a.batch = c.batch;
    a.tilesM = (c.Ci + tile - 1) / tile; a.tilesN = (c.Ck + tile - 1) / tile;
    a.mode_count = sc.mode_count;
    const int64_t tiles = (int64_t)a.tilesM * a.tilesN * c.batch;
    const Split split = sc.split ? choose_split(tiles, c.Cj, small) : Split{1, tiles};
    a.kparts = split.kparts;
    a.n_whole = (int32_t)split.n_whole;
    a.scratch = split.kparts > 1 ? sc.split : nullptr;
    a.counters = split.kparts > 1 ? sc.counters : nullptr;
}

// Eq. 2 for a call with little work: one launch of the kernel that gives every wavefront a small tile
// of its own.  It judges overflow from the values it stages, so no measuring pass is needed; with
// `verify` the ranges in `promised` (lo A, hi A, lo w, hi w, lo B, hi B) are checked as well.
bool wave_call(const NodeCall& c, int64_t max_updates) {
    return (int64_t)c.batch * c.Ci * c.Cj * c.Ck <= max_updates;
}

hipError_t enqueue_node_wave(const NodeCall& c, const NodeScratch& sc, const int64_t* promised, hipStream_t st) {
    const int rb = wave_tile_rb((int64_t)((c.Ci + 15) / 16) * ((c.Ck + 15) / 16) * c.batch, c.Cj);
    const int ts = 8 * rb;
    NodeArgs a{};
    a.base.A = c.A; a.base.w = c.w; a.base.B = c.B; a.base.out = c.out; a.base.arg = c.arg;
    a.base.flag = sc.flag;
    a.base.loA = a.base.loW = a.base.loB = (int32_t)kI32Min;
    a.base.hiA = a.base.hiW = a.base.hiB = (int32_t)kI32Max;
    if (promised) {
        a.base.loA = (int32_t)promised[0]; a.base.hiA = (int32_t)promised[1]; a.base.loW = (int32_t)promised[2];
        a.base.hiW = (int32_t)promised[3]; a.base.loB = (int32_t)promised[4]; a.base.hiB = (int32_t)promised[5];
    }
    a.sA = (int64_t)c.Ci * c.Cj; a.sw = c.Cj; a.sB = (int64_t)c.Cj * c.Ck; a.sO = (int64_t)c.Ci * c.Ck;
    a.Ci = c.Ci; a.Cj = c.Cj; a.Ck = c.Ck; a.batch = c.batch;
    a.tilesM = (c.Ci + ts - 1) / ts; a.tilesN = (c.Ck + ts - 1) / ts;
    a.total_tiles = (int32_t)((int64_t)a.tilesM * a.tilesN * c.batch);     // a tile holds at least one cell: <= 2^27
    a.mode_count = sc.mode_count;
    return launch_minplus_wave(a, nullptr, c.arg ? kModePlain : kModeValue, rb, st, promised != nullptr);
}

// Eq. 2 with nothing known about the values: {min, max} of A, w and B are measured on the device,
// by a pass over every product or by the product kernel's workgroups themselves (see below).  With
// an argmin output the arithmetic variant depends on the ranges: every workgroup picks it from the
// ranges it is given or has taken and runs the matching body of the kernel.  Nothing comes back to
// the host.
hipError_t enqueue_node_measured(const NodeCall& c, const NodeScratch& sc, hipStream_t st) {
    const bool small = want_small_tiles(c.Ci, c.Cj, c.Ck, c.batch);
    NodeArgs a{};
    a.base.loA = a.base.loW = a.base.loB = (int32_t)kI32Min;
    a.base.hiA = a.base.hiW = a.base.hiB = (int32_t)kI32Max;
    // Where the ranges come from.  Every workgroup can take them from the strips its own tile reads:
    // no launches ahead of the product kernel, but a strip is scanned by every tile of its row or
    // column.  That pays for launches bound by latency (few tiles, a scan of moderate size: 10 x 256^3
    // 34.7 -> 30.7 us, 9 x 512^3 82 -> 76) and for batches of small products, whose strips are shared by
    // at most two tiles (4096 x 256^3: 3.37 -> 3.24 ms).  Otherwise one pass over A, w and B measures
    // every product once (a 2048^3 product would scan 32 times its inputs; 64 x (512, 100, 512), 4096
    // tiles of three stages each, ran 18 % slower scanning).
    const int64_t ts = small ? kTileSmall : kTileLarge;
    const int64_t tm = (c.Ci + ts - 1) / ts, tn = (c.Ck + ts - 1) / ts, tiles = tm * tn * c.batch;
    const int64_t scan_bytes = tiles * 2 * ts * c.Cj * 4;
    a.self_measure = (tm <= 2 && tn <= 2) || (tiles <= 1024 && scan_bytes <= ((int64_t)160 << 20)) ? 1 : 0;
    if (!a.self_measure) {
        int32_t *sA = sc.stats, *sW = sc.stats + 2 * (int64_t)c.batch, *sB = sc.stats + 4 * (int64_t)c.batch;
        hipError_t e = launch_init_workspace(sc.stats, 3 * c.batch, nullptr, nullptr, 0, st);
        if (e == hipSuccess) e = launch_ranges(c.A, c.batch, (int64_t)c.Ci * c.Cj, sA, st);
        if (e == hipSuccess) e = launch_ranges(c.w, c.batch, c.Cj, sW, st);
        if (e == hipSuccess) e = launch_ranges(c.B, c.batch, (int64_t)c.Cj * c.Ck, sB, st);
        if (e != hipSuccess) return e;
        a.base.rngA = sA; a.base.rngW = sW; a.base.rngB = sB;
        a.sR = 2;
    }
    if (!c.arg) {       // minimum only: one variant, the ranges serve the overflow test
        fill_common(a, c, sc, small);
        return launch_minplus(a, kModeValue, small, st);
    }
    a.auto_row = keyed_row_pays(c.Ci, c.Cj, c.Ck, c.batch) ? 1 : 0;
    a.auto_limit = small ? kKeyedMaxSpreadSmall : kKeyedMaxSpreadLarge;
    fill_common(a, c, sc, small);
    return launch_minplus(a, kModeAuto, small, st);
}

lwp_status check_node_call(lwp_ctx* ctx, const NodeCall& c) {
    if (c.batch < 1 || c.Ci < 1 || c.Cj < 1 || c.Ck < 1) return fail(ctx, LWP_E_INVAL, "sizes must be positive");
    if (c.Cj > kMaxConfigs) return fail(ctx, LWP_E_INVAL, "Cj exceeds 65536");
    if (!c.A || !c.w || !c.B || !c.out) return fail(ctx, LWP_E_INVAL, "null table pointer");
    if (((uintptr_t)c.A | (uintptr_t)c.w | (uintptr_t)c.B | (uintptr_t)c.out | (uintptr_t)c.arg) & 3)
        return fail(ctx, LWP_E_INVAL, "table pointer not 4-byte aligned");
    if ((int64_t)((c.Ci + kTileSmall - 1) / kTileSmall) * ((c.Ck + kTileSmall - 1) / kTileSmall) * c.batch > 0x7fffffffLL)
        return fail(ctx, LWP_E_INVAL, "too many output tiles");
    return LWP_OK;
}

// ---- scratch of the entry point that allocates nothing -------------------------------------------
// One array per GPU, held from the moment the library's code is loaded on it until the process ends:
//   [0, 6 * kNoAllocMaxBatch)   measured ranges of A, w, B per product
//   then kSplitMaxTiles         arrival counters of split tiles
//   then                        split-tile scratch for kSplitMaxWorkgroups parts
constexpr int64_t kNoAllocStatsInts = 6 * (int64_t)LWP_NOALLOC_MAX_BATCH;
constexpr int64_t kNoAllocInts = kNoAllocStatsInts + kSplitMaxTiles + (int64_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart;
static __device__ __align__(256) int32_t scratch[kNoAllocInts];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each GPU, once known

// Device address of this GPU's copy of `scratch` (the array's name is only a host-side handle).
// `device` must be the current device.
hipError_t scratch_on_device(int device, int32_t** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = static_cast<int32_t*>(ptr);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

}  // namespace

namespace lwp {
// Set-up hook for lwp_create: looks the scratch array up on the context's device, so that a later
// lwp_eliminate_node_noalloc on that device finds everything ready.
hipError_t prepare_noalloc_scratch(int device) {
    int32_t* p = nullptr;
    return scratch_on_device(device, &p);
}
}  // namespace lwp

extern "C" {

lwp_status lwp_eliminate_node_noalloc(void* hip_stream, int32_t batch, int32_t Ci, int32_t Cj, int32_t Ck,
                                      const int32_t* d_A, const int32_t* d_w, const int32_t* d_B,
                                      int32_t* d_out, int32_t* d_argmin, int32_t* d_status) {
    const NodeCall c{batch, Ci, Cj, Ck, d_A, d_w, d_B, d_out, d_argmin};
    if (lwp_status s = check_node_call(nullptr, c)) return s;
    if (((uintptr_t)d_status) & 3) return LWP_E_INVAL;
    if (batch > LWP_NOALLOC_MAX_BATCH) return LWP_E_TOO_LARGE;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return LWP_E_HIP;
    int32_t* base = nullptr;
    if (scratch_on_device(device, &base) != hipSuccess) { (void)hipGetLastError(); return LWP_E_HIP; }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int32_t* counters = base + kNoAllocStatsInts;
    // the array keeps what the last call left: the ranges are initialised by the measuring pass; the
    // counters are zero after every complete launch, and are cleared here in case one was cut short
    if (launch_fill_i32(counters, kSplitMaxTiles, 0, st) != hipSuccess) { (void)hipGetLastError(); return LWP_E_HIP; }
    const NodeScratch sc{base, counters + kSplitMaxTiles, counters, d_status, nullptr};
    if (enqueue_node_measured(c, sc, st) != hipSuccess) { (void)hipGetLastError(); return LWP_E_HIP; }
    return LWP_OK;
}

// ---- Eq. 2 -------------------------------------------------------------------------------------
lwp_status lwp_eliminate_node(lwp_ctx* ctx, int32_t batch, int32_t Ci, int32_t Cj, int32_t Ck,
                              const int32_t* d_A, const int32_t* d_w, const int32_t* d_B,
                              int32_t* d_out, int32_t* d_argmin) {
    if (lwp_status s = check_ctx(ctx)) return s;
    const NodeCall c{batch, Ci, Cj, Ck, d_A, d_w, d_B, d_out, d_argmin};
    if (lwp_status s = check_node_call(ctx, c)) return s;
    if (lwp_status s = ensure_state(ctx)) return s;
    if (ctx->wave_kernel && wave_call(c, kWaveMaxUpdates)) {
        const NodeScratch sc{nullptr, nullptr, nullptr, ctx->dstate, ctx->dstate + 1};
        ScopedTimer tm(ctx, 0, (int64_t)batch * Ci * Cj * Ck, false);
        LWP_HIP(ctx, enqueue_node_wave(c, sc, nullptr, ctx->stream));
        return LWP_OK;
    }
    if (lwp_status s = ensure_workspace(ctx, 6 * (size_t)batch * sizeof(int32_t))) return s;
    if (lwp_status s = ensure_split_buffers(ctx)) return s;
    const NodeScratch sc{reinterpret_cast<int32_t*>(ctx->ws), ctx->split,
                         ctx->split + (size_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart, ctx->dstate, ctx->dstate + 1};
    ScopedTimer tm(ctx, 0, (int64_t)batch * Ci * Cj * Ck, false);
    LWP_HIP(ctx, enqueue_node_measured(c, sc, ctx->stream));
    return LWP_OK;
}

lwp_status lwp_eliminate_node_bounded(lwp_ctx* ctx, int32_t batch, int32_t Ci, int32_t Cj, int32_t Ck,
                                      const int32_t* d_A, const int32_t* d_w, const int32_t* d_B,
                                      int32_t* d_out, int32_t* d_argmin, const int32_t* bounds) {
    if (lwp_status s = check_ctx(ctx)) return s;
    const NodeCall c{batch, Ci, Cj, Ck, d_A, d_w, d_B, d_out, d_argmin};
    if (lwp_status s = check_node_call(ctx, c)) return s;
    if (!bounds) return fail(ctx, LWP_E_INVAL, "null bounds");
    const Range rA{bounds[0], bounds[1]}, rw{bounds[2], bounds[3]}, rB{bounds[4], bounds[5]};
    if (rA.lo > rA.hi || rw.lo > rw.hi || rB.lo > rB.hi) return fail(ctx, LWP_E_INVAL, "a promised range is empty");
    if (!fits(rA.lo + rw.lo + rB.lo) || !fits(rA.hi + rw.hi + rB.hi) || !fits(rA.lo + rw.lo) || !fits(rA.hi + rw.hi))
        return fail(ctx, LWP_E_OVERFLOW, "A + w + B may leave int32 within the promised ranges");
    if (lwp_status s = ensure_state(ctx)) return s;
    // (a call of at most four 64 x 64 tiles with long rows stays there up to the general limit: with so
    // few tiles the tiled kernel cannot spread the rows over the chip -- 64 x 16384 x 64: 107 against 167 us)
    const int64_t tiles64 = (int64_t)((Ci + 63) / 64) * ((Ck + 63) / 64) * batch;
    if (ctx->wave_kernel && wave_call(c, tiles64 <= kWaveFewTiles ? kWaveMaxUpdates : kWaveMaxUpdatesBounded)) {
        const NodeScratch sc{nullptr, nullptr, nullptr, ctx->dstate, ctx->dstate + 1};
        const int64_t promised[6] = {rA.lo, rA.hi, rw.lo, rw.hi, rB.lo, rB.hi};
        ScopedTimer tm(ctx, 0, (int64_t)batch * Ci * Cj * Ck, false);
        LWP_HIP(ctx, enqueue_node_wave(c, sc, promised, ctx->stream));
        return LWP_OK;
    }
    if (lwp_status s = ensure_split_buffers(ctx)) return s;
    const NodeScratch sc{nullptr, ctx->split, ctx->split + (size_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart,
                         ctx->dstate, ctx->dstate + 1};
    // the host knows the ranges, so it picks the variant: packed keys on the preferred tile size if
    // the spread allows, else on 128 x 128 tiles (one more bit) if those still fill the chip, else
    // keys re-based per row, else compare/select; without an argmin output the minimum-only variant
    const bool prefer_small = want_small_tiles(Ci, Cj, Ck, batch);
    const bool value_only = (d_argmin == nullptr);
    const int64_t spread = (rA.hi + rw.hi - rA.lo - rw.lo) + (rB.hi - rB.lo);   // promised ranges need not be attained
    const bool keyed = !value_only && (spread <= kKeyedMaxSpreadSmall ||
                       (spread <= kKeyedMaxSpreadLarge && (!prefer_small || large_tiles(Ci, Ck, batch) >= 512)));
    const bool keyed_row = !value_only && !keyed && keyed_row_spread(rB) <= kKeyedMaxSpreadSmall &&
                           keyed_row_pays(Ci, Cj, Ck, batch);
    const bool small = keyed_row || (prefer_small && (value_only || spread <= kKeyedMaxSpreadSmall || !keyed));
    NodeArgs a{};
    a.base.loA = (int32_t)rA.lo; a.base.hiA = (int32_t)rA.hi; a.base.loW = (int32_t)rw.lo; a.base.hiW = (int32_t)rw.hi;
    a.base.loB = (int32_t)rB.lo; a.base.hiB = (int32_t)rB.hi;
    fill_common(a, c, sc, small);
    const int mode = value_only ? kModeValue : (keyed ? kModeKeyed : (keyed_row ? kModeKeyedRow : kModePlain));
    ScopedTimer tm(ctx, 0, (int64_t)batch * Ci * Cj * Ck, keyed || keyed_row);
    LWP_HIP(ctx, launch_minplus(a, mode, small, ctx->stream, /*verify=*/true));
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
    if (lwp_status s = ensure_state(ctx)) return s;
    const int64_t cells = (int64_t)batch * Ci * Cj;
    ScopedTimer tm(ctx, 1, cells, false);
    LWP_HIP(ctx, launch_edge_sum_pair(d_e1, d_e2, d_out, cells, ctx->dstate, ctx->stream));
    return LWP_OK;
}

}  // extern "C"
