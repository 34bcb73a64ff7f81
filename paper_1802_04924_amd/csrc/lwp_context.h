// The library's context and the helpers every translation unit behind the C ABI shares: error
// recording, the context's growing device workspace and pinned staging buffer, the split-tile
// buffers, launch timing, and the policy that picks a min-plus kernel variant.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <string>
#include <vector>

#include "lwp.h"
#include "lwp_kernels.h"

struct lwp_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;
    char* ws = nullptr;        // device workspace
    size_t ws_bytes = 0;
    char* pin = nullptr;       // pinned host staging (descriptor upload, small read-backs)
    size_t pin_bytes = 0;
    int32_t* split = nullptr;  // scratch + per-tile counters of split tiles (see minplus.hip)
    // device words of the single-step entry points, which only enqueue: [0] error bits set by their
    // kernels (1: a sum may leave int32, 2: an element outside the ranges the caller promised),
    // reported and cleared by lwp_synchronize; [1 + mode] products that ran on each kernel variant
    int32_t* dstate = nullptr;
    int32_t* hstate = nullptr;     // pinned host word lwp_synchronize reads the error bits back through
    // a search on this context met tables too wide for packed keys on global offsets: later searches
    // do not try those first (see Search::run)
    bool keys_failed = false;
    bool single_launch = true;     // LWP_OPT_SINGLE_LAUNCH
    bool wave_kernel = true;       // LWP_OPT_SMALL_PRODUCT_KERNEL
    bool profiling = false;
    struct Timed { hipEvent_t a, b; int kind; int64_t work; bool keyed; };
    std::vector<Timed> timed;
    lwp_profile prof{};
};

namespace lwp {

constexpr int64_t kI32Max = 2147483647LL, kI32Min = -2147483648LL;
constexpr int kMaxConfigs = 65536;

// Records `why` as the context's last error and returns `s`.
lwp_status fail(lwp_ctx* ctx, lwp_status s, const std::string& why);

#define LWP_HIP(ctx, call)                                                                     \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return ::lwp::fail(ctx, e_ == hipErrorOutOfMemory ? LWP_E_NOMEM : LWP_E_HIP,       \
                               std::string(#call) + ": " + hipGetErrorString(e_));             \
    } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Clears the last error and makes the context's device current.
lwp_status check_ctx(lwp_ctx* ctx);
// Grow-only buffers of the context (a growth synchronises the stream and reallocates).
lwp_status ensure_workspace(lwp_ctx* ctx, size_t bytes);
lwp_status ensure_pinned(lwp_ctx* ctx, size_t bytes);
// Scratch and arrival counters of split tiles, allocated on first use; set_split points a
// launch at them.
// How a launch's tiles are split: the first n_whole tiles have one workgroup each, the others kparts.
struct Split { int kparts; int64_t n_whole; };
lwp_status ensure_split_buffers(lwp_ctx* ctx);
// Looks up, once per device, the scratch array of the entry point that allocates nothing
// (lwp_eliminate.cpp); `device` must be current.
hipError_t prepare_noalloc_scratch(int device);
constexpr int kStateInts = 8;
lwp_status ensure_state(lwp_ctx* ctx);
void set_split(lwp_ctx* ctx, NodeArgs& a, Split split);

// Brackets one launch with HIP events while profiling is on (kind 0: node elimination with
// `work` cell updates, kind 1: edge elimination with `work` cells).
struct ScopedTimer {
    lwp_ctx* ctx;
    size_t idx = (size_t)-1;
    ScopedTimer(lwp_ctx* c, int kind, int64_t work, bool keyed);
    ~ScopedTimer();
};
// Synchronises and folds the recorded events into ctx->prof.
lwp_status drain_profile(lwp_ctx* ctx);

// ---- choice of the min-plus kernel variant -----------------------------------------------------
struct Range { int64_t lo, hi; };
inline bool fits(int64_t v) { return v >= kI32Min && v <= kI32Max; }

// The same for keys re-based per output row: the row's minimum re-bases to 0 and everything more
// than B's spread above it is clamped, so only B's spread counts.
inline int64_t keyed_row_spread(Range rB) { return 2 * (rB.hi - rB.lo) + 1; }
// Their extra pass over A pays once a launch is bound by arithmetic rather than by latency
// (measured: no gain for launches of a few 163^3 products, 2.3x for 2048^3).
inline bool keyed_row_pays(int32_t Ci, int32_t Cj, int32_t Ck, int64_t batch) {
    return (int64_t)Ci * Cj * Ck * batch >= ((int64_t)1 << 28);
}

// Tile choice.  Measured on MI355X the 64 x 64 variant (4 waves per SIMD, 32-deep stages) matches or
// beats the 128 x 128 variant except for launches of very many tiles (batches of thousands of
// products), where its four times as many workgroup start-ups cost about 1 %; it also quantises a
// launch four times finer, which matters when a launch is only a few waves of workgroups.
inline int64_t large_tiles(int32_t Ci, int32_t Ck, int64_t batch) {
    return (int64_t)((Ci + kTileLarge - 1) / kTileLarge) * ((Ck + kTileLarge - 1) / kTileLarge) * batch;
}
inline bool want_small_tiles(int32_t Ci, int32_t Cj, int32_t Ck, int64_t batch) {
    (void)Cj;
    return large_tiles(Ci, Ck, batch) < 2048;
}

// Split tiles: a launch with few 64 x 64 tiles lets several workgroups share a tile, each with a
// part of the c range of at least two stages of 32 candidates.
// The kernel is bound by instruction issue: a compute unit works a tile off in the same time however
// many workgroups keep it company (512 candidates: 21 us), so a launch takes as long as the compute
// unit with the most tiles -- measured: 512 tiles 63 us, 576 to 768 tiles 86, 832 to 1024 106.  A
// launch of more tiles than compute units therefore gives every unit the same number of whole tiles
// and shares the tiles left over (a launch of 4160 tiles: 64 of them), with the number of parts that
// spreads them most evenly; each further part adds to the merging, which the small term below stands
// for.  (576 tiles: 90 -> 69 us; 320: 53 -> 43; 1344: 139 -> 130.)
// Up to two tiles per compute unit in whole rounds, all tiles are shared, by the same rule (one 512^3
// product, 64 tiles: 19.8 -> 18.4 us with 4 parts instead of 8; 192 tiles: 4 parts instead of 2, 38 -> 32 us).
constexpr int64_t kComputeUnits = 256;
inline Split choose_split(int64_t tiles, int32_t Cj, bool small_tiles) {
    if (!small_tiles) return {1, tiles};
    const int64_t nstages = (Cj + 31) / 32;
    const bool leftover = tiles > kComputeUnits && tiles % kComputeUnits != 0;
    // (two whole tiles per unit come out slightly behind four halves: 64 against 62 us)
    const int64_t shared = leftover ? tiles % kComputeUnits : (tiles <= kSplitMaxTiles ? tiles : 0);
    if (shared == 0) return {1, tiles};
    const int64_t kmax = std::min<int64_t>({kSplitMaxParts, kSplitMaxWorkgroups / shared, nstages / 2});
    // time of the shared tiles in units of one tile's: the compute unit with the most parts (a part is
    // a whole number of stages), plus a little for every further part to merge.  Leftover tiles may also stay whole (one more tile's
    // time); a launch of at most a tile per unit is always split (a lone workgroup does not keep a
    // compute unit busy).
    // (A compute unit with one workgroup runs at 0.77 of the rate it reaches with four, with two at
    // 0.95: slopes of launch time over the number of candidates, 64 / 256 / 1024 tiles.)
    int64_t k = 1;
    double best = leftover ? 1.0 : 1e9;
    const int64_t whole_per_unit = (tiles - shared) / kComputeUnits;
    for (int64_t q = 2; q <= kmax; ++q) {
        const int64_t parts = (shared * q + kComputeUnits - 1) / kComputeUnits;      // on the fullest unit
        const int64_t resident = whole_per_unit + parts;
        const double rate = resident >= 3 ? 1.0 : (resident == 2 ? 0.95 : 0.77);
        const double part = (double)((nstages + q - 1) / q) / (double)nstages;        // of a tile: whole stages
        const double cost = (double)parts * part / rate + 0.03 * (double)(q - 1);
        if (cost < best - 1e-9) { best = cost; k = q; }
    }
    if (k < 2) return {1, tiles};
    return {(int)k, tiles - shared};
}

}  // namespace lwp
