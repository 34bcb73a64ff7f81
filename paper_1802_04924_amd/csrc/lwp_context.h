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
// Measured: splitting pays while tiles x parts stays around 1024 workgroups (4 per compute unit).
// A launch of more tiles runs in rounds of kWorkgroupSlots workgroups; if its last round is less than
// half full, the tiles of that round are shared instead, so that the round ends sooner (a launch of
// 4160 tiles would otherwise take five rounds for the work of 4.06).  A compute unit works a tile off
// in the same time however many workgroups keep it company (the kernel is bound by instruction
// issue), so a launch really takes as long as the compute unit with the most tiles: of a last round
// that is more than half full, the tiles left over once every compute unit has had the same number
// of whole ones are shared (576 tiles of 512 candidates: 90 -> 69 us).
constexpr int64_t kWorkgroupSlots = 1024;      // 256 compute units x 4 resident workgroups of 64 x 64 tiles
constexpr int64_t kComputeUnits = 256;
inline Split choose_split(int64_t tiles, int32_t Cj, bool small_tiles) {
    if (!small_tiles) return {1, tiles};
    const int64_t nstages = (Cj + 31) / 32;
    int64_t shared = tiles <= kSplitMaxTiles ? tiles : tiles % kWorkgroupSlots;
    if (shared > kSplitMaxTiles) shared %= kComputeUnits;
    if (shared == 0 || shared > kSplitMaxTiles) return {1, tiles};
    // parts per tile: enough for a part on every compute unit, no more (more parts only add to the
    // merging: one 512^3 product 19.8 -> 18.4 us with 4 instead of 8, two 28.6 -> 26.0 with 2), or
    // the few more that put the same number of parts on every compute unit (192 tiles: 2 parts each
    // make 384 = one or two per unit, 4 make three per unit: 38 -> 32 us)
    int64_t fill = std::max<int64_t>(2, (kComputeUnits + shared - 1) / shared);
    for (int64_t k2 = 2; k2 <= kSplitMaxParts; ++k2)
        if ((shared * k2) % kComputeUnits == 0) { fill = std::max(fill, k2); break; }   // the same number of parts on every compute unit
    const int64_t k = std::min<int64_t>({kSplitMaxParts, kSplitMaxWorkgroups / shared, nstages / 2, fill});
    if (k < 2) return {1, tiles};
    return {(int)k, tiles - shared};
}

}  // namespace lwp
