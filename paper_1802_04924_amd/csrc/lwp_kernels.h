// Device-side entry points of the strategy search, as host-callable launchers.
// Every launcher only enqueues on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace lwp {

// ---- node elimination (Eq. 2) --------------------------------------------------------------
// One product of a batched launch.  [loX, hiX] are ranges the caller guarantees for the entries
// of A, w and B; rngA / rngB optionally point at a measured {min, max} pair in device memory
// (written by the launch that produced the table, earlier on the same stream) and can only
// tighten them; rngW likewise for w.  rngOut, if set, receives {min, max} of `out` by atomics and must have been
// initialised to {INT32_MAX, INT32_MIN}.  The packed-key variant needs
//   min(hiA + hiW - loA - loW, (hiA - loA) + (hiB - loB) + 1) + (hiB - loB) <= kKeyedMaxSpread*.
struct NodeDesc {
    const int32_t* A;
    const int32_t* w;
    const int32_t* B;
    int32_t* out;
    int32_t* arg;      // may be null
    int32_t loA, hiA, loW, hiW, loB, hiB;
    const int32_t* rngA;
    const int32_t* rngB;
    const int32_t* rngW;
    int32_t* rngOut;
    int32_t* flag;     // optional: OR-ed with 1 if max A + max w + max B (measured) may leave int32
                       // (2: a promised range broken, 4: skipped by a speculative launch; see NodeArgs)
    int32_t Ci, Cj, Ck;   // shape of this product; read only by launches of mixed shapes
    // Output cells of the products before this one within the round a search runs it in (saturating
    // at 2^30).  Read only by the single-workgroup search, which deals a round's cells to its threads.
    int32_t cell_begin;
    int32_t pad[2];
};
static_assert(sizeof(NodeDesc) == 128, "descriptor layout");

struct NodeArgs {
    const NodeDesc* descs;   // device array [batch], or null for strided addressing
    NodeDesc base;           // strided addressing: product 0
    int64_t sA, sw, sB, sO;  // strided addressing: element strides between products
    int64_t sR;              // strided addressing: int32 elements between the products' measured range pairs
                             // (base.rngA / rngW / rngB point at product 0's pairs; 0 = one pair for all)
    int32_t Ci, Cj, Ck, batch;
    int32_t tilesM, tilesN;  // output tiles of the chosen tile size per product
    // Mixed shapes (64 x 64 tiles, descriptor addressing only): product q has its own shape in
    // descs[q] and owns tiles [tile_begin[q], tile_begin[q+1]) of the launch; tile_begin is a
    // device array of batch + 1 ascending entries and total_tiles = tile_begin[batch].  Ci, Cj, Ck,
    // tilesM and tilesN above are then ignored.
    const int32_t* tile_begin;
    int32_t total_tiles;
    // Split tiles (64 x 64 tiles only): with kparts > 1 the launch's first n_whole tiles have one
    // workgroup each and every later ("shared") tile has kparts workgroups.  scratch holds
    // shared tiles * kparts * 2 * 16 * 256 int32; counters one zeroed int32 per shared tile (left zeroed).
    int32_t kparts, n_whole;
    int32_t* scratch;
    int32_t* counters;
    // kModeAuto: the variant is decided on the device, per product, from the measured ranges (see
    // auto_variant in minplus.hip).  auto_limit: largest spread packed keys on global offsets may
    // have at this launch's tile size; auto_row: keys re-based per row are among the candidates.
    int32_t auto_row;
    // kModeKeyed launched without knowing the ranges: a product whose measured ranges do not allow
    // packed keys is skipped -- its outputs are NOT written -- and 4 is OR-ed into its `flag`
    int32_t speculative;
    int64_t auto_limit;
    // optional: element `mode` is incremented once per product that this launch works on
    int32_t* mode_count;
    // non-zero: nothing is known or has been measured about the values; every workgroup takes the
    // ranges of the strips of A and B and of the w its tile reads, in place of the descriptor's bounds
    // and measured ranges (which are ignored).  Not with promised ranges (verify).
    int32_t self_measure;
};
constexpr int64_t kSplitScratchIntsPerPart = 2 * 16 * 256;
// Capacity of the split-tile buffers every caller of launch_minplus provides: scratch for
// kSplitMaxWorkgroups parts, one counter for each of kSplitMaxTiles tiles.  A split launch must
// stay within both (the launcher refuses one that does not).
constexpr int kSplitMaxParts = 8, kSplitMaxWorkgroups = 1024, kSplitMaxTiles = 512;

constexpr int kTileLarge = 128, kTileSmall = 64, kNodeThreads = 256;
// largest spread the packed keys can hold: 27 bits with 128 x 128 tiles (16-deep stages), 26 bits
// with 64 x 64 tiles (32-deep stages)
constexpr int64_t kKeyedMaxSpreadLarge = (1ll << 27) - 2, kKeyedMaxSpreadSmall = (1ll << 26) - 2;

// mode: packed keys (needs the spread bound above), plain int32 compare/select (any values), or
// value-only (minimum without argmin, any values; `arg` is ignored).  small_tiles selects 64 x 64
// output tiles instead of 128 x 128; tilesM / tilesN in args must match.
// kModeKeyedRow: packed keys whose A side is re-based per output row (64 x 64 tiles only): needs
//   2 * (hiB - loB) + 1 <= kKeyedMaxSpreadSmall and nothing of A or w beyond A + w fitting int32.
// kModeAuto: keyed, keyed per row or plain, picked per product on the device from the ranges the
//   descriptors point at (args.auto_limit, args.auto_row); mode_count then counts by picked variant.
constexpr int kModeKeyed = 0, kModePlain = 1, kModeValue = 2, kModeKeyedRow = 3, kModeAuto = 4;
// verify: the ranges in the descriptors are promises of the caller, not measurements (they need not
// be attained, and rngA / rngW / rngB must be null).  The kernel then checks every element of A, w
// and B it stages against them and ORs 2 into `flag` on a violation (results are then meaningless
// but every access stays in bounds); the keyed variant needs
//   (hiA + hiW - loA - loW) + (hiB - loB) <= kKeyedMaxSpread*.
// Strided addressing only, not with mixed shapes.
hipError_t launch_minplus(const NodeArgs& args, int mode, bool small_tiles, hipStream_t stream, bool verify = false);

// The same product for launches too small for the tiled kernel: one wavefront per 8 x 8 (rb = 1) or
// 16 x 16 (rb = 2) output tile, nothing shared between wavefronts.  mode: kModePlain or kModeValue.
// Addressing as launch_minplus (descriptors or strides; descriptors must carry Ci / Cj / Ck), with
// tile counts in units of this kernel's tiles: tilesM / tilesN per product for one shape, or
// tile_begin (batch + 1 ascending entries) for mixed shapes; total_tiles = all tiles of the launch.
// flag, rngOut and mode_count behave as in launch_minplus (overflow is judged from the values each
// wavefront stages, not from the descriptors' ranges, which are ignored); rngOut is best left null
// unless a consumer needs the measured range (thousands of wavefronts then share two atomics);
// no split tiles (kparts <= 1).
// h_descs (optional, with descriptor addressing): a host copy of args.descs[0 .. batch); its first
// kWaveInlineDescs entries are passed in the kernel arguments and not read from device memory.
// verify: the descriptors' ranges are promises of the caller; every wavefront compares the values
// it stages with them and ORs 2 into `flag` on a violation (all of A, w and B is staged by some
// wavefront of the product).
constexpr int kWaveInlineDescs = 6;
hipError_t launch_minplus_wave(const NodeArgs& args, const NodeDesc* h_descs, int mode, int rb, hipStream_t stream,
                               bool verify = false);
// When a launch goes to this kernel (measured on MI355X, launches back to back): its cell updates
// together stay below kWaveMaxUpdates -- beyond that the tiled kernel's arithmetic rate wins over its
// start-up latency.  (However long the products' rows: a launch within that limit with many candidates
// has few tiles, and then four wavefronts share each.)  A caller that promises value ranges gets the
// tiled kernel's packed keys in a single launch without any measuring pass, which is faster from
// kWaveMaxUpdatesBounded on.  Tile size: with at least kWaveFillTiles tiles of 16 x 16 those are used
// (every SIMD still gets two wavefronts' worth); so are they when there are few of them (up to
// kWaveSplitTiles16, which four wavefronts share each) and rows are long enough that a quarter of
// the candidates still fills a wavefront's pipeline -- a 16 x 16 tile loads half as much per update;
// else 8 x 8 (four times as many, smaller pieces to spread over the chip).
constexpr int64_t kWaveMaxUpdates = (int64_t)3 << 25, kWaveMaxUpdatesBounded = (int64_t)1 << 25;
constexpr int64_t kWaveFewTiles = 4;       // calls with promised ranges and at most this many 64 x 64 tiles: kWaveMaxUpdates
constexpr int64_t kWaveFillTiles = 2048;
// four wavefronts per tile: a launch of at most this many tiles of 8 x 8, or of 16 x 16
constexpr int kWaveSplitTiles = 1024, kWaveSplitTiles16 = 1536;
constexpr int64_t kWaveSharedMinTiles = 64, kWaveSharedMinCj = 200;
// mean_cj: candidates per output cell, averaged over the launch
inline int wave_tile_rb(int64_t tiles_16x16, int64_t mean_cj) {
    if (tiles_16x16 >= kWaveFillTiles) return 2;
    if (tiles_16x16 > kWaveSharedMinTiles && tiles_16x16 <= kWaveSplitTiles16 && mean_cj >= kWaveSharedMinCj) return 2;
    return 1;
}

// ---- edge elimination (Eq. 3) --------------------------------------------------------------
// out = sum of n_src tables of `cells` elements.  srcs indexes a device array of table pointers.
struct EdgeDesc {
    int32_t* out;
    int32_t* rngOut;     // optional {min, max} of out, by atomics (see NodeDesc)
    int32_t* flag;       // optional: OR-ed with 1 if a sum leaves int32
    int64_t cells;       // elements of every table of this group
    int32_t first_src;   // index into the pointer array
    int32_t n_src;
};
// max_cells: the largest `cells` among the descriptors (sizes the grid).
hipError_t launch_edge_sum_desc(const EdgeDesc* d_descs, const int32_t* const* d_src_ptrs, int32_t n_desc,
                                int64_t max_cells, hipStream_t stream);
// flag (optional) is OR-ed with 1 if a sum leaves int32 (the wrapped sum is stored).
hipError_t launch_edge_sum_pair(const int32_t* e1, const int32_t* e2, int32_t* out, int64_t cells, int32_t* flag,
                                hipStream_t stream);

// p[0..n) = value (a fill kernel: also safe inside a captured graph, unlike a memset node).
hipError_t launch_fill_i32(int32_t* d_p, int64_t n, int32_t value, hipStream_t stream);
// dst[0..bytes) = src[0..bytes) by a kernel (bytes a multiple of 16, both 16-byte aligned); src may be
// pinned host memory the device can read.  For small blocks on the critical path of a search: a
// runtime copy of more than a few kilobytes goes through the DMA engine and takes about 15 us.
hipError_t launch_copy_block(const void* src, void* dst, size_t bytes, hipStream_t stream);

// ---- value ranges ----------------------------------------------------------------------------
// One launch that prepares a search: stats[2*t] = INT32_MAX, stats[2*t+1] = INT32_MIN for
// t < n_tables; *flag = 0 (if given); keys[k] = all ones for k < n_keys (if given).
hipError_t launch_init_workspace(int32_t* d_stats, int32_t n_tables, int32_t* d_flag, unsigned long long* d_keys,
                                 int32_t n_keys, hipStream_t stream);
// stats[2*t] = min, stats[2*t+1] = max of table t (tables of `cells` elements each, dense one
// after another), by atomics onto initialised pairs: for t < n_tables, or, if d_which (device array of
// n_tables table numbers) is given, for the tables it lists.
hipError_t launch_ranges(const int32_t* d_tables, int32_t n_tables, int64_t cells, int32_t* d_stats,
                         hipStream_t stream, const int32_t* d_which = nullptr);
// The same for tables of different sizes: table t is elements [d_off[t], d_off[t+1]) of d_tables
// (d_off: device array of offsets, one more than there are tables); max_cells sizes the grid.
hipError_t launch_ranges_var(const int32_t* d_tables, const int64_t* d_off, int32_t n_tables, int64_t max_cells,
                             int32_t* d_stats, hipStream_t stream, const int32_t* d_which = nullptr);
// First launch of a search: w = tc + ts, row by row; row v is elements [v*C, (v+1)*C), or
// [d_node_off[v], d_node_off[v+1]) if d_node_off (device, n_nodes + 1 offsets) is given.  Stats pair
// w_pair0 + v receives {min, max} of row v of w, or {INT32_MAX, INT32_MIN} if a sum of that row
// leaves int32; all other of the n_pairs stats pairs are initialised for atomic min/max and
// keys[0..n_keys) to all ones.  *d_flag (optional) is set to 0.
// Optionally the launch also copies up_bytes (a multiple of 16, both addresses 16-byte aligned) from
// up_src -- pinned host memory the device can read -- to up_dst: a small descriptor block then needs no
// copy of its own.  The range must not hold d_node_off (other workgroups of the launch read that).
hipError_t launch_prepare_search(const int32_t* tc, const int32_t* ts, int32_t* w, int32_t n_nodes, int32_t C,
                                 const int64_t* d_node_off, int32_t* d_stats, int32_t n_pairs, int32_t w_pair0,
                                 unsigned long long* d_keys, int32_t n_keys, int32_t* d_flag, hipStream_t stream,
                                 const void* up_src = nullptr, void* up_dst = nullptr, size_t up_bytes = 0);

// ---- residual graph and back-substitution (Alg. 1, enumeration of the final graph and undo) --
struct PairDesc {       // residual component with two nodes joined by one edge
    const int32_t* T;   // [Ci][Ck]
    const int32_t* wi;  // t_c + t_s of the source node [Ci]
    const int32_t* wk;  // of the destination node [Ck]
    int32_t src, dst, Ci, Ck;
};
struct SingleDesc {     // residual isolated node
    const int32_t* w;   // [C]
    int32_t node, C;
};
// Residual component with K > 2 nodes: all strategies are enumerated (their number <= 2^32).  Node
// q of the component is digit q of the flat strategy index (radix Cn[q]), digit 0 (lowest node id)
// most significant.  Edge x joins digits src_pos[x] -> dst_pos[x] with table tab[x]
// [Cn[src_pos[x]]][Cn[dst_pos[x]]].
constexpr int kCompMaxNodes = 12, kCompMaxEdges = 32;
struct CompDesc {
    const int32_t* tab[kCompMaxEdges];
    const int32_t* w[kCompMaxNodes];
    int32_t node[kCompMaxNodes];
    int32_t Cn[kCompMaxNodes];
    int8_t src_pos[kCompMaxEdges], dst_pos[kCompMaxEdges];
    int32_t K, n_edges;
};
struct UndoDesc {       // one node elimination of the log
    const int32_t* arg; // [Ci][Ck] stored argmin, or null: recompute from the three tables below
    const int32_t* A;   // table of the in-edge (i,j) at the time of the elimination [Ci][Cj]
    const int32_t* w;   // t_c + t_s of node j [Cj]
    const int32_t* B;   // table of the out-edge (j,k) [Cj][Ck]
    int32_t j, i, k, round;
    int32_t Cj, Ck;
    int32_t first;      // index of the first entry of this entry's round (entries are ordered by round)
    int32_t pad;
};
static_assert(sizeof(UndoDesc) == 64, "descriptor layout");
// keys[p] is a 64-bit (cost, flat index) minimum per component, initialised to all ones.
// d_flag (optional) is OR-ed with 1 if a sum leaves int32.  max_rows / max_c size the grids.
hipError_t launch_pair_min(const PairDesc* d_pairs, int32_t n_pairs, int32_t max_rows,
                           unsigned long long* d_keys, int32_t* d_flag, hipStream_t stream);
hipError_t launch_single_min(const SingleDesc* d_singles, int32_t n_singles, int32_t max_c,
                             unsigned long long* d_keys /* after the pairs */, hipStream_t stream);
// One launch per component; n_prefix = product of Cn[0..K-2]; key = d_keys[index of the component].
hipError_t launch_component_min(const CompDesc* d_comp, unsigned long long n_prefix,
                                unsigned long long* d_key, int32_t* d_flag, hipStream_t stream);
// Decodes the component minima (keys: pairs, then singles, then enumerated components), then
// walks the undo list backwards (entries of one round are independent).
// result[0] = total cost low word, result[1] = high word, result[2..2+n_nodes) = strategy,
// result[2+n_nodes] = *d_flag (0 if d_flag is null), OR 1 if one of the n_nodes stats pairs starting
// at d_wstats is the impossible {INT32_MAX, INT32_MIN} (a row of t_c + t_s left int32).
// h_result (optional): pinned host memory the device can write; receives a copy of the 3 + n_nodes
// result words before the kernel ends.
hipError_t launch_back_substitute(const PairDesc* d_pairs, int32_t n_pairs, const SingleDesc* d_singles,
                                  int32_t n_singles, const CompDesc* d_comps, int32_t n_comps,
                                  const unsigned long long* d_keys,
                                  const UndoDesc* d_undo, int32_t n_undo, int32_t n_nodes,
                                  const int32_t* d_flag, const int32_t* d_wstats, int32_t* d_result,
                                  int32_t* h_result, hipStream_t stream);

// ---- a whole small search in one launch (one workgroup) -------------------------------------------
// The descriptors are those of the general path; rounds[r] names the edge-sum groups and the node
// eliminations of round r (ranges into `edges` / `nodes`).  NodeDesc.Ci/Cj/Ck and cell_begin must be
// set; ranges, rngOut and per-descriptor flags are ignored (overflow is found exactly and OR-ed into
// *flag, which the kernel first clears).  w receives t_c + t_s for all n_w entries.  Every table a
// descriptor points at must lie in w, in tx (the caller's tables) or in slots (the intermediate
// ones): the kernel works on copies of the three regions in LDS.  keys: one per component.
// result / host_result as launch_back_substitute.
// A descriptor block of at most kTinyInlineBytes can travel in the kernel arguments instead of device
// memory (inline_block = 1): the search then needs no upload before its one launch.  The eight
// descriptor pointers (rounds ... undo) are then byte offsets into that block, cast to pointers.
constexpr int kTinyInlineBytes = 3584;
// All tables of such a search together (t_c + t_s rows, the caller's t_x, the intermediate tables) must
// fit this many words: the workgroup keeps them in LDS.
constexpr int kTinyLdsWords = 32768;
struct TinyRound { int32_t g0, g1, n0, n1; };
struct TinyArgs {
    const int32_t* tc;
    const int32_t* ts;
    int32_t* w;
    int64_t n_w;
    const int32_t* tx;       // the caller's edge tables, and the intermediate tables: where they start
    const int32_t* slots;    // and how many words they have
    int64_t n_tx, n_slots;
    const TinyRound* rounds;
    int32_t n_rounds;
    const NodeDesc* nodes;
    const EdgeDesc* edges;
    const int32_t* const* srcs;
    const PairDesc* pairs;
    const SingleDesc* singles;
    const CompDesc* comps;
    int32_t n_pairs, n_singles, n_comps;
    unsigned long long* keys;
    const UndoDesc* undo;
    int32_t n_undo, n_nodes;
    int32_t* flag;
    int32_t* result;
    int32_t* host_result;
    int32_t inline_block;
    int32_t up_n16;          // set by launch_tiny_search: 16-byte words of the descriptor block the kernel
    const void* up_src;      // copies from up_src (host, pinned) to up_dst (device) before it starts
    void* up_dst;
};
// d_block / h_block: the descriptor block on the device (what the pointers in args point into) and its
// host copy, block_bytes long.  If h_block is given and the block is small enough it is passed in the
// kernel arguments and the device copy is not read (it need not have been uploaded).
constexpr bool tiny_block_fits_arguments(size_t block_bytes) { return block_bytes <= (size_t)kTinyInlineBytes; }
// A larger block (of whole 16-byte words, up to a megabyte) the kernel copies itself from h_block (pinned
// host memory) to d_block; only a block that is neither needs uploading before the launch.
constexpr bool tiny_block_copied_by_kernel(size_t block_bytes) { return block_bytes % 16 == 0 && block_bytes <= ((size_t)1 << 20); }
hipError_t launch_tiny_search(const TinyArgs& args, const void* d_block, const void* h_block, size_t block_bytes,
                              hipStream_t stream);

// ---- VALU issue-rate probe ---------------------------------------------------------------------
// `blocks` workgroups of 256 threads each run `iters` iterations of a register-only add + three-way
// min loop; per iteration and thread alu_probe_instr_per_iter() VALU instructions that perform the
// arithmetic of alu_probe_updates_per_iter() cell updates.  d_out: one uint32 (never written in
// practice).
hipError_t launch_alu_probe(uint32_t* d_out, int blocks, int iters, hipStream_t stream);
int alu_probe_instr_per_iter();
int alu_probe_updates_per_iter();

}  // namespace lwp
