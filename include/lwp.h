/*
 * lwp.h -- C ABI of the layer-wise-parallelism strategy search for one AMD MI355X (gfx950).
 *
 * The library finds, for a computation graph whose nodes are layers and whose edges are
 * tensors, one parallelization configuration per layer minimising the cost model of the
 * paper (Sec. 5.1, Eq. 1) with the graph search of Sec. 5.2 (Alg. 1): node eliminations
 * (Eq. 2), edge eliminations (Eq. 3), solution of the small residual graph and undoing the
 * eliminations in reverse order.
 *
 * Conventions
 *   - All costs are int32 nanoseconds.  Sums are exact; every minimum takes the LOWEST index
 *     among equal candidates.  A sum that could leave int32 is refused (LWP_E_OVERFLOW): for a
 *     node elimination the test is max A + max w + max B (and the minima) over the tables' actual
 *     value ranges, measured on the device; edge sums and the residual-graph sums are tested
 *     element by element.  The test is sufficient, not necessary.
 *   - A cost table of an edge e = (l_i, l_j) is row-major [cfg of l_i][cfg of l_j].
 *   - "DEVICE" pointers are HIP device memory on the context's device, owned by the caller;
 *     the library never frees or keeps them.  "HOST" pointers are ordinary host memory.
 *   - Every kernel is enqueued on the context's stream.  lwp_eliminate_node, _node_bounded and
 *     lwp_eliminate_edge only enqueue and return (the first call of a size may grow a buffer of
 *     the context, which waits for the stream once); what their kernels find on the device -- a
 *     sum that may leave int32, a value outside promised ranges -- is reported by the next
 *     lwp_synchronize.  lwp_build_cost_tables returns after the stream has drained; a search
 *     returns once its last kernel has delivered the result to the host (the kernel writes it
 *     into pinned memory, the status word last, and the host waits for that word): nothing of
 *     the search is still reading the caller's tables then, though the kernel may not have
 *     retired yet -- later work on the stream is ordered behind it as usual.
 *   - Errors are return codes; on error the outputs are untouched unless stated.  Argument
 *     and graph validation happen before any GPU work.  lwp_last_error gives the reason.
 *   - A context must not be used from two threads at once.
 */
#ifndef LWP_H
#define LWP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lwp_ctx lwp_ctx;

typedef enum {
    LWP_OK = 0,
    LWP_E_INVAL = -1,          /* null pointer, non-positive size, misaligned pointer        */
    LWP_E_GRAPH = -2,          /* endpoint out of range, self loop, cycle                    */
    LWP_E_NOT_REDUCIBLE = -3,  /* a residual component is too large to enumerate             */
    LWP_E_OVERFLOW = -4,       /* the tables' value ranges do not keep every sum inside int32 */
    LWP_E_NOMEM = -5,          /* device or host allocation failed                           */
    LWP_E_HIP = -6,            /* a HIP runtime call failed                                  */
    LWP_E_TOO_LARGE = -7       /* a size exceeds the fixed capacity of lwp_eliminate_node_noalloc */
} lwp_status;

/* Order of eliminations (the paper leaves the choice open, Alg. 2 "if there exists ...").
 * Every round first merges all parallel edges (E-phase), then eliminates nodes (N-phase):
 *   LWP_SCHEDULE_ROUNDS     scan nodes in ascending id, take every eligible node none of whose
 *                           two neighbours was taken in this round; all taken nodes are
 *                           eliminated by one batched launch;
 *   LWP_SCHEDULE_LEFT_FOLD  take only the lowest-id eligible node per round;
 *   LWP_SCHEDULE_NONE       eliminate nothing: the baseline the paper compares its algorithm with
 *                           (Sec. 5.2, last paragraph; Table 3), which finds the optimum of the
 *                           ORIGINAL graph by enumerating every strategy.  Each connected component
 *                           is enumerated on the device like a residual component (same limits:
 *                           12 nodes, 32 edges, 2^32 strategies); among equal optima the
 *                           lexicographically lowest strategy, lower node id more significant. */
typedef enum { LWP_SCHEDULE_ROUNDS = 0, LWP_SCHEDULE_LEFT_FOLD = 1, LWP_SCHEDULE_NONE = 2 } lwp_schedule;

/* ---- context --------------------------------------------------------------------------- */

/* Creates a context bound to HIP device `device` and stream `hip_stream` (a hipStream_t cast
 * to void*, NULL = the default stream).  The context owns a device workspace that grows on
 * demand and is released by lwp_destroy. */
lwp_status lwp_create(lwp_ctx **out, int device, void *hip_stream);
void lwp_destroy(lwp_ctx *ctx);
/* Human-readable reason of the last failure on ctx; valid until the next call on ctx. */
const char *lwp_last_error(const lwp_ctx *ctx);
const char *lwp_status_string(lwp_status s);
/* Blocks until the context's stream has drained, then reports what the kernels of
 * lwp_eliminate_node, lwp_eliminate_node_bounded and lwp_eliminate_edge enqueued since the last
 * lwp_synchronize found: LWP_E_OVERFLOW if a sum of one of them may have left int32,
 * LWP_E_INVAL if one met a value outside the ranges its caller promised; the outputs of such
 * an elimination are invalid.  The record is cleared by the call. */
lwp_status lwp_synchronize(lwp_ctx *ctx);

/* Options of a context.  LWP_OPT_SINGLE_LAUNCH (default 1): a search whose whole work is a few
 * hundred thousand operations and whose tables fit 32768 words together (the sizes the paper itself searches: a
 * handful of devices, tens of configurations per layer) runs as one launch of one workgroup
 * instead of a dozen dependent launches; 0 sends every search down the general path.  Results are
 * identical.
 * LWP_OPT_SMALL_PRODUCT_KERNEL (default 1): node eliminations with little work -- one call, or one
 * round of a search, below 100 million (3 * 2^25) cell updates (2^25 for a call with promised
 * ranges and more than four 64 x 64 output tiles) -- run on a kernel that gives every wavefront a
 * small output tile of its own instead of the tiled kernel, whose launch would be mostly latency
 * at that size; 0 sends every node elimination to the tiled kernel.  Results are identical; the overflow
 * test of the small-product kernel is the same formula applied to the values each wavefront reads,
 * so it is at least as tight. */
typedef enum { LWP_OPT_SINGLE_LAUNCH = 0, LWP_OPT_SMALL_PRODUCT_KERNEL = 1 } lwp_option;
lwp_status lwp_set_option(lwp_ctx *ctx, int32_t option, int32_t value);

/* ---- node elimination (Sec. 5.2, Eq. 2; argmin of Thm. 3 in the appendix) ---------------- */

/* For every b in [0,batch):
 *   out[b][a][k] = min_c ( A[b][a][c] + w[b][c] + B[b][c][k] ),  argmin[b][a][k] = lowest such c
 * A = table of the in-edge (l_i,l_j), w = t_c(l_j,.) + t_s(l_j,.), B = table of the out-edge.
 * DEVICE, dense, row-major: A [batch][Ci][Cj], w [batch][Cj], B [batch][Cj][Ck],
 * out [batch][Ci][Ck], argmin [batch][Ci][Ck] (may be NULL: then only the minimum is computed,
 * by a variant without argmin bookkeeping).  out/argmin must not overlap the inputs.  Sizes: batch, Ci, Cj, Ck >= 1, Cj <= 65536.
 * Enqueues and returns.  Nothing is assumed about the values: their ranges are measured on the
 * device -- by one pass over A, w and B of every product, or, where that is cheaper (few output
 * tiles, or products of at most two tiles a side), by every workgroup of the product kernel over
 * the rows of A, the columns of B and the w that its tile reads -- and the product kernel picks
 * its arithmetic variant from them, also on the device (a call with little work needs neither:
 * see LWP_OPT_SMALL_PRODUCT_KERNEL).  If max A + max w + max B (or the minima) over what was
 * measured could leave int32 the next lwp_synchronize returns LWP_E_OVERFLOW. */
lwp_status lwp_eliminate_node(lwp_ctx *ctx, int32_t batch, int32_t Ci, int32_t Cj, int32_t Ck,
                              const int32_t *d_A, const int32_t *d_w, const int32_t *d_B,
                              int32_t *d_out, int32_t *d_argmin);

/* The same for a caller that knows ranges of the values (cost tables come out of a cost model with
 * known bounds, Sec. 5.1): bounds HOST [6] = {lo A, hi A, lo w, hi w, lo B, hi B}, inclusive, valid
 * for every product.  The measuring pass is skipped and the host picks the kernel variant, so the
 * call costs one launch.  Returns LWP_E_OVERFLOW at once if hi A + hi w + hi B (or the minima)
 * leaves int32.  The kernel checks every element it reads against the promise; a violation makes
 * the outputs invalid and the next lwp_synchronize return LWP_E_INVAL. */
lwp_status lwp_eliminate_node_bounded(lwp_ctx *ctx, int32_t batch, int32_t Ci, int32_t Cj, int32_t Ck,
                                      const int32_t *d_A, const int32_t *d_w, const int32_t *d_B,
                                      int32_t *d_out, int32_t *d_argmin, const int32_t *bounds);

/* lwp_eliminate_node for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  No context: the kernels are enqueued on
 * hip_stream (a hipStream_t, NULL = the default stream) of the CURRENT device, and the device memory
 * they need beyond the operands -- measured ranges, arrival counters and partial results of split
 * tiles -- is a fixed array inside the library's device code (about 32.1 MiB per GPU, held from the
 * first use of the library on that GPU until the process ends).  The call itself allocates and
 * frees nothing; the array's address is looked up once per device, by lwp_create or by the first
 * call on that device.  Limits: batch <= LWP_NOALLOC_MAX_BATCH, else LWP_E_TOO_LARGE (Ci, Cj, Ck as
 * for lwp_eliminate_node).  Same results as lwp_eliminate_node, bit for bit.  Enqueues and returns.
 * d_status: DEVICE int32 owned by the caller, or NULL; bit 0 is OR-ed in if a sum of some product
 * may leave int32 (the call never clears it).  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams, or threads) race and give wrong results. */
#define LWP_NOALLOC_MAX_BATCH 4096
lwp_status lwp_eliminate_node_noalloc(void *hip_stream, int32_t batch, int32_t Ci, int32_t Cj, int32_t Ck,
                                      const int32_t *d_A, const int32_t *d_w, const int32_t *d_B,
                                      int32_t *d_out, int32_t *d_argmin, int32_t *d_status);

/* ---- edge elimination (Sec. 5.2, Eq. 3) -------------------------------------------------- */

/* out[b][i][j] = e1[b][i][j] + e2[b][i][j].  DEVICE, dense [batch][Ci][Cj]; out may alias e1 or
 * e2.  Enqueues and returns; if a sum leaves int32 (the wrapped value is stored) the next
 * lwp_synchronize returns LWP_E_OVERFLOW. */
lwp_status lwp_eliminate_edge(lwp_ctx *ctx, int32_t batch, int32_t Ci, int32_t Cj,
                              const int32_t *d_e1, const int32_t *d_e2, int32_t *d_out);

/* ---- whole search (Sec. 5.2, Alg. 1) ----------------------------------------------------- */

/* One entry of the elimination log, in execution order.
 * kind 0: node elimination of node j between i and k; in-edge e1 = (i,j), out-edge e2 = (j,k);
 *         the new edge (i,k) keeps the id e1.
 * kind 1: edge elimination; edge e2 is added into e1 (both (i,k)); the sum keeps the id e1; j = -1.
 * round: index of the schedule round the step belongs to. */
typedef struct { int32_t kind, j, i, k, e1, e2, round; } lwp_step;

/* Host-only: computes the elimination schedule of a graph (no GPU, no context).
 * edges: HOST [n_edges][2] = (src, dst), node ids in [0,n_nodes), parallel edges allowed.
 * steps: HOST, room for max(n_edges,1) entries, may be NULL.  n_steps / n_rounds / n_residual_nodes
 * may be NULL.  Returns LWP_E_GRAPH for a bad endpoint, self loop or cycle and
 * LWP_E_NOT_REDUCIBLE if a connected component of the residual graph has more than 12 nodes or
 * 32 edges (components of one node, of two nodes and one edge, and larger ones that will be
 * enumerated are all fine). */
lwp_status lwp_plan_graph(int32_t n_nodes, int32_t n_edges, const int32_t *edges, int32_t schedule,
                          lwp_step *steps, int32_t *n_steps, int32_t *n_rounds,
                          int32_t *n_residual_nodes);

/* Finds a strategy minimising Eq. 1.
 * edges HOST [n_edges][2]; every node has C configurations (1 <= C <= 65536).
 * d_tc, d_ts DEVICE [n_nodes][C]; d_tx DEVICE [n_edges][C][C]; read-only.
 * out_cost HOST int32: t_o of the returned strategy; out_strategy HOST [n_nodes]: configuration
 * index per node.  Among optimal strategies the one produced by the schedule and the
 * lowest-index rule is returned.  The residual graph (Alg. 1, "enumerating all possible
 * candidate strategies") is solved per connected component: a node, a pair joined by one edge
 * (lowest flat index of (source cfg, destination cfg)), or, for K > 2 nodes, enumeration of all
 * C^K strategies (lexicographically lowest optimum, lower node id more significant), which needs
 * C^K <= 2^32, else LWP_E_NOT_REDUCIBLE.  Blocking. */
lwp_status lwp_search_graph(lwp_ctx *ctx, int32_t n_nodes, int32_t n_edges, const int32_t *edges,
                            int32_t C, const int32_t *d_tc, const int32_t *d_ts, const int32_t *d_tx,
                            int32_t schedule, int32_t *out_cost, int32_t *out_strategy);

/* How the undo pass (Alg. 1, last loop) obtains the configuration c_j of an eliminated node:
 *   LWP_UNDO_STORED     every node elimination stores its argmin table (one int32 [C][C] each),
 *                       the undo pass looks c_j up;
 *   LWP_UNDO_RECOMPUTE  as the paper describes it (Table 2: undoing costs O(EC)): eliminations keep
 *                       only the minimum, their input tables stay alive, and the undo pass
 *                       recomputes c_j = argmin_c { A[c_i][c] + w[c] + B[c][c_k] } (lowest c).
 *                       The elimination kernel then needs no argmin bookkeeping and runs at its
 *                       full rate for any int32 value range.
 * Both return the same strategy. */
typedef enum { LWP_UNDO_STORED = 0, LWP_UNDO_RECOMPUTE = 1 } lwp_undo;
/* lwp_search_graph with the undo mode chosen by the caller (lwp_search_graph uses STORED). */
lwp_status lwp_search_graph_ex(lwp_ctx *ctx, int32_t n_nodes, int32_t n_edges, const int32_t *edges,
                               int32_t C, const int32_t *d_tc, const int32_t *d_ts, const int32_t *d_tx,
                               int32_t schedule, int32_t undo, int32_t *out_cost, int32_t *out_strategy);

/* The search when the layers' configuration sets differ in size (Sec. 3: each layer l has its own
 * set of configurations; Sec. 5 enumerates them per layer type, so e.g. a fully-connected layer has
 * fewer than a convolution).  C_node HOST [n_nodes]: node v has C_node[v] configurations
 * (1 <= C_node[v] <= 65536).  d_tc, d_ts DEVICE: the nodes' rows concatenated in node order
 * (row v has C_node[v] entries); d_tx DEVICE: the edges' tables concatenated in edge order, table e
 * row-major [C_node[src_e]][C_node[dst_e]].  Everything else as lwp_search_graph_ex, with "C^K"
 * read as the product of the component's C_node.  With all C_node equal it is the same call as
 * lwp_search_graph_ex (which is implemented by it). */
lwp_status lwp_search_graph_ragged(lwp_ctx *ctx, int32_t n_nodes, int32_t n_edges, const int32_t *edges,
                                   const int32_t *C_node, const int32_t *d_tc, const int32_t *d_ts,
                                   const int32_t *d_tx, int32_t schedule, int32_t undo,
                                   int32_t *out_cost, int32_t *out_strategy);

/* A search prepared once and run many times on tables that change in place (the cost tables are
 * re-measured or rebuilt for another batch size or machine while the graph stays; Sec. 5.1, 5.2).
 * lwp_search_plan_create fixes graph, configuration counts (as lwp_search_graph_ragged), table
 * ADDRESSES and schedule, allocates the plan's own workspace and does all host-side work --
 * schedule, buffer plan, descriptors, their upload -- once.  That is possible with recomputed
 * undo (LWP_UNDO_RECOMPUTE): value-only eliminations and device-side overflow checks leave
 * nothing for the host to decide from the tables' values.  lwp_search_plan_run enqueues the
 * launch sequence on the context's stream, waits for it and returns what lwp_search_graph_ragged
 * would return for the tables' present contents.  Blocking.  A plan belongs to its context:
 * destroy it before the context. */
typedef struct lwp_search_plan lwp_search_plan;
lwp_status lwp_search_plan_create(lwp_ctx *ctx, int32_t n_nodes, int32_t n_edges, const int32_t *edges,
                                  const int32_t *C_node, const int32_t *d_tc, const int32_t *d_ts,
                                  const int32_t *d_tx, int32_t schedule, lwp_search_plan **out);
lwp_status lwp_search_plan_run(lwp_search_plan *plan, int32_t *out_cost, int32_t *out_strategy);
void lwp_search_plan_destroy(lwp_search_plan *plan);

/* Host-only: bytes of device workspace lwp_search_graph(_ex) needs for this graph (0 on a graph it
 * would refuse). */
size_t lwp_search_workspace_bytes(int32_t n_nodes, int32_t n_edges, const int32_t *edges, int32_t C,
                                  int32_t schedule);
size_t lwp_search_workspace_bytes_ex(int32_t n_nodes, int32_t n_edges, const int32_t *edges, int32_t C,
                                     int32_t schedule, int32_t undo);
size_t lwp_search_workspace_bytes_ragged(int32_t n_nodes, int32_t n_edges, const int32_t *edges,
                                         const int32_t *C_node, int32_t schedule, int32_t undo);

/* ---- cost tables (Sec. 5.1: t_c, t_s, t_x) ----------------------------------------------- */

/* One layer: kind 0 = 2D convolution, 1 = 2D pooling, 2 = fully connected.  N = batch size;
 * input tensor N x Cin x Hin x Win, output N x Cout x Hout x Wout; kernel kh x kw, stride
 * sh x sw, padding ph x pw.  A fully connected layer reads its whole input per sample. */
typedef struct {
    int32_t kind, N, Cin, Hin, Win, Cout, Hout, Wout, kh, kw, sh, sw, ph, pw;
} lwp_layer;
/* One configuration (Sec. 4): degrees of parallelism in the sample, height, width and channel
 * dimensions of the layer's OUTPUT tensor; its n*h*w*c equal parts are placed on the devices
 * dev_offset, dev_offset+1, ... in the order ((i_n*h + i_h)*w + i_w)*c + i_c.  n == 0 marks a
 * padding row that is invalid for every layer. */
typedef struct { int32_t n, h, w, c, dev_offset, pad; } lwp_config;
typedef struct {
    int32_t n_devices;
    int32_t flop_per_ns;    /* per-device compute rate           */
    int32_t byte_per_ns;    /* bandwidth of every device link    */
    int32_t invalid_cost;   /* t_c of a configuration a layer cannot use */
} lwp_machine;

/* Evaluates the analytic cost model for every layer and configuration (pair).
 * layers HOST [n_layers]; edges HOST [n_edges][2]; cfgs HOST [C]; outputs DEVICE
 * d_tc, d_ts [n_layers][C], d_tx [n_edges][C][C].  Blocking.
 *   t_c = round(work / (n*h*w*c * flop_per_ns)), work = forward + backward operations of the layer;
 *   t_s = round(4 * parameters * (r-1) / (r * byte_per_ns)), r = n*h*w parameter replicas;
 *   t_x = round(4 * elements a consumer part reads from another device / byte_per_ns);
 *   a configuration a layer cannot use gets t_c = invalid_cost, t_s = 0 and t_x = 0.
 * Returns LWP_E_OVERFLOW if a cost exceeds int32 (the tables then hold truncated values),
 * LWP_E_INVAL if a producer's output shape differs from its consumer's input shape. */
lwp_status lwp_build_cost_tables(lwp_ctx *ctx, const lwp_layer *layers, int32_t n_layers,
                                 const int32_t *edges, int32_t n_edges, const lwp_config *cfgs,
                                 int32_t C, const lwp_machine *machine,
                                 int32_t *d_tc, int32_t *d_ts, int32_t *d_tx);

/* The same with a configuration list per layer (Sec. 4: the configurations of a layer depend on
 * its parallelizable dimensions, Table 1).  C_node HOST [n_layers]; cfgs HOST: the layers' lists
 * one after another (layer l has C_node[l] rows, 1..65535).  Outputs DEVICE in the layout
 * lwp_search_graph_ragged takes: d_tc, d_ts the layers' rows concatenated, d_tx the edges' tables
 * [C_node[src]][C_node[dst]] concatenated. */
lwp_status lwp_build_cost_tables_ragged(lwp_ctx *ctx, const lwp_layer *layers, int32_t n_layers,
                                        const int32_t *edges, int32_t n_edges, const lwp_config *cfgs,
                                        const int32_t *C_node, const lwp_machine *machine,
                                        int32_t *d_tc, int32_t *d_ts, int32_t *d_tx);

/* The cost model on a device graph (Sec. 4: each connection (d_i, d_j) has a bandwidth b(d_i, d_j);
 * Sec. 5.1, assumption 2: moving s bytes over it takes s / b) and with measured compute times
 * (Sec. 5.1: t_c is the measured time of the layer under the configuration).
 * bandwidth HOST [n_devices][n_devices]: b(u, v) in byte per ns from device u (row, the sender) to
 * device v (column), positive for u != v, the diagonal is ignored; all entries must have a common
 * multiple of at most 2^20 (the sums below are exact). */
typedef struct {
    int32_t n_devices;
    int32_t flop_per_ns;    /* per-device compute rate of the analytic t_c; unused with measured t_c */
    int32_t invalid_cost;   /* t_c of a configuration a layer cannot use                            */
    int32_t pad;
    const int32_t *bandwidth;
} lwp_device_graph;
/* Arguments and table layout as lwp_build_cost_tables_ragged.  measured_tc HOST, laid out like d_tc,
 * or NULL: if given, t_c of every configuration its layer can use is copied from it (entries must be
 * >= 0) instead of the analytic value.
 *   t_x = round( sum over (producer part on device u, consumer part on device v != u) of
 *         4 * elements the consumer part reads from the producer part / b(u, v) );
 *   t_s = max over the devices u holding parameters of round( sum over the other r - 1 devices v that
 *         hold a replica of the same parameters of (4 * parameters / r) / b(u, v) );
 * with one bandwidth for all connections both are the formulas of lwp_build_cost_tables.  Blocking. */
lwp_status lwp_build_cost_tables_graph(lwp_ctx *ctx, const lwp_layer *layers, int32_t n_layers,
                                       const int32_t *edges, int32_t n_edges, const lwp_config *cfgs,
                                       const int32_t *C_node, const lwp_device_graph *graph,
                                       const int32_t *measured_tc,
                                       int32_t *d_tc, int32_t *d_ts, int32_t *d_tx);

/* Host-only: the configurations of one layer on a machine of n_devices (Sec. 4, Table 1; equal
 * partitioning): every (n, h, w, c) of power-of-two degrees with n*h*w*c = d <= n_devices, no degree
 * above the extent it splits (N, Hout, Wout, Cout), h = w = 1 for a fully connected layer, once
 * per device block [k*d, (k+1)*d) inside the machine.  Ascending (n, h, w, c, dev_offset).
 * *count receives the number of configurations; at most `capacity` rows are written to out
 * (out may be NULL if capacity is 0). */
lwp_status lwp_enumerate_configs(const lwp_layer *layer, int32_t n_devices, lwp_config *out,
                                 int32_t capacity, int32_t *count);

/* ---- measurement ------------------------------------------------------------------------- */

/* Accumulated since the last lwp_profile_reset while profiling is on: every node-elimination
 * launch is bracketed by HIP events on the context's stream. */
typedef struct {
    int64_t node_launches;     /* min-plus kernel launches                         */
    int64_t node_cell_updates; /* sum of batch*Ci*Cj*Ck over those launches        */
    double node_ms;            /* sum of their durations (HIP events)              */
    int64_t edge_launches;
    int64_t edge_cells;
    double edge_ms;
    int64_t keyed_launches;    /* node launches that used the packed-key variant (whole searches and
                                  lwp_eliminate_node_bounded, where the host picks the variant)      */
    /* products of lwp_eliminate_node(_bounded) per kernel variant since the last reset (the variant
     * of lwp_eliminate_node is picked on the device, per product): packed keys on global offsets,
     * packed keys re-based per row, compare/select, minimum only */
    int64_t products_keyed, products_keyed_row, products_plain, products_value;
} lwp_profile;
/* Runs a register-only loop of the min-plus kernel's two inner instructions (32-bit add, three-way
 * unsigned min; no memory traffic) on every compute unit and reports the rate the device
 * sustains: VALU lane-operations per second (instructions x 64 lanes) and the cell updates per
 * second those instructions amount to (1.5 instructions per update).  The measured counterpart
 * of the datasheet-derived peak the roofline fraction is quoted against.
 * Blocking (a few milliseconds). */
lwp_status lwp_measure_valu_rate(lwp_ctx *ctx, double *lane_ops_per_s, double *cell_updates_per_s);
lwp_status lwp_profile_enable(lwp_ctx *ctx, int32_t on);
lwp_status lwp_profile_reset(lwp_ctx *ctx);
/* Synchronises the stream, then fills *out. */
lwp_status lwp_profile_read(lwp_ctx *ctx, lwp_profile *out);

#ifdef __cplusplus
}
#endif
#endif /* LWP_H */
