// Analytic cost model (Sec. 5.1): the three cost functions t_c(l,c), t_s(l,c), t_x(e,c_i,c_j)
// evaluated for every layer / configuration (pair).  The paper measures t_c on the device and
// derives t_x and t_s from "data to be moved / bandwidth"; this file uses closed forms:
//   t_c = work / (degree * device rate), t_s = replicated parameter bytes / bandwidth,
//   t_x = bytes the consumer's parts read from OTHER devices / bandwidth.
// All arithmetic is integer (int64 intermediates, half-up rounding), so results are exact.
//
// t_x is not evaluated as a double loop over (producer part, consumer part).  Because the
// producer's parts partition its output tensor, the volume read by all consumer parts is a
// product of per-dimension sums; what stays on the same device is subtracted part by part
// (a producer part shares a device with at most one consumer part).
//
// With a device graph (Sec. 4: every connection (d_i, d_j) has its own bandwidth; lwp_build_cost_tables_graph)
// a transfer's time depends on both of its ends, so the volume between every pair of parts is
// weighted by L / b(u, v), L the least common multiple of the bandwidths (the sum of fractions stays
// an exact integer until one final division): the consumer's parts are walked dimension by dimension
// and whole subtrees without overlap are skipped.  t_c may then come from the caller's measurements.
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "lwp.h"
#include "lwp_context.h"

namespace {

enum { KIND_CONV = 0, KIND_POOL = 1, KIND_FC = 2 };

__host__ __device__ inline long long div_round(long long num, long long den) { return (num + den / 2) / den; }

__device__ inline bool row_valid(const lwp_layer& L, const lwp_config& c, int n_devices) {
    if (c.n <= 0 || c.h <= 0 || c.w <= 0 || c.c <= 0) return false;
    if (c.n > L.N || c.c > L.Cout || c.h > L.Hout || c.w > L.Wout) return false;
    if (L.kind == KIND_FC && (c.h != 1 || c.w != 1)) return false;
    const long long d = (long long)c.n * c.h * c.w * c.c;
    return c.dev_offset >= 0 && c.dev_offset + d <= n_devices;
}

struct Span { long long lo, hi; };
__device__ inline Span split(int t, int g, int D) { return {(long long)t * D / g, (long long)(t + 1) * D / g}; }
__device__ inline Span window(Span o, int s, int p, int k, int Din) {
    const long long lo = o.lo * s - p, hi = (o.hi - 1) * s - p + k;
    return {lo < 0 ? 0 : lo, hi > Din ? Din : hi};
}
__device__ inline long long common(Span a, Span b) {
    const long long lo = a.lo > b.lo ? a.lo : b.lo, hi = a.hi < b.hi ? a.hi : b.hi;
    return hi > lo ? hi - lo : 0;
}
// what consumer part index t (of g) reads along one spatial axis of its input
__device__ inline Span spatial_need(const lwp_layer& L, bool height, int t, int g) {
    if (L.kind == KIND_FC) return {0, height ? L.Hin : L.Win};
    return height ? window(split(t, g, L.Hout), L.sh, L.ph, L.kh, L.Hin)
                  : window(split(t, g, L.Wout), L.sw, L.pw, L.kw, L.Win);
}

// Where layer l finds its configurations and its rows: configurations cfgs[cfg_off .. + C),
// outputs t_c, t_s at element out_off.  One shared list: cfg_off = 0 for every layer.
struct LayerSlice { int64_t cfg_off, out_off; int32_t C, pad; };

// grid: x over the configurations of a layer, y = layer
__global__ void node_costs_kernel(const lwp_layer* __restrict__ layers, const LayerSlice* __restrict__ slices,
                                  const lwp_config* __restrict__ cfgs, lwp_machine m,
                                  int32_t* __restrict__ tc, int32_t* __restrict__ ts, int32_t* __restrict__ flag) {
    const LayerSlice sl = slices[blockIdx.y];
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= sl.C) return;
    const int64_t x = sl.out_off + r;
    const lwp_layer L = layers[blockIdx.y];
    const lwp_config c = cfgs[sl.cfg_off + r];
    long long work, params;
    if (L.kind == KIND_CONV) {
        work = 6ll * L.N * L.Cout * L.Hout * L.Wout * L.Cin * L.kh * L.kw;
        params = 4ll * ((long long)L.Cout * L.Cin * L.kh * L.kw + L.Cout);
    } else if (L.kind == KIND_FC) {
        const long long fan_in = (long long)L.Cin * L.Hin * L.Win;
        work = 6ll * L.N * fan_in * L.Cout;
        params = 4ll * (fan_in * L.Cout + L.Cout);
    } else {
        work = 2ll * L.N * L.Cout * L.Hout * L.Wout * L.kh * L.kw;
        params = 0;
    }
    long long vc = m.invalid_cost, vs = 0;
    if (row_valid(L, c, m.n_devices)) {
        const long long degree = (long long)c.n * c.h * c.w * c.c;
        const long long replicas = (long long)c.n * c.h * c.w;
        vc = div_round(work, degree * m.flop_per_ns);
        vs = div_round(params * (replicas - 1), replicas * m.byte_per_ns);
    }
    if (vc > 2147483647ll || vs > 2147483647ll) atomicOr(flag, 1);
    tc[x] = (int32_t)vc;
    ts[x] = (int32_t)vs;
}

// grid: x over consumer configurations, y over producer configurations (both sized for the
// largest list), z = edge; table e starts at element tx_off[e]
__global__ void edge_costs_kernel(const lwp_layer* __restrict__ layers, const LayerSlice* __restrict__ slices,
                                  const int32_t* __restrict__ edges, const int64_t* __restrict__ tx_off,
                                  const lwp_config* __restrict__ cfgs, lwp_machine m,
                                  int32_t* __restrict__ tx, int32_t* __restrict__ flag) {
    const int e = blockIdx.z;
    const int b = blockIdx.x * blockDim.x + threadIdx.x;     // consumer configuration
    const int a = blockIdx.y;                                // producer configuration
    const LayerSlice sa = slices[edges[2 * e]], sb = slices[edges[2 * e + 1]];
    if (a >= sa.C || b >= sb.C) return;
    const lwp_layer P = layers[edges[2 * e]];
    const lwp_layer Q = layers[edges[2 * e + 1]];
    const lwp_config ca = cfgs[sa.cfg_off + a], cb = cfgs[sb.cfg_off + b];
    long long cells = 0;
    if (row_valid(P, ca, m.n_devices) && row_valid(Q, cb, m.n_devices)) {
        // volume read by all consumer parts, wherever it lives
        long long vol_c = (Q.kind == KIND_POOL) ? Q.Cin : (long long)cb.c * Q.Cin;
        long long vol_h = 0, vol_w = 0;
        for (int t = 0; t < cb.h; ++t) { const Span s = spatial_need(Q, true, t, cb.h); vol_h += s.hi - s.lo; }
        for (int t = 0; t < cb.w; ++t) { const Span s = spatial_need(Q, false, t, cb.w); vol_w += s.hi - s.lo; }
        const long long everything = (long long)Q.N * vol_c * vol_h * vol_w;
        // minus what a consumer part finds on its own device
        long long local = 0;
        const int da = ca.n * ca.h * ca.w * ca.c, db = cb.n * cb.h * cb.w * cb.c;
        for (int p = 0; p < da; ++p) {
            const int q = ca.dev_offset + p - cb.dev_offset;
            if (q < 0 || q >= db) continue;
            int r = p;
            const int pc = r % ca.c; r /= ca.c;
            const int pw = r % ca.w; r /= ca.w;
            const int ph = r % ca.h; const int pn = r / ca.h;
            r = q;
            const int qc = r % cb.c; r /= cb.c;
            const int qw = r % cb.w; r /= cb.w;
            const int qh = r % cb.h; const int qn = r / cb.h;
            const Span need_c = (Q.kind == KIND_POOL) ? split(qc, cb.c, Q.Cout) : Span{0, Q.Cin};
            local += common(split(pn, ca.n, P.N), split(qn, cb.n, Q.N)) *
                     common(split(pc, ca.c, P.Cout), need_c) *
                     common(split(ph, ca.h, P.Hout), spatial_need(Q, true, qh, cb.h)) *
                     common(split(pw, ca.w, P.Wout), spatial_need(Q, false, qw, cb.w));
        }
        cells = everything - local;
    }
    const long long v = div_round(4 * cells, m.byte_per_ns);
    if (v > 2147483647ll) atomicOr(flag, 1);
    tx[tx_off[e] + (int64_t)a * sb.C + b] = (int32_t)v;
}

// ---- device graph ----------------------------------------------------------------------------
// wgt [n_devices][n_devices] = L / b(u, v) (0 on the diagonal); measured (optional) replaces the
// analytic t_c of usable configurations.
struct GraphArgs { const int32_t* wgt; const int32_t* measured; int64_t L; int32_t n_devices, flop_per_ns, invalid_cost, pad; };

__device__ inline void part_index(const lwp_config& c, int p, int& in, int& ih, int& iw, int& ic) {
    ic = p % c.c; p /= c.c;
    iw = p % c.w; p /= c.w;
    ih = p % c.h; in = p / c.h;
}

__global__ void node_costs_graph_kernel(const lwp_layer* __restrict__ layers, const LayerSlice* __restrict__ slices,
                                        const lwp_config* __restrict__ cfgs, GraphArgs g,
                                        int32_t* __restrict__ tc, int32_t* __restrict__ ts, int32_t* __restrict__ flag) {
    const LayerSlice sl = slices[blockIdx.y];
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= sl.C) return;
    const int64_t x = sl.out_off + r;
    const lwp_layer L = layers[blockIdx.y];
    const lwp_config c = cfgs[sl.cfg_off + r];
    long long work, params;
    if (L.kind == KIND_CONV) {
        work = 6ll * L.N * L.Cout * L.Hout * L.Wout * L.Cin * L.kh * L.kw;
        params = 4ll * ((long long)L.Cout * L.Cin * L.kh * L.kw + L.Cout);
    } else if (L.kind == KIND_FC) {
        const long long fan_in = (long long)L.Cin * L.Hin * L.Win;
        work = 6ll * L.N * fan_in * L.Cout;
        params = 4ll * (fan_in * L.Cout + L.Cout);
    } else {
        work = 2ll * L.N * L.Cout * L.Hout * L.Wout * L.kh * L.kw;
        params = 0;
    }
    long long vc = g.invalid_cost, vs = 0;
    if (row_valid(L, c, g.n_devices)) {
        const int replicas = c.n * c.h * c.w;
        if (g.measured) {
            vc = g.measured[x];
            if (vc < 0) atomicOr(flag, 2);
        } else vc = div_round(work, (long long)replicas * c.c * g.flop_per_ns);
        // the holders of one channel part's parameters sit c devices apart; every one of them sends an
        // r-th of its gradients to each of the others, and the slowest sender finishes last
        for (int ic = 0; ic < c.c; ++ic)
            for (int s = 0; s < replicas; ++s) {
                const int u = c.dev_offset + s * c.c + ic;
                long long inv = 0;
                for (int t = 0; t < replicas; ++t)
                    if (t != s) inv += g.wgt[(int64_t)u * g.n_devices + c.dev_offset + t * c.c + ic];
                const long long v = div_round(params * inv, (long long)replicas * g.L);
                vs = v > vs ? v : vs;
            }
    }
    if (vc > 2147483647ll || vs > 2147483647ll) atomicOr(flag, 1);
    tc[x] = (int32_t)vc;
    ts[x] = (int32_t)vs;
}

__global__ void edge_costs_graph_kernel(const lwp_layer* __restrict__ layers, const LayerSlice* __restrict__ slices,
                                        const int32_t* __restrict__ edges, const int64_t* __restrict__ tx_off,
                                        const lwp_config* __restrict__ cfgs, GraphArgs g,
                                        int32_t* __restrict__ tx, int32_t* __restrict__ flag) {
    const int e = blockIdx.z;
    const int b = blockIdx.x * blockDim.x + threadIdx.x;     // consumer configuration
    const int a = blockIdx.y;                                // producer configuration
    const LayerSlice sa = slices[edges[2 * e]], sb = slices[edges[2 * e + 1]];
    if (a >= sa.C || b >= sb.C) return;
    const lwp_layer P = layers[edges[2 * e]];
    const lwp_layer Q = layers[edges[2 * e + 1]];
    const lwp_config ca = cfgs[sa.cfg_off + a], cb = cfgs[sb.cfg_off + b];
    long long scaled = 0;                                    // sum of elements * L / b(u, v)
    if (row_valid(P, ca, g.n_devices) && row_valid(Q, cb, g.n_devices)) {
        const int da = ca.n * ca.h * ca.w * ca.c;
        for (int p = 0; p < da; ++p) {
            int pn, ph, pw, pc;
            part_index(ca, p, pn, ph, pw, pc);
            const Span tn = split(pn, ca.n, P.N), th = split(ph, ca.h, P.Hout), tw = split(pw, ca.w, P.Wout),
                       tcs = split(pc, ca.c, P.Cout);
            const int32_t* wrow = g.wgt + (int64_t)(ca.dev_offset + p) * g.n_devices + cb.dev_offset;
            for (int qn = 0; qn < cb.n; ++qn) {
                const long long on = common(tn, split(qn, cb.n, Q.N));
                if (!on) continue;
                for (int qh = 0; qh < cb.h; ++qh) {
                    const long long oh = on * common(th, spatial_need(Q, true, qh, cb.h));
                    if (!oh) continue;
                    for (int qw = 0; qw < cb.w; ++qw) {
                        const long long ow = oh * common(tw, spatial_need(Q, false, qw, cb.w));
                        if (!ow) continue;
                        for (int qc = 0; qc < cb.c; ++qc) {
                            const Span need_c = (Q.kind == KIND_POOL) ? split(qc, cb.c, Q.Cout) : Span{0, Q.Cin};
                            // the weight of a device with itself is 0: what is local costs nothing
                            scaled += ow * common(tcs, need_c) * wrow[((qn * cb.h + qh) * cb.w + qw) * cb.c + qc];
                        }
                    }
                }
            }
        }
    }
    const long long v = div_round(4 * scaled, g.L);
    if (v > 2147483647ll) atomicOr(flag, 1);
    tx[tx_off[e] + (int64_t)a * sb.C + b] = (int32_t)v;
}

}  // namespace

namespace {

struct GraphHost { std::vector<int32_t> wgt; int64_t L; const int32_t* measured; int64_t rows; };

// cfg_rows: total rows in cfgs.  shared: every layer uses rows [0, Cn[0]).  graph (optional): weights
// of a device graph and measured t_c; machine->byte_per_ns is then unused.
lwp_status build_tables(lwp_ctx* ctx, const lwp_layer* layers, int32_t n_layers, const int32_t* edges,
                        int32_t n_edges, const lwp_config* cfgs, const int32_t* Cn, bool shared,
                        const lwp_machine* machine, int32_t* d_tc, int32_t* d_ts, int32_t* d_tx,
                        const GraphHost* graph = nullptr) {
    if (machine->n_devices < 1 || machine->flop_per_ns < 1 || machine->byte_per_ns < 1 || machine->invalid_cost < 0)
        return lwp::fail(ctx, LWP_E_INVAL, "machine constants must be positive");
    for (int32_t l = 0; l < n_layers; ++l) {
        const lwp_layer& L = layers[l];
        if (L.kind < KIND_CONV || L.kind > KIND_FC) return lwp::fail(ctx, LWP_E_INVAL, "unknown layer kind");
        if (L.N < 1 || L.Cin < 1 || L.Hin < 1 || L.Win < 1 || L.Cout < 1 || L.Hout < 1 || L.Wout < 1 || L.kh < 1 ||
            L.kw < 1 || L.sh < 1 || L.sw < 1 || L.ph < 0 || L.pw < 0)
            return lwp::fail(ctx, LWP_E_INVAL, "layer extents must be positive");
        if (Cn[l] < 1 || Cn[l] > 65535) return lwp::fail(ctx, LWP_E_INVAL, "a layer needs 1..65535 configurations");
    }
    for (int32_t e = 0; e < n_edges; ++e) {
        const int32_t p = edges[2 * e], q = edges[2 * e + 1];
        if (p < 0 || p >= n_layers || q < 0 || q >= n_layers || p == q)
            return lwp::fail(ctx, LWP_E_GRAPH, "edge endpoint out of range");
        const lwp_layer &P = layers[p], &Q = layers[q];
        if (P.N != Q.N || P.Cout != Q.Cin || P.Hout != Q.Hin || P.Wout != Q.Win)
            return lwp::fail(ctx, LWP_E_INVAL, "producer output and consumer input shapes differ");
    }
    std::vector<LayerSlice> slices((size_t)n_layers);
    std::vector<int64_t> tx_off((size_t)(n_edges > 0 ? n_edges : 1));
    int64_t rows = 0, cfg_rows = 0;
    int32_t c_max = 1;
    for (int32_t l = 0; l < n_layers; ++l) {
        slices[l] = {shared ? 0 : rows, rows, Cn[l], 0};
        rows += Cn[l];
        c_max = Cn[l] > c_max ? Cn[l] : c_max;
    }
    cfg_rows = shared ? Cn[0] : rows;
    int64_t cells = 0;
    for (int32_t e = 0; e < n_edges; ++e) { tx_off[e] = cells; cells += (int64_t)Cn[edges[2 * e]] * Cn[edges[2 * e + 1]]; }

    hipStream_t st = ctx->stream;
    const size_t bl = (size_t)n_layers * sizeof(lwp_layer), bs = (size_t)n_layers * sizeof(LayerSlice),
                 bc = (size_t)cfg_rows * sizeof(lwp_config), be = (size_t)(n_edges > 0 ? n_edges : 1) * 2 * sizeof(int32_t),
                 bo = tx_off.size() * sizeof(int64_t);
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    const size_t off_s = up(bl), off_c = off_s + up(bs), off_e = off_c + up(bc), off_o = off_e + up(be), off_f = off_o + up(bo);
    const size_t bw_bytes = graph ? graph->wgt.size() * sizeof(int32_t) : 0;
    const size_t bm_bytes = (graph && graph->measured) ? (size_t)rows * sizeof(int32_t) : 0;
    const size_t off_w = off_f + 256, off_m = off_w + up(bw_bytes);
    char* d = nullptr;
    if (hipMalloc(&d, off_m + up(bm_bytes) + 256) != hipSuccess) { (void)hipGetLastError(); return lwp::fail(ctx, LWP_E_NOMEM, "descriptor upload buffer"); }
    lwp_status result = LWP_OK;
    int32_t flag = 0;
    hipError_t herr = hipSuccess;
    auto ok = [&](hipError_t e) { if (e != hipSuccess && herr == hipSuccess) herr = e; return e == hipSuccess; };
    if (ok(hipMemcpyAsync(d, layers, bl, hipMemcpyHostToDevice, st)) &&
        ok(hipMemcpyAsync(d + off_s, slices.data(), bs, hipMemcpyHostToDevice, st)) &&
        ok(hipMemcpyAsync(d + off_c, cfgs, bc, hipMemcpyHostToDevice, st)) &&
        (n_edges == 0 || ok(hipMemcpyAsync(d + off_e, edges, (size_t)n_edges * 2 * sizeof(int32_t), hipMemcpyHostToDevice, st))) &&
        (n_edges == 0 || ok(hipMemcpyAsync(d + off_o, tx_off.data(), (size_t)n_edges * sizeof(int64_t), hipMemcpyHostToDevice, st))) &&
        (bw_bytes == 0 || ok(hipMemcpyAsync(d + off_w, graph->wgt.data(), bw_bytes, hipMemcpyHostToDevice, st))) &&
        (bm_bytes == 0 || ok(hipMemcpyAsync(d + off_m, graph->measured, bm_bytes, hipMemcpyHostToDevice, st))) &&
        ok(hipMemsetAsync(d + off_f, 0, sizeof(int32_t), st))) {
        const lwp_layer* dl = reinterpret_cast<const lwp_layer*>(d);
        const LayerSlice* ds = reinterpret_cast<const LayerSlice*>(d + off_s);
        const lwp_config* dc = reinterpret_cast<const lwp_config*>(d + off_c);
        const int32_t* de = reinterpret_cast<const int32_t*>(d + off_e);
        const int64_t* dof = reinterpret_cast<const int64_t*>(d + off_o);
        int32_t* df = reinterpret_cast<int32_t*>(d + off_f);
        GraphArgs ga{};
        if (graph)
            ga = {reinterpret_cast<const int32_t*>(d + off_w), bm_bytes ? reinterpret_cast<const int32_t*>(d + off_m) : nullptr,
                  graph->L, machine->n_devices, machine->flop_per_ns, machine->invalid_cost, 0};
        for (int32_t l0 = 0; l0 < n_layers && herr == hipSuccess; l0 += 65535) {
            const int32_t nl = (n_layers - l0) < 65535 ? (n_layers - l0) : 65535;
            if (graph)
                hipLaunchKernelGGL(node_costs_graph_kernel, dim3((c_max + 255) / 256, nl), dim3(256), 0, st, dl + l0, ds + l0,
                                   dc, ga, d_tc, d_ts, df);
            else
                hipLaunchKernelGGL(node_costs_kernel, dim3((c_max + 255) / 256, nl), dim3(256), 0, st, dl + l0, ds + l0, dc,
                                   *machine, d_tc, d_ts, df);
            ok(hipGetLastError());
        }
        for (int32_t e0 = 0; e0 < n_edges && herr == hipSuccess; e0 += 65535) {
            const int32_t ne = (n_edges - e0) < 65535 ? (n_edges - e0) : 65535;
            if (graph)
                hipLaunchKernelGGL(edge_costs_graph_kernel, dim3((c_max + 63) / 64, c_max, ne), dim3(64), 0, st, dl, ds,
                                   de + 2 * (size_t)e0, dof + e0, dc, ga, d_tx, df);
            else
                hipLaunchKernelGGL(edge_costs_kernel, dim3((c_max + 255) / 256, c_max, ne), dim3(256), 0, st, dl, ds,
                                   de + 2 * (size_t)e0, dof + e0, dc, *machine, d_tx, df);
            ok(hipGetLastError());
        }
        ok(hipMemcpyAsync(&flag, df, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    }
    ok(hipStreamSynchronize(st));
    (void)hipFree(d);
    if (herr != hipSuccess) return lwp::fail(ctx, LWP_E_HIP, hipGetErrorString(herr));
    if (flag & 2) result = lwp::fail(ctx, LWP_E_INVAL, "a measured t_c is negative");
    else if (flag) result = lwp::fail(ctx, LWP_E_OVERFLOW, "a cost does not fit int32 nanoseconds");
    return result;
}

}  // namespace

extern "C" lwp_status lwp_build_cost_tables(lwp_ctx* ctx, const lwp_layer* layers, int32_t n_layers,
                                            const int32_t* edges, int32_t n_edges, const lwp_config* cfgs,
                                            int32_t C, const lwp_machine* machine,
                                            int32_t* d_tc, int32_t* d_ts, int32_t* d_tx) {
    if (!ctx) return LWP_E_INVAL;
    if (lwp_status rc = lwp::check_ctx(ctx)) return rc;
    if (!layers || !cfgs || !machine || !d_tc || !d_ts || (n_edges > 0 && (!edges || !d_tx)))
        return lwp::fail(ctx, LWP_E_INVAL, "null pointer");
    if (n_layers < 1 || n_edges < 0 || C < 1 || C > 65535)
        return lwp::fail(ctx, LWP_E_INVAL, "bad sizes");
    const std::vector<int32_t> Cn((size_t)n_layers, C);
    return build_tables(ctx, layers, n_layers, edges, n_edges, cfgs, Cn.data(), true, machine, d_tc, d_ts, d_tx);
}

extern "C" lwp_status lwp_build_cost_tables_ragged(lwp_ctx* ctx, const lwp_layer* layers, int32_t n_layers,
                                                   const int32_t* edges, int32_t n_edges, const lwp_config* cfgs,
                                                   const int32_t* C_node, const lwp_machine* machine,
                                                   int32_t* d_tc, int32_t* d_ts, int32_t* d_tx) {
    if (!ctx) return LWP_E_INVAL;
    if (lwp_status rc = lwp::check_ctx(ctx)) return rc;
    if (!layers || !cfgs || !C_node || !machine || !d_tc || !d_ts || (n_edges > 0 && (!edges || !d_tx)))
        return lwp::fail(ctx, LWP_E_INVAL, "null pointer");
    if (n_layers < 1 || n_edges < 0) return lwp::fail(ctx, LWP_E_INVAL, "bad sizes");
    return build_tables(ctx, layers, n_layers, edges, n_edges, cfgs, C_node, false, machine, d_tc, d_ts, d_tx);
}

// Sec. 4: the device graph gives every connection (d_i, d_j) its own bandwidth; Sec. 5.1: t_c is
// measured on the device.  See the header for the readings.
extern "C" lwp_status lwp_build_cost_tables_graph(lwp_ctx* ctx, const lwp_layer* layers, int32_t n_layers,
                                                  const int32_t* edges, int32_t n_edges, const lwp_config* cfgs,
                                                  const int32_t* C_node, const lwp_device_graph* dg,
                                                  const int32_t* measured_tc,
                                                  int32_t* d_tc, int32_t* d_ts, int32_t* d_tx) {
    if (!ctx) return LWP_E_INVAL;
    if (lwp_status rc = lwp::check_ctx(ctx)) return rc;
    if (!layers || !cfgs || !C_node || !dg || !dg->bandwidth || !d_tc || !d_ts || (n_edges > 0 && (!edges || !d_tx)))
        return lwp::fail(ctx, LWP_E_INVAL, "null pointer");
    if (n_layers < 1 || n_edges < 0) return lwp::fail(ctx, LWP_E_INVAL, "bad sizes");
    if (dg->n_devices < 1 || dg->n_devices > 4096) return lwp::fail(ctx, LWP_E_INVAL, "a device graph has 1..4096 devices");
    const int32_t D = dg->n_devices;
    GraphHost gh;
    gh.L = 1;
    auto gcd = [](int64_t a, int64_t b) { while (b) { const int64_t t = a % b; a = b; b = t; } return a; };
    for (int32_t u = 0; u < D; ++u)
        for (int32_t v = 0; v < D; ++v) {
            if (u == v) continue;
            const int64_t b = dg->bandwidth[(size_t)u * D + v];
            if (b < 1) return lwp::fail(ctx, LWP_E_INVAL, "every connection of the device graph needs a positive bandwidth");
            gh.L = gh.L / gcd(gh.L, b) * b;
            if (gh.L > (1 << 20))
                return lwp::fail(ctx, LWP_E_INVAL, "the bandwidths have no common multiple below 2^20 (exact sums of transfer times need one)");
        }
    gh.wgt.assign((size_t)D * D, 0);
    for (int32_t u = 0; u < D; ++u)
        for (int32_t v = 0; v < D; ++v)
            if (u != v) gh.wgt[(size_t)u * D + v] = (int32_t)(gh.L / dg->bandwidth[(size_t)u * D + v]);
    gh.measured = measured_tc;
    const lwp_machine m{dg->n_devices, dg->flop_per_ns, 1, dg->invalid_cost};
    return build_tables(ctx, layers, n_layers, edges, n_edges, cfgs, C_node, false, &m, d_tc, d_ts, d_tx, &gh);
}

// Sec. 4 / Table 1: a configuration gives a degree of parallelism to every parallelizable
// dimension of the layer's output (sample, height, width, channel; a fully connected layer has
// only sample and channel), partitions being equal.  Enumerated here: power-of-two degrees whose
// product d fits the machine and that do not exceed the layer's extents, on every device block
// [k*d, (k+1)*d).  Ascending (n, h, w, c, offset).
extern "C" lwp_status lwp_enumerate_configs(const lwp_layer* layer, int32_t n_devices, lwp_config* out,
                                            int32_t capacity, int32_t* count) {
    if (!layer || !count || n_devices < 1 || capacity < 0 || (capacity > 0 && !out)) return LWP_E_INVAL;
    if (layer->kind < KIND_CONV || layer->kind > KIND_FC || layer->N < 1 || layer->Cout < 1 || layer->Hout < 1 ||
        layer->Wout < 1)
        return LWP_E_INVAL;
    const bool fc = layer->kind == KIND_FC;
    int64_t found = 0;
    for (int64_t n = 1; n <= n_devices && n <= layer->N; n <<= 1)
        for (int64_t h = 1; n * h <= n_devices && h <= (fc ? 1 : layer->Hout); h <<= 1)
            for (int64_t w = 1; n * h * w <= n_devices && w <= (fc ? 1 : layer->Wout); w <<= 1)
                for (int64_t c = 1; n * h * w * c <= n_devices && c <= layer->Cout; c <<= 1) {
                    const int64_t degree = n * h * w * c;
                    for (int64_t block = 0; (block + 1) * degree <= n_devices; ++block, ++found)
                        if (found < capacity) out[found] = {(int32_t)n, (int32_t)h, (int32_t)w, (int32_t)c, (int32_t)(block * degree), 0};
                }
    if (found > 2147483647ll) return LWP_E_INVAL;
    *count = (int32_t)found;
    return LWP_OK;
}
