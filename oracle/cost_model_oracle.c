/*
 * CPU oracle of the analytic cost model (TEST INFRASTRUCTURE, not the product).
 *
 * Sec. 5.1 defines three cost functions; the paper measures t_c on the device and does not
 * print formulas for t_x and t_s beyond saying that each is a data volume divided by a known
 * bandwidth.  The readings implemented here:
 *
 *   configuration (Sec. 4): degrees (n, h, w, c) over the sample, height, width and channel
 *     dimensions of the layer's OUTPUT tensor, equal partitioning: part t of g over an extent
 *     D is [floor(t*D/g), floor((t+1)*D/g)).  The d = n*h*w*c parts sit on devices
 *     dev_offset + ((i_n*h + i_h)*w + i_w)*c + i_c.  A row is invalid for a layer if it is a
 *     padding row (n == 0), if a degree exceeds the extent, if the block leaves the machine, or
 *     if it splits height/width of a fully connected layer (Table 1).
 *   t_c = round(F / (d * flop_per_ns)); F = forward + backward work: 3 * 2*N*Cout*Hout*Wout*Cin*kh*kw
 *     for a convolution, 3 * 2*N*(Cin*Hin*Win)*Cout for a fully connected layer,
 *     2 * N*Cout*Hout*Wout*kh*kw for pooling.  Invalid rows get machine.invalid_cost.
 *   t_s = round(P * (r-1) / (r * byte_per_ns)); P = 4 bytes * (weights + biases), r = n*h*w the
 *     number of parameter replicas (a channel split partitions the parameters; Sec. 3, Fig. 2).
 *   t_x = round(bytes / byte_per_ns); bytes = 4 * sum over (producer part p, consumer part q) on
 *     DIFFERENT devices of |T(p) ^ R(q)|, T(p) the producer's output part, R(q) the region of that
 *     tensor the consumer part reads: its samples; all input channels (pooling: its own channels);
 *     the window-expanded, clipped spatial range (fully connected: everything).
 *   Rounding is half-up in integers: (num + den/2) / den.  Invalid rows/columns of t_x are 0.
 *
 * With a device graph (Sec. 4: every connection (d_i, d_j) has its own bandwidth b(d_i, d_j); Sec. 5.1,
 * assumption 2: moving s bytes over it takes s / b) -- orc_build_cost_tables_graph:
 *   t_x = round( sum over (producer part p on device u, consumer part q on device v != u) of
 *         4 * |T(p) ^ R(q)| / b(u, v) ): the transfers of one tensor are added up, each over its own
 *         connection (with one bandwidth for all pairs this is the formula above);
 *   t_s = max over the devices u that hold parameters of round( sum over the other devices v holding a
 *         replica of the same parameters of (P / r) / b(u, v) ): every replica sends an r-th of its
 *         gradients to each of the others (each serves an r-th of the parameters, in the paper's
 *         words a parameter server for it); devices work at the same time, the slowest finishes last
 *         (with one bandwidth: P * (r-1) / (r * b), the formula above);
 *   t_c = a table of measured times handed in by the caller (Sec. 5.1: "processing the layer under
 *         that configuration multiple times on the device and measuring"), or the analytic value.
 *   Sums of fractions with different denominators are exact: with L the least common multiple of
 *   all bandwidths, s / b = s * (L / b) / L, and one division by L (half-up) ends the sum.
 *
 * Absolute values are PARITY UNPINNED against the paper (its t_c are device measurements); the
 * tests pin this file through closed forms and conservation properties instead.
 */
#include <stdint.h>
#include <stdlib.h>

#define ORC_OK 0
#define ORC_E_INVAL (-1)
#define ORC_E_OVERFLOW (-4)

typedef struct { int32_t kind, N, Cin, Hin, Win, Cout, Hout, Wout, kh, kw, sh, sw, ph, pw; } orc_layer;
typedef struct { int32_t n, h, w, c, dev_offset, pad; } orc_config;
typedef struct { int32_t n_devices, flop_per_ns, byte_per_ns, invalid_cost; } orc_machine;

enum { KIND_CONV = 0, KIND_POOL = 1, KIND_FC = 2 };

static int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }
static int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }
static int64_t round_div(int64_t num, int64_t den) { return (num + den / 2) / den; }

static int config_valid(const orc_layer *L, const orc_config *c, const orc_machine *m)
{
    if (c->n <= 0 || c->h <= 0 || c->w <= 0 || c->c <= 0) return 0;
    if (c->n > L->N || c->c > L->Cout || c->h > L->Hout || c->w > L->Wout) return 0;
    if (L->kind == KIND_FC && (c->h != 1 || c->w != 1)) return 0;
    int64_t d = (int64_t)c->n * c->h * c->w * c->c;
    if (c->dev_offset < 0 || c->dev_offset + d > m->n_devices) return 0;
    return 1;
}

static void part(int t, int g, int D, int64_t *lo, int64_t *hi)
{
    *lo = (int64_t)t * D / g;
    *hi = (int64_t)(t + 1) * D / g;
}

/* input range read by output range [o0,o1) of a window op with stride s, padding p, kernel k */
static void window(int64_t o0, int64_t o1, int s, int p, int k, int Din, int64_t *lo, int64_t *hi)
{
    *lo = imax(0, o0 * s - p);
    *hi = imin(Din, (o1 - 1) * s - p + k);
}

static int64_t overlap(int64_t a0, int64_t a1, int64_t b0, int64_t b1)
{
    return imax(0, imin(a1, b1) - imax(a0, b0));
}

/* The three tables when layer l has its own list of configurations: rows
 * cfgs[cfg_off[l] .. cfg_off[l] + Cn[l]).  t_c and t_s are the layers' rows one after another
 * (row l starts at node_off[l]); t_x holds the edges' tables [Cn[src]][Cn[dst]] one after another
 * (table e starts at tx_off[e]). */
static int build_tables(const orc_layer *layers, int n_layers, const int32_t *edges, int n_edges,
                        const orc_config *cfgs, const int64_t *cfg_off, const int32_t *Cn,
                        const int64_t *node_off, const int64_t *tx_off, const orc_machine *m,
                        int32_t *tc, int32_t *ts, int32_t *tx)
{
    if (n_layers <= 0 || m->flop_per_ns <= 0 || m->byte_per_ns <= 0) return ORC_E_INVAL;
    for (int l = 0; l < n_layers; ++l) if (Cn[l] <= 0) return ORC_E_INVAL;
    int overflow = 0;
    for (int l = 0; l < n_layers; ++l) {
        const orc_layer *L = &layers[l];
        const int C = Cn[l];
        int64_t F, P;
        if (L->kind == KIND_CONV) {
            F = 3 * 2 * (int64_t)L->N * L->Cout * L->Hout * L->Wout * L->Cin * L->kh * L->kw;
            P = 4 * ((int64_t)L->Cout * L->Cin * L->kh * L->kw + L->Cout);
        } else if (L->kind == KIND_FC) {
            F = 3 * 2 * (int64_t)L->N * ((int64_t)L->Cin * L->Hin * L->Win) * L->Cout;
            P = 4 * ((int64_t)L->Cout * L->Cin * L->Hin * L->Win + L->Cout);
        } else if (L->kind == KIND_POOL) {
            F = 2 * (int64_t)L->N * L->Cout * L->Hout * L->Wout * L->kh * L->kw;
            P = 0;
        } else return ORC_E_INVAL;
        for (int r = 0; r < C; ++r) {
            const orc_config *c = &cfgs[cfg_off[l] + r];
            int64_t vc = m->invalid_cost, vs = 0;
            if (config_valid(L, c, m)) {
                int64_t d = (int64_t)c->n * c->h * c->w * c->c;
                int64_t rep = (int64_t)c->n * c->h * c->w;
                vc = round_div(F, d * m->flop_per_ns);
                vs = round_div(P * (rep - 1), rep * m->byte_per_ns);
            }
            if (vc > INT32_MAX || vs > INT32_MAX) overflow = 1;
            tc[node_off[l] + r] = (int32_t)vc;
            ts[node_off[l] + r] = (int32_t)vs;
        }
    }
    for (int e = 0; e < n_edges; ++e) {
        int pi = edges[2 * e], ci = edges[2 * e + 1];
        if (pi < 0 || pi >= n_layers || ci < 0 || ci >= n_layers) return ORC_E_INVAL;
        const orc_layer *Pl = &layers[pi], *Cl = &layers[ci];
        /* the tensor on the edge: the producer's output is the consumer's input */
        if (Pl->N != Cl->N || Pl->Cout != Cl->Cin || Pl->Hout != Cl->Hin || Pl->Wout != Cl->Win) return ORC_E_INVAL;
        const int Ca = Cn[pi], Cb = Cn[ci];
#pragma omp parallel for schedule(dynamic, 4) reduction(| : overflow)
        for (int a = 0; a < Ca; ++a) {
            const orc_config *ca = &cfgs[cfg_off[pi] + a];
            for (int b = 0; b < Cb; ++b) {
                const orc_config *cb = &cfgs[cfg_off[ci] + b];
                int64_t cells = 0;
                if (config_valid(Pl, ca, m) && config_valid(Cl, cb, m)) {
                    for (int pn = 0; pn < ca->n; ++pn) for (int ph = 0; ph < ca->h; ++ph)
                    for (int pw = 0; pw < ca->w; ++pw) for (int pc = 0; pc < ca->c; ++pc) {
                        int devp = ca->dev_offset + ((pn * ca->h + ph) * ca->w + pw) * ca->c + pc;
                        int64_t tn0, tn1, th0, th1, tw0, tw1, tc0, tc1;
                        part(pn, ca->n, Pl->N, &tn0, &tn1);
                        part(ph, ca->h, Pl->Hout, &th0, &th1);
                        part(pw, ca->w, Pl->Wout, &tw0, &tw1);
                        part(pc, ca->c, Pl->Cout, &tc0, &tc1);
                        for (int qn = 0; qn < cb->n; ++qn) for (int qh = 0; qh < cb->h; ++qh)
                        for (int qw = 0; qw < cb->w; ++qw) for (int qc = 0; qc < cb->c; ++qc) {
                            int devq = cb->dev_offset + ((qn * cb->h + qh) * cb->w + qw) * cb->c + qc;
                            if (devq == devp) continue;          /* already local */
                            int64_t rn0, rn1, rh0, rh1, rw0, rw1, rc0, rc1, o0, o1;
                            part(qn, cb->n, Cl->N, &rn0, &rn1);
                            if (Cl->kind == KIND_FC) {
                                rc0 = 0; rc1 = Cl->Cin; rh0 = 0; rh1 = Cl->Hin; rw0 = 0; rw1 = Cl->Win;
                            } else {
                                if (Cl->kind == KIND_POOL) part(qc, cb->c, Cl->Cout, &rc0, &rc1);
                                else { rc0 = 0; rc1 = Cl->Cin; }
                                part(qh, cb->h, Cl->Hout, &o0, &o1);
                                window(o0, o1, Cl->sh, Cl->ph, Cl->kh, Cl->Hin, &rh0, &rh1);
                                part(qw, cb->w, Cl->Wout, &o0, &o1);
                                window(o0, o1, Cl->sw, Cl->pw, Cl->kw, Cl->Win, &rw0, &rw1);
                            }
                            cells += overlap(tn0, tn1, rn0, rn1) * overlap(tc0, tc1, rc0, rc1) *
                                     overlap(th0, th1, rh0, rh1) * overlap(tw0, tw1, rw0, rw1);
                        }
                    }
                }
                int64_t v = round_div(4 * cells, m->byte_per_ns);
                if (v > INT32_MAX) overflow = 1;
                tx[tx_off[e] + (int64_t)a * Cb + b] = (int32_t)v;
            }
        }
    }
    return overflow ? ORC_E_OVERFLOW : ORC_OK;
}

/* One list of C configurations shared by all layers: t_c, t_s [n_layers][C], t_x [n_edges][C][C]. */
int orc_build_cost_tables(const orc_layer *layers, int n_layers, const int32_t *edges, int n_edges,
                          const orc_config *cfgs, int C, const orc_machine *m,
                          int32_t *tc, int32_t *ts, int32_t *tx)
{
    if (n_layers <= 0 || C <= 0 || n_edges < 0) return ORC_E_INVAL;
    int64_t *cfg_off = calloc((size_t)n_layers, sizeof(int64_t));
    int64_t *node_off = malloc((size_t)n_layers * sizeof(int64_t));
    int64_t *tx_off = malloc((size_t)(n_edges + 1) * sizeof(int64_t));
    int32_t *Cn = malloc((size_t)n_layers * sizeof(int32_t));
    for (int l = 0; l < n_layers; ++l) { node_off[l] = (int64_t)l * C; Cn[l] = C; }
    for (int e = 0; e < n_edges; ++e) tx_off[e] = (int64_t)e * C * C;
    int rc = build_tables(layers, n_layers, edges, n_edges, cfgs, cfg_off, Cn, node_off, tx_off, m, tc, ts, tx);
    free(cfg_off); free(node_off); free(tx_off); free(Cn);
    return rc;
}

/* Per-layer lists, concatenated in layer order in cfgs; Cn[l] rows for layer l. */
int orc_build_cost_tables_ragged(const orc_layer *layers, int n_layers, const int32_t *edges, int n_edges,
                                 const orc_config *cfgs, const int32_t *Cn, const orc_machine *m,
                                 int32_t *tc, int32_t *ts, int32_t *tx)
{
    if (n_layers <= 0 || n_edges < 0) return ORC_E_INVAL;
    for (int e = 0; e < n_edges; ++e)
        if (edges[2 * e] < 0 || edges[2 * e] >= n_layers || edges[2 * e + 1] < 0 || edges[2 * e + 1] >= n_layers)
            return ORC_E_INVAL;
    int64_t *cfg_off = malloc((size_t)(n_layers + 1) * sizeof(int64_t));
    int64_t *tx_off = malloc((size_t)(n_edges + 1) * sizeof(int64_t));
    cfg_off[0] = 0;
    for (int l = 0; l < n_layers; ++l) cfg_off[l + 1] = cfg_off[l] + Cn[l];
    tx_off[0] = 0;
    for (int e = 0; e < n_edges; ++e) tx_off[e + 1] = tx_off[e] + (int64_t)Cn[edges[2 * e]] * Cn[edges[2 * e + 1]];
    int rc = build_tables(layers, n_layers, edges, n_edges, cfgs, cfg_off, Cn, cfg_off, tx_off, m, tc, ts, tx);
    free(cfg_off); free(tx_off);
    return rc;
}

/* The configurations of one layer (Sec. 4: a degree of parallelism per parallelizable dimension,
 * Table 1; equal partitioning): all (n, h, w, c) of powers of two whose product d does not exceed
 * the number of devices and whose degrees do not exceed the layer's extents (a fully connected
 * layer splits only sample and channel), each with every device block [offset, offset + d) whose
 * offset is a multiple of d.  Order: ascending (n, h, w, c, offset).
 * Returns the count; writes at most cap rows. */
int orc_enumerate_configs(const orc_layer *L, int n_devices, orc_config *out, int cap)
{
    int count = 0;
    for (int n = 1; n <= n_devices && n <= L->N; n *= 2)
        for (int h = 1; n * h <= n_devices && h <= L->Hout; h *= 2)
            for (int w = 1; n * h * w <= n_devices && w <= L->Wout; w *= 2)
                for (int c = 1; n * h * w * c <= n_devices && c <= L->Cout; c *= 2) {
                    if (L->kind == KIND_FC && (h != 1 || w != 1)) continue;
                    const int d = n * h * w * c;
                    for (int off = 0; off + d <= n_devices; off += d) {
                        if (count < cap) {
                            orc_config r = { n, h, w, c, off, 0 };
                            out[count] = r;
                        }
                        ++count;
                    }
                }
    return count;
}


/* ---- device graph and measured t_c ------------------------------------------------------------ */

static int64_t gcd64(int64_t a, int64_t b) { while (b) { int64_t t = a % b; a = b; b = t; } return a; }

static int in_config(const orc_config *c, int dev, int *in_, int *ih, int *iw, int *ic)
{
    int64_t d = (int64_t)c->n * c->h * c->w * c->c;
    int p = dev - c->dev_offset;
    if (p < 0 || p >= d) return 0;
    *ic = p % c->c; p /= c->c;
    *iw = p % c->w; p /= c->w;
    *ih = p % c->h; *in_ = p / c->h;
    return 1;
}

/* Per-layer configuration lists as orc_build_cost_tables_ragged takes them; bw [n_devices][n_devices]
 * holds b(u, v) in bytes per ns for the connection from device u (row) to device v (column), the
 * diagonal is ignored; measured_tc (may be NULL) has the layout of tc and replaces the analytic t_c
 * of every configuration its layer can use. */
int orc_build_cost_tables_graph(const orc_layer *layers, int n_layers, const int32_t *edges, int n_edges,
                                const orc_config *cfgs, const int32_t *Cn, int n_devices, int flop_per_ns,
                                int invalid_cost, const int32_t *bw, const int32_t *measured_tc,
                                int32_t *tc, int32_t *ts, int32_t *tx)
{
    if (n_layers <= 0 || n_edges < 0 || n_devices <= 0 || flop_per_ns <= 0) return ORC_E_INVAL;
    int64_t L = 1;                                 /* least common multiple of the bandwidths */
    for (int u = 0; u < n_devices; ++u)
        for (int v = 0; v < n_devices; ++v) {
            if (u == v) continue;
            int64_t b = bw[u * n_devices + v];
            if (b <= 0) return ORC_E_INVAL;
            L = L / gcd64(L, b) * b;
            if (L > (1 << 20)) return ORC_E_INVAL;
        }
    for (int e = 0; e < n_edges; ++e)
        if (edges[2 * e] < 0 || edges[2 * e] >= n_layers || edges[2 * e + 1] < 0 || edges[2 * e + 1] >= n_layers)
            return ORC_E_INVAL;
    const orc_machine m = { n_devices, flop_per_ns, 1, invalid_cost };    /* for config_valid */
    int overflow = 0;
    int64_t off = 0;
    for (int l = 0; l < n_layers; ++l) {
        const orc_layer *Ly = &layers[l];
        int64_t F, P;
        if (Ly->kind == KIND_CONV) {
            F = 3 * 2 * (int64_t)Ly->N * Ly->Cout * Ly->Hout * Ly->Wout * Ly->Cin * Ly->kh * Ly->kw;
            P = 4 * ((int64_t)Ly->Cout * Ly->Cin * Ly->kh * Ly->kw + Ly->Cout);
        } else if (Ly->kind == KIND_FC) {
            F = 3 * 2 * (int64_t)Ly->N * ((int64_t)Ly->Cin * Ly->Hin * Ly->Win) * Ly->Cout;
            P = 4 * ((int64_t)Ly->Cout * Ly->Cin * Ly->Hin * Ly->Win + Ly->Cout);
        } else if (Ly->kind == KIND_POOL) {
            F = 2 * (int64_t)Ly->N * Ly->Cout * Ly->Hout * Ly->Wout * Ly->kh * Ly->kw;
            P = 0;
        } else return ORC_E_INVAL;
        if (Cn[l] <= 0) return ORC_E_INVAL;
        for (int r = 0; r < Cn[l]; ++r) {
            const orc_config *c = &cfgs[off + r];
            int64_t vc = invalid_cost, vs = 0;
            if (config_valid(Ly, c, &m)) {
                int64_t d = (int64_t)c->n * c->h * c->w * c->c;
                int64_t rep = (int64_t)c->n * c->h * c->w;
                if (measured_tc) {
                    vc = measured_tc[off + r];
                    if (vc < 0) return ORC_E_INVAL;
                } else vc = round_div(F, d * flop_per_ns);
                /* every device u of the configuration against the other holders of its parameters:
                 * the parts that differ from u's only in the sample, height or width index */
                for (int u = c->dev_offset; u < c->dev_offset + d; ++u) {
                    int un = 0, uh = 0, uw = 0, uc = 0, vn = 0, vh = 0, vw = 0, vcx = 0;
                    in_config(c, u, &un, &uh, &uw, &uc);
                    int64_t inv = 0;                        /* sum of L / b(u, v) */
                    for (int v = c->dev_offset; v < c->dev_offset + d; ++v) {
                        in_config(c, v, &vn, &vh, &vw, &vcx);
                        if (v == u || vcx != uc) continue;
                        inv += L / bw[u * n_devices + v];
                    }
                    int64_t t = round_div(P * inv, rep * L);
                    vs = imax(vs, t);
                }
            }
            if (vc > INT32_MAX || vs > INT32_MAX) overflow = 1;
            tc[off + r] = (int32_t)vc;
            ts[off + r] = (int32_t)vs;
        }
        off += Cn[l];
    }
    int64_t *cfg_off = malloc((size_t)(n_layers + 1) * sizeof(int64_t));
    cfg_off[0] = 0;
    for (int l = 0; l < n_layers; ++l) cfg_off[l + 1] = cfg_off[l] + Cn[l];
    int64_t tx_off = 0;
    for (int e = 0; e < n_edges; ++e) {
        int pi = edges[2 * e], ci = edges[2 * e + 1];
        const orc_layer *Pl = &layers[pi], *Cl = &layers[ci];
        if (Pl->N != Cl->N || Pl->Cout != Cl->Cin || Pl->Hout != Cl->Hin || Pl->Wout != Cl->Win) { free(cfg_off); return ORC_E_INVAL; }
        const int Ca = Cn[pi], Cb = Cn[ci];
        for (int a = 0; a < Ca; ++a) {
            const orc_config *ca = &cfgs[cfg_off[pi] + a];
            for (int b = 0; b < Cb; ++b) {
                const orc_config *cb = &cfgs[cfg_off[ci] + b];
                int64_t scaled = 0;                         /* sum of 4 * cells * L / b(u, v) */
                if (config_valid(Pl, ca, &m) && config_valid(Cl, cb, &m)) {
                    int64_t da = (int64_t)ca->n * ca->h * ca->w * ca->c, db = (int64_t)cb->n * cb->h * cb->w * cb->c;
                    for (int u = ca->dev_offset; u < ca->dev_offset + da; ++u)
                        for (int v = cb->dev_offset; v < cb->dev_offset + db; ++v) {
                            if (u == v) continue;                /* already local */
                            int pn = 0, ph = 0, pw = 0, pc = 0, qn = 0, qh = 0, qw = 0, qc = 0;
                            in_config(ca, u, &pn, &ph, &pw, &pc);
                            in_config(cb, v, &qn, &qh, &qw, &qc);
                            int64_t tn0, tn1, th0, th1, tw0, tw1, tc0, tc1;
                            part(pn, ca->n, Pl->N, &tn0, &tn1);
                            part(ph, ca->h, Pl->Hout, &th0, &th1);
                            part(pw, ca->w, Pl->Wout, &tw0, &tw1);
                            part(pc, ca->c, Pl->Cout, &tc0, &tc1);
                            int64_t rn0, rn1, rh0, rh1, rw0, rw1, rc0, rc1, o0, o1;
                            part(qn, cb->n, Cl->N, &rn0, &rn1);
                            if (Cl->kind == KIND_FC) {
                                rc0 = 0; rc1 = Cl->Cin; rh0 = 0; rh1 = Cl->Hin; rw0 = 0; rw1 = Cl->Win;
                            } else {
                                if (Cl->kind == KIND_POOL) part(qc, cb->c, Cl->Cout, &rc0, &rc1);
                                else { rc0 = 0; rc1 = Cl->Cin; }
                                part(qh, cb->h, Cl->Hout, &o0, &o1);
                                window(o0, o1, Cl->sh, Cl->ph, Cl->kh, Cl->Hin, &rh0, &rh1);
                                part(qw, cb->w, Cl->Wout, &o0, &o1);
                                window(o0, o1, Cl->sw, Cl->pw, Cl->kw, Cl->Win, &rw0, &rw1);
                            }
                            int64_t cells = overlap(tn0, tn1, rn0, rn1) * overlap(tc0, tc1, rc0, rc1) *
                                            overlap(th0, th1, rh0, rh1) * overlap(tw0, tw1, rw0, rw1);
                            scaled += 4 * cells * (L / bw[u * n_devices + v]);
                        }
                }
                int64_t t = round_div(scaled, L);
                if (t > INT32_MAX) overflow = 1;
                tx[tx_off + (int64_t)a * Cb + b] = (int32_t)t;
            }
        }
        tx_off += (int64_t)Ca * Cb;
    }
    free(cfg_off);
    return overflow ? ORC_E_OVERFLOW : ORC_OK;
}
