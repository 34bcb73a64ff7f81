/*
 * CPU oracle for the layer-wise-parallelism strategy search.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * straightforward implementation of what the GPU library computes, written
 * from the paper's equations so that a reader can check it by eye.  It shares
 * no code with the HIP path.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * What follows the paper:
 *   orc_strategy_cost    Eq. 1   (objective t_o of a complete strategy)
 *   orc_minplus_argmin   Eq. 2   (node elimination; argmin of Thm. 3 / Eq. of the appendix)
 *   orc_edge_sum         Eq. 3   (edge elimination)
 *   orc_search           Alg. 1  (eliminate, solve the residual graph, undo in reverse)
 *
 * Readings where the paper is silent:
 *   - costs are int32 nanoseconds, sums are exact; a sum that leaves int32 is an error;
 *   - every min takes the LOWEST index among equal candidates (strict '<' in ascending order);
 *   - the order of eliminations is the written canonical schedule implemented in orc_search;
 *   - the residual graph is solved per connected component: one node, a pair joined by one edge
 *     (lowest flat index of (source cfg, destination cfg)), or outright enumeration of larger
 *     components (lexicographically lowest optimum, lower node id more significant).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_E_INVAL (-1)
#define ORC_E_NOT_REDUCIBLE (-3)
#define ORC_E_OVERFLOW (-4)
#define ORC_E_NOMEM (-5)

#define ORC_SCHEDULE_ROUNDS 0
#define ORC_SCHEDULE_LEFT_FOLD 1
#define ORC_SCHEDULE_NONE 2          /* no elimination at all: the baseline of Sec. 5.2 / Table 3 */

static int fits_i32(int64_t v) { return v >= INT32_MIN && v <= INT32_MAX; }

/* Eq. 1: t_o = sum_l (t_c(l,S_l) + t_s(l,S_l)) + sum_{e=(i,j)} t_x(e,S_i,S_j).
 * Node l has Cn[l] configurations.  tc, ts: the rows of all nodes one after another; tx: the
 * tables of all edges one after another, table e is [Cn[src]][Cn[dst]]; result in 64 bits. */
int orc_strategy_cost_ragged(int n_nodes, int n_edges, const int32_t *edges, const int32_t *Cn,
                             const int32_t *tc, const int32_t *ts, const int32_t *tx,
                             const int32_t *S, int64_t *out_cost)
{
    int64_t t = 0;
    size_t off = 0;
    for (int l = 0; l < n_nodes; ++l) {
        if (S[l] < 0 || S[l] >= Cn[l]) return ORC_E_INVAL;
        t += (int64_t)tc[off + S[l]] + (int64_t)ts[off + S[l]];
        off += (size_t)Cn[l];
    }
    off = 0;
    for (int e = 0; e < n_edges; ++e) {
        int i = edges[2 * e], j = edges[2 * e + 1];
        t += tx[off + (size_t)S[i] * Cn[j] + S[j]];
        off += (size_t)Cn[i] * Cn[j];
    }
    *out_cost = t;
    return ORC_OK;
}

/* Eq. 2 for one eliminated node l_j:
 *   out[a][b] = min_c ( A[a][c] + w[c] + B[c][b] ),   arg[a][b] = lowest c attaining it,
 * A = t_x(e_1) [Ci][Cj], w = t_c(l_j)+t_s(l_j) [Cj], B = t_x(e_2) [Cj][Ck].
 * For one row a the candidates are visited in ascending c, so strict '<' keeps the lowest c. */
int orc_minplus_argmin(int Ci, int Cj, int Ck, const int32_t *A, const int32_t *w,
                       const int32_t *B, int32_t *out, int32_t *arg)
{
    if (Ci < 0 || Cj <= 0 || Ck < 0) return ORC_E_INVAL;
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int a = 0; a < Ci; ++a) {
        int32_t *best = out + (size_t)a * Ck;
        int32_t *bidx = arg + (size_t)a * Ck;
        for (int c = 0; c < Cj; ++c) {
            int64_t left = (int64_t)A[(size_t)a * Cj + c] + (int64_t)w[c];
            const int32_t *Brow = B + (size_t)c * Ck;
            for (int b = 0; b < Ck; ++b) {
                int64_t s = left + (int64_t)Brow[b];
                if (!fits_i32(s)) overflow = 1;
                if (c == 0 || s < (int64_t)best[b]) {
                    best[b] = (int32_t)s;
                    bidx[b] = c;
                }
            }
        }
    }
    return overflow ? ORC_E_OVERFLOW : ORC_OK;
}

/* Eq. 3: out = e1 + e2 elementwise over [Ci][Cj]. */
int orc_edge_sum(int Ci, int Cj, const int32_t *e1, const int32_t *e2, int32_t *out)
{
    int overflow = 0;
    size_t n = (size_t)Ci * Cj;
    for (size_t t = 0; t < n; ++t) {
        int64_t s = (int64_t)e1[t] + (int64_t)e2[t];
        if (!fits_i32(s)) overflow = 1;
        out[t] = (int32_t)s;
    }
    return overflow ? ORC_E_OVERFLOW : ORC_OK;
}

/* Residual pair (Alg. 1, enumeration of the final graph with K = 2):
 *   min_{a,b} wi[a] + T[a][b] + wk[b] over T [Ci][Ck], lowest flat index a*Ck+b among equals. */
int orc_final_pair(int Ci, int Ck, const int32_t *wi, const int32_t *T, const int32_t *wk,
                   int64_t *out_cost, int32_t *out_a, int32_t *out_b)
{
    int64_t best = 0;
    int ba = -1, bb = -1, overflow = 0;
    for (int a = 0; a < Ci; ++a)
        for (int b = 0; b < Ck; ++b) {
            int64_t s = (int64_t)wi[a] + (int64_t)T[(size_t)a * Ck + b] + (int64_t)wk[b];
            if (!fits_i32(s)) overflow = 1;
            if (ba < 0 || s < best) { best = s; ba = a; bb = b; }
        }
    *out_cost = best; *out_a = ba; *out_b = bb;
    return overflow ? ORC_E_OVERFLOW : ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1                                                               */
/* ------------------------------------------------------------------------- */

/* One log entry.  kind 0 = node elimination of node j between i and k, using
 * in-edge e1=(i,j) and out-edge e2=(j,k); the new edge (i,k) keeps the id e1.
 * kind 1 = edge elimination: edge e2 is added into e1 (same endpoints i,k),
 * the sum keeps the id e1; j is -1.  'round' counts schedule rounds from 0. */
typedef struct { int32_t kind, j, i, k, e1, e2, round; } orc_step;

typedef struct {
    int32_t src, dst;
    int32_t *tab;      /* current C x C table of this edge           */
    int owned;         /* 1 if tab was allocated here (not an input) */
    int alive;
} live_edge;

static int cmp_edge_group(const void *pa, const void *pb, void *ctx)
{
    const live_edge *E = (const live_edge *)ctx;
    int a = *(const int *)pa, b = *(const int *)pb;
    if (E[a].src != E[b].src) return E[a].src < E[b].src ? -1 : 1;
    if (E[a].dst != E[b].dst) return E[a].dst < E[b].dst ? -1 : 1;
    return a < b ? -1 : (a > b);
}

/* simple insertion sort with context (n is small: number of live edges) */
static void sort_ids(int *ids, int n, const live_edge *E)
{
    for (int x = 1; x < n; ++x) {
        int v = ids[x], y = x - 1;
        while (y >= 0 && cmp_edge_group(&ids[y], &v, (void *)E) > 0) { ids[y + 1] = ids[y]; --y; }
        ids[y + 1] = v;
    }
}

/*
 * Alg. 1.  Canonical schedule (the paper leaves the choice of the eliminated
 * node/edge open; this is the written rule both implementations follow):
 *
 *   repeat rounds until a round changes nothing:
 *     E-phase  for every (src,dst) group of live edges holding >= 2 edges, in
 *              ascending (src,dst): add the edges with higher ids, in ascending
 *              id order, into the lowest id (Eq. 3 applied pairwise);
 *     N-phase  scan nodes in ascending id; node j is eligible if it has exactly
 *              one live in-edge (i,j) and one live out-edge (j,k);
 *                ROUNDS:    select j unless i or k was selected in this round;
 *                LEFT_FOLD: select only the first eligible node;
 *              then eliminate every selected node by Eq. 2 (new edge keeps the
 *              in-edge's id).
 *
 * Each connected component of the residual graph is minimised on its own (a
 * node, a pair joined by one edge, or enumeration of all C^K strategies of a
 * larger component, K <= 16 and at most 2^32 strategies here).  The eliminations are then
 * undone in reverse order:
 * S[j] = arg_j[S[i]][S[k]].
 *
 * steps (optional, room for n_edges entries) receives the log; n_steps and
 * n_rounds (optional) its length and the number of rounds that did work.
 */
int orc_search_ragged(int n_nodes, int n_edges, const int32_t *edges, const int32_t *Cn,
                      const int32_t *tc, const int32_t *ts, const int32_t *tx, int schedule,
                      int64_t *out_cost, int32_t *S, orc_step *steps, int32_t *n_steps, int32_t *n_rounds)
{
    if (n_nodes <= 0 || n_edges < 0) return ORC_E_INVAL;
    int rc = ORC_OK;
    size_t total_w = 0;
    for (int l = 0; l < n_nodes; ++l) { if (Cn[l] <= 0) return ORC_E_INVAL; total_w += (size_t)Cn[l]; }
    size_t *woff = (size_t *)malloc(sizeof(size_t) * (size_t)n_nodes);   /* start of node l's row of w */
    int32_t *w = (int32_t *)malloc(total_w * sizeof(int32_t));
    live_edge *E = (live_edge *)calloc((size_t)(n_edges > 0 ? n_edges : 1), sizeof(live_edge));
    orc_step *log = (orc_step *)calloc((size_t)(n_edges > 0 ? n_edges : 1), sizeof(orc_step));
    int32_t **argtab = (int32_t **)calloc((size_t)(n_edges > 0 ? n_edges : 1), sizeof(int32_t *));
    char *dead = (char *)calloc((size_t)n_nodes, 1);
    char *sel = (char *)malloc((size_t)n_nodes);
    int *indeg = (int *)malloc(sizeof(int) * n_nodes), *outdeg = (int *)malloc(sizeof(int) * n_nodes);
    /* per node during the elimination phase; reused per residual component for its member nodes
     * (ine) and its live edges (oute), of which there can be more than nodes */
    size_t n_slots = (size_t)(n_nodes > n_edges ? n_nodes : n_edges);
    int *ine = (int *)malloc(sizeof(int) * n_nodes), *oute = (int *)malloc(sizeof(int) * n_slots);
    int *ids = (int *)malloc(sizeof(int) * (n_edges > 0 ? n_edges : 1));
    int nlog = 0, rounds = 0;
    if (!woff || !w || !E || !log || !argtab || !dead || !sel || !indeg || !outdeg || !ine || !oute || !ids) {
        rc = ORC_E_NOMEM; goto done;
    }

    /* w = t_c + t_s: Eq. 1 and Eq. 2 only ever use the sum. */
    for (size_t t = 0; t < total_w; ++t) {
        int64_t s = (int64_t)tc[t] + (int64_t)ts[t];
        if (!fits_i32(s)) { rc = ORC_E_OVERFLOW; goto done; }
        w[t] = (int32_t)s;
    }
    { size_t o = 0; for (int l = 0; l < n_nodes; ++l) { woff[l] = o; o += (size_t)Cn[l]; } }
    {
        size_t o = 0;       /* table e is [Cn[src]][Cn[dst]], tables one after another */
        for (int e = 0; e < n_edges; ++e) {
            E[e].src = edges[2 * e]; E[e].dst = edges[2 * e + 1];
            if (E[e].src < 0 || E[e].src >= n_nodes || E[e].dst < 0 || E[e].dst >= n_nodes ||
                E[e].src == E[e].dst) { rc = ORC_E_INVAL; goto done; }
            E[e].tab = (int32_t *)(tx + o);
            E[e].owned = 0; E[e].alive = 1;
            o += (size_t)Cn[E[e].src] * Cn[E[e].dst];
        }
    }

    for (;;) {
        int changed = 0;
        /* The baseline the paper compares with (Sec. 5.2, last paragraph; Table 3) searches the
         * original graph: nothing is eliminated and every strategy of it is enumerated below. */
        if (schedule == ORC_SCHEDULE_NONE) break;
        /* ---- E-phase: merge parallel edges (Eq. 3) ---- */
        int nl = 0;
        for (int e = 0; e < n_edges; ++e) if (E[e].alive) ids[nl++] = e;
        sort_ids(ids, nl, E);
        for (int x = 0; x < nl;) {
            int y = x + 1;
            while (y < nl && E[ids[y]].src == E[ids[x]].src && E[ids[y]].dst == E[ids[x]].dst) ++y;
            int keep = ids[x];
            for (int z = x + 1; z < y; ++z) {
                int other = ids[z];
                int32_t *sum = (int32_t *)malloc((size_t)Cn[E[keep].src] * Cn[E[keep].dst] * sizeof(int32_t));
                if (!sum) { rc = ORC_E_NOMEM; goto done; }
                int r = orc_edge_sum(Cn[E[keep].src], Cn[E[keep].dst], E[keep].tab, E[other].tab, sum);
                if (E[keep].owned) free(E[keep].tab);
                if (E[other].owned) free(E[other].tab);
                E[keep].tab = sum; E[keep].owned = 1;
                E[other].alive = 0; E[other].tab = NULL; E[other].owned = 0;
                log[nlog++] = (orc_step){1, -1, E[keep].src, E[keep].dst, keep, other, rounds};
                changed = 1;
                if (r != ORC_OK) { rc = r; goto done; }
            }
            x = y;
        }
        /* ---- N-phase: choose independent eligible nodes, then apply Eq. 2 ---- */
        for (int l = 0; l < n_nodes; ++l) { indeg[l] = outdeg[l] = 0; ine[l] = oute[l] = -1; sel[l] = 0; }
        for (int e = 0; e < n_edges; ++e) if (E[e].alive) {
            outdeg[E[e].src]++; oute[E[e].src] = e;
            indeg[E[e].dst]++;  ine[E[e].dst] = e;
        }
        for (int j = 0; j < n_nodes; ++j) {
            if (dead[j] || indeg[j] != 1 || outdeg[j] != 1) continue;
            int i = E[ine[j]].src, k = E[oute[j]].dst;
            if (sel[i] || sel[k]) continue;
            sel[j] = 1;
            if (schedule == ORC_SCHEDULE_LEFT_FOLD) break;
        }
        for (int j = 0; j < n_nodes; ++j) {
            if (!sel[j]) continue;
            int e1 = ine[j], e2 = oute[j];
            int i = E[e1].src, k = E[e2].dst;
            int32_t *nt = (int32_t *)malloc((size_t)Cn[i] * Cn[k] * sizeof(int32_t));
            int32_t *na = (int32_t *)malloc((size_t)Cn[i] * Cn[k] * sizeof(int32_t));
            if (!nt || !na) { free(nt); free(na); rc = ORC_E_NOMEM; goto done; }
            int r = orc_minplus_argmin(Cn[i], Cn[j], Cn[k], E[e1].tab, w + woff[j], E[e2].tab, nt, na);
            if (E[e1].owned) free(E[e1].tab);
            if (E[e2].owned) free(E[e2].tab);
            E[e1].tab = nt; E[e1].owned = 1; E[e1].dst = k;
            E[e2].alive = 0; E[e2].tab = NULL; E[e2].owned = 0;
            dead[j] = 1;
            argtab[nlog] = na;
            log[nlog++] = (orc_step){0, j, i, k, e1, e2, rounds};
            changed = 1;
            if (r != ORC_OK) { rc = r; goto done; }
        }
        if (!changed) break;
        ++rounds;
    }

    /* ---- residual graph (Alg. 1: enumerate all strategies of the final graph) ----
     * Connected components are independent.  One node: min_a w[a].  Two nodes joined by one edge:
     * orc_final_pair.  Anything larger is enumerated outright, configurations of the lower node id
     * varying slowest, so that strict '<' keeps the lexicographically lowest optimum. */
    {
        int *comp = indeg;                       /* reused: component label per node */
        int64_t total = 0;
        for (int l = 0; l < n_nodes; ++l) { comp[l] = dead[l] ? -1 : l; S[l] = -1; }
        for (int changed = 1; changed;) {        /* label propagation; graphs here are tiny */
            changed = 0;
            for (int e = 0; e < n_edges; ++e) if (E[e].alive) {
                int a = comp[E[e].src], b = comp[E[e].dst];
                if (a != b) { int m = a < b ? a : b; comp[E[e].src] = comp[E[e].dst] = m; changed = 1; }
            }
        }
        for (int root = 0; root < n_nodes; ++root) {
            if (dead[root] || comp[root] != root) continue;
            int K = 0, ne = 0;
            for (int l = 0; l < n_nodes; ++l) if (comp[l] == root) ine[K++] = l;      /* ine reused: member nodes, ascending */
            for (int e = 0; e < n_edges; ++e) if (E[e].alive && comp[E[e].src] == root) oute[ne++] = e;   /* oute reused */
            int64_t c = 0;
            if (K == 1) {
                int l = ine[0], best = 0;
                for (int q = 1; q < Cn[l]; ++q) if (w[woff[l] + q] < w[woff[l] + best]) best = q;
                c = w[woff[l] + best]; S[l] = best;
            } else if (K == 2 && ne == 1 && schedule != ORC_SCHEDULE_NONE) {   /* the baseline enumerates in node order */
                int e = oute[0]; int32_t a, b;
                int r = orc_final_pair(Cn[E[e].src], Cn[E[e].dst], w + woff[E[e].src], E[e].tab, w + woff[E[e].dst], &c, &a, &b);
                if (r != ORC_OK) { rc = r; goto done; }
                S[E[e].src] = a; S[E[e].dst] = b;
            } else {
                /* number of strategies of the component, counted in 64 bits */
                uint64_t n_assign = 1;
                if (K > 16 || ne > 64) { rc = ORC_E_NOT_REDUCIBLE; goto done; }
                for (int q = 0; q < K; ++q) {
                    n_assign *= (uint64_t)Cn[ine[q]];
                    if (n_assign > ((uint64_t)1 << 32)) { rc = ORC_E_NOT_REDUCIBLE; goto done; }
                }
                int bestd[16], pos_of_src[64], pos_of_dst[64];
                for (int x = 0; x < ne; ++x)
                    for (int q = 0; q < K; ++q) {
                        if (ine[q] == E[oute[x]].src) pos_of_src[x] = q;
                        if (ine[q] == E[oute[x]].dst) pos_of_dst[x] = q;
                    }
                /* The configurations of the component's first node are independent slices of the
                 * enumeration: each slice keeps its own first optimum (threads share the slices),
                 * and the slices are then compared in ascending order with strict '<', which is
                 * the order one odometer over all K digits would visit them in. */
                int C0 = Cn[ine[0]];
                int64_t *slice_cost = (int64_t *)malloc(sizeof(int64_t) * (size_t)C0);
                int32_t *slice_digits = (int32_t *)malloc(sizeof(int32_t) * 16 * (size_t)C0);
                if (!slice_cost || !slice_digits) { free(slice_cost); free(slice_digits); rc = ORC_E_NOMEM; goto done; }
                int overflow = 0;
#pragma omp parallel for schedule(dynamic) reduction(| : overflow)
                for (int d0 = 0; d0 < C0; ++d0) {
                    int digit[16];
                    int64_t bc = 0;
                    int have = 0;
                    digit[0] = d0;
                    for (int q = 1; q < K; ++q) digit[q] = 0;
                    for (;;) {
                        int64_t t = 0;
                        for (int q = 0; q < K; ++q) t += w[woff[ine[q]] + digit[q]];
                        for (int x = 0; x < ne; ++x)
                            t += E[oute[x]].tab[(size_t)digit[pos_of_src[x]] * Cn[E[oute[x]].dst] + digit[pos_of_dst[x]]];
                        if (!fits_i32(t)) overflow = 1;
                        if (!have || t < bc) {
                            bc = t; have = 1;
                            for (int q = 0; q < K; ++q) slice_digits[(size_t)d0 * 16 + q] = digit[q];
                        }
                        int q = K - 1;                           /* odometer: last node fastest */
                        while (q >= 1 && ++digit[q] == Cn[ine[q]]) digit[q--] = 0;
                        if (q < 1) break;
                    }
                    slice_cost[d0] = bc;
                }
                for (int d0 = 0; d0 < C0; ++d0)
                    if (d0 == 0 || slice_cost[d0] < c) {
                        c = slice_cost[d0];
                        for (int q = 0; q < K; ++q) bestd[q] = slice_digits[(size_t)d0 * 16 + q];
                    }
                free(slice_cost); free(slice_digits);
                if (overflow) { rc = ORC_E_OVERFLOW; goto done; }
                for (int q = 0; q < K; ++q) S[ine[q]] = bestd[q];
            }
            total += c;
        }
        if (!fits_i32(total)) { rc = ORC_E_OVERFLOW; goto done; }
        *out_cost = total;
    }
    /* ---- undo in reverse order ---- */
    for (int t = nlog - 1; t >= 0; --t) {
        if (log[t].kind != 0) continue;                    /* edge eliminations change nothing */
        S[log[t].j] = argtab[t][(size_t)S[log[t].i] * Cn[log[t].k] + S[log[t].k]];
    }

done:
    if (steps && rc == ORC_OK) memcpy(steps, log, sizeof(orc_step) * nlog);
    if (n_steps) *n_steps = nlog;
    if (n_rounds) *n_rounds = rounds;
    if (E) for (int e = 0; e < n_edges; ++e) if (E[e].owned) free(E[e].tab);
    if (argtab) for (int t = 0; t < n_edges; ++t) free(argtab[t]);
    free(woff); free(w); free(E); free(log); free(argtab); free(dead); free(sel);
    free(indeg); free(outdeg); free(ine); free(oute); free(ids);
    return rc;
}

/* The same with one configuration count C for every node: tc, ts [N][C], tx [E][C][C]. */
int orc_search(int n_nodes, int n_edges, const int32_t *edges, int C,
               const int32_t *tc, const int32_t *ts, const int32_t *tx, int schedule,
               int64_t *out_cost, int32_t *S, orc_step *steps, int32_t *n_steps, int32_t *n_rounds)
{
    if (n_nodes <= 0 || C <= 0) return ORC_E_INVAL;
    int32_t *Cn = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_nodes);
    if (!Cn) return ORC_E_NOMEM;
    for (int l = 0; l < n_nodes; ++l) Cn[l] = C;
    int rc = orc_search_ragged(n_nodes, n_edges, edges, Cn, tc, ts, tx, schedule, out_cost, S, steps, n_steps, n_rounds);
    free(Cn);
    return rc;
}

int orc_strategy_cost(int n_nodes, int n_edges, const int32_t *edges, int C,
                      const int32_t *tc, const int32_t *ts, const int32_t *tx,
                      const int32_t *S, int64_t *out_cost)
{
    if (n_nodes <= 0 || C <= 0) return ORC_E_INVAL;
    int32_t *Cn = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_nodes);
    if (!Cn) return ORC_E_NOMEM;
    for (int l = 0; l < n_nodes; ++l) Cn[l] = C;
    int rc = orc_strategy_cost_ragged(n_nodes, n_edges, edges, Cn, tc, ts, tx, S, out_cost);
    free(Cn);
    return rc;
}
