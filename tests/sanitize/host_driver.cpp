// Host-only exercise of the CPU oracle (oracle/*.c) and of the library's elimination scheduler
// (csrc/lwp_plan.cpp) for a build with -fsanitize=address,undefined: random graphs (valid, cyclic,
// with bad endpoints), random tables with heavy ties, per-node configuration counts, both schedules.
// Besides whatever the sanitizers report (signed overflow in the oracle IS the overflow
// precondition), it checks what must hold of any run: the scheduler's step log equals the oracle's,
// and the oracle's cost equals Eq. 1 of the strategy it returns.  No GPU call, no HIP header.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "lwp_plan.h"

extern "C" {
typedef struct { int32_t kind, j, i, k, e1, e2, round; } orc_step;
int orc_search_ragged(int n_nodes, int n_edges, const int32_t* edges, const int32_t* Cn, const int32_t* tc,
                      const int32_t* ts, const int32_t* tx, int schedule, int64_t* out_cost, int32_t* S,
                      orc_step* steps, int32_t* n_steps, int32_t* n_rounds);
int orc_strategy_cost_ragged(int n_nodes, int n_edges, const int32_t* edges, const int32_t* Cn, const int32_t* tc,
                             const int32_t* ts, const int32_t* tx, const int32_t* S, int64_t* out_cost);
int orc_minplus_argmin(int Ci, int Cj, int Ck, const int32_t* A, const int32_t* w, const int32_t* B, int32_t* out,
                       int32_t* arg);
int orc_edge_sum(int Ci, int Cj, const int32_t* e1, const int32_t* e2, int32_t* out);
typedef struct { int32_t kind, N, Cin, Hin, Win, Cout, Hout, Wout, kh, kw, sh, sw, ph, pw; } orc_layer;
typedef struct { int32_t n, h, w, c, dev_offset, pad; } orc_config;
typedef struct { int32_t n_devices, flop_per_ns, byte_per_ns, invalid_cost; } orc_machine;
int orc_enumerate_configs(const orc_layer* L, int n_devices, orc_config* out, int cap);
int orc_build_cost_tables_ragged(const orc_layer* layers, int n_layers, const int32_t* edges, int n_edges,
                                 const orc_config* cfgs, const int32_t* Cn, const orc_machine* m, int32_t* tc,
                                 int32_t* ts, int32_t* tx);
}

#define CHECK(cond, ...)                                      \
    do {                                                      \
        if (!(cond)) {                                        \
            std::fprintf(stderr, "FAILED %s: ", #cond);       \
            std::fprintf(stderr, __VA_ARGS__);                \
            std::fprintf(stderr, "\n");                       \
            std::exit(1);                                     \
        }                                                     \
    } while (0)

int main() {
    std::mt19937 rng(20180213);
    long searched = 0, refused = 0, irreducible = 0;
    for (int it = 0; it < 2000; ++it) {
        const int n = 1 + rng() % 14;
        const int e = rng() % 22;
        std::vector<int32_t> edges(2 * (size_t)e), Cn(n);
        for (auto& c : Cn) c = 1 + rng() % (n > 8 ? 3 : 5);    // residual components are enumerated outright
        const int kind = rng() % 8;             // 0: arbitrary endpoints (cycles, self loops), 1: a bad endpoint, else a DAG
        for (int q = 0; q < e; ++q) {
            int a = rng() % n, b = rng() % n;
            if (kind >= 2 && n > 1) {
                while (a == b) b = rng() % n;
                if (a > b) std::swap(a, b);
            }
            edges[2 * q] = a; edges[2 * q + 1] = b;
        }
        if (kind == 1 && e > 0) edges[rng() % (2 * e)] = (rng() % 2) ? -1 : n;
        const int hi = (rng() % 3 == 0) ? 1 : 1000;      // heavy ties every third graph
        size_t rows = 0, cells = 0;
        for (int v = 0; v < n; ++v) rows += Cn[v];
        bool endpoints_ok = true;
        for (int q = 0; q < 2 * e; ++q) endpoints_ok = endpoints_ok && edges[q] >= 0 && edges[q] < n;
        for (int q = 0; q < e && endpoints_ok; ++q) cells += (size_t)Cn[edges[2 * q]] * Cn[edges[2 * q + 1]];
        std::vector<int32_t> tc(rows), ts(rows), tx(cells ? cells : 1);
        for (auto& x : tc) x = rng() % (hi + 1);
        for (auto& x : ts) x = rng() % (hi + 1);
        for (auto& x : tx) x = rng() % (hi + 1);
        for (int sched = 0; sched < 2; ++sched) {
            lwp::Plan plan;
            std::string err;
            const lwp_status ps = lwp::make_plan(n, e, edges.data(), sched, plan, err);
            if (ps == LWP_E_GRAPH || ps == LWP_E_INVAL) { ++refused; continue; }
            if (ps == LWP_E_NOT_REDUCIBLE) { ++irreducible; continue; }
            CHECK(ps == LWP_OK, "make_plan returned %d", (int)ps);
            std::vector<orc_step> log(e > 0 ? e : 1);
            std::vector<int32_t> S(n);
            int64_t cost = 0, again = 0;
            int32_t ns = 0, nr = 0;
            const int rc = orc_search_ragged(n, e, edges.data(), Cn.data(), tc.data(), ts.data(), tx.data(), sched, &cost,
                                             S.data(), log.data(), &ns, &nr);
            CHECK(rc == 0, "oracle search returned %d on a graph the scheduler accepts", rc);
            CHECK((size_t)ns == plan.steps.size() && nr == plan.n_rounds, "log lengths differ: %d/%zu steps, %d/%d rounds",
                  ns, plan.steps.size(), nr, plan.n_rounds);
            for (int q = 0; q < ns; ++q) {
                const lwp_step& a = plan.steps[q];
                const orc_step& b = log[q];
                CHECK(a.kind == b.kind && a.j == b.j && a.i == b.i && a.k == b.k && a.e1 == b.e1 && a.e2 == b.e2 &&
                      a.round == b.round, "step %d differs", q);
            }
            CHECK(orc_strategy_cost_ragged(n, e, edges.data(), Cn.data(), tc.data(), ts.data(), tx.data(), S.data(), &again) == 0,
                  "strategy out of range");
            CHECK(again == cost, "Eq. 1 of the returned strategy is %lld, the search says %lld", (long long)again, (long long)cost);
            ++searched;
        }
    }
    // Eq. 2 / Eq. 3 at the edges of int32: the oracle must report, not overflow
    {
        const int32_t big = INT32_MAX, small = INT32_MIN;
        std::vector<int32_t> A{big, small, 5, -5}, w{big, small}, B{big, 7, small, -7}, out(4), arg(4);
        CHECK(orc_minplus_argmin(2, 2, 2, A.data(), w.data(), B.data(), out.data(), arg.data()) == -4, "overflow not reported");
        CHECK(orc_edge_sum(2, 2, A.data(), B.data(), out.data()) == -4, "overflow not reported");
    }
    // cost model: random layers, every enumerated configuration, consecutive layers as edges
    for (int it = 0; it < 40; ++it) {
        const int L = 2 + rng() % 3, ndev = 1 << (rng() % 4);
        std::vector<orc_layer> layers(L);
        int C = 3 + rng() % 30, H = 4 + rng() % 20;
        const int N = 1 + rng() % 16;
        for (int l = 0; l < L; ++l) {
            const int kind = (l == L - 1) ? 2 : (int)(rng() % 2);
            const int k = 1 + 2 * (rng() % 2), s = 1 + rng() % 2, p = k / 2;
            orc_layer& x = layers[l];
            x.kind = kind; x.N = N; x.Cin = C; x.Hin = H; x.Win = H;
            x.kh = x.kw = kind == 2 ? 1 : k; x.sh = x.sw = kind == 2 ? 1 : s; x.ph = x.pw = kind == 2 ? 0 : p;
            x.Cout = kind == 1 ? C : 2 + (int)(rng() % 40);
            x.Hout = x.Wout = kind == 2 ? 1 : (H + 2 * p - x.kh) / x.sh + 1;
            C = x.Cout; H = x.Hout;
        }
        std::vector<int32_t> edges, Cn(L);
        for (int l = 0; l + 1 < L; ++l) { edges.push_back(l); edges.push_back(l + 1); }
        std::vector<orc_config> cfgs;
        for (int l = 0; l < L; ++l) {
            const int cnt = orc_enumerate_configs(&layers[l], ndev, nullptr, 0);
            CHECK(cnt >= 1, "a layer without configurations");
            std::vector<orc_config> mine(cnt);
            CHECK(orc_enumerate_configs(&layers[l], ndev, mine.data(), cnt) == cnt, "count changed");
            Cn[l] = cnt;
            cfgs.insert(cfgs.end(), mine.begin(), mine.end());
        }
        size_t rows = 0, cells = 0;
        for (int l = 0; l < L; ++l) rows += Cn[l];
        for (int l = 0; l + 1 < L; ++l) cells += (size_t)Cn[l] * Cn[l + 1];
        std::vector<int32_t> tc(rows), ts(rows), tx(cells);
        const orc_machine m{ndev, 10000, 10, 1 << 28};
        const int rc = orc_build_cost_tables_ragged(layers.data(), L, edges.data(), L - 1, cfgs.data(), Cn.data(), &m, tc.data(),
                                                    ts.data(), tx.data());
        CHECK(rc == 0, "cost model returned %d", rc);
        for (auto x : tc) CHECK(x >= 0, "negative t_c");
        for (auto x : tx) CHECK(x >= 0, "negative t_x");
    }
    std::printf("sanitized host run ok: %ld searches checked, %ld graphs refused, %ld not reducible\n", searched, refused,
                irreducible);
    return 0;
}
