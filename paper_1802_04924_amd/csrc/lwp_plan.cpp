// Canonical elimination schedule.  The paper only says "if there exists a node / two edges"
// (Alg. 2); the rule below fixes the choice so that results are reproducible:
//
//   repeat rounds until a round changes nothing
//     E-phase: for every (src,dst) with >= 2 live parallel edges, ascending (src,dst): the
//              edges with higher ids are added, ascending, into the lowest id (Eq. 3);
//     N-phase: nodes in ascending id; j is eligible with exactly one live in-edge (i,j) and
//              one live out-edge (j,k).  ROUNDS takes j unless i or k was taken in this round
//              (the taken nodes share no edge, so they are eliminated together); LEFT_FOLD
//              takes the first eligible node only.  The new edge (i,k) keeps the in-edge's id.
#include "lwp_plan.h"

#include <algorithm>
#include <utility>

namespace lwp {

namespace {
struct Edge { int32_t src, dst; bool live; };
}

lwp_status make_plan(int32_t n_nodes, int32_t n_edges, const int32_t* edges, int32_t schedule,
                     Plan& plan, std::string& err) {
    plan = Plan();
    if (n_nodes <= 0 || n_edges < 0 || (n_edges > 0 && !edges)) { err = "bad graph sizes"; return LWP_E_INVAL; }
    if (schedule != LWP_SCHEDULE_ROUNDS && schedule != LWP_SCHEDULE_LEFT_FOLD && schedule != LWP_SCHEDULE_NONE) {
        err = "unknown schedule";
        return LWP_E_INVAL;
    }
    std::vector<Edge> E(n_edges);
    for (int32_t e = 0; e < n_edges; ++e) {
        int32_t s = edges[2 * e], d = edges[2 * e + 1];
        if (s < 0 || s >= n_nodes || d < 0 || d >= n_nodes) { err = "edge endpoint out of range"; return LWP_E_GRAPH; }
        if (s == d) { err = "self loop"; return LWP_E_GRAPH; }
        E[e] = {s, d, true};
    }
    {   // acyclicity (Kahn), successors in compressed rows
        std::vector<int32_t> indeg(n_nodes, 0), first(n_nodes + 1, 0), succ(n_edges), order;
        for (auto& e : E) { indeg[e.dst]++; first[e.src + 1]++; }
        for (int32_t v = 0; v < n_nodes; ++v) first[v + 1] += first[v];
        std::vector<int32_t> fill(first.begin(), first.end() - 1);
        for (auto& e : E) succ[fill[e.src]++] = e.dst;
        order.reserve(n_nodes);
        for (int32_t v = 0; v < n_nodes; ++v) if (!indeg[v]) order.push_back(v);
        for (size_t head = 0; head < order.size(); ++head) {
            const int32_t v = order[head];
            for (int32_t x = first[v]; x < first[v + 1]; ++x) if (--indeg[succ[x]] == 0) order.push_back(succ[x]);
        }
        if ((int32_t)order.size() != n_nodes) { err = "graph has a cycle"; return LWP_E_GRAPH; }
    }

    // Every round walks only what is still alive: the live edges (ascending id) and the nodes not yet
    // eliminated (ascending id), both compacted after the round -- a schedule in rounds halves a chain
    // every time, so the whole plan costs about what its first round does.
    std::vector<char> gone(n_nodes, 0), taken(n_nodes, 0);
    std::vector<int32_t> n_in(n_nodes, 0), n_out(n_nodes, 0), e_in(n_nodes), e_out(n_nodes), start_of(n_nodes);
    std::vector<int32_t> live_e(n_edges), live_v(n_nodes), by_src(n_edges), chosen;
    for (int32_t e = 0; e < n_edges; ++e) live_e[e] = e;
    for (int32_t v = 0; v < n_nodes; ++v) live_v[v] = v;
    // degrees and, where the degree is one, the edge (n_in / n_out of live nodes are zero beforehand)
    auto count_degrees = [&]() {
        bool several_out = false;
        for (int32_t e : live_e) if (E[e].live) {
            const int32_t s = E[e].src, d = E[e].dst;
            several_out |= (++n_out[s] == 2);
            e_out[s] = e;
            ++n_in[d];
            e_in[d] = e;
        }
        return several_out;
    };
    int32_t round = 0;
    plan.steps.reserve(n_edges);
    for (;;) {
        // the exhaustive baseline (Sec. 5.2, Table 3) searches the original graph: no eliminations
        if (schedule == LWP_SCHEDULE_NONE) break;
        bool worked = false;
        // E-phase.  Parallel edges need a source with several live out-edges; then: the live edges of
        // every source, ascending id, ordered by destination; equal (src, dst) form a group.  Sources
        // ascending, destinations ascending within a source.
        if (count_degrees()) {
            int32_t run = 0;
            for (int32_t v : live_v) { run += n_out[v]; start_of[v] = run; }
            for (size_t x = live_e.size(); x-- > 0;) by_src[--start_of[E[live_e[x]].src]] = live_e[x];
            bool merged = false;
            for (int32_t v : live_v) {
                const int32_t cnt = n_out[v];
                if (cnt < 2) continue;
                int32_t* first = by_src.data() + start_of[v];
                std::stable_sort(first, first + cnt, [&](int32_t a, int32_t b2) { return E[a].dst < E[b2].dst; });
                for (int32_t g0 = 0; g0 < cnt;) {
                    int32_t g1 = g0 + 1;
                    while (g1 < cnt && E[first[g1]].dst == E[first[g0]].dst) ++g1;
                    for (int32_t z = g0 + 1; z < g1; ++z) {
                        plan.steps.push_back({1, -1, v, E[first[g0]].dst, first[g0], first[z], round});
                        E[first[z]].live = false;
                        ++plan.n_edge_steps;
                        merged = true;
                    }
                    g0 = g1;
                }
            }
            if (merged) {               // the degrees again, without the merged edges
                worked = true;
                for (int32_t v : live_v) n_in[v] = n_out[v] = 0;
                count_degrees();
            }
        }
        // N-phase
        chosen.clear();
        for (int32_t j : live_v) {
            if (n_in[j] != 1 || n_out[j] != 1) continue;
            int32_t i = E[e_in[j]].src, k = E[e_out[j]].dst;
            if (taken[i] || taken[k]) continue;
            taken[j] = 1;
            chosen.push_back(j);
            if (schedule == LWP_SCHEDULE_LEFT_FOLD) break;
        }
        for (int32_t j : chosen) {
            int32_t e1 = e_in[j], e2 = e_out[j];
            int32_t i = E[e1].src, k = E[e2].dst;
            plan.steps.push_back({0, j, i, k, e1, e2, round});
            E[e1].dst = k;
            E[e2].live = false;
            gone[j] = 1;
            ++plan.n_node_steps;
            worked = true;
        }
        if (!worked) break;
        live_e.erase(std::remove_if(live_e.begin(), live_e.end(), [&](int32_t e) { return !E[e].live; }), live_e.end());
        size_t keep = 0;
        for (int32_t v : live_v) {
            if (gone[v]) continue;
            n_in[v] = n_out[v] = 0;
            taken[v] = 0;
            live_v[keep++] = v;
        }
        live_v.resize(keep);
        ++round;
    }
    plan.n_rounds = round;

    // residual graph: connected components over the live edges
    std::vector<int32_t> label(n_nodes);
    for (int32_t v = 0; v < n_nodes; ++v) label[v] = gone[v] ? -1 : v;
    for (bool changed = true; changed;) {
        changed = false;
        for (int32_t e = 0; e < n_edges; ++e) if (E[e].live) {
            int32_t a = label[E[e].src], b = label[E[e].dst];
            if (a != b) { label[E[e].src] = label[E[e].dst] = std::min(a, b); changed = true; }
        }
    }
    for (int32_t root = 0; root < n_nodes; ++root) {
        if (gone[root] || label[root] != root) continue;
        ResidualComponent c;
        for (int32_t v = root; v < n_nodes; ++v) if (label[v] == root) c.nodes.push_back(v);
        for (int32_t e = 0; e < n_edges; ++e) if (E[e].live && label[E[e].src] == root) {
            c.edges.push_back(e); c.esrc.push_back(E[e].src); c.edst.push_back(E[e].dst);
        }
        if (c.nodes.size() == 1) plan.singles.push_back(root);
        else if (c.nodes.size() == 2 && c.edges.size() == 1 && schedule != LWP_SCHEDULE_NONE)   // (the baseline enumerates in node order)
            plan.pairs.push_back({c.edges[0], c.esrc[0], c.edst[0]});
        else if ((int)c.nodes.size() > kMaxComponentNodes || (int)c.edges.size() > kMaxComponentEdges) {
            err = "a residual component has more than " + std::to_string(kMaxComponentNodes) + " nodes or " +
                  std::to_string(kMaxComponentEdges) + " edges";
            return LWP_E_NOT_REDUCIBLE;
        } else plan.comps.push_back(std::move(c));
    }
    return LWP_OK;
}

}  // namespace lwp
