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
#include <map>
#include <queue>
#include <utility>

namespace lwp {

namespace {
struct Edge { int32_t src, dst; bool live; };
}

lwp_status make_plan(int32_t n_nodes, int32_t n_edges, const int32_t* edges, int32_t schedule,
                     Plan& plan, std::string& err) {
    plan = Plan();
    if (n_nodes <= 0 || n_edges < 0 || (n_edges > 0 && !edges)) { err = "bad graph sizes"; return LWP_E_INVAL; }
    if (schedule != LWP_SCHEDULE_ROUNDS && schedule != LWP_SCHEDULE_LEFT_FOLD) { err = "unknown schedule"; return LWP_E_INVAL; }
    std::vector<Edge> E(n_edges);
    for (int32_t e = 0; e < n_edges; ++e) {
        int32_t s = edges[2 * e], d = edges[2 * e + 1];
        if (s < 0 || s >= n_nodes || d < 0 || d >= n_nodes) { err = "edge endpoint out of range"; return LWP_E_GRAPH; }
        if (s == d) { err = "self loop"; return LWP_E_GRAPH; }
        E[e] = {s, d, true};
    }
    {   // acyclicity (Kahn)
        std::vector<int32_t> indeg(n_nodes, 0);
        std::vector<std::vector<int32_t>> succ(n_nodes);
        for (auto& e : E) { indeg[e.dst]++; succ[e.src].push_back(e.dst); }
        std::queue<int32_t> q;
        for (int32_t v = 0; v < n_nodes; ++v) if (!indeg[v]) q.push(v);
        int32_t seen = 0;
        while (!q.empty()) {
            int32_t v = q.front(); q.pop(); ++seen;
            for (int32_t u : succ[v]) if (--indeg[u] == 0) q.push(u);
        }
        if (seen != n_nodes) { err = "graph has a cycle"; return LWP_E_GRAPH; }
    }

    std::vector<char> gone(n_nodes, 0), taken(n_nodes, 0);
    std::vector<int32_t> n_in(n_nodes), n_out(n_nodes), e_in(n_nodes), e_out(n_nodes);
    int32_t round = 0;
    for (;;) {
        bool worked = false;
        // E-phase
        std::map<std::pair<int32_t, int32_t>, std::vector<int32_t>> groups;
        for (int32_t e = 0; e < n_edges; ++e) if (E[e].live) groups[{E[e].src, E[e].dst}].push_back(e);
        for (auto& g : groups) {
            const std::vector<int32_t>& ids = g.second;       // ascending by construction
            for (size_t z = 1; z < ids.size(); ++z) {
                plan.steps.push_back({1, -1, g.first.first, g.first.second, ids[0], ids[z], round});
                E[ids[z]].live = false;
                ++plan.n_edge_steps;
                worked = true;
            }
        }
        // N-phase
        for (int32_t v = 0; v < n_nodes; ++v) { n_in[v] = n_out[v] = 0; taken[v] = 0; }
        for (int32_t e = 0; e < n_edges; ++e) if (E[e].live) {
            n_out[E[e].src]++; e_out[E[e].src] = e;
            n_in[E[e].dst]++;  e_in[E[e].dst] = e;
        }
        std::vector<int32_t> chosen;
        for (int32_t j = 0; j < n_nodes; ++j) {
            if (gone[j] || n_in[j] != 1 || n_out[j] != 1) continue;
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
        else if (c.nodes.size() == 2 && c.edges.size() == 1) plan.pairs.push_back({c.edges[0], c.esrc[0], c.edst[0]});
        else if ((int)c.nodes.size() > kMaxComponentNodes || (int)c.edges.size() > kMaxComponentEdges) {
            err = "a residual component has more than " + std::to_string(kMaxComponentNodes) + " nodes or " +
                  std::to_string(kMaxComponentEdges) + " edges";
            return LWP_E_NOT_REDUCIBLE;
        } else plan.comps.push_back(std::move(c));
    }
    return LWP_OK;
}

}  // namespace lwp
