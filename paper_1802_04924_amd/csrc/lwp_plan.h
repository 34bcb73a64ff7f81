// Host-side elimination scheduler (Alg. 1, elimination phase; Alg. 2 in the appendix).
// Which node or edge can be eliminated depends only on the topology, never on table values,
// so the whole schedule is computed on the CPU before anything is launched.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "lwp.h"

namespace lwp {

struct ResidualPair { int32_t edge, src, dst; };
// A residual component with more than two nodes (or more than one edge): solved by enumerating
// all strategies of its nodes (Alg. 1, "enumerating all possible candidate strategies").
struct ResidualComponent {
    std::vector<int32_t> nodes;   // ascending ids; the lowest id is the most significant digit
    std::vector<int32_t> edges;   // live edge ids inside the component
    std::vector<int32_t> esrc, edst;   // endpoints of those edges (current, after eliminations)
};
constexpr int kMaxComponentNodes = 12, kMaxComponentEdges = 32;

struct Plan {
    std::vector<lwp_step> steps;          // execution order
    int32_t n_rounds = 0;                 // rounds that did work
    std::vector<ResidualPair> pairs;      // residual components with two nodes (one live edge)
    std::vector<int32_t> singles;         // residual isolated nodes
    std::vector<ResidualComponent> comps; // residual components that need enumeration
    int32_t n_node_steps = 0, n_edge_steps = 0;
};

// Validates the graph (endpoints, self loops, acyclicity) and runs the canonical schedule.
lwp_status make_plan(int32_t n_nodes, int32_t n_edges, const int32_t* edges, int32_t schedule,
                     Plan& plan, std::string& err);

}  // namespace lwp
