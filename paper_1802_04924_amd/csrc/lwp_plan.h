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

struct Plan {
    std::vector<lwp_step> steps;          // execution order
    int32_t n_rounds = 0;                 // rounds that did work
    std::vector<ResidualPair> pairs;      // residual components with two nodes (one live edge)
    std::vector<int32_t> singles;         // residual isolated nodes
    int32_t n_node_steps = 0, n_edge_steps = 0;
};

// Validates the graph (endpoints, self loops, acyclicity) and runs the canonical schedule.
lwp_status make_plan(int32_t n_nodes, int32_t n_edges, const int32_t* edges, int32_t schedule,
                     Plan& plan, std::string& err);

}  // namespace lwp
