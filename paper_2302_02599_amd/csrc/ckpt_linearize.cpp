// Host-side network linearisation: cuts a computation DAG, given in topological order,
// into the node groups that become the stages of a chain (Sections "Linearization",
// "Common Node" and the algorithm of "Full Set of Linearization Rules").
#include <cstdint>
#include <vector>

#include "ckpt_dp.h"

extern "C" int ckpt_linearize(int n, const int32_t* child_ptr, const int32_t* child_idx, const uint8_t* flags,
                              int32_t* group_of_node, uint8_t* is_common) {
    if (n < 0 || !child_ptr || !flags || !group_of_node || !is_common) return CKPT_E_ARG;
    if (child_ptr[0] != 0) return CKPT_E_ARG;
    for (int v = 0; v < n; ++v) {
        if (child_ptr[v + 1] < child_ptr[v]) return CKPT_E_ARG;
        if (child_ptr[v + 1] > child_ptr[v] && !child_idx) return CKPT_E_ARG;
        for (int e = child_ptr[v]; e < child_ptr[v + 1]; ++e)
            if (child_idx[e] <= v || child_idx[e] >= n) return CKPT_E_ARG;  // not a topological order
    }
    // One pass in node order.  pending[v] = dependencies of v not yet released; open = number
    // of nodes with pending > 0 (the "pool" is empty iff open == 0).
    std::vector<int32_t> pending(n, 0);
    std::vector<uint8_t> tracked(n, 0);
    int open = 0, groups = 0;
    for (int v = 0; v < n; ++v) is_common[v] = (flags[v] & CKPT_NODE_COMMON_SEED) ? 1 : 0;
    // the release step walks a node's parents: build the reverse adjacency once
    std::vector<int32_t> par_ptr(n + 1, 0);
    for (int e = 0; e < child_ptr[n]; ++e) ++par_ptr[child_idx[e] + 1];
    for (int v = 0; v < n; ++v) par_ptr[v + 1] += par_ptr[v];
    std::vector<int32_t> par_idx(child_ptr[n]), fill(par_ptr.begin(), par_ptr.end() - 1);
    for (int v = 0; v < n; ++v)
        for (int e = child_ptr[v]; e < child_ptr[v + 1]; ++e) par_idx[fill[child_idx[e]]++] = v;

    for (int v = 0; v < n; ++v) group_of_node[v] = -1;
    std::vector<int32_t> current;
    for (int v = 0; v < n; ++v) {
        if (flags[v] & CKPT_NODE_PLACEHOLDER) continue;
        bool parents_common = true;
        for (int e = par_ptr[v]; e < par_ptr[v + 1]; ++e) {
            const int p = par_idx[e];
            if (!is_common[p]) parents_common = false;
            if (tracked[p] && --pending[p] == 0) --open;
        }
        current.push_back(v);
        bool sticky = false;
        int deps = 0;
        for (int e = child_ptr[v]; e < child_ptr[v + 1]; ++e) {
            const uint8_t cf = flags[child_idx[e]];
            if (cf & (CKPT_NODE_IN_PLACE | CKPT_NODE_COMM)) sticky = true;
            if (!(cf & CKPT_NODE_PLACEHOLDER)) ++deps;
        }
        if (open == 0 && !sticky) {
            for (int u : current) group_of_node[u] = groups;
            ++groups;
            current.clear();
        }
        if ((flags[v] & CKPT_NODE_NON_DIFF) || parents_common) {
            is_common[v] = 1;
        } else if (deps > 0) {
            tracked[v] = 1;
            pending[v] = deps;
            ++open;
        }
    }
    if (!current.empty()) {
        for (int u : current) group_of_node[u] = groups;
        ++groups;
    }
    return groups;
}
