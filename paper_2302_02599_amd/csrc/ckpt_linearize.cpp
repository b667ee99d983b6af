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
    // One forward sweep over the CSR adjacency, no reverse edges and no dependency pool:
    //   - a node is common when it is seeded, non-differentiable, or has no non-common parent;
    //     every non-common node (placeholders included) counts itself into its children;
    //   - an examined, non-common node keeps dependencies outstanding until its last examined
    //     child has been appended, so "no dependency outstanding after v" is a running maximum
    //     of those last uses (horizon) that does not pass v.
    std::vector<int32_t> noncommon_parents(n, 0);
    int groups = 0;
    int32_t horizon = -1;
    bool open_group = false;
    for (int v = 0; v < n; ++v) {
        const bool placeholder = flags[v] & CKPT_NODE_PLACEHOLDER;
        const bool common = (flags[v] & CKPT_NODE_COMMON_SEED) ||
                            (!placeholder && ((flags[v] & CKPT_NODE_NON_DIFF) || noncommon_parents[v] == 0));
        is_common[v] = common ? 1 : 0;
        bool sticky = false;
        int32_t last_use = -1;
        for (int e = child_ptr[v]; e < child_ptr[v + 1]; ++e) {
            const int c = child_idx[e];
            if (!common) ++noncommon_parents[c];
            if (flags[c] & (CKPT_NODE_IN_PLACE | CKPT_NODE_COMM)) sticky = true;
            if (!(flags[c] & CKPT_NODE_PLACEHOLDER) && c > last_use) last_use = c;
        }
        if (placeholder) {
            group_of_node[v] = -1;
            continue;
        }
        group_of_node[v] = groups;
        open_group = true;
        if (horizon <= v && !sticky) {  // nothing outstanding, no child that sticks to v: v ends its group
            ++groups;
            open_group = false;
        }
        if (!common && last_use > horizon) horizon = last_use;
    }
    return groups + (open_group ? 1 : 0);
}
