// Weighted spanning trees of the rank graph: the hand-over between tree
// packing and scheduling (paper section 3.1: arborescences T_i with weights w_i).
#pragma once
#include <array>
#include <cstdint>
#include <vector>

#include "../../include/blink.h"

namespace blink {

using ParentVec = std::array<int8_t, BLINK_MAX_RANKS>;  // parent[v]; -1 at the root; unused tail = -2

struct Trees {
    int k = 0;
    std::vector<int> root;
    std::vector<ParentVec> parent;
    std::vector<double> weight;
    int count() const { return static_cast<int>(root.size()); }
};

// true iff following parents from every vertex reaches `root` (k-1 arcs, no cycle).
bool is_spanning_tree(int k, int root, const ParentVec& parent);

// children of every vertex in ascending id
std::vector<std::vector<int>> children(int k, const ParentVec& parent);

// Tree packing entry point used by the C ABI (pack.cpp).
blink_status_t pack_trees(int k, int m, const int32_t* src, const int32_t* dst, const double* cap,
                          int root, double eps, double prune_tol, Trees& out);

}  // namespace blink

struct blink_trees {
    blink::Trees t;
};
