// Maximum-weight matching in a general graph, for the per-round matchings of the
// schedule generator for even rank counts that are not powers of two (App. D).
//
// Two solvers over the same dense, symmetric weight table (0 = no edge):
//   - an exact recursion over subsets, whose choice among equally heavy matchings
//     is fixed (lowest vertex: unmatched first, then partners ascending; first
//     best wins), for up to 20 vertices;
//   - Edmonds' blossom algorithm in its O(V^3) primal-dual form (the App. D
//     reference for the matching step), for any size; which of several equally
//     heavy matchings it returns is not specified.
#pragma once
#include <cstdint>
#include <vector>

namespace sar {

// weight[a * k + b] for vertices a, b < k; symmetric, non-negative.
// mate[a] receives a's partner or -1.  Returns the matching's weight.
int64_t max_weight_matching_subsets(int k, const std::vector<int64_t>& weight, std::vector<int>& mate);
int64_t max_weight_matching_blossom(int k, const std::vector<int64_t>& weight, std::vector<int>& mate);

constexpr int kMaxSubsetVertices = 20;

}  // namespace sar
