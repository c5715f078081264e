// Host side of the multi-colour spanning trees (Section 4.2): who sums what for which colour.
//
// For each colour the nodes form a complete k-ary tree in breadth-first (heap) order:
// position p has children at positions k*p+1 .. k*p+k (those below n).  Positions
// 0 .. s-1 are the non-leaf ones, s = ceil((n-1)/k).  Colour c places node (p + c*s) mod n at
// position p, so the non-leaf nodes of colour c are the s consecutive nodes starting at c*s:
// disjoint across colours exactly when k*s <= n, which is also the fewest nodes any k such
// trees can do with.  Nothing here touches the GPU.
#include "mc_internal.h"

namespace {

// s: non-leaf positions per tree; false when disjoint sets cannot exist.
bool plan(int32_t n, int32_t k, int64_t* s_out) {
    if (n < 1 || k < 1) return false;
    const int64_t s = (int64_t(n) - 1 + k - 1) / k;
    if (int64_t(k) * s > n) return false;
    *s_out = s;
    return true;
}

}  // namespace

extern "C" {

int mc_colour_trees(int32_t n_nodes, int32_t k_colours, int32_t* parent) {
    int64_t s = 0;
    if (!parent || !plan(n_nodes, k_colours, &s)) return MC_ERR_INVALID_ARG;
    const int64_t n = n_nodes, k = k_colours;
    for (int64_t c = 0; c < k; ++c) {
        int32_t* row = parent + c * n;
        const int64_t shift = (c * s) % n;
        for (int64_t p = 0; p < n; ++p) {
            const int64_t node = (p + shift) % n;
            row[node] = p == 0 ? -1 : int32_t(((p - 1) / k + shift) % n);
        }
    }
    return MC_OK;
}

int mc_rank_roles(int32_t n_nodes, int32_t k_colours, int32_t rank, int32_t* role,
                  int32_t* n_children, int32_t* children) {
    int64_t s = 0;
    if (!role || !n_children || !children || !plan(n_nodes, k_colours, &s)) return MC_ERR_INVALID_ARG;
    if (rank < 0 || rank >= n_nodes) return MC_ERR_INVALID_ARG;
    const int64_t n = n_nodes, k = k_colours;
    for (int64_t c = 0; c < k; ++c) {
        const int64_t shift = (c * s) % n;
        const int64_t p = ((int64_t(rank) - shift) % n + n) % n;  // this rank's position in tree c
        int32_t cnt = 0;
        for (int64_t j = 1; j <= k; ++j) {
            const int64_t q = k * p + j;
            children[c * k + (j - 1)] = q < n ? int32_t((q + shift) % n) : -1;
            if (q < n) ++cnt;
        }
        n_children[c] = cnt;
        role[c] = p == 0 ? MC_ROLE_ROOT : (cnt > 0 ? MC_ROLE_INNER : MC_ROLE_LEAF);
    }
    return MC_OK;
}

}  // extern "C"
