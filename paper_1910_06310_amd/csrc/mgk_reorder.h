// Vertex orderings for tile packing (Section IV-A).  Host only.
#ifndef MGK_REORDER_H
#define MGK_REORDER_H

#include <stdint.h>

#include <vector>

// Undirected graph in CSR form over both directions of every edge.
struct MgkAdj {
    int n = 0;
    std::vector<int32_t> ptr;  // n + 1
    std::vector<int32_t> idx;  // neighbours
};

// Each function returns perm with perm[old_id] = new_id, a bijection on [0, n).
std::vector<int32_t> mgk_order_identity(int n);
// Reverse Cuthill-McKee: breadth-first from a pseudo-peripheral vertex of each
// component, neighbours by increasing degree, order reversed.
std::vector<int32_t> mgk_order_rcm(const MgkAdj& g);
// Partition-based reordering: a perfectly balanced K = ceil(n/t)-way partition
// (all parts of size t except possibly the last) that aims at the fewest
// pairs of distinct parts joined by an edge (Eq. 3); part k occupies new ids
// [k t, (k+1) t).
std::vector<int32_t> mgk_order_pbr(const MgkAdj& g, int t);

// Space-filling-curve order for vertices with coordinates (Section IV-A): each of the
// `dim` (1..3) coordinates is scaled to the graph's bounding box and quantised to 10
// bits (21 / dim bits), the bits of the coordinates are interleaved (Morton, Z-order),
// and the vertices are numbered by that key (ties in the given order).
// coords[v * dim + a], all finite.
std::vector<int32_t> mgk_order_morton(int n, int dim, const float* coords);

// Number of ordered pairs (k, l), k != l, of t-blocks of the new numbering
// that are joined by at least one edge: the non-empty off-diagonal tiles.
int64_t mgk_count_offdiag_tiles(const MgkAdj& g, const std::vector<int32_t>& perm, int t);

#endif
