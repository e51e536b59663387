// Internal layouts shared by the host packer and the HIP kernels.
// Not part of the public ABI.
#ifndef MGK_INTERNAL_H
#define MGK_INTERNAL_H

#include <stdint.h>

#if defined(__HIPCC__)
#define MGK_HD __host__ __device__
#else
#define MGK_HD
#endif

// One graph of a batch, as the device sees it (32 bytes).  All offsets index
// the batch-wide arrays of MgkBatchDev.
struct MgkGraphDesc {
    int32_t n;            // vertices
    int32_t nnz;          // stored nonzeros of the symmetric A (2 per edge)
    int32_t n_tiles;      // non-empty octiles
    int32_t n_tile_rows;  // ceil(n / 8)
    int32_t voff;         // first vertex in the per-vertex arrays
    int32_t zoff;         // first packed nonzero in w[] / e[]
    int32_t toff;         // first tile in tiles[]
    int32_t roff;         // first entry in trow_ptr[] (n_tile_rows + 1 entries)
};

// One non-empty octile (Section IV-A/B): tile coordinates, occupancy bitmap
// (bit 8*r + c <-> element (r, c) of the tile) and where its packed nonzeros
// start, relative to the graph's zoff.  Tiles of a graph are sorted by
// (tile_row, tile_col); nonzeros inside a tile are packed in bit order.
struct MgkTile {
    uint16_t tr, tc;
    uint32_t nzoff;
    uint64_t bitmap;
};

struct MgkBatchDev {
    const MgkGraphDesc* graphs;
    const MgkTile* tiles;
    const float* w;          // packed edge weights A_ij
    const float* e;          // packed edge labels E_ij
    const int32_t* vlabel;   // vertex labels (stored order)
    const float* rowsum;     // sum_j A_ij per vertex; d_i = rowsum + q (Eq. 1)
    const float* start;      // starting probability p_i
    const int32_t* rowptr;   // per vertex: nonzeros of the graph in rows before it
    const int32_t* trow_ptr; // per graph: tile-row pointers into its tile list
};

// One unit of work: solve the pair (outer graph g1 of batch X, inner graph g2
// of batch Y) and write the value to out0 (and out1 if >= 0).
struct MgkJob {
    int32_t g1, g2;
    int32_t out0, out1;
};

enum { MGK_EK_CONST = 0, MGK_EK_SE = 1 };

struct MgkParams {
    float q;          // stopping probability
    float h;          // vertex kernel off-diagonal value
    float e_scale;    // sqrt(alpha * log2(e)): kappa_e = exp2(-((e-e')*e_scale)^2)
    float e_shift;    // common shift applied to labels before scaling
    float ke_const;   // constant edge kernel value
    float rtol2;      // rtol^2
    int32_t max_iter; // <= 0: automatic
    int32_t edge_kernel;
};

// ---- LDS plan of the on-chip solver (one workgroup per pair) ---------------
// words (4 bytes each):
//   x, r, p, a, M            5 * N            N = n1 * n2
//   rowptr1                  n1 + 1
//   ent1 (outer graph)       4 * z1           {p-row byte offset, label, weight, -}
//   ent2 (inner graph)       4 * z2           {i'*4, j'*4, label, log2 weight}
//   reduction scratch        64
static inline MGK_HD int64_t mgk_small_lds_words(int64_t n1, int64_t n2, int64_t z1, int64_t z2) {
    int64_t words = 5 * n1 * n2 + (n1 + 1);
    words = (words + 3) & ~(int64_t)3;  // ent arrays are 16-byte aligned
    words += 4 * z1 + 4 * z2 + 64;
    return words;
}

#define MGK_LDS_LIMIT_BYTES (160 * 1024)

#endif
