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

// One graph of a batch, as the device sees it (40 bytes).  All offsets index
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
    int32_t max_deg;      // largest number of nonzeros in a row
    int32_t lane_len;     // lane slots of the graph as inner operand (multiple of 64)
    int32_t loff;         // first lane slot of the graph in batch-wide expanded inner lists
    int32_t regs_runs;    // longest run of outer nonzeros of one wavefront under regs_split:
                          // 4 wavefronts in bits 0-15, 8 wavefronts in bits 16-31
};

// Lane layout of a graph used as the inner operand of the on-chip XMV: the
// nonzeros of a row occupy adjacent lanes, and the sum over a row is a DPP
// shift-and-add inside one 16-lane row of a wavefront.  In a graph whose rows
// all have at most 16 nonzeros no row crosses a group of 16 lanes (a row that
// does not fit the rest of a group starts the next one), so every y_ii' has one
// writer.  A graph with longer rows needs atomic adds anyway (a long row is cut
// into several runs); there the rows are packed without gaps and every row that
// crosses a group boundary is cut at it.
#define MGK_LANE_GROUP 16

// Where nonzero `rank` of a row of `deg` nonzeros sits when the row starts at lane
// slot `first`: its position in its run (the part of the row inside one lane group),
// whether it is the last of the run, whether the row has more than one run.
struct MgkRunPos {
    uint32_t rank, last, cut;
};
static inline MGK_HD MgkRunPos mgk_run_pos(int first, int rank, int deg) {
    const int pos = first + rank;
    const int group = pos & ~(MGK_LANE_GROUP - 1);
    MgkRunPos r;
    r.rank = (uint32_t)(pos - (first > group ? first : group));
    r.last = (rank + 1 == deg || pos - group == MGK_LANE_GROUP - 1) ? 1u : 0u;
    r.cut = (first & (MGK_LANE_GROUP - 1)) + deg > MGK_LANE_GROUP ? 1u : 0u;
    return r;
}

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
    const int32_t* lanepos;  // per vertex: first lane slot of its row (inner operand layout)
    const int32_t* trow_ptr; // per graph: tile-row pointers into its tile list
    const int32_t* tile_graph; // per tile: the graph it belongs to
    const int32_t* iperm;    // per vertex: original id of the stored vertex
    const struct MgkEntry* list_outer;  // per nonzero (CSR order, index zoff + k), see MgkEntry
    const struct MgkEntry* list_inner;  // per lane slot (index loff + slot)
    const int32_t* regs_split;  // per graph MGK_REGS_SPLIT_STRIDE row boundaries, see below
    const float* attr_outer;  // label attribute a of nonzero k (CSR order): attr_outer[a * nnz_total + zoff + k]
    const float* attr_inner;  // the same in lane order: attr_inner[a * lanes_total + loff + slot], 0 on idle slots
    const struct MgkSellDesc* sell_desc;    // per graph, see MgkSellDesc
    const struct MgkSellVertex* sell_vtx;   // records of the owner-computes solver
    const struct MgkSellNbr* sell_nbr;
    int32_t n_graphs, n_tiles_total, nnz_total, lanes_total;
    int32_t label_dim;        // attributes per edge label (1 for plain scalar labels)
    int32_t uniform_start;    // 1: no starting probabilities were given, p_i = 1/n on every graph
};

// One unit of work: solve the pair (outer graph g1 of batch X, inner graph g2
// of batch Y) and write the value to out0 (and to out1 if >= 0).  out1 == -2
// marks a job whose outer graph is the *second* graph of the requested pair
// (the orientation was exchanged); only the nodal output cares.
struct MgkJob {
    int32_t g1, g2;
    int32_t out0, out1;
};
#define MGK_OUT1_NONE (-1)
#define MGK_OUT1_SWAPPED (-2)

// Device pointers the solvers write to.  iters, flags, nodal may be null.
// nodal: solution x of pair k (original vertex numbering of the requested pair,
// row-major n x n') starts at nodal + nodal_off[out0].
struct MgkOutputs {
    float* K;
    int32_t* iters;
    int32_t* flags;
    float* nodal;
    const int64_t* nodal_off;
};

// Edge base kernels (Appendix B).  SE, POLY and CONST take one label per edge;
// KRON_SE and RCONV_SE take label_dim attributes (parts) per edge.
enum { MGK_EK_CONST = 0, MGK_EK_SE = 1, MGK_EK_POLY = 2, MGK_EK_KRON_SE = 3, MGK_EK_RCONV_SE = 4 };
#define MGK_MAX_LABEL_DIM 4
#define MGK_POLY_MAX_COEF 9

struct MgkParams {
    float q;          // stopping probability
    float h;          // vertex kernel off-diagonal value
    float e_scale;    // SE: sqrt(alpha * log2(e)), kappa_e = exp2(-((e-e')*e_scale)^2); POLY: 1 / rho
    float e_shift;    // common shift applied to labels before scaling
    float ke_const;   // constant edge kernel value
    float rtol2;      // rtol^2
    int32_t max_iter; // <= 0: automatic
    int32_t edge_kernel;
    int32_t label_dim;                     // attributes per edge label the kernel reads
    float attr_scale[MGK_MAX_LABEL_DIM];   // KRON_SE: sqrt(alpha_a log2(e)) per attribute; RCONV_SE: [0] for all parts
    float poly_c[MGK_POLY_MAX_COEF];       // POLY: sum_i poly_c[i] r^i on r = |e-e'| / rho < 1, zero-padded
};

#if defined(__HIPCC__)
// Compact polynomial radial basis kernel on the prescaled difference d = (e - e') / rho:
// Horner over all MGK_POLY_MAX_COEF coefficients (the unused high ones are 0), and
// 0 from |d| = 1 on.
__device__ __forceinline__ float mgk_poly_kernel(float d, const float* c) {
    const float r = __builtin_fabsf(d);
    const float rc = __builtin_fminf(r, 1.0f);
    float v = c[MGK_POLY_MAX_COEF - 1];
#pragma unroll
    for (int i = MGK_POLY_MAX_COEF - 2; i >= 0; --i) v = __builtin_fmaf(v, rc, c[i]);
    return r < 1.0f ? v : 0.0f;
}
#endif

// ---- LDS plan of the on-chip solver (one workgroup per pair) ---------------
// All offsets in 4-byte words from the start of dynamic LDS.  Computed the same
// way on the host (to size the launch) and in the kernel.
struct MgkSmallPlan {
    int32_t p, y;            // vectors, padded to waves * 64 * ept words each
    int32_t ent1, ent2;      // expanded nonzeros, 4 words each
    int32_t attr1;           // label attributes of the outer nonzeros, attr_dim arrays of z1pad words
    int32_t rowend;          // bit k set: outer entry k is the last of its row
    int32_t tiles1, tiles2;  // staged octile headers, 4 words each
    int32_t vtx1, vtx2;      // per vertex: d_i, start probability, label
    int32_t red;             // reduction scratch, 64 words
    int32_t total;           // words
    int32_t z1pad;           // outer entries padded (multiple of 4, + 4 spare)
    int32_t share;           // nominal outer entries per wave
    int32_t rowend_words;
};

// attr_dim: attributes per edge label for the kernels over label attributes, else 0
static inline MGK_HD MgkSmallPlan mgk_small_plan(int32_t n1, int32_t n2, int32_t z1,
                                                 int32_t lane_len2, int32_t t1, int32_t t2,
                                                 int32_t waves, int32_t ept, int32_t attr_dim) {
    MgkSmallPlan L;
    const int32_t np = waves * 64 * ept;   // >= n1 * n2: every thread owns ept elements
    (void)n1;
    L.z1pad = ((z1 + 3) & ~3) + 4;
    L.share = (z1 + waves - 1) / waves;
    if (L.share < 1) L.share = 1;
    L.rowend_words = L.z1pad / 32 + 2;
    L.p = 0;
    L.y = np;
    L.ent1 = 2 * np;
    L.attr1 = L.ent1 + 4 * L.z1pad;
    L.ent2 = L.attr1 + attr_dim * L.z1pad;
    L.rowend = L.ent2 + 4 * lane_len2;
    L.tiles1 = L.rowend + ((L.rowend_words + 3) & ~3);
    L.tiles2 = L.tiles1 + 4 * t1;
    L.vtx1 = L.tiles2 + 4 * t2;
    L.vtx2 = L.vtx1 + 3 * n1;
    L.red = L.vtx2 + 3 * n2;
    L.total = L.red + 64;
    return L;
}

// Largest product size N = n n' the on-chip solver takes: 16 waves x 16
// elements per thread.
#define MGK_SMALL_MAX_N (16 * 64 * 16)

#define MGK_LDS_LIMIT_BYTES (160 * 1024)

// ---- register-resident on-chip solver ----------------------------------------
// Four or eight wavefronts per pair.  Each wavefront owns a run of whole outer
// rows of at most SMAX nonzeros and keeps the off-diagonal matrix entries
// A_ij A'_i'j' kappa_e(E_ij, E'_i'j') of (its outer nonzeros) x (all inner lane
// slots) in registers for the whole solve; the inner graph takes `chunks`
// 64-lane chunks and has rows of at most 4 nonzeros.  LDS holds p, y, x and a
// dump area (each padded to the register blocks), the per-vertex data of both graphs and the
// reduction scratch.
#define MGK_REGS_SMAX_W4 24      // longest run of outer nonzeros per wavefront, 4 wavefronts
#define MGK_REGS_SMAX_W8 20      // the same with 8 wavefronts
#define MGK_REGS_MAX_CHUNKS 2
#define MGK_REGS_MAX_EPT 8
#define MGK_REGS_MAX_DEG 4       // inner rows: two shift-and-add steps

struct MgkRegsPlan {
    int32_t p, y, x, dump, vtx1, vtx2, red, total;  // words
};

static inline MGK_HD MgkRegsPlan mgk_regs_plan(int32_t n1, int32_t n2, int32_t waves, int32_t ept) {
    MgkRegsPlan L;
    const int32_t np = waves * 64 * ept;
    L.p = 0;
    L.y = np;
    L.x = 2 * np;
    L.dump = 3 * np;   // same shape as y, 2 np behind it: where lanes that hold no row sum store
    L.vtx1 = 4 * np;
    L.vtx2 = L.vtx1 + 3 * n1;
    L.red = (L.vtx2 + 3 * n2 + 3) & ~3;
    L.total = L.red + 64;
    return L;
}

// ---- owner-computes on-chip solver (graphs of at most 64 vertices, degree <= 4) ----
// Every element (i, i') of the product vectors has one owning lane, which keeps the
// off-diagonal entries of its row of the system -- deg(i) deg(i') of them, about four on
// molecule-like graphs -- in registers together with the LDS address of the element of p
// each one multiplies.  Lanes that work side by side must own rows of equal length, so
// the vertices of a graph are sorted by degree (descending) at load and grouped: groups
// of 4 when the graph is the outer operand, groups of 8 when it is the inner one.  A
// "tile" is (outer group U) x (inner group V): 32 elements = one half of a wavefront,
// all of whose rows have at most maxdeg(U) * maxdeg(V) entries.  Tiles are enumerated by
// (maxdeg(U) descending, maxdeg(V) descending); tile number h is held by lanes
// 32 (h & 1) .. + 31 of a wavefront (mgk_sell_wave_of) in its vector slot (h / 2) / W, lane
// 8 u + v owning (vertex u of U, vertex v of V).  An element's p value lives in LDS at
// a word that is 8 u + v modulo 32, so its bank is 8 (k & 3) + (k' & 7) for sorted positions k, k':
// a gather by the 32 lanes of a tile is free of bank conflicts when the a-th neighbours
// of the 4 outer vertices sit at positions distinct mod 4 and the b-th neighbours of the
// 8 inner vertices at positions distinct mod 8 (the loader orders the vertices inside a
// degree class, and each vertex's neighbour list, toward that).
#define MGK_SELL_MAX_N 64        // vertices per graph
#define MGK_SELL_MAX_DEG 4
#define MGK_SELL_OUTER_GROUP 4
#define MGK_SELL_INNER_GROUP 8

// Per graph: where its records start (8 ceil(n / 8) vertex records, 4 neighbour records
// each) and how many outer / inner groups have each maximum degree 0..4.  ok == 0: the
// graph does not qualify (too many vertices or a vertex of higher degree).
struct MgkSellDesc {
    int32_t voff;
    uint32_t ga03;   // groups of 4 whose maximum degree is 0..3, one byte each
    uint32_t gb03;   // groups of 8 whose maximum degree is 0..3
    uint32_t hi;     // groups of 4 with maximum degree 4 | groups of 8 with maximum degree 4 << 8 | ok << 16
};
static inline MGK_HD int mgk_sell_ga(const MgkSellDesc& d, int deg) {
    return (int)((deg < 4 ? d.ga03 >> (8 * deg) : d.hi) & 0xffu);
}
static inline MGK_HD int mgk_sell_gb(const MgkSellDesc& d, int deg) {
    return (int)((deg < 4 ? d.gb03 >> (8 * deg) : d.hi >> 8) & 0xffu);
}
static inline MGK_HD bool mgk_sell_ok(const MgkSellDesc& d) { return ((d.hi >> 16) & 1u) != 0u; }
// Vertex at sorted position k: row sum of A, starting probability, label, and
// (vertex id in stored order) | degree << 16.  Positions >= n are padding (degree 0, id 0xffff).
struct alignas(16) MgkSellVertex {
    float rowsum, start;
    int32_t label;
    uint32_t id_deg;
};
// a-th neighbour of the vertex at sorted position k (record 4 k + a): the neighbour's
// sorted position, A_ij, E_ij.  a >= degree: weight 0, position k itself.
struct alignas(16) MgkSellNbr {
    uint32_t pos;
    float w, e;
    uint32_t pad;
};

// Tiles 2 s and 2 s + 1 share vector slot s / W of wavefront s % W, counted back and forth
// (W - 1 - s % W in odd rounds): rows get shorter with s, and this way no wavefront takes
// the longest rows of every round.
static inline MGK_HD int mgk_sell_wave_of(int s, int waves) {
    const int m = s / waves, j = s - m * waves;
    return (m & 1) ? waves - 1 - j : j;
}

// LDS plan of the owner-computes solver, in words.
struct MgkSellPlan {
    int32_t p, y, x;          // slot layout, waves * 64 * ept words each
    int32_t vtx1, nbr1, vtx2, nbr2;
    int32_t table, rankof;    // tile number -> (U, V, A, B); U * G2 + V -> byte address of the tile's 32 words of p
    int32_t sched;            // per wavefront and slot: entries | (entries per outer neighbour) << 8
    int32_t misfit;           // per wavefront: 1 when its rows do not fit the launch shape
    int32_t red, total;
};
static inline MGK_HD MgkSellPlan mgk_sell_plan(int32_t n1, int32_t n2, int32_t waves, int32_t ept) {
    MgkSellPlan L;
    const int32_t np = waves * 64 * ept;
    const int32_t r1 = (n1 + 7) & ~7, r2 = (n2 + 7) & ~7;   // staged records per graph
    const int32_t tiles = ((n1 + 3) / 4) * ((n2 + 7) / 8);
    L.p = 0;
    L.y = np;
    L.x = 2 * np;
    L.vtx1 = 3 * np;
    L.nbr1 = L.vtx1 + 4 * r1;
    L.vtx2 = L.nbr1 + 16 * r1;
    L.nbr2 = L.vtx2 + 4 * r2;
    L.table = L.nbr2 + 16 * r2;
    L.rankof = L.table + ((tiles + 3) & ~3);
    L.sched = L.rankof + ((tiles + 3) & ~3);
    L.misfit = L.sched + waves * ept;
    L.red = (L.misfit + waves + 3) & ~3;
    L.total = L.red + 64;
    return L;
}

// Order of the tile classes (A, B) = (largest degree of the outer group, of the inner
// group): classes with entries first, by A descending then B descending, then the classes
// without entries (A or B zero: isolated vertices) in the same order.  True when class
// (a, b) comes before class (A, B).
static inline MGK_HD bool mgk_sell_class_before(int a, int b, int A, int B) {
    const bool z = a * b == 0, Z = A * B == 0;
    if (z != Z) return Z;
    return a > A || (a == A && b > B);
}

// Walk of the tiles of a pair in the order the kernel numbers them, for the host planner
// (does the pair fit a launch shape?): returns the largest number of entry registers any
// wavefront needs with `waves` wavefronts, the number of vector slots per lane in *slots
// and the entries all wavefronts execute together in *executed.
static inline int32_t mgk_sell_need(const MgkSellDesc& o, const MgkSellDesc& i, int32_t waves, int32_t* slots,
                                    int32_t* executed) {
    int32_t per_wave[16] = {0};
    int32_t h = 0, prevA = 0, prevB = 0;
    for (int pass = 0; pass < 2; ++pass)   // classes with entries, then those without
        for (int A = MGK_SELL_MAX_DEG; A >= 0; --A)
            for (int B = MGK_SELL_MAX_DEG; B >= 0; --B) {
                if ((A * B == 0) != (pass == 1)) continue;
                const int32_t cnt = mgk_sell_ga(o, A) * mgk_sell_gb(i, B);
                for (int32_t k = 0; k < cnt; ++k, ++h) {
                    if (h & 1) {
                        const int32_t a = A > prevA ? A : prevA, b = B > prevB ? B : prevB;
                        per_wave[mgk_sell_wave_of(h >> 1, waves)] += a * b;
                    } else {
                        prevA = A;
                        prevB = B;
                    }
                }
            }
    if (h & 1) per_wave[mgk_sell_wave_of(h >> 1, waves)] += prevA * prevB;
    int32_t need = 0, sum = 0;
    for (int w = 0; w < waves; ++w) { need = per_wave[w] > need ? per_wave[w] : need; sum += per_wave[w]; }
    *slots = ((h + 1) / 2 + waves - 1) / waves;
    if (executed) *executed = sum;
    return need;
}

// ---- solver with vectors in global memory (pairs too large for LDS) ---------
// Expanded nonzero lists of a whole batch, rebuilt per call because the label
// scaling depends on the edge-kernel parameters:
//   outer list (CSR order, index zoff + position): {col, scaled label or
//     weight, log2 weight, row}
//   inner list (lane layout, index loff + slot): {row, col | rank in run << 24
//     | row longer than a lane group << 30 | last of run << 31, scaled label or
//     weight, log2 weight (the weight itself for the kernels that multiply by it)}
struct alignas(16) MgkEntry {
    uint32_t x, y, z, w;
};

// Parameter-free nonzero lists written once at load (list_outer / list_inner of
// MgkBatchDev) for the register-resident on-chip solver, which reads a graph's
// nonzeros straight into lanes:
//   list_outer[zoff + k], CSR order: {row, col, label bits, weight bits | bit 31
//     set when k is the last nonzero of its row (weights are > 0)}
//   list_inner[loff + slot], lane layout: {row | rank in run << 20 | row longer
//     than a lane group << 30 | last of run << 31, col, label bits, weight bits
//     (0.0f for an idle slot)}

// Outer rows of a graph divided among the wavefronts of the register-resident solver
// (whole rows, contiguous, the most loaded wavefront as light as possible; written at
// load): regs_split[g * MGK_REGS_SPLIT_STRIDE + k], k = 0..4: wavefront w of 4 owns
// rows [b[w], b[w+1]); k = 5..13: the same for 8 wavefronts.
#define MGK_REGS_SPLIT_STRIDE 14
#define MGK_REGS_SPLIT_W8 5

struct MgkExpanded {
    const MgkEntry* outer;
    const MgkEntry* inner;
};

// Octiles of a batch expanded to dense 8x8 blocks (64 floats per tile each).
struct MgkDenseTiles {
    const float* w;    // A_ij, 0 where absent
    const float* e;    // scaled label, 0 where absent
    const float* lw;   // log2 A_ij, -inf where absent
};

// One pair solved with global-memory vectors.  Vector v of the pair starts at
// vec + v * npad floats: 0 x, 1 r, 2 p, 3 M, 4 y (also holds z).
struct MgkLargePair {
    int32_t g1, g2;        // outer graph (batch X), inner graph (batch Y)
    int32_t n1, n2;
    int64_t vec;           // offset of the pair's vectors in the scratch array (floats)
    int32_t npad;          // n1 * n2 rounded up to 64
    int32_t out0, out1;
    int32_t max_iter;
    int32_t nsteps;        // DPP steps for the inner row sums
    int32_t atomic_rows;   // inner graph has rows longer than a lane group
};

// Scalars of one pair in the global-memory solver.  The three sums of iteration `it` go
// to slot it & 1 of their pair of accumulators; the other slot is cleared meanwhile, by a
// kernel that runs when nobody reads it (no separate scalar kernels, no host round trip):
//   rz[it & 1]        r^T z after the update of iteration it; rz[(it + 1) & 1] is the one
//                     of the iteration before (rho of Alg. 1; the set-up puts it in rz[1])
//   pa[it & 1]        p^T a of iteration it
//   rr[it & 1]        r^T r after the update of iteration it
struct MgkPairState {
    float rz[2], pa[2], rr[2];
    float bb;       // b^T b
    float kval;
    int32_t iters, done, flag;
    int32_t growth; // bits of max_i x_i / (M^{-1} b)_i >= 1: how far the solution exceeds the Jacobi guess
};

// A pair whose solution exceeds M^{-1} b by more than this factor somewhere is checked
// after the solve: one more product gives the true residual b - S x in fp32, and if
// (true relative residual) x (that factor) exceeds MGK_VERIFY_ACCURACY the pair's flag
// becomes 3.  Below the threshold even a residual at fp32 rounding level cannot move the
// value by that much, so nothing is checked.
#define MGK_VERIFY_GROWTH 32.0f
#define MGK_VERIFY_ACCURACY 1e-4f

#define MGK_LARGE_ROWS_PER_BLOCK 8    // outer rows per workgroup of the large XMV
#define MGK_LARGE_CHUNKS_PER_WAVE 2   // 64-lane chunks of the inner layout per wave
#define MGK_LARGE_WAVES 4
#define MGK_ROWS_MAX_BATCH 64         // rows of p (= outer nonzeros) staged at a time by the row-staged XMV

#endif
