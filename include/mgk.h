/* mgk.h - C ABI of the MI355X marginalized-graph-kernel solver.
 *
 * The library evaluates the marginalized graph kernel between labeled graphs
 * (paper Section II-B, Eq. 1)
 *
 *     K(G,G') = p_x^T ( D_x V_x^{-1} - A_x (.) E_x )^{-1} D_x q_x
 *
 * by running the Jacobi-preconditioned conjugate-gradient iteration of
 * Alg. 1 on the tensor-product system of each requested pair, with the
 * off-diagonal product (A (x) A') (.) (E (x)k E') p formed from the two graphs
 * (Alg. 2, Section III) instead of from a stored N x N matrix: regenerated in
 * every iteration, or, for pairs of small graphs, generated once per solve
 * into registers (mgk_set_product_cache).  Graphs are
 * held on the device as coordinate lists of non-empty 8x8 tiles ("octiles",
 * Section III-D) with a 64-bit occupancy bitmap and packed nonzeros per tile
 * (Section IV-A/B), after an optional partition-based vertex reordering
 * (Section IV-A, Eq. 3).
 *
 * Conventions
 *  - Every entry point returns an mgk_status and never throws or aborts across
 *    the ABI.  mgk_last_error() gives a message for the last failure on a ctx.
 *  - "host" pointers are ordinary CPU memory, read before the call returns and
 *    never retained.  "device" pointers are GPU global memory on the ctx's
 *    device (for example a torch tensor's data_ptr()); the caller owns them.
 *  - Kernels are enqueued on the HIP stream passed as `stream` (a hipStream_t
 *    cast to void*, NULL = the null stream).  Results are valid once the caller
 *    has synchronised that stream.
 *  - A ctx is bound to one device and is not thread-safe.  Batches belong to
 *    the ctx that loaded them.
 *  - Calls that include pairs too large for the on-chip solver synchronise the
 *    stream before returning (iterations are enqueued without waiting, as many
 *    as the previous such call needed; then the host reads how many pairs still
 *    iterate, normally once per call)
 *    and allocate device scratch owned by the ctx (5 vectors of n n' floats per
 *    such pair, plus expanded nonzero lists of the batches).  Such pairs are
 *    solved in groups of at most 4096 pairs and 8 GiB of vectors.
 *  - Non-convergence is data, not an error: the pair's flag is set to 1 and the
 *    value of the last iterate is still written.  Flag 2 with a NaN value marks
 *    a pair that a kernel refused because it did not fit the launch shape the
 *    host chose for it (an internal error; it is never solved in part).  Flag 3
 *    (pairs solved with vectors in global memory): the iteration met the stop
 *    test of Alg. 1 on its recursively updated residual, but the solution is
 *    more than 32 times the Jacobi guess M^{-1} b somewhere and the residual
 *    b - S x recomputed with one more product is so large in fp32 that the
 *    value may be off by more than 1e-4 relative (an ill-conditioned pair, for
 *    example a dense graph against itself with all base kernels equal to 1).
 *  - Precision: fp32 on the device.  Product index of (i,i') is i*n'+i'.
 */
#ifndef MGK_H
#define MGK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mgk_ctx mgk_ctx;     /* opaque: parameters, device scratch, error text */
typedef struct mgk_batch mgk_batch; /* opaque: a packed (and reordered) set of graphs  */

typedef enum {
    MGK_OK = 0,
    MGK_EINVAL = 1,  /* bad argument or invalid graph                     */
    MGK_ENOMEM = 2,  /* host or device allocation failed                  */
    MGK_EDEVICE = 3, /* a HIP call failed                                 */
    MGK_ESTATE = 4,  /* object used with the wrong ctx / after free       */
    MGK_ELIMIT = 5   /* a pair is larger than this build can solve        */
} mgk_status;

/* vertex reordering applied when a batch is loaded (Section IV-A) */
enum { MGK_REORDER_NONE = 0, MGK_REORDER_PBR = 1, MGK_REORDER_RCM = 2,
       MGK_REORDER_MORTON = 3 /* only through mgk_load_graphs_embedded */ };
/* tile-pair primitive selection (Section IV-B, "hybrid dense-sparse") */
enum { MGK_TILE_AUTO = 0, MGK_TILE_SPARSE = 1, MGK_TILE_DENSE = 2, MGK_TILE_SPARSE_GATHER = 3 };

/* Create a context on HIP device `device`.  *out is NULL on failure.
 * device = -1 creates a host-only context: graphs can be loaded, reordered,
 * packed and inspected, nothing is copied to a GPU, and the solve calls
 * return MGK_ESTATE. */
mgk_status mgk_create(mgk_ctx** out, int device);
void mgk_destroy(mgk_ctx* ctx);
/* Message of the last failed call on ctx (ctx-owned, valid until the next call). */
const char* mgk_last_error(const mgk_ctx* ctx);

/* ---- base kernels and solver parameters (Section II-B, Alg. 1) -------------
 * Vertex kernel: kappa_v(v,v') = 1 if v == v' else h, 0 < h <= 1.
 * Edge kernel, square exponential (Appendix B): exp(-(e-e')^2 / (2 l^2)), l > 0.
 * Edge kernel, constant: kappa_e == c, 0 <= c <= 1 (c = 1, h = 1 gives Eq. 2).
 * Stopping probability q > 0, the same on every vertex; d_i = sum_j A_ij + q.
 * Solver: stop when r^T r <= rtol^2 b^T b (b = D_x q_x) or after max_iter
 * iterations (max_iter <= 0: 2 N capped at 1000).  Defaults: h = 1, constant
 * edge kernel c = 1, q = 0.05, rtol = 1e-6. */
mgk_status mgk_set_vertex_kernel_delta(mgk_ctx* ctx, float h);
mgk_status mgk_set_edge_kernel_se(mgk_ctx* ctx, float length_scale);
mgk_status mgk_set_edge_kernel_const(mgk_ctx* ctx, float c);
/* More edge base kernels (the examples of Appendix B).  Values must stay in
 * [0, 1] and the kernel positive definite for Eq. 1 to be SPD (Section II-B).
 *
 * poly: compact polynomial radial basis kernel on scalar labels,
 *   kappa_e(e, e') = sum_{i < n_coef} coef[i] r^i  for r = |e - e'| / rho < 1,
 *   and 0 for r >= 1 (compact support of radius rho > 0).  n_coef in 1..9
 *   (coef is copied).  Rejected with MGK_EINVAL if the polynomial leaves
 *   [0, 1] anywhere on 0 <= r <= 1 (checked on a grid of 4097 points).
 *   Example: Wendland's (1-r)^4 (4r+1) = {1, 0, -10, 20, -15, 4}.
 * kron_se: Kronecker-product kernel over labels with `dim` real attributes,
 *   kappa_e = prod_a exp(-(e_a - e'_a)^2 / (2 length_scale[a]^2)), dim in 1..4.
 * rconv_se: R-convolution kernel over labels made of `dim` parts,
 *   kappa_e = (1 / dim^2) sum_a sum_b exp(-(e_a - e'_b)^2 / (2 length_scale^2));
 *   the factor 1 / dim^2 keeps the range inside [0, 1].  dim in 1..4.
 * The last two need batches loaded with the same number of attributes per
 * edge (mgk_load_graphs_attr); a solve with another batch fails with
 * MGK_ESTATE.  All three run in both on-chip solvers and in the sparse
 * product of the global-memory solver; the dense tile-pair product is built
 * for poly only (pairs of well-filled graphs take the sparse product with the
 * other two). */
mgk_status mgk_set_edge_kernel_poly(mgk_ctx* ctx, int32_t n_coef, const float* coef, float rho);
mgk_status mgk_set_edge_kernel_kron_se(mgk_ctx* ctx, int32_t dim, const float* length_scale);
mgk_status mgk_set_edge_kernel_rconv_se(mgk_ctx* ctx, int32_t dim, float length_scale);
mgk_status mgk_set_stop_prob(mgk_ctx* ctx, float q);
mgk_status mgk_set_solver(mgk_ctx* ctx, float rtol, int32_t max_iter);
/* Tile-pair primitive of the global-memory solver: sparse (only the nnz * nnz'
 * products of the nonzeros), dense (all 4096 products of every pair of
 * non-empty octiles, no gathers), or automatic per graph pair from the mean
 * fill of the two graphs' octiles.  The sparse product stages the rows of p
 * that a row of the outer graph needs in LDS whenever a row of p (4 n' bytes)
 * fits in 120 KB; MGK_TILE_SPARSE_GATHER forces the variant that gathers p from
 * global memory instead (always used for larger n').  The on-chip solvers always use the sparse product. */
mgk_status mgk_set_tile_path(mgk_ctx* ctx, int32_t mode);
/* Tuning knobs, safe to leave alone.  waves_per_pair: wavefronts of the
 * workgroup that solves one on-chip pair (1, 2, 4, 8 or 16; 0 = automatic by
 * product size).  A pair too large for the requested size gets the next
 * larger one that fits. */
mgk_status mgk_set_launch(mgk_ctx* ctx, int32_t waves_per_pair);
/* Pairs with n n' <= max_product are solved on chip (one workgroup per pair,
 * vectors in LDS and registers); larger pairs keep their vectors in global
 * memory and run one kernel per step of Alg. 1.  Default and upper bound:
 * 16384.  0 sends every pair to the global-memory solver. */
mgk_status mgk_set_onchip_limit(mgk_ctx* ctx, int32_t max_product);
/* On-chip solver, where the off-diagonal entries A_ij A'_i'j' kappa_e(E_ij,
 * E'_i'j') come from in each iteration.  0: regenerated from the two graphs in
 * every product, as Alg. 2 does.  1 (default): for a pair small enough that its
 * nnz * nnz' entries fit in the vector registers of one workgroup they are
 * generated once per solve and kept there (they are never written to memory);
 * other pairs are handled as with 0.  3: as 1, but pairs of graphs with at most
 * 64 vertices of degree at most 4 (edge kernels on scalar labels) go to a second
 * entry-keeping kernel in which every lane owns whole rows of the system; it is
 * slower on the benchmark workloads and kept for comparison (2 is accepted and
 * means 1).  All give the same iterates up to the rounding of the entries.
 * Ignored while mgk_set_launch forces a workgroup size. */
mgk_status mgk_set_product_cache(mgk_ctx* ctx, int32_t enable);
/* Order of the on-chip jobs inside a launch (Section V-B, dynamic scheduling).
 * 1 (default): most expensive pairs first, so that the hardware dispatcher,
 * which hands workgroups to compute units as they free up, ends the launch with
 * the cheapest pairs.  0: in the order the pairs were given.  The values do not
 * depend on it. */
mgk_status mgk_set_schedule(mgk_ctx* ctx, int32_t cost_sorted);

/* ---- graphs -----------------------------------------------------------------
 * Load n_graphs graphs given in flat host arrays (all caller-owned, copied):
 *   vtx_off[n_graphs+1]   prefix offsets into the per-vertex arrays
 *   vtx_label[sum n]      integer vertex labels
 *   start_prob[sum n]     starting probabilities p, or NULL for 1/n
 *   edge_off[n_graphs+1]  prefix offsets into the per-edge arrays
 *   src, dst              endpoints, ids local to the graph; each undirected
 *                         edge listed once in either orientation
 *   weight                A_ij > 0, or NULL for 1
 *   edge_label            E_ij, or NULL for 0 (unlabeled)
 * Rejected with MGK_EINVAL: empty graph, endpoint out of range, self loop,
 * duplicate edge, weight that is not finite and positive, non-finite label
 * or probability.  The graphs are reordered (`reorder`), cut into octiles,
 * empty octiles dropped, and copied to the device. */
mgk_status mgk_load_graphs(mgk_ctx* ctx, int32_t n_graphs,
                           const int64_t* vtx_off, const int32_t* vtx_label,
                           const float* start_prob,
                           const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                           const float* weight, const float* edge_label,
                           int32_t reorder, mgk_batch** out);
/* The same with label_dim (1..4) attributes per edge label:
 * edge_label[(sum m) * label_dim], the attributes of an edge adjacent.
 * mgk_load_graphs is label_dim = 1.  The octiles (mgk_batch_get_tiles) hold
 * attribute 0. */
mgk_status mgk_load_graphs_attr(mgk_ctx* ctx, int32_t n_graphs,
                                const int64_t* vtx_off, const int32_t* vtx_label,
                                const float* start_prob,
                                const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                                const float* weight, int32_t label_dim, const float* edge_label,
                                int32_t reorder, mgk_batch** out);
/* Graphs whose vertices come with coordinates (coords[(sum n) * coord_dim], coord_dim
 * 1..3, finite): as mgk_load_graphs, with the vertices of every graph numbered along the
 * Morton (Z-order) curve through the graph's bounding box, the space-filling-curve
 * ordering of Section IV-A (10 bits per coordinate in 2 and 3 dimensions). */
mgk_status mgk_load_graphs_embedded(mgk_ctx* ctx, int32_t n_graphs,
                                    const int64_t* vtx_off, const int32_t* vtx_label,
                                    const float* start_prob,
                                    const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                                    const float* weight, const float* edge_label,
                                    int32_t coord_dim, const float* coords, mgk_batch** out);
void mgk_free_batch(mgk_ctx* ctx, mgk_batch* batch);

/* Totals over the batch (any pointer may be NULL): graphs, vertices, stored
 * nonzeros (2 per edge), non-empty octiles, and non-empty off-diagonal
 * octiles (twice the objective of Eq. 3 for the ordering in use). */
mgk_status mgk_batch_stats(const mgk_batch* batch, int64_t* n_graphs, int64_t* n_vertices,
                           int64_t* nnz, int64_t* n_tiles, int64_t* n_offdiag_tiles);
/* perm[vtx_off[g] + old_id] = new (stored) id of that vertex in graph g. */
mgk_status mgk_batch_permutation(const mgk_batch* batch, int32_t* perm_host);
/* Host copy of graph g's packed form, for inspection and tests.  tile_row,
 * tile_col, bitmap: [*n_tiles]; w, e: [*nnz] packed tile by tile in bit order
 * (bit 8*r+c of the bitmap <-> row 8*tile_row+r, column 8*tile_col+c).
 * Pass NULL arrays to query the counts only. */
mgk_status mgk_batch_get_tiles(const mgk_batch* batch, int32_t g, int32_t* n_tiles, int32_t* nnz,
                               int32_t* tile_row, int32_t* tile_col, uint64_t* bitmap,
                               float* w, float* e);

/* ---- kernel values ----------------------------------------------------------
 * mgk_gram: all pairs of one batch.  K_dev[G*G] row-major, both triangles
 * written (K[i][j] == K[j][i] bit for bit: each unordered pair is solved
 * once).  iters_dev / flag_dev: optional [G*G] int32 arrays receiving the
 * number of PCG iterations and 0 (converged) / 1 (stopped at max_iter).
 * The job list of the batch is built on the first call and kept. */
mgk_status mgk_gram(mgk_ctx* ctx, mgk_batch* batch, float* K_dev,
                    int32_t* iters_dev, int32_t* flag_dev, void* stream);

/* mgk_pairs: K_dev[k] = K(X[i_host[k]], Y[j_host[k]]), k < n_pairs.  Y may be
 * the same batch as X.  i_host / j_host are host arrays.  Outputs as above,
 * length n_pairs. */
mgk_status mgk_pairs(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                     const int32_t* i_host, const int32_t* j_host, float* K_dev,
                     int32_t* iters_dev, int32_t* flag_dev, void* stream);

/* mgk_pairs_dev: mgk_pairs with the index arrays in device memory (int32, on the
 * ctx's device, written before work enqueued on `stream` so far completes).  The
 * launch shape of a pair is chosen on the host from the sizes of its two graphs
 * (Section V-B), so the indices are copied to the host first: the call
 * synchronises `stream` once before it enqueues the solve. */
mgk_status mgk_pairs_dev(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                         const int32_t* i_dev, const int32_t* j_dev, float* K_dev,
                         int32_t* iters_dev, int32_t* flag_dev, void* stream);

/* mgk_pairs_noalloc: mgk_pairs for callers that cannot allocate device memory (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same
 * arguments, same kernels and bit-identical values, but the call makes no hipMalloc /
 * hipFree (nor any other allocating HIP or library call): the job list its kernels read
 * lives in a fixed 1 MiB array in device memory that every GPU the library runs on holds
 * until the process ends.  Limits: at most 65536 pairs per call, and every pair must be
 * solvable on chip (n n' <= the on-chip limit); otherwise MGK_ELIMIT and nothing is
 * enqueued.  All calls on a GPU share that one array, which keeps the jobs of the last
 * call: calls that overlap in time on the same GPU (other streams, other contexts,
 * other threads) race on it; within one context a call first waits for the previous
 * mgk_pairs_noalloc call's stream.  The index arrays are copied to the device from the
 * caller's host memory and the stream is synchronised once before the kernels start,
 * as in mgk_pairs. */
mgk_status mgk_pairs_noalloc(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                             const int32_t* i_host, const int32_t* j_host, float* K_dev,
                             int32_t* iters_dev, int32_t* flag_dev, void* stream);

/* mgk_pairs_nodal: as mgk_pairs, and also the node-wise similarity (Section I):
 * the solution x = V_x r_inf of Eq. 1 itself.  For pair k the n x n' values, in
 * the caller's original vertex numbering, row-major (vertex i of the X graph,
 * vertex i' of the Y graph at i*n'+i'), are written at x_dev + x_off_host[k]
 * (x_off_host: host array of n_pairs offsets in floats; the regions must not
 * overlap).  K_dev[k] = sum_ii' p_i p'_i' x_ii'. */
mgk_status mgk_pairs_nodal(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                           const int32_t* i_host, const int32_t* j_host, float* K_dev, float* x_dev,
                           const int64_t* x_off_host, int32_t* iters_dev, int32_t* flag_dev,
                           void* stream);

/* Which kernels the last mgk_gram / mgk_pairs* call on ctx enqueued (for measurement
 * reports): one text line per launch shape, "<kernel and template arguments> pairs=<n>
 * entries_cached=<0|1>" (entries_cached: the off-diagonal entries are kept in registers
 * instead of being regenerated in every product of Alg. 2).  Copies at most capacity - 1
 * characters and a terminating 0 into buf (host memory, may be NULL) and returns the size
 * needed including the 0, or -1 for a null ctx. */
int64_t mgk_launch_log(const mgk_ctx* ctx, char* buf, int64_t capacity);

/* Normalised Gram matrix (Section "Related Work"): K[i][j] /= sqrt(K[i][i] K[j][j])
 * in place on the n x n row-major device matrix K_dev. */
mgk_status mgk_normalize_gram(mgk_ctx* ctx, int32_t n, float* K_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MGK_H */
