// Solver for pairs whose vectors do not fit on chip: x, r, p, M, y live in
// global memory and each step of Alg. 1 is a kernel over all such pairs of a
// call.  The XMV (Alg. 2) uses the same lane scheme as the on-chip solver:
// inner nonzeros one per lane with rows in adjacent lanes, outer nonzeros
// streamed as wave-uniform operands, one kappa_e evaluation and one gathered
// p_jj' per nonzero pair, DPP row sums at the end of every outer row, a single
// writer per y_ii'.  Here the entry lists come from global memory (expanded
// once per call by mgk_expand_kernel) and p is gathered from global memory.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mgk_internal.h"
#include "mgk_launch.h"

namespace {

constexpr int kWaves = MGK_LARGE_WAVES;
constexpr int kThreads = kWaves * 64;

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
    return v + __int_as_float(moved);
}

__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_add<0xB1>(v);
    v = dpp_add<0x4E>(v);
    v = dpp_add<0x141>(v);
    v = dpp_add<0x140>(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (r0 + r1) + (r2 + r3);
}

// sum over the workgroup, then one atomic per workgroup into *dst
__device__ __forceinline__ void block_accumulate(float v, float* dst, float* red) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += red[w];
        atomicAdd(dst, s);
    }
    __syncthreads();
}

template <int DIST>
__device__ __forceinline__ float row_shr(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x110 + DIST, 0xf, 0xf, true));
}

// ---- expansion of the octiles of a whole batch --------------------------------
// idle lane slots of the inner lists: weight 0 (`aux` = its log2, -inf, or the weight
// itself for the kernels that multiply by it), never the end of a run
__global__ void mgk_fill_idle_kernel(uint4* inner, int n, uint32_t aux) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n) inner[k] = make_uint4(0u, 0u, 0u, aux);
}

// one wave per octile, lane <-> bit of the bitmap
template <int EK>
__global__ __launch_bounds__(256) void mgk_expand_kernel(MgkBatchDev B, MgkParams prm, uint4* outer,
                                                         uint4* inner) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= B.n_tiles_total) return;
    const MgkGraphDesc g = B.graphs[B.tile_graph[t]];
    const MgkTile tile = B.tiles[t];
    const int r = lane >> 3, c = lane & 7;
    int prior = 0;  // nonzeros of this row in earlier tiles of the same tile row
    for (int tp = t - 1; tp >= g.toff && B.tiles[tp].tr == tile.tr; --tp)
        prior += __popc((uint32_t)(B.tiles[tp].bitmap >> (8 * r)) & 0xffu);
    if (!((tile.bitmap >> lane) & 1ull)) return;
    const int row = (int)tile.tr * 8 + r, col = (int)tile.tc * 8 + c;
    const int k = g.zoff + (int)tile.nzoff + __popcll(tile.bitmap & ((1ull << lane) - 1ull));
    const float w = B.w[k];
    const float el = (B.e[k] - prm.e_shift) * prm.e_scale;
    const int rp0 = B.rowptr[g.voff + row];
    const int rp1 = (row + 1 < g.n) ? B.rowptr[g.voff + row + 1] : g.nnz;
    const uint32_t rowbyte = (uint32_t)(tile.bitmap >> (8 * r)) & 0xffu;
    const int rank = prior + __popc(rowbyte & ((1u << c) - 1u));
    // fourth word: log2 weight where the weight is folded into an exponent, else the weight
    const float lw = (EK == MGK_EK_POLY || EK == MGK_EK_RCONV_SE) ? w : __log2f(w);
    const float lab = EK == MGK_EK_CONST ? w : el;
    outer[g.zoff + rp0 + rank] = make_uint4((uint32_t)col, __float_as_uint(lab), __float_as_uint(lw), (uint32_t)row);
    const int first = B.lanepos[g.voff + row];
    const MgkRunPos rp = mgk_run_pos(first, rank, rp1 - rp0);
    inner[g.loff + first + rank] =
        make_uint4((uint32_t)row, (uint32_t)col | (rp.rank << 24) | (rp.cut << 30) | (rp.last << 31), __float_as_uint(lab),
                   __float_as_uint(lw));
}

// ---- Alg. 1 set-up -------------------------------------------------------------
__global__ __launch_bounds__(256) void mgk_large_init_kernel(MgkBatchDev X, MgkBatchDev Y,
                                                             const MgkLargePair* pairs,
                                                             MgkPairState* state, float* vec,
                                                             MgkParams prm) {
    __shared__ float red[8];
    const MgkLargePair P = pairs[blockIdx.y];
    const int N = P.n1 * P.n2;
    const MgkGraphDesc g1 = X.graphs[P.g1], g2 = Y.graphs[P.g2];
    float* x = vec + P.vec;
    float* r = x + P.npad;
    float* p = r + P.npad;
    float* M = p + P.npad;
    float* y = M + P.npad;
    const float qq = prm.q * prm.q;
    float s_rz = 0.f, s_bb = 0.f;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < P.npad; idx += gridDim.x * blockDim.x) {
        float b = 0.f, z0 = 0.f, m = 1.f;
        if (idx < N) {
            const int i = idx / P.n2, ip = idx - i * P.n2;
            const float d1 = X.rowsum[g1.voff + i] + prm.q, d2 = Y.rowsum[g2.voff + ip] + prm.q;
            const float kv = (X.vlabel[g1.voff + i] == Y.vlabel[g2.voff + ip]) ? 1.f : prm.h;
            const float dd = d1 * d2;
            m = dd / kv;
            b = dd * qq;
            z0 = kv * qq;
        }
        x[idx] = 0.f; r[idx] = b; p[idx] = z0; M[idx] = m; y[idx] = 0.f;
        s_rz = __builtin_fmaf(b, z0, s_rz);
        s_bb = __builtin_fmaf(b, b, s_bb);
    }
    block_accumulate(s_rz, &state[blockIdx.y].rz[1], red);   // rho of iteration 0
    block_accumulate(s_bb, &state[blockIdx.y].bb, red);
}

// ---- XMV ---------------------------------------------------------------------------
// grid.y = pair; grid.x enumerates (outer row block, group of inner chunks).
template <bool WEIGHTED, int EK>
__global__ __launch_bounds__(kThreads) void mgk_large_xmv_kernel(
    MgkBatchDev X, MgkBatchDev Y, MgkExpanded EX, MgkExpanded EY, const MgkLargePair* pairs,
    const MgkPairState* state, float* vec, MgkParams prm) {
    if (state[blockIdx.y].done) return;
    const float ke_c = prm.ke_const;
    constexpr bool ATTR = EK == MGK_EK_KRON_SE || EK == MGK_EK_RCONV_SE;   // labels with D attributes
    const int D = prm.label_dim;
    const MgkLargePair P = pairs[blockIdx.y];
    const MgkGraphDesc g1 = X.graphs[P.g1], g2 = Y.graphs[P.g2];
    const int chunks = g2.lane_len / 64;
    constexpr int CPB = kWaves * MGK_LARGE_CHUNKS_PER_WAVE;   // chunks per workgroup
    const int chunk_groups = (chunks + CPB - 1) / CPB;
    const int row_blocks = (P.n1 + MGK_LARGE_ROWS_PER_BLOCK - 1) / MGK_LARGE_ROWS_PER_BLOCK;
    if ((int)blockIdx.x >= row_blocks * chunk_groups) return;
    const int rb = blockIdx.x / chunk_groups, cg = blockIdx.x - rb * chunk_groups;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row0 = rb * MGK_LARGE_ROWS_PER_BLOCK;
    const int row1 = min(row0 + MGK_LARGE_ROWS_PER_BLOCK, P.n1);
    const float* p = vec + P.vec + 2 * (int64_t)P.npad;
    float* y = vec + P.vec + 4 * (int64_t)P.npad;
    const uint4* outer = reinterpret_cast<const uint4*>(EX.outer) + g1.zoff;
    const uint4* inner = reinterpret_cast<const uint4*>(EY.inner) + g2.loff;
    const int32_t* rowptr1 = X.rowptr + g1.voff;
    const int n2 = P.n2;

    for (int cc = 0; cc < MGK_LARGE_CHUNKS_PER_WAVE; ++cc) {
        const int c = (cg * kWaves + wave) * MGK_LARGE_CHUNKS_PER_WAVE + cc;
        if (c >= chunks) break;
        const uint4 e2 = inner[c * 64 + lane];
        const int ip = (int)e2.x, jp = (int)(e2.y & 0xffffffu);
        const uint32_t rank = (e2.y >> 24) & 0xfu;
        const bool last = (e2.y >> 31) != 0u;
        const float el2 = __uint_as_float(e2.z);
        const float lw2 = __uint_as_float(e2.w);
        const float m1 = rank >= 1 ? 1.f : 0.f, m2 = rank >= 2 ? 1.f : 0.f;
        const float m4 = rank >= 4 ? 1.f : 0.f, m8 = rank >= 8 ? 1.f : 0.f;
        float e2a[MGK_MAX_LABEL_DIM] = {0.f, 0.f, 0.f, 0.f};   // this lane's attributes, prescaled
        if (ATTR) {
#pragma unroll
            for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                if (a < D)
                    e2a[a] = Y.attr_inner[(int64_t)a * Y.lanes_total + g2.loff + c * 64 + lane] * prm.attr_scale[a];
        }
        const float* ao = X.attr_outer + g1.zoff;   // outer attributes, raw: plane a at a * nnz_total
        const float w2s = lw2 / (float)(D * D);     // R-convolution: A'_i'j' / D^2 (0 on idle lanes)
        for (int i = row0; i < row1; ++i) {
            const int kb = rowptr1[i];
            const int ke = (i + 1 < P.n1) ? rowptr1[i + 1] : g1.nnz;
            if (kb == ke) continue;
            float acc = 0.f;
            for (int k = kb; k < ke; ++k) {
                const uint4 e1 = outer[k];   // wave-uniform
                const float pv = p[(int64_t)e1.x * n2 + jp];
                if (EK == MGK_EK_SE) {
                    const float d = el2 - __uint_as_float(e1.y);
                    float t;
                    if (WEIGHTED) t = __builtin_fmaf(-d, d, lw2 + __uint_as_float(e1.z));
                    else t = __builtin_fmaf(-d, d, lw2);
                    acc = __builtin_fmaf(__builtin_amdgcn_exp2f(t), pv, acc);
                } else if (EK == MGK_EK_POLY) {
                    float cu = mgk_poly_kernel(el2 - __uint_as_float(e1.y), prm.poly_c);
                    if (WEIGHTED) cu *= __uint_as_float(e1.z);
                    acc = __builtin_fmaf(cu, pv, acc);
                } else if (EK == MGK_EK_KRON_SE) {
                    // exp2(log2 A + log2 A' - sum_a (s_a (e_a - e'_a))^2); k is wave-uniform
                    float t = WEIGHTED ? lw2 + __uint_as_float(e1.z) : lw2;
#pragma unroll
                    for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                        if (a < D) {
                            const float d = __builtin_fmaf(ao[(int64_t)a * X.nnz_total + k], -prm.attr_scale[a], e2a[a]);
                            t = __builtin_fmaf(-d, d, t);
                        }
                    acc = __builtin_fmaf(__builtin_amdgcn_exp2f(t), pv, acc);
                } else if (EK == MGK_EK_RCONV_SE) {
                    float sum = 0.f;
#pragma unroll
                    for (int b = 0; b < MGK_MAX_LABEL_DIM; ++b)
                        if (b < D) {
                            const float e1b = ao[(int64_t)b * X.nnz_total + k] * prm.attr_scale[0];
#pragma unroll
                            for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                                if (a < D) {
                                    const float d = e2a[a] - e1b;
                                    sum += __builtin_amdgcn_exp2f(-d * d);
                                }
                        }
                    if (WEIGHTED) sum *= __uint_as_float(e1.z);
                    acc = __builtin_fmaf(sum, pv, acc);
                } else {
                    acc = __builtin_fmaf(WEIGHTED ? __uint_as_float(e1.y) : 1.f, pv, acc);
                }
            }
            if (EK == MGK_EK_CONST) acc *= ke_c * el2;
            if (EK == MGK_EK_POLY) acc *= lw2;          // A'_i'j' (0 on idle lanes)
            if (EK == MGK_EK_RCONV_SE) acc *= w2s;
            if (P.nsteps > 0) acc = __builtin_fmaf(m1, row_shr<1>(acc), acc);
            if (P.nsteps > 1) acc = __builtin_fmaf(m2, row_shr<2>(acc), acc);
            if (P.nsteps > 2) acc = __builtin_fmaf(m4, row_shr<4>(acc), acc);
            if (P.nsteps > 3) acc = __builtin_fmaf(m8, row_shr<8>(acc), acc);
            if (last) {
                float* dst = y + ((int64_t)i * n2 + ip);
                // pairs with long inner rows add everywhere (y is cleared after every product):
                // measured faster than atomics on the long-row lanes and plain stores on the rest
                if (P.atomic_rows) atomicAdd(dst, acc);
                else *dst = acc;
            }
        }
    }
}

// ---- XMV with the needed rows of p staged in LDS -------------------------------------------
// One workgroup per outer row i (grid.y = pair).  The rows p_j. of the neighbours j of i are
// copied to LDS with coalesced loads, as many at a time as fit (`lds_floats` / n'), and every
// (outer nonzero, inner nonzero) product then gathers p_jj' from LDS instead of from global
// memory: a row is read from memory once and gathered from z' times (z' nonzeros of the
// inner graph), so the 64-lane gathers no longer go through the L2.  Lane scheme, base kernel
// evaluation and row sums as in mgk_large_xmv_kernel; the waves of the workgroup take the
// 64-lane chunks of the inner graph in turn.  For the edge kernels over label attributes
// the batch's outer attributes are staged (prescaled) next to the outer entries.
// This lane's inner entries of chunks c0 .. c0 + CB - 1 (idle entries past `chunks`).
template <int CB>
__device__ __forceinline__ void rows_load(uint4 (&e2v)[CB], const uint4* inner, int c0, int chunks, int lane) {
#pragma unroll
    for (int b = 0; b < CB; ++b)
        e2v[b] = c0 + b < chunks ? inner[(c0 + b) * 64 + lane] : make_uint4(0u, 0u, 0u, 0u);
}

// All passes of one wave over a staged batch, CB chunks each; the inner entries of the
// next pass are in flight during the products of this one.
template <int CB, bool WEIGHTED, int EK, typename PASS>
__device__ __forceinline__ void rows_sweep(const uint4* inner, int wave, int nwaves, int chunks, int lane,
                                           const PASS& pass) {
    uint4 nxt[CB];
    rows_load<CB>(nxt, inner, wave * CB, chunks, lane);
    for (int c0 = wave * CB; c0 < chunks; c0 += nwaves * CB) {
        uint4 cur[CB];
#pragma unroll
        for (int b = 0; b < CB; ++b) cur[b] = nxt[b];
        if (c0 + nwaves * CB < chunks) rows_load<CB>(nxt, inner, c0 + nwaves * CB, chunks, lane);
        pass(cur, c0);
    }
}

// The products of one pass: this wave's CB chunks of the inner lane layout (chunk c0 + b,
// idle past `chunks`) against the nb outer entries of the staged batch.  The weight A_ij
// of an outer entry is already in its staged row of p.  The labels of the batch sit in
// LDS as a plain array padded to a multiple of four with entries whose kernel value is
// exactly 0, and are read four at a time: one 16-byte
// broadcast read serves 4 * CB products, where a read of a whole 16-byte entry per product
// occupied the LDS twice as long as the gather of p it accompanied.
template <int CB, bool WEIGHTED, int EK>
__device__ __forceinline__ void rows_pass(const MgkBatchDev& Y, const MgkGraphDesc& g2,
                                          const MgkLargePair& P, const MgkParams& prm,
                                          const uint4 (&e2v)[CB], int c0, int chunks, int lane,
                                          const float* prow, const float* olab,
                                          const float* oattr, int nb, int n2, float* yrow,
                                          bool first_batch) {
    constexpr bool ATTR = EK == MGK_EK_KRON_SE || EK == MGK_EK_RCONV_SE;
    const int D = prm.label_dim;
    int ip[CB];
    uint32_t rank[CB];
    bool last[CB];
    float el2[CB], lw2[CB], acc[CB];
    const char* pb[CB];
    float e2a[CB][MGK_MAX_LABEL_DIM];   // this lane's attributes, prescaled
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        const bool on = c0 + b < chunks;
        const uint4 e2 = e2v[b];
        ip[b] = (int)e2.x;
        pb[b] = reinterpret_cast<const char*>(prow) + (e2.y & 0xffffffu) * 4u;
        rank[b] = (e2.y >> 24) & 0xfu;
        last[b] = (e2.y >> 31) != 0u;
        el2[b] = __uint_as_float(e2.z);
        lw2[b] = __uint_as_float(e2.w);
        acc[b] = 0.f;
#pragma unroll
        for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a) {
            e2a[b][a] = 0.f;
            if (ATTR && on && a < D)
                e2a[b][a] = Y.attr_inner[(int64_t)a * Y.lanes_total + g2.loff + (c0 + b) * 64 + lane] *
                            prm.attr_scale[EK == MGK_EK_RCONV_SE ? 0 : a];
        }
    }
    const uint32_t n2x4 = (uint32_t)n2 * 4u;
    for (int r0 = 0; r0 < nb; r0 += 4) {
        const float4 l4 = *reinterpret_cast<const float4*>(olab + r0);   // wave-uniform broadcast
        const float lab[4] = {l4.x, l4.y, l4.z, l4.w};
        float pv[4][CB];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t off = (uint32_t)min(r0 + u, nb - 1) * n2x4;   // past the batch: its last row
#pragma unroll
            for (int b = 0; b < CB; ++b) pv[u][b] = *reinterpret_cast<const float*>(pb[b] + off);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + u;   // < the padded batch length
#pragma unroll
            for (int b = 0; b < CB; ++b) {
                float cu;
                if (EK == MGK_EK_SE) {
                    const float d = el2[b] - lab[u];
                    cu = __builtin_amdgcn_exp2f(__builtin_fmaf(-d, d, lw2[b]));
                } else if (EK == MGK_EK_POLY) {
                    cu = mgk_poly_kernel(el2[b] - lab[u], prm.poly_c);
                } else if (EK == MGK_EK_KRON_SE) {
                    float t = lw2[b];
#pragma unroll
                    for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                        if (a < D) {
                            const float d = e2a[b][a] - oattr[a * MGK_ROWS_MAX_BATCH + r];
                            t = __builtin_fmaf(-d, d, t);
                        }
                    cu = __builtin_amdgcn_exp2f(t);
                } else if (EK == MGK_EK_RCONV_SE) {
                    cu = 0.f;
#pragma unroll
                    for (int q = 0; q < MGK_MAX_LABEL_DIM; ++q)
                        if (q < D) {
                            const float e1b = oattr[q * MGK_ROWS_MAX_BATCH + r];
#pragma unroll
                            for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                                if (a < D) {
                                    const float d = e2a[b][a] - e1b;
                                    cu += __builtin_amdgcn_exp2f(-d * d);
                                }
                        }
                } else {
                    cu = lab[u];   // 1, 0 past the batch
                }
                acc[b] = __builtin_fmaf(cu, pv[u][b], acc[b]);
            }
        }
    }
    const float w2div = 1.0f / (float)(D * D);
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        float v = acc[b];
        if (EK == MGK_EK_CONST) v *= prm.ke_const * el2[b];
        if (EK == MGK_EK_POLY) v *= lw2[b];
        if (EK == MGK_EK_RCONV_SE) v *= lw2[b] * w2div;   // A'_i'j' / D^2 (0 on idle lanes)
        if (P.nsteps > 0) v = __builtin_fmaf(rank[b] >= 1 ? 1.f : 0.f, row_shr<1>(v), v);
        if (P.nsteps > 1) v = __builtin_fmaf(rank[b] >= 2 ? 1.f : 0.f, row_shr<2>(v), v);
        if (P.nsteps > 2) v = __builtin_fmaf(rank[b] >= 4 ? 1.f : 0.f, row_shr<4>(v), v);
        if (P.nsteps > 3) v = __builtin_fmaf(rank[b] >= 8 ? 1.f : 0.f, row_shr<8>(v), v);
        if (last[b]) {
            float* dst = yrow + ip[b];
            // pairs with long inner rows add everywhere (y is cleared after every product)
            if (P.atomic_rows) atomicAdd(dst, v);
            else if (first_batch) *dst = v;
            else *dst += v;                   // same lane, later batch of this row
        }
    }
}

// CB: chunks of the inner layout per pass.  A kernel parameter, not a run-time choice: the
// register count of a kernel is that of its widest path, and the workloads with short rows
// of p (several workgroups per CU) need the small one.
template <bool WEIGHTED, int EK, int CB>
__global__ __launch_bounds__(1024) void mgk_large_xmv_rows_kernel(
    MgkBatchDev X, MgkBatchDev Y, MgkExpanded EX, MgkExpanded EY, const MgkLargePair* pairs,
    const MgkPairState* state, float* vec, MgkParams prm, int lds_floats) {
    extern __shared__ __align__(16) float prow[];
    constexpr bool ATTR = EK == MGK_EK_KRON_SE || EK == MGK_EK_RCONV_SE;   // labels with D attributes
    if (state[blockIdx.y].done) return;
    const int D = prm.label_dim;
    const MgkLargePair P = pairs[blockIdx.y];
    const int i = blockIdx.x;
    if (i >= P.n1) return;
    const MgkGraphDesc g1 = X.graphs[P.g1], g2 = Y.graphs[P.g2];
    const int32_t* rowptr1 = X.rowptr + g1.voff;
    const int kb = rowptr1[i];
    const int ke = (i + 1 < P.n1) ? rowptr1[i + 1] : g1.nnz;
    if (kb == ke) return;   // whole workgroup: y_i. stays 0
    const int n2 = P.n2;
    const int chunks = g2.lane_len / 64;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    // the host sizes LDS for at least one row of p, plus MGK_ROWS_MAX_BATCH outer entries
    const int bmax = min(max(lds_floats / n2, 1), MGK_ROWS_MAX_BATCH);
    // labels of the batch's outer entries (1 for the constant kernel), their weights A_ij,
    // the rows j of p they multiply, then their label attributes, prescaled:
    // oattr[a * MGK_ROWS_MAX_BATCH + r]
    float* olab = prow + ((lds_floats + 3) & ~3);   // read four at a time: 16-byte aligned
    float* ow = olab + MGK_ROWS_MAX_BATCH;
    int* oj = reinterpret_cast<int*>(olab + 2 * MGK_ROWS_MAX_BATCH);
    float* oattr = olab + MGK_ROWS_MAX_BATCH * 4;
    const float* p = vec + P.vec + 2 * (int64_t)P.npad;
    float* y = vec + P.vec + 4 * (int64_t)P.npad;
    const uint4* outer = reinterpret_cast<const uint4*>(EX.outer) + g1.zoff;
    const uint4* inner = reinterpret_cast<const uint4*>(EY.inner) + g2.loff;
    float* yrow = y + (int64_t)i * n2;
    for (int b0 = kb; b0 < ke; b0 += bmax) {
        const int nb = min(bmax, ke - b0);
        if (b0 > kb) __syncthreads();   // every wave is done with the rows staged before
        // the outer entries go to LDS too: in the product loop they are wave-uniform
        // operands, and a global load of one address by 64 lanes costs a full memory access
        if ((int)threadIdx.x < ((nb + 3) & ~3)) {
            const int t = threadIdx.x;
            if (t < nb) {
                const uint4 e = outer[b0 + t];
                olab[t] = EK == MGK_EK_CONST ? 1.f : __uint_as_float(e.y);
                // the entry carries log2 A_ij where the weight is folded into an exponent
                ow[t] = !WEIGHTED ? 1.f
                        : EK == MGK_EK_CONST ? __uint_as_float(e.y)
                        : (EK == MGK_EK_SE || EK == MGK_EK_KRON_SE) ? __builtin_amdgcn_exp2f(__uint_as_float(e.z))
                        : __uint_as_float(e.z);
                oj[t] = (int)e.x;
            } else {   // padding: a label so far away that kappa_e is exactly 0
                olab[t] = EK == MGK_EK_CONST ? 0.f : 1e18f;
            }
            if (ATTR) {
#pragma unroll
                for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                    if (a < D)
                        oattr[a * MGK_ROWS_MAX_BATCH + t] = t < nb
                            ? X.attr_outer[(int64_t)a * X.nnz_total + g1.zoff + b0 + t] *
                              prm.attr_scale[EK == MGK_EK_RCONV_SE ? 0 : a]
                            : 1e18f;
            }
        }
        // Short rows: the rows of p of the whole batch as one index space, four elements in
        // flight per thread, so that the loads of different rows do not wait for each other
        // (config 2 at density 0.2: 18.6 -> 15.6 ms).  The row of an index comes from a
        // floating-point quotient (exact at these sizes) and one correction.
        __syncthreads();   // oj, ow
        // Row r of the batch is A_ij p_j. for its outer entry (i, j): the weight is applied
        // once per element of the row here instead of once per product below.
        if ((n2 & 3) == 0 && n2 >= (int)blockDim.x) {
            // long rows, 16-byte aligned: one after the other, every thread busy in each
            for (int r = 0; r < nb; ++r) {
                const float4* s4 = reinterpret_cast<const float4*>(p + (int64_t)oj[r] * n2);
                float4* d4 = reinterpret_cast<float4*>(prow + r * n2);
                const float wr = ow[r];
                for (int t = threadIdx.x; t < (n2 >> 2); t += blockDim.x) {
                    float4 v = s4[t];
                    if (WEIGHTED) { v.x *= wr; v.y *= wr; v.z *= wr; v.w *= wr; }
                    d4[t] = v;
                }
            }
        } else if ((n2 & 3) == 0) {
            const int n2q = n2 >> 2, total = nb * n2q;
            const float inv = 1.0f / (float)n2q;
            const float4* p4 = reinterpret_cast<const float4*>(p);
            float4* d4 = reinterpret_cast<float4*>(prow);
            for (int idx0 = threadIdx.x; idx0 < total; idx0 += 4 * blockDim.x) {
                float4 v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = idx0 + q * (int)blockDim.x;
                    if (idx < total) {
                        int r = (int)(((float)idx + 0.5f) * inv);
                        r += (idx - r * n2q >= n2q) - (idx - r * n2q < 0);   // guards the rounding
                        v[q] = p4[(int64_t)oj[r] * n2q + (idx - r * n2q)];
                        if (WEIGHTED) {
                            const float wr = ow[r];
                            v[q].x *= wr; v[q].y *= wr; v[q].z *= wr; v[q].w *= wr;
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = idx0 + q * (int)blockDim.x;
                    if (idx < total) d4[idx] = v[q];
                }
            }
        } else {
            const int total = nb * n2;
            const float inv = 1.0f / (float)n2;
            for (int idx0 = threadIdx.x; idx0 < total; idx0 += 4 * blockDim.x) {
                float v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = idx0 + q * (int)blockDim.x;
                    if (idx < total) {
                        int r = (int)(((float)idx + 0.5f) * inv);
                        r += (idx - r * n2 >= n2) - (idx - r * n2 < 0);
                        v[q] = p[(int64_t)oj[r] * n2 + (idx - r * n2)];
                        if (WEIGHTED) v[q] *= ow[r];
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = idx0 + q * (int)blockDim.x;
                    if (idx < total) prow[idx] = v[q];
                }
            }
        }
        __syncthreads();
        const bool first = b0 == kb;
        rows_sweep<CB, WEIGHTED, EK>(inner, wave, nwaves, chunks, lane, [&](const uint4 (&e2v)[CB], int c0) {
            rows_pass<CB, WEIGHTED, EK>(Y, g2, P, prm, e2v, c0, chunks, lane, prow, olab, oattr, nb, n2, yrow, first);
        });
    }
}

// ---- dense tile-pair XMV (Section III-D "tiling-blocking" primitive as a function) ------
// Octiles expanded to dense 8x8 blocks: weight (0 where absent), scaled label,
// log2 weight (-inf where absent), 64 floats each per tile.
template <int EK>
__global__ __launch_bounds__(256) void mgk_expand_dense_kernel(MgkBatchDev B, MgkParams prm, float* dw,
                                                               float* de, float* dlw) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= B.n_tiles_total) return;
    const MgkGraphDesc g = B.graphs[B.tile_graph[t]];
    const MgkTile tile = B.tiles[t];
    float w = 0.f, el = 0.f, lw = __uint_as_float(0xff800000u);
    if ((tile.bitmap >> lane) & 1ull) {
        const int k = g.zoff + (int)tile.nzoff + __popcll(tile.bitmap & ((1ull << lane) - 1ull));
        w = B.w[k];
        el = (B.e[k] - prm.e_shift) * prm.e_scale;
        lw = __log2f(w);
    }
    dw[(int64_t)t * 64 + lane] = w;
    de[(int64_t)t * 64 + lane] = el;
    dlw[(int64_t)t * 64 + lane] = lw;
}

// One wave per 8x8 block of outputs (tile row I of G x tile row I' of G'), lane
// (i, i') = (lane / 8, lane % 8).  For every pair of non-empty tiles (T in row
// I, T' in row I') the 64 p values of block (J, J') are staged in LDS and read
// back as broadcasts; the lane keeps row i of T and row i' of T' in registers:
//   y_ii' += sum_j A_ij sum_j' A'_i'j' kappa_e(E_ij, E'_i'j') p_jj'
// with A' folded into the exponent.  3 VALU + 1 exp per product, no gathers, no
// row sums; every product of the 8x8x8x8 block is evaluated, present or not.
template <int EK>
__global__ __launch_bounds__(256) void mgk_large_xmv_dense_kernel(
    MgkBatchDev X, MgkBatchDev Y, MgkDenseTiles DX, MgkDenseTiles DY, const MgkLargePair* pairs,
    const MgkPairState* state, float* vec, MgkParams prm) {
    __shared__ __align__(16) float ptile[4][64];
    if (state[blockIdx.y].done) return;
    const float ke_c = prm.ke_const;
    const MgkLargePair P = pairs[blockIdx.y];
    const MgkGraphDesc g1 = X.graphs[P.g1], g2 = Y.graphs[P.g2];
    const int ntr1 = g1.n_tile_rows, ntr2 = g2.n_tile_rows;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ot = blockIdx.x * 4 + wave;        // output block index
    if (ot >= ntr1 * ntr2) return;
    const int I = ot / ntr2, Ip = ot - I * ntr2;
    const int i = lane >> 3, ip = lane & 7;
    const float* p = vec + P.vec + 2 * (int64_t)P.npad;
    float* y = vec + P.vec + 4 * (int64_t)P.npad;
    const int n1 = P.n1, n2 = P.n2;
    const int32_t* trp1 = X.trow_ptr + g1.roff;
    const int32_t* trp2 = Y.trow_ptr + g2.roff;
    const int t1b = trp1[I], t1e = trp1[I + 1];
    const int t2b = trp2[Ip], t2e = trp2[Ip + 1];
    // Sums are kept in levels (product row -> tile pair -> outer tile -> total): a single
    // running fp32 sum over the up to n n' products of a dense row would carry a rounding
    // bias of their count times half an ulp, which ill-conditioned pairs amplify.
    float acc = 0.f;
    float* pt = ptile[wave];
    for (int t1 = t1b; t1 < t1e; ++t1) {
        float acc_t1 = 0.f;
        const int gt1 = g1.toff + t1;
        const int J = X.tiles[gt1].tc;
        float wr[8], er[8];
        {
            const float4* a = reinterpret_cast<const float4*>(DX.w + (int64_t)gt1 * 64 + i * 8);
            const float4* b = reinterpret_cast<const float4*>(DX.e + (int64_t)gt1 * 64 + i * 8);
            const float4 a0 = a[0], a1 = a[1], b0 = b[0], b1 = b[1];
            wr[0] = a0.x; wr[1] = a0.y; wr[2] = a0.z; wr[3] = a0.w; wr[4] = a1.x; wr[5] = a1.y; wr[6] = a1.z; wr[7] = a1.w;
            er[0] = b0.x; er[1] = b0.y; er[2] = b0.z; er[3] = b0.w; er[4] = b1.x; er[5] = b1.y; er[6] = b1.z; er[7] = b1.w;
        }
        const int prow = J * 8 + i;               // this lane's row of the p block (as loader)
        for (int t2 = t2b; t2 < t2e; ++t2) {
            const int gt2 = g2.toff + t2;
            const int Jp = Y.tiles[gt2].tc;
            float f2[8], e2[8];                   // log2 weight (or weight) and label of row i' of T'
            {
                const float* src = EK == MGK_EK_SE ? DY.lw : DY.w;
                const float4* a = reinterpret_cast<const float4*>(src + (int64_t)gt2 * 64 + ip * 8);
                const float4* b = reinterpret_cast<const float4*>(DY.e + (int64_t)gt2 * 64 + ip * 8);
                const float4 a0 = a[0], a1 = a[1], b0 = b[0], b1 = b[1];
                f2[0] = a0.x; f2[1] = a0.y; f2[2] = a0.z; f2[3] = a0.w; f2[4] = a1.x; f2[5] = a1.y; f2[6] = a1.z; f2[7] = a1.w;
                e2[0] = b0.x; e2[1] = b0.y; e2[2] = b0.z; e2[3] = b0.w; e2[4] = b1.x; e2[5] = b1.y; e2[6] = b1.z; e2[7] = b1.w;
            }
            const int pcol = Jp * 8 + ip;
            const float pv = (prow < n1 && pcol < n2) ? p[(int64_t)prow * n2 + pcol] : 0.f;
            __builtin_amdgcn_wave_barrier();
            pt[lane] = pv;
            __builtin_amdgcn_wave_barrier();
            float acc_pair = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float4 pa = *reinterpret_cast<const float4*>(pt + j * 8);
                const float4 pb = *reinterpret_cast<const float4*>(pt + j * 8 + 4);
                const float pj[8] = {pa.x, pa.y, pa.z, pa.w, pb.x, pb.y, pb.z, pb.w};
                float s = 0.f;
#pragma unroll
                for (int jp = 0; jp < 8; ++jp) {
                    if (EK == MGK_EK_SE) {
                        const float d = e2[jp] - er[j];
                        s = __builtin_fmaf(__builtin_amdgcn_exp2f(__builtin_fmaf(-d, d, f2[jp])), pj[jp], s);
                    } else if (EK == MGK_EK_POLY) {
                        s = __builtin_fmaf(mgk_poly_kernel(e2[jp] - er[j], prm.poly_c) * f2[jp], pj[jp], s);
                    } else {
                        s = __builtin_fmaf(f2[jp], pj[jp], s);
                    }
                }
                acc_pair = __builtin_fmaf(wr[j], s, acc_pair);
            }
            acc_t1 += acc_pair;
        }
        acc += acc_t1;
    }
    if (EK == MGK_EK_CONST) acc *= ke_c;
    const int row = I * 8 + i, col = Ip * 8 + ip;
    if (row < n1 && col < n2) y[(int64_t)row * n2 + col] = acc;
}

// ---- p^T a with a = M p - y ---------------------------------------------------------
// Also clears the accumulators of r^T z and r^T r that the update of this iteration adds to
// (their values, from two iterations ago, were last read by the kernel before this one).
__global__ __launch_bounds__(256) void mgk_large_dot_kernel(const MgkLargePair* pairs,
                                                            MgkPairState* state, const float* vec, int it) {
    __shared__ float red[8];
    MgkPairState& st = state[blockIdx.y];
    if (st.done) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) { st.rz[it & 1] = 0.f; st.rr[it & 1] = 0.f; }
    const MgkLargePair P = pairs[blockIdx.y];
    const float* p = vec + P.vec + 2 * (int64_t)P.npad;
    const float* M = p + P.npad;
    const float* y = M + P.npad;
    float s = 0.f;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < P.npad; idx += gridDim.x * blockDim.x) {
        const float pv = p[idx];
        s = __builtin_fmaf(pv, __builtin_fmaf(M[idx], pv, -y[idx]), s);
    }
    block_accumulate(s, &st.pa[it & 1], red);
}

// ---- alpha = rho / p^T a; x += alpha p; r -= alpha a; z = M^{-1} r (stored over y);
//      rho' = r^T z; r^T r.  Clears the accumulator of the next iteration's p^T a.
__global__ __launch_bounds__(256) void mgk_large_update_kernel(const MgkLargePair* pairs,
                                                               MgkPairState* state, float* vec, int it) {
    __shared__ float red[8];
    MgkPairState& st = state[blockIdx.y];
    if (st.done) return;
    const MgkLargePair P = pairs[blockIdx.y];
    const float alpha = st.rz[(it + 1) & 1] / st.pa[it & 1];
    if (blockIdx.x == 0 && threadIdx.x == 0) st.pa[(it + 1) & 1] = 0.f;
    float* x = vec + P.vec;
    float* r = x + P.npad;
    const float* p = r + P.npad;
    const float* M = p + P.npad;
    float* y = const_cast<float*>(M) + P.npad;
    float s_rz = 0.f, s_rr = 0.f;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < P.npad; idx += gridDim.x * blockDim.x) {
        const float pv = p[idx], m = M[idx];
        const float av = __builtin_fmaf(m, pv, -y[idx]);
        x[idx] = __builtin_fmaf(alpha, pv, x[idx]);
        const float rv = __builtin_fmaf(-alpha, av, r[idx]);
        r[idx] = rv;
        const float zv = rv / m;
        y[idx] = zv;
        s_rz = __builtin_fmaf(rv, zv, s_rz);
        s_rr = __builtin_fmaf(rv, rv, s_rr);
    }
    block_accumulate(s_rz, &st.rz[it & 1], red);
    block_accumulate(s_rr, &st.rr[it & 1], red);
}

// ---- stop test; beta = rho' / rho; p = z + beta p; y cleared for the next product.
// Every workgroup takes the same decision from the sums of this iteration, which no one
// writes during this kernel; one thread per pair records it (a workgroup that starts after
// that and sees the pair marked done would have stopped anyway).
__global__ __launch_bounds__(256) void mgk_large_pupdate_kernel(const MgkLargePair* pairs,
                                                                MgkPairState* state, float* vec, int it,
                                                                float rtol2, int* n_active) {
    MgkPairState& st = state[blockIdx.y];
    if (st.done) return;
    const MgkLargePair P = pairs[blockIdx.y];
    const float rz = st.rz[it & 1], rho = st.rz[(it + 1) & 1];
    const bool converged = st.rr[it & 1] <= rtol2 * st.bb;
    const bool stop = converged || it + 1 >= P.max_iter;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st.iters = it + 1;
        if (stop) {
            st.flag = converged ? 0 : 1;
            st.done = 1;
            atomicSub(n_active, 1);
            atomicMax(n_active + 1, it + 1);   // most iterations any pair of the call needed
        }
    }
    if (stop) return;
    const float beta = rz / rho;
    float* p = vec + P.vec + 2 * (int64_t)P.npad;
    float* y = p + 2 * (int64_t)P.npad;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < P.npad; idx += gridDim.x * blockDim.x) {
        p[idx] = __builtin_fmaf(beta, p[idx], y[idx]);
        y[idx] = 0.f;
    }
}

// ---- K = p_x^T x; the nodal solution; how far x exceeds the Jacobi guess M^{-1} b ------------
__global__ __launch_bounds__(256) void mgk_large_final_kernel(MgkBatchDev X, MgkBatchDev Y,
                                                              const MgkLargePair* pairs,
                                                              MgkPairState* state, const float* vec,
                                                              MgkOutputs out, MgkParams prm) {
    __shared__ float red[8];
    const MgkLargePair P = pairs[blockIdx.y];
    const int N = P.n1 * P.n2;
    const MgkGraphDesc g1 = X.graphs[P.g1], g2 = Y.graphs[P.g2];
    const float* x = vec + P.vec;
    float* nodal = out.nodal ? out.nodal + out.nodal_off[P.out0] : nullptr;
    const bool swapped = P.out1 == MGK_OUT1_SWAPPED;
    const float inv_qq = 1.0f / (prm.q * prm.q), inv_h = 1.0f / prm.h;
    float s = 0.f, growth = 0.f;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < N; idx += gridDim.x * blockDim.x) {
        const int i = idx / P.n2, ip = idx - i * P.n2;
        const float xv = x[idx];
        s = __builtin_fmaf(X.start[g1.voff + i] * Y.start[g2.voff + ip], xv, s);
        // (M^{-1} b)_ii' = kappa_v q^2
        const bool same = X.vlabel[g1.voff + i] == Y.vlabel[g2.voff + ip];
        growth = fmaxf(growth, xv * inv_qq * (same ? 1.f : inv_h));
        if (nodal) {
            const int64_t oi = X.iperm[g1.voff + i], oip = Y.iperm[g2.voff + ip];
            nodal[swapped ? oip * P.n1 + oi : oi * P.n2 + oip] = xv;
        }
    }
    // positive floats order like their bit patterns
    growth = fmaxf(growth, 0.f);
    for (int off = 32; off > 0; off >>= 1) growth = fmaxf(growth, __shfl_xor(growth, off));
    if ((threadIdx.x & 63) == 0 && growth > 0.f) atomicMax(&state[blockIdx.y].growth, __float_as_int(growth));
    block_accumulate(s, &state[blockIdx.y].kval, red);
}

// ---- check of pairs with a large growth factor: y = XMV(x), true residual b - (M x - y) ----
// Marks those pairs as running again (done = 0) with p = x and y = 0, so that the product
// kernels of one more launch take them; all other pairs stay done.
__global__ __launch_bounds__(256) void mgk_large_verify_prepare_kernel(const MgkLargePair* pairs,
                                                                       MgkPairState* state, float* vec) {
    MgkPairState& st = state[blockIdx.y];
    if (__int_as_float(st.growth) <= MGK_VERIFY_GROWTH) return;
    const MgkLargePair P = pairs[blockIdx.y];
    const float* x = vec + P.vec;
    float* p = vec + P.vec + 2 * (int64_t)P.npad;
    float* y = p + 2 * (int64_t)P.npad;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < P.npad; idx += gridDim.x * blockDim.x) {
        p[idx] = x[idx];
        y[idx] = 0.f;
    }
    // every workgroup of the pair writes the same values; the product kernels come later
    if (threadIdx.x == 0) { st.done = 0; st.rr[0] = 0.f; }
}

__global__ __launch_bounds__(256) void mgk_large_verify_residual_kernel(MgkBatchDev X, MgkBatchDev Y,
                                                                        const MgkLargePair* pairs,
                                                                        MgkPairState* state, const float* vec,
                                                                        MgkParams prm) {
    __shared__ float red[8];
    MgkPairState& st = state[blockIdx.y];
    if (st.done) return;   // only the pairs under check are marked as running
    const MgkLargePair P = pairs[blockIdx.y];
    const int N = P.n1 * P.n2;
    const MgkGraphDesc g1 = X.graphs[P.g1], g2 = Y.graphs[P.g2];
    const float* x = vec + P.vec;
    const float* M = x + 3 * (int64_t)P.npad;
    const float* y = M + P.npad;
    const float qq = prm.q * prm.q;
    float s = 0.f;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < N; idx += gridDim.x * blockDim.x) {
        const int i = idx / P.n2, ip = idx - i * P.n2;
        const bool same = X.vlabel[g1.voff + i] == Y.vlabel[g2.voff + ip];
        const float m = M[idx];
        const float b = m * (same ? qq : prm.h * qq);            // b = M kappa_v q^2 = d d' q^2
        const float rho = b - __builtin_fmaf(m, x[idx], -y[idx]);
        s = __builtin_fmaf(rho, rho, s);
    }
    block_accumulate(s, &st.rr[0], red);
}

// Per-pair outputs.  A checked pair whose true residual, times its growth factor, says that
// the value may be off by more than MGK_VERIFY_ACCURACY gets flag 3.
__global__ void mgk_large_store_kernel(const MgkLargePair* pairs, MgkPairState* state,
                                       int n_pairs, MgkOutputs out) {
    float* K = out.K;
    int32_t* iters = out.iters;
    int32_t* flags = out.flags;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_pairs) return;
    const MgkLargePair P = pairs[k];
    MgkPairState& s = state[k];
    int flag = s.flag;
    if (!s.done) {   // was under check
        const float growth = __int_as_float(s.growth);
        const float rel = sqrtf(s.rr[0] / s.bb);
        if (flag == 0 && rel * growth > MGK_VERIFY_ACCURACY) flag = 3;
        s.done = 1;
    }
    K[P.out0] = s.kval;
    if (P.out1 >= 0) K[P.out1] = s.kval;
    if (iters) { iters[P.out0] = s.iters; if (P.out1 >= 0) iters[P.out1] = s.iters; }
    if (flags) { flags[P.out0] = flag; if (P.out1 >= 0) flags[P.out1] = flag; }
}

// ---- normalised Gram matrix: K_ij / sqrt(K_ii K_jj) --------------------------------------
__global__ void mgk_diag_kernel(const float* K, float* diag, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) diag[i] = K[(int64_t)i * n + i];
}

__global__ void mgk_normalize_kernel(float* K, const float* diag, int n) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= (int64_t)n * n) return;
    const int i = (int)(k / n), j = (int)(k - (int64_t)i * n);
    K[k] = K[k] / sqrtf(diag[i] * diag[j]);
}

}  // namespace

// ---- launchers -----------------------------------------------------------------------------
hipError_t mgk_launch_expand(const MgkBatchDev& B, const MgkParams& prm, MgkEntry* outer_, MgkEntry* inner_,
                             hipStream_t stream) {
    uint4* outer = reinterpret_cast<uint4*>(outer_);
    uint4* inner = reinterpret_cast<uint4*>(inner_);
    if (B.lanes_total > 0)
        hipLaunchKernelGGL(mgk_fill_idle_kernel, dim3((B.lanes_total + 255) / 256), dim3(256), 0, stream,
                           inner, B.lanes_total,
                           (prm.edge_kernel == MGK_EK_POLY || prm.edge_kernel == MGK_EK_RCONV_SE) ? 0u : 0xff800000u);
    if (B.n_tiles_total > 0) {
        const dim3 grid((B.n_tiles_total + 3) / 4);
        switch (prm.edge_kernel) {
#define MGK_EXPAND(EKV) \
    case EKV: hipLaunchKernelGGL(mgk_expand_kernel<EKV>, grid, dim3(256), 0, stream, B, prm, outer, inner); break;
            MGK_EXPAND(MGK_EK_SE) MGK_EXPAND(MGK_EK_CONST) MGK_EXPAND(MGK_EK_POLY)
            MGK_EXPAND(MGK_EK_KRON_SE) MGK_EXPAND(MGK_EK_RCONV_SE)
#undef MGK_EXPAND
            default: return hipErrorInvalidValue;
        }
    }
    return hipGetLastError();
}

hipError_t mgk_launch_expand_dense(const MgkBatchDev& B, const MgkParams& prm, float* dw, float* de,
                                   float* dlw, hipStream_t stream) {
    if (B.n_tiles_total > 0) {
        const dim3 grid((B.n_tiles_total + 3) / 4);
        if (prm.edge_kernel == MGK_EK_SE)
            hipLaunchKernelGGL(mgk_expand_dense_kernel<MGK_EK_SE>, grid, dim3(256), 0, stream, B, prm, dw, de, dlw);
        else
            hipLaunchKernelGGL(mgk_expand_dense_kernel<MGK_EK_CONST>, grid, dim3(256), 0, stream, B, prm, dw, de, dlw);
    }
    return hipGetLastError();
}

hipError_t mgk_launch_large_init(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkLargePair* pairs,
                                 MgkPairState* state, float* vec, const MgkParams& prm, int n_pairs,
                                 int vec_blocks, hipStream_t stream) {
    hipLaunchKernelGGL(mgk_large_init_kernel, dim3(vec_blocks, n_pairs), dim3(256), 0, stream, X, Y, pairs,
                       state, vec, prm);
    return hipGetLastError();
}

static hipError_t launch_large_xmv(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkExpanded& EX,
                                   const MgkExpanded& EY, const MgkLargePair* pairs,
                                   MgkPairState* state, float* vec, const MgkParams& prm,
                                   bool weighted, int n_pairs, int xmv_blocks, const MgkDenseTiles* DX,
                                   const MgkDenseTiles* DY, int rows_threads, int rows_lds_bytes,
                                   int rows_chunks, hipStream_t stream);

hipError_t mgk_launch_large_iteration(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkExpanded& EX,
                                      const MgkExpanded& EY, const MgkLargePair* pairs,
                                      MgkPairState* state, float* vec, const MgkParams& prm,
                                      bool weighted, int n_pairs, int xmv_blocks, int vec_blocks,
                                      int* n_active, int it, const MgkDenseTiles* DX,
                                      const MgkDenseTiles* DY, int rows_threads, int rows_lds_bytes,
                                      int rows_chunks, hipStream_t stream) {
    const dim3 gv(vec_blocks, n_pairs);
    hipError_t e = launch_large_xmv(X, Y, EX, EY, pairs, state, vec, prm, weighted, n_pairs, xmv_blocks, DX, DY,
                                    rows_threads, rows_lds_bytes, rows_chunks, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mgk_large_dot_kernel, gv, dim3(256), 0, stream, pairs, state, vec, it);
    hipLaunchKernelGGL(mgk_large_update_kernel, gv, dim3(256), 0, stream, pairs, state, vec, it);
    hipLaunchKernelGGL(mgk_large_pupdate_kernel, gv, dim3(256), 0, stream, pairs, state, vec, it, prm.rtol2, n_active);
    return hipGetLastError();
}

// The product y = XMV(p) for every pair that is marked as running.
static hipError_t launch_large_xmv(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkExpanded& EX,
                                   const MgkExpanded& EY, const MgkLargePair* pairs,
                                   MgkPairState* state, float* vec, const MgkParams& prm,
                                   bool weighted, int n_pairs, int xmv_blocks, const MgkDenseTiles* DX,
                                   const MgkDenseTiles* DY, int rows_threads, int rows_lds_bytes,
                                   int rows_chunks, hipStream_t stream) {
    const dim3 gx(xmv_blocks, n_pairs);
    if (DX == nullptr && rows_threads > 0) {
        // xmv_blocks = largest number of outer rows of a pair
#define MGK_ROWS_GO(WT, EKV, CBV, SLOT) \
    { \
        auto kern = mgk_large_xmv_rows_kernel<WT, EKV, CBV>; \
        static bool configured = false; \
        if (!configured) { \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, MGK_LDS_LIMIT_BYTES); \
            if (e != hipSuccess) return e; \
            configured = true; \
        } \
        hipLaunchKernelGGL(kern, gx, dim3(rows_threads), rows_lds_bytes + 16 + MGK_ROWS_MAX_BATCH * (4 + MGK_MAX_LABEL_DIM) * sizeof(float), stream, X, Y, EX, EY, pairs, state, vec, prm, rows_lds_bytes / 4); \
    }
#define MGK_ROWS(EKV) \
    case EKV: \
        if (rows_chunks >= 4) { if (weighted) MGK_ROWS_GO(true, EKV, 4, 0) else MGK_ROWS_GO(false, EKV, 4, 1) } \
        else if (rows_chunks >= 2) { if (weighted) MGK_ROWS_GO(true, EKV, 2, 2) else MGK_ROWS_GO(false, EKV, 2, 3) } \
        else { if (weighted) MGK_ROWS_GO(true, EKV, 1, 4) else MGK_ROWS_GO(false, EKV, 1, 5) } \
        break;
        switch (prm.edge_kernel) {
            MGK_ROWS(MGK_EK_SE) MGK_ROWS(MGK_EK_CONST) MGK_ROWS(MGK_EK_POLY)
            MGK_ROWS(MGK_EK_KRON_SE) MGK_ROWS(MGK_EK_RCONV_SE)
            default: return hipErrorInvalidValue;
        }
#undef MGK_ROWS_GO
#undef MGK_ROWS
    } else if (DX != nullptr) {
        if (prm.edge_kernel == MGK_EK_SE)
            hipLaunchKernelGGL(mgk_large_xmv_dense_kernel<MGK_EK_SE>, gx, dim3(256), 0, stream, X, Y, *DX, *DY, pairs, state, vec, prm);
        else if (prm.edge_kernel == MGK_EK_POLY)
            hipLaunchKernelGGL(mgk_large_xmv_dense_kernel<MGK_EK_POLY>, gx, dim3(256), 0, stream, X, Y, *DX, *DY, pairs, state, vec, prm);
        else if (prm.edge_kernel == MGK_EK_CONST)
            hipLaunchKernelGGL(mgk_large_xmv_dense_kernel<MGK_EK_CONST>, gx, dim3(256), 0, stream, X, Y, *DX, *DY, pairs, state, vec, prm);
        else
            return hipErrorInvalidValue;   // kernels over label attributes use the sparse product
    } else {
#define MGK_XMV(EKV) \
    case EKV: \
        if (weighted) hipLaunchKernelGGL((mgk_large_xmv_kernel<true, EKV>), gx, dim3(kThreads), 0, stream, X, Y, EX, EY, pairs, state, vec, prm); \
        else hipLaunchKernelGGL((mgk_large_xmv_kernel<false, EKV>), gx, dim3(kThreads), 0, stream, X, Y, EX, EY, pairs, state, vec, prm); \
        break;
        switch (prm.edge_kernel) {
            MGK_XMV(MGK_EK_SE) MGK_XMV(MGK_EK_CONST) MGK_XMV(MGK_EK_POLY) MGK_XMV(MGK_EK_KRON_SE) MGK_XMV(MGK_EK_RCONV_SE)
            default: return hipErrorInvalidValue;
        }
#undef MGK_XMV
    }
    return hipGetLastError();
}

hipError_t mgk_launch_large_final(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkExpanded& EX,
                                  const MgkExpanded& EY, const MgkLargePair* pairs, MgkPairState* state,
                                  float* vec, const MgkParams& prm, bool weighted, int n_pairs, int xmv_blocks,
                                  int vec_blocks, const MgkDenseTiles* DX, const MgkDenseTiles* DY,
                                  int rows_threads, int rows_lds_bytes, int rows_chunks, const MgkOutputs& out,
                                  hipStream_t stream) {
    const dim3 gv(vec_blocks, n_pairs);
    hipLaunchKernelGGL(mgk_large_final_kernel, gv, dim3(256), 0, stream, X, Y, pairs, state, vec, out, prm);
    // one more product and the true residual for the pairs whose solution grew far beyond the
    // Jacobi guess (none on well-conditioned workloads: these launches then return at once)
    hipLaunchKernelGGL(mgk_large_verify_prepare_kernel, gv, dim3(256), 0, stream, pairs, state, vec);
    hipError_t e = launch_large_xmv(X, Y, EX, EY, pairs, state, vec, prm, weighted, n_pairs, xmv_blocks, DX, DY,
                                    rows_threads, rows_lds_bytes, rows_chunks, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mgk_large_verify_residual_kernel, gv, dim3(256), 0, stream, X, Y, pairs, state, vec, prm);
    hipLaunchKernelGGL(mgk_large_store_kernel, dim3((n_pairs + 63) / 64), dim3(64), 0, stream, pairs, state,
                       n_pairs, out);
    return hipGetLastError();
}

hipError_t mgk_launch_normalize(float* K, float* diag, int n, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(mgk_diag_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, K, diag, n);
    const int64_t nn = (int64_t)n * n;
    hipLaunchKernelGGL(mgk_normalize_kernel, dim3((unsigned)((nn + 255) / 256)), dim3(256), 0, stream, K, diag, n);
    return hipGetLastError();
}
