// On-chip solver: one workgroup runs the whole preconditioned CG iteration
// (Alg. 1) for one graph pair.  The search direction p and the off-diagonal
// product y live in LDS; x, r, M and the owner's copies of p and z live in
// registers, EPT elements per thread.
//
// The off-diagonal product of Alg. 1 (the XMV of Alg. 2) is formed on the fly.
// The octiles of both graphs are expanded once per pair into LDS entry lists
// (Section IV-B: stored compact, expanded on chip).  The inner graph's
// nonzeros then sit one per lane in registers, rows in adjacent lanes; the
// outer graph's nonzeros are streamed from LDS as wave-uniform operands in row
// order, four at a time so that their LDS reads overlap.  Each (outer, inner)
// nonzero pair costs one kappa_e evaluation, one gathered read of p_jj' and
// one fused multiply-add into a register that lasts for the outer row i.  At
// the end of the row the lanes of each inner row i' are summed with DPP
// shifts and one lane stores y_ii'.  Every y_ii' has exactly one writer, so no
// atomics are needed (LDS float atomics cost ~200 clocks per wavefront
// instruction on this chip, against 2 for a store).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mgk_internal.h"
#include "mgk_launch.h"
#include "mgk_wave.h"

namespace {

// Expand packed nonzero k of a graph (one thread per nonzero) into the entry
// list of its graph: find its octile in the staged tile list, its bit in the
// occupancy bitmap, and from the bitmaps of the tile row its position in the
// row.  (Octiles of these graphs hold only a few nonzeros, so a thread per
// nonzero wastes far fewer lanes than a lane per bit of every bitmap.)
// Outer graph: CSR order, entry = {byte offset of p row j, scaled label (or
// weight for the constant kernel), log2 weight (the weight itself for the
// polynomial kernel), byte offset of y row i};
// `rowend` gets bit k set when entry k is the last of its row.
// Inner graph: lane layout (rows in adjacent lanes inside groups of 16), entry
// = {i'*4 | rank in run << 20 | row-longer-than-16 << 30 | last-of-run << 31,
// j'*4, scaled label or weight, log2 weight}.
// PLANES (outer graph only): the four words of entry k go to four arrays of `stride`
// words each (word w of entry k at ent[w * stride + k]) instead of one 16-byte record.
template <bool OUTER, bool WEIGHTED, int EK, bool PLANES>
__device__ __forceinline__ void expand_nonzero(const MgkBatchDev& B, const MgkGraphDesc& g,
                                               const MgkTile* tiles_lds, int k, uint4* ent,
                                               uint32_t* rowend, int n_inner, const MgkParams& prm,
                                               int stride) {
    int lo = 0, hi = g.n_tiles;   // last tile whose first packed nonzero is <= k
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int)tiles_lds[mid].nzoff <= k) lo = mid; else hi = mid;
    }
    const int t = lo;
    const MgkTile tile = tiles_lds[t];
    int rest = k - (int)tile.nzoff;   // index of the nonzero among the set bits of the bitmap
    int r = 0;
    uint32_t rowbyte = (uint32_t)tile.bitmap & 0xffu;
    while (rest >= __popc(rowbyte)) {  // ends: the tile holds more than `rest` nonzeros
        rest -= __popc(rowbyte);
        ++r;
        rowbyte = (uint32_t)(tile.bitmap >> (8 * r)) & 0xffu;
    }
    uint32_t bits = rowbyte;
    for (int q = 0; q < rest; ++q) bits &= bits - 1u;
    const int c = __ffs(bits) - 1;
    const int row = (int)tile.tr * 8 + r, col = (int)tile.tc * 8 + c;
    int rank = rest;                  // position inside the row: earlier tiles of the tile row first
    for (int tp = t - 1; tp >= 0 && tiles_lds[tp].tr == tile.tr; --tp)
        rank += __popc((uint32_t)(tiles_lds[tp].bitmap >> (8 * r)) & 0xffu);
    const float w = B.w[g.zoff + k];
    const float el = (B.e[g.zoff + k] - prm.e_shift) * prm.e_scale;
    const int rp0 = B.rowptr[g.voff + row];
    const int rp1 = (row + 1 < g.n) ? B.rowptr[g.voff + row + 1] : g.nnz;
    uint4 v;
    if (OUTER) {
        const int pos = rp0 + rank;
        v.x = (uint32_t)(col * n_inner * 4);
        v.y = __float_as_uint(EK == MGK_EK_CONST ? w : el);
        v.z = __float_as_uint((EK == MGK_EK_POLY || EK == MGK_EK_RCONV_SE) ? w : WEIGHTED ? __log2f(w) : 0.f);
        v.w = (uint32_t)(row * n_inner * 4);
        if (PLANES) {
            uint32_t* words = reinterpret_cast<uint32_t*>(ent);
            words[pos] = v.x;
            words[stride + pos] = v.y;
            words[2 * stride + pos] = v.z;
            words[3 * stride + pos] = v.w;
        } else {
            ent[pos] = v;
        }
        if (pos + 1 == rp1) atomicOr(&rowend[pos >> 5], 1u << (pos & 31));
    } else {
        const int lp = B.lanepos[g.voff + row];
        const int deg = rp1 - rp0;
        const MgkRunPos rp = mgk_run_pos(lp, rank, deg);   // cut: the row has several runs
        v.x = (uint32_t)(row * 4) | (rp.rank << 20) | (rp.cut << 30) | (rp.last << 31);
        v.y = (uint32_t)(col * 4);
        v.z = __float_as_uint(EK == MGK_EK_CONST ? w : el);
        v.w = __float_as_uint((EK == MGK_EK_POLY || EK == MGK_EK_RCONV_SE) ? w : WEIGHTED ? __log2f(w) : 0.f);
        ent[lp + rank] = v;
    }
}

// position of the first set bit at or after `from` in a bit array of `words` words; `none` if absent
__device__ __forceinline__ int next_set_bit(const uint32_t* bits, int words, int from, int none) {
    int wi = from >> 5;
    if (wi >= words) return none;
    uint32_t cur = bits[wi] & (0xffffffffu << (from & 31));
    while (true) {
        if (cur) return wi * 32 + __ffs(cur) - 1;
        if (++wi >= words) return none;
        cur = bits[wi];
    }
}

// One XMV (Alg. 2) over this wave's share [kbeg, kend) of the outer nonzeros and CB
// chunks of 64 inner lane slots starting at ent2c[0] (this lane's slot of the first):
// y_ii' = sum_{j,j'} A_ij A'_i'j' kappa_e(E_ij, E'_i'j') p_jj'.  NSTEPS DPP
// shift-and-add steps sum the lanes of each inner row (rows of up to 2^NSTEPS
// nonzeros).  Every outer entry is a 16-byte broadcast read, which costs the LDS
// twice what a conflict-free gather of p does: with CB chunks per pass it is
// read 1/CB as often.
// ATOMIC: the wave's share may begin and end inside an outer row.  kfirst is the
// first row end of the share if that row began in the previous wave's share (-1
// otherwise), force_end says that the share ends inside a row; the sums of both
// rows are added to y atomically, like those of inner rows cut into several runs.
// What the kernels over label attributes read beside the entries: attribute a of outer
// nonzero k, prescaled, at outer[a * z1pad + k] (LDS); attribute a of this lane's inner
// nonzero of the chunk at inner[a * inner_stride] (global memory, 0 on idle slots).
struct MgkAttrArgs {
    const float* outer;
    const float* inner;
    int64_t inner_stride;
    int dim;
    float scale[MGK_MAX_LABEL_DIM];
};

template <int CB, int NSTEPS, bool WEIGHTED, int EK, bool ATOMIC>
__device__ __forceinline__ void xmv_chunks(const uint4* ent1, const uint4* ent2c, const uint32_t* rowend,
                                           const char* pbytes, char* ybytes, int kbeg, int kend,
                                           int kfirst, bool force_end, float ke_c, const float* pc,
                                           int z1pad, const MgkAttrArgs& at) {
    static_assert(CB == 1 || CB == 2 || CB == 4, "one, two or four chunks per pass");
    constexpr bool ATTR = EK == MGK_EK_KRON_SE || EK == MGK_EK_RCONV_SE;
    uint32_t ip4[CB], jp4[CB], rank[CB];
    bool last[CB], longrow[CB];
    float el2[CB], lw2[CB], acc[CB];
    float e2a[CB][MGK_MAX_LABEL_DIM];   // this lane's attributes, prescaled
#pragma unroll
    for (int b = 0; b < CB; ++b)
#pragma unroll
        for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
            e2a[b][a] = ATTR && a < at.dim ? at.inner[a * at.inner_stride + 64 * b] * at.scale[a] : 0.f;
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        const uint4 e2 = ent2c[64 * b];
        ip4[b] = e2.x & 0xfffffu;
        jp4[b] = e2.y;
        rank[b] = (e2.x >> 20) & 0xffu;
        last[b] = (e2.x >> 31) != 0u;
        longrow[b] = ((e2.x >> 30) & 1u) != 0u;
        el2[b] = __uint_as_float(e2.z);
        lw2[b] = __uint_as_float(e2.w);
        acc[b] = 0.f;
    }
    // multipliers of the shift-and-add steps: 1 where the lane DIST places lower belongs
    // to the same run.  Short rows end every few entries: kept in registers; with long
    // rows (NSTEPS > 2) the ends are rare and the masks are made when needed.
    float m1[CB], m2[CB];
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        m1[b] = rank[b] >= 1 ? 1.f : 0.f;
        m2[b] = rank[b] >= 2 ? 1.f : 0.f;
    }
    for (int k0 = kbeg; k0 < kend; k0 += 32) {
        // row-end bits of entries k0 .. k0+31
        const uint32_t lo = __builtin_amdgcn_readfirstlane(rowend[k0 >> 5]);
        const uint32_t hi = __builtin_amdgcn_readfirstlane(rowend[(k0 >> 5) + 1]);
        uint32_t window = (uint32_t)((((uint64_t)hi << 32) | lo) >> (k0 & 31));
        const int kstop = min(k0 + 32, kend);
        if (kstop - k0 < 32) window &= (1u << (kstop - k0)) - 1u;
        if (ATOMIC && force_end && kstop == kend) window |= 1u << (kend - 1 - k0);
        for (int k = k0; k < kstop; k += 4, window >>= 4) {
            uint4 e1[4];
            float pv[4][CB], cu[4][CB];
            if constexpr (ATOMIC) {
                // four arrays instead of records: one broadcast read brings a word of four
                // entries (k is a multiple of 4 here); the offset of the row of y is read
                // where a row ends, which is rare in graphs with long rows
                const uint32_t* words = reinterpret_cast<const uint32_t*>(ent1);
                const uint4 x4 = *reinterpret_cast<const uint4*>(words + k);
                const uint4 y4 = *reinterpret_cast<const uint4*>(words + z1pad + k);
                e1[0].x = x4.x; e1[1].x = x4.y; e1[2].x = x4.z; e1[3].x = x4.w;
                e1[0].y = y4.x; e1[1].y = y4.y; e1[2].y = y4.z; e1[3].y = y4.w;
                if (WEIGHTED && EK != MGK_EK_CONST) {
                    const uint4 z4 = *reinterpret_cast<const uint4*>(words + 2 * z1pad + k);
                    e1[0].z = z4.x; e1[1].z = z4.y; e1[2].z = z4.z; e1[3].z = z4.w;
                }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) e1[u] = ent1[k + u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int b = 0; b < CB; ++b)
                    pv[u][b] = *reinterpret_cast<const float*>(pbytes + (e1[u].x + jp4[b]));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
#pragma unroll
                for (int b = 0; b < CB; ++b) {
                    if (EK == MGK_EK_SE) {
                        const float d = el2[b] - __uint_as_float(e1[u].y);
                        float t;
                        if (WEIGHTED) t = __builtin_fmaf(-d, d, lw2[b] + __uint_as_float(e1[u].z));
                        else t = __builtin_fmaf(-d, d, lw2[b]);  // lw2: 0, or -inf on idle lanes
                        cu[u][b] = __builtin_amdgcn_exp2f(t);
                    } else if (EK == MGK_EK_POLY) {
                        cu[u][b] = mgk_poly_kernel(el2[b] - __uint_as_float(e1[u].y), pc);
                        if (WEIGHTED) cu[u][b] *= __uint_as_float(e1[u].z);     // A_ij
                    } else if (EK == MGK_EK_KRON_SE) {
                        // product of square exponentials over the attributes: one exponent
                        float t = WEIGHTED ? lw2[b] + __uint_as_float(e1[u].z) : lw2[b];
#pragma unroll
                        for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                            if (a < at.dim) {
                                const float d = e2a[b][a] - at.outer[a * z1pad + k + u];
                                t = __builtin_fmaf(-d, d, t);
                            }
                        cu[u][b] = __builtin_amdgcn_exp2f(t);
                    } else if (EK == MGK_EK_RCONV_SE) {
                        // sum over all pairs of parts; A'_i'j' / D^2 is applied at the row end
                        float sum = 0.f;
#pragma unroll
                        for (int q = 0; q < MGK_MAX_LABEL_DIM; ++q)
                            if (q < at.dim) {
                                const float e1q = at.outer[q * z1pad + k + u];
#pragma unroll
                                for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                                    if (a < at.dim) {
                                        const float d = e2a[b][a] - e1q;
                                        sum += __builtin_amdgcn_exp2f(-d * d);
                                    }
                            }
                        cu[u][b] = WEIGHTED ? sum * __uint_as_float(e1[u].z) : sum;
                    } else {
                        cu[u][b] = WEIGHTED ? __uint_as_float(e1[u].y) : 1.f;  // A_ij
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
#pragma unroll
                for (int b = 0; b < CB; ++b) acc[b] = __builtin_fmaf(cu[u][b], pv[u][b], acc[b]);
                if ((window >> u) & 1u) {   // end of outer row i: sum over each inner row
                    // wave-uniform: this wave holds only a part of outer row i
                    const bool part = ATOMIC && (k + u == kfirst || (force_end && k + u == kend - 1));
                    const uint32_t yoff = ATOMIC ? reinterpret_cast<const uint32_t*>(ent1)[3 * z1pad + k + u]
                                                 : e1[u].w;
#pragma unroll
                    for (int b = 0; b < CB; ++b) {
                        if (EK == MGK_EK_CONST) acc[b] *= ke_c * el2[b];  // el2 = A'_i'j' (0 on idle lanes)
                        if (EK == MGK_EK_POLY) acc[b] *= lw2[b];           // lw2 = A'_i'j' (0 on idle lanes)
                        if (EK == MGK_EK_RCONV_SE) acc[b] *= lw2[b] * (1.0f / (float)(at.dim * at.dim));
                    }
                    if constexpr (CB == 1) {
                        if (NSTEPS > 0) acc[0] = shr_fmac<1>(acc[0], m1[0]);
                        if (NSTEPS > 1) acc[0] = shr_fmac<2>(acc[0], m2[0]);
                        if (NSTEPS > 2) acc[0] = shr_fmac<4>(acc[0], rank[0] >= 4 ? 1.f : 0.f);
                        if (NSTEPS > 3) acc[0] = shr_fmac<8>(acc[0], rank[0] >= 8 ? 1.f : 0.f);
                    } else {
#pragma unroll
                        for (int b = 0; b < CB; b += 2) {
                            if (NSTEPS > 0) shr_fmac_pair<1>(acc[b], acc[b + 1], m1[b], m1[b + 1]);
                            if (NSTEPS > 1) shr_fmac_pair<2>(acc[b], acc[b + 1], m2[b], m2[b + 1]);
                            if (NSTEPS > 2) shr_fmac_pair<4>(acc[b], acc[b + 1], rank[b] >= 4 ? 1.f : 0.f,
                                                             rank[b + 1] >= 4 ? 1.f : 0.f);
                            if (NSTEPS > 3) shr_fmac_pair<8>(acc[b], acc[b + 1], rank[b] >= 8 ? 1.f : 0.f,
                                                             rank[b + 1] >= 8 ? 1.f : 0.f);
                        }
                    }
#pragma unroll
                    for (int b = 0; b < CB; ++b) {
                        if (last[b]) {
                            float* dst = reinterpret_cast<float*>(ybytes + (yoff + ip4[b]));
                            if (ATOMIC && (longrow[b] || part))   // several sums add up to one y_ii'
                                __hip_atomic_fetch_add(dst, acc[b], __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_WORKGROUP);
                            else
                                *dst = acc[b];
                        }
                        acc[b] = 0.f;
                    }
                }
            }
        }
    }
}

// The whole inner lane layout (len2 slots, a multiple of 64): four chunks per pass,
// then two, then one for what is left.
template <int NSTEPS, bool WEIGHTED, int EK, bool ATOMIC>
__device__ __forceinline__ void xmv_pass(const uint4* ent1, const uint4* ent2, const uint32_t* rowend,
                                         const char* pbytes, char* ybytes, int len2, int kbeg,
                                         int kend, int kfirst, bool force_end, float ke_c,
                                         const float* pc, int lane, int z1pad, MgkAttrArgs at) {
    // A kernel's register count is that of its widest path: four chunks per pass only in
    // the kernels for graphs with long rows, whose inner layouts have many chunks; one for
    // the kernels over label attributes, which hold up to four attributes per chunk.
    constexpr bool ATTR = EK == MGK_EK_KRON_SE || EK == MGK_EK_RCONV_SE;
    constexpr int CBMAX = ATTR ? 1 : ATOMIC ? 4 : 2;
    const float* inner0 = at.inner;   // attribute 0 of lane slot `lane`
    int c = 0;
    if constexpr (CBMAX >= 4)
        for (; c + 256 <= len2; c += 256)
            xmv_chunks<4, NSTEPS, WEIGHTED, EK, ATOMIC>(ent1, ent2 + c + lane, rowend, pbytes, ybytes,
                                                        kbeg, kend, kfirst, force_end, ke_c, pc, z1pad, at);
    if constexpr (CBMAX >= 2)
        for (; c + 128 <= len2; c += 128)
            xmv_chunks<2, NSTEPS, WEIGHTED, EK, ATOMIC>(ent1, ent2 + c + lane, rowend, pbytes, ybytes,
                                                        kbeg, kend, kfirst, force_end, ke_c, pc, z1pad, at);
    for (; c < len2; c += 64) {
        if (ATTR) at.inner = inner0 + c;
        xmv_chunks<1, NSTEPS, WEIGHTED, EK, ATOMIC>(ent1, ent2 + c + lane, rowend, pbytes, ybytes,
                                                    kbeg, kend, kfirst, force_end, ke_c, pc, z1pad, at);
    }
}

// ATOMIC: the inner graph has rows longer than 16 nonzeros; the runs of those rows are
// combined with float atomics and y is cleared by its reader every iteration.
template <int WAVES, int EPT, bool WEIGHTED, int EK, bool ATOMIC>
__global__ __launch_bounds__(WAVES * 64) void mgk_pcg_small(
    MgkBatchDev X, MgkBatchDev Y, const MgkJob* __restrict__ jobs, MgkParams prm, MgkOutputs out) {
    extern __shared__ __align__(16) uint32_t lds[];
    constexpr int NT = WAVES * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    const MgkJob job = jobs[blockIdx.x];
    const MgkGraphDesc g1 = X.graphs[job.g1];
    const MgkGraphDesc g2 = Y.graphs[job.g2];
    const int n1 = g1.n, n2 = g2.n, N = n1 * n2, z1 = g1.nnz, len2 = g2.lane_len;
    constexpr bool ATTR = EK == MGK_EK_KRON_SE || EK == MGK_EK_RCONV_SE;   // labels with several attributes
    const int attr_dim = ATTR ? prm.label_dim : 0;
    const MgkSmallPlan L = mgk_small_plan(n1, n2, z1, len2, g1.n_tiles, g2.n_tiles, WAVES, EPT, attr_dim);

    float* p = reinterpret_cast<float*>(lds + L.p);
    float* y = reinterpret_cast<float*>(lds + L.y);
    uint4* ent1 = reinterpret_cast<uint4*>(lds + L.ent1);
    uint4* ent2 = reinterpret_cast<uint4*>(lds + L.ent2);
    uint32_t* rowend = lds + L.rowend;
    float* oattr = reinterpret_cast<float*>(lds + L.attr1);
    MgkTile* tl1 = reinterpret_cast<MgkTile*>(lds + L.tiles1);
    MgkTile* tl2 = reinterpret_cast<MgkTile*>(lds + L.tiles2);
    float* dq1 = reinterpret_cast<float*>(lds + L.vtx1);           // d_i = rowsum + q
    float* st1 = dq1 + n1;                                         // start probability
    int* lb1 = reinterpret_cast<int*>(st1 + n1);                   // vertex label
    float* dq2 = reinterpret_cast<float*>(lds + L.vtx2);
    float* st2 = dq2 + n2;
    int* lb2 = reinterpret_cast<int*>(st2 + n2);
    float* red = reinterpret_cast<float*>(lds + L.red);

    // ---- stage tiles and per-vertex data; clear row-end bits, entries and y ----
    for (int t = tid; t < g1.n_tiles; t += NT) tl1[t] = X.tiles[g1.toff + t];
    for (int t = tid; t < g2.n_tiles; t += NT) tl2[t] = Y.tiles[g2.toff + t];
    for (int v = tid; v < n1; v += NT) {
        dq1[v] = X.rowsum[g1.voff + v] + prm.q;
        st1[v] = X.start[g1.voff + v];
        lb1[v] = X.vlabel[g1.voff + v];
    }
    for (int v = tid; v < n2; v += NT) {
        dq2[v] = Y.rowsum[g2.voff + v] + prm.q;
        st2[v] = Y.start[g2.voff + v];
        lb2[v] = Y.vlabel[g2.voff + v];
    }
    for (int k = tid; k < L.rowend_words; k += NT) rowend[k] = 0u;
    // spare outer entries past z1 (read by the 4-wide loop, never used) and idle
    // lane slots of the inner layout: weight 0, address 0, never the end of a run
    for (int k = z1 + tid; k < L.z1pad; k += NT) {
        if (ATOMIC) {   // entries as four arrays of z1pad words, see xmv_chunks
            uint32_t* words = reinterpret_cast<uint32_t*>(ent1);
            words[k] = words[L.z1pad + k] = words[2 * L.z1pad + k] = words[3 * L.z1pad + k] = 0u;
        } else {
            ent1[k] = make_uint4(0u, 0u, 0u, 0u);
        }
    }
    // label attributes of the outer nonzeros (CSR order, as the entries), prescaled
    if (ATTR) {
        for (int a = 0; a < attr_dim; ++a) {
            const float sc = prm.attr_scale[EK == MGK_EK_RCONV_SE ? 0 : a];
            for (int k = tid; k < L.z1pad; k += NT)
                oattr[a * L.z1pad + k] = k < z1 ? X.attr_outer[(int64_t)a * X.nnz_total + g1.zoff + k] * sc : 0.f;
        }
    }
    // idle slots: log2 w = -inf, or w = 0 where the entry carries the weight itself
    for (int k = tid; k < len2; k += NT) ent2[k] = make_uint4(0u, 0u, 0u, (EK == MGK_EK_POLY || EK == MGK_EK_RCONV_SE) ? 0u : 0xff800000u);
#pragma unroll
    for (int m = 0; m < EPT; ++m) y[tid + m * NT] = 0.f;  // entries no row pair reaches stay 0
    __syncthreads();

    // ---- expand the octiles, one thread per packed nonzero --------------------
    for (int k = tid; k < z1 + g2.nnz; k += NT) {
        if (k < z1)
            expand_nonzero<true, WEIGHTED, EK, ATOMIC>(X, g1, tl1, k, ent1, rowend, n2, prm, L.z1pad);
        else
            expand_nonzero<false, WEIGHTED, EK, false>(Y, g2, tl2, k - z1, ent2, nullptr, n2, prm, 0);
    }

    // ---- Alg. 1 set-up: M = D_x V_x^{-1}, x = 0, r = b = D_x q_x, z = M^{-1} r,
    //      p = z, rho = r^T z ----------------------------------------------------
    float xr[EPT], rr_[EPT], Mr[EPT], pr[EPT], zr[EPT];
    const float qq = prm.q * prm.q;
    const float inv_n2 = 1.0f / (float)n2;
    const float inv_h = 1.0f / prm.h;
    float s_rz = 0.f, s_bb = 0.f;
#pragma unroll
    for (int m = 0; m < EPT; ++m) {
        const int idx = tid + m * NT;
        const bool ok = idx < N;
        const int ic = ok ? idx : 0;
        const int i = (int)(((float)ic + 0.5f) * inv_n2);
        const int ip = ic - i * n2;
        const bool same = lb1[i] == lb2[ip];
        const float dd = dq1[i] * dq2[ip];
        const float b = ok ? dd * qq : 0.f;
        const float z0 = ok ? (same ? qq : prm.h * qq) : 0.f;  // M^{-1} b = kappa_v q q'
        Mr[m] = ok ? (same ? dd : dd * inv_h) : 1.f;           // d d' / kappa_v
        xr[m] = 0.f;
        rr_[m] = b;
        pr[m] = z0;
        p[idx] = z0;   // p and y are padded to NT * EPT; the padding stays 0
        s_rz = __builtin_fmaf(b, z0, s_rz);
        s_bb = __builtin_fmaf(b, b, s_bb);
    }
    block_sum2<WAVES>(s_rz, s_bb, red, wave, lane);
    float rho = s_rz;
    const float thresh = prm.rtol2 * s_bb;
    int max_iter = prm.max_iter;
    if (max_iter <= 0) max_iter = min(2 * N, 1000);
    __syncthreads();  // entries, row-end bits and p are complete

    // ---- this wave's share of the outer nonzeros: whole rows, about z1 / WAVES
    //      (ATOMIC: exactly that many, rounded up to the groups of four the XMV reads;
    //      the rows cut by a share boundary are completed with atomic adds)
    int kbeg = 0, kend = z1, kfirst = -1;
    bool force_end = false;
    if (WAVES > 1) {
        if (ATOMIC) {
            const int share4 = (L.share + 3) & ~3;
            kbeg = min(wave * share4, z1);
            kend = min(kbeg + share4, z1);
            if (kbeg < kend) {
                if (kbeg > 0 && !((rowend[(kbeg - 1) >> 5] >> ((kbeg - 1) & 31)) & 1u))
                    kfirst = next_set_bit(rowend, L.rowend_words, kbeg, z1);
                force_end = !((rowend[(kend - 1) >> 5] >> ((kend - 1) & 31)) & 1u);
            }
            kfirst = __builtin_amdgcn_readfirstlane(kfirst);
            force_end = __builtin_amdgcn_readfirstlane((int)force_end) != 0;
        } else {
            if (wave > 0) kbeg = next_set_bit(rowend, L.rowend_words, wave * L.share - 1, z1 - 1) + 1;
            if (wave < WAVES - 1) kend = next_set_bit(rowend, L.rowend_words, (wave + 1) * L.share - 1, z1 - 1) + 1;
        }
        kbeg = __builtin_amdgcn_readfirstlane(min(kbeg, z1));
        kend = __builtin_amdgcn_readfirstlane(min(kend, z1));
    }
    const int nsteps = g2.max_deg <= 1 ? 0 : g2.max_deg <= 2 ? 1 : g2.max_deg <= 4 ? 2
                     : g2.max_deg <= 8 ? 3 : 4;

    const char* pbytes = reinterpret_cast<const char*>(p);
    char* ybytes = reinterpret_cast<char*>(y);
    const float ke_c = prm.ke_const;
    MgkAttrArgs at;
    at.outer = oattr;
    at.inner = Y.attr_inner + g2.loff + lane;
    at.inner_stride = Y.lanes_total;
    at.dim = attr_dim;
#pragma unroll
    for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a) at.scale[a] = prm.attr_scale[EK == MGK_EK_RCONV_SE ? 0 : a];

    int it = 0;
    int flag = 1;
    while (it < max_iter) {
        // ---- XMV (Alg. 2): y_ii' = sum_{j,j'} A_ij A'_i'j' kappa_e(E_ij,E'_i'j') p_jj'
        switch (nsteps) {
            case 0: xmv_pass<0, WEIGHTED, EK, ATOMIC>(ent1, ent2, rowend, pbytes, ybytes, len2, kbeg, kend, kfirst, force_end, ke_c, prm.poly_c, lane, L.z1pad, at); break;
            case 1: xmv_pass<1, WEIGHTED, EK, ATOMIC>(ent1, ent2, rowend, pbytes, ybytes, len2, kbeg, kend, kfirst, force_end, ke_c, prm.poly_c, lane, L.z1pad, at); break;
            case 2: xmv_pass<2, WEIGHTED, EK, ATOMIC>(ent1, ent2, rowend, pbytes, ybytes, len2, kbeg, kend, kfirst, force_end, ke_c, prm.poly_c, lane, L.z1pad, at); break;
            case 3: xmv_pass<3, WEIGHTED, EK, ATOMIC>(ent1, ent2, rowend, pbytes, ybytes, len2, kbeg, kend, kfirst, force_end, ke_c, prm.poly_c, lane, L.z1pad, at); break;
            default: xmv_pass<4, WEIGHTED, EK, ATOMIC>(ent1, ent2, rowend, pbytes, ybytes, len2, kbeg, kend, kfirst, force_end, ke_c, prm.poly_c, lane, L.z1pad, at); break;
        }
        __syncthreads();

        // ---- a = M p - y ; alpha = rho / p^T a
        float s_pa = 0.f;
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            const float yv = y[tid + m * NT];
            if (ATOMIC) y[tid + m * NT] = 0.f;
            zr[m] = __builtin_fmaf(Mr[m], pr[m], -yv);
            s_pa = __builtin_fmaf(pr[m], zr[m], s_pa);
        }
        const float pa = block_sum<WAVES>(s_pa, red + 32, wave, lane);
        const float alpha = rho * __builtin_amdgcn_rcpf(pa);

        // ---- x += alpha p; r -= alpha a; z = M^{-1} r; rho' = r^T z
        float s_rz2 = 0.f, s_rr = 0.f;
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            xr[m] = __builtin_fmaf(alpha, pr[m], xr[m]);
            const float rv = __builtin_fmaf(-alpha, zr[m], rr_[m]);
            rr_[m] = rv;
            const float zv = rv * __builtin_amdgcn_rcpf(Mr[m]);
            zr[m] = zv;
            s_rz2 = __builtin_fmaf(rv, zv, s_rz2);
            s_rr = __builtin_fmaf(rv, rv, s_rr);
        }
        block_sum2<WAVES>(s_rz2, s_rr, red, wave, lane);
        ++it;

        // ---- p = z + beta p (also after the last iteration, where it is not used: the
        //      loop then has a single exit and the register blocks stay in place)
        const float beta = s_rz2 * __builtin_amdgcn_rcpf(rho);
        rho = s_rz2;
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            const float pn = __builtin_fmaf(beta, pr[m], zr[m]);
            pr[m] = pn;
            p[tid + m * NT] = pn;
        }
        __syncthreads();
        if (s_rr <= thresh) { flag = 0; break; }
    }

    // ---- K = p_x^T x (Eq. 1)
    float s_k = 0.f;
#pragma unroll
    for (int m = 0; m < EPT; ++m) {
        const int idx = tid + m * NT;
        const int ic = idx < N ? idx : 0;
        const int i = (int)(((float)ic + 0.5f) * inv_n2);
        const int ip = ic - i * n2;
        s_k = __builtin_fmaf(st1[i] * st2[ip], xr[m], s_k);  // x is 0 beyond N
    }
    const float Kval = block_sum<WAVES>(s_k, red + 48, wave, lane);
    if (tid == 0) {
        out.K[job.out0] = Kval;
        if (job.out1 >= 0) out.K[job.out1] = Kval;
        if (out.iters) {
            out.iters[job.out0] = it;
            if (job.out1 >= 0) out.iters[job.out1] = it;
        }
        if (out.flags) {
            out.flags[job.out0] = flag;
            if (job.out1 >= 0) out.flags[job.out1] = flag;
        }
    }
    // ---- nodal similarity: x itself, in the original numbering of the requested pair
    if (out.nodal) {
        float* dst = out.nodal + out.nodal_off[job.out0];
        const bool swapped = job.out1 == MGK_OUT1_SWAPPED;
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            const int idx = tid + m * NT;
            if (idx < N) {
                const int i = (int)(((float)idx + 0.5f) * inv_n2);
                const int ip = idx - i * n2;
                const int oi = X.iperm[g1.voff + i], oip = Y.iperm[g2.voff + ip];
                dst[swapped ? oip * n1 + oi : oi * n2 + oip] = xr[m];
            }
        }
    }
}

template <int WAVES, int EPT, bool WEIGHTED, int EK, bool ATOMIC>
hipError_t launch_one(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkJob* jobs, int n_jobs,
                      const MgkParams& prm, size_t lds_bytes, const MgkOutputs& out, hipStream_t stream) {
    auto kern = mgk_pcg_small<WAVES, EPT, WEIGHTED, EK, ATOMIC>;
    static bool configured = false;  // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           MGK_LDS_LIMIT_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(n_jobs), dim3(WAVES * 64), lds_bytes, stream, X, Y, jobs, prm, out);
    return hipGetLastError();
}

template <int WAVES, int EPT>
hipError_t launch_we(bool weighted, bool atomic_rows, int ek, const MgkBatchDev& X,
                     const MgkBatchDev& Y, const MgkJob* jobs, int n_jobs, const MgkParams& prm,
                     size_t lds_bytes, const MgkOutputs& out, hipStream_t stream) {
#define MGK_GO(WT, EKV, AT) \
    return launch_one<WAVES, EPT, WT, EKV, AT>(X, Y, jobs, n_jobs, prm, lds_bytes, out, stream)
    if (ek == MGK_EK_SE) {
        if (weighted) { if (atomic_rows) MGK_GO(true, MGK_EK_SE, true); MGK_GO(true, MGK_EK_SE, false); }
        if (atomic_rows) MGK_GO(false, MGK_EK_SE, true);
        MGK_GO(false, MGK_EK_SE, false);
    }
    if (ek == MGK_EK_POLY) {
        if (weighted) { if (atomic_rows) MGK_GO(true, MGK_EK_POLY, true); MGK_GO(true, MGK_EK_POLY, false); }
        if (atomic_rows) MGK_GO(false, MGK_EK_POLY, true);
        MGK_GO(false, MGK_EK_POLY, false);
    }
    if (ek == MGK_EK_KRON_SE) {
        if (weighted) { if (atomic_rows) MGK_GO(true, MGK_EK_KRON_SE, true); MGK_GO(true, MGK_EK_KRON_SE, false); }
        if (atomic_rows) MGK_GO(false, MGK_EK_KRON_SE, true);
        MGK_GO(false, MGK_EK_KRON_SE, false);
    }
    if (ek == MGK_EK_RCONV_SE) {
        if (weighted) { if (atomic_rows) MGK_GO(true, MGK_EK_RCONV_SE, true); MGK_GO(true, MGK_EK_RCONV_SE, false); }
        if (atomic_rows) MGK_GO(false, MGK_EK_RCONV_SE, true);
        MGK_GO(false, MGK_EK_RCONV_SE, false);
    }
    if (ek != MGK_EK_CONST) return hipErrorInvalidValue;
    if (weighted) { if (atomic_rows) MGK_GO(true, MGK_EK_CONST, true); MGK_GO(true, MGK_EK_CONST, false); }
    if (atomic_rows) MGK_GO(false, MGK_EK_CONST, true);
    MGK_GO(false, MGK_EK_CONST, false);
#undef MGK_GO
}

}  // namespace

#ifndef MGK_SMALL_WAVES
#error "compile with -DMGK_SMALL_WAVES=<1|2|4|8|16>"
#endif

#define MGK_CAT2(a, b) a##b
#define MGK_CAT(a, b) MGK_CAT2(a, b)

// One translation unit per workgroup size keeps the build parallel; the finer register
// blocks of the four-wavefront size (6, 10, 14 elements per thread: the common size class)
// are a unit of their own, compiled with -DMGK_SMALL_FINE.
#ifdef MGK_SMALL_FINE
hipError_t mgk_launch_small_w4_fine(
    int ept, bool weighted, bool atomic_rows, const MgkBatchDev& X, const MgkBatchDev& Y,
    const MgkJob* jobs_dev, int n_jobs, const MgkParams& prm, size_t lds_bytes,
    const MgkOutputs& out, hipStream_t stream) {
    static_assert(MGK_SMALL_WAVES == 4, "finer register blocks exist for four wavefronts only");
    if (n_jobs <= 0) return hipSuccess;
    switch (ept) {
        case 6: return launch_we<4, 6>(weighted, atomic_rows, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 10: return launch_we<4, 10>(weighted, atomic_rows, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 14: return launch_we<4, 14>(weighted, atomic_rows, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        default: return hipErrorInvalidValue;
    }
}
#else
hipError_t MGK_CAT(mgk_launch_small_w, MGK_SMALL_WAVES)(
    int ept, bool weighted, bool atomic_rows, const MgkBatchDev& X, const MgkBatchDev& Y,
    const MgkJob* jobs_dev, int n_jobs, const MgkParams& prm, size_t lds_bytes,
    const MgkOutputs& out, hipStream_t stream) {
    if (n_jobs <= 0) return hipSuccess;
    constexpr int W = MGK_SMALL_WAVES;
    if constexpr (W == 16) {  // 16 x 64 x 10 elements hold a pair of 96-vertex graphs
        if (ept == 10)
            return launch_we<W, 10>(weighted, atomic_rows, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
    }
    switch (ept) {
        case 4: return launch_we<W, 4>(weighted, atomic_rows, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 12: return launch_we<W, 12>(weighted, atomic_rows, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 8: return launch_we<W, 8>(weighted, atomic_rows, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        case 16: return launch_we<W, 16>(weighted, atomic_rows, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
        default: return hipErrorInvalidValue;
    }
}
#endif
