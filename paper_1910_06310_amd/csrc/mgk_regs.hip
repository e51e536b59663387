// Register-resident on-chip solver: one workgroup of four or eight wavefronts
// runs the whole preconditioned CG iteration (Alg. 1) for one graph pair whose
// off-diagonal matrix fits in the register file.
//
// Alg. 2 regenerates the entries A_ij A'_i'j' kappa_e(E_ij, E'_i'j') in every
// iteration because the N x N matrix cannot be kept in memory.  For a pair of
// small graphs the nonzero ones (nnz x nnz' of them, a few thousand) do fit in
// the 512 KB of vector registers of a compute unit, so they are generated once
// per solve, straight into registers, and never touch memory at all: each lane
// owns one nonzero (i', j') of the inner graph per 64-lane chunk, each
// wavefront owns a run of whole rows of the outer graph, and register
// kap[c][k] of a lane holds the entry for the wavefront's k-th outer nonzero
// and the lane's inner nonzero of chunk c.  One XMV then costs, per entry, an
// address add, a gathered LDS read of p_jj' and a multiply-add; the loop over k
// is unrolled completely so that the register index is static.  The sum over
// the lanes of an inner row at the end of an outer row (DPP shift-and-add) and
// the vector part of the iteration follow the streaming kernel; the edge base
// kernel appears only in the one-off fill of the registers, so every base
// kernel runs the same iteration.  x is kept in LDS beside p and y (it is
// touched once per iteration), r, M, the owner's p and z in registers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mgk_internal.h"
#include "mgk_launch.h"
#include "mgk_wave.h"

namespace {

// value of v in lane k (k a compile-time constant after unrolling)
__device__ __forceinline__ uint32_t lane_value(uint32_t v, int k) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, k);
}
__device__ __forceinline__ float lane_value(float v, int k) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), k));
}

// The loops over the wave's outer nonzeros are unrolled by template recursion,
// four nonzeros per step, so that every index into the register array kap is a
// compile-time constant.

// Matrix entries of outer nonzeros K0 .. SMAX-1 (lanes K0.. of e1s / l1) against this
// lane's inner nonzeros: square-exponential kernel on prescaled labels,
// exp2(log2 A + log2 A' - (e - e')^2).  Lanes of e1s past the wave's run hold a huge
// label and idle inner slots hold l2 = -inf, so both give exactly 0.
template <int K0, int SMAX, int C, bool WEIGHTED>
__device__ __forceinline__ void fill_se(float (&kap)[C][SMAX], int S, const float (&e2s)[C],
                                        const float (&l2)[C], float e1s, float l1) {
    if constexpr (K0 < SMAX) {
        if (K0 < S) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float e1 = lane_value(e1s, K0 + u);
                const float la = WEIGHTED ? lane_value(l1, K0 + u) : 0.f;
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const float d = e2s[c] - e1;
                    kap[c][K0 + u] = __builtin_amdgcn_exp2f(__builtin_fmaf(-d, d, WEIGHTED ? l2[c] + la : l2[c]));
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < C; ++c) kap[c][K0 + u] = 0.f;
        }
        fill_se<K0 + 4, SMAX, C, WEIGHTED>(kap, S, e2s, l2, e1s, l1);
    }
}

// the same for the constant edge kernel: A_ij * (A'_i'j' kappa_e); w1 is 0 past the run
template <int K0, int SMAX, int C>
__device__ __forceinline__ void fill_const(float (&kap)[C][SMAX], int S, const float (&w2c)[C], float w1) {
    if constexpr (K0 < SMAX) {
        if (K0 < S) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float wa = lane_value(w1, K0 + u);
#pragma unroll
                for (int c = 0; c < C; ++c) kap[c][K0 + u] = w2c[c] * wa;
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < C; ++c) kap[c][K0 + u] = 0.f;
        }
        fill_const<K0 + 4, SMAX, C>(kap, S, w2c, w1);
    }
}

// compact polynomial kernel on labels prescaled by 1 / rho; wprod = A_ij A'_i'j' per lane
// pair (0 on idle slots and past the run)
template <int K0, int SMAX, int C>
__device__ __forceinline__ void fill_poly(float (&kap)[C][SMAX], int S, const float (&e2s)[C],
                                          const float (&w2)[C], float e1s, float w1, const float* pc) {
    if constexpr (K0 < SMAX) {
        if (K0 < S) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float e1 = lane_value(e1s, K0 + u);
                const float wa = lane_value(w1, K0 + u);
#pragma unroll
                for (int c = 0; c < C; ++c)
                    kap[c][K0 + u] = mgk_poly_kernel(e2s[c] - e1, pc) * (w2[c] * wa);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < C; ++c) kap[c][K0 + u] = 0.f;
        }
        fill_poly<K0 + 4, SMAX, C>(kap, S, e2s, w2, e1s, w1, pc);
    }
}

// Kernels over labels with D attributes, each prescaled by sqrt(log2(e) / (2 l_a^2)).
// RCONV false: Kronecker product of square exponentials, exp2(log2 A + log2 A' -
// sum_a (e_a - e'_a)^2), with l1 / l2 the log2 weights (-inf on idle slots; lanes past
// the run carry a huge attribute 0).  RCONV true: (A A' / D^2) sum_a sum_b
// exp2(-(e_a - e'_b)^2), with l1 / l2 the weights themselves (0 where there is no entry).
template <int K0, int SMAX, int C, bool RCONV>
__device__ __forceinline__ void fill_attr(float (&kap)[C][SMAX], int S, int D,
                                          const float (&e2a)[C][MGK_MAX_LABEL_DIM], const float (&l2)[C],
                                          const float (&e1a)[MGK_MAX_LABEL_DIM], float l1) {
    if constexpr (K0 < SMAX) {
        if (K0 < S) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float e1[MGK_MAX_LABEL_DIM];
#pragma unroll
                for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a) e1[a] = a < D ? lane_value(e1a[a], K0 + u) : 0.f;
                const float la = lane_value(l1, K0 + u);
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    if (RCONV) {
                        float sum = 0.f;
#pragma unroll
                        for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
#pragma unroll
                            for (int b = 0; b < MGK_MAX_LABEL_DIM; ++b)
                                if (a < D && b < D) {
                                    const float d = e2a[c][a] - e1[b];
                                    sum += __builtin_amdgcn_exp2f(-d * d);
                                }
                        kap[c][K0 + u] = sum * (l2[c] * la);
                    } else {
                        float t = l2[c] + la;
#pragma unroll
                        for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a)
                            if (a < D) {
                                const float d = e2a[c][a] - e1[a];
                                t = __builtin_fmaf(-d, d, t);
                            }
                        kap[c][K0 + u] = __builtin_amdgcn_exp2f(t);
                    }
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < C; ++c) kap[c][K0 + u] = 0.f;
        }
        fill_attr<K0 + 4, SMAX, C, RCONV>(kap, S, D, e2a, l2, e1a, l1);
    }
}

// per-lane constants of the inner nonzeros, one set per chunk
template <int C>
struct InnerLanes {
    uint32_t jp[C];                   // byte offset of column j' in a row of p
    uint32_t ip[C];                   // byte offset of row i' in a row of y; lanes that are not the
                                      // last of their run point the same distance into the dump area
    float m1[C], m2[C];               // 1 if the lane is at least that far into its run, else 0
};

// Gathered reads of p for outer nonzeros K0 .. K0+3 (lanes past the wave's run hold
// offset 0, so the reads stay inside p).
template <int K0, int C, int SMAX>
__device__ __forceinline__ void gather4(float (&pv)[4][C], const InnerLanes<C>& in,
                                        const uint32_t (&s_poff)[SMAX], const char* pbytes) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint32_t po = s_poff[K0 + u];
#pragma unroll
        for (int c = 0; c < C; ++c)
            pv[u][c] = *reinterpret_cast<const float*>(pbytes + (po + in.jp[c]));
    }
}

// acc[c] += m1 * (acc[c] one lane down) and then += m2 * (two lanes down), inside rows of
// 16 lanes: the sum over an inner row of at most 4 nonzeros arrives in its last lane.
// The DPP reads need two wait states after the write of the register they read; with two
// chunks the steps of one chunk fill part of the other's.
template <int C>
__device__ __forceinline__ void row_sums(float (&acc)[C], const InnerLanes<C>& in) {
    static_assert(C == 1 || C == 2, "one or two chunks");
    if constexpr (C == 1) {
        asm volatile(
            "s_nop 1\n\tv_fmac_f32_dpp %0, %0, %1 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "s_nop 1\n\tv_fmac_f32_dpp %0, %0, %2 row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1"
            : "+v"(acc[0])
            : "v"(in.m1[0]), "v"(in.m2[0]));
    } else {
        asm volatile(
            "s_nop 1\n\tv_fmac_f32_dpp %0, %0, %2 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %1, %1, %3 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "s_nop 0\n\tv_fmac_f32_dpp %0, %0, %4 row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %1, %1, %5 row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1"
            : "+v"(acc[0]), "+v"(acc[1])
            : "v"(in.m1[0]), "v"(in.m1[1]), "v"(in.m2[0]), "v"(in.m2[1]));
    }
}

// Multiply-add of outer nonzeros K0 .. K0+3 (p values already read into pv); at the
// end of an outer row (wave-uniform test) each inner row is summed over its lanes
// (rows of at most 4 nonzeros: two shift-and-add steps) and y_ii' stored from the
// last lane of the row.
template <int K0, int SMAX, int C>
__device__ __forceinline__ void use4(const float (&kap)[C][SMAX], const InnerLanes<C>& in,
                                     float (&acc)[C], const float (&pv)[4][C], uint64_t rowmask,
                                     uint32_t v_yoff, char* ybytes) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int c = 0; c < C; ++c) acc[c] = __builtin_fmaf(kap[c][K0 + u], pv[u][c], acc[c]);
        if ((rowmask >> (K0 + u)) & 1ull) {
            const uint32_t yo = lane_value(v_yoff, K0 + u);
            row_sums<C>(acc, in);
#pragma unroll
            for (int c = 0; c < C; ++c) {
                // every lane stores: the last lane of an inner row to y_ii', the others to
                // the same place in a dump area behind y (no divergent region)
                *reinterpret_cast<float*>(ybytes + (yo + in.ip[c])) = acc[c];
                acc[c] = 0.f;
            }
        }
    }
}

// XMV steps K0 .. (K0 < S on entry): the reads of p for the next four outer
// nonzeros are issued before the four already read are used, so that the LDS
// latency overlaps the arithmetic.
template <int K0, int SMAX, int C>
__device__ __forceinline__ void xmv_steps(const float (&kap)[C][SMAX], const InnerLanes<C>& in,
                                          float (&acc)[C], const float (&pv)[4][C], int S,
                                          uint64_t rowmask, const uint32_t (&s_poff)[SMAX],
                                          uint32_t v_yoff, const char* pbytes, char* ybytes) {
    if constexpr (K0 + 4 < SMAX) {
        if (K0 + 4 < S) {   // wave-uniform
            float nx[4][C];
            gather4<K0 + 4, C, SMAX>(nx, in, s_poff, pbytes);
            use4<K0, SMAX, C>(kap, in, acc, pv, rowmask, v_yoff, ybytes);
            xmv_steps<K0 + 4, SMAX, C>(kap, in, acc, nx, S, rowmask, s_poff, v_yoff, pbytes, ybytes);
            return;
        }
    }
    use4<K0, SMAX, C>(kap, in, acc, pv, rowmask, v_yoff, ybytes);
}

template <int W, int SMAX, int EPT, int C>
__global__ __launch_bounds__(W * 64) void mgk_pcg_regs(MgkBatchDev X, MgkBatchDev Y,
                                                   const MgkJob* __restrict__ jobs, MgkParams prm,
                                                   MgkOutputs out, int weighted) {
    extern __shared__ __align__(16) uint32_t lds[];
    constexpr int NT = W * 64;
    constexpr int NP = NT * EPT;   // p, y and x are padded to the register blocks
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const MgkJob job = jobs[blockIdx.x];
    const MgkGraphDesc g1 = X.graphs[job.g1];
    const MgkGraphDesc g2 = Y.graphs[job.g2];
    const int n1 = g1.n, n2 = g2.n, N = n1 * n2, z1 = g1.nnz, len2 = g2.lane_len;
    const MgkRegsPlan L = mgk_regs_plan(n1, n2, W, EPT);

    float* p = reinterpret_cast<float*>(lds);          // L.p == 0
    float* y = reinterpret_cast<float*>(lds) + NP;     // L.y == NP
    float* x = reinterpret_cast<float*>(lds) + 2 * NP; // L.x == 2 NP; 3 NP .. 4 NP: dump area
    float* dq1 = reinterpret_cast<float*>(lds + L.vtx1);   // d_i = rowsum + q
    float* st1 = dq1 + n1;                                 // start probability
    int* lb1 = reinterpret_cast<int*>(st1 + n1);           // vertex label
    float* dq2 = reinterpret_cast<float*>(lds + L.vtx2);
    float* st2 = dq2 + n2;
    int* lb2 = reinterpret_cast<int*>(st2 + n2);
    float* red = reinterpret_cast<float*>(lds + L.red);

    // ---- stage per-vertex data; clear y (entries no row pair reaches stay 0) ----
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
#pragma unroll
    for (int m = 0; m < EPT; ++m) y[tid + m * NT] = 0.f;
    if (tid == 0) red[63] = 0.f;

    // ---- this wave's outer rows: whole rows, divided at load so that the most loaded
    //      wavefront is as light as possible
    const int32_t* split = X.regs_split + (int64_t)job.g1 * MGK_REGS_SPLIT_STRIDE + (W == 8 ? MGK_REGS_SPLIT_W8 : 0);
    const int rbeg = split[wave], rend = split[wave + 1];
    int kbeg = rbeg < n1 ? X.rowptr[g1.voff + rbeg] : z1;
    int kend = rend < n1 ? X.rowptr[g1.voff + rend] : z1;
    kbeg = __builtin_amdgcn_readfirstlane(kbeg);
    kend = __builtin_amdgcn_readfirstlane(kend);
    // The host only sends pairs whose runs fit the unrolled loop.  Should one not fit, the
    // solve goes on with the part that does (so that every loop stays in bounds) and the
    // pair's outputs are replaced at the end: value NaN, flag 2, never a value computed
    // with part of the matrix.  red[63] is cleared before the staging barrier below.
    const bool misfit = kend - kbeg > SMAX;
    const int S = min(kend - kbeg, SMAX);

    // lane l < S holds the wave's l-th outer nonzero
    const bool live1 = lane < S;
    const MgkEntry o = live1 ? X.list_outer[g1.zoff + kbeg + lane] : MgkEntry{0u, 0u, 0u, 0u};
    const uint32_t v_poff = o.y * (uint32_t)(n2 * 4);   // byte offset of row j of p
    const uint32_t v_yoff = o.x * (uint32_t)(n2 * 4);   // byte offset of row i of y
    const uint64_t rowmask = __ballot(live1 && (o.w >> 31) != 0u);
    const float w1 = live1 ? __uint_as_float(o.w & 0x7fffffffu) : 0.f;
    // lanes past the run: a label so far away that kappa_e underflows to exactly 0
    const float e1s = live1 ? (__uint_as_float(o.z) - prm.e_shift) * prm.e_scale : 1e18f;
    const float l1 = weighted ? __log2f(live1 ? w1 : 1.f) : 0.f;

    // ---- inner nonzeros of this lane, one per chunk; matrix entries into registers --
    InnerLanes<C> in;
    float kap[C][SMAX];
    {
        float e2s[C], l2[C], w2c[C], w2r[C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int slot = c * 64 + lane;
            const MgkEntry e = slot < len2 ? Y.list_inner[g2.loff + slot] : MgkEntry{0u, 0u, 0u, 0u};
            in.ip[c] = (e.x & 0xfffffu) * 4u + ((e.x >> 31) != 0u ? 0u : (uint32_t)(2 * NP * 4));
            in.jp[c] = e.y * 4u;
            const uint32_t rank = (e.x >> 20) & 0xffu;
            in.m1[c] = rank >= 1 ? 1.f : 0.f;
            in.m2[c] = rank >= 2 ? 1.f : 0.f;
            const float w2 = __uint_as_float(e.w);   // 0 on idle slots
            e2s[c] = (__uint_as_float(e.z) - prm.e_shift) * prm.e_scale;
            l2[c] = w2 > 0.f ? (weighted ? __log2f(w2) : 0.f) : -__builtin_inff();
            w2c[c] = w2 * prm.ke_const;
            w2r[c] = w2;
        }
        if (prm.edge_kernel == MGK_EK_SE) {
            if (weighted) fill_se<0, SMAX, C, true>(kap, S, e2s, l2, e1s, l1);
            else fill_se<0, SMAX, C, false>(kap, S, e2s, l2, e1s, l1);
        } else if (prm.edge_kernel == MGK_EK_CONST) {
            fill_const<0, SMAX, C>(kap, S, w2c, w1);
        } else if (prm.edge_kernel == MGK_EK_POLY) {
            fill_poly<0, SMAX, C>(kap, S, e2s, w2r, e1s, w1, prm.poly_c);
        } else {
            // labels with D attributes, from the attribute planes of the two lists
            const int D = prm.label_dim;
            const bool rconv = prm.edge_kernel == MGK_EK_RCONV_SE;
            float e1a[MGK_MAX_LABEL_DIM], e2a[C][MGK_MAX_LABEL_DIM], f2[C];
#pragma unroll
            for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a) {
                const bool on = a < D;
                const float raw1 = on && live1 ? X.attr_outer[(int64_t)a * X.nnz_total + g1.zoff + kbeg + lane] : 0.f;
                e1a[a] = raw1 * prm.attr_scale[a];
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const int slot = c * 64 + lane;
                    const float raw2 = on && slot < len2 ? Y.attr_inner[(int64_t)a * Y.lanes_total + g2.loff + slot] : 0.f;
                    e2a[c][a] = raw2 * prm.attr_scale[a];
                }
            }
            if (rconv) {
                const float inv = 1.0f / (float)(D * D);
#pragma unroll
                for (int c = 0; c < C; ++c) f2[c] = w2r[c] * inv;   // 0 on idle slots
                fill_attr<0, SMAX, C, true>(kap, S, D, e2a, f2, e1a, w1);   // w1 is 0 past the run
            } else {
                if (!live1) e1a[0] = 1e18f;   // past the run: kappa_e underflows to exactly 0
                const float la = weighted ? __log2f(live1 ? w1 : 1.f) : 0.f;
                fill_attr<0, SMAX, C, false>(kap, S, D, e2a, l2, e1a, la);
            }
        }
    }
    __syncthreads();   // per-vertex data staged
    if (misfit && lane == 0) red[63] = 1.f;   // wave-uniform, after the barrier that follows the clearing

    // ---- Alg. 1 set-up: M = D_x V_x^{-1}, x = 0, r = b = D_x q_x, z = M^{-1} r,
    //      p = z, rho = r^T z ----------------------------------------------------
    float rr_[EPT], Mr[EPT], pr[EPT], zr[EPT];   // x stays in LDS: touched once per iteration
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
        const int i2 = ic - i * n2;
        const bool same = lb1[i] == lb2[i2];
        const float dd = dq1[i] * dq2[i2];
        const float b = ok ? dd * qq : 0.f;
        const float z0 = ok ? (same ? qq : prm.h * qq) : 0.f;  // M^{-1} b = kappa_v q q'
        Mr[m] = ok ? (same ? dd : dd * inv_h) : 1.f;           // d d' / kappa_v
        rr_[m] = b;
        pr[m] = z0;
        p[idx] = z0;                                           // padding holds 0
        x[idx] = 0.f;
        s_rz = __builtin_fmaf(b, z0, s_rz);
        s_bb = __builtin_fmaf(b, b, s_bb);
    }
    block_sum2<W>(s_rz, s_bb, red, wave, lane);
    float rho = s_rz;
    const float thresh = prm.rtol2 * s_bb;
    int max_iter = prm.max_iter;
    if (max_iter <= 0) max_iter = min(2 * N, 1000);
    __syncthreads();  // p and the cleared y are complete

    const char* pbytes = reinterpret_cast<const char*>(p);
    char* ybytes = reinterpret_cast<char*>(y);
    // byte offset of row j of p for each of the wave's outer nonzeros, in scalar
    // registers for the whole solve (entries past the run read row 0); the offsets of the
    // rows of y, needed at row ends only, stay in lanes: the scalar file does not hold both
    uint32_t s_poff[SMAX];
#pragma unroll
    for (int k = 0; k < SMAX; ++k) s_poff[k] = lane_value(v_poff, k);

    int it = 0;
    int flag = 1;
    while (it < max_iter) {
        // ---- XMV: y_ii' = sum_{j,j'} A_ij A'_i'j' kappa_e(E_ij,E'_i'j') p_jj', entries from registers
        if (S > 0) {
            float acc[C], pv[4][C];
#pragma unroll
            for (int c = 0; c < C; ++c) acc[c] = 0.f;
            gather4<0, C, SMAX>(pv, in, s_poff, pbytes);
            xmv_steps<0, SMAX, C>(kap, in, acc, pv, S, rowmask, s_poff, v_yoff, pbytes, ybytes);
        }
        __syncthreads();

        // ---- a = M p - y ; alpha = rho / p^T a
        float s_pa = 0.f;
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            zr[m] = __builtin_fmaf(Mr[m], pr[m], -y[tid + m * NT]);
            s_pa = __builtin_fmaf(pr[m], zr[m], s_pa);
        }
        const float pa = block_sum<W>(s_pa, red + 32, wave, lane);
        const float alpha = rho * __builtin_amdgcn_rcpf(pa);

        // ---- x += alpha p; r -= alpha a; z = M^{-1} r; rho' = r^T z
        float s_rz2 = 0.f, s_rr = 0.f;
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            x[tid + m * NT] = __builtin_fmaf(alpha, pr[m], x[tid + m * NT]);
            const float rv = __builtin_fmaf(-alpha, zr[m], rr_[m]);
            rr_[m] = rv;
            const float zv = rv * __builtin_amdgcn_rcpf(Mr[m]);   // 1/M is hoisted by the compiler
            zr[m] = zv;
            s_rz2 = __builtin_fmaf(rv, zv, s_rz2);
            s_rr = __builtin_fmaf(rv, rv, s_rr);
        }
        block_sum2<W>(s_rz2, s_rr, red, wave, lane);
        ++it;

        // ---- p = z + beta p (also after the last iteration, where it is not used: the
        //      loop then has a single exit and the register blocks stay in place)
        const float beta = s_rz2 * __builtin_amdgcn_rcpf(rho);
        rho = s_rz2;
        // written as an instruction with the register of p as destination: the compiler's
        // own choice accumulates into the register of z and copies it back, EPT moves per
        // iteration
        float beta_v = beta;
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            asm("v_fma_f32 %0, %1, %0, %2" : "+v"(pr[m]) : "v"(beta_v), "v"(zr[m]));
            p[tid + m * NT] = pr[m];
        }
        __syncthreads();
        if (s_rr <= thresh) { flag = 0; break; }
    }

    // ---- K = p_x^T x (Eq. 1); every thread reads back the x elements it wrote
    float s_k = 0.f;
    if (X.uniform_start && Y.uniform_start) {   // p_x = 1 / (n n') everywhere
#pragma unroll
        for (int m = 0; m < EPT; ++m) s_k += x[tid + m * NT];   // x is 0 beyond N
        s_k *= inv_n2 * (1.0f / (float)n1);
    } else {
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            const int idx = tid + m * NT;
            const int ic = idx < N ? idx : 0;
            const int i = (int)(((float)ic + 0.5f) * inv_n2);
            const int i2 = ic - i * n2;
            s_k = __builtin_fmaf(st1[i] * st2[i2], x[idx], s_k);  // x is 0 beyond N
        }
    }
    float Kval = block_sum<W>(s_k, red + 48, wave, lane);
    if (tid == 0) {
        if (red[63] != 0.f) {   // some wavefront's run did not fit
            Kval = __builtin_nanf("");
            flag = 2;
        }
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
                const int i2 = idx - i * n2;
                const int oi = X.iperm[g1.voff + i], oi2 = Y.iperm[g2.voff + i2];
                dst[swapped ? oi2 * n1 + oi : oi * n2 + oi2] = x[idx];
            }
        }
    }
}

template <int W, int SMAX, int EPT, int C>
hipError_t launch_one(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkJob* jobs, int n_jobs,
                      const MgkParams& prm, bool weighted, size_t lds_bytes, const MgkOutputs& out,
                      hipStream_t stream) {
    auto kern = mgk_pcg_regs<W, SMAX, EPT, C>;
    static bool configured = false;  // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           MGK_LDS_LIMIT_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(n_jobs), dim3(W * 64), lds_bytes, stream, X, Y, jobs, prm, out,
                       weighted ? 1 : 0);
    return hipGetLastError();
}

}  // namespace

#if !defined(MGK_REGS_CHUNKS) || !defined(MGK_REGS_WAVES)
#error "compile with -DMGK_REGS_WAVES=<4|8> -DMGK_REGS_CHUNKS=<1|2>"
#endif

#define MGK_CAT2(a, b, c, d) a##b##c##d
#define MGK_CAT(a, b, c, d) MGK_CAT2(a, b, c, d)

// One translation unit per (wavefronts, chunk count) keeps the build parallel.
hipError_t MGK_CAT(mgk_launch_regs_w, MGK_REGS_WAVES, _c, MGK_REGS_CHUNKS)(
    int ept, bool weighted, const MgkBatchDev& X, const MgkBatchDev& Y, const MgkJob* jobs_dev,
    int n_jobs, const MgkParams& prm, size_t lds_bytes, const MgkOutputs& out, hipStream_t stream) {
    if (n_jobs <= 0) return hipSuccess;
    constexpr int C = MGK_REGS_CHUNKS;
    constexpr int W = MGK_REGS_WAVES;
    constexpr int SMAX = W == 4 ? MGK_REGS_SMAX_W4 : MGK_REGS_SMAX_W8;
    switch (ept) {
#define MGK_CASE(E) \
    case E: return launch_one<W, SMAX, E, C>(X, Y, jobs_dev, n_jobs, prm, weighted, lds_bytes, out, stream);
        MGK_CASE(1) MGK_CASE(2) MGK_CASE(3) MGK_CASE(4) MGK_CASE(5) MGK_CASE(6) MGK_CASE(7) MGK_CASE(8)
#undef MGK_CASE
        default: return hipErrorInvalidValue;
    }
}
