// Owner-computes on-chip solver: one workgroup runs the whole preconditioned CG
// iteration (Alg. 1) for a pair of small graphs of bounded degree, and every lane owns
// rows of the system.
//
// On molecule-like graphs (mean degree 2) a row of the off-diagonal matrix
// (A (x) A') (.) (E (x)k E') has deg(i) deg(i') = about four entries, so the product of
// Alg. 2 is a sparse matrix-vector product with very short rows.  Here the matrix is
// kept row by row: the lane that owns element (i, i') holds the entries of its row and
// the LDS address of the element of p each one multiplies in registers, generated once
// per solve, and one product costs a gathered LDS read and a multiply-add per entry; no
// sums across lanes, no atomics.  Lanes of a wavefront run in lock step, so they must
// own rows of (nearly) equal length: the loader sorts each graph's vertices by degree
// and the kernel hands out the elements tile by tile (4 outer x 8 inner vertices of equal
// maximum degree, see mgk_internal.h), longest rows first.  The entry registers of a
// lane are one flat array over all its rows; a 64-bit mask, the same for the whole
// wavefront, marks where a row ends, there the sum is stored and cleared.  The vector
// part of the iteration works on the same lane = row assignment, so the product never
// leaves the lane except through that store.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mgk_internal.h"
#include "mgk_launch.h"
#include "mgk_wave.h"

namespace {

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// kappa_e of two prescaled labels for the kernels on scalar labels
__device__ __forceinline__ float edge_kernel_value(int kind, float e1, float e2, const MgkParams& prm) {
    const float d = e2 - e1;
    if (kind == MGK_EK_SE) return __builtin_amdgcn_exp2f(-d * d);
    if (kind == MGK_EK_POLY) return mgk_poly_kernel(d, prm.poly_c);
    return prm.ke_const;
}

// Gathered reads of p for entries T0 .. T0+3.
template <int T0, int R>
__device__ __forceinline__ void gather4(float (&pv)[4], const uint32_t (&addr)[R], const char* pbytes) {
#pragma unroll
    for (int u = 0; u < 4; ++u) pv[u] = *reinterpret_cast<const float*>(pbytes + addr[T0 + u]);
}

// Multiply-adds of entries T0 .. T0+3; where a row ends (wave-uniform mask) the sum goes
// to the lane's next y slot and is cleared.
template <int T0, int R>
__device__ __forceinline__ void use4(const float (&kap)[R], const float (&pv)[4], float& acc,
                                     uint64_t ends, uint32_t& yaddr, char* ybytes, int stride_bytes) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        acc = __builtin_fmaf(kap[T0 + u], pv[u], acc);
        if ((ends >> (T0 + u)) & 1ull) {
            *reinterpret_cast<float*>(ybytes + yaddr) = acc;
            yaddr += (uint32_t)stride_bytes;
            acc = 0.f;
        }
    }
}

// Entries T0 .. of the lane's rows (T0 < total on entry): the reads of the next four
// are issued before the four already read are used.
template <int T0, int R>
__device__ __forceinline__ void xmv_steps(const float (&kap)[R], const uint32_t (&addr)[R],
                                          const float (&pv)[4], float& acc, int total, uint64_t ends,
                                          uint32_t& yaddr, const char* pbytes, char* ybytes, int stride_bytes) {
    if constexpr (T0 + 4 < R) {
        if (T0 + 4 < total) {   // wave-uniform
            float nx[4];
            gather4<T0 + 4, R>(nx, addr, pbytes);
            use4<T0, R>(kap, pv, acc, ends, yaddr, ybytes, stride_bytes);
            xmv_steps<T0 + 4, R>(kap, addr, nx, acc, total, ends, yaddr, pbytes, ybytes, stride_bytes);
            return;
        }
    }
    use4<T0, R>(kap, pv, acc, ends, yaddr, ybytes, stride_bytes);
}

template <int W, int EPT, int R>
__global__ __launch_bounds__(W * 64) void mgk_pcg_sell(MgkBatchDev X, MgkBatchDev Y,
                                                   const MgkJob* __restrict__ jobs, MgkParams prm,
                                                   MgkOutputs out) {
    static_assert(R % 4 == 0 && R <= 64, "entry registers: a multiple of 4, one mask bit each");
    static_assert((W & (W - 1)) == 0 && W <= 16, "wavefronts: a power of two");
    extern __shared__ __align__(16) uint32_t lds[];
    constexpr int NT = W * 64;
    constexpr int NP = NT * EPT;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);

    const MgkJob job = jobs[blockIdx.x];
    const MgkGraphDesc g1 = X.graphs[job.g1];
    const MgkGraphDesc g2 = Y.graphs[job.g2];
    const MgkSellDesc s1 = X.sell_desc[job.g1];
    const MgkSellDesc s2 = Y.sell_desc[job.g2];
    const int n1 = g1.n, n2 = g2.n;
    const int G1 = (n1 + 3) >> 2, G2 = (n2 + 7) >> 3, H = G1 * G2;   // outer groups, inner groups, tiles
    const int r1 = (n1 + 7) & ~7, r2 = (n2 + 7) & ~7;                // staged records
    const MgkSellPlan L = mgk_sell_plan(n1, n2, W, EPT);

    float* p = reinterpret_cast<float*>(lds);            // L.p == 0
    float* y = reinterpret_cast<float*>(lds) + NP;
    float* x = reinterpret_cast<float*>(lds) + 2 * NP;
    uint4* vtx1 = reinterpret_cast<uint4*>(lds + L.vtx1);   // {d_i, start, label, id | deg << 16}
    uint4* nbr1 = reinterpret_cast<uint4*>(lds + L.nbr1);   // {tile-row part of the tile index, A_ij, scaled E_ij, bytes inside the tile}
    uint4* vtx2 = reinterpret_cast<uint4*>(lds + L.vtx2);
    uint4* nbr2 = reinterpret_cast<uint4*>(lds + L.nbr2);
    uint32_t* table = lds + L.table;
    uint32_t* rankof = lds + L.rankof;
    float* red = reinterpret_cast<float*>(lds + L.red);
    const int kind = prm.edge_kernel;

    // ---- stage both graphs' records; d_i = rowsum + q; labels prescaled; a neighbour at
    //      sorted position k of the outer graph contributes (k / 4) G2 to the tile index and
    //      32 (k & 3) bytes to the address, one of the inner graph k / 8 and 4 (k & 7) bytes
    {
        const uint4* sv1 = reinterpret_cast<const uint4*>(X.sell_vtx + s1.voff);
        const uint4* sn1 = reinterpret_cast<const uint4*>(X.sell_nbr + 4 * (int64_t)s1.voff);
        const uint4* sv2 = reinterpret_cast<const uint4*>(Y.sell_vtx + s2.voff);
        const uint4* sn2 = reinterpret_cast<const uint4*>(Y.sell_nbr + 4 * (int64_t)s2.voff);
        for (int k = tid; k < r1; k += NT) {
            uint4 v = sv1[k];
            v.x = __float_as_uint(__uint_as_float(v.x) + prm.q);
            vtx1[k] = v;
        }
        for (int k = tid; k < r2; k += NT) {
            uint4 v = sv2[k];
            v.x = __float_as_uint(__uint_as_float(v.x) + prm.q);
            vtx2[k] = v;
        }
        for (int k = tid; k < 4 * r1; k += NT) {
            const uint4 v = sn1[k];
            uint4 o;
            o.x = (v.x >> 2) * (uint32_t)G2;
            o.y = v.y;
            o.z = __float_as_uint((__uint_as_float(v.z) - prm.e_shift) * prm.e_scale);
            o.w = (v.x & 3u) * 32u;
            nbr1[k] = o;
        }
        for (int k = tid; k < 4 * r2; k += NT) {
            const uint4 v = sn2[k];
            uint4 o;
            o.x = v.x >> 3;
            o.y = v.y;
            o.z = __float_as_uint((__uint_as_float(v.z) - prm.e_shift) * prm.e_scale);
            o.w = (v.x & 7u) * 4u;
            nbr2[k] = o;
        }
    }
    // ---- number the tiles: class (A, B) = (largest degree in outer group U, in inner group V)
    //      in the order of mgk_sell_class_before, inside a class U-major.  table[h]: the tile
    //      with number h; rankof[U G2 + V]: where that tile's 32 elements of p start in LDS
    for (int t = tid; t < H; t += NT) {
        const int U = t / G2, V = t - U * G2;
        const int A = (int)(X.sell_vtx[s1.voff + 4 * U].id_deg >> 16);
        const int B = (int)(Y.sell_vtx[s2.voff + 8 * V].id_deg >> 16);
        int before = 0, firstU = 0, firstV = 0;
#pragma unroll
        for (int a = MGK_SELL_MAX_DEG; a >= 0; --a) {
#pragma unroll
            for (int b = MGK_SELL_MAX_DEG; b >= 0; --b)
                if (mgk_sell_class_before(a, b, A, B)) before += mgk_sell_ga(s1, a) * mgk_sell_gb(s2, b);
            if (a > A) firstU += mgk_sell_ga(s1, a);
            if (a > B) firstV += mgk_sell_gb(s2, a);
        }
        const int h = before + (U - firstU) * mgk_sell_gb(s2, B) + (V - firstV);
        table[h] = (uint32_t)U | ((uint32_t)V << 8) | ((uint32_t)A << 16) | ((uint32_t)B << 24);
        const int sl = h >> 1, m = sl / W;
        rankof[t] = (uint32_t)(m * NT + mgk_sell_wave_of(sl, W) * 64 + (h & 1) * 32) * 4u;
    }
    __syncthreads();

    // ---- this wavefront's slots: slot m holds tiles 2 s and 2 s + 1, s = m W + (wave, counted
    //      back and forth); its rows take (largest A) x (largest B) of the two tiles entries.
    //      Tiles with entries come first, so a wavefront's slots with entries are its first
    //      ones.  The schedule goes to LDS, where the fill reads it by slot number.
    const int half = lane >> 5, lu = (lane >> 3) & 3, lv = lane & 7;
    const int S = (H + 1) >> 1;   // slots of the pair
    uint32_t* sched = lds + L.sched + wave * EPT;
    int total = 0, nslots = 0;
#pragma unroll
    for (int m = 0; m < EPT; ++m) {
        const int sl = m * W + ((m & 1) ? W - 1 - wave : wave);
        const int h0 = 2 * sl;
        const uint32_t t0 = h0 < H ? table[h0] : 0u, t1 = h0 + 1 < H ? table[h0 + 1] : 0u;
        const int Aw = uniform((int)max((t0 >> 16) & 0xffu, (t1 >> 16) & 0xffu));
        const int Bw = uniform((int)max(t0 >> 24, t1 >> 24));
        if (lane == 0) sched[m] = (uint32_t)(Aw * Bw) | ((uint32_t)Bw << 8);
        total += Aw * Bw;
        if (sl < S) nslots = m + 1;
    }
    // the host only sends pairs that fit; every wavefront reports whether it does
    if (lane == 0) lds[L.misfit + wave] = (total > R || W * EPT < S) ? 1u : 0u;
    if (total > R) total = 0;   // nothing is solved then
    // wave-uniform by construction; said again so that they stay in scalar registers
    total = uniform(total);
    nslots = uniform(nslots);

    // ---- Alg. 1 set-up on the lane's elements.  M = D_x V_x^{-1}, x = 0, r = b = D_x q_x,
    //      z = M^{-1} r, p = z, rho = r^T z
    float rr_[EPT], Mr[EPT], Mi[EPT], pr[EPT];
    const float qq = prm.q * prm.q;
    const float inv_h = 1.0f / prm.h;
    float s_rz = 0.f, s_bb = 0.f;
#pragma unroll
    for (int m = 0; m < EPT; ++m) {
        const int h = 2 * (m * W + ((m & 1) ? W - 1 - wave : wave)) + half;
        const uint32_t te = h < H ? table[h] : 0u;
        const int k1 = 4 * (int)(te & 0xffu) + lu, k2 = 8 * (int)((te >> 8) & 0xffu) + lv;
        const bool ok = h < H && k1 < n1 && k2 < n2;
        const uint4 a = vtx1[ok ? k1 : 0], b = vtx2[ok ? k2 : 0];
        const bool same = a.z == b.z;
        const float dd = __uint_as_float(a.x) * __uint_as_float(b.x);
        const float bv = ok ? dd * qq : 0.f;
        const float z0 = ok ? (same ? qq : prm.h * qq) : 0.f;   // M^{-1} b = kappa_v q q'
        Mr[m] = ok ? (same ? dd : dd * inv_h) : 1.f;            // d d' / kappa_v
        Mi[m] = __builtin_amdgcn_rcpf(Mr[m]);
        rr_[m] = bv;
        pr[m] = z0;
        p[tid + m * NT] = z0;
        x[tid + m * NT] = 0.f;
        y[tid + m * NT] = 0.f;   // rows without entries are never stored by the product
        s_rz = __builtin_fmaf(bv, z0, s_rz);
        s_bb = __builtin_fmaf(bv, bv, s_bb);
    }

    // ---- fill the entry registers.  Entry t of the wavefront is (slot m, neighbour a of the
    //      lane's outer vertex, neighbour b of its inner vertex) with m, a, b wave-uniform
    //      counters; a vertex with fewer neighbours has records of weight 0 there.
    float kap[R];
    uint32_t addr[R];
    uint64_t ends = 0;
    {
        const char* n1b = reinterpret_cast<const char*>(nbr1);
        const char* n2b = reinterpret_cast<const char*>(nbr2);
        int m = 0, a = 0, b = 0, Bcur = 1, left = 0;
        uint32_t base1 = 0, base2 = 0;   // byte offsets of the lane's outer / inner neighbour records
        float live = 0.f;                // 0 on lanes whose half of the slot has no tile
        auto load_slot = [&](int mm) {   // mm wave-uniform
            const uint32_t sc = (uint32_t)uniform((int)sched[mm]);
            left = (int)(sc & 0xffu);
            Bcur = (int)(sc >> 8);
            const int h = 2 * (mm * W + ((mm & 1) ? W - 1 - wave : wave)) + half;
            const uint32_t te = h < H ? table[h] : 0u;
            base1 = (4u * (te & 0xffu) + (uint32_t)lu) * 64u;
            base2 = (8u * ((te >> 8) & 0xffu) + (uint32_t)lv) * 64u;
            live = h < H ? 1.f : 0.f;
        };
        if (total > 0) load_slot(0);
        uint4 o1 = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int t = 0; t < R; ++t) {
            if (t < total) {   // wave-uniform, as are the counters
                m = uniform(m);
                a = uniform(a);
                b = uniform(b);
                left = uniform(left);
                Bcur = uniform(Bcur);
                if (b == 0) o1 = *reinterpret_cast<const uint4*>(n1b + base1 + (uint32_t)a * 16u);
                const uint4 o2 = *reinterpret_cast<const uint4*>(n2b + base2 + (uint32_t)b * 16u);
                const float w12 = __uint_as_float(o1.y) * __uint_as_float(o2.y) * live;   // 0 past either degree
                kap[t] = w12 * edge_kernel_value(kind, __uint_as_float(o1.z), __uint_as_float(o2.z), prm);
                addr[t] = rankof[o1.x + o2.x] + o1.w + o2.w;
                ++b;
                if (b == Bcur) { b = 0; ++a; }
                if (--left == 0) {
                    ends |= 1ull << t;
                    a = 0;
                    b = 0;
                    ++m;
                    if (t + 1 < total) load_slot(m);
                }
            } else {
                kap[t] = 0.f;
                addr[t] = 0u;
            }
        }
    }

    ends = ((uint64_t)(uint32_t)uniform((int)(uint32_t)(ends >> 32)) << 32) | (uint32_t)uniform((int)(uint32_t)ends);

    block_sum2<W>(s_rz, s_bb, red, wave, lane);   // barrier inside: p, x and the fit reports are complete
    {
        uint32_t misfit = 0u;
#pragma unroll
        for (int w = 0; w < W; ++w) misfit |= lds[L.misfit + w];
        misfit = (uint32_t)uniform((int)misfit);
        if (misfit != 0u) {   // the same in every thread: value NaN, flag 2, nothing solved in part
            if (tid == 0) {
                const float bad = __builtin_nanf("");
                out.K[job.out0] = bad;
                if (job.out1 >= 0) out.K[job.out1] = bad;
                if (out.iters) { out.iters[job.out0] = 0; if (job.out1 >= 0) out.iters[job.out1] = 0; }
                if (out.flags) { out.flags[job.out0] = 2; if (job.out1 >= 0) out.flags[job.out1] = 2; }
            }
            return;
        }
    }
    float rho = s_rz;
    const float thresh = prm.rtol2 * s_bb;
    int max_iter = prm.max_iter;
    if (max_iter <= 0) max_iter = min(2 * n1 * n2, 1000);

    const char* pbytes = reinterpret_cast<const char*>(p);
    char* ybytes = reinterpret_cast<char*>(y);

    int it = 0;
    int flag = 1;
    uint32_t ends_lo = (uint32_t)ends, ends_hi = (uint32_t)(ends >> 32);
    while (it < max_iter) {
        // The row-end tests below are a bit test and a branch on scalar registers each.  The
        // empty statement keeps them inside the loop: hoisted, they become one 64-bit lane
        // mask per entry, more than the scalar register file holds.
        asm volatile("" : "+s"(ends_lo), "+s"(ends_hi), "+s"(total));
        const uint64_t ends_now = ((uint64_t)ends_hi << 32) | ends_lo;
        // ---- XMV: y_ii' = sum_{j,j'} A_ij A'_i'j' kappa_e(E_ij,E'_i'j') p_jj', one row per slot
        if (total > 0) {
            float acc = 0.f, pv[4];
            uint32_t yaddr = (uint32_t)tid * 4u;   // the rows with entries are the lane's first slots
            gather4<0, R>(pv, addr, pbytes);
            xmv_steps<0, R>(kap, addr, pv, acc, total, ends_now, yaddr, pbytes, ybytes, NT * 4);
        }
        // ---- a = M p - y ; alpha = rho / p^T a   (y was written by this very lane)
        float s_pa = 0.f;
#pragma unroll
        for (int m = 0; m < EPT; ++m)
            if (m < nslots) {   // wave-uniform
                const float av = __builtin_fmaf(Mr[m], pr[m], -y[tid + m * NT]);
                s_pa = __builtin_fmaf(pr[m], av, s_pa);
            }
        const float pa = block_sum<W>(s_pa, red + 32, wave, lane);
        const float alpha = rho * __builtin_amdgcn_rcpf(pa);

        // ---- x += alpha p; r -= alpha a; z = M^{-1} r; rho' = r^T z.  a is formed again from
        //      y (a register per slot less than keeping it across the sum)
        float s_rz2 = 0.f, s_rr = 0.f;
#pragma unroll
        for (int m = 0; m < EPT; ++m)
            if (m < nslots) {
                const float av = __builtin_fmaf(Mr[m], pr[m], -y[tid + m * NT]);
                x[tid + m * NT] = __builtin_fmaf(alpha, pr[m], x[tid + m * NT]);
                const float rv = __builtin_fmaf(-alpha, av, rr_[m]);
                rr_[m] = rv;
                const float zv = rv * Mi[m];
                s_rz2 = __builtin_fmaf(rv, zv, s_rz2);
                s_rr = __builtin_fmaf(rv, rv, s_rr);
            }
        block_sum2<W>(s_rz2, s_rr, red, wave, lane);
        ++it;

        // ---- p = z + beta p
        const float beta = s_rz2 * __builtin_amdgcn_rcpf(rho);
        rho = s_rz2;
#pragma unroll
        for (int m = 0; m < EPT; ++m)
            if (m < nslots) {
                pr[m] = __builtin_fmaf(beta, pr[m], rr_[m] * Mi[m]);
                p[tid + m * NT] = pr[m];
            }
        __syncthreads();
        if (s_rr <= thresh) { flag = 0; break; }
    }

    // ---- K = p_x^T x (Eq. 1)
    float s_k = 0.f;
#pragma unroll
    for (int m = 0; m < EPT; ++m) {
        const int h = 2 * (m * W + ((m & 1) ? W - 1 - wave : wave)) + half;
        const uint32_t te = h < H ? table[h] : 0u;
        const int k1 = 4 * (int)(te & 0xffu) + lu, k2 = 8 * (int)((te >> 8) & 0xffu) + lv;
        const bool ok = h < H && k1 < n1 && k2 < n2;
        const float st = ok ? __uint_as_float(vtx1[k1].y) * __uint_as_float(vtx2[k2].y) : 0.f;
        s_k = __builtin_fmaf(st, x[tid + m * NT], s_k);
    }
    const float Kval = block_sum<W>(s_k, red + 48, wave, lane);
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
            const int h = 2 * (m * W + ((m & 1) ? W - 1 - wave : wave)) + half;
            const uint32_t te = h < H ? table[h] : 0u;
            const int k1 = 4 * (int)(te & 0xffu) + lu, k2 = 8 * (int)((te >> 8) & 0xffu) + lv;
            if (h < H && k1 < n1 && k2 < n2) {
                const int i = (int)(vtx1[k1].w & 0xffffu), i2 = (int)(vtx2[k2].w & 0xffffu);   // stored order
                const int oi = X.iperm[g1.voff + i], oi2 = Y.iperm[g2.voff + i2];
                dst[swapped ? oi2 * n1 + oi : oi * n2 + oi2] = x[tid + m * NT];
            }
        }
    }
}

template <int W, int EPT, int R>
hipError_t launch_one(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkJob* jobs, int n_jobs,
                      const MgkParams& prm, size_t lds_bytes, const MgkOutputs& out, hipStream_t stream) {
    auto kern = mgk_pcg_sell<W, EPT, R>;
    static bool configured = false;  // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           MGK_LDS_LIMIT_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(n_jobs), dim3(W * 64), lds_bytes, stream, X, Y, jobs, prm, out);
    return hipGetLastError();
}

}  // namespace

#if !defined(MGK_SELL_WAVES)
#error "compile with -DMGK_SELL_WAVES=<4|8|16>"
#endif

#define MGK_CAT2(a, b) a##b
#define MGK_CAT(a, b) MGK_CAT2(a, b)
#define MGK_SELL_SHAPES_OF2(W) MGK_SELL_SHAPES_W##W
#define MGK_SELL_SHAPES_OF(W) MGK_SELL_SHAPES_OF2(W)

// One translation unit per workgroup size keeps the build parallel.
hipError_t MGK_CAT(mgk_launch_sell_w, MGK_SELL_WAVES)(
    int ept, int regs, const MgkBatchDev& X, const MgkBatchDev& Y, const MgkJob* jobs_dev, int n_jobs,
    const MgkParams& prm, size_t lds_bytes, const MgkOutputs& out, hipStream_t stream) {
    if (n_jobs <= 0) return hipSuccess;
#define MGK_CASE(WW, E, RR) \
    if (ept == E && regs == RR) return launch_one<WW, E, RR>(X, Y, jobs_dev, n_jobs, prm, lds_bytes, out, stream);
    MGK_SELL_SHAPES_OF(MGK_SELL_WAVES)(MGK_CASE)
#undef MGK_CASE
    return hipErrorInvalidValue;
}
