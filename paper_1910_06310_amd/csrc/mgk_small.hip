// On-chip solver: one workgroup runs the whole preconditioned CG iteration
// (Alg. 1) for one graph pair with every vector resident in LDS.
//
// The off-diagonal product of Alg. 1 (the XMV of Alg. 2) is formed on the fly:
// the inner graph's nonzeros live one per lane, the outer graph's nonzeros are
// streamed from LDS as wave-uniform operands, and each (outer nonzero, inner
// nonzero) pair costs one kappa_e evaluation, one gathered read of p_jj' and
// one fused multiply-add.  Contributions to a_ii' are kept in a register while
// the outer row i lasts and then added to LDS with one float atomic.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mgk_internal.h"
#include "mgk_launch.h"

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <int WAVES>
__device__ __forceinline__ float block_sum(float v, float* red, int wave, int lane) {
    v = wave_sum(v);
    if (WAVES == 1) return v;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) s += red[w];
    return s;
}

// Expand the octiles of one graph row into LDS entries (Section IV-B: tiles
// are stored compact and expanded on chip).  `row` is a vertex of graph g.
template <bool OUTER, bool WEIGHTED, int EK>
__device__ __forceinline__ void expand_row(const MgkBatchDev& B, const MgkGraphDesc& g, int row,
                                           uint4* ent, int n_inner, const MgkParams& prm) {
    const int tr = row >> 3, r = row & 7;
    const int32_t* trp = B.trow_ptr + g.roff;
    const int t0 = trp[tr], t1 = trp[tr + 1];
    int pos = B.rowptr[g.voff + row];
    for (int t = t0; t < t1; ++t) {
        const MgkTile tile = B.tiles[g.toff + t];
        uint32_t byte = (uint32_t)(tile.bitmap >> (8 * r)) & 0xffu;
        if (!byte) continue;
        const uint64_t below = tile.bitmap & ((1ull << (8 * r)) - 1ull);
        int k = g.zoff + (int)tile.nzoff + __popcll(below);
        while (byte) {
            const int c = __ffs(byte) - 1;
            byte &= byte - 1;
            const int col = (int)tile.tc * 8 + c;
            const float w = B.w[k];
            const float el = (B.e[k] - prm.e_shift) * prm.e_scale;
            ++k;
            uint4 v;
            if (OUTER) {
                v.x = (uint32_t)(col * n_inner * 4);  // byte offset of p row `col`
                v.y = __float_as_uint(el);
                v.z = __float_as_uint(WEIGHTED ? __log2f(w) : 0.f);
                v.w = __float_as_uint(w);
            } else {
                v.x = (uint32_t)(row * 4);
                v.y = (uint32_t)(col * 4);
                v.z = __float_as_uint(EK == MGK_EK_SE ? el : w);
                v.w = __float_as_uint(WEIGHTED ? __log2f(w) : 0.f);
            }
            ent[pos++] = v;
        }
    }
}

template <int WAVES, bool WEIGHTED, int EK>
__global__ __launch_bounds__(WAVES * 64) void mgk_pcg_small(
    MgkBatchDev X, MgkBatchDev Y, const MgkJob* __restrict__ jobs, MgkParams prm,
    float* __restrict__ K_out, int32_t* __restrict__ iters_out, int32_t* __restrict__ flag_out) {
    extern __shared__ __align__(16) uint32_t lds[];
    constexpr int NT = WAVES * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    const MgkJob job = jobs[blockIdx.x];
    const MgkGraphDesc g1 = X.graphs[job.g1];
    const MgkGraphDesc g2 = Y.graphs[job.g2];
    const int n1 = g1.n, n2 = g2.n, N = n1 * n2, z1 = g1.nnz, z2 = g2.nnz;

    float* x = reinterpret_cast<float*>(lds);
    float* r = x + N;
    float* p = r + N;
    float* a = p + N;
    float* M = a + N;
    int* rowptr1 = reinterpret_cast<int*>(M + N);
    uint4* ent1 = reinterpret_cast<uint4*>(lds + ((5 * N + n1 + 1 + 3) & ~3));
    uint4* ent2 = ent1 + z1;
    float* red = reinterpret_cast<float*>(ent2 + z2);

    // ---- expand both graphs into LDS --------------------------------------
    for (int row = tid; row < n1 + n2; row += NT) {
        if (row < n1) {
            rowptr1[row] = X.rowptr[g1.voff + row];
            expand_row<true, WEIGHTED, EK>(X, g1, row, ent1, n2, prm);
        } else {
            expand_row<false, WEIGHTED, EK>(Y, g2, row - n1, ent2, n2, prm);
        }
    }
    if (tid == 0) rowptr1[n1] = z1;

    // ---- Alg. 1 set-up: M = D_x V_x^{-1}, x = 0, r = b = D_x q_x, z = M^{-1} r,
    //      p = z, rho = r^T z.  a is preset to M p so that the XMV only has to
    //      subtract the off-diagonal product (a = M p - L p). -----------------
    const float qq = prm.q * prm.q;
    float s_rz = 0.f, s_bb = 0.f;
    for (int idx = tid; idx < N; idx += NT) {
        const int i = idx / n2, ip = idx - i * n2;
        const float d1 = X.rowsum[g1.voff + i] + prm.q;
        const float d2 = Y.rowsum[g2.voff + ip] + prm.q;
        const float kv = (X.vlabel[g1.voff + i] == Y.vlabel[g2.voff + ip]) ? 1.f : prm.h;
        const float dd = d1 * d2;
        const float b = dd * qq;
        const float z0 = kv * qq;          // M^{-1} b
        M[idx] = dd / kv;
        x[idx] = 0.f;
        r[idx] = b;
        p[idx] = z0;
        a[idx] = b;                        // M p
        s_rz += b * z0;
        s_bb += b * b;
    }
    float rho = block_sum<WAVES>(s_rz, red, wave, lane);
    const float bb = block_sum<WAVES>(s_bb, red + 16, wave, lane);
    const float thresh = prm.rtol2 * bb;
    int max_iter = prm.max_iter;
    if (max_iter <= 0) max_iter = min(2 * N, 1000);
    __syncthreads();

    const char* pbytes = reinterpret_cast<const char*>(p);
    char* abytes = reinterpret_cast<char*>(a);
    const float ke_c = prm.ke_const;

    int it = 0;
    int flag = 1;
    while (it < max_iter) {
        // ---- XMV (Alg. 2): a_ii' -= sum_{j,j'} A_ij A'_i'j' kappa_e(E_ij,E'_i'j') p_jj'
        for (int c = 0; c < z2; c += 64) {
            const int k2 = c + lane;
            const bool act = k2 < z2;
            const uint4 e2 = ent2[act ? k2 : 0];
            const uint32_t ip4 = e2.x, jp4 = e2.y;
            const float el2 = __uint_as_float(e2.z);
            const float lw2 = __uint_as_float(e2.w);
            for (int i = wave; i < n1; i += WAVES) {
                const int kb = __builtin_amdgcn_readfirstlane(rowptr1[i]);
                const int ke = __builtin_amdgcn_readfirstlane(rowptr1[i + 1]);
                if (kb == ke) continue;
                float acc = 0.f;
                for (int k = kb; k < ke; ++k) {
                    const uint4 e1 = ent1[k];
                    const float pv = *reinterpret_cast<const float*>(pbytes + (e1.x + jp4));
                    if (EK == MGK_EK_SE) {
                        const float d = el2 - __uint_as_float(e1.y);
                        float t;
                        if (WEIGHTED) t = __builtin_fmaf(-d, d, lw2 + __uint_as_float(e1.z));
                        else t = -d * d;
                        acc = __builtin_fmaf(__builtin_amdgcn_exp2f(t), pv, acc);
                    } else {
                        if (WEIGHTED) acc = __builtin_fmaf(__uint_as_float(e1.w), pv, acc);
                        else acc += pv;
                    }
                }
                if (EK == MGK_EK_CONST) {
                    acc *= WEIGHTED ? ke_c * el2 : ke_c;  // el2 holds A'_i'j' for the constant kernel
                }
                if (act) {
                    float* dst = reinterpret_cast<float*>(abytes + (i * n2 * 4 + ip4));
                    __hip_atomic_fetch_add(dst, -acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
        }
        __syncthreads();

        // ---- alpha = rho / p^T a
        float s_pa = 0.f;
        for (int idx = tid; idx < N; idx += NT) s_pa += p[idx] * a[idx];
        const float pa = block_sum<WAVES>(s_pa, red + 32, wave, lane);
        const float alpha = rho / pa;

        // ---- x += alpha p; r -= alpha a; z = M^{-1} r (kept in a); rho' = r^T z
        float s_rz2 = 0.f, s_rr = 0.f;
        for (int idx = tid; idx < N; idx += NT) {
            x[idx] = __builtin_fmaf(alpha, p[idx], x[idx]);
            const float rv = __builtin_fmaf(-alpha, a[idx], r[idx]);
            r[idx] = rv;
            const float zv = rv * __builtin_amdgcn_rcpf(M[idx]);
            a[idx] = zv;
            s_rz2 = __builtin_fmaf(rv, zv, s_rz2);
            s_rr = __builtin_fmaf(rv, rv, s_rr);
        }
        const float rho2 = block_sum<WAVES>(s_rz2, red, wave, lane);
        const float rr = block_sum<WAVES>(s_rr, red + 16, wave, lane);
        ++it;
        if (rr <= thresh) { flag = 0; break; }

        // ---- p = z + beta p ; a = M p
        const float beta = rho2 / rho;
        rho = rho2;
        for (int idx = tid; idx < N; idx += NT) {
            const float pn = __builtin_fmaf(beta, p[idx], a[idx]);
            p[idx] = pn;
            a[idx] = M[idx] * pn;
        }
        __syncthreads();
    }

    // ---- K = p_x^T x (Eq. 1)
    float s_k = 0.f;
    for (int idx = tid; idx < N; idx += NT) {
        const int i = idx / n2, ip = idx - i * n2;
        s_k += X.start[g1.voff + i] * Y.start[g2.voff + ip] * x[idx];
    }
    const float Kval = block_sum<WAVES>(s_k, red + 48, wave, lane);
    if (tid == 0) {
        K_out[job.out0] = Kval;
        if (job.out1 >= 0) K_out[job.out1] = Kval;
        if (iters_out) {
            iters_out[job.out0] = it;
            if (job.out1 >= 0) iters_out[job.out1] = it;
        }
        if (flag_out) {
            flag_out[job.out0] = flag;
            if (job.out1 >= 0) flag_out[job.out1] = flag;
        }
    }
}

template <int WAVES, bool WEIGHTED, int EK>
hipError_t launch_one(const MgkBatchDev& X, const MgkBatchDev& Y, const MgkJob* jobs, int n_jobs,
                      const MgkParams& prm, size_t lds_bytes, float* K, int32_t* iters,
                      int32_t* flags, hipStream_t stream) {
    auto kern = mgk_pcg_small<WAVES, WEIGHTED, EK>;
    static size_t configured = 0;  // per instantiation
    if (lds_bytes > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           MGK_LDS_LIMIT_BYTES);
        if (e != hipSuccess) return e;
        configured = MGK_LDS_LIMIT_BYTES;
    }
    hipLaunchKernelGGL(kern, dim3(n_jobs), dim3(WAVES * 64), lds_bytes, stream, X, Y, jobs, prm, K,
                       iters, flags);
    return hipGetLastError();
}

template <int WAVES>
hipError_t launch_w(bool weighted, int ek, const MgkBatchDev& X, const MgkBatchDev& Y,
                    const MgkJob* jobs, int n_jobs, const MgkParams& prm, size_t lds_bytes, float* K,
                    int32_t* iters, int32_t* flags, hipStream_t stream) {
    if (ek == MGK_EK_SE) {
        if (weighted) return launch_one<WAVES, true, MGK_EK_SE>(X, Y, jobs, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        return launch_one<WAVES, false, MGK_EK_SE>(X, Y, jobs, n_jobs, prm, lds_bytes, K, iters, flags, stream);
    }
    if (weighted) return launch_one<WAVES, true, MGK_EK_CONST>(X, Y, jobs, n_jobs, prm, lds_bytes, K, iters, flags, stream);
    return launch_one<WAVES, false, MGK_EK_CONST>(X, Y, jobs, n_jobs, prm, lds_bytes, K, iters, flags, stream);
}

}  // namespace

hipError_t mgk_launch_small(int waves, bool weighted, const MgkBatchDev& X, const MgkBatchDev& Y,
                            const MgkJob* jobs_dev, int n_jobs, const MgkParams& prm,
                            size_t lds_bytes, float* K, int32_t* iters, int32_t* flags,
                            hipStream_t stream) {
    if (n_jobs <= 0) return hipSuccess;
    switch (waves) {
        case 1: return launch_w<1>(weighted, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        case 2: return launch_w<2>(weighted, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        case 4: return launch_w<4>(weighted, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        case 8: return launch_w<8>(weighted, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        case 16: return launch_w<16>(weighted, prm.edge_kernel, X, Y, jobs_dev, n_jobs, prm, lds_bytes, K, iters, flags, stream);
        default: return hipErrorInvalidValue;
    }
}
