// Wavefront-level helpers shared by the on-chip kernels: DPP reductions and the
// masked shift-and-add step that sums the lanes of an inner row.
#ifndef MGK_WAVE_H
#define MGK_WAVE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// ---- wavefront reductions with DPP (no LDS traffic) --------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
    return v + __int_as_float(moved);
}

__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror
    v = dpp_add<0x140>(v);  // row_mirror: every lane holds the sum of its row of 16
    // row_bcast:15 into rows 1 and 3, then row_bcast:31 into rows 2 and 3: lane 63 holds the
    // total.  Written out so that each step is one DPP add (rows outside the row mask keep
    // their value); the wait states a DPP read needs after a VALU write are explicit.
    asm("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                 "s_nop 0"   // one more before the lane read below
                 : "+v"(v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Sum of the 8 (or 16) values held by 8 (16) adjacent lanes, in every one of them.
template <int COUNT>
__device__ __forceinline__ float group_sum(float t) {
    static_assert(COUNT == 8 || COUNT == 16, "group of 8 or 16 lanes");
    t = dpp_add<0xB1>(t);   // quad_perm [1,0,3,2]
    t = dpp_add<0x4E>(t);   // quad_perm [2,3,0,1]
    t = dpp_add<0x141>(t);  // row_half_mirror
    if (COUNT == 16) t = dpp_add<0x140>(t);  // row_mirror
    return t;
}

// Sum over the workgroup.  Every wave leaves its partial in red[wave]; after the
// barrier either every thread adds the few partials itself, or (8 and 16 waves)
// the lanes of a wave read one partial each and add them with DPP steps.  All
// waves add in the same order, so all hold the same bits.
template <int WAVES>
__device__ __forceinline__ float block_sum(float v, float* red, int wave, int lane) {
    v = wave_sum(v);
    if (WAVES == 1) return v;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    if constexpr (WAVES >= 8) {
        const float t = group_sum<WAVES>(red[lane & (WAVES - 1)]);
        return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), 0));
    } else {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) s += red[w];
        return s;
    }
}

// Two sums at once; red needs 32 floats.
template <int WAVES>
__device__ __forceinline__ void block_sum2(float& u, float& v, float* red, int wave, int lane) {
    u = wave_sum(u);
    v = wave_sum(v);
    if (WAVES == 1) return;
    if (lane == 0) { red[wave] = u; red[16 + wave] = v; }
    __syncthreads();
    if constexpr (WAVES >= 8) {
        // lanes 0..15 (8 waves: 0..7) gather u's partials, lanes 16..31 (8..15) v's
        const float t = group_sum<WAVES>(red[(lane & (WAVES - 1)) + ((lane & WAVES) ? 16 : 0)]);
        u = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), 0));
        v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), WAVES));
    } else {
        float su = 0.f, sv = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) { su += red[w]; sv += red[16 + w]; }
        u = su;
        v = sv;
    }
}

// acc += m * (acc of the lane DIST places lower in the same 16-lane row, 0 if none):
// one step of the masked shift-and-add that sums the lanes of an inner row.  A
// single DPP multiply-add; the two wait states a DPP read needs after a VALU
// write of the same register are spelled out because the instruction is
// emitted by hand.
template <int DIST>
__device__ __forceinline__ float shr_fmac(float acc, float m) {
    asm volatile("s_nop 1\n\tv_fmac_f32_dpp %0, %0, %1 row_shr:%2 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(acc)
                 : "v"(m), "n"(DIST));
    return acc;
}

// The same step on two accumulators at once: the second instruction fills one of the
// wait states of the first one's successor.
template <int DIST>
__device__ __forceinline__ void shr_fmac_pair(float& acc0, float& acc1, float m0, float m1) {
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %0, %2 row_shr:%4 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %1, %1, %3 row_shr:%4 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(acc0), "+v"(acc1)
                 : "v"(m0), "v"(m1), "n"(DIST));
}

}  // namespace

#endif
