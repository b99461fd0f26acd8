// Cross-lane building blocks shared by the kernels that walk the ELL slices (SpMM, SDDMM and
// the backward kernel that does both): entry hand-over inside groups of four lanes, sums over
// the 16 lanes of a lane group, and the fold of a spread quad.
#pragma once
#include "common.h"

namespace mst {

// A lane's 16 bytes of the batch of four pairs that starts at pair p (p the same in all lanes): a buffer
// load from a 256-byte descriptor of the batch (scalar registers) at the lane's byte offset, so that no
// 64-bit lane address of the entry array has to be kept or added to.
typedef uint32_t walk_u32x4 __attribute__((ext_vector_type(4)));
__device__ inline uint4 load_batch(const uint4* __restrict__ ent, int p, uint32_t lane_byte) {
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(ent + (int64_t)p * 4), 0, 256, 0x00020000);
    const walk_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)lane_byte, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// A pair's eight partial sums (32 bytes at `slots`, the same address in all lanes): the storing lanes
// write theirs with a buffer store at their byte offset -- again no 64-bit lane address.
__device__ inline void store_pair_slot(float* slots, uint32_t lane_byte, float v) {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(slots, 0, 32, 0x00020000);
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rs, (int)lane_byte, 0, 0);
}

// value of v in lane JJ of this lane's aligned group of four lanes
template <int JJ>
__device__ inline uint32_t quad_bcast(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, JJ * 0x55, 0xf, 0xf, true);
}

// Four FMAs whose common factor W comes from lane JJ of the group of four lanes through the
// DPP operand of v_fmac_f32 (no separate broadcast move).  The leading s_nop covers the two
// wait states a DPP read needs after a VALU write of its source, whatever was scheduled
// in front of the block.
#define MST_FMA4_BC(JJ, A0, A1, A2, A3, W, X)                                                   \
    asm("s_nop 1\n\t"                                                                           \
        "v_fmac_f32_dpp %0, %4, %5 quad_perm:[" #JJ "," #JJ "," #JJ "," #JJ "] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t" \
        "v_fmac_f32_dpp %1, %4, %6 quad_perm:[" #JJ "," #JJ "," #JJ "," #JJ "] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t" \
        "v_fmac_f32_dpp %2, %4, %7 quad_perm:[" #JJ "," #JJ "," #JJ "," #JJ "] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t" \
        "v_fmac_f32_dpp %3, %4, %8 quad_perm:[" #JJ "," #JJ "," #JJ "," #JJ "] row_mask:0xf bank_mask:0xf bound_ctrl:1"     \
        : "+v"(A0), "+v"(A1), "+v"(A2), "+v"(A3)                                                \
        : "v"(W), "v"(X.x), "v"(X.y), "v"(X.z), "v"(X.w))

// A spread quad (one long row dealt over the four lane groups): lane group 0 takes the sum
// of the four lane groups' accumulators, the others -- whose output positions belong to
// empty rows -- take zero.  `spread` is the same in every lane of the wavefront.
template <int NACC>
__device__ inline void fold_spread(float (&acc)[NACC], int spread, int g) {
    if (!__builtin_amdgcn_readfirstlane(spread)) return;
#pragma unroll
    for (int e = 0; e < NACC; ++e) {
        float v = acc[e];
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        acc[e] = (g == 0) ? v : 0.f;
    }
}

// p[0] + p[stride] + ... + p[(ntile - 1) stride], added in that order (the order is part of the
// result); sixteen loads are in flight before the first add, a one-by-one loop waits for each.
__device__ inline float ordered_plane_sum(const float* __restrict__ p, int64_t stride, int ntile) {
    float sum = 0.f;
    int t = 0;
    for (; t + 16 <= ntile; t += 16) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = p[(int64_t)(t + u) * stride];
#pragma unroll
        for (int u = 0; u < 16; ++u) sum += v[u];
    }
    for (; t < ntile; ++t) sum += p[(int64_t)t * stride];
    return sum;
}

template <int CTRL>
__device__ inline float dpp_add(float x) {
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sums of a and b over each row of 16 lanes with six adds / selects instead of eight:
// after the first exchange the lower eight lanes go on with a, the upper eight with b.
// The sum of a ends up in lanes 0..7 of the row, the sum of b in lanes 8..15.
__device__ inline float row_sum_pair(float a, float b, bool upper_half) {
    a = dpp_add<0x128>(a);                 // row_ror:8   lane s += lane s ^ 8
    b = dpp_add<0x128>(b);
    float c = upper_half ? b : a;
    c = dpp_add<0x141>(c);                 // row_half_mirror   lane s += lane 7 - s of its half
    c = dpp_add<0xB1>(c);                  // quad_perm:[1,0,3,2]
    c = dpp_add<0x4E>(c);                  // quad_perm:[2,3,0,1]
    return c;
}

}  // namespace mst
