// Cooperative load of one [TT tokens x KC indices] block of a row-major activation
// matrix into the transposed, swizzled LDS tile described at lds_off().
#pragma once
#include "common.h"

namespace mst {

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// four consecutive elements A[row, k .. k+3] as fp32; zero outside [0,T) x [0,K)
template <typename TIn>
__device__ inline float4 load_quad(const TIn* __restrict__ A, int64_t lda, int row, int k, int T, int K,
                                   bool vec_ok);

template <>
__device__ inline float4 load_quad<float>(const float* __restrict__ A, int64_t lda, int row, int k, int T,
                                          int K, bool vec_ok) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row >= T || k >= K) return v;
    const float* p = A + (int64_t)row * lda + k;
    if (vec_ok && k + 3 < K) return *reinterpret_cast<const float4*>(p);
    v.x = p[0];
    if (k + 1 < K) v.y = p[1];
    if (k + 2 < K) v.z = p[2];
    if (k + 3 < K) v.w = p[3];
    return v;
}

template <>
__device__ inline float4 load_quad<uint16_t>(const uint16_t* __restrict__ A, int64_t lda, int row, int k,
                                             int T, int K, bool vec_ok) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row >= T || k >= K) return v;
    const uint16_t* p = A + (int64_t)row * lda + k;
    if (vec_ok && k + 3 < K) {
        const uint2 u = *reinterpret_cast<const uint2*>(p);
        v.x = __uint_as_float(u.x << 16);
        v.y = __uint_as_float(u.x & 0xFFFF0000u);
        v.z = __uint_as_float(u.y << 16);
        v.w = __uint_as_float(u.y & 0xFFFF0000u);
        return v;
    }
    v.x = bf16_to_f32(p[0]);
    if (k + 1 < K) v.y = bf16_to_f32(p[1]);
    if (k + 2 < K) v.z = bf16_to_f32(p[2]);
    if (k + 3 < K) v.w = bf16_to_f32(p[3]);
    return v;
}

// NTHREADS threads fill tile[KC][TT] from A[t0 .. t0+TT) x [k0 .. k0+KC).
// Work item = (token pair tp, quad q): two 16-byte row reads, four 8-byte LDS stores.
template <typename TIn, int NTHREADS>
__device__ inline void load_tile(float* tile, const TIn* __restrict__ A, int64_t lda, int t0, int k0, int T,
                                 int K, bool vec_ok, int tid) {
    constexpr int QUADS = KC / 4;              // 32
    constexpr int ITEMS = (TT / 2) * QUADS;    // 2048
    static_assert(ITEMS % NTHREADS == 0, "tile loader needs a divisor thread count");
    char* base = reinterpret_cast<char*>(tile);
#pragma unroll
    for (int it = 0; it < ITEMS / NTHREADS; ++it) {
        const int item = it * NTHREADS + tid;
        const int q = item & (QUADS - 1);
        const int tp = item / QUADS;
        const int row = t0 + 2 * tp, k = k0 + 4 * q;
        const float4 a = load_quad<TIn>(A, lda, row, k, T, K, vec_ok);
        const float4 b = load_quad<TIn>(A, lda, row + 1, k, T, K, vec_ok);
        const uint32_t kl = 4u * q;
        // rows kl .. kl+3 share the swizzle q (kl >> 2 == q)
        const uint32_t slot = ((uint32_t)tp ^ (uint32_t)q) << 3;
        *reinterpret_cast<float2*>(base + (((kl + 0) << 9) | slot)) = make_float2(a.x, b.x);
        *reinterpret_cast<float2*>(base + (((kl + 1) << 9) | slot)) = make_float2(a.y, b.y);
        *reinterpret_cast<float2*>(base + (((kl + 2) << 9) | slot)) = make_float2(a.z, b.z);
        *reinterpret_cast<float2*>(base + (((kl + 3) << 9) | slot)) = make_float2(a.w, b.w);
    }
}

// XCD-aware block -> (token tile, row slab): consecutive blocks go to the 8 XCDs in turn,
// so the slabs of one token tile are given block ids that land on the same XCD and
// share that XCD's L2 copy of the activation tile.
__device__ inline bool block_to_tile(int nslab, int ntile, int& tile, int& slab) {
    const int b = blockIdx.x;
    const int xcd = b & 7, q = b >> 3;
    tile = (q / nslab) * 8 + xcd;
    slab = q % nslab;
    return tile < ntile;
}
inline unsigned grid_for(int ntile, int nslab) { return (unsigned)(cdiv(ntile, 8) * 8 * nslab); }

// four view entries fetched with one scalar load
struct __attribute__((aligned(32))) Ent4 {
    uint32_t off0, w0, off1, w1, off2, w2, off3, w3;
};

}  // namespace mst
