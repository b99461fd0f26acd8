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

// unchecked 16-byte (fp32) / 8-byte (bf16) read of A[row, k .. k+3]
template <typename TIn>
__device__ inline float4 load_quad_fast(const TIn* __restrict__ p);
template <>
__device__ inline float4 load_quad_fast<float>(const float* __restrict__ p) {
    return *reinterpret_cast<const float4*>(p);
}
template <>
__device__ inline float4 load_quad_fast<uint16_t>(const uint16_t* __restrict__ p) {
    const uint2 u = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u),
                       __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xFFFF0000u));
}

// Four consecutive elements as fp32 through a buffer load: the address is the descriptor's base (scalar
// registers) plus a 32-bit byte offset per lane, so no 64-bit lane address has to live across the walk.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <typename TIn>
__device__ inline float4 buffer_quad(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off);
template <>
__device__ inline float4 buffer_quad<float>(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_off, 0, 0);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
template <>
__device__ inline float4 buffer_quad<uint16_t>(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off) {
    const u32x2 u = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)byte_off, 0, 0);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u),
                       __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xFFFF0000u));
}
// descriptor of `bytes` bytes from p (raw buffer: no stride, offsets beyond `bytes` read zero)
__device__ inline __amdgpu_buffer_rsrc_t buffer_of(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// All threads of the workgroup fill tile[KC][TT] from A[t0 .. t0+TT) x [k0 .. k0+KC).
// Work item = (token quad tq, index quad kq): four 16-byte row reads (consecutive lanes
// read consecutive 16 bytes of a row), transposed in registers, eight 8-byte LDS stores.
// 1024 items per tile.  A tile that lies wholly inside the matrix (and rows that allow
// vector reads) takes the branch-free path: all four reads of an item are in flight at
// once, one memory round trip per tile.  Edge tiles take the checked path.
template <typename TIn, int NTHREADS>
__device__ inline void load_tile(float* tile, const TIn* __restrict__ A, int64_t lda, int t0, int k0, int T,
                                 int K, bool vec_ok, int tid) {
    constexpr int ITEMS = (TT / 4) * (KC / 4);
    static_assert(ITEMS % NTHREADS == 0, "tile loader needs a thread count that divides 1024");
    char* base = reinterpret_cast<char*>(tile);
    const bool interior = vec_ok && t0 + TT <= T && k0 + KC <= K;     // uniform over the workgroup
    // The lane's offsets are worked out again for every tile (a dozen VALU instructions): as values that
    // do not change round the chunk loop they would be kept in registers across the walk, which has none
    // to spare -- they ended up in scratch memory and were read back before every tile.
    asm volatile("" : "+v"(tid));
#pragma unroll
    for (int it = 0; it < ITEMS / NTHREADS; ++it) {
        const int item = it * NTHREADS + tid;
        const int kq = item & (KC / 4 - 1);
        const int tq = item / (KC / 4);
        const int row = t0 + 4 * tq, k = k0 + 4 * kq;
        // rows 4kq .. 4kq+3 share the swizzle kq & 15
        const uint32_t slot = ((uint32_t)(tq >> 4) << 8) | ((uint32_t)((tq & 15) ^ (kq & 15)) << 4);
        const uint32_t kl = 4u * kq;
        if (interior) {
            // buffer loads from the tile's corner (the same for every lane: scalar registers) with a 32-bit
            // lane offset, instead of a 64-bit address per lane and row kept alive round the chunk loop
            const TIn* corner = A + (int64_t)t0 * lda + k0;
            const uint32_t ld = (uint32_t)lda * (uint32_t)sizeof(TIn);
            const __amdgpu_buffer_rsrc_t rs = buffer_of(corner, (uint32_t)(TT - 1) * ld + (uint32_t)(KC * sizeof(TIn)));
            const uint32_t o = (uint32_t)(4 * tq) * ld + (uint32_t)(4 * kq * sizeof(TIn));
            const float4 r0 = buffer_quad<TIn>(rs, o);
            const float4 r1 = buffer_quad<TIn>(rs, o + ld);
            const float4 r2 = buffer_quad<TIn>(rs, o + 2 * ld);
            const float4 r3 = buffer_quad<TIn>(rs, o + 3 * ld);
            *reinterpret_cast<float4*>(base + (((kl + 0) << 9) | slot)) = make_float4(r0.x, r1.x, r2.x, r3.x);
            *reinterpret_cast<float4*>(base + (((kl + 1) << 9) | slot)) = make_float4(r0.y, r1.y, r2.y, r3.y);
            *reinterpret_cast<float4*>(base + (((kl + 2) << 9) | slot)) = make_float4(r0.z, r1.z, r2.z, r3.z);
            *reinterpret_cast<float4*>(base + (((kl + 3) << 9) | slot)) = make_float4(r0.w, r1.w, r2.w, r3.w);
            continue;
        }
        // two token rows at a time (8 live registers): 8-byte halves of the 16-byte slot
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float4 a = load_quad<TIn>(A, lda, row + 2 * h, k, T, K, vec_ok);
            const float4 b = load_quad<TIn>(A, lda, row + 2 * h + 1, k, T, K, vec_ok);
            const uint32_t sl = slot | (uint32_t)(h << 3);
            *reinterpret_cast<float2*>(base + (((kl + 0) << 9) | sl)) = make_float2(a.x, b.x);
            *reinterpret_cast<float2*>(base + (((kl + 1) << 9) | sl)) = make_float2(a.y, b.y);
            *reinterpret_cast<float2*>(base + (((kl + 2) << 9) | sl)) = make_float2(a.z, b.z);
            *reinterpret_cast<float2*>(base + (((kl + 3) << 9) | sl)) = make_float2(a.w, b.w);
        }
    }
}

// token index (inside the tile) of a lane's e-th value, e = 0..7, s = lane & 15
__device__ inline int lane_token(int s, int e) { return (e < 4) ? 4 * s + e : 64 + 4 * s + (e - 4); }

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

}  // namespace mst
