// Strided attention pattern of Sec. 3.3 as a byte mask: M[i][j] = 1 iff j <= i and
// (i - j < l or (i - j) mod l = 0).  Write-only and HBM-bound: a thread produces 16
// consecutive bytes of a row and stores them as one 16-byte word (rows are 16-byte
// aligned when L is a multiple of 16; other lengths take the byte path).
#include "common.h"

namespace mst {

__device__ inline uint32_t keep(int i, int64_t j, int l) {
    if (j > i) return 0u;
    const int back = i - (int)j;
    return (back < l || back % l == 0) ? 1u : 0u;
}

// One row per blockIdx.y.  The window and the causal cut are comparisons; the strided
// positions j = i - k l of a 16-byte group are found from one remainder per thread and set
// bit by bit (at most one of them when l >= 16).
__global__ void k_strided_mask16(uint8_t* __restrict__ M, int L, int l) {
    const int i = blockIdx.y;
    const int j0 = (blockIdx.x * blockDim.x + threadIdx.x) * 16;
    if (j0 >= L) return;
    uint64_t w[2] = {0, 0};
    if (j0 <= i) {
        const int lo = i - l + 1;                            // first position of the window
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const int j = j0 + b;
            if (j >= lo && j <= i) w[b >> 3] |= 1ull << (8 * (b & 7));
        }
        // positions congruent to i modulo l: the first at or after j0, then every l-th
        const int r = i % l, m0 = j0 % l;
        int h = (r >= m0) ? r - m0 : r - m0 + l;             // offset inside the group
        const int last = min(15, i - j0);
        for (; h <= last; h += l) {
            if (h < 8) w[0] |= 1ull << (8 * h);
            else w[1] |= 1ull << (8 * (h - 8));
        }
    }
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 v = {(uint32_t)w[0], (uint32_t)(w[0] >> 32), (uint32_t)w[1], (uint32_t)(w[1] >> 32)};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(M + (int64_t)i * L + j0));
}

__global__ void k_strided_mask1(uint8_t* __restrict__ M, int L, int l) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)L * L) return;
    M[id] = (uint8_t)keep((int)(id / L), id % L, l);
}

}  // namespace mst

extern "C" int mst_strided_attention_mask(uint8_t* M_dev, int L, int stride, mst_stream_t stream) {
    using namespace mst;
    if (!M_dev || L < 1 || L > 32768 || stride < 1) return MST_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(M_dev) % 16 != 0) return MST_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (L % 16 == 0) {
        const int per_row = L / 16;
        const int threads = per_row >= 256 ? 256 : 64;
        k_strided_mask16<<<dim3((unsigned)cdiv(per_row, threads), (unsigned)L), threads, 0, s>>>(M_dev, L, stride);
    } else {
        const int64_t n = (int64_t)L * L;
        k_strided_mask1<<<(unsigned)cdiv(n, 256), 256, 0, s>>>(M_dev, L, stride);
    }
    MST_LAUNCH_CHECK();
    return MST_OK;
}
