// SDDMM over the active index list:  dW[o, i] = sum_t dY[t, o] X[t, i]  for the active
// (o, i) only (the weight-gradient half of the backward pass; App. "FLOP Calculation",
// backward = 2 x forward).
//
// Same decomposition as the SpMM: a workgroup owns TT = 128 tokens and a slab of 8*RW
// rows of the row view, stages chunks of X in LDS and walks its rows' entries.  A lane
// keeps dY for its two tokens and its wavefront's RW rows in registers; per entry it reads
// its two X values from LDS, forms the two products and the wavefront sums them with a
// DPP scan (no LDS traffic).  Lane 63 stores the per-(token tile, entry) partial sums; a
// second kernel adds the partials of all token tiles in a fixed order (deterministic,
// no floating-point atomics) and writes the result at the entry's canonical position.
#include "tile_loader.h"

namespace mst {

template <int CTRL, int ROW_MASK>
__device__ inline float dpp_add(float x) {
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, true);
    return x + __int_as_float(y);
}

// sum over the 64 lanes, valid in lane 63
__device__ inline float wave_sum_to_last(float x) {
    x = dpp_add<0x111, 0xf>(x);   // row_shr:1
    x = dpp_add<0x112, 0xf>(x);   // row_shr:2
    x = dpp_add<0x114, 0xf>(x);   // row_shr:4
    x = dpp_add<0x118, 0xf>(x);   // row_shr:8   -> lane 15 of each row of 16 holds the row sum
    x = dpp_add<0x142, 0xa>(x);   // row_bcast:15 into rows 1 and 3
    x = dpp_add<0x143, 0xc>(x);   // row_bcast:31 into rows 2 and 3 -> lane 63 holds the total
    return x;
}

template <typename TIn>
__device__ inline float load_act(const TIn* p);
template <>
__device__ inline float load_act<float>(const float* p) { return *p; }
template <>
__device__ inline float load_act<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }

template <int RW, typename TIn>
__global__ __launch_bounds__(512) void k_sddmm(const TIn* __restrict__ X, const TIn* __restrict__ dY,
                                               const int* __restrict__ ptr, const Ent4* __restrict__ ent4,
                                               float* __restrict__ partial, int64_t capv, int T, int K, int R,
                                               int Rpad, int nchunk, int nslab, int ntile, int vec_ok) {
    __shared__ float tile[KC * TT];
    int tile_id, slab;
    if (!block_to_tile(nslab, ntile, tile_id, slab)) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = tile_id * TT;
    const int r0 = slab * (8 * RW) + wave * RW;
    const uint32_t lane8 = (uint32_t)lane << 3;
    const char* tb = reinterpret_cast<const char*>(tile);
    float* pt = partial + (int64_t)tile_id * capv;

    // dY for this lane's two tokens and the wavefront's rows
    float2 dy[RW];
    const int ta = t0 + 2 * lane;
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        float a = 0.f, b = 0.f;
        if (r0 + r < R) {
            if (ta < T) a = load_act<TIn>(dY + (int64_t)ta * R + r0 + r);
            if (ta + 1 < T) b = load_act<TIn>(dY + (int64_t)(ta + 1) * R + r0 + r);
        }
        dy[r] = make_float2(a, b);
    }

    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) __syncthreads();
        load_tile<TIn, 512>(tile, X, K, t0, c * KC, T, K, vec_ok != 0, tid);
        __syncthreads();
        const int* p = ptr + (int64_t)c * Rpad + r0;
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            const int beg = p[r], end = p[r + 1];
            const Ent4* eg = ent4 + (beg >> 2);
            const int ng = (end - beg) >> 2;
            Ent4 cur = eg[0];
            for (int g = 0; g < ng; ++g) {
                const Ent4 nxt = eg[g + 1];
                const float2 x0 = *reinterpret_cast<const float2*>(tb + (lane8 ^ cur.off0));
                const float2 x1 = *reinterpret_cast<const float2*>(tb + (lane8 ^ cur.off1));
                const float2 x2 = *reinterpret_cast<const float2*>(tb + (lane8 ^ cur.off2));
                const float2 x3 = *reinterpret_cast<const float2*>(tb + (lane8 ^ cur.off3));
                float4 s;
                s.x = wave_sum_to_last(fmaf(dy[r].y, x0.y, dy[r].x * x0.x));
                s.y = wave_sum_to_last(fmaf(dy[r].y, x1.y, dy[r].x * x1.x));
                s.z = wave_sum_to_last(fmaf(dy[r].y, x2.y, dy[r].x * x2.x));
                s.w = wave_sum_to_last(fmaf(dy[r].y, x3.y, dy[r].x * x3.x));
                if (lane == 63) *reinterpret_cast<float4*>(pt + beg + 4 * g) = s;
                cur = nxt;
            }
        }
    }
}

// dW[perm[e]] = sum over token tiles of partial[tile][e], tiles added in ascending order
__global__ void k_sddmm_reduce(const float* __restrict__ partial, int64_t capv, int ntile,
                               const int* __restrict__ ptr, int64_t nseg, const int* __restrict__ perm,
                               float* __restrict__ dW) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= ptr[nseg]) return;
    const int p = perm[e];
    if (p < 0) return;
    float s = 0.f;
    for (int t = 0; t < ntile; ++t) s += partial[(int64_t)t * capv + e];
    dW[p] = s;
}

template <int RW, typename TIn>
static int launch_sddmm(const mst_layer* L, const TIn* dY, const TIn* X, float* dW, int T,
                        const Workspace& ws, hipStream_t s) {
    const View& v = L->row;
    const int ntile = (int)cdiv(T, TT);
    const int nslab = (int)cdiv(v.R, 8 * RW);
    const int vec_ok = (v.K % 4 == 0) ? 1 : 0;
    k_sddmm<RW, TIn><<<grid_for(ntile, nslab), 512, 0, s>>>(X, dY, v.ptr, reinterpret_cast<const Ent4*>(v.ent),
                                                           ws.partial, v.capv, T, v.K, v.R, v.Rpad, v.nchunk,
                                                           nslab, ntile, vec_ok);
    MST_LAUNCH_CHECK();
    const int64_t upper = L->nnz + (SEG_PAD - 1) * (int64_t)v.nchunk * v.R;
    k_sddmm_reduce<<<(unsigned)cdiv(upper, 256), 256, 0, s>>>(ws.partial, v.capv, ntile, v.ptr, v.nseg, v.perm, dW);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int sddmm(const mst_layer* L, const void* dY, const void* X, float* dW, int T, mst_dtype act,
          const Workspace& ws, hipStream_t s) {
    if (L->nnz == 0) return MST_OK;
    const int64_t ntile = cdiv(T, TT);
    const int rw = (ntile * cdiv(L->O, 8 * 16) >= 512) ? 16 : 8;
    if (act == MST_F32) {
        const float* y = static_cast<const float*>(dY);
        const float* x = static_cast<const float*>(X);
        return rw == 16 ? launch_sddmm<16, float>(L, y, x, dW, T, ws, s) : launch_sddmm<8, float>(L, y, x, dW, T, ws, s);
    }
    const uint16_t* y = static_cast<const uint16_t*>(dY);
    const uint16_t* x = static_cast<const uint16_t*>(X);
    return rw == 16 ? launch_sddmm<16, uint16_t>(L, y, x, dW, T, ws, s)
                    : launch_sddmm<8, uint16_t>(L, y, x, dW, T, ws, s);
}

}  // namespace mst
