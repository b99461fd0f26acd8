// SDDMM over the active index list:  dW[o, i] = sum_t dY[t, o] X[t, i]  for the active
// (o, i) only (the weight-gradient half of the backward pass; App. "FLOP Calculation",
// backward = 2 x forward).
//
// Same decomposition as the SpMM: a workgroup owns TT = 128 tokens and a slab of 8*RW
// rows of the row view, stages chunks of X in LDS and walks its rows' entries.  A lane
// keeps dY for its two tokens and its wavefront's RW rows in registers; per entry it reads
// its two X values from LDS, forms the two products and the wavefront sums them, four
// entries at a time, with DPP exchanges and one MFMA (no LDS traffic).  Lane 0 stores the
// per-(token tile, entry) partial sums; a
// second kernel adds the partials of all token tiles in a fixed order (deterministic,
// no floating-point atomics) and writes the result at the entry's canonical position.
#include "tile_loader.h"

namespace mst {

typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ inline float dpp_mov(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sums four per-lane values over the 64 lanes at once; the four totals come back in
// lane 0 (components 0..3).  Two butterfly levels fold the four registers into one whose
// lane l carries a partial of value l % 4 (quad_perm exchanges), two row rotations sum
// the quads of each row of 16 lanes, and one 16x16x4 MFMA against a matrix of ones adds
// the four rows: D[i][j] = sum_k x[lane i + 16k], rows 0..3 of D sit in lane 0's registers.
__device__ inline floatx4 wave_sum4(float p0, float p1, float p2, float p3, int lane) {
    const bool b0 = lane & 1, b1 = lane & 2;
    const float q01 = (b0 ? p1 : p0) + dpp_mov<0xB1>(b0 ? p0 : p1);     // quad_perm [1,0,3,2]
    const float q23 = (b0 ? p3 : p2) + dpp_mov<0xB1>(b0 ? p2 : p3);
    float x = (b1 ? q23 : q01) + dpp_mov<0x4E>(b1 ? q01 : q23);         // quad_perm [2,3,0,1]
    x += dpp_mov<0x124>(x);                                              // row_ror:4
    x += dpp_mov<0x128>(x);                                              // row_ror:8
    floatx4 z = {0.f, 0.f, 0.f, 0.f};
    return __builtin_amdgcn_mfma_f32_16x16x4f32(x, 1.0f, z, 0, 0, 0);
}

template <typename TIn>
__device__ inline float load_act(const TIn* p);
template <>
__device__ inline float load_act<float>(const float* p) { return *p; }
template <>
__device__ inline float load_act<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }

template <int RWMAX, typename TIn>
__global__ __launch_bounds__(512) void k_sddmm(const TIn* __restrict__ X, const TIn* __restrict__ dY,
                                               const int* __restrict__ ptr, const Ent4* __restrict__ ent4,
                                               float* __restrict__ partial, int64_t capv, int T, int K, int R,
                                               int Rpad, int nchunk, int nslab, int ntile, int rw, int vec_ok) {
    __shared__ float tile[KC * TT];
    int tile_id, slab;
    if (!block_to_tile(nslab, ntile, tile_id, slab)) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = tile_id * TT;
    const int r0 = slab * (8 * rw) + wave * rw;
    const uint32_t lane8 = (uint32_t)lane << 3;
    const char* tb = reinterpret_cast<const char*>(tile);
    float4* pt = reinterpret_cast<float4*>(partial + (int64_t)tile_id * capv);

    // dY for this lane's two tokens and the wavefront's rows
    float2 dy[RWMAX];
    const int ta = t0 + 2 * lane;
#pragma unroll
    for (int r = 0; r < RWMAX; ++r) {
        float a = 0.f, b = 0.f;
        if (r < rw && r0 + r < R) {
            if (ta < T) a = load_act<TIn>(dY + (int64_t)ta * R + r0 + r);
            if (ta + 1 < T) b = load_act<TIn>(dY + (int64_t)(ta + 1) * R + r0 + r);
        }
        dy[r] = make_float2(a, b);
    }

    const int pl = r0 + min(lane, rw);
    int pv = ptr[pl];
    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) __syncthreads();
        load_tile<TIn, 512>(tile, X, K, t0, c * KC, T, K, vec_ok != 0, tid);
        const int pv_next = (c + 1 < nchunk) ? ptr[(int64_t)(c + 1) * Rpad + pl] : 0;
        int g = __builtin_amdgcn_readlane(pv, 0) >> 2;
        Ent4 cur = ent4[g];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < RWMAX; ++r) {
            if (r < rw) {
                const int gend = __builtin_amdgcn_readlane(pv, r + 1) >> 2;
                for (; g < gend; ++g) {
                    const Ent4 nxt = ent4[g + 1];
                    const float2 x0 = *reinterpret_cast<const float2*>(tb + (lane8 ^ cur.off0));
                    const float2 x1 = *reinterpret_cast<const float2*>(tb + (lane8 ^ cur.off1));
                    const float2 x2 = *reinterpret_cast<const float2*>(tb + (lane8 ^ cur.off2));
                    const float2 x3 = *reinterpret_cast<const float2*>(tb + (lane8 ^ cur.off3));
                    const floatx4 s = wave_sum4(fmaf(dy[r].y, x0.y, dy[r].x * x0.x),
                                                fmaf(dy[r].y, x1.y, dy[r].x * x1.x),
                                                fmaf(dy[r].y, x2.y, dy[r].x * x2.x),
                                                fmaf(dy[r].y, x3.y, dy[r].x * x3.x), lane);
                    if (lane == 0) pt[g] = make_float4(s[0], s[1], s[2], s[3]);
                    cur = nxt;
                }
            }
        }
        pv = pv_next;
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

int pick_rows_per_wave(int T, int R, int nw, int rw_max, double stage_cost);   // spmm.hip

template <typename TIn>
static int launch_sddmm(const mst_layer* L, const TIn* dY, const TIn* X, float* dW, int T,
                        const Workspace& ws, hipStream_t s) {
    const View& v = L->row;
    const int rw = pick_rows_per_wave(T, v.R, 8, 16, 6.0);
    const int ntile = (int)cdiv(T, TT);
    const int nslab = (int)cdiv(v.R, 8 * rw);
    const int vec_ok = (v.K % 4 == 0) ? 1 : 0;
    k_sddmm<16, TIn><<<grid_for(ntile, nslab), 512, 0, s>>>(X, dY, v.ptr, reinterpret_cast<const Ent4*>(v.ent),
                                                           ws.partial, v.capv, T, v.K, v.R, v.Rpad, v.nchunk,
                                                           nslab, ntile, rw, vec_ok);
    MST_LAUNCH_CHECK();
    const int64_t upper = L->nnz + (SEG_PAD - 1) * (int64_t)v.nchunk * v.R;
    k_sddmm_reduce<<<(unsigned)cdiv(upper, 256), 256, 0, s>>>(ws.partial, v.capv, ntile, v.ptr, v.nseg, v.perm, dW);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int sddmm(const mst_layer* L, const void* dY, const void* X, float* dW, int T, mst_dtype act,
          const Workspace& ws, hipStream_t s) {
    if (L->nnz == 0) return MST_OK;
    if (act == MST_F32)
        return launch_sddmm<float>(L, static_cast<const float*>(dY), static_cast<const float*>(X), dW, T, ws, s);
    return launch_sddmm<uint16_t>(L, static_cast<const uint16_t*>(dY), static_cast<const uint16_t*>(X), dW, T, ws, s);
}

}  // namespace mst
