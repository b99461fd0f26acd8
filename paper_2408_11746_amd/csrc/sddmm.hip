// SDDMM over the active index list:  dW[o, i] = sum_t dY[t, o] X[t, i]  for the active
// (o, i) only (the weight-gradient half of the backward pass; App. "FLOP Calculation",
// backward = 2 x forward).
//
// Same decomposition and lane mapping as the SpMM: a workgroup owns TT = 128 tokens and
// a row block (or half of one) of the driving view per wavefront, stages chunks of one
// dense operand in LDS and walks the ELL slices (written below for the row view: X is
// staged, dY sits in registers; the col view swaps the two).  A lane keeps dY of its 8 tokens for the 4 rows of its lane group in
// registers; entries reach the lanes as in the SpMM (batches of four pairs, handed round
// the groups of four lanes through DPP operands); per step a lane reads its 8 X values of the entry's column from LDS, forms the
// 8-term dot product and the 16 lanes of the group add their parts with four DPP row
// shifts -- all four lane groups (four entries) at once, no LDS traffic.  Lane 15 of
// each group stores the per-(token tile, entry slot) partial sums; a second kernel adds
// the partials of all token tiles in a fixed order (deterministic, no floating-point
// atomics) and writes the result at the entry's canonical position.
#include "tile_loader.h"

namespace mst {

template <int CTRL>
__device__ inline float dpp_add(float x) {
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// sum over each row of 16 lanes, valid in the row's last lane
__device__ inline float row_sum_to_last(float x) {
    x = dpp_add<0x111>(x);   // row_shr:1
    x = dpp_add<0x112>(x);   // row_shr:2
    x = dpp_add<0x114>(x);   // row_shr:4
    x = dpp_add<0x118>(x);   // row_shr:8
    return x;
}

template <typename TIn>
__device__ inline float load_act(const TIn* p);
template <>
__device__ inline float load_act<float>(const float* p) { return *p; }
template <>
__device__ inline float load_act<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }

// value of v in lane JJ of this lane's aligned group of four lanes
template <int JJ>
__device__ inline uint32_t quad_bcast(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, JJ * 0x55, 0xf, 0xf, true);
}

#define MST_DOT(JJ, OFF, DY, RES)                                                    \
    do {                                                                             \
        const uint32_t a_ = lane16 ^ quad_bcast<JJ>(OFF);                                        \
        const float4 xa = *reinterpret_cast<const float4*>(tb + a_);                 \
        const float4 xb = *reinterpret_cast<const float4*>(tb + a_ + 256);           \
        float d_ = DY[0] * xa.x;                                                     \
        d_ = fmaf(DY[1], xa.y, d_); d_ = fmaf(DY[2], xa.z, d_); d_ = fmaf(DY[3], xa.w, d_); \
        d_ = fmaf(DY[4], xb.x, d_); d_ = fmaf(DY[5], xb.y, d_);                      \
        d_ = fmaf(DY[6], xb.z, d_); d_ = fmaf(DY[7], xb.w, d_);                      \
        RES = row_sum_to_last(d_);                                                   \
    } while (0)

// partial sums of the pair held by lane JJ of each group of four lanes
#define MST_DOT_PAIR(JJ, DY, P)                                                      \
    do {                                                                             \
        float r0, r1;                                                                \
        MST_DOT(JJ, cur.x, DY, r0);                                                  \
        MST_DOT(JJ, cur.z, DY, r1);                                                  \
        if (s == 15) pt[(int64_t)(P) * 4 + g] = make_float2(r0, r1);                 \
    } while (0)

constexpr int NW = 16;      // wavefronts per workgroup

// QW = quads per wavefront (4: a whole row block, 2: half of one), as in the SpMM
template <typename TIn, int QW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(8, 8)))
void k_sddmm(const TIn* __restrict__ X /* staged operand [T x K] */, const TIn* __restrict__ dY /* register operand [T x R] */,
             const int* __restrict__ ptr,
             const uint4* __restrict__ ent, const int* __restrict__ rowmap, float* __restrict__ partial, int64_t slots_stride, int T, int K,
             int R, int NBpad, int nchunk, int nslab, int ntile, int vec_ok) {
    __shared__ float tile[KC * TT];
    int tile_id, slab;
    if (!block_to_tile(nslab, ntile, tile_id, slab)) return;
    const int tid = threadIdx.x;
    constexpr int nw = NW;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = tile_id * TT;
    constexpr int WPB = 4 / QW;
    const int blk = (slab * nw + wave) / WPB;
    const int q0 = (wave % WPB) * QW;
    const int g = lane >> 4, s = lane & 15;
    const uint32_t lane16 = (uint32_t)s << 4;
    const char* tb = reinterpret_cast<const char*>(tile);
    const int eoff = (lane & 3) * 4 + g;              // this lane's 16 bytes of a batch of four pairs
    // partial sums of this token tile, viewed as float2[] indexed by pair * 4 + g
    float2* pt = reinterpret_cast<float2*>(partial + (int64_t)tile_id * slots_stride);

    // dY of this lane's 8 tokens for the rows of rank 4 (q0 + q) + g of the block
    float dy[QW][8];
    int rsel[QW];
#pragma unroll
    for (int q = 0; q < QW; ++q) rsel[q] = rowmap[blk * RB + 4 * (q0 + q) + g];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int t = t0 + lane_token(s, e);
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            float v = 0.f;
            if (t < T && rsel[q] < R) v = load_act<TIn>(dY + (int64_t)t * R + rsel[q]);
            dy[q][e] = v;
        }
    }

    const int pl = blk * 4 + q0 + min(lane, QW);
    int pv = ptr[pl];
    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) __syncthreads();
        load_tile<TIn, NW * 64>(tile, X, K, t0, c * KC, T, K, vec_ok != 0, tid);
        const int pv_next = (c + 1 < nchunk) ? ptr[(int64_t)(c + 1) * NBpad * 4 + pl] : 0;
        int p = __builtin_amdgcn_readlane(pv, 0);
        uint4 nxt = ent[(int64_t)p * 4 + eoff];
        __syncthreads();
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            const int pend = __builtin_amdgcn_readlane(pv, q + 1);
            while (p < pend) {
                const uint4 cur = nxt;
                const int pn = min(p + 4, pend);
                nxt = ent[(int64_t)pn * 4 + eoff];
                MST_DOT_PAIR(0, dy[q], p);
                if (p + 1 < pend) {
                    MST_DOT_PAIR(1, dy[q], p + 1);
                    if (p + 2 < pend) {
                        MST_DOT_PAIR(2, dy[q], p + 2);
                        if (p + 3 < pend) MST_DOT_PAIR(3, dy[q], p + 3);
                    }
                }
                p = pn;
            }
        }
        pv = pv_next;
    }
}

// dW[perm[e]] = sum over token tiles of partial[tile][e], tiles added in ascending order
__global__ void k_sddmm_reduce(const float* __restrict__ partial, int64_t slots_stride, int ntile,
                               const int* __restrict__ ptr, int64_t nseg, const int* __restrict__ perm,
                               float* __restrict__ dW) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)ptr[nseg] * 8) return;
    const int p = perm[e];
    if (p < 0) return;
    float sum = 0.f;
    for (int t = 0; t < ntile; ++t) sum += partial[(int64_t)t * slots_stride + e];
    dW[p] = sum;
}

// The product is symmetric in its two dense operands: either view can drive it.  The view
// with more rows is used (more workgroups, fewer chunks): the row view stages X and keeps
// dY in registers, the col view stages dY and keeps X in registers.
template <typename TIn>
static int launch_sddmm(const mst_layer* L, const TIn* dY, const TIn* X, float* dW, int T,
                        const Workspace& ws, hipStream_t s) {
    const bool use_col = L->I > L->O;
    const View& v = use_col ? L->col : L->row;
    const TIn* staged = use_col ? dY : X;
    const TIn* inreg = use_col ? X : dY;
    const int ntile = (int)cdiv(T, TT);
    const int qw = pick_quads(T, v.NB);
    const int nslab = (int)cdiv(v.NB, NW * qw / 4);
    const int vec_ok = (v.K % 4 == 0) ? 1 : 0;
    const int64_t stride = v.cap_pairs * 8;
    if (qw == 4)
        k_sddmm<TIn, 4><<<grid_for(ntile, nslab), NW * 64, 0, s>>>(staged, inreg, v.ptr, v.ent, v.rowmap, ws.partial, stride, T,
                                                                  v.K, v.R, v.NBpad, v.nchunk, nslab, ntile, vec_ok);
    else
        k_sddmm<TIn, 2><<<grid_for(ntile, nslab), NW * 64, 0, s>>>(staged, inreg, v.ptr, v.ent, v.rowmap, ws.partial, stride, T,
                                                                  v.K, v.R, v.NBpad, v.nchunk, nslab, ntile, vec_ok);
    MST_LAUNCH_CHECK();
    const int64_t upper = 4 * (L->nnz + (int64_t)v.nchunk * v.NB * 4);
    k_sddmm_reduce<<<(unsigned)cdiv(upper, 256), 256, 0, s>>>(ws.partial, stride, ntile, v.ptr, v.nseg, v.perm, dW);
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
