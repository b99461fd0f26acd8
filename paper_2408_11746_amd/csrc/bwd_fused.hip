// Both gradients of a layer from ONE walk of the col view (S = W^T, rows = input index i,
// contraction over the output index o; App. "FLOP Calculation": backward = 2 x forward):
//
//   dX[t, i] = sum_o dY[t, o] W[o, i]          (the input gradient, an SpMM over the col view)
//   dW[o, i] = sum_t dY[t, o] X[t, i]          (the weight gradient at the active positions)
//
// The two products read the same staged operand: a workgroup stages chunks of dY for its
// 128 tokens in LDS and walks the ELL slices of its quads once; the eight dY values a lane
// reads for an entry feed both the eight FMAs of the input gradient (weight handed round
// through the DPP operand, as in the SpMM) and the 8-term dot product with the lane's X
// values (summed over the 16 lanes of a lane group as in the SDDMM).  Per entry that halves
// the LDS reads, the entry fetches and the staging of dY against the two separate kernels.
// Every sum is formed in the order the separate kernels use (dX: a row's entries in stored
// order; dW: 128-token partial sums added in ascending tile order by the second kernel), so
// the results are those of the SpMM, bit for bit, and of the SDDMM when it is driven by the
// col view.
#include <algorithm>

#include "tile_loader.h"
#include "walk_ops.h"

namespace mst {

// one entry {OFF, W} held by lane JJ of the group of four lanes: both products
#define MSTF_STEP(JJ, OFF, W, XR, ACC, RES)                                           \
    do {                                                                             \
        const uint32_t a_ = lane16 ^ quad_bcast<JJ>(OFF);                            \
        const float4 ya = *reinterpret_cast<const float4*>(tb + a_);                 \
        const float4 yb = *reinterpret_cast<const float4*>(tb + a_ + 256);           \
        float d_ = XR[0] * ya.x;                                                     \
        d_ = fmaf(XR[1], ya.y, d_); d_ = fmaf(XR[2], ya.z, d_); d_ = fmaf(XR[3], ya.w, d_); \
        d_ = fmaf(XR[4], yb.x, d_); d_ = fmaf(XR[5], yb.y, d_);                      \
        d_ = fmaf(XR[6], yb.z, d_); d_ = fmaf(XR[7], yb.w, d_);                      \
        RES = d_;                                                                    \
        MST_FMA4_BC(JJ, ACC[0], ACC[1], ACC[2], ACC[3], W, ya);                     \
        MST_FMA4_BC(JJ, ACC[4], ACC[5], ACC[6], ACC[7], W, yb);                     \
    } while (0)

#define MSTF_PAIR(JJ, XR, ACC, P)                                                    \
    do {                                                                             \
        float r0, r1;                                                                \
        MSTF_STEP(JJ, cur.x, cur.y, XR, ACC, r0);                                    \
        MSTF_STEP(JJ, cur.z, cur.w, XR, ACC, r1);                                    \
        const float r_ = row_sum_pair(r0, r1, upper);                                \
        if (storer) store_pair_slot(pt + (int64_t)(P) * 8, pbyte, r_);                      \
    } while (0)

// NWF wavefronts per workgroup, QW quads per wavefront (consecutive quads): the slab of a
// workgroup is 4 NWF QW rows.  Two workgroups share a CU: 16 wavefronts of 64 registers or
// 8 wavefronts of 128.
template <typename TIn, int NWF, int QW>
__global__ __launch_bounds__(NWF * 64) __attribute__((amdgpu_waves_per_eu(NWF / 2, NWF / 2)))
void k_bwd_fused(const TIn* __restrict__ dY /* staged [T x K] */, const TIn* __restrict__ X /* registers [T x R] */,
                 const int* __restrict__ ptr, const uint4* __restrict__ ent, const int* __restrict__ rowmap,
                 float* __restrict__ dX /* [T x R], or [nsplit][T x R] partial input gradients */,
                 float* __restrict__ partial, int64_t slots_stride,
                 int T, int K, int R, int NBpad, int nchunk, int nslab, int ntile, int vec_ok, int vec_reg,
                 int chunks_per_split) {
    __shared__ float tile[KC * TT];
    int tile_id, slab;
    if (!block_to_tile(nslab, ntile, tile_id, slab)) return;
    const int tid = threadIdx.x;
    constexpr int nthreads = NWF * 64;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = tile_id * TT;
    const int fq = (slab * NWF + wave) * QW;          // this wavefront's first quad (4 * block + quad)
    const int g = lane >> 4, s = lane & 15;
    const uint32_t lane16 = (uint32_t)s << 4;
    const char* tb = reinterpret_cast<const char*>(tile);
    const uint32_t ebyte = (uint32_t)((lane & 3) * 4 + g) * 16u;
    const bool upper = (s & 8) != 0;
    const bool storer = (s & 7) == 0;
    const uint32_t pbyte = (uint32_t)(g * 2 + (s >> 3)) * 4u;
    float* pt = partial + (int64_t)tile_id * slots_stride;

    constexpr int SLAB_ROWS = NWF * QW * 4;
    constexpr int NCH = SLAB_ROWS / 4;
    const int row0 = slab * SLAB_ROWS;

    // ---- X of this lane's 8 tokens for the row of each of its quads, through LDS (the
    // staging layout of the epilogue below); a spread quad works on the row of lane group 0
    float xr[QW][8];
    {
        int rin[QW];
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            const int rm = rowmap[(fq + q) * 4 + g], rm0 = rowmap[(fq + q) * 4];
            rin[q] = (((rm & SPREAD_FLAG) ? rm0 : rm) & ~SPREAD_FLAG) - row0;
        }
        float* stf = tile;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (h) __syncthreads();
            for (int item = tid; item < 64 * NCH; item += nthreads) {
                const int tl = item / NCH, j = item % NCH;
                const int t = t0 + 64 * h + tl;
                const int row = row0 + 4 * j;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (t < T && row < R) v = load_quad<TIn>(X, R, t, row, T, R, vec_reg != 0);
                *reinterpret_cast<float4*>(stf + (tl * 64 + (j ^ ((tl >> 2) & 15))) * 4) = v;
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < QW; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    xr[q][4 * h + e] = stf[((4 * s + e) * 64 + ((rin[q] >> 2) ^ s)) * 4 + (rin[q] & 3)];
        }
    }

    float acc[QW][8];
#pragma unroll
    for (int q = 0; q < QW; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;

    // blockIdx.y takes a range of chunks (short batches: more workgroups than tiles x slabs).
    // An entry lies in one chunk, so its weight gradient is complete in one workgroup; the
    // input gradient of a range is a partial sum, written to its own [T x R] plane.
    const int c_begin = blockIdx.y * chunks_per_split;
    const int c_end = min(nchunk, c_begin + chunks_per_split);
    dX += (int64_t)blockIdx.y * T * R;
    // first pairs of this wavefront's quads 0 .. QW of a chunk: the same for all lanes, read by scalar
    // loads one chunk ahead
    const int* pw = ptr + fq;
    int pb[QW + 1];
#pragma unroll
    for (int q = 0; q <= QW; ++q) pb[q] = (pw + (int64_t)c_begin * NBpad * 4)[q];
    for (int c = c_begin; c < c_end; ++c) {
        __syncthreads();
        load_tile<TIn, NWF * 64>(tile, dY, K, t0, c * KC, T, K, vec_ok != 0, tid);
        int pb_next[QW + 1];
        const int* pwn = pw + (int64_t)(c + 1 < c_end ? c + 1 : c) * NBpad * 4;
#pragma unroll
        for (int q = 0; q <= QW; ++q) pb_next[q] = pwn[q];
        int p = pb[0];
        uint4 nxt = load_batch(ent, p, ebyte);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            const int pend = pb[q + 1];
            while (p < pend) {
                const uint4 cur = nxt;
                const int pn = min(p + 4, pend);
                nxt = load_batch(ent, pn, ebyte);
                MSTF_PAIR(0, xr[q], acc[q], p);
                if (p + 1 < pend) {
                    MSTF_PAIR(1, xr[q], acc[q], p + 1);
                    if (p + 2 < pend) {
                        MSTF_PAIR(2, xr[q], acc[q], p + 2);
                        if (p + 3 < pend) MSTF_PAIR(3, xr[q], acc[q], p + 3);
                    }
                }
                p = pn;
            }
        }
#pragma unroll
        for (int q = 0; q <= QW; ++q) pb[q] = pb_next[q];
    }

    // ---- input gradient out: through LDS, 64 tokens at a time (token tl owns 1 KB, the
    // 16-byte chunk j of rows 4j..4j+3 of the slab at slot j ^ ((tl >> 2) & 15))
    // (the rows of the accumulators are read from the row map again, and the lane constants worked out
    // again, rather than kept in registers across the walk)
    int tid_e = threadIdx.x;
    asm volatile("" : "+v"(tid_e));
    const int g_e = (tid_e >> 4) & 3, s_e = tid_e & 15;
    int rout[QW];
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int rm = rowmap[(fq + q) * 4 + g_e];
        fold_spread(acc[q], rm & SPREAD_FLAG, g_e);
        rout[q] = (rm & ~SPREAD_FLAG) - row0;
    }
    float* stf = tile;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int tl = 4 * s_e + e;
#pragma unroll
            for (int q = 0; q < QW; ++q)
                stf[(tl * 64 + ((rout[q] >> 2) ^ s_e)) * 4 + (rout[q] & 3)] = acc[q][4 * h + e];
        }
        __syncthreads();
        for (int item = tid_e; item < 64 * NCH; item += nthreads) {
            const int tl = item / NCH, j = item % NCH;
            const int t = t0 + 64 * h + tl;
            const int row = row0 + 4 * j;
            if (t >= T || row >= R) continue;
            const float4 v = *reinterpret_cast<const float4*>(stf + (tl * 64 + (j ^ ((tl >> 2) & 15))) * 4);
            float* o = dX + (int64_t)t * R + row;
            if (vec_reg && row + 3 < R) {
                typedef float f4 __attribute__((ext_vector_type(4)));
                f4 vv = {v.x, v.y, v.z, v.w};
                __builtin_nontemporal_store(vv, reinterpret_cast<f4*>(o));
            } else {
                __builtin_nontemporal_store(v.x, o);
                if (row + 1 < R) __builtin_nontemporal_store(v.y, o + 1);
                if (row + 2 < R) __builtin_nontemporal_store(v.z, o + 2);
                if (row + 3 < R) __builtin_nontemporal_store(v.w, o + 3);
            }
        }
    }
}

// dW[perm[e]] = sum over token tiles of partial[tile][e], tiles added in ascending order
__global__ void k_bwd_fused_reduce(const float* __restrict__ partial, int64_t slots_stride, int ntile,
                                   const int* __restrict__ ptr, int64_t nseg, const int* __restrict__ perm,
                                   float* __restrict__ dW) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)ptr[nseg] * 8) return;
    const int p = perm[e];
    if (p < 0) return;
    dW[p] = ordered_plane_sum(partial + e, slots_stride, ntile);
}

// dX[k] = sum of the nsplit partial planes, added in ascending order
__global__ void k_sum_planes(const float* __restrict__ planes, int64_t n, int nsplit, float* __restrict__ out) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n) return;
    float sum = planes[k];
    for (int z = 1; z < nsplit; ++z) sum += planes[(int64_t)z * n + k];
    out[k] = sum;
}

template <typename TIn, int NWF, int QW>
static void launch_fused(const View& v, const TIn* dY, const TIn* X, float* dX, float* partial, int T, int nsplit,
                         hipStream_t s) {
    const int ntile = (int)cdiv(T, TT);
    const int nslab = (int)cdiv((int64_t)v.NB * 4, NWF * QW);
    const int cps = (int)cdiv(v.nchunk, nsplit);
    k_bwd_fused<TIn, NWF, QW><<<dim3(grid_for(ntile, nslab), (unsigned)nsplit), NWF * 64, 0, s>>>(
        dY, X, v.ptr, v.ent, v.rowmap, dX, partial, v.cap_pairs * 8, T, v.K, v.R, v.NBpad, v.nchunk, nslab, ntile,
        (v.K % 4 == 0) ? 1 : 0, (v.R % 4 == 0) ? 1 : 0, cps);
}

// Launch shapes: 8 wavefronts x 3, 4 or 5 quads (96-, 128-, 160-row slabs, up to 128 registers per lane)
// or 16 wavefronts x 1 or 2 quads (64- / 128-row slabs, 64 registers per lane).  All give the same results.
struct FusedShape {
    int waves, quads;
};
static FusedShape g_forced_fused = {0, 0};

int bwd_fused_force_shape(int waves, int quads) {
    const bool ok = (waves == 0 && quads == 0) || (waves == 8 && quads >= 3 && quads <= 5) || (waves == 16 && quads <= 2 && quads >= 1);
    if (!ok) return MST_ERR_ARG;
    g_forced_fused = {waves, quads};
    return MST_OK;
}

// The shared walk is used at every density of the sparse path: over GPT-2 small / medium /
// large shapes it beats the two separate kernels by 1.16 on average at density 0.02 and 1.26
// at 0.20 (uniform masks), and equals them on power-law masks at 0.02.
bool bwd_fused_pays(const mst_layer*) { return true; }

// Cost of one workgroup (walk, staging of dY, the X rows of the slab, per-chunk overhead and a
// fixed amount per quad segment a wavefront walks) times the rounds its grid needs on 256 CUs x 2
// workgroups, as for the SpMM launch shapes; one set of constants for the shapes of 8 wavefronts,
// one for those of 16, fitted to timings of the five shapes on twelve GPT-2 small / medium / large
// layer shapes at densities 0.02 .. 0.10 and 4096 .. 16384 tokens on MI355X (144 cases: the choice
// is 0.2 % slower than the best shape on average, 7 % at worst; 16 x 2 is the best in two thirds).
static FusedShape pick_fused_shape(int T, int R, int K, double density) {
    if (g_forced_fused.waves != 0) return g_forced_fused;
    struct Cls {
        double kWalk, kStage, kReg, kChunk, kLoneTail, kLoneOnly, kSeg;
    };
    static const Cls cls[2] = {{5.675e-5, 6.23e-5, 7.598e-4, 1.352, 0.633, 0.762, 0.287},     // 8 wavefronts
                               {4.706e-5, 5.52e-5, 7.846e-4, 1.225, 0.580, 0.698, 0.392}};    // 16 wavefronts
    static const FusedShape cand[] = {{8, 3}, {8, 4}, {8, 5}, {16, 1}, {16, 2}};
    const int64_t nchunk = cdiv(K, KC), ntile = cdiv(T, TT);
    FusedShape best = cand[3];
    double best_cost = 0.0;
    for (const FusedShape& sh : cand) {
        const Cls& c = cls[sh.waves == 8 ? 0 : 1];
        const int rows = sh.waves * sh.quads * 4;
        const int64_t nslab = cdiv(R, rows), nwg = ntile * nslab;
        const double rows_eff = (double)R / (double)nslab;
        const double wg = TT * (rows_eff * density * K * c.kWalk + (double)nchunk * KC * c.kStage + rows * c.kReg) +
                          c.kChunk * (double)nchunk + c.kSeg * (double)sh.quads * (double)nchunk;
        const int64_t full = nwg / 512, rest = nwg % 512;
        double rounds;
        if (full == 0) rounds = rest <= 256 ? c.kLoneOnly : 1.0;
        else rounds = (double)full + (rest == 0 ? 0.0 : rest <= 256 ? c.kLoneTail : 1.0);
        const double cost = wg * rounds;
        if (best_cost == 0.0 || cost < best_cost) {
            best_cost = cost;
            best = sh;
        }
    }
    return best;
}

// Short batches leave most CUs without a workgroup and every workgroup with a long chain of
// chunks: the chunk range is then split over up to 8 workgroups (as many as keep the grid
// within one round and the partial input gradients within `plane_floats`).  A forced launch
// shape runs unsplit.
static int pick_chunk_split(int T, const View& v, size_t plane_floats) {
    if (g_forced_fused.waves != 0) return 1;
    const int64_t nwg = cdiv(T, TT) * cdiv(v.R, 64);
    if (nwg > 256 || v.nchunk < 12) return 1;     // short chunk chains gain less than the extra pass costs
    int64_t n = std::min<int64_t>({8, v.nchunk / 2, 512 / nwg, (int64_t)(plane_floats / ((size_t)T * v.R))});
    if (n < 2) return 1;
    const int64_t cps = cdiv(v.nchunk, n);
    return (int)cdiv(v.nchunk, cps);                  // no empty range
}

template <typename TIn>
static int launch_fused_any(const View& v, const TIn* dY, const TIn* X, float* dX, const Workspace& ws, int T,
                            double density, hipStream_t s) {
    const int nsplit = pick_chunk_split(T, v, ws.gemm_floats);
    if (nsplit > 1) {
        launch_fused<TIn, 16, 1>(v, dY, X, ws.gemm, ws.partial, T, nsplit, s);
        MST_LAUNCH_CHECK();
        const int64_t n = (int64_t)T * v.R;
        k_sum_planes<<<(unsigned)cdiv(n, 256), 256, 0, s>>>(ws.gemm, n, nsplit, dX);
        MST_LAUNCH_CHECK();
        return MST_OK;
    }
    const FusedShape sh = pick_fused_shape(T, v.R, v.K, density);
    if (sh.waves == 16 && sh.quads == 2) launch_fused<TIn, 16, 2>(v, dY, X, dX, ws.partial, T, 1, s);
    else if (sh.waves == 8 && sh.quads == 5) launch_fused<TIn, 8, 5>(v, dY, X, dX, ws.partial, T, 1, s);
    else if (sh.waves == 8 && sh.quads == 4) launch_fused<TIn, 8, 4>(v, dY, X, dX, ws.partial, T, 1, s);
    else if (sh.waves == 8) launch_fused<TIn, 8, 3>(v, dY, X, dX, ws.partial, T, 1, s);
    else launch_fused<TIn, 16, 1>(v, dY, X, dX, ws.partial, T, 1, s);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int bwd_fused(const mst_layer* L, const void* dY, const void* X, float* dX, float* dW, int T, mst_dtype act,
              const Workspace& ws, hipStream_t s) {
    const View& v = L->col;
    const double density = (double)L->nnz / (double)L->N;
    const int rc = (act == MST_F32)
        ? launch_fused_any<float>(v, static_cast<const float*>(dY), static_cast<const float*>(X), dX, ws, T, density, s)
        : launch_fused_any<uint16_t>(v, static_cast<const uint16_t*>(dY), static_cast<const uint16_t*>(X), dX, ws, T,
                                     density, s);
    if (rc != MST_OK) return rc;
    if (L->nnz > 0) {
        const int64_t upper = 4 * (L->nnz + (int64_t)v.nchunk * v.NB * 4);
        k_bwd_fused_reduce<<<(unsigned)cdiv(upper, 256), 256, 0, s>>>(ws.partial, v.cap_pairs * 8, (int)cdiv(T, TT), v.ptr,
                                                                      v.nseg, v.perm, dW);
        MST_LAUNCH_CHECK();
    }
    return MST_OK;
}

}  // namespace mst
