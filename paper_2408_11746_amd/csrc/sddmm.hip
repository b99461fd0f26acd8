// SDDMM over the active index list:  dW[o, i] = sum_t dY[t, o] X[t, i]  for the active
// (o, i) only (the weight-gradient half of the backward pass; App. "FLOP Calculation",
// backward = 2 x forward).
//
// Same decomposition and lane mapping as the SpMM: a workgroup owns TT = 128 tokens and
// two to four quads of the driving view per wavefront, stages chunks of one dense operand
// in LDS and walks the ELL slices (written below for the row view: X is staged, dY sits in
// registers; the col view swaps the two).  A lane keeps dY of its 8 tokens for the row of
// its lane group in every quad (brought in through LDS so that the global reads are
// contiguous); entries reach the lanes as in the SpMM (batches of four pairs, handed round
// the groups of four lanes through DPP operands).  Per step a lane reads its 8 X values
// of the entry's column from LDS and forms the 8-term dot product; the sums over the 16
// lanes of a group are taken for the two entries of a pair together with DPP adds -- all
// four lane groups at once, no LDS traffic.  One lane per entry stores the per-(token
// tile, entry slot) partial sum; a second kernel adds the partials of all token tiles in a
// fixed order (deterministic, no floating-point atomics) and writes the result at the
// entry's canonical position.
#include "tile_loader.h"
#include "walk_ops.h"

namespace mst {

// this lane's share (8 tokens) of the dot product of one entry
#define MST_DOT(JJ, OFF, DY, RES)                                                    \
    do {                                                                             \
        const uint32_t a_ = lane16 ^ quad_bcast<JJ>(OFF);                            \
        const float4 xa = *reinterpret_cast<const float4*>(tb + a_);                 \
        const float4 xb = *reinterpret_cast<const float4*>(tb + a_ + 256);           \
        float d_ = DY[0] * xa.x;                                                     \
        d_ = fmaf(DY[1], xa.y, d_); d_ = fmaf(DY[2], xa.z, d_); d_ = fmaf(DY[3], xa.w, d_); \
        d_ = fmaf(DY[4], xb.x, d_); d_ = fmaf(DY[5], xb.y, d_);                      \
        d_ = fmaf(DY[6], xb.z, d_); d_ = fmaf(DY[7], xb.w, d_);                      \
        RES = d_;                                                                    \
    } while (0)

// partial sums of the pair held by lane JJ of each group of four lanes: lane 0 of a lane
// group stores the first entry's sum, lane 8 the second's
#define MST_DOT_PAIR(JJ, DY, P)                                                      \
    do {                                                                             \
        float r0, r1;                                                                \
        MST_DOT(JJ, cur.x, DY, r0);                                                  \
        MST_DOT(JJ, cur.z, DY, r1);                                                  \
        const float r_ = row_sum_pair(r0, r1, upper);                                \
        if (storer) store_pair_slot(pt + (int64_t)(P) * 8, pbyte, r_);                      \
    } while (0)

constexpr int NW = 16;      // wavefronts per workgroup

// One driving view's operands: its ELL arrays, the dense operand it stages in LDS and the one
// its lanes keep in registers.
template <typename TIn>
struct SddmmSide {
    const TIn* __restrict__ staged;      // [T x K]
    const TIn* __restrict__ inreg;       // [T x R]
    const int* __restrict__ ptr;
    const uint4* __restrict__ ent;
    const int* __restrict__ rowmap;
    const int* __restrict__ perm;
    int64_t slots_stride;                // partial-sum slots per token tile
    int64_t nseg;
    int K, R, NBpad, nchunk, nslab, vec_ok, vec_reg;
};

// QW = quads per wavefront (consecutive quads, which may cross row blocks): the slab of a
// workgroup is 64 QW rows of the driving view
template <typename TIn, int QW>
__device__ __forceinline__ void sddmm_side(const SddmmSide<TIn>& a, float* __restrict__ tile, float* __restrict__ partial,
                                           int T, int ntile) {
    const TIn* __restrict__ X = a.staged;
    const TIn* __restrict__ dY = a.inreg;
    const int* __restrict__ ptr = a.ptr;
    const uint4* __restrict__ ent = a.ent;
    const int* __restrict__ rowmap = a.rowmap;
    const int64_t slots_stride = a.slots_stride;
    const int K = a.K, R = a.R, NBpad = a.NBpad, nchunk = a.nchunk, nslab = a.nslab;
    const int vec_ok = a.vec_ok, vec_reg = a.vec_reg;
    int tile_id, slab;
    if (!block_to_tile(nslab, ntile, tile_id, slab)) return;
    const int tid = threadIdx.x;
    constexpr int nthreads = NW * 64;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = tile_id * TT;
    const int fq = (slab * NW + wave) * QW;           // this wavefront's first quad (4 * block + quad)
    const int g = lane >> 4, s = lane & 15;
    const uint32_t lane16 = (uint32_t)s << 4;
    const char* tb = reinterpret_cast<const char*>(tile);
    const uint32_t ebyte = (uint32_t)((lane & 3) * 4 + g) * 16u;              // this lane's 16 bytes of a batch of four pairs
    const bool upper = (s & 8) != 0;
    const bool storer = (s & 7) == 0;
    const uint32_t pbyte = (uint32_t)(g * 2 + (s >> 3)) * 4u;               // slot of this lane's sum inside a pair's eight
    // partial sums of this token tile: eight per pair, (lane group, step of the pair)
    float* pt = partial + (int64_t)tile_id * slots_stride;

    // ---- register operand: dY of this lane's 8 tokens for the row of each of its quads.
    // It comes in through LDS, 64 tokens at a time: the workgroup reads the slab's columns
    // of 64 token rows as whole contiguous runs into the staging layout the SpMM epilogue
    // uses (token tl owns 1 KB, the 16-byte chunk j of rows 4j..4j+3 at slot
    // j ^ ((tl >> 2) & 15)), then every lane picks its rows' values.
    constexpr int SLAB_ROWS = NW * QW * 4;
    constexpr int NCH = SLAB_ROWS / 4;
    const int row0 = slab * SLAB_ROWS;
    float dy[QW][8];
    int rloc[QW];
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        // a spread quad: all four lane groups work on the row of lane group 0
        const int rm = rowmap[(fq + q) * 4 + g], rm0 = rowmap[(fq + q) * 4];
        rloc[q] = (((rm & SPREAD_FLAG) ? rm0 : rm) & ~SPREAD_FLAG) - row0;
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
            if (t < T && row < R) v = load_quad<TIn>(dY, R, t, row, T, R, vec_reg != 0);
            *reinterpret_cast<float4*>(stf + (tl * 64 + (j ^ ((tl >> 2) & 15))) * 4) = v;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < QW; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                dy[q][4 * h + e] = stf[((4 * s + e) * 64 + ((rloc[q] >> 2) ^ s)) * 4 + (rloc[q] & 3)];
    }

    // first pairs of this wavefront's quads 0 .. QW of a chunk: the same for all lanes, read by scalar
    // loads one chunk ahead
    const int* pw = ptr + fq;
    int pb[QW + 1];
#pragma unroll
    for (int q = 0; q <= QW; ++q) pb[q] = pw[q];
    for (int c = 0; c < nchunk; ++c) {
        __syncthreads();
        load_tile<TIn, NW * 64>(tile, X, K, t0, c * KC, T, K, vec_ok != 0, tid);
        int pb_next[QW + 1];
        const int* pwn = pw + (int64_t)(c + 1 < nchunk ? c + 1 : c) * NBpad * 4;
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
#pragma unroll
        for (int q = 0; q <= QW; ++q) pb[q] = pb_next[q];
    }
}

// Either view can drive the product; which one does is a device-side flag set when the views
// were built.  One launch serves both: its grid covers the larger of the two, and every
// workgroup takes the side the flag names (QW0 quads per wavefront for the row view, QW1
// for the col view).
template <typename TIn, int QW0, int QW1>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(8, 8)))
void k_sddmm(const SddmmSide<TIn> row, const SddmmSide<TIn> col, float* __restrict__ partial, int T, int ntile,
             const int* __restrict__ choice) {
    __shared__ float tile[KC * TT];
    if (*choice) sddmm_side<TIn, QW1>(col, tile, partial, T, ntile);
    else sddmm_side<TIn, QW0>(row, tile, partial, T, ntile);
}

// dW[perm[e]] = sum over token tiles of partial[tile][e], tiles added in ascending order
template <typename TIn>
__global__ void k_sddmm_reduce(const float* __restrict__ partial, int ntile, const SddmmSide<TIn> row,
                               const SddmmSide<TIn> col, float* __restrict__ dW, const int* __restrict__ choice) {
    const bool c = *choice != 0;                      // field by field: the arguments stay in scalar registers
    const int* __restrict__ ptr = c ? col.ptr : row.ptr;
    const int* __restrict__ perm = c ? col.perm : row.perm;
    const int64_t nseg = c ? col.nseg : row.nseg;
    const int64_t slots_stride = c ? col.slots_stride : row.slots_stride;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)ptr[nseg] * 8) return;
    const int p = perm[e];
    if (p < 0) return;
    dW[p] = ordered_plane_sum(partial + e, slots_stride, ntile);
}

// Quads per wavefront (2, 3 or 4: slabs of 128, 192 or 256 rows), by the cost model of the
// SpMM launch shapes: the cost of one workgroup (walk, staging of both dense operands,
// per-chunk overhead) times the rounds the grid needs on 256 CUs x 2 workgroups, a last
// round with at most one workgroup per CU costing less.  Constants fitted to timings of
// GPT-2 small / medium / large layer shapes at densities 0.02 .. 0.10 on MI355X.  Every
// choice adds the same terms in the same order.
static int pick_sddmm_quads(int T, int R, int K, double density) {
    const double kWalk = 3.71e-5, kStage = 3.0e-5, kReg = 9.96e-4, kChunk = 1.57;
    const double kLoneTail = 0.51, kLoneOnly = 0.58;
    const int64_t nchunk = cdiv(K, KC), ntile = cdiv(T, TT);
    int best = 4;
    double best_cost = 0.0;
    for (int qw = 2; qw <= 4; ++qw) {
        const int rows = NW * qw * 4;
        const int64_t nslab = cdiv(R, rows), nwg = ntile * nslab;
        const double rows_eff = (double)R / (double)nslab;
        const double wg = TT * (rows_eff * density * K * kWalk + (double)nchunk * KC * kStage + rows * kReg) +
                          kChunk * (double)nchunk;
        const int64_t full = nwg / 512, rest = nwg % 512;
        double rounds;
        if (full == 0) rounds = rest <= 256 ? kLoneOnly : 1.0;
        else rounds = (double)full + (rest == 0 ? 0.0 : rest <= 256 ? kLoneTail : 1.0);
        const double cost = wg * rounds;
        if (best_cost == 0.0 || cost < best_cost) {
            best_cost = cost;
            best = qw;
        }
    }
    return best;
}

template <typename TIn, int QW0, int QW1>
static void launch_k(const SddmmSide<TIn>& row, const SddmmSide<TIn>& col, float* partial, int T, int ntile,
                     const int* choice, hipStream_t s) {
    const unsigned grid = std::max(grid_for(ntile, row.nslab), grid_for(ntile, col.nslab));
    k_sddmm<TIn, QW0, QW1><<<grid, NW * 64, 0, s>>>(row, col, partial, T, ntile, choice);
}

template <typename TIn, int QW0>
static void launch_q(int qw1, const SddmmSide<TIn>& row, const SddmmSide<TIn>& col, float* partial, int T, int ntile,
                     const int* choice, hipStream_t s) {
    if (qw1 == 4) launch_k<TIn, QW0, 4>(row, col, partial, T, ntile, choice, s);
    else if (qw1 == 3) launch_k<TIn, QW0, 3>(row, col, partial, T, ntile, choice, s);
    else launch_k<TIn, QW0, 2>(row, col, partial, T, ntile, choice, s);
}

// The product is symmetric in its two dense operands: either view can drive it.  The row
// view stages X and keeps dY in registers, the col view stages dY and keeps X in registers.
// The host does not know which one the layer uses (that would take a synchronisation after
// the views were built), so it passes both sides to one launch of each kernel.
template <typename TIn>
static int launch_sddmm(const mst_layer* L, const TIn* dY, const TIn* X, float* dW, int T,
                        const Workspace& ws, hipStream_t s) {
    const int ntile = (int)cdiv(T, TT);
    SddmmSide<TIn> side[2];
    int qw[2];
    int64_t upper = 0;
    for (int me = 0; me < 2; ++me) {
        const View& v = me ? L->col : L->row;
        qw[me] = pick_sddmm_quads(T, v.R, v.K, (double)L->nnz / ((double)v.R * (double)v.K));
        SddmmSide<TIn>& a = side[me];
        a.staged = me ? dY : X;
        a.inreg = me ? X : dY;
        a.ptr = v.ptr;
        a.ent = v.ent;
        a.rowmap = v.rowmap;
        a.perm = v.perm;
        a.slots_stride = v.cap_pairs * 8;
        a.nseg = v.nseg;
        a.K = v.K;
        a.R = v.R;
        a.NBpad = v.NBpad;
        a.nchunk = v.nchunk;
        a.nslab = (int)cdiv((int64_t)v.NB * 4, NW * qw[me]);
        a.vec_ok = (v.K % 4 == 0) ? 1 : 0;
        a.vec_reg = (v.R % 4 == 0) ? 1 : 0;
        upper = std::max(upper, 4 * (L->nnz + (int64_t)v.nchunk * v.NB * 4));
    }
    if (qw[0] == 4) launch_q<TIn, 4>(qw[1], side[0], side[1], ws.partial, T, ntile, L->sddmm_view, s);
    else if (qw[0] == 3) launch_q<TIn, 3>(qw[1], side[0], side[1], ws.partial, T, ntile, L->sddmm_view, s);
    else launch_q<TIn, 2>(qw[1], side[0], side[1], ws.partial, T, ntile, L->sddmm_view, s);
    MST_LAUNCH_CHECK();
    k_sddmm_reduce<TIn><<<(unsigned)cdiv(upper, 256), 256, 0, s>>>(ws.partial, ntile, side[0], side[1], dW, L->sddmm_view);
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
