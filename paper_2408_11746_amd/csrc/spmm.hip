// SpMM:  out[T x R] = A[T x K] * S^T  with S [R x K] unstructured-sparse.
// Serves the forward product (S = W, A = X; App. "FLOP Calculation" Eq. (1)) and the
// input gradient (S = W^T, A = dY; the first half of the backward pass).
//
// A workgroup of 16 wavefronts owns a tile of tokens (128 in k_spmm, 64 in k_spmm64) and a
// slab of rows (64 rows per quad-per-wavefront: 128 .. 512).  It walks the contraction index
// in chunks of KC: the chunk of A is staged (transposed) in LDS, then each wavefront walks
// the ELL slices of its quads.  A wavefront is four lane groups of 16 lanes; in one step
// each lane group multiplies ONE entry (its own row of the quad) with all tokens of the
// tile, 8 (4) per lane.  The entries {offset, weight} come straight from global memory:
// a lane loads 16 bytes (one pair of its lane group) of a batch of four pairs, the next
// batch is in flight while the current one is used, and the four lanes of a group of four
// hand their pairs round through DPP operands of the address XOR and of the FMAs.  The
// activations come from 16-byte LDS reads; the accumulators of a row stay in registers for
// the whole K loop.  Nothing in the inner loop touches LDS for entries, the scalar unit or
// a lane outside the group of four.  The result tile leaves through LDS so that global
// stores are contiguous runs of the slab's columns.
#include "tile_loader.h"
#include "walk_ops.h"

namespace mst {

// one step: entry {OFF, W} as held by lane JJ of the group of four lanes
#define MST_STEP(JJ, OFF, W, ACC)                                                    \
    do {                                                                             \
        const uint32_t a_ = lane16 ^ quad_bcast<JJ>(OFF);                            \
        const float4 xa = *reinterpret_cast<const float4*>(tb + a_);                 \
        const float4 xb = *reinterpret_cast<const float4*>(tb + a_ + 256);           \
        MST_FMA4_BC(JJ, ACC[0], ACC[1], ACC[2], ACC[3], W, xa);                      \
        MST_FMA4_BC(JJ, ACC[4], ACC[5], ACC[6], ACC[7], W, xb);                      \
    } while (0)

// the pair held by lane JJ of each group of four lanes: both of its steps
#define MST_PAIR(JJ, ACC)                                                            \
    do {                                                                             \
        MST_STEP(JJ, cur.x, cur.y, ACC);                                             \
        MST_STEP(JJ, cur.z, cur.w, ACC);                                             \
    } while (0)

constexpr int NW = 16;      // wavefronts per workgroup

// QW = quads per wavefront (2, 3 or 4 consecutive quads, which may cross row blocks): the
// slab of a workgroup is 64 QW rows.
template <typename TIn, int QW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_spmm(
    const TIn* __restrict__ A, const int* __restrict__ ptr, const uint4* __restrict__ ent,
    const int* __restrict__ rowmap, float* __restrict__ out,
    int T, int K, int R, int NBpad, int nchunk, int nslab, int ntile, int vec_ok, int vec_store) {
    __shared__ float tile[KC * TT];
    int tile_id, slab;
    if (!block_to_tile(nslab, ntile, tile_id, slab)) return;
    const int tid = threadIdx.x;
    constexpr int nthreads = NW * 64, nw = NW;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = tile_id * TT;
    const int fq = (slab * nw + wave) * QW;           // this wavefront's first quad (4 * block + quad)
    const int g = lane >> 4, s = lane & 15;
    const uint32_t lane16 = (uint32_t)s << 4;
    const char* tb = reinterpret_cast<const char*>(tile);
    // a batch is four consecutive pairs: lane (g, j = lane & 3) holds lane group g's
    // 16 bytes of pair j of the batch, the four lanes of a group of four hand them round
    const uint32_t ebyte = (uint32_t)((lane & 3) * 4 + g) * 16u;

    float acc[QW][8];
#pragma unroll
    for (int q = 0; q < QW; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;

    // first pairs of this wavefront's quads 0 .. QW of the current chunk: the same for all lanes, so they
    // come through scalar loads into scalar registers, one chunk ahead
    const int* pw = ptr + fq;
    int pb[QW + 1];
#pragma unroll
    for (int q = 0; q <= QW; ++q) pb[q] = pw[q];
    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) __syncthreads();
        load_tile<TIn, NW * 64>(tile, A, K, t0, c * KC, T, K, vec_ok != 0, tid);
        int pb_next[QW + 1];
        const int* pwn = pw + (int64_t)(c + 1 < nchunk ? c + 1 : c) * NBpad * 4;
#pragma unroll
        for (int q = 0; q <= QW; ++q) pb_next[q] = pwn[q];
        int p = pb[0];
        uint4 nxt = load_batch(ent, p, ebyte);               // (reads past the end stay in the tail)
        __syncthreads();
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            const int pend = pb[q + 1];
            while (p < pend) {
                // batch = pairs p .. p+3 of this slice; the following batch starts at p + 4
                // or, when the slice ends before that, at the first pair of the next slice
                const uint4 cur = nxt;
                const int pn = min(p + 4, pend);
                nxt = load_batch(ent, pn, ebyte);            // (at most 4 pairs past the end: next block or tail)
                MST_PAIR(0, acc[q]);
                if (p + 1 < pend) {
                    MST_PAIR(1, acc[q]);
                    if (p + 2 < pend) {
                        MST_PAIR(2, acc[q]);
                        if (p + 3 < pend) MST_PAIR(3, acc[q]);
                    }
                }
                p = pn;
            }
        }
#pragma unroll
        for (int q = 0; q <= QW; ++q) pb[q] = pb_next[q];
    }

    // (the epilogue works its lane constants out again instead of keeping the prologue's alive --
    // in scratch memory -- across the chunk loop)
    int tid_e = threadIdx.x;
    asm volatile("" : "+v"(tid_e));
    const int g_e = (tid_e >> 4) & 3, s_e = tid_e & 15;

    // rows of this lane's accumulators: place g of quad fq + q
    int rloc[QW];
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int rm = rowmap[(fq + q) * 4 + g_e];
        fold_spread(acc[q], rm & SPREAD_FLAG, g_e);
        rloc[q] = rm & ~SPREAD_FLAG;
    }

    // ---- epilogue: through LDS, 64 tokens at a time, so that each token's outputs of the
    // whole slab leave as one contiguous run.  Staging layout: token tl (0..63) owns 1 KB;
    // the 16-byte chunk j (rows 4j..4j+3 of the slab) sits at slot j ^ ((tl >> 2) & 15).
    constexpr int SLAB_ROWS = NW * QW * 4;
    const int row0 = slab * SLAB_ROWS;                // first row of the slab
#pragma unroll
    for (int q = 0; q < QW; ++q) rloc[q] -= row0;     // position inside the slab's token row
    float* stf = tile;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        __syncthreads();                              // tile / previous half no longer read
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int tl = 4 * s_e + e;
#pragma unroll
            for (int q = 0; q < QW; ++q)
                stf[(tl * 64 + ((rloc[q] >> 2) ^ s_e)) * 4 + (rloc[q] & 3)] = acc[q][4 * h + e];
        }
        __syncthreads();
        constexpr int NCH = SLAB_ROWS / 4;            // 16-byte chunks per token row of the slab
        for (int item = tid_e; item < 64 * NCH; item += nthreads) {
            const int tl = item / NCH, j = item % NCH;
            const int t = t0 + 64 * h + tl;
            const int row = row0 + 4 * j;
            if (t >= T || row >= R) continue;
            const float4 v = *reinterpret_cast<const float4*>(stf + (tl * 64 + (j ^ ((tl >> 2) & 15))) * 4);
            float* o = out + (int64_t)t * R + row;
            // streaming stores: the output is not read again by this kernel and should not
            // push the activation tiles out of the L2
            if (vec_store && row + 3 < R) {
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

// ---- 64-token variant.  Same walk with half as many tokens per lane (one 16-byte LDS read
// and four FMAs per step); a wavefront owns QW consecutive quads, which may cross row
// blocks, so a workgroup's slab is 64 QW rows (128 .. 512).  Twice as many token tiles and
// the free choice of QW let the grid match the chip where the 128-token kernel leaves
// CUs idle, and a wide slab re-reads the activations less often.  The tile uses the first
// 256 bytes of every 512-byte row of the 128-token layout, so the entries' stored offsets
// serve both kernels.
#define MST_STEP64(JJ, OFF, W, ACC)                                                  \
    do {                                                                             \
        const uint32_t a_ = lane16 ^ quad_bcast<JJ>(OFF);                            \
        const float4 xa = *reinterpret_cast<const float4*>(tb + a_);                 \
        MST_FMA4_BC(JJ, ACC[0], ACC[1], ACC[2], ACC[3], W, xa);                      \
    } while (0)
#define MST_PAIR64(JJ, ACC)                                                          \
    do {                                                                             \
        MST_STEP64(JJ, cur.x, cur.y, ACC);                                           \
        MST_STEP64(JJ, cur.z, cur.w, ACC);                                           \
    } while (0)

constexpr int TT64 = 64;

// 64 tokens x KC indices into the first half of each tile row.  Work item = (token quad,
// index quad, row pair): two 16-byte row reads, four 8-byte LDS stores; 1024 items.
template <typename TIn>
__device__ inline void load_tile64(float* tile, const TIn* __restrict__ A, int64_t lda, int t0, int k0, int T,
                                   int K, bool vec_ok, int tid) {
    char* base = reinterpret_cast<char*>(tile);
    asm volatile("" : "+v"(tid));                     // (offsets worked out per tile, see load_tile)
    const int kq = tid & 31, h = (tid >> 5) & 1, tq = tid >> 6;
    const int row = t0 + 4 * tq + 2 * h, k = k0 + 4 * kq;
    float4 a, b;
    if (vec_ok && t0 + TT64 <= T && k0 + KC <= K) {       // uniform: tile wholly inside the matrix
        const TIn* corner = A + (int64_t)t0 * lda + k0;     // scalar; the lane adds a 32-bit byte offset
        const uint32_t ld = (uint32_t)lda * (uint32_t)sizeof(TIn);
        const __amdgpu_buffer_rsrc_t rs = buffer_of(corner, (uint32_t)(TT64 - 1) * ld + (uint32_t)(KC * sizeof(TIn)));
        const uint32_t o = (uint32_t)(4 * tq + 2 * h) * ld + (uint32_t)(4 * kq * sizeof(TIn));
        a = buffer_quad<TIn>(rs, o);
        b = buffer_quad<TIn>(rs, o + ld);
    } else {
        a = load_quad<TIn>(A, lda, row, k, T, K, vec_ok);
        b = load_quad<TIn>(A, lda, row + 1, k, T, K, vec_ok);
    }
    const uint32_t sl = ((uint32_t)(tq ^ (kq & 15)) << 4) | (uint32_t)(h << 3);
    const uint32_t kl = 4u * kq;
    *reinterpret_cast<float2*>(base + (((kl + 0) << 9) | sl)) = make_float2(a.x, b.x);
    *reinterpret_cast<float2*>(base + (((kl + 1) << 9) | sl)) = make_float2(a.y, b.y);
    *reinterpret_cast<float2*>(base + (((kl + 2) << 9) | sl)) = make_float2(a.z, b.z);
    *reinterpret_cast<float2*>(base + (((kl + 3) << 9) | sl)) = make_float2(a.w, b.w);
}

template <typename TIn, int QW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_spmm64(
    const TIn* __restrict__ A, const int* __restrict__ ptr, const uint4* __restrict__ ent,
    const int* __restrict__ rowmap, float* __restrict__ out,
    int T, int K, int R, int NBpad, int nchunk, int nslab, int ntile, int vec_ok, int vec_store) {
    __shared__ float tile[KC * TT];
    int tile_id, slab;
    if (!block_to_tile(nslab, ntile, tile_id, slab)) return;
    const int tid = threadIdx.x;
    constexpr int nthreads = NW * 64;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = tile_id * TT64;
    const int fq = (slab * NW + wave) * QW;           // this wavefront's first quad (4 * block + quad)
    const int g = lane >> 4, s = lane & 15;
    const uint32_t lane16 = (uint32_t)s << 4;
    const char* tb = reinterpret_cast<const char*>(tile);
    const uint32_t ebyte = (uint32_t)((lane & 3) * 4 + g) * 16u;

    float acc[QW][4];
#pragma unroll
    for (int q = 0; q < QW; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[q][e] = 0.f;

    const int* pw = ptr + fq;                         // (scalar loads, one chunk ahead, as in k_spmm)
    int pb[QW + 1];
#pragma unroll
    for (int q = 0; q <= QW; ++q) pb[q] = pw[q];
    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) __syncthreads();
        load_tile64<TIn>(tile, A, K, t0, c * KC, T, K, vec_ok != 0, tid);
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
                MST_PAIR64(0, acc[q]);
                if (p + 1 < pend) {
                    MST_PAIR64(1, acc[q]);
                    if (p + 2 < pend) {
                        MST_PAIR64(2, acc[q]);
                        if (p + 3 < pend) MST_PAIR64(3, acc[q]);
                    }
                }
                p = pn;
            }
        }
#pragma unroll
        for (int q = 0; q <= QW; ++q) pb[q] = pb_next[q];
    }

    // ---- epilogue: through LDS in passes of 256 slab rows; as in the 128-token kernel a
    // token owns 1 KB of staging and chunk j (rows 4j..4j+3 of the pass) sits at slot
    // j ^ ((token >> 2) & 15)
    constexpr int SLAB_ROWS = NW * QW * 4;
    constexpr int NPASS = (SLAB_ROWS + 255) / 256;
    const int row0 = slab * SLAB_ROWS;
    int tid_e = threadIdx.x;                          // (lane constants worked out again, as in k_spmm)
    asm volatile("" : "+v"(tid_e));
    const int g_e = (tid_e >> 4) & 3, s_e = tid_e & 15;
    int rloc[QW];
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int rm = rowmap[(fq + q) * 4 + g_e];
        fold_spread(acc[q], rm & SPREAD_FLAG, g_e);
        rloc[q] = (rm & ~SPREAD_FLAG) - row0;
    }
    float* stf = tile;
#pragma unroll
    for (int h = 0; h < NPASS; ++h) {
        __syncthreads();
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            if (NPASS > 1 && ((wave * QW + q) >> 6) != h) continue;      // quad's block lies in another pass
            const int rl = rloc[q] - 256 * h;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                stf[((4 * s_e + e) * 64 + ((rl >> 2) ^ s_e)) * 4 + (rl & 3)] = acc[q][e];
        }
        __syncthreads();
        const int NCH = (SLAB_ROWS - 256 * h < 256 ? SLAB_ROWS - 256 * h : 256) / 4;   // constant after unrolling
        for (int item = tid_e; item < 64 * NCH; item += nthreads) {
            const int tl = item / NCH, j = item % NCH;
            const int t = t0 + tl;
            const int row = row0 + 256 * h + 4 * j;
            if (t >= T || row >= R) continue;
            const float4 v = *reinterpret_cast<const float4*>(stf + (tl * 64 + (j ^ ((tl >> 2) & 15))) * 4);
            float* o = out + (int64_t)t * R + row;
            if (vec_store && row + 3 < R) {
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

template <typename TIn, int QW>
static void launch64(const View& v, const TIn* A, float* out, int T, hipStream_t s) {
    const int ntile = (int)cdiv(T, TT64);
    const int nslab = (int)cdiv((int64_t)v.NB * 4, NW * QW);
    k_spmm64<TIn, QW><<<grid_for(ntile, nslab), NW * 64, 0, s>>>(A, v.ptr, v.ent, v.rowmap, out, T, v.K, v.R, v.NBpad,
                                                                v.nchunk, nslab, ntile, (v.K % 4 == 0) ? 1 : 0,
                                                                (v.R % 4 == 0) ? 1 : 0);
}

// Launch shape: tokens per workgroup (128 or 64) and quads per wavefront.  Every candidate
// computes the same sums in the same order, so the choice changes speed only.  The cost of a
// candidate is the cost of one workgroup -- walk (proportional to its entries x tokens),
// activation staging (tokens x K) and output (tokens x rows) -- times the number of
// rounds its grid needs on 256 CUs x 2 workgroups; a last round that leaves every CU at
// most one workgroup costs less than a full one.  A wavefront also pays a fixed amount per
// quad segment it walks (pointer and first entry batch, padding to an even step count), which
// at densities of a few percent decides for few quads per wavefront.  The constants were fitted
// to timings of 138 cases (GPT-2 small / medium / large layer shapes, T = 512 .. 16384, densities
// 0.01 .. 0.10: the range the sparse kernels serve) on MI355X: the chosen shape is 1.6 % slower
// than the best one on average, 12 % at worst (timed again on the present kernels).
struct SpmmShape {
    int tt, qw;
};
static SpmmShape g_forced = {0, 0};

static SpmmShape pick_shape(int T, int R, int K, double density) {
    if (g_forced.tt != 0) return g_forced;
    static const SpmmShape cand[] = {{128, 2}, {128, 3}, {128, 4}, {64, 2}, {64, 3}, {64, 4}, {64, 6}, {64, 8}};
    const double kWalk = 2.2e-5, kStage = 0.0, kOut = 2.69e-4, kChunk = 1.31;
    const double kLoneTail = 0.68, kLoneOnly = 0.71, k64 = 0.893, kSeg128 = 0.49, kSeg64 = 0.35;
    const int64_t nchunk = cdiv(K, KC);
    SpmmShape best = cand[0];
    double best_cost = 0.0;
    for (const SpmmShape& c : cand) {
        const int rows = NW * c.qw * 4;
        const int64_t nslab = cdiv(R, rows), ntile = cdiv(T, c.tt), nwg = ntile * nslab;
        const double rows_eff = (double)R / (double)nslab;
        const double wg = c.tt * (rows_eff * density * K * kWalk * (c.tt == 64 ? k64 : 1.0) +
                                  (double)nchunk * KC * kStage + rows * kOut) + kChunk * (double)nchunk +
                          (double)c.qw * (double)nchunk * (c.tt == 128 ? kSeg128 : kSeg64);
        const int64_t full = nwg / 512, rest = nwg % 512;
        double rounds;
        if (full == 0) rounds = rest <= 256 ? kLoneOnly : 1.0;
        else rounds = (double)full + (rest == 0 ? 0.0 : rest <= 256 ? kLoneTail : 1.0);
        const double cost = wg * rounds;
        if (best_cost == 0.0 || cost < best_cost) {
            best_cost = cost;
            best = c;
        }
    }
    return best;
}

template <typename TIn>
static int launch_spmm(const View& v, const TIn* A, float* out, int T, int64_t nnz, hipStream_t s) {
    const double density = (double)nnz / ((double)v.R * (double)v.K);
    const SpmmShape sh = pick_shape(T, v.R, v.K, density);
    if (sh.tt == 64) {
        switch (sh.qw) {
            case 2: launch64<TIn, 2>(v, A, out, T, s); break;
            case 3: launch64<TIn, 3>(v, A, out, T, s); break;
            case 4: launch64<TIn, 4>(v, A, out, T, s); break;
            case 6: launch64<TIn, 6>(v, A, out, T, s); break;
            default: launch64<TIn, 8>(v, A, out, T, s); break;
        }
        MST_LAUNCH_CHECK();
        return MST_OK;
    }
    const int ntile = (int)cdiv(T, TT);
    const int nslab = (int)cdiv((int64_t)v.NB * 4, NW * sh.qw);
    const int vec_ok = (v.K % 4 == 0) ? 1 : 0;
    const int vec_store = (v.R % 4 == 0) ? 1 : 0;
    if (sh.qw == 4)
        k_spmm<TIn, 4><<<grid_for(ntile, nslab), NW * 64, 0, s>>>(A, v.ptr, v.ent, v.rowmap, out, T, v.K, v.R, v.NBpad, v.nchunk,
                                                                 nslab, ntile, vec_ok, vec_store);
    else if (sh.qw == 3)
        k_spmm<TIn, 3><<<grid_for(ntile, nslab), NW * 64, 0, s>>>(A, v.ptr, v.ent, v.rowmap, out, T, v.K, v.R, v.NBpad, v.nchunk,
                                                                 nslab, ntile, vec_ok, vec_store);
    else
        k_spmm<TIn, 2><<<grid_for(ntile, nslab), NW * 64, 0, s>>>(A, v.ptr, v.ent, v.rowmap, out, T, v.K, v.R, v.NBpad, v.nchunk,
                                                                 nslab, ntile, vec_ok, vec_store);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int spmm(const View& v, const void* A, float* out, int T, int64_t nnz, mst_dtype act, hipStream_t s) {
    if (act == MST_F32) return launch_spmm<float>(v, static_cast<const float*>(A), out, T, nnz, s);
    return launch_spmm<uint16_t>(v, static_cast<const uint16_t*>(A), out, T, nnz, s);
}

int spmm_force_shape(int tt, int qw) {
    if (tt == 0 && qw == 0) {
        g_forced = {0, 0};
        return MST_OK;
    }
    const bool ok = (tt == 128 && (qw == 2 || qw == 3 || qw == 4)) ||
                    (tt == 64 && (qw == 2 || qw == 3 || qw == 4 || qw == 6 || qw == 8));
    if (!ok) return MST_ERR_ARG;
    g_forced = {tt, qw};
    return MST_OK;
}

}  // namespace mst
