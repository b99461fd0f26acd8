// Row-split SpMM:  out[T x R] = A[T x K] * S^T  with S [R x K] unstructured-sparse.
// Serves the forward product (S = W, A = X; App. "FLOP Calculation" Eq. (1)) and the
// input gradient (S = W^T, A = dY; the first half of the backward pass).
//
// One workgroup owns TT = 128 tokens and a slab of 8*rw rows of S.  It walks the
// contraction index in chunks of KC: the chunk of A is staged (transposed) in LDS, then
// each wavefront walks the entries of its RW rows in that chunk.  A lane keeps two
// tokens; an entry costs one scalar-fetched {offset, weight}, one 8-byte LDS read and
// two FMAs into the row's accumulator pair, which stays in registers for the whole K loop.
#include "tile_loader.h"

namespace mst {

// entries of one group against the staged tile, accumulated into one row's pair
#define MST_SPMM_GROUP(E)                                                                     \
    do {                                                                                      \
        const float2 x0 = *reinterpret_cast<const float2*>(tb + (lane8 ^ (E).off0));          \
        const float2 x1 = *reinterpret_cast<const float2*>(tb + (lane8 ^ (E).off1));          \
        const float2 x2 = *reinterpret_cast<const float2*>(tb + (lane8 ^ (E).off2));          \
        const float2 x3 = *reinterpret_cast<const float2*>(tb + (lane8 ^ (E).off3));          \
        const float w0 = __uint_as_float((E).w0), w1 = __uint_as_float((E).w1);               \
        const float w2 = __uint_as_float((E).w2), w3 = __uint_as_float((E).w3);               \
        acc[r].x = fmaf(w0, x0.x, acc[r].x); acc[r].y = fmaf(w0, x0.y, acc[r].y);             \
        acc[r].x = fmaf(w1, x1.x, acc[r].x); acc[r].y = fmaf(w1, x1.y, acc[r].y);             \
        acc[r].x = fmaf(w2, x2.x, acc[r].x); acc[r].y = fmaf(w2, x2.y, acc[r].y);             \
        acc[r].x = fmaf(w3, x3.x, acc[r].x); acc[r].y = fmaf(w3, x3.y, acc[r].y);             \
    } while (0)

// NW wavefronts per workgroup; RWMAX bounds the accumulator registers; rw <= RWMAX (a
// multiple of 4) is the number of rows a wavefront actually owns, chosen on the host so
// that the grid fills the chip.  Two variants are built: 16 wavefronts x 12 rows at
// <= 64 VGPRs (two workgroups = 32 wavefronts per CU hide the latency of the scalar entry
// fetches), and 8 wavefronts x 32 rows for very sparse layers, where re-reading the
// activation tile for many narrow slabs would cost more than the entry work.
template <int NW, int RWMAX, int MINB, typename TIn>
__global__ __launch_bounds__(NW * 64, MINB) void k_spmm(const TIn* __restrict__ A, const int* __restrict__ ptr,
                                                        const Ent4* __restrict__ ent4, float* __restrict__ out,
                                                        int T, int K, int R, int Rpad, int nchunk, int nslab,
                                                        int ntile, int rw, int vec_ok, int vec_store) {
    __shared__ float tile[KC * TT];
    int tile_id, slab;
    if (!block_to_tile(nslab, ntile, tile_id, slab)) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = tile_id * TT;
    const int r0 = slab * (NW * rw) + wave * rw;
    const uint32_t lane8 = (uint32_t)lane << 3;
    const char* tb = reinterpret_cast<const char*>(tile);

    float2 acc[RWMAX];
#pragma unroll
    for (int r = 0; r < RWMAX; ++r) acc[r] = make_float2(0.f, 0.f);

    // lane r keeps the wavefront's segment pointer r of the current chunk
    const int pl = r0 + min(lane, rw);
    int pv = ptr[pl];
    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) __syncthreads();
        load_tile<TIn, NW * 64>(tile, A, K, t0, c * KC, T, K, vec_ok != 0, tid);
        const int pv_next = (c + 1 < nchunk) ? ptr[(int64_t)(c + 1) * Rpad + pl] : 0;
        // the wavefront's entries of this chunk are contiguous: one running group pointer,
        // the next group is always in flight while the current one is multiplied
        int g = __builtin_amdgcn_readlane(pv, 0) >> 2;
        const Ent4* pe = ent4 + g;
        Ent4 cur = pe[0];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < RWMAX; ++r) {
            if (r < rw) {
                const int gend = __builtin_amdgcn_readlane(pv, r + 1) >> 2;
                int n = gend - g;
                g = gend;
                for (; n >= 2; n -= 2) {           // two groups per trip
                    const Ent4 other = pe[1];
                    MST_SPMM_GROUP(cur);
                    cur = pe[2];
                    MST_SPMM_GROUP(other);
                    pe += 2;
                }
                if (n > 0) {
                    const Ent4 nxt = pe[1];
                    MST_SPMM_GROUP(cur);
                    cur = nxt;
                    pe += 1;
                }
            }
        }
        pv = pv_next;
    }

    // lane l holds tokens t0 + 2l and t0 + 2l + 1 for rows r0 .. r0 + rw - 1
    const int ta = t0 + 2 * lane;
    if (vec_store && r0 + rw <= R) {
#pragma unroll
        for (int r = 0; r < RWMAX; r += 4) {
            if (r < rw) {
                if (ta < T)
                    *reinterpret_cast<float4*>(out + (int64_t)ta * R + r0 + r) =
                        make_float4(acc[r].x, acc[r + 1].x, acc[r + 2].x, acc[r + 3].x);
                if (ta + 1 < T)
                    *reinterpret_cast<float4*>(out + (int64_t)(ta + 1) * R + r0 + r) =
                        make_float4(acc[r].y, acc[r + 1].y, acc[r + 2].y, acc[r + 3].y);
            }
        }
    } else {
#pragma unroll
        for (int r = 0; r < RWMAX; ++r) {
            if (r < rw && r0 + r < R) {
                if (ta < T) out[(int64_t)ta * R + r0 + r] = acc[r].x;
                if (ta + 1 < T) out[(int64_t)(ta + 1) * R + r0 + r] = acc[r].y;
            }
        }
    }
}

// Rows per wavefront (multiple of 4, <= rw_max).  The grid is ntile * ceil(R / (nw rw))
// workgroups running two per CU; the model charges each round of 512 workgroups
// rw units of entry work plus a fixed cost for staging the tile, and picks the minimum.
int pick_rows_per_wave(int T, int R, int nw, int rw_max, double stage_cost) {
    const int64_t ntile = cdiv(T, TT);
    int best = 4;
    double best_cost = 1e300;
    for (int rw = 4; rw <= rw_max; rw += 4) {
        const int64_t items = ntile * cdiv(R, nw * rw);
        const double rounds = (double)cdiv(items, 512);
        const double cost = rounds * (rw + stage_cost);
        if (cost < best_cost - 1e-9) { best_cost = cost; best = rw; }
    }
    return best;
}

template <typename TIn>
static int launch_spmm(const View& v, const TIn* A, float* out, int T, int64_t nnz, hipStream_t s) {
    const int ntile = (int)cdiv(T, TT);
    const int vec_ok = (v.K % 4 == 0) ? 1 : 0;
    const int vec_store = (v.R % 4 == 0) ? 1 : 0;
    const Ent4* e4 = reinterpret_cast<const Ent4*>(v.ent);
    const double per_seg = (double)nnz / ((double)v.R * v.nchunk);      // entries per (row, chunk)
    if (per_seg >= 4.0) {
        const int rw = pick_rows_per_wave(T, v.R, 16, 12, 3.0);
        const int nslab = (int)cdiv(v.R, 16 * rw);
        k_spmm<16, 12, 2, TIn><<<grid_for(ntile, nslab), 1024, 0, s>>>(A, v.ptr, e4, out, T, v.K, v.R, v.Rpad,
                                                                      v.nchunk, nslab, ntile, rw, vec_ok, vec_store);
    } else {
        const int rw = pick_rows_per_wave(T, v.R, 8, 32, 6.0);
        const int nslab = (int)cdiv(v.R, 8 * rw);
        k_spmm<8, 32, 1, TIn><<<grid_for(ntile, nslab), 512, 0, s>>>(A, v.ptr, e4, out, T, v.K, v.R, v.Rpad,
                                                                    v.nchunk, nslab, ntile, rw, vec_ok, vec_store);
    }
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int spmm(const View& v, const void* A, float* out, int T, int64_t nnz, mst_dtype act, hipStream_t s) {
    if (act == MST_F32) return launch_spmm<float>(v, static_cast<const float*>(A), out, T, nnz, s);
    return launch_spmm<uint16_t>(v, static_cast<const uint16_t*>(A), out, T, nnz, s);
}

}  // namespace mst
