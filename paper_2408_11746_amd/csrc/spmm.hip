// Row-split SpMM:  out[T x R] = A[T x K] * S^T  with S [R x K] unstructured-sparse.
// Serves the forward product (S = W, A = X; App. "FLOP Calculation" Eq. (1)) and the
// input gradient (S = W^T, A = dY; the first half of the backward pass).
//
// One workgroup owns TT = 128 tokens and a slab of 8*RW rows of S.  It walks the
// contraction index in chunks of KC: the chunk of A is staged (transposed) in LDS, then
// each wavefront walks the entries of its RW rows in that chunk.  A lane keeps two
// tokens; an entry costs one scalar-fetched {offset, weight}, one 8-byte LDS read and
// two FMAs into the row's accumulator pair, which stays in registers for the whole K loop.
#include "tile_loader.h"

namespace mst {

template <int RW, typename TIn>
__global__ __launch_bounds__(512) void k_spmm(const TIn* __restrict__ A, const int* __restrict__ ptr,
                                              const Ent4* __restrict__ ent4, float* __restrict__ out,
                                              int T, int K, int R, int Rpad, int nchunk, int nslab, int ntile,
                                              int vec_ok, int vec_store) {
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

    float2 acc[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) acc[r] = make_float2(0.f, 0.f);

    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) __syncthreads();
        load_tile<TIn, 512>(tile, A, K, t0, c * KC, T, K, vec_ok != 0, tid);
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
                const float w0 = __uint_as_float(cur.w0), w1 = __uint_as_float(cur.w1);
                const float w2 = __uint_as_float(cur.w2), w3 = __uint_as_float(cur.w3);
                acc[r].x = fmaf(w0, x0.x, acc[r].x); acc[r].y = fmaf(w0, x0.y, acc[r].y);
                acc[r].x = fmaf(w1, x1.x, acc[r].x); acc[r].y = fmaf(w1, x1.y, acc[r].y);
                acc[r].x = fmaf(w2, x2.x, acc[r].x); acc[r].y = fmaf(w2, x2.y, acc[r].y);
                acc[r].x = fmaf(w3, x3.x, acc[r].x); acc[r].y = fmaf(w3, x3.y, acc[r].y);
                cur = nxt;
            }
        }
    }

    // lane l holds tokens t0 + 2l and t0 + 2l + 1 for rows r0 .. r0 + RW - 1
    const int ta = t0 + 2 * lane;
    if (vec_store && r0 + RW <= R) {
        if (ta < T) {
            float4* o = reinterpret_cast<float4*>(out + (int64_t)ta * R + r0);
#pragma unroll
            for (int r = 0; r < RW; r += 4) o[r >> 2] = make_float4(acc[r].x, acc[r + 1].x, acc[r + 2].x, acc[r + 3].x);
        }
        if (ta + 1 < T) {
            float4* o = reinterpret_cast<float4*>(out + (int64_t)(ta + 1) * R + r0);
#pragma unroll
            for (int r = 0; r < RW; r += 4) o[r >> 2] = make_float4(acc[r].y, acc[r + 1].y, acc[r + 2].y, acc[r + 3].y);
        }
    } else {
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            if (r0 + r < R) {
                if (ta < T) out[(int64_t)ta * R + r0 + r] = acc[r].x;
                if (ta + 1 < T) out[(int64_t)(ta + 1) * R + r0 + r] = acc[r].y;
            }
        }
    }
}

template <int RW, typename TIn>
static int launch_spmm(const View& v, const TIn* A, float* out, int T, hipStream_t s) {
    const int ntile = (int)cdiv(T, TT);
    const int nslab = (int)cdiv(v.R, 8 * RW);
    const int vec_ok = (v.K % 4 == 0) ? 1 : 0;
    const int vec_store = (v.R % 4 == 0) ? 1 : 0;
    k_spmm<RW, TIn><<<grid_for(ntile, nslab), 512, 0, s>>>(A, v.ptr, reinterpret_cast<const Ent4*>(v.ent), out, T,
                                                          v.K, v.R, v.Rpad, v.nchunk, nslab, ntile, vec_ok,
                                                          vec_store);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

// rows per wavefront: wide slabs re-read the activation tile less often; narrow ones
// give enough workgroups to fill 256 CUs twice when T * R is small
static int pick_rw(int T, int R) {
    const int64_t ntile = cdiv(T, TT);
    for (int rw : {32, 16}) {
        if (ntile * cdiv(R, 8 * rw) >= 512) return rw;
    }
    return 8;
}

int spmm(const View& v, const void* A, float* out, int T, mst_dtype act, hipStream_t s) {
    const int rw = pick_rw(T, v.R);
    if (act == MST_F32) {
        const float* a = static_cast<const float*>(A);
        if (rw == 32) return launch_spmm<32, float>(v, a, out, T, s);
        if (rw == 16) return launch_spmm<16, float>(v, a, out, T, s);
        return launch_spmm<8, float>(v, a, out, T, s);
    }
    const uint16_t* a = static_cast<const uint16_t*>(A);
    if (rw == 32) return launch_spmm<32, uint16_t>(v, a, out, T, s);
    if (rw == 16) return launch_spmm<16, uint16_t>(v, a, out, T, s);
    return launch_spmm<8, uint16_t>(v, a, out, T, s);
}

}  // namespace mst
