// Heavy rows of the forward product Y = X (W . M)^T (App. "FLOP Calculation" Eq. (1)).
//
// With power-law row lengths a few dozen rows of W hold most of the nonzeros (rows that are a
// quarter full or entirely full next to thousands of rows with a handful of entries).  In the
// row view they would make a few quads hundreds of steps long while every other wavefront of
// the workgroup waits at the chunk barriers.  Such rows -- at most HEAVY_MAX, chosen when the
// row view is built -- are left out of the view and kept as a small dense matrix
// Hd [HEAVY_MAX x I] (zero at inactive positions); their outputs Y[:, h] are a dense
// contraction on the matrix cores: fp32 operands split into bf16 hi + lo, three
// v_mfma_f32_32x32x16_bf16 per 16 k (two when X is bfloat16), fp32 accumulation, the same
// arithmetic as the dense GEMM kernels.  The sparse kernel writes zeros to those columns of Y
// first (the rows look empty to it); this kernel, launched after it on the same stream,
// overwrites them.  The count and the list live in device memory (an update never reads them
// back): for a layer the rule applies to, the kernel is launched after every sparse forward and
// returns at once when the layer has no heavy row at the moment.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "split_bf16.h"

namespace mst {

constexpr int HT = 32;           // tokens per workgroup
constexpr int HK = 128;          // k per step: two LDS rows of 64 bf16 per tile row (two halves)

// eight consecutive k of a row as fp32 (row == nullptr or k past the row's end: zeros)
__device__ inline void heavy_load8(const float* __restrict__ row, int k, int I, bool vec, float4& a, float4& b) {
    a = make_float4(0.f, 0.f, 0.f, 0.f);
    b = a;
    if (row == nullptr || k >= I) return;
    if (vec && k + 8 <= I) {
        a = *reinterpret_cast<const float4*>(row + k);
        b = *reinterpret_cast<const float4*>(row + k + 4);
        return;
    }
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = k + j < I ? row[k + j] : 0.f;
    a = make_float4(v[0], v[1], v[2], v[3]);
    b = make_float4(v[4], v[5], v[6], v[7]);
}
// the same for bfloat16 storage: the eight values as they are (one 16-byte LDS unit)
__device__ inline uint4 heavy_load8(const uint16_t* __restrict__ row, int k, int I, bool vec) {
    uint4 r = make_uint4(0u, 0u, 0u, 0u);
    if (row == nullptr || k >= I) return r;
    if (vec && k + 8 <= I) return *reinterpret_cast<const uint4*>(row + k);
    uint32_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = k + j < I ? (uint32_t)row[k + j] : 0u;
    return make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
}

__device__ inline void heavy_stage_f32(char* hi, char* lo, uint32_t addr, const float4& a, const float4& b) {
    uint4 h, l;
    split_pair(a.x, a.y, h.x, l.x);
    split_pair(a.z, a.w, h.y, l.y);
    split_pair(b.x, b.y, h.z, l.z);
    split_pair(b.z, b.w, h.w, l.w);
    *reinterpret_cast<uint4*>(hi + addr) = h;
    *reinterpret_cast<uint4*>(lo + addr) = l;
}

template <typename TA> struct HeavyRegs;
template <> struct HeavyRegs<float> { float4 a[2]; float4 b[2][2]; };
template <> struct HeavyRegs<uint16_t> { uint4 a; float4 b[2][2]; };

// Workgroup = 32 tokens x up to 64 heavy rows (T / 32 workgroups: two per CU at T = 16384, which
// is what keeps the memory side busy -- a workgroup has one fetch in flight at a time).  Wavefronts
// 0 and 1 own one 32 x 32 MFMA tile each (rows 0..31 and 32..63 of the heavy list; the second idles
// when the list is short), all four stage.  k steps of 128 through one LDS stage, per half of
// 64 k: A hi, A lo (32 rows of 128 bytes), B hi, B lo (64 rows); the next step's operands travel in
// registers while this one is multiplied.  A: thread tid stages unit tid & 7 of row tid >> 3; B:
// unit idx & 7 of row idx >> 3, idx = it * 256 + tid: eight threads read 256 consecutive bytes.
template <typename TA>
__global__ __launch_bounds__(256) void k_heavy_fwd(const TA* __restrict__ X, const float* __restrict__ Hd,
                                                   const int* __restrict__ heavy, float* __restrict__ Y, int T, int I,
                                                   int O, int vec_x, int vec_h) {
    const int nh = min(heavy[0], HEAVY_MAX);
    if (nh <= 0) return;
    constexpr uint32_t PA = HT * 128, PB = HEAVY_MAX * 128;      // bytes of an A plane, of a B plane
    constexpr uint32_t HALF = 2 * PA + 2 * PB;                   // one half's four planes
    __shared__ __attribute__((aligned(16))) char lds[2 * HALF];
    __shared__ int col_s[HEAVY_MAX];
    char* const Ah = lds;
    char* const Al = lds + PA;
    char* const Bh = lds + 2 * PA;
    char* const Bl = lds + 2 * PA + PB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = (wave & 1) * 32;
    const int lk = lane >> 5, lm = lane & 31;
    const int m0 = blockIdx.x * HT;
    if (tid < HEAVY_MAX) col_s[tid] = tid < nh ? heavy[1 + tid] : 0;
    const bool active = wave < 2 && wn < nh;

    const int ua = tid & 7, ra = tid >> 3;
    const uint32_t addr_a = bf_unit(ra, ua);
    const TA* const arow = m0 + ra < T ? X + (int64_t)(m0 + ra) * I : nullptr;
    const float* brow[2];
    uint32_t addr_b[2];
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int r = (it * 256 + tid) >> 3;
        addr_b[it] = bf_unit(r, ua);
        brow[it] = r < nh ? Hd + (int64_t)r * I : nullptr;
    }
    HeavyRegs<TA> rg[2];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            const int k = k0 + 64 * hf + 8 * ua;
            if constexpr (std::is_same<TA, float>::value) heavy_load8(arow, k, I, vec_x != 0, rg[hf].a[0], rg[hf].a[1]);
            else rg[hf].a = heavy_load8(arow, k, I, vec_x != 0);
#pragma unroll
            for (int it = 0; it < 2; ++it) heavy_load8(brow[it], k, I, vec_h != 0, rg[hf].b[it][0], rg[hf].b[it][1]);
        }
    };
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    fetch(0);
    for (int k0 = 0; k0 < I; k0 += HK) {
        __syncthreads();                                  // the stage is free (and col_s is written)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            if constexpr (std::is_same<TA, float>::value) heavy_stage_f32(Ah, Al, hf * HALF + addr_a, rg[hf].a[0], rg[hf].a[1]);
            else *reinterpret_cast<uint4*>(Ah + hf * HALF + addr_a) = rg[hf].a;
#pragma unroll
            for (int it = 0; it < 2; ++it) heavy_stage_f32(Bh, Bl, hf * HALF + addr_b[it], rg[hf].b[it][0], rg[hf].b[it][1]);
        }
        __syncthreads();
        if (k0 + HK < I) fetch(k0 + HK);
        if (active) {
#pragma unroll
            for (int ks = 0; ks < 16; ks += 2) {          // 16 k per MFMA: units ks + lk of half ks >> 3
                const uint32_t hoff = (ks >> 3) * HALF;
                const uint32_t oa = hoff + bf_unit(lm, (ks & 7) + lk), ob = hoff + bf_unit(wn + lm, (ks & 7) + lk);
                const bf16x8 ah = *reinterpret_cast<const bf16x8*>(Ah + oa);
                const bf16x8 bh = *reinterpret_cast<const bf16x8*>(Bh + ob);
                const bf16x8 bl = *reinterpret_cast<const bf16x8*>(Bl + ob);
                if constexpr (std::is_same<TA, float>::value) {
                    const bf16x8 al = *reinterpret_cast<const bf16x8*>(Al + oa);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc, 0, 0, 0);
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc, 0, 0, 0);
            }
        }
    }
    if (!active) return;
    // D layout of the 32x32 MFMA: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
    const int n = wn + lm;
    if (n >= nh) return;
    const int col = col_s[n];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int m = m0 + 8 * (v >> 2) + 4 * lk + (v & 3);
        if (m < T) Y[(int64_t)m * O + col] = acc[v];
    }
}

// Hd from the canonical arrays: block j fills row j
__global__ __launch_bounds__(256) void k_heavy_fill(const int* __restrict__ heavy, const int* __restrict__ rowptr,
                                                    const int* __restrict__ flat, const float* __restrict__ vals, int I,
                                                    float* __restrict__ Hd) {
    heavy_fill_row((int)blockIdx.x, heavy, rowptr, flat, vals, I, Hd);
}

// The rows that leave the row view: rowcnt[r] >= thr, the first HEAVY_MAX of them in row order.
// heavy[0] = their count, heavy[1 + j] = the j-th such row (0 past the count), heavy[1 + HEAVY_MAX] =
// their entries in total; their per-chunk counts are cleared, so that the view's ranking and
// pointers see empty rows.  One block.
__global__ __launch_bounds__(1024) void k_mark_heavy(const int* __restrict__ rowcnt, int O, int thr, int* __restrict__ segcnt,
                                                     int nchunk, int Rpad, int* __restrict__ heavy) {
    __shared__ int wsum[16];
    __shared__ int entries_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) entries_s = 0;
    __syncthreads();
    int base = 0;
    for (int r0 = 0; r0 < O && base < HEAVY_MAX; r0 += 1024) {
        const int r = r0 + tid;
        const bool is = r < O && rowcnt[r] >= thr;
        const unsigned long long bal = __ballot(is);
        if (lane == 0) wsum[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) before += wsum[w];
            total += wsum[w];
        }
        const int pos = base + before + __popcll(bal & ((1ull << lane) - 1ull));
        if (is && pos < HEAVY_MAX) {
            heavy[1 + pos] = r;
            atomicAdd(&entries_s, rowcnt[r]);
            for (int c = 0; c < nchunk; ++c) segcnt[(size_t)c * Rpad + r] = 0;
        }
        base += total;
        __syncthreads();
    }
    const int n = min(base, HEAVY_MAX);
    if (tid == 0) { heavy[0] = n; heavy[1 + HEAVY_MAX] = entries_s; }
    if (tid >= n && tid < HEAVY_MAX) heavy[1 + tid] = 0;
}

static int g_heavy_rows = 1;     // 0 off, 1 large layers whose loaded mask has heavy rows, 2 every layer
int heavy_rows_mode() { return g_heavy_rows; }

int heavy_rows_enable(int on) {
    if (on < 0 || on > 2) return MST_ERR_ARG;
    g_heavy_rows = on;
    return MST_OK;
}

// Row length from which a row counts as heavy: a quarter of the row and four times the mean row
// (no row of a uniformly random mask comes near it), never below 32.  INT_MAX for a layer the rule
// does not apply to (mst_layer::heavy_on, decided by mst_layer_load_dense).
int heavy_threshold(const mst_layer* L) {
    if (!L->heavy_on || !L->Hd || L->O < 1) return 0x7FFFFFFF;
    const int64_t mean4 = 4 * cdiv(L->nnz, L->O);
    return (int)std::min<int64_t>(0x7FFFFFFF, std::max<int64_t>(std::max<int64_t>(L->I / 4, mean4), 32));
}

int heavy_mark(const mst_layer* L, const Workspace& ws, int Rpad, hipStream_t s) {
    k_mark_heavy<<<1, 1024, 0, s>>>(ws.rowcnt, L->O, heavy_threshold(L), ws.segcnt, L->row.nchunk, Rpad, L->heavy);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int heavy_fill(const mst_layer* L, hipStream_t s) {
    k_heavy_fill<<<HEAVY_MAX, 256, 0, s>>>(L->heavy, L->rowptr, L->flat, L->vals, L->I, L->Hd);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int heavy_fwd(const mst_layer* L, const void* X, float* Y, int T, mst_dtype act, hipStream_t s) {
    const unsigned grid = (unsigned)cdiv(T, HT);
    const int vec_h = L->I % 4 == 0;
    if (act == MST_BF16)
        k_heavy_fwd<uint16_t><<<grid, 256, 0, s>>>((const uint16_t*)X, L->Hd, L->heavy, Y, T, L->I, L->O, L->I % 8 == 0, vec_h);
    else
        k_heavy_fwd<float><<<grid, 256, 0, s>>>((const float*)X, L->Hd, L->heavy, Y, T, L->I, L->O, L->I % 4 == 0, vec_h);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

}  // namespace mst
