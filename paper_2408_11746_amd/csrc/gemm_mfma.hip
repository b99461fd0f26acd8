// Dense fp32-accumulating GEMMs on the CDNA matrix cores: v_mfma_f32_32x32x2f32 for fp32
// operands, v_mfma_f32_32x32x16_bf16 when both operands are bfloat16.
//
// Used where a dense contraction really is the work: the dense weight gradient
// G = dY^T X that scores gradient-based growth (Algorithm 1, ArgTopK of |grad|; the dense
// gradient Sec. 2 says such growth needs), and the three products of a layer whose
// density is high (start of warm-up / end of restoration, Sec. 3.1).
//
// C[M x N] = sum_k A'[k][m] B'[k][n].  Each operand is given either k-major (element
// (k, m) at src[k*ld + m]) or m-major (src[m*ld + k]); both are staged k-major in LDS.
// Workgroup tile 128 x 128 x 16, four wavefronts of 64 x 64 (2 x 2 MFMA tiles each).
// Optional split of the k range over blockIdx.x (fastest index: consecutive workgroups go
// to the 8 XCDs in turn, so an XCD's L2 mostly sees one k range of the operands instead of
// all of them) into separate partial outputs that a
// second kernel adds in a fixed order.
#include <type_traits>
#include "common.h"
#include "split_bf16.h"

namespace mst {

constexpr int BM = 128, BN = 128;      // bf16 kernel tile
constexpr int BK = 16;                 // k per LDS tile of the fp32 kernel

template <typename TIn>
__device__ inline float to_f32(TIn v);
template <>
__device__ inline float to_f32<float>(float v) { return v; }
template <>
__device__ inline float to_f32<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// four consecutive source elements; the 16-byte path needs all four in range and aligned
template <typename TIn>
__device__ inline void load4(const TIn* __restrict__ p, int n_valid, bool vec, float* v);
template <>
__device__ inline void load4<float>(const float* __restrict__ p, int n_valid, bool vec, float* v) {
    if (vec && n_valid >= 4) {
        const float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        return;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = j < n_valid ? p[j] : 0.f;
}
template <>
__device__ inline void load4<uint16_t>(const uint16_t* __restrict__ p, int n_valid, bool vec, float* v) {
    if (vec && n_valid >= 4) {
        const uint2 q = *reinterpret_cast<const uint2*>(p);
        v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xFFFF0000u);
        v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xFFFF0000u);
        return;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = j < n_valid ? to_f32<uint16_t>(p[j]) : 0.f;
}

// One operand tile [BK x W] (k-major in LDS, row stride W + 4) handled by NT threads:
// IPT items of four elements per thread.
template <int W, int NT> struct TileShape {
    static constexpr int LD = W + 4;
    static constexpr int IPT = BK * W / 4 / NT;
    static_assert(BK * W / 4 % NT == 0, "tile does not divide over the threads");
};

template <typename TIn, bool KMAJOR, int W, int NT>
__device__ inline void fetch_tile(const TIn* __restrict__ src, int64_t ld, int k0, int m0, int Kdim, int Mdim,
                                  int tid, bool vec, float (&v)[4 * TileShape<W, NT>::IPT]) {
    constexpr int IPT = TileShape<W, NT>::IPT;
#pragma unroll
    for (int it = 0; it < IPT; ++it) {
        const int idx = it * NT + tid;
        if (KMAJOR) {            // item = (k, group of 4 m): a wavefront reads whole rows
            const int k = k0 + idx / (W / 4), m = m0 + ((idx % (W / 4)) << 2);
            const int nv = (k < Kdim) ? max(0, min(4, Mdim - m)) : 0;
            if (nv > 0) load4<TIn>(src + (int64_t)k * ld + m, nv, vec, &v[it * 4]);
            else { v[it * 4] = v[it * 4 + 1] = v[it * 4 + 2] = v[it * 4 + 3] = 0.f; }
        } else {                 // item = (m, group of 4 k)
            const int m = m0 + idx / (BK / 4), k = k0 + ((idx % (BK / 4)) << 2);
            const int nv = (m < Mdim) ? max(0, min(4, Kdim - k)) : 0;
            if (nv > 0) load4<TIn>(src + (int64_t)m * ld + k, nv, vec, &v[it * 4]);
            else { v[it * 4] = v[it * 4 + 1] = v[it * 4 + 2] = v[it * 4 + 3] = 0.f; }
        }
    }
}

template <bool KMAJOR, int W, int NT>
__device__ inline void stage_tile(float* lds, int tid, const float (&v)[4 * TileShape<W, NT>::IPT]) {
    constexpr int IPT = TileShape<W, NT>::IPT, LD = TileShape<W, NT>::LD;
#pragma unroll
    for (int it = 0; it < IPT; ++it) {
        const int idx = it * NT + tid;
        if (KMAJOR) {
            const int k = idx / (W / 4), m = (idx % (W / 4)) << 2;
            *reinterpret_cast<float4*>(lds + k * LD + m) =
                make_float4(v[it * 4 + 0], v[it * 4 + 1], v[it * 4 + 2], v[it * 4 + 3]);
        } else {
            const int m = idx / (BK / 4), k = (idx % (BK / 4)) << 2;
#pragma unroll
            for (int j = 0; j < 4; ++j) lds[(k + j) * LD + m] = v[it * 4 + j];
        }
    }
}

// TM x 128 workgroup tile, TM / 64 x 2 wavefronts of 64 x 64 each
template <typename TA, bool A_KMAJOR, typename TB, bool B_KMAJOR, int TM>
__global__ __launch_bounds__(TM * 2) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_gemm(const TA* __restrict__ A, int64_t lda,
                                                 const TB* __restrict__ B, int64_t ldb,
                                                 float* __restrict__ C, int M, int N, int Kdim, int k_per_split,
                                                 int64_t split_stride, int vec_a, int vec_b) {
    constexpr int NT = TM * 2, TNW = 128;
    typedef TileShape<TM, NT> SA;
    typedef TileShape<TNW, NT> SB;
    __shared__ float As[2][BK * SA::LD];
    __shared__ float Bs[2][BK * SB::LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int m0 = blockIdx.z * TM, n0 = blockIdx.y * TNW;
    const int kbeg = blockIdx.x * k_per_split;
    const int kend = min(Kdim, kbeg + k_per_split);
    float* Cz = C + (int64_t)blockIdx.x * split_stride;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Two LDS buffers, one barrier per step: while buffer b is multiplied, the registers
    // (tile s + 1, fetched during step s - 1) go to buffer b ^ 1 and tile s + 2 is fetched.
    float ra[4 * SA::IPT], rb[4 * SB::IPT];
    fetch_tile<TA, A_KMAJOR, TM, NT>(A, lda, kbeg, m0, kend, M, tid, vec_a != 0, ra);
    fetch_tile<TB, B_KMAJOR, TNW, NT>(B, ldb, kbeg, n0, kend, N, tid, vec_b != 0, rb);
    stage_tile<A_KMAJOR, TM, NT>(As[0], tid, ra);
    stage_tile<B_KMAJOR, TNW, NT>(Bs[0], tid, rb);
    if (kbeg + BK < kend) {
        fetch_tile<TA, A_KMAJOR, TM, NT>(A, lda, kbeg + BK, m0, kend, M, tid, vec_a != 0, ra);
        fetch_tile<TB, B_KMAJOR, TNW, NT>(B, ldb, kbeg + BK, n0, kend, N, tid, vec_b != 0, rb);
    }
    __syncthreads();
    const int lk = lane >> 5, lm = lane & 31;
    int buf = 0;
    for (int k0 = kbeg; k0 < kend; k0 += BK, buf ^= 1) {
        const float* as = As[buf];
        const float* bs = Bs[buf];
        if (k0 + BK < kend) {                  // the next tile goes to the other buffer ...
            stage_tile<A_KMAJOR, TM, NT>(As[buf ^ 1], tid, ra);
            stage_tile<B_KMAJOR, TNW, NT>(Bs[buf ^ 1], tid, rb);
            if (k0 + 2 * BK < kend) {          // ... and the one after it starts to travel
                fetch_tile<TA, A_KMAJOR, TM, NT>(A, lda, k0 + 2 * BK, m0, kend, M, tid, vec_a != 0, ra);
                fetch_tile<TB, B_KMAJOR, TNW, NT>(B, ldb, k0 + 2 * BK, n0, kend, N, tid, vec_b != 0, rb);
            }
        }
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const float a0 = as[(kk + lk) * SA::LD + wm + lm];
            const float a1 = as[(kk + lk) * SA::LD + wm + 32 + lm];
            const float b0 = bs[(kk + lk) * SB::LD + wn + lm];
            const float b1 = bs[(kk + lk) * SB::LD + wn + 32 + lm];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
    }

    // D layout of the 32x32 MFMA: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                const int n = n0 + wn + j * 32 + lm;
                if (m < M && n < N) Cz[(int64_t)m * N + n] = acc[i][j][v];
            }
}

// ---- bf16 x bf16 -> fp32, both operands k-major (the dense gradient G = dY^T X with
// bfloat16 activations).  v_mfma_f32_32x32x16_bf16 wants, per lane, 8 consecutive k of one
// row, so the k-major source is transposed on its way into LDS: a thread fetches an
// [8 k x 8 m] patch with eight 16-byte loads (threads 0..127 the A tile, 128..255 the B
// tile; a wavefront reads four 256-byte row pieces per load), transposes it in registers
// and stores eight 16-byte rows [m][8 k].  Workgroup tile 128 x 128 x 64; an LDS row is 64 k
// = 128 bytes = eight 16-byte units, unit u of row m is kept at position u ^ ((m >> 1) & 7):
// the MFMA operand reads of 16 consecutive rows then cover all banks once.
constexpr int BKH = 64;            // k per LDS tile


// thread -> patch: 16 patches along m x 8 along k, for the A tile (tid < 128) or the B tile
__device__ inline void fetch_patch(const uint16_t* __restrict__ src, int64_t ld, int k0, int m0, int Kdim,
                                   int Mdim, int p, bool vec_ok, uint4 (&d)[8]) {
    const int mq = p & 15, kg = p >> 4;
    const int m = m0 + 8 * mq;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        const int k = k0 + 8 * kg + kk;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (k < Kdim && m < Mdim) {
            const uint16_t* q = src + (int64_t)k * ld + m;
            if (vec_ok && m + 8 <= Mdim) {
                v = *reinterpret_cast<const uint4*>(q);
            } else {
                uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (m + j < Mdim) w[j >> 1] |= (uint32_t)q[j] << (16 * (j & 1));
                v = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
        d[kk] = v;
    }
}

// d[kk] holds 8 m of row k0 + kk; LDS row m gets its 8 k as one 16-byte unit
__device__ inline uint32_t half_of(const uint4& v, int r) {      // element r (0..7) of the 8 packed in v
    const uint32_t word = (r >> 1) == 0 ? v.x : (r >> 1) == 1 ? v.y : (r >> 1) == 2 ? v.z : v.w;
    return (r & 1) ? (word >> 16) : (word & 0xFFFFu);
}
__device__ inline void stage_patch(char* lds, int p, const uint4 (&d)[8]) {
    const int mq = p & 15, kg = p >> 4;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const uint4 out = make_uint4(half_of(d[0], r) | (half_of(d[1], r) << 16), half_of(d[2], r) | (half_of(d[3], r) << 16),
                                     half_of(d[4], r) | (half_of(d[5], r) << 16), half_of(d[6], r) | (half_of(d[7], r) << 16));
        *reinterpret_cast<uint4*>(lds + bf_unit(8 * mq + r, kg)) = out;
    }
}

__global__ __launch_bounds__(256) void k_gemm_tn_bf16(const uint16_t* __restrict__ A, int64_t lda,
                                                      const uint16_t* __restrict__ B, int64_t ldb,
                                                      float* __restrict__ C, int M, int N, int Kdim,
                                                      int k_per_split, int64_t split_stride, int vec_a,
                                                      int vec_b) {
    __shared__ __attribute__((aligned(16))) char As[BM * 128];
    __shared__ __attribute__((aligned(16))) char Bs[BN * 128];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int m0 = blockIdx.z * BM, n0 = blockIdx.y * BN;
    const int kbeg = blockIdx.x * k_per_split;
    const int kend = min(Kdim, kbeg + k_per_split);
    float* Cz = C + (int64_t)blockIdx.x * split_stride;
    // this thread's operand tile
    const bool mine_a = tid < 128;
    const int p = tid & 127;
    const uint16_t* src = mine_a ? A : B;
    const int64_t ld = mine_a ? lda : ldb;
    const int o0 = mine_a ? m0 : n0, odim = mine_a ? M : N;
    const bool vec = mine_a ? vec_a != 0 : vec_b != 0;
    char* dst = mine_a ? As : Bs;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 rp[8];
    fetch_patch(src, ld, kbeg, o0, kend, odim, p, vec, rp);
    const int lk = lane >> 5, lm = lane & 31;
    for (int k0 = kbeg; k0 < kend; k0 += BKH) {
        __syncthreads();
        stage_patch(dst, p, rp);
        __syncthreads();
        if (k0 + BKH < kend) fetch_patch(src, ld, k0 + BKH, o0, kend, odim, p, vec, rp);
#pragma unroll
        for (int ks = 0; ks < BKH / 8; ks += 2) {          // 16 k per MFMA: units ks + lk
            const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(As + bf_unit(wm + lm, ks + lk));
            const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(As + bf_unit(wm + 32 + lm, ks + lk));
            const bf16x8 b0 = *reinterpret_cast<const bf16x8*>(Bs + bf_unit(wn + lm, ks + lk));
            const bf16x8 b1 = *reinterpret_cast<const bf16x8*>(Bs + bf_unit(wn + 32 + lm, ks + lk));
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                const int n = n0 + wn + j * 32 + lm;
                if (m < M && n < N) Cz[(int64_t)m * N + n] = acc[i][j][v];
            }
}

// ---- fp32 x fp32 -> fp32 on the bf16 matrix cores: every operand element x is split while it
// is staged into hi = bf16(x) and lo = bf16(x - hi) (x - hi is exact in fp32), and a product is
// formed as hi*hi + hi*lo + lo*hi with fp32 accumulation: three v_mfma_f32_32x32x16_bf16 (16x
// the rate of the fp32 MFMA each) instead of eight v_mfma_f32_32x32x2f32 per 16 k.  What is
// dropped (lo*lo and the second-order residue of the split) is below 2^-16 of a product, far
// inside the 1e-4 bound of the fp32 results and of the same order as the rounding of an fp32
// accumulation over thousands of terms.  Workgroup tile 128 x 128 x 64, four wavefronts of
// 64 x 64; LDS holds the hi and lo halves of both operand tiles in the bf16 kernel's layout
// (64 KB).  Either operand may be k-major (element (k, m) at src[k*ld + m]: an [8 k x 4 m]
// patch per thread is transposed in registers) or m-major (src[m*ld + k]: eight consecutive k
// per thread go to LDS as they are).  Only for shapes whose tiles are whole (M, N multiples
// of 128, k ranges multiples of 64, rows 16-byte aligned); everything else takes k_gemm.
constexpr int SPK = 64;


template <bool KMAJOR>
__device__ inline void split_fetch(const float* __restrict__ src, int64_t ld, int k0, int m0, int p, float4 (&r)[8]) {
    if (KMAJOR) {                       // patch: k = k0 + 8 kg .. + 7, m = m0 + 4 mq .. + 3
        const int mq = p & 31, kg = p >> 5;
        const float* q = src + (int64_t)(k0 + 8 * kg) * ld + m0 + 4 * mq;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) r[kk] = *reinterpret_cast<const float4*>(q + (int64_t)kk * ld);
    } else {                            // four units of eight consecutive k: unit index it * 256 + p
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int idx = it * 256 + p, m = idx >> 3, u = idx & 7;
            const float* q = src + (int64_t)(m0 + m) * ld + k0 + 8 * u;
            r[2 * it] = *reinterpret_cast<const float4*>(q);
            r[2 * it + 1] = *reinterpret_cast<const float4*>(q + 4);
        }
    }
}

__device__ inline float f4_at(const float4& v, int j) { return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w; }
__device__ inline uint32_t u4_at(const uint4& v, int j) { return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w; }

template <bool KMAJOR>
__device__ inline void split_stage(char* hi_lds, char* lo_lds, int p, const float4 (&r)[8]) {
    if (KMAJOR) {
        const int mq = p & 31, kg = p >> 5;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint4 h, l;
            split_pair(f4_at(r[0], j), f4_at(r[1], j), h.x, l.x);
            split_pair(f4_at(r[2], j), f4_at(r[3], j), h.y, l.y);
            split_pair(f4_at(r[4], j), f4_at(r[5], j), h.z, l.z);
            split_pair(f4_at(r[6], j), f4_at(r[7], j), h.w, l.w);
            const uint32_t a = bf_unit(4 * mq + j, kg);
            *reinterpret_cast<uint4*>(hi_lds + a) = h;
            *reinterpret_cast<uint4*>(lo_lds + a) = l;
        }
    } else {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int idx = it * 256 + p, m = idx >> 3, u = idx & 7;
            uint4 h, l;
            split_pair(r[2 * it].x, r[2 * it].y, h.x, l.x);
            split_pair(r[2 * it].z, r[2 * it].w, h.y, l.y);
            split_pair(r[2 * it + 1].x, r[2 * it + 1].y, h.z, l.z);
            split_pair(r[2 * it + 1].z, r[2 * it + 1].w, h.w, l.w);
            const uint32_t a = bf_unit(m, u);
            *reinterpret_cast<uint4*>(hi_lds + a) = h;
            *reinterpret_cast<uint4*>(lo_lds + a) = l;
        }
    }
}

template <bool A_KMAJOR, bool B_KMAJOR>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k_gemm_split(const float* __restrict__ A, int64_t lda, const float* __restrict__ B, int64_t ldb,
                  float* __restrict__ C, int M, int N, int Kdim, int k_per_split, int64_t split_stride) {
    __shared__ __attribute__((aligned(16))) char lds[4 * BM * 128];      // A hi, A lo, B hi, B lo
    char* const Ah = lds;
    char* const Al = lds + BM * 128;
    char* const Bh = lds + 2 * BM * 128;
    char* const Bl = lds + 3 * BM * 128;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    // Workgroup -> (output tile, k range).  Consecutive workgroup ids go to the 8 XCDs in turn;
    // each XCD has its own L2.  XCD x is given the tiles x Q .. x Q + Q - 1 (m-tile major, so they
    // share a few row panels of A and the column panels of B) and walks them one k range after
    // the other: the workgroups resident on an XCD at a time read the same operand panels at
    // the same k, and an XCD reads only its share of A.
    const int gn = N / BN, ntiles = (M / BM) * gn, nsplit = (Kdim + k_per_split - 1) / k_per_split;
    const int Q = (ntiles + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int split = slot / Q, tile_id = xcd * Q + slot % Q;
    if (tile_id >= ntiles || split >= nsplit) return;
    const int m0 = (tile_id / gn) * BM, n0 = (tile_id % gn) * BN;
    const int kbeg = split * k_per_split;
    const int kend = min(Kdim, kbeg + k_per_split);
    float* Cz = C + (int64_t)split * split_stride;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    float4 ra[8], rb[8];
    split_fetch<A_KMAJOR>(A, lda, kbeg, m0, tid, ra);
    split_fetch<B_KMAJOR>(B, ldb, kbeg, n0, tid, rb);
    const int lk = lane >> 5, lm = lane & 31;
    for (int k0 = kbeg; k0 < kend; k0 += SPK) {
        __syncthreads();
        split_stage<A_KMAJOR>(Ah, Al, tid, ra);
        split_stage<B_KMAJOR>(Bh, Bl, tid, rb);
        __syncthreads();
        if (k0 + SPK < kend) {
            split_fetch<A_KMAJOR>(A, lda, k0 + SPK, m0, tid, ra);
            split_fetch<B_KMAJOR>(B, ldb, k0 + SPK, n0, tid, rb);
        }
#pragma unroll
        for (int ks = 0; ks < SPK / 8; ks += 2) {          // 16 k per MFMA: units ks + lk
            const uint32_t ua0 = bf_unit(wm + lm, ks + lk), ua1 = bf_unit(wm + 32 + lm, ks + lk);
            const uint32_t ub0 = bf_unit(wn + lm, ks + lk), ub1 = bf_unit(wn + 32 + lm, ks + lk);
            const bf16x8 a0h = *reinterpret_cast<const bf16x8*>(Ah + ua0), a0l = *reinterpret_cast<const bf16x8*>(Al + ua0);
            const bf16x8 a1h = *reinterpret_cast<const bf16x8*>(Ah + ua1), a1l = *reinterpret_cast<const bf16x8*>(Al + ua1);
            const bf16x8 b0h = *reinterpret_cast<const bf16x8*>(Bh + ub0), b0l = *reinterpret_cast<const bf16x8*>(Bl + ub0);
            const bf16x8 b1h = *reinterpret_cast<const bf16x8*>(Bh + ub1), b1l = *reinterpret_cast<const bf16x8*>(Bl + ub1);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0l, b0h, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0l, b1h, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1l, b0h, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1l, b1h, acc[1][1], 0, 0, 0);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, b0l, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, b1l, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1h, b0l, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1h, b1l, acc[1][1], 0, 0, 0);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, b0h, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, b1h, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1h, b0h, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1h, b1h, acc[1][1], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                const int n = n0 + wn + j * 32 + lm;
                Cz[(int64_t)m * N + n] = acc[i][j][v];
            }
}

// ---- the same product with a 256 x 256 workgroup tile: half the operand bytes per flop of the
// 128 x 128 kernel, whose speed is set by what the CUs can pull from L2, not by the matrix
// cores.  512 threads = 8 wavefronts (4 along m x 2 along n) of 64 x 128 (2 x 4 MFMA tiles, 128
// accumulator registers), k steps of 32 through TWO LDS stages of 64 KB (hi and lo halves of a
// 256 x 32 tile of each operand): one barrier per step; the registers fetched during step s
// (tile s + 2) are split and stored into the free stage at the start of step s + 1.
// Threads 0..255 stage A, 256..511 stage B.  LDS rows are 32 k = 64 bytes = four 16-byte
// units; row m sits at position rho(m) (the two low bit pairs of m swapped inside its group of
// 16) and its unit u at (u ^ (rho >> 2) ^ (rho >> 4)) & 3: the MFMA operand reads of 16
// consecutive rows, the k-major stores (rows four apart) and the m-major stores (four rows x
// four units) each cover all banks once.
constexpr int BM2 = 256, BN2 = 256, SPK2 = 32;

// Tile number -> tile coordinates for the 256-row kernels.  Tiles are numbered in bands of four tile
// rows, column by column inside a band: the 32 tiles an XCD works on at a time then span about
// 4 rows x 8 columns instead of 2 x 20, so its L2 is filled with 12 operand panels instead of 22.
constexpr int TILE_BAND = 4;
__device__ inline void tile_coords(int tile_id, int gm, int gn, int& mi, int& ni) {
    const int band = tile_id / (TILE_BAND * gn), rem = tile_id - band * TILE_BAND * gn;
    const int hgt = min(TILE_BAND, gm - band * TILE_BAND);
    ni = rem / hgt;
    mi = band * TILE_BAND + rem - ni * hgt;
}

__device__ inline uint32_t bf_unit32(int m, int u) {
    const int rho = (m & ~15) | ((m & 3) << 2) | ((m >> 2) & 3);
    return (uint32_t)(rho * 64 + (((u ^ (rho >> 2) ^ (rho >> 4)) & 3) << 4));
}

// Staging roles.  A thread stages four "pieces" per step; a piece is one 16-byte LDS unit in each
// half (eight consecutive k of one row), made of four hi/lo pairs.
//   operands of equal layout: threads 0..255 stage A, 256..511 stage B, p = tid & 255;
//     k-major: registers r[kk] = four consecutive rows (m0 + 4 mq ..) at k0 + 8 kg + kk; piece j =
//              row 4 mq + j, unit kg;
//     m-major: r[2 it], r[2 it + 1] = eight consecutive k (unit u) of row m(it); piece it.
//   mixed (A m-major, B k-major): every thread stages two pieces of each, h = tid >> 8:
//     r[0..3] as the m-major case for it = 2 h, 2 h + 1; r[4 + t] = two consecutive rows
//     (n0 + 4 mq + 2 h ..) at k = k0 + 8 kg + 2 t (.xy) and + 2 t + 1 (.zw); pieces 2, 3 = those rows.
__device__ inline int mmajor_row(int p, int it) { return 64 * it + 16 * (p >> 6) + 4 * ((p >> 2) & 3) + ((p >> 4) & 3); }

// hi/lo pair q (0..3) of piece `piece` (0..3).  LAYOUT 0: k-major, 1: m-major, 2: mixed.
template <int LAYOUT>
__device__ inline void split256_pair(const float4 (&r)[8], int piece, int q, uint32_t& hi, uint32_t& lo) {
    if (LAYOUT == 0) {
        split_pair(f4_at(r[2 * q], piece), f4_at(r[2 * q + 1], piece), hi, lo);
    } else if (LAYOUT == 1 || piece < 2) {
        const float4& v = r[2 * piece + (q >> 1)];
        if (q & 1) split_pair(v.z, v.w, hi, lo);
        else split_pair(v.x, v.y, hi, lo);
    } else {
        const float4& v = r[4 + q];
        if (piece == 2) split_pair(v.x, v.z, hi, lo);
        else split_pair(v.y, v.w, hi, lo);
    }
}
// byte offset of that piece inside one half of its operand's tile
template <int LAYOUT>
__device__ inline uint32_t split256_unit(int p, int h, int piece) {
    if (LAYOUT == 0) return bf_unit32(4 * (p & 63) + piece, p >> 6);
    if (LAYOUT == 1) return bf_unit32(mmajor_row(p, piece), p & 3);
    if (piece < 2) return bf_unit32(mmajor_row(p, 2 * h + piece), p & 3);
    return bf_unit32(4 * (p & 63) + 2 * h + piece - 2, p >> 6);
}

template <bool A_KMAJOR, bool B_KMAJOR>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k_gemm_split256(const float* __restrict__ A, int64_t lda, const float* __restrict__ B, int64_t ldb,
                     float* __restrict__ C, int M, int N, int Kdim, int k_per_split, int64_t split_stride, int sched) {
    constexpr int PLANE = BM2 * 64;                                       // one half (hi or lo) of one operand tile
    __shared__ __attribute__((aligned(16))) char lds[2 * 4 * PLANE];     // [stage][A hi, A lo, B hi, B lo]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 128;
    const int gn = N / BN2, ntiles = (M / BM2) * gn;
    // This workgroup's one or two segments (tile, k range, partial-output plane).
    int nseg = 1, seg_tile[2], seg_kb[2], seg_ke[2], seg_plane[2];
    if (sched == 0) {
        // XCD x takes tiles x Q .. x Q + Q - 1, one k range after the other
        const int nsplit = (Kdim + k_per_split - 1) / k_per_split;
        const int Q = (ntiles + 7) >> 3;
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int split = slot / Q, tile_id = xcd * Q + slot % Q;
        if (tile_id >= ntiles || split >= nsplit) return;
        seg_tile[0] = tile_id;
        seg_kb[0] = split * k_per_split;
        seg_ke[0] = min(Kdim, seg_kb[0] + k_per_split);
        seg_plane[0] = split;
    } else {
        // Five workgroups per two tiles (about 100 tiles on 256 CUs: two k ranges per tile fill 78 % of
        // the CUs, three need a second round).  Both tiles are cut into the same three k ranges [0, x),
        // [x, 2 x), [2 x, K) with x = k_per_split a little more than a third (so that the shorter last range
        // makes up for a second start-up and output): workgroups 0, 1 take the first two ranges of tile A,
        // 3, 4 those of tile B, workgroup 2 the last range of A and then of B.  Every tile ends with three
        // partial planes in ascending k order, as with three plain k ranges, and neighbouring workgroups walk
        // the same k range at the same time (they share operand tiles in L2).
        // (an XCD takes 32 consecutive work items)
        const int item = (blockIdx.x & 7) * 32 + (blockIdx.x >> 3);
        const int g = item / 5, r = item % 5, x = k_per_split;
        if ((blockIdx.x >> 3) >= 32 || 2 * g + 1 >= ntiles) return;
        const int tA = 2 * g, tB = 2 * g + 1;
        const int range = r < 2 ? r : r == 2 ? 2 : r - 3;        // 0, 1, 2 (both tiles), 0, 1
        seg_tile[0] = r < 3 ? tA : tB;
        seg_plane[0] = range;
        seg_kb[0] = range * x;
        seg_ke[0] = range == 2 ? Kdim : (range + 1) * x;
        if (r == 2) {
            nseg = 2;
            seg_tile[1] = tB;
            seg_plane[1] = 2;
            seg_kb[1] = 2 * x;
            seg_ke[1] = Kdim;
        }
    }
    int m0 = 0, n0 = 0, kbeg = 0, kend = 0;
    float* Cz = C;

    floatx16 acc[2][4];

    static_assert(A_KMAJOR == B_KMAJOR || (!A_KMAJOR && B_KMAJOR), "layouts: TN, NT or NN");
    constexpr int LAYOUT = A_KMAJOR == B_KMAJOR ? (A_KMAJOR ? 0 : 1) : 2;
    // h is uniform per wavefront: operand base and row pitch stay scalar, a load's address is a
    // scalar base (advanced per step) plus a per-thread 32-bit byte offset fixed for the kernel
    const int h = __builtin_amdgcn_readfirstlane(tid >> 8), p = tid & 255;
    const int64_t pa = 4 * lda, pb = 4 * ldb;         // row pitches in bytes
    const char* base0 = nullptr;                      // equal layouts: this thread's operand; mixed: A
    const char* base1 = nullptr;                      // mixed: B
    const int64_t pitch0 = LAYOUT == 2 ? pa : (h == 0 ? pa : pb);
    uint32_t voff[4];
    if (LAYOUT == 0) {
        voff[0] = (uint32_t)(8 * (p >> 6) * pitch0 + 16 * (p & 63));
    } else if (LAYOUT == 1) {
#pragma unroll
        for (int it = 0; it < 4; ++it) voff[it] = (uint32_t)(mmajor_row(p, it) * pitch0 + 32 * (p & 3));
    } else {
#pragma unroll
        for (int t = 0; t < 2; ++t) voff[t] = (uint32_t)(mmajor_row(p, 2 * h + t) * pa + 32 * (p & 3));
        voff[2] = (uint32_t)(8 * (p >> 6) * pb + 16 * (p & 63) + 8 * h);
    }
    auto set_tile = [&]() {                           // operand bases of the tile at (m0, n0)
        if (LAYOUT == 0) {
            base0 = reinterpret_cast<const char*>(h == 0 ? A + m0 : B + n0);
        } else if (LAYOUT == 1) {
            base0 = reinterpret_cast<const char*>(h == 0 ? A : B) + (int64_t)(h == 0 ? m0 : n0) * pitch0;
        } else {
            base0 = reinterpret_cast<const char*>(A) + (int64_t)m0 * pa;
            base1 = reinterpret_cast<const char*>(B + n0);
        }
    };
    auto fetch = [&](int k0, float4 (&r)[8]) __attribute__((always_inline)) {
        if (LAYOUT == 0) {
            const char* row = base0 + (int64_t)k0 * pitch0;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) r[kk] = *reinterpret_cast<const float4*>(row + kk * pitch0 + voff[0]);
        } else if (LAYOUT == 1) {
            const char* col = base0 + 4 * (int64_t)k0;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                r[2 * it] = *reinterpret_cast<const float4*>(col + voff[it]);
                r[2 * it + 1] = *reinterpret_cast<const float4*>(col + voff[it] + 16);
            }
        } else {
            const char* col = base0 + 4 * (int64_t)k0;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                r[2 * t] = *reinterpret_cast<const float4*>(col + voff[t]);
                r[2 * t + 1] = *reinterpret_cast<const float4*>(col + voff[t] + 16);
            }
            const char* row = base1 + (int64_t)k0 * pb;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float2 e = *reinterpret_cast<const float2*>(row + (2 * t) * pb + voff[2]);
                const float2 o = *reinterpret_cast<const float2*>(row + (2 * t + 1) * pb + voff[2]);
                r[4 + t] = make_float4(e.x, e.y, o.x, o.y);
            }
        }
    };
    const int lk = lane >> 5, lm = lane & 31;
    uint32_t wr_unit[4];                              // this thread's four LDS units of a stage (hi half)
#pragma unroll
    for (int pc = 0; pc < 4; ++pc) {
        const int plane = LAYOUT == 2 ? (pc < 2 ? 0 : 2 * PLANE) : (h == 0 ? 0 : 2 * PLANE);
        wr_unit[pc] = plane + split256_unit<LAYOUT>(p, h, pc);
    }
    auto stage = [&](int buf, const float4 (&r)[8]) __attribute__((always_inline)) {
        char* const wr = lds + buf * 4 * PLANE;
#pragma unroll
        for (int pc = 0; pc < 4; ++pc) {
            uint4 hv, lv;
            split256_pair<LAYOUT>(r, pc, 0, hv.x, lv.x);
            split256_pair<LAYOUT>(r, pc, 1, hv.y, lv.y);
            split256_pair<LAYOUT>(r, pc, 2, hv.z, lv.z);
            split256_pair<LAYOUT>(r, pc, 3, hv.w, lv.w);
            *reinterpret_cast<uint4*>(wr + wr_unit[pc]) = hv;
            *reinterpret_cast<uint4*>(wr + PLANE + wr_unit[pc]) = lv;
        }
    };
    float4 r[8];
    // One k step on LDS stage `buf`: 48 MFMAs in four groups (ks, jp) of twelve; the three products
    // of an accumulator are four MFMAs apart (back to back they would wait for each other).
    // With STAGE the tile held in r is split and stored into the other LDS stage during groups
    // 2 and 3: two pairs after every three MFMAs, fenced so that the order survives scheduling.
    // An MFMA occupies the matrix pipe for 32 cycles and the wavefront issues the conversions
    // meanwhile.  With FETCH the registers are refilled (tile at knext) once the last pair is split.
    auto step = [&](int buf, auto stage_c, auto fetch_c, int knext) __attribute__((always_inline)) {
        constexpr bool STAGE = decltype(stage_c)::value, FETCH = decltype(fetch_c)::value;
        const char* Ah = lds + buf * 4 * PLANE;
        const char* Al = Ah + PLANE;
        const char* Bh = Ah + 2 * PLANE;
        const char* Bl = Ah + 3 * PLANE;
        char* const wr = lds + (buf ^ 1) * 4 * PLANE;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {              // 16 k per MFMA: units 2 ks + lk
            bf16x8 ah[2], al[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t ua = bf_unit32(wm + 32 * i + lm, 2 * ks + lk);
                ah[i] = *reinterpret_cast<const bf16x8*>(Ah + ua);
                al[i] = *reinterpret_cast<const bf16x8*>(Al + ua);
            }
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                bf16x8 bh[2], bl[2];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const uint32_t ub = bf_unit32(wn + 32 * (2 * jp + jj) + lm, 2 * ks + lk);
                    bh[jj] = *reinterpret_cast<const bf16x8*>(Bh + ub);
                    bl[jj] = *reinterpret_cast<const bf16x8*>(Bl + ub);
                }
                uint32_t hw[4], lw[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
#pragma unroll
                    for (int e = 3 * c; e < 3 * c + 3; ++e) {
                        const int t = e >> 2, jj = (e >> 1) & 1, i = e & 1;
                        acc[i][2 * jp + jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            t == 0 ? al[i] : ah[i], t == 1 ? bl[jj] : bh[jj], acc[i][2 * jp + jj], 0, 0, 0);
                    }
                    if (STAGE && ks == 1) {
                        const int piece = 2 * jp + (c >> 1), q0 = 2 * (c & 1);
#pragma unroll
                        for (int q = q0; q < q0 + 2; ++q) split256_pair<LAYOUT>(r, piece, q, hw[q], lw[q]);
                        if (c & 1) {
                            *reinterpret_cast<uint4*>(wr + wr_unit[piece]) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                            *reinterpret_cast<uint4*>(wr + PLANE + wr_unit[piece]) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
                        }
                    }
                    // scalar work, global loads and LDS reads may still move across
                    __builtin_amdgcn_sched_barrier(0x124);
                }
            }
        }
        if (FETCH) fetch(knext, r);
    };
    using std::true_type;
    using std::false_type;

    for (int sg = 0; sg < nseg; ++sg) {
        const int tile_id = seg_tile[sg];
        int mi, ni;
        tile_coords(tile_id, M / BM2, gn, mi, ni);
        m0 = mi * BM2;
        n0 = ni * BN2;
        kbeg = seg_kb[sg];
        kend = seg_ke[sg];
        Cz = C + (int64_t)seg_plane[sg] * split_stride;
        set_tile();
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

        fetch(kbeg, r);
        stage(0, r);
        if (kbeg + SPK2 < kend) fetch(kbeg + SPK2, r);
        __syncthreads();
        int buf = 0, k0 = kbeg;
        for (; k0 + 2 * SPK2 < kend; k0 += SPK2, buf ^= 1) {
            step(buf, true_type{}, true_type{}, k0 + 2 * SPK2);
            __syncthreads();
        }
        if (k0 + SPK2 < kend) {                       // last but one step: nothing left to fetch
            step(buf, true_type{}, false_type{}, 0);
            __syncthreads();
            buf ^= 1;
        }
        step(buf, false_type{}, false_type{}, 0);     // last step

#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                    const int n = n0 + wn + j * 32 + lm;
                    Cz[(int64_t)m * N + n] = acc[i][j][v];
                }
        if (sg + 1 < nseg) __syncthreads();           // the next segment reuses the LDS stages
    }
}

// Y = X Wd^T and dX = dY Wd with BFLOAT16 activations (A m-major, bfloat16) and the fp32 dense
// weight copy (B m-major for NT, k-major for NN): A is exact in bfloat16, so a term is
// a b_hi + a b_lo, two MFMAs, and A's tile is copied to LDS as it is (one 16-byte unit = eight k of
// one row).  Tile, wavefront layout, LDS stages and swizzle of k_gemm_split256; every thread
// stages two units of A (rows mmajor_row(p, 2 h + t), unit p & 3) and two pieces of B (m-major:
// the same rows and unit; k-major: the patch 8 k x 2 columns of the mixed form there).  A step
// is 32 MFMAs; the eight hi/lo pairs of the next B tile follow every second MFMA of its second half.
template <bool B_KMAJOR>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k_gemm_a16_256(const uint16_t* __restrict__ A, int64_t lda, const float* __restrict__ B, int64_t ldb,
                    float* __restrict__ C, int M, int N, int Kdim) {
    constexpr int PLANE = BM2 * 64;
    __shared__ __attribute__((aligned(16))) char lds[2 * 4 * PLANE];     // [stage][A, (unused), B hi, B lo]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 128;
    const int gn = N / BN2, ntiles = (M / BM2) * gn;
    const int Q = (ntiles + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tile_id = xcd * Q + slot;
    if (slot >= Q || tile_id >= ntiles) return;
    int mi, ni;
    tile_coords(tile_id, M / BM2, gn, mi, ni);
    const int m0 = mi * BM2, n0 = ni * BN2;

    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int h = __builtin_amdgcn_readfirstlane(tid >> 8), p = tid & 255;
    const int64_t pa = 2 * lda, pb = 4 * ldb;
    const char* const base_a = reinterpret_cast<const char*>(A) + (int64_t)m0 * pa;
    const char* const base_b = B_KMAJOR ? reinterpret_cast<const char*>(B + n0)
                                        : reinterpret_cast<const char*>(B) + (int64_t)n0 * pb;
    uint32_t voff_a[2], voff_b[2], wr_a[2], wr_b[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int row = mmajor_row(p, 2 * h + t);
        voff_a[t] = (uint32_t)(row * pa + 16 * (p & 3));
        wr_a[t] = bf_unit32(row, p & 3);
        if (!B_KMAJOR) {
            voff_b[t] = (uint32_t)(row * pb + 32 * (p & 3));
            wr_b[t] = 2 * PLANE + bf_unit32(row, p & 3);
        } else {
            wr_b[t] = 2 * PLANE + bf_unit32(4 * (p & 63) + 2 * h + t, p >> 6);
        }
    }
    if (B_KMAJOR) {
        voff_b[0] = (uint32_t)(8 * (p >> 6) * pb + 16 * (p & 63) + 8 * h);
        voff_b[1] = 0;
    }
    uint4 ra[2];
    float4 rb[4];
    auto fetch = [&](int k0) __attribute__((always_inline)) {
        const char* ca = base_a + 2 * (int64_t)k0;
#pragma unroll
        for (int t = 0; t < 2; ++t) ra[t] = *reinterpret_cast<const uint4*>(ca + voff_a[t]);
        if (!B_KMAJOR) {
            const char* cb = base_b + 4 * (int64_t)k0;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                rb[2 * t] = *reinterpret_cast<const float4*>(cb + voff_b[t]);
                rb[2 * t + 1] = *reinterpret_cast<const float4*>(cb + voff_b[t] + 16);
            }
        } else {
            const char* row = base_b + (int64_t)k0 * pb;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float2 e = *reinterpret_cast<const float2*>(row + (2 * t) * pb + voff_b[0]);
                const float2 o = *reinterpret_cast<const float2*>(row + (2 * t + 1) * pb + voff_b[0]);
                rb[t] = make_float4(e.x, e.y, o.x, o.y);
            }
        }
    };
    // pair q (0..3) of B piece pc (0..1)
    auto pair_b = [&](int pc, int q, uint32_t& hi, uint32_t& lo) __attribute__((always_inline)) {
        if (!B_KMAJOR) {
            const float4& v = rb[2 * pc + (q >> 1)];
            if (q & 1) split_pair(v.z, v.w, hi, lo);
            else split_pair(v.x, v.y, hi, lo);
        } else {
            const float4& v = rb[q];
            if (pc == 0) split_pair(v.x, v.z, hi, lo);
            else split_pair(v.y, v.w, hi, lo);
        }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
        char* const wr = lds + buf * 4 * PLANE;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            *reinterpret_cast<uint4*>(wr + wr_a[t]) = ra[t];
            uint4 hv, lv;
            pair_b(t, 0, hv.x, lv.x);
            pair_b(t, 1, hv.y, lv.y);
            pair_b(t, 2, hv.z, lv.z);
            pair_b(t, 3, hv.w, lv.w);
            *reinterpret_cast<uint4*>(wr + wr_b[t]) = hv;
            *reinterpret_cast<uint4*>(wr + PLANE + wr_b[t]) = lv;
        }
    };
    const int lk = lane >> 5, lm = lane & 31;
    auto step = [&](int buf, auto stage_c, auto fetch_c, int knext) __attribute__((always_inline)) {
        constexpr bool STAGE = decltype(stage_c)::value, FETCH = decltype(fetch_c)::value;
        const char* Ap = lds + buf * 4 * PLANE;
        const char* Bh = Ap + 2 * PLANE;
        const char* Bl = Ap + 3 * PLANE;
        char* const wr = lds + (buf ^ 1) * 4 * PLANE;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 a[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(Ap + bf_unit32(wm + 32 * i + lm, 2 * ks + lk));
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                bf16x8 bh[2], bl[2];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const uint32_t ub = bf_unit32(wn + 32 * (2 * jp + jj) + lm, 2 * ks + lk);
                    bh[jj] = *reinterpret_cast<const bf16x8*>(Bh + ub);
                    bl[jj] = *reinterpret_cast<const bf16x8*>(Bl + ub);
                }
                uint32_t hw[4], lw[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
#pragma unroll
                    for (int e = 2 * c; e < 2 * c + 2; ++e) {           // e = 4 t + 2 jj + i: a b_lo first, then a b_hi
                        const int t = e >> 2, jj = (e >> 1) & 1, i = e & 1;
                        acc[i][2 * jp + jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], t == 0 ? bl[jj] : bh[jj],
                                                                                      acc[i][2 * jp + jj], 0, 0, 0);
                    }
                    if (STAGE && ks == 1) {
                        pair_b(jp, c, hw[c], lw[c]);                    // piece jp: its four pairs over this group's chunks
                        if (c == 3) {
                            *reinterpret_cast<uint4*>(wr + wr_a[jp]) = ra[jp];
                            *reinterpret_cast<uint4*>(wr + wr_b[jp]) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                            *reinterpret_cast<uint4*>(wr + PLANE + wr_b[jp]) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0x124);
                }
            }
        }
        if (FETCH) fetch(knext);
    };
    using std::true_type;
    using std::false_type;

    fetch(0);
    stage(0);
    if (SPK2 < Kdim) fetch(SPK2);
    __syncthreads();
    int buf = 0, k0 = 0;
    for (; k0 + 2 * SPK2 < Kdim; k0 += SPK2, buf ^= 1) {
        step(buf, true_type{}, true_type{}, k0 + 2 * SPK2);
        __syncthreads();
    }
    if (k0 + SPK2 < Kdim) {
        step(buf, true_type{}, false_type{}, 0);
        __syncthreads();
        buf ^= 1;
    }
    step(buf, false_type{}, false_type{}, 0);

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                const int n = n0 + wn + j * 32 + lm;
                C[(int64_t)m * N + n] = acc[i][j][v];
            }
}

// The same split product on a 256 x 160 or 256 x 192 workgroup tile: for outputs 1280 wide (five
// 256-tiles across leave 160 tiles for 256 CUs at T = 8192; eight 160-tiles across give 256) and
// for outputs 2304 or 3072 wide (288 / 384 tiles of 256 x 256 need two rounds of which the second is
// an eighth / half full; 384 / 512 tiles of 256 x 192 fill one and a half / two).  A m-major
// (NT and NN products).  Eight wavefronts stacked along m, each 32 rows x 160 (192) columns (5 (6) MFMA
// tiles, 80 (96) accumulator registers); per 16-k slice a wavefront reads 2 A and 10 (12) B fragments for
// 15 (18) MFMAs, issued product-major so that the three products of an accumulator are five (six) apart.
// Staging roles (p = tid & 255, h = tid >> 8, uniform per wavefront):
//   m-major B (NT): threads 0..255 stage A as in k_gemm_split256; of threads 256..511 the first
//     160 (192) stage B, unit p & 3 of rows 16 (p >> 4) + 4 ((p >> 2) & 3) + it, it = 0..3; the other
//     96 (64) repeat the first ones (same loads, same LDS values), so the loop has no predicate.
//   k-major B (NN): every thread stages two m-major pieces of A (it = 2 h, 2 h + 1) and two columns
//     of B: the patch 8 k x 2 columns (k group tid / 80 (96), columns 2 (tid % 80 (96)) ..) of the
//     first 320 (384) threads, repeated by the rest; registers as the mixed form of k_gemm_split256.
// The next tile is split and stored during the second 16-k slice, one pair after every MFMA.
// (Measured and dropped for a k-major B: four-byte loads that give both roles one register
// form, and a mask-select between the two forms: both leave the loads too little time.)
constexpr int BN3 = 160;          // (the narrower of the two widths; whole-tile test of the dispatch)
template <int BNW, bool B_KMAJOR>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k_gemm_split_n160(const float* __restrict__ A, int64_t lda, const float* __restrict__ B, int64_t ldb,
                       float* __restrict__ C, int M, int N, int Kdim, int k_per_split, int64_t split_stride) {
    constexpr int PLANE = BM2 * 64;
    constexpr int LAYOUT = B_KMAJOR ? 2 : 1;
    __shared__ __attribute__((aligned(16))) char lds[2 * 4 * PLANE];     // [stage][A hi, A lo, B hi, B lo]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave * 32;
    constexpr int NJ = BNW / 32;
    static_assert(BNW == 160 || BNW == 192, "five or six MFMA tiles across");
    const int gn = N / BNW, ntiles = (M / BM2) * gn, nsplit = (Kdim + k_per_split - 1) / k_per_split;
    const int Q = (ntiles + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int split = slot / Q, tile_id = xcd * Q + slot % Q;
    if (tile_id >= ntiles || split >= nsplit) return;
    int mi, ni;
    tile_coords(tile_id, M / BM2, gn, mi, ni);
    const int m0 = mi * BM2, n0 = ni * BNW;
    const int kbeg = split * k_per_split;
    const int kend = min(Kdim, kbeg + k_per_split);
    float* Cz = C + (int64_t)split * split_stride;

    floatx16 acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    const int h = __builtin_amdgcn_readfirstlane(tid >> 8), p = tid & 255;
    const int64_t pa = 4 * lda, pb = 4 * ldb;
    const char* base0;                                // NT: this thread's operand; NN: A
    const char* base1 = nullptr;                      // NN: B
    uint32_t voff[4], wr_unit[4];
    if (LAYOUT == 1) {
        if (h == 0) {
            base0 = reinterpret_cast<const char*>(A) + (int64_t)m0 * pa;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                voff[it] = (uint32_t)(mmajor_row(p, it) * pa + 32 * (p & 3));
                wr_unit[it] = bf_unit32(mmajor_row(p, it), p & 3);
            }
        } else {
            const int q = p < BNW ? p : p - BNW;
            base0 = reinterpret_cast<const char*>(B) + (int64_t)n0 * pb;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int row = 16 * (q >> 4) + 4 * ((q >> 2) & 3) + it;
                voff[it] = (uint32_t)(row * pb + 32 * (q & 3));
                wr_unit[it] = 2 * PLANE + bf_unit32(row, q & 3);
            }
        }
    } else {
        base0 = reinterpret_cast<const char*>(A) + (int64_t)m0 * pa;
        base1 = reinterpret_cast<const char*>(B + n0);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            voff[t] = (uint32_t)(mmajor_row(p, 2 * h + t) * pa + 32 * (p & 3));
            wr_unit[t] = bf_unit32(mmajor_row(p, 2 * h + t), p & 3);
        }
        const int q = tid < 2 * BNW ? tid : tid - 2 * BNW, nq = q % (BNW / 2), kg = q / (BNW / 2);
        voff[2] = (uint32_t)(8 * kg * pb + 8 * nq);
        voff[3] = 0;
        wr_unit[2] = 2 * PLANE + bf_unit32(2 * nq, kg);
        wr_unit[3] = 2 * PLANE + bf_unit32(2 * nq + 1, kg);
    }
    float4 r[8];
    auto fetch = [&](int k0) __attribute__((always_inline)) {
        const char* col = base0 + 4 * (int64_t)k0;
        if (LAYOUT == 1) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                r[2 * it] = *reinterpret_cast<const float4*>(col + voff[it]);
                r[2 * it + 1] = *reinterpret_cast<const float4*>(col + voff[it] + 16);
            }
        } else {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                r[2 * t] = *reinterpret_cast<const float4*>(col + voff[t]);
                r[2 * t + 1] = *reinterpret_cast<const float4*>(col + voff[t] + 16);
            }
            const char* row = base1 + (int64_t)k0 * pb;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float2 e = *reinterpret_cast<const float2*>(row + (2 * t) * pb + voff[2]);
                const float2 o = *reinterpret_cast<const float2*>(row + (2 * t + 1) * pb + voff[2]);
                r[4 + t] = make_float4(e.x, e.y, o.x, o.y);
            }
        }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
        char* const wr = lds + buf * 4 * PLANE;
#pragma unroll
        for (int pc = 0; pc < 4; ++pc) {
            uint4 hv, lv;
            split256_pair<LAYOUT>(r, pc, 0, hv.x, lv.x);
            split256_pair<LAYOUT>(r, pc, 1, hv.y, lv.y);
            split256_pair<LAYOUT>(r, pc, 2, hv.z, lv.z);
            split256_pair<LAYOUT>(r, pc, 3, hv.w, lv.w);
            *reinterpret_cast<uint4*>(wr + wr_unit[pc]) = hv;
            *reinterpret_cast<uint4*>(wr + PLANE + wr_unit[pc]) = lv;
        }
    };
    const int lk = lane >> 5, lm = lane & 31;
    auto step = [&](int buf, auto stage_c, auto fetch_c, int knext) __attribute__((always_inline)) {
        constexpr bool STAGE = decltype(stage_c)::value, FETCH = decltype(fetch_c)::value;
        const char* Ah = lds + buf * 4 * PLANE;
        const char* Al = Ah + PLANE;
        const char* Bh = Ah + 2 * PLANE;
        const char* Bl = Ah + 3 * PLANE;
        char* const wr = lds + (buf ^ 1) * 4 * PLANE;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const uint32_t ua = bf_unit32(wm + lm, 2 * ks + lk);
            const bf16x8 ah = *reinterpret_cast<const bf16x8*>(Ah + ua);
            const bf16x8 al = *reinterpret_cast<const bf16x8*>(Al + ua);
            bf16x8 bh[NJ], bl[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint32_t ub = bf_unit32(32 * j + lm, 2 * ks + lk);
                bh[j] = *reinterpret_cast<const bf16x8*>(Bh + ub);
                bl[j] = *reinterpret_cast<const bf16x8*>(Bl + ub);
            }
            uint32_t hw[4], lw[4];
#pragma unroll
            for (int e = 0; e < 3 * NJ; ++e) {                      // e = NJ t + j; products t: lo.hi, hi.lo, hi.hi
                const int t = e / NJ, j = e % NJ;
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t == 0 ? al : ah, t == 1 ? bl[j] : bh[j], acc[j], 0, 0, 0);
                if (STAGE && ks == 1) {
                    // pair e after MFMA e (with 15 MFMAs the sixteenth pair goes with the last, with 18 the last two
                    // carry none); a piece's two units leave after its fourth pair
#pragma unroll
                    for (int pr = e; pr < ((3 * NJ < 16 && e == 3 * NJ - 1) ? 16 : (e < 16 ? e + 1 : e)); ++pr) {
                        split256_pair<LAYOUT>(r, pr >> 2, pr & 3, hw[pr & 3], lw[pr & 3]);
                        if ((pr & 3) == 3) {
                            *reinterpret_cast<uint4*>(wr + wr_unit[pr >> 2]) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                            *reinterpret_cast<uint4*>(wr + PLANE + wr_unit[pr >> 2]) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0x124);
            }
        }
        if (FETCH) fetch(knext);
    };
    using std::true_type;
    using std::false_type;

    fetch(kbeg);
    stage(0);
    if (kbeg + SPK2 < kend) fetch(kbeg + SPK2);
    __syncthreads();
    int buf = 0, k0 = kbeg;
    for (; k0 + 2 * SPK2 < kend; k0 += SPK2, buf ^= 1) {
        step(buf, true_type{}, true_type{}, k0 + 2 * SPK2);
        __syncthreads();
    }
    if (k0 + SPK2 < kend) {
        step(buf, true_type{}, false_type{}, 0);
        __syncthreads();
        buf ^= 1;
    }
    step(buf, false_type{}, false_type{}, 0);

#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + wm + 8 * (v >> 2) + 4 * lk + (v & 3);
            const int n = n0 + j * 32 + lm;
            Cz[(int64_t)m * N + n] = acc[j][v];
        }
}

// G = A^T B with BOTH operands bfloat16 and k-major (A [K x M], B [K x N]): the same 256 x 256
// workgroup tile, eight wavefronts of 64 x 128 and two LDS stages as k_gemm_split256, k steps of
// 64: the two planes of an operand hold its k halves (0..31, 32..63) instead of hi and lo, one
// MFMA product per term.  A thread stages a patch of 8 k x 8 rows: eight 16-byte loads, an
// 8 x 8 halfword transpose in registers (v_perm_b32), eight 16-byte LDS units (one per row).
// Staging of the next tile is spread over the second half of a step's MFMAs, as there.
// (Four wavefronts of 128 x 128 with the accumulators in the accumulation half of the
// register file measured 15 % slower: one wavefront per SIMD leaves every wait exposed.)
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k_gemm_tn_bf16_256(const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ B, int64_t ldb,
                        float* __restrict__ C, int M, int N, int Kdim, int k_per_split, int64_t split_stride) {
    constexpr int PLANE = BM2 * 64, KS = 64;
    __shared__ __attribute__((aligned(16))) char lds[2 * 4 * PLANE];     // [stage][A k<32, A k>=32, B k<32, B k>=32]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 128;
    const int gn = N / BN2, ntiles = (M / BM2) * gn, nsplit = (Kdim + k_per_split - 1) / k_per_split;
    const int Q = (ntiles + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int split = slot / Q, tile_id = xcd * Q + slot % Q;
    if (tile_id >= ntiles || split >= nsplit) return;
    int mi, ni;
    tile_coords(tile_id, M / BM2, gn, mi, ni);
    const int m0 = mi * BM2, n0 = ni * BN2;
    const int kbeg = split * k_per_split;
    const int kend = min(Kdim, kbeg + k_per_split);
    float* Cz = C + (int64_t)split * split_stride;

    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // h: 0 stages A, 1 stages B; uniform per wavefront, so base and row pitch stay scalar and a
    // load's address is scalar row + per-thread 32-bit offset
    const int h = __builtin_amdgcn_readfirstlane(tid >> 8), p = tid & 255, mq = p & 31, kg = p >> 5;
    const int64_t pitch = 2 * (h == 0 ? lda : ldb);
    const char* const sbase = reinterpret_cast<const char*>(h == 0 ? A + m0 : B + n0);
    const uint32_t voff = (uint32_t)(8 * kg * pitch + 16 * mq);
    uint4 r[8];
    auto fetch = [&](int k0) __attribute__((always_inline)) {
        const char* row = sbase + (int64_t)k0 * pitch;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) r[kk] = *reinterpret_cast<const uint4*>(row + kk * pitch + voff);
    };
    const uint32_t wr_plane = (uint32_t)((2 * h + (kg >> 2)) * PLANE);
    uint32_t wr_unit[8];                              // row 8 mq + j, unit kg & 3
#pragma unroll
    for (int j = 0; j < 8; ++j) wr_unit[j] = wr_plane + bf_unit32(8 * mq + j, kg & 3);
    // row j of the patch: halfword j of the eight registers, k ascending
    auto piece = [&](int j) __attribute__((always_inline)) -> uint4 {
        const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
        uint32_t o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t w0 = u4_at(r[2 * d], j >> 1), w1 = u4_at(r[2 * d + 1], j >> 1);
            o[d] = __builtin_amdgcn_perm(w1, w0, sel);
        }
        return make_uint4(o[0], o[1], o[2], o[3]);
    };
    const int lk = lane >> 5, lm = lane & 31;
    // one k step (64) on LDS stage buf: four groups (k half, 16-k slice) of eight MFMAs; with STAGE
    // groups 2 and 3 each store four rows of the next tile, one row after every two MFMAs
    auto step = [&](int buf, auto stage_c, auto fetch_c, int knext) __attribute__((always_inline)) {
        constexpr bool STAGE = decltype(stage_c)::value, FETCH = decltype(fetch_c)::value;
        const char* base = lds + buf * 4 * PLANE;
        char* const wr = lds + (buf ^ 1) * 4 * PLANE;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const char* Ap = base + (g >> 1) * PLANE;
            const char* Bp = base + (2 + (g >> 1)) * PLANE;
            const int ks = g & 1;
            bf16x8 a[2], b[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(Ap + bf_unit32(wm + 32 * i + lm, 2 * ks + lk));
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = *reinterpret_cast<const bf16x8*>(Bp + bf_unit32(wn + 32 * j + lm, 2 * ks + lk));
#pragma unroll
            for (int c = 0; c < 4; ++c) {
#pragma unroll
                for (int e = 2 * c; e < 2 * c + 2; ++e)
                    acc[e & 1][e >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[e & 1], b[e >> 1], acc[e & 1][e >> 1], 0, 0, 0);
                if (STAGE && g >= 2) {
                    const int j = 4 * (g - 2) + c;
                    *reinterpret_cast<uint4*>(wr + wr_unit[j]) = piece(j);
                }
                __builtin_amdgcn_sched_barrier(0x124);     // scalar work, global loads and LDS reads may still move
            }
        }
        if (FETCH) fetch(knext);
    };
    using std::true_type;
    using std::false_type;

    fetch(kbeg);
#pragma unroll
    for (int j = 0; j < 8; ++j) *reinterpret_cast<uint4*>(lds + wr_unit[j]) = piece(j);
    if (kbeg + KS < kend) fetch(kbeg + KS);
    __syncthreads();
    int buf = 0, k0 = kbeg;
    for (; k0 + 2 * KS < kend; k0 += KS, buf ^= 1) {
        step(buf, true_type{}, true_type{}, k0 + 2 * KS);
        __syncthreads();
    }
    if (k0 + KS < kend) {
        step(buf, true_type{}, false_type{}, 0);
        __syncthreads();
        buf ^= 1;
    }
    step(buf, false_type{}, false_type{}, 0);

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                const int n = n0 + wn + j * 32 + lm;
                Cz[(int64_t)m * N + n] = acc[i][j][v];
            }
}

// C[i] = part[i] + part[stride + i] + ... (nsplit planes, added in ascending order)
__global__ void k_splitk_reduce(const float* __restrict__ part, int64_t stride, int nsplit,
                                float* __restrict__ C, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int z = 0; z < nsplit; ++z) s += part[(int64_t)z * stride + i];
    C[i] = s;
}
// the same with four consecutive outputs per thread (n and stride multiples of 4, 16-byte aligned
// bases): 16-byte loads, a quarter of the threads
__global__ void k_splitk_reduce4(const float* __restrict__ part, int64_t stride, int nsplit,
                                 float* __restrict__ C, int64_t n4) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    const float4* p = reinterpret_cast<const float4*>(part) + i;
    const int64_t s4 = stride >> 2;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    int z = 0;
    for (; z + 4 <= nsplit; z += 4) {
        const float4 a = p[(int64_t)z * s4], b = p[(int64_t)(z + 1) * s4], c = p[(int64_t)(z + 2) * s4], d = p[(int64_t)(z + 3) * s4];
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
        s.x += b.x; s.y += b.y; s.z += b.z; s.w += b.w;
        s.x += c.x; s.y += c.y; s.z += c.z; s.w += c.w;
        s.x += d.x; s.y += d.y; s.z += d.z; s.w += d.w;
    }
    for (; z < nsplit; ++z) {
        const float4 a = p[(int64_t)z * s4];
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
    reinterpret_cast<float4*>(C)[i] = s;
}
static int sum_split_planes(const float* part, int64_t stride, int nsplit, float* C, int64_t n, hipStream_t s) {
    if (n % 4 == 0 && stride % 4 == 0 && aligned16(part) && aligned16(C))
        k_splitk_reduce4<<<(unsigned)cdiv(n / 4, 256), 256, 0, s>>>(part, stride, nsplit, C, n / 4);
    else
        k_splitk_reduce<<<(unsigned)cdiv(n, 256), 256, 0, s>>>(part, stride, nsplit, C, n);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

// Number of k ranges (blockIdx.x) a GEMM of `tiles` output tiles is split into.  A CU holds
// `wg_per_cu` workgroups; the grid should fill 256 x wg_per_cu places a whole number of
// times.  Cost of a choice = (k steps per workgroup x step_us + wg_us) x rounds, a last
// partial round counting `last[]` by quarters of the places it fills, plus the pass that
// adds the partial outputs.  Constants fitted to timings of the dense gradient at GPT-2
// small / medium / large shapes (fp32 kernel: 2.7 % rms error; bf16 kernel: 9 %).
struct SplitModel {
    int wg_per_cu, bk;
    double step_us, wg_us, sum_us_per_float, last[3];
};
static const SplitModel kSplitF32 = {4, BK, 4.63, 10.7, 5e-7, {0.44, 0.63, 0.84}};
static const SplitModel kSplitBf16 = {3, BKH, 2.08, 3.0, 1.8e-6, {0.69, 0.76, 0.86}};

static int pick_nsplit(int64_t tiles, int Kdim, const SplitModel& md, int64_t max_split) {
    const int64_t places = 256 * md.wg_per_cu;
    int best = 1;
    double best_cost = 0.0;
    const int64_t hi = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(16, max_split), Kdim / 256));
    for (int ns = 1; ns <= hi; ++ns) {
        const int64_t n = tiles * ns, full = n / places, rest = n % places;
        const double steps = (double)cdiv(cdiv(Kdim, ns), md.bk);
        const double frac = (double)rest / (double)places;
        const double last = rest == 0 ? 0.0 : frac <= 0.25 ? md.last[0] : frac <= 0.5 ? md.last[1] : frac <= 0.75 ? md.last[2] : 1.0;
        const double cost = (steps * md.step_us + md.wg_us) * ((double)full + last) +
                            (ns > 1 ? md.sum_us_per_float * (double)ns * (double)tiles * 128.0 * 128.0 : 0.0);
        if (best_cost == 0.0 || cost < best_cost) {
            best_cost = cost;
            best = ns;
        }
    }
    return best;
}

// `left_unsummed`: if not null the partial outputs of a split stay in split_ws and their number
// is returned there (1: the result is in C); otherwise they are added into C.
template <typename TA, bool AK, typename TB, bool BKM>
static int launch(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int M, int N, int Kdim,
                  float* split_ws, int64_t split_ws_floats, int* left_unsummed, hipStream_t s) {
    // (a 256 x 128 tile was measured: a third less operand traffic per flop, no gain in time)
    const int tm = 128;
    const int gm = (int)cdiv(M, tm), gn = (int)cdiv(N, 128);
    const int64_t mn = (int64_t)M * N;
    const int nsplit0 = split_ws ? pick_nsplit((int64_t)gm * gn, Kdim, kSplitF32, split_ws_floats / mn) : 1;
    const int kps = (int)(cdiv(cdiv(Kdim, nsplit0), BK) * BK);
    const int nsplit = (int)cdiv(Kdim, kps);
    dim3 grid(nsplit, gn, gm);
    float* dst = nsplit > 1 ? split_ws : C;
    // 16-byte loads need every row start aligned: leading dimension a multiple of 4
    // elements (the k ranges of the splits start at multiples of BK)
    const int vec_a = (lda % 4 == 0) ? 1 : 0, vec_b = (ldb % 4 == 0) ? 1 : 0;
    k_gemm<TA, AK, TB, BKM, 128><<<grid, 256, 0, s>>>((const TA*)A, lda, (const TB*)B, ldb, dst, M, N, Kdim, kps, mn,
                                                     vec_a, vec_b);
    MST_LAUNCH_CHECK();
    if (left_unsummed) {
        *left_unsummed = nsplit;
        return MST_OK;
    }
    if (nsplit > 1) {
        const int rcs = sum_split_planes(split_ws, mn, nsplit, C, mn, s);
        if (rcs != MST_OK) return rcs;
    }
    return MST_OK;
}

// Workgroup tile and split count of the bf16-split kernels, chosen together.  Tiles are dealt to
// the XCDs in equal shares (Q each).  An XCD has 32 CUs: 64 places for the 128-tile kernel (two
// workgroups per CU), 32 for the 256-tile kernel, so what matters is how many rounds Q x splits
// needs on ONE XCD.  Modelled time = rounds x (k steps per workgroup + start-up and output of a
// workgroup, in steps) x time of a step, plus the traffic of the partial outputs.  Constants
// from timings on MI355X: a 64-k step of two co-resident 128 x 128 tiles 3.3 us, a 32-k step of
// a 256 x 256 tile 2.0 us (1.6x the work per CU and time), of a 256 x 160 tile 1.8 us and of a
// 256 x 192 tile 2.1 us (less work per staged byte: they pay only where they fill CUs that the 256
// tile leaves idle), start-up + output 7, 13, 7 and 7 steps.
// The model reproduces the measured times of the GPT-2 small / large products within 15 % and
// orders the candidates as measured.
struct SplitPlan {
    int tile, nsplit;
};
static SplitPlan plan_split(int M, int N, int Kdim, int64_t max_split, bool summed, bool allow128, bool allow256,
                            bool allow160, bool allow192) {
    static const int cand[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    SplitPlan best{0, 1};
    double best_cost = 0.0;
    for (int tile : {128, 256, 160, 192}) {           // 160, 192: 256 rows x 160 / 192 columns (A m-major only)
        if (tile == 128 ? !allow128 : tile == 256 ? !allow256 : tile == 160 ? !allow160 : !allow192) continue;
        const int tm = tile == 128 ? 128 : 256, tn = tile;
        const int kstep = tile == 128 ? SPK : 32, places = tile == 128 ? 64 : 32;
        const double unit_us = tile == 128 ? 3.3 : tile == 256 ? 2.0 : tile == 160 ? 1.8 : 2.1, wg_steps = tile == 128 ? 7.0 : tile == 256 ? 13.0 : 7.0;
        if (M % tm != 0 || N % tn != 0 || Kdim % kstep != 0) continue;
        const int64_t Q = cdiv((int64_t)(M / tm) * (N / tn), 8);
        for (int ns : cand) {
            if (ns > 1 && (ns > max_split || Kdim / ns < 512)) continue;
            const double steps = (double)cdiv(cdiv(Kdim, ns), kstep);
            double cost = (double)cdiv(Q * ns, places) * (steps + wg_steps) * unit_us;
            // partial outputs: written and read once each, plus the sum's write (4 B at about 4 TB/s);
            // left unsummed they are read sparsely by the caller's gather
            if (ns > 1) cost += 1.0e-6 * (double)M * (double)N * (summed ? ns + 1.0 : 0.25 * ns);
            if (best.tile == 0 || cost < best_cost) {
                best_cost = cost;
                best = SplitPlan{tile, ns};
            }
        }
    }
    return best;
}
static int g_gemm_fp32_only = 0;          // test hook: 1 = never use the bf16-split kernel
static int g_last_tile = 0;               // workgroup tile of the last split-kernel launch (128 / 256 / 160), 0: another kernel
static int g_sched52 = 1;                 // test hook: 0 = never the five-for-two schedule
static int g_split_tile = 0;              // test hook: 0 = automatic, 128 / 256 / 160 / 192 = that workgroup tile when the shape allows it

int gemm_last_tile() { return g_last_tile; }

int gemm_force_fp32_mfma(int on) {       // 0 automatic, 1 fp32 MFMA kernel, 128 / 256 / 160: split kernel with that tile
    if (on == 52 || on == -52) {                    // (the other settings stay as they are)
        g_sched52 = on > 0;
        return MST_OK;
    }
    g_gemm_fp32_only = on == 1 ? 1 : 0;
    g_split_tile = (on == 128 || on == 256 || on == 160 || on == 192) ? on : 0;
    return MST_OK;
}

// whole tiles of one of the split kernels: 128 x 128 (256 x 256 is a subset) or, for an m-major A, 256 x 160
static bool split_ok(int M, int N, int Kdim, int64_t lda, int64_t ldb, bool a_kmajor) {
    if (g_gemm_fp32_only || Kdim % SPK != 0 || lda % 4 != 0 || ldb % 4 != 0) return false;
    return (M % BM == 0 && N % BN == 0) || (!a_kmajor && M % BM2 == 0 && (N % BN3 == 0 || N % 192 == 0));
}

template <bool AK, bool BKM>
static int launch_split(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int M, int N, int Kdim,
                        float* split_ws, int64_t split_ws_floats, int* left_unsummed, hipStream_t s) {
    const int64_t mn = (int64_t)M * N;
    const int pin = g_split_tile;
    SplitPlan plan = plan_split(M, N, Kdim, split_ws ? split_ws_floats / mn : 1, left_unsummed == nullptr,
                                pin == 0 || pin == 128, pin == 0 || pin == 256, !AK && (pin == 0 || pin == 160),
                                !AK && (pin == 0 || pin == 192));
    if (plan.tile == 0)                               // the pinned tile does not fit this shape: any that does
        plan = plan_split(M, N, Kdim, split_ws ? split_ws_floats / mn : 1, left_unsummed == nullptr, true, true, !AK, !AK);
    const int tile = plan.tile, nsplit0 = plan.nsplit;
    g_last_tile = tile;
    const int kstep = tile == 128 ? SPK : SPK2;
    const int kps = (int)(cdiv(cdiv(Kdim, nsplit0), kstep) * kstep);
    const int nsplit = (int)cdiv(Kdim, kps);
    const int tm = tile == 128 ? 128 : 256;
    const unsigned grid = (unsigned)(8 * cdiv((int64_t)(M / tm) * (N / tile), 8) * nsplit);
    float* dst = nsplit > 1 ? split_ws : C;
    // About 100 tiles of 256 x 256 with two k ranges each leave a fifth of the CUs idle: five
    // workgroups per two tiles instead (k_gemm_split256, sched = 1), three partial planes per tile.
    const int64_t tiles256 = (int64_t)(M / BM2) * (N / BN2);
    const int S = Kdim / SPK2, x_steps = (int)cdiv(2 * S + 13, 5);
    if (tile == 256 && nsplit == 2 && g_sched52 && split_ws && split_ws_floats / mn >= 3 && tiles256 % 2 == 0 &&
        tiles256 * 5 / 2 <= 256 && tiles256 * 2 <= 218 && S - 2 * x_steps >= 8) {
        k_gemm_split256<AK, BKM><<<256u, 512, 0, s>>>((const float*)A, lda, (const float*)B, ldb, split_ws,
                                                                              M, N, Kdim, x_steps * SPK2, mn, 1);
        MST_LAUNCH_CHECK();
        if (left_unsummed) {
            *left_unsummed = 3;
            return MST_OK;
        }
        const int rcs = sum_split_planes(split_ws, mn, 3, C, mn, s);
        if (rcs != MST_OK) return rcs;
        return MST_OK;
    }
    if (tile == 160) {
        if constexpr (!AK)
            k_gemm_split_n160<160, BKM><<<grid, 512, 0, s>>>((const float*)A, lda, (const float*)B, ldb, dst, M, N, Kdim, kps, mn);
    } else if (tile == 192) {
        if constexpr (!AK)
            k_gemm_split_n160<192, BKM><<<grid, 512, 0, s>>>((const float*)A, lda, (const float*)B, ldb, dst, M, N, Kdim, kps, mn);
    } else if (tile == 256)
        k_gemm_split256<AK, BKM><<<grid, 512, 0, s>>>((const float*)A, lda, (const float*)B, ldb, dst, M, N, Kdim, kps, mn, 0);
    else
        k_gemm_split<AK, BKM><<<grid, 256, 0, s>>>((const float*)A, lda, (const float*)B, ldb, dst, M, N, Kdim, kps, mn);
    MST_LAUNCH_CHECK();
    if (left_unsummed) {
        *left_unsummed = nsplit;
        return MST_OK;
    }
    if (nsplit > 1) {
        const int rcs = sum_split_planes(split_ws, mn, nsplit, C, mn, s);
        if (rcs != MST_OK) return rcs;
    }
    return MST_OK;
}

// bfloat16 activations x fp32 dense weights on whole 256 x 256 tiles (16-byte loads of eight bfloat16: K % 32)
static bool a16_ok(int M, int N, int Kdim) {
    return !g_gemm_fp32_only && g_split_tile != 128 && M % BM2 == 0 && N % BN2 == 0 && Kdim % SPK2 == 0;
}
template <bool BKM>
static int launch_a16(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int M, int N, int Kdim,
                      int* left_unsummed, hipStream_t s) {
    const unsigned grid = (unsigned)(8 * cdiv((int64_t)(M / BM2) * (N / BN2), 8));
    k_gemm_a16_256<BKM><<<grid, 512, 0, s>>>((const uint16_t*)A, lda, (const float*)B, ldb, C, M, N, Kdim);
    MST_LAUNCH_CHECK();
    g_last_tile = 256;
    if (left_unsummed) *left_unsummed = 1;
    return MST_OK;
}

static int launch_tn_bf16(const void* A, const void* B, float* C, int M, int N, int Kdim, float* split_ws,
                          int64_t split_ws_floats, int* left_unsummed, hipStream_t s) {
    const int gm = (int)cdiv(M, BM), gn = (int)cdiv(N, BN);
    const int64_t mn = (int64_t)M * N;
    if (g_split_tile != 128 && M % BM2 == 0 && N % BN2 == 0 && Kdim % 64 == 0 &&
        (g_split_tile == 256 || (int64_t)(M / BM2) * (N / BN2) >= 8)) {
        // whole 256 x 256 tiles: the two-stage kernel; split count from the same per-XCD round model
        // (a 64-k step takes about 1.3 us, start-up and output of a workgroup about 16 steps)
        static const int cand[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
        const int64_t Q = cdiv((int64_t)(M / BM2) * (N / BN2), 8), max_split = split_ws ? split_ws_floats / mn : 1;
        int ns_best = 1;
        double best_cost = 0.0;
        for (int ns : cand) {
            if (ns > 1 && (ns > max_split || Kdim / ns < 512)) continue;
            double cost = (double)cdiv(Q * ns, 32) * ((double)cdiv(cdiv(Kdim, ns), 64) + 16.0) * 1.3;
            if (ns > 1) cost += 1.0e-6 * (double)mn * (left_unsummed ? 0.25 * ns : ns + 1.0);
            if (best_cost == 0.0 || cost < best_cost) {
                best_cost = cost;
                ns_best = ns;
            }
        }
        const int kps = (int)(cdiv(cdiv(Kdim, ns_best), 64) * 64);
        const int nsplit = (int)cdiv(Kdim, kps);
        const unsigned grid = (unsigned)(8 * Q * nsplit);
        float* dst = nsplit > 1 ? split_ws : C;
        k_gemm_tn_bf16_256<<<grid, 512, 0, s>>>((const uint16_t*)A, M, (const uint16_t*)B, N, dst, M, N, Kdim, kps, mn);
        MST_LAUNCH_CHECK();
        if (left_unsummed) {
            *left_unsummed = nsplit;
            return MST_OK;
        }
        if (nsplit > 1) {
            const int rcs = sum_split_planes(split_ws, mn, nsplit, C, mn, s);
            if (rcs != MST_OK) return rcs;
        }
        return MST_OK;
    }
    const int nsplit0 = split_ws ? pick_nsplit((int64_t)gm * gn, Kdim, kSplitBf16, split_ws_floats / mn) : 1;
    const int kps = (int)(cdiv(cdiv(Kdim, nsplit0), BKH) * BKH);
    const int nsplit = (int)cdiv(Kdim, kps);
    dim3 grid(nsplit, gn, gm);
    float* dst = nsplit > 1 ? split_ws : C;
    // 16-byte loads of 8 elements need leading dimensions that are multiples of 8 (bases are 16-byte aligned)
    k_gemm_tn_bf16<<<grid, 256, 0, s>>>((const uint16_t*)A, M, (const uint16_t*)B, N, dst, M, N, Kdim, kps, mn,
                                        (M % 8 == 0) ? 1 : 0, (N % 8 == 0) ? 1 : 0);
    MST_LAUNCH_CHECK();
    if (left_unsummed) {
        *left_unsummed = nsplit;
        return MST_OK;
    }
    if (nsplit > 1) {
        const int rcs = sum_split_planes(split_ws, mn, nsplit, C, mn, s);
        if (rcs != MST_OK) return rcs;
    }
    return MST_OK;
}

// TN: C[M x N] = A^T B, A [K x M], B [K x N]          (G = dY^T X)
// NT: C[M x N] = A B^T, A [M x K], B [N x K] (fp32)   (Y = X Wd^T)
// NN: C[M x N] = A B,   A [M x K], B [K x N] (fp32)   (dX = dY Wd)
int gemm_mfma(GemmKind kind, const void* A, mst_dtype a_dt, const void* B, mst_dtype b_dt, float* C,
              int M, int N, int Kdim, float* split_ws, int64_t split_ws_floats, hipStream_t s, int* left_unsummed) {
    const bool ab = a_dt == MST_BF16, bb = b_dt == MST_BF16;
    g_last_tile = 0;
    switch (kind) {
        case GEMM_TN:
            if (ab != bb) return MST_ERR_ARG;
            if (ab) return launch_tn_bf16(A, B, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
            if (split_ok(M, N, Kdim, M, N, true))
                return launch_split<true, true>(A, M, B, N, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
            return launch<float, true, float, true>(A, M, B, N, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
        case GEMM_NT:
            if (bb) return MST_ERR_ARG;
            if (ab && a16_ok(M, N, Kdim)) return launch_a16<false>(A, Kdim, B, Kdim, C, M, N, Kdim, left_unsummed, s);
            if (ab) return launch<uint16_t, false, float, false>(A, Kdim, B, Kdim, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
            if (split_ok(M, N, Kdim, Kdim, Kdim, false))
                return launch_split<false, false>(A, Kdim, B, Kdim, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
            return launch<float, false, float, false>(A, Kdim, B, Kdim, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
        case GEMM_NN:
            if (bb) return MST_ERR_ARG;
            if (ab && a16_ok(M, N, Kdim)) return launch_a16<true>(A, Kdim, B, N, C, M, N, Kdim, left_unsummed, s);
            if (ab) return launch<uint16_t, false, float, true>(A, Kdim, B, N, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
            if (split_ok(M, N, Kdim, Kdim, N, false))
                return launch_split<false, true>(A, Kdim, B, N, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
            return launch<float, false, float, true>(A, Kdim, B, N, C, M, N, Kdim, split_ws, split_ws_floats, left_unsummed, s);
    }
    return MST_ERR_ARG;
}

}  // namespace mst
