// Exact k-selection with index tie-break, and the device side of one Mixed-Growing
// update (Algorithm 1: ArgTopK of -|theta . M|, ArgTopK of |grad| over the inactive
// positions, RandK over the rest, then the mask / weight update).
//
// Each of the three selections is "the k candidates with the smallest (key, index)":
//   prune   candidates = active weights,            key = |w| bits            (32 bit)
//   grad    candidates = inactive positions,        key = 0x7FFFFFFF - |g| bits (32 bit)
//   random  candidates = inactive, not grad-grown,  key = SplitMix64(seed)[f]  (64 bit)
// A most-significant-digit radix select (8-bit digits, one histogram pass per digit)
// finds the k-th smallest key tau on the device; a last ordered pass takes every key
// below tau and, among the keys equal to tau, the lowest indices until k are taken.
// Nothing is read back to the host.
#include "common.h"

namespace mst {

__device__ inline uint32_t abs_bits(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

__device__ inline uint64_t splitmix64_at(uint64_t seed, uint64_t f) {
    uint64_t z = seed + (f + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct PruneKeys {
    typedef uint32_t key_t;
    const float* vals;
    __device__ bool get(int64_t k, key_t& key) const { key = abs_bits(vals[k]); return true; }
};
struct GradKeys {
    typedef uint32_t key_t;
    const float* G;
    const uint8_t* mask;
    __device__ bool get(int64_t f, key_t& key) const {
        if (mask[f]) return false;
        key = 0x7FFFFFFFu - abs_bits(G[f]);
        return true;
    }
};
struct RandKeys {
    typedef uint64_t key_t;
    const uint8_t* mask;
    const uint8_t* sel;
    uint64_t seed;
    __device__ bool get(int64_t f, key_t& key) const {
        if (mask[f] || sel[f]) return false;
        key = splitmix64_at(seed, (uint64_t)f);
        return true;
    }
};

// state words: [0] key prefix fixed so far, [1] how many still to take inside the prefix,
// from word 8 on: 256 uint32 histogram bins
__global__ void k_select_init(uint64_t* state, uint64_t k) {
    if (threadIdx.x == 0) { state[0] = 0; state[1] = k; }
    reinterpret_cast<uint32_t*>(state + 8)[threadIdx.x] = 0;
}

template <typename KS>
__global__ void k_select_hist(KS ks, int64_t n, uint64_t* __restrict__ state, int shift, int first) {
    typedef typename KS::key_t key_t;
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;          // blockDim.x == 256
    __syncthreads();
    const key_t prefix = (key_t)state[0];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        key_t key;
        if (!ks.get(i, key)) continue;
        // (x >> shift) >> 8 keeps every shift amount below the key width
        if (!first && ((key >> shift) >> 8) != ((prefix >> shift) >> 8)) continue;
        atomicAdd(&h[(uint32_t)(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    const uint32_t c = h[threadIdx.x];
    if (c) atomicAdd(reinterpret_cast<uint32_t*>(state + 8) + threadIdx.x, c);
}

// picks the digit that contains the k-th smallest key and clears the histogram
// (256 threads: inclusive scan of the bins, the first bin whose running total reaches k)
__global__ void k_select_pick(uint64_t* __restrict__ state, int shift) {
    __shared__ uint32_t wsum[4];
    __shared__ int pick_bin;
    __shared__ uint32_t pick_before;
    uint32_t* hist = reinterpret_cast<uint32_t*>(state + 8);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint32_t c = hist[t];
    uint32_t x = c;
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) wsum[wave] = x;
    if (t == 0) { pick_bin = 255; pick_before = 0; }
    __syncthreads();
    uint32_t incl = x;
    for (int w = 0; w < wave; ++w) incl += wsum[w];
    const uint64_t k = state[1];
    // exactly one bin has (total before it) < k <= (total including it)
    if ((uint64_t)(incl - c) < k && (uint64_t)incl >= k) { pick_bin = t; pick_before = incl - c; }
    __syncthreads();
    if (t == 0) {
        state[0] |= (uint64_t)pick_bin << shift;
        state[1] = k - pick_before;
    }
    hist[t] = 0;
}

// per block of SELECT_BLOCK indices: how many candidates carry exactly the threshold key
template <typename KS>
__global__ void k_select_ties(KS ks, int64_t n, const uint64_t* __restrict__ state, int* __restrict__ blk) {
    typedef typename KS::key_t key_t;
    __shared__ int cnt;
    if (threadIdx.x == 0) cnt = 0;
    __syncthreads();
    const key_t tau = (key_t)state[0];
    const int64_t base = (int64_t)blockIdx.x * SELECT_BLOCK;
    int mine = 0;
    for (int j = threadIdx.x; j < SELECT_BLOCK; j += blockDim.x) {
        const int64_t i = base + j;
        key_t key;
        if (i < n && ks.get(i, key) && key == tau) ++mine;
    }
    if (mine) atomicAdd(&cnt, mine);
    __syncthreads();
    if (threadIdx.x == 0) blk[blockIdx.x] = cnt;
}

// flags[i] = code for every selected index; 256 threads, 8 consecutive indices each
template <typename KS>
__global__ void k_select_flag(KS ks, int64_t n, const uint64_t* __restrict__ state,
                              const int* blk_excl, uint8_t* flags, uint8_t code) {
    typedef typename KS::key_t key_t;
    constexpr int PER = SELECT_BLOCK / 256;
    __shared__ int wsum[4];
    const key_t tau = (key_t)state[0];
    const int64_t need = (int64_t)state[1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t base = (int64_t)blockIdx.x * SELECT_BLOCK + (int64_t)tid * PER;
    bool cand[PER];
    key_t key[PER];
    int eq = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int64_t i = base + j;
        cand[j] = i < n && ks.get(i, key[j]);
        if (cand[j] && key[j] == tau) ++eq;
    }
    int x = eq;                                  // inclusive scan of eq over the block
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    int64_t rank = (int64_t)blk_excl[blockIdx.x] + (x - eq);
    for (int w = 0; w < wave; ++w) rank += wsum[w];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        if (!cand[j]) continue;
        bool take = key[j] < tau;
        if (key[j] == tau) { take = rank < need; ++rank; }
        if (take) flags[base + j] = code;
    }
}

int scan_excl_i32(const int* in, int* out, int64_t n, hipStream_t s);   // layer.hip

template <typename KS>
static int select_smallest(KS ks, int64_t n, int64_t k, uint8_t* flags, uint8_t code, const Workspace& ws,
                           hipStream_t s) {
    typedef typename KS::key_t key_t;
    if (k <= 0 || n <= 0) return MST_OK;
    uint64_t* state = ws.sel_state;
    k_select_init<<<1, 256, 0, s>>>(state, (uint64_t)k);
    MST_LAUNCH_CHECK();
    const unsigned hist_blocks = (unsigned)std::min<int64_t>(cdiv(n, 256 * 8), 2048);
    const int bits = (int)sizeof(key_t) * 8;
    for (int shift = bits - 8; shift >= 0; shift -= 8) {
        k_select_hist<KS><<<hist_blocks, 256, 0, s>>>(ks, n, state, shift, shift == bits - 8 ? 1 : 0);
        MST_LAUNCH_CHECK();
        k_select_pick<<<1, 256, 0, s>>>(state, shift);
        MST_LAUNCH_CHECK();
    }
    const int64_t nblk = cdiv(n, SELECT_BLOCK);
    int* blk = reinterpret_cast<int*>(ws.blk);
    k_select_ties<KS><<<(unsigned)nblk, 256, 0, s>>>(ks, n, state, blk);
    MST_LAUNCH_CHECK();
    int rc = scan_excl_i32(blk, blk, nblk, s);
    if (rc != MST_OK) return rc;
    k_select_flag<KS><<<(unsigned)nblk, 256, 0, s>>>(ks, n, state, blk, flags, code);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

// kept weights go to the dense scratch, pruned positions leave the mask
__global__ void k_apply_prune(const float* __restrict__ vals, const int* __restrict__ flat,
                              const uint8_t* __restrict__ psel, int64_t nnz, float* __restrict__ Wd,
                              uint8_t* __restrict__ mask) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    const int f = flat[k];
    if (psel[k]) mask[f] = 0;
    else Wd[f] = vals[k];
}

__global__ void k_apply_grow(const uint8_t* __restrict__ sel, int64_t n, uint8_t* __restrict__ mask) {
    const int64_t f = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (f < n && sel[f]) mask[f] = 1;
}

int mask_update_device(mst_layer* L, const float* G, const mst_update_stats& st, uint64_t seed,
                       const Workspace& ws, hipStream_t s) {
    const int64_t N = L->N, nnz = L->nnz;
    int rc;
    if ((rc = fill_u32(ws.sel, 0u, cdiv(N, 4), s)) != MST_OK) return rc;
    if ((rc = fill_u32(ws.psel, 0u, cdiv(nnz > 0 ? nnz : 1, 4), s)) != MST_OK) return rc;
    if ((rc = fill_u32(ws.Wd, 0u, N, s)) != MST_OK) return rc;

    if ((rc = select_smallest(PruneKeys{L->vals}, nnz, st.n_prune, ws.psel, 1, ws, s)) != MST_OK) return rc;
    if ((rc = select_smallest(GradKeys{G, L->mask}, N, st.n_grad, ws.sel, 2, ws, s)) != MST_OK) return rc;
    if ((rc = select_smallest(RandKeys{L->mask, ws.sel, seed}, N, st.n_rand, ws.sel, 3, ws, s)) != MST_OK) return rc;

    if (nnz > 0) {
        k_apply_prune<<<(unsigned)cdiv(nnz, 256), 256, 0, s>>>(L->vals, L->flat, ws.psel, nnz, ws.Wd, L->mask);
        MST_LAUNCH_CHECK();
    }
    if (st.n_grow > 0) {
        k_apply_grow<<<(unsigned)cdiv(N, 256), 256, 0, s>>>(ws.sel, N, L->mask);
        MST_LAUNCH_CHECK();
    }
    L->nnz = st.nnz_after;
    return build_views(L, ws.Wd, ws, s);
}

}  // namespace mst
