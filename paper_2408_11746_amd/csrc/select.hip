// Exact k-selection with index tie-break, and the device side of one Mixed-Growing
// update (Algorithm 1: ArgTopK of -|theta . M|, ArgTopK of |grad| over the inactive
// positions, RandK over the rest, then the mask / weight update).
//
// Each of the three selections is "the k candidates with the smallest (key, index)":
//   prune   candidates = active weights,            key = |w| bits            (32 bit)
//   grad    candidates = inactive positions,        key = 0x7FFFFFFF - |g| bits (32 bit)
//   random  candidates = inactive, not grad-grown,  key = SplitMix64(seed)[f]  (64 bit)
// A most-significant-digit radix select (8-bit digits, one kernel per digit: histogram,
// then the last block to finish picks the bin; the search stops early when a bin holds
// exactly the keys still wanted) finds the k-th smallest key tau on the device; a last ordered pass takes every key
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
// |w| + lambda |grad|, both roundings explicit (no contraction into one fused operation);
// a non-negative float orders like its bit pattern
struct ScoredPruneKeys {
    typedef uint32_t key_t;
    const float* vals;
    const int* flat;
    const float* G;
    float lambda;
    __device__ bool get(int64_t k, key_t& key) const {
        key = __float_as_uint(__fadd_rn(fabsf(vals[k]), __fmul_rn(lambda, fabsf(G[flat[k]]))));
        return true;
    }
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

// State of one selection (uint64 words): [0] key prefix fixed so far, [1] how many still to
// take inside the prefix, [2] mode (0: keys below [0] are taken and the first [1] keys equal
// to it; 1: every key <= [0] is taken, the search ended early), [3] count of the
// histogram blocks that have finished; from word 8 on: SEL_BINS uint32 histogram bins.
// All states of an update are set by k_update_init.

// One digit of the search: every block adds its LDS histogram of the digit (of the keys
// that match the prefix) to the global one; the block that finishes last picks the bin that
// contains the k-th smallest key, extends the prefix and clears the histogram for the next
// digit.  If that bin holds exactly the number of keys still wanted, all of them are taken
// and the remaining digits are skipped (mode 1): with 64-bit random keys this happens after
// three of the six digits.
constexpr int SEL_NT = 1024;     // threads of a histogram block (16 wavefronts share one LDS histogram)

// The LDS histogram keeps one copy of every bin per lane (h[bin][lane], 64 KB): a
// wavefront's 64 atomic adds always go to 64 different banks, whatever the keys are.  With
// a single copy the hot bins of the leading digits (exponent bits of |w| and |grad|)
// serialise the whole pass.
template <typename KS>
__global__ __launch_bounds__(SEL_NT) void k_select_digit(KS ks, int64_t n, uint64_t* __restrict__ state, int shift,
                                                         int width, int first) {
    typedef typename KS::key_t key_t;
    __shared__ uint32_t h[SEL_BINS * 64];
    __shared__ uint32_t wsum[4];
    __shared__ int is_last, pick_bin;
    __shared__ uint32_t pick_before, pick_count;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (state[2] != 0) return;                       // search already over (same value for every thread)
    for (int i = tid; i < SEL_BINS * 64; i += SEL_NT) h[i] = 0;
    __syncthreads();
    const key_t prefix = (key_t)state[0];
    const uint32_t mask = (1u << width) - 1u;
    const int64_t stride = (int64_t)gridDim.x * SEL_NT;
    for (int64_t i = (int64_t)blockIdx.x * SEL_NT + tid; i < n; i += stride) {
        key_t key;
        if (!ks.get(i, key)) continue;
        if (!first && (key >> (shift + width)) != (prefix >> (shift + width))) continue;
        atomicAdd(&h[(((uint32_t)(key >> shift) & mask) << 6) | lane], 1u);
    }
    __syncthreads();
    uint32_t* ghist = reinterpret_cast<uint32_t*>(state + 8);
    if (tid < SEL_BINS) {                            // sum of the bin's 64 copies, each thread starting at another bank
        uint32_t c = 0;
        for (int r = 0; r < 64; ++r) c += h[(tid << 6) | ((r + tid) & 63)];
        // The blocks talk through device-scope atomics only (performed at the level all XCDs
        // share).  The add returns its old value, so it has been performed when the thread
        // reaches the barrier; the ticket of thread 0 comes after the barrier and the last
        // block reads the bins with atomic loads: no cache write-back fence is needed (on
        // this multi-die GPU a device-scope fence per block costs more than the pass).
        uint32_t old = 0;
        if (c) old = atomicAdd(&ghist[tid], c);
        asm volatile("" ::"v"(old));
    }
    __syncthreads();
    if (tid == 0) {
        const unsigned long long ticket = atomicAdd(reinterpret_cast<unsigned long long*>(state + 3), 1ull);
        is_last = ticket == (unsigned long long)gridDim.x - 1ull;
    }
    __syncthreads();
    if (!is_last) return;
    // ---- pick (the first 256 threads, one bin each): the bin with (total before it) < k <= (total including it)
    uint32_t c = 0, x = 0;
    if (tid < SEL_BINS) {
        c = __hip_atomic_load(&ghist[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        x = c;
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(x, d, 64);
            if (lane >= d) x += y;
        }
        if (lane == 63) wsum[wave] = x;
    }
    if (tid == 0) { pick_bin = SEL_BINS - 1; pick_before = 0; pick_count = 0; }
    __syncthreads();
    const uint64_t k = state[1];
    if (tid < SEL_BINS) {
        uint32_t incl = x;
        for (int w = 0; w < wave; ++w) incl += wsum[w];
        if ((uint64_t)(incl - c) < k && (uint64_t)incl >= k) { pick_bin = tid; pick_before = incl - c; pick_count = c; }
        ghist[tid] = 0;
    }
    __syncthreads();
    if (tid == 0) {
        uint64_t pre = state[0] | ((uint64_t)pick_bin << shift);
        const uint64_t need = k - pick_before;
        if (need == (uint64_t)pick_count) {          // the whole bin is wanted: no ties to break
            pre |= shift ? ((1ull << shift) - 1ull) : 0ull;
            state[2] = 1;
        }
        state[0] = pre;
        state[1] = need;
        state[3] = 0;
    }
}

// per block of SELECT_BLOCK indices: how many candidates carry exactly the threshold key
template <typename KS>
__global__ void k_select_ties(KS ks, int64_t n, const uint64_t* __restrict__ state, int* __restrict__ blk) {
    typedef typename KS::key_t key_t;
    __shared__ int cnt;
    if (state[2] != 0) return;                       // no ties to break
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

// flags[i] = code for every selected index; 256 threads, 8 consecutive indices each.  Keys
// equal to the threshold are taken in index order: a key's rank is the count of such keys
// in the blocks before this one (summed here from the per-block counts) plus those before
// it inside the block.
template <typename KS>
__global__ void k_select_flag(KS ks, int64_t n, const uint64_t* __restrict__ state,
                              const int* __restrict__ blk, uint8_t* flags, uint8_t code) {
    typedef typename KS::key_t key_t;
    constexpr int PER = SELECT_BLOCK / 256;
    __shared__ int wsum[4];
    __shared__ int64_t before_s[4];
    const key_t tau = (key_t)state[0];
    const int64_t need = (int64_t)state[1];
    const bool all_le = state[2] != 0;
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
    if (all_le) {
#pragma unroll
        for (int j = 0; j < PER; ++j)
            if (cand[j] && key[j] <= tau) flags[base + j] = code;
        return;
    }
    int64_t prev = 0;                            // threshold keys in the blocks before this one
    for (int bb = tid; bb < (int)blockIdx.x; bb += 256) prev += blk[bb];
    for (int d = 32; d >= 1; d >>= 1) prev += __shfl_xor(prev, d, 64);
    if (lane == 0) before_s[wave] = prev;
    int x = eq;                                  // inclusive scan of eq over the block
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    int64_t rank = before_s[0] + before_s[1] + before_s[2] + before_s[3] + (x - eq);
    for (int w = 0; w < wave; ++w) rank += wsum[w];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        if (!cand[j]) continue;
        bool take = key[j] < tau;
        if (key[j] == tau) { take = rank < need; ++rank; }
        if (take) flags[base + j] = code;
    }
}

template <typename KS>
static int select_smallest(KS ks, int64_t n, int64_t k, uint8_t* flags, uint8_t code, uint64_t* state,
                           const Workspace& ws, hipStream_t s) {
    typedef typename KS::key_t key_t;
    if (k <= 0 || n <= 0) return MST_OK;
    const unsigned hist_blocks = (unsigned)std::min<int64_t>(cdiv(n, SEL_NT * 4), 512);   // two per CU (64 KB of LDS each)
    const int bits = (int)sizeof(key_t) * 8;
    for (int top = bits; top > 0; top -= SEL_DIGIT_BITS) {       // digit = bits [shift, top)
        const int shift = std::max(0, top - SEL_DIGIT_BITS);
        k_select_digit<KS><<<hist_blocks, SEL_NT, 0, s>>>(ks, n, state, shift, top - shift, top == bits ? 1 : 0);
        MST_LAUNCH_CHECK();
    }
    const int64_t nblk = cdiv(n, SELECT_BLOCK);
    int* blk = reinterpret_cast<int*>(ws.blk);
    k_select_ties<KS><<<(unsigned)nblk, 256, 0, s>>>(ks, n, state, blk);
    MST_LAUNCH_CHECK();
    k_select_flag<KS><<<(unsigned)nblk, 256, 0, s>>>(ks, n, state, blk, flags, code);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

// start of an update: flags, dense scratch and the three selection states
__global__ void k_update_init(uint32_t* __restrict__ sel, int64_t sel_words, uint32_t* __restrict__ psel,
                              int64_t psel_words, uint32_t* __restrict__ Wd, int64_t n,
                              uint64_t* __restrict__ state, uint64_t k0, uint64_t k1, uint64_t k2) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) Wd[i] = 0u;
    if (i < sel_words) sel[i] = 0u;
    if (i < psel_words) psel[i] = 0u;
    if (i < (int64_t)SEL_STATES * SEL_STATE_WORDS) {
        const int w = (int)(i % SEL_STATE_WORDS), which = (int)(i / SEL_STATE_WORDS);
        state[i] = (w == 1) ? (which == 0 ? k0 : which == 1 ? k1 : k2) : 0ull;
    }
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
    uint64_t* st0 = ws.sel_state;
    k_update_init<<<(unsigned)cdiv(std::max<int64_t>(N, (int64_t)SEL_STATES * SEL_STATE_WORDS), 256), 256, 0, s>>>(
        reinterpret_cast<uint32_t*>(ws.sel), cdiv(N, 4), reinterpret_cast<uint32_t*>(ws.psel),
        cdiv(nnz > 0 ? nnz : 1, 4), reinterpret_cast<uint32_t*>(ws.Wd), N, st0, (uint64_t)st.n_prune,
        (uint64_t)st.n_grad, (uint64_t)st.n_rand);
    MST_LAUNCH_CHECK();

    if (L->prune_lambda == 0.f)
        rc = select_smallest(PruneKeys{L->vals}, nnz, st.n_prune, ws.psel, 1, st0, ws, s);
    else
        rc = select_smallest(ScoredPruneKeys{L->vals, L->flat, G, L->prune_lambda}, nnz, st.n_prune, ws.psel, 1, st0, ws, s);
    if (rc != MST_OK) return rc;
    if ((rc = select_smallest(GradKeys{G, L->mask}, N, st.n_grad, ws.sel, 2, st0 + SEL_STATE_WORDS, ws, s)) != MST_OK)
        return rc;
    if ((rc = select_smallest(RandKeys{L->mask, ws.sel, seed}, N, st.n_rand, ws.sel, 3, st0 + 2 * SEL_STATE_WORDS, ws,
                              s)) != MST_OK)
        return rc;

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
