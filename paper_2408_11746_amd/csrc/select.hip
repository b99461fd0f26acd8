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

// A key source answers get(i, key): is index i a candidate, and with which key.  get4 does the
// same for the four indices i .. i+3 of an aligned group (i a multiple of 4, all below n) with
// vector loads where the arrays allow it.
struct PruneKeys {
    typedef uint32_t key_t;
    const float* vals;
    __device__ bool get(int64_t k, key_t& key) const { key = abs_bits(vals[k]); return true; }
    __device__ void get4(int64_t k, key_t (&key)[4], bool (&ok)[4]) const {
        const float4 v = *reinterpret_cast<const float4*>(vals + k);
        key[0] = abs_bits(v.x); key[1] = abs_bits(v.y); key[2] = abs_bits(v.z); key[3] = abs_bits(v.w);
        ok[0] = ok[1] = ok[2] = ok[3] = true;
    }
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
    __device__ void get4(int64_t k, key_t (&key)[4], bool (&ok)[4]) const {
#pragma unroll
        for (int u = 0; u < 4; ++u) ok[u] = get(k + u, key[u]);
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
    __device__ void get4(int64_t f, key_t (&key)[4], bool (&ok)[4]) const {
        const uint32_t m = *reinterpret_cast<const uint32_t*>(mask + f);
        const float4 g = *reinterpret_cast<const float4*>(G + f);
        key[0] = 0x7FFFFFFFu - abs_bits(g.x); key[1] = 0x7FFFFFFFu - abs_bits(g.y);
        key[2] = 0x7FFFFFFFu - abs_bits(g.z); key[3] = 0x7FFFFFFFu - abs_bits(g.w);
        ok[0] = (m & 0xFFu) == 0; ok[1] = (m & 0xFF00u) == 0; ok[2] = (m & 0xFF0000u) == 0; ok[3] = (m & 0xFF000000u) == 0;
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
    __device__ void get4(int64_t f, key_t (&key)[4], bool (&ok)[4]) const {
        const uint32_t m = *reinterpret_cast<const uint32_t*>(mask + f) | *reinterpret_cast<const uint32_t*>(sel + f);
        ok[0] = (m & 0xFFu) == 0; ok[1] = (m & 0xFF00u) == 0; ok[2] = (m & 0xFF0000u) == 0; ok[3] = (m & 0xFF000000u) == 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) key[u] = ok[u] ? splitmix64_at(seed, (uint64_t)(f + u)) : 0ull;
    }
};

// keys of the aligned group of four indices starting at i4 (any of them may lie past n)
template <typename KS>
__device__ inline void keys_of_group(const KS& ks, int64_t i4, int64_t n, typename KS::key_t (&key)[4], bool (&ok)[4]) {
    if (i4 + 3 < n) {
        ks.get4(i4, key, ok);
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) ok[u] = i4 + u < n && ks.get(i4 + u, key[u]);
    }
}

// State of one selection (uint64 words): [0] key prefix fixed so far, [1] how many still to
// take inside the prefix, [2] mode (0: keys below [0] are taken and the first [1] keys equal
// to it in index order; 1: every key <= [0] is taken, the search ended early; 2: keys below
// [0] and keys equal to it with index <= [6]), [3] count of the histogram blocks that have
// finished, [4] length of the candidate list of the random selection, [6] index cut of mode 2;
// from word 8 on: the uint32 histogram bins.  All states of an update are set by k_update_init.

constexpr int SEL_NT = 1024;     // threads of a histogram block (16 wavefronts share one LDS histogram)
constexpr int SEL_GCOPIES = 8;   // copies of the global histogram of a digit pass

// One digit of the search by block `blk` of `nblk`: every block adds its LDS histogram of the
// digit (of the keys that match the prefix) to the global one; the block that finishes last
// picks the bin that contains the k-th smallest key, extends the prefix and clears the
// histogram for the next digit.  If that bin holds exactly the number of keys still wanted,
// all of them are taken and the remaining digits are skipped (mode 1).
// The LDS histogram keeps one copy of every bin per lane (h[bin][lane], 64 KB): a
// wavefront's 64 atomic adds always go to 64 different banks, whatever the keys are.  With
// a single copy the hot bins of the leading digits (exponent bits of |w| and |grad|)
// serialise the whole pass.
struct DigitShared {
    uint32_t h[SEL_BINS * 64];
    uint32_t wsum[4];
    int is_last, pick_bin;
    uint32_t pick_before, pick_count;
};

template <typename KS>
__device__ void select_digit_block(KS ks, int64_t n, uint64_t* __restrict__ state, int shift, int width, int first,
                                   int blk, int nblk, DigitShared& sh) {
    typedef typename KS::key_t key_t;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (state[2] != 0) return;                       // search already over (same value for every thread)
    for (int i = tid; i < SEL_BINS * 64; i += SEL_NT) sh.h[i] = 0;
    __syncthreads();
    const key_t prefix = (key_t)state[0];
    const uint32_t mask = (1u << width) - 1u;
    const int64_t stride = (int64_t)nblk * SEL_NT * 4;
    // a thread takes aligned groups of four consecutive indices (vector loads), two groups per round
    for (int64_t i0 = ((int64_t)blk * SEL_NT + tid) * 4; i0 < n; i0 += 2 * stride) {
        key_t key[2][4];
        bool ok[2][4];
        keys_of_group(ks, i0, n, key[0], ok[0]);
        if (i0 + stride < n) keys_of_group(ks, i0 + stride, n, key[1], ok[1]);
        else ok[1][0] = ok[1][1] = ok[1][2] = ok[1][3] = false;
#pragma unroll
        for (int v = 0; v < 2; ++v)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (!ok[v][u]) continue;
                if (!first && (key[v][u] >> (shift + width)) != (prefix >> (shift + width))) continue;
                atomicAdd(&sh.h[(((uint32_t)(key[v][u] >> shift) & mask) << 6) | lane], 1u);
            }
    }
    __syncthreads();
    // the global histogram has SEL_GCOPIES copies (block b adds to copy b mod SEL_GCOPIES): hundreds of
    // blocks adding to the same 256 addresses would queue up at the memory side
    uint32_t* ghist = reinterpret_cast<uint32_t*>(state + 8);
    uint32_t* gmine = ghist + (blk % SEL_GCOPIES) * SEL_BINS;
    if (tid < SEL_BINS) {                            // sum of the bin's 64 copies, each thread starting at another bank
        uint32_t c = 0;
        for (int r = 0; r < 64; ++r) c += sh.h[(tid << 6) | ((r + tid) & 63)];
        // The blocks talk through device-scope atomics only (performed at the level all XCDs
        // share).  The add returns its old value, so it has been performed when the thread
        // reaches the barrier; the ticket of thread 0 comes after the barrier and the last
        // block reads the bins with atomic loads: no cache write-back fence is needed (on
        // this multi-die GPU a device-scope fence per block costs more than the pass).
        uint32_t old = 0;
        if (c) old = atomicAdd(&gmine[tid], c);
        asm volatile("" ::"v"(old));
    }
    __syncthreads();
    if (tid == 0) {
        const unsigned long long ticket = atomicAdd(reinterpret_cast<unsigned long long*>(state + 3), 1ull);
        sh.is_last = ticket == (unsigned long long)nblk - 1ull;
    }
    __syncthreads();
    if (!sh.is_last) return;
    // ---- pick (the first 256 threads, one bin each): the bin with (total before it) < k <= (total including it)
    uint32_t c = 0, x = 0;
    if (tid < SEL_BINS) {
#pragma unroll
        for (int g = 0; g < SEL_GCOPIES; ++g)
            c += __hip_atomic_load(&ghist[g * SEL_BINS + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        x = c;
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(x, d, 64);
            if (lane >= d) x += y;
        }
        if (lane == 63) sh.wsum[wave] = x;
    }
    if (tid == 0) { sh.pick_bin = SEL_BINS - 1; sh.pick_before = 0; sh.pick_count = 0; }
    __syncthreads();
    const uint64_t k = state[1];
    if (tid < SEL_BINS) {
        uint32_t incl = x;
        for (int w = 0; w < wave; ++w) incl += sh.wsum[w];
        if ((uint64_t)(incl - c) < k && (uint64_t)incl >= k) { sh.pick_bin = tid; sh.pick_before = incl - c; sh.pick_count = c; }
#pragma unroll
        for (int g = 0; g < SEL_GCOPIES; ++g) ghist[g * SEL_BINS + tid] = 0;
    }
    __syncthreads();
    if (tid == 0) {
        uint64_t pre = state[0] | ((uint64_t)sh.pick_bin << shift);
        const uint64_t need = k - sh.pick_before;
        if (need == (uint64_t)sh.pick_count) {       // the whole bin is wanted: no ties to break
            pre |= shift ? ((1ull << shift) - 1ull) : 0ull;
            state[2] = 1;
        }
        state[0] = pre;
        state[1] = need;
        state[3] = 0;
    }
}

// Two independent selections (the prune set and the gradient-growth set of one update) share
// their digit passes: blocks [0, nb0) work on the first, the others on the second.
template <typename KS0, typename KS1>
__global__ __launch_bounds__(SEL_NT) void k_select_digit2(KS0 ks0, int64_t n0, uint64_t* __restrict__ st0, int nb0, int shift0,
                                                          int width0, KS1 ks1, int64_t n1, uint64_t* __restrict__ st1, int nb1,
                                                          int shift1, int width1, int first) {
    __shared__ DigitShared sh;
    if ((int)blockIdx.x < nb0) select_digit_block(ks0, n0, st0, shift0, width0, first, (int)blockIdx.x, nb0, sh);
    else select_digit_block(ks1, n1, st1, shift1, width1, first, (int)blockIdx.x - nb0, nb1, sh);
}

// per block of SELECT_BLOCK indices: how many candidates carry exactly the threshold key
template <typename KS>
__device__ void select_ties_block(KS ks, int64_t n, const uint64_t* __restrict__ state, int* __restrict__ blk, int b, int& cnt) {
    typedef typename KS::key_t key_t;
    if (state[2] != 0) return;                       // no ties to break
    if (threadIdx.x == 0) cnt = 0;
    __syncthreads();
    const key_t tau = (key_t)state[0];
    const int64_t base = (int64_t)b * SELECT_BLOCK;
    int mine = 0;
    for (int j = threadIdx.x; j < SELECT_BLOCK; j += blockDim.x) {
        const int64_t i = base + j;
        key_t key;
        if (i < n && ks.get(i, key) && key == tau) ++mine;
    }
    if (mine) atomicAdd(&cnt, mine);
    __syncthreads();
    if (threadIdx.x == 0) blk[b] = cnt;
}

template <typename KS0, typename KS1>
__global__ void k_select_ties2(KS0 ks0, int64_t n0, const uint64_t* __restrict__ st0, int* __restrict__ blk0, int nb0,
                               KS1 ks1, int64_t n1, const uint64_t* __restrict__ st1, int* __restrict__ blk1) {
    __shared__ int cnt;
    if ((int)blockIdx.x < nb0) select_ties_block(ks0, n0, st0, blk0, (int)blockIdx.x, cnt);
    else select_ties_block(ks1, n1, st1, blk1, (int)blockIdx.x - nb0, cnt);
}

// What the flag pass of a selection does with index i beyond flags[i] = code for a selected one.
struct FlagSink {
    uint8_t* flags;
    uint8_t code;
    int full;            // 1: every index below n gets its flag (0 if not selected); 0: only the selected ones are written
    uint8_t* grow_mask;  // not null: a selected position becomes active ...
    float* grow_w;       // ... and its weight in the dense scratch starts at zero
    __device__ void put(int64_t i, bool take) const {
        if (take) {
            flags[i] = code;
            if (grow_mask) { grow_mask[i] = 1; grow_w[i] = 0.f; }
        } else if (full) {
            flags[i] = 0;
        }
    }
};

// flags of block b; 256 threads, 8 consecutive indices each.  Keys equal to the threshold are
// taken in index order: a key's rank is the count of such keys in the blocks before this one
// (summed here from the per-block counts) plus those before it inside the block.
template <typename KS>
__device__ void select_flag_block(KS ks, int64_t n, const uint64_t* __restrict__ state, const int* __restrict__ blk,
                                  const FlagSink& sink, int b, int* wsum, int64_t* before_s) {
    typedef typename KS::key_t key_t;
    constexpr int PER = SELECT_BLOCK / 256;
    const key_t tau = (key_t)state[0];
    const int64_t need = (int64_t)state[1];
    const int mode = (int)state[2];
    const int64_t cut = (int64_t)state[6];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t base = (int64_t)b * SELECT_BLOCK + (int64_t)tid * PER;
    bool cand[PER];
    key_t key[PER];
    int eq = 0;
    static_assert(PER == 8, "two aligned groups of four per thread");
    {
        key_t k4[2][4];
        bool o4[2][4];
        keys_of_group(ks, base, n, k4[0], o4[0]);
        keys_of_group(ks, base + 4, n, k4[1], o4[1]);
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            cand[j] = o4[j >> 2][j & 3];
            key[j] = k4[j >> 2][j & 3];
            if (cand[j] && key[j] == tau) ++eq;
        }
    }
    if (mode != 0) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int64_t i = base + j;
            if (i >= n) continue;
            bool take = cand[j] && key[j] <= tau;
            if (mode == 2 && take && key[j] == tau) take = i <= cut;
            sink.put(i, take);
        }
        return;
    }
    int64_t prev = 0;                            // threshold keys in the blocks before this one
    for (int bb = tid; bb < b; bb += 256) prev += blk[bb];
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
        const int64_t i = base + j;
        if (i >= n) continue;
        bool take = false;
        if (cand[j]) {
            take = key[j] < tau;
            if (key[j] == tau) { take = rank < need; ++rank; }
        }
        sink.put(i, take);
    }
}

template <typename KS0, typename KS1>
__global__ __launch_bounds__(256) void k_select_flag2(KS0 ks0, int64_t n0, const uint64_t* __restrict__ st0,
                                                      const int* __restrict__ blk0, FlagSink sink0, int nb0, KS1 ks1, int64_t n1,
                                                      const uint64_t* __restrict__ st1, const int* __restrict__ blk1,
                                                      FlagSink sink1) {
    __shared__ int wsum[4];
    __shared__ int64_t before_s[4];
    if ((int)blockIdx.x < nb0) select_flag_block(ks0, n0, st0, blk0, sink0, (int)blockIdx.x, wsum, before_s);
    else select_flag_block(ks1, n1, st1, blk1, sink1, (int)blockIdx.x - nb0, wsum, before_s);
}

template <typename KS>
__global__ __launch_bounds__(256) void k_select_flag(KS ks, int64_t n, const uint64_t* __restrict__ state,
                                                     const int* __restrict__ blk, FlagSink sink) {
    __shared__ int wsum[4];
    __shared__ int64_t before_s[4];
    select_flag_block(ks, n, state, blk, sink, (int)blockIdx.x, wsum, before_s);
}

// ---- the random selection.  Its keys are 64-bit hashes of the index: uniform, and distinct for
// distinct indices.  One pass builds the histogram of the top 10 bits (no hot bins, so one
// LDS copy per block) and picks the bin of the k-th key; one pass appends the candidates of
// that bin -- about n / 1024 of them -- to a list; one block finishes the search on the list
// (seven more 8-bit digits, then the index cut among equal keys).  Selected positions are marked
// where they are decided: candidates below the picked bin by the list pass, those inside it by
// the finishing block.  Three launches whatever the keys are.
constexpr int RAND_TOP_BITS = 10, RAND_BINS = 1 << RAND_TOP_BITS, RAND_SHIFT = 64 - RAND_TOP_BITS;

struct RandItem {
    uint64_t key;
    int64_t f;
};

__global__ __launch_bounds__(SEL_NT) void k_rand_hist(RandKeys ks, int64_t n, uint64_t* __restrict__ state) {
    __shared__ uint32_t h[RAND_BINS];
    __shared__ uint32_t part[16];
    __shared__ int is_last;
    const int tid = threadIdx.x;
    for (int i = tid; i < RAND_BINS; i += SEL_NT) h[i] = 0;
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * SEL_NT * 4;
    for (int64_t i0 = ((int64_t)blockIdx.x * SEL_NT + tid) * 4; i0 < n; i0 += stride) {
        uint64_t key[4];
        bool ok[4];
        keys_of_group(ks, i0, n, key, ok);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (ok[u]) atomicAdd(&h[(uint32_t)(key[u] >> RAND_SHIFT)], 1u);
    }
    __syncthreads();
    uint32_t* ghist = reinterpret_cast<uint32_t*>(state + 8);
    for (int i = tid; i < RAND_BINS; i += SEL_NT) {
        const uint32_t c = h[i];
        uint32_t old = 0;
        if (c) old = atomicAdd(&ghist[i], c);
        asm volatile("" ::"v"(old));
    }
    __syncthreads();
    if (tid == 0) {
        const unsigned long long ticket = atomicAdd(reinterpret_cast<unsigned long long*>(state + 3), 1ull);
        is_last = ticket == (unsigned long long)gridDim.x - 1ull;
    }
    __syncthreads();
    if (!is_last) return;
    // pick: thread t owns bin t
    static_assert(RAND_BINS == SEL_NT, "one bin per thread");
    uint32_t c[1], tot = 0;
    c[0] = __hip_atomic_load(&ghist[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    tot = c[0];
    // exclusive scan of the 1024 threads' sums: inside each wavefront, then over the 16 wavefronts
    const int lane = tid & 63, wave = tid >> 6;
    uint32_t x = tot;
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) part[wave] = x;
    __syncthreads();
    uint32_t woff = 0;
    for (int w = 0; w < wave; ++w) woff += part[w];
    const uint64_t k = state[1];
    uint64_t before = (uint64_t)woff + x - tot;
    for (int u = 0; u < 1; ++u) {
        if (before < k && before + c[u] >= k) {       // exactly one thread when 1 <= k <= number of candidates
            const uint64_t need = k - before;
            uint64_t pre = (uint64_t)tid << RAND_SHIFT;
            if (need == (uint64_t)c[u]) {             // the whole bin is wanted
                pre |= (1ull << RAND_SHIFT) - 1ull;
                state[2] = 1;
            }
            state[0] = pre;
            state[1] = need;
        }
        before += c[u];
    }
    if (tid == 0) { state[3] = 0; state[4] = 0; }
}

// block of 1024 threads, 16 indices each.  Candidates in a bin below the picked one are selected on
// the spot; those of the picked bin (about 16 per block) are gathered in LDS and appended to the
// list with ONE add to its length (an add per hit would queue up at the counter)
constexpr int COMPACT_PER_BLOCK = SEL_NT * 16, COMPACT_STAGE = 512;
__global__ __launch_bounds__(SEL_NT) void k_rand_compact(RandKeys ks, int64_t n, uint64_t* __restrict__ state,
                                                         RandItem* __restrict__ list, FlagSink sink) {
    __shared__ RandItem stage[COMPACT_STAGE];
    __shared__ unsigned int nstage;
    __shared__ unsigned long long base_s;
    const bool whole_bin = state[2] != 0;            // every candidate of the picked bin is wanted: no list
    const int tid = threadIdx.x;
    if (tid == 0) nstage = 0;
    __syncthreads();
    const uint64_t top = state[0] >> RAND_SHIFT;
    unsigned long long* len = reinterpret_cast<unsigned long long*>(state + 4);
    const int64_t b0 = (int64_t)blockIdx.x * COMPACT_PER_BLOCK;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t i4 = b0 + ((int64_t)r * SEL_NT + tid) * 4;
        if (i4 >= n) continue;
        uint64_t key[4];
        bool ok[4];
        keys_of_group(ks, i4, n, key, ok);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (!ok[u]) continue;
            const uint64_t bin = key[u] >> RAND_SHIFT;
            if (bin < top || (whole_bin && bin == top)) {     // decided here: selected (each thread owns its indices)
                sink.put(i4 + u, true);
                continue;
            }
            if (bin != top) continue;
            const unsigned int at = atomicAdd(&nstage, 1u);
            if (at < COMPACT_STAGE) stage[at] = RandItem{key[u], i4 + u};
            else list[atomicAdd(len, 1ull)] = RandItem{key[u], i4 + u};      // (a block with more hits than the stage holds)
        }
    }
    __syncthreads();
    const unsigned int m = min(nstage, (unsigned int)COMPACT_STAGE);
    if (tid == 0 && m) base_s = atomicAdd(len, (unsigned long long)m);
    __syncthreads();
    for (unsigned int i = tid; i < m; i += SEL_NT) list[base_s + i] = stage[i];
}

// one block: the state[1]-th smallest (key, index) of the list decides the threshold.  Lists of up to
// RAND_LDS_KEYS items (the usual case by far) are searched in LDS.
constexpr int RAND_LDS_KEYS = 7168;
__global__ __launch_bounds__(SEL_NT) void k_rand_finish(uint64_t* __restrict__ state, const RandItem* __restrict__ list,
                                                        FlagSink sink) {
    __shared__ uint64_t keys[RAND_LDS_KEYS];
    __shared__ uint32_t h[SEL_BINS];
    __shared__ uint32_t wtot[4];
    __shared__ uint64_t prefix_s, need_s;
    __shared__ int done_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (state[2] != 0) return;
    const int64_t c = (int64_t)state[4];
    const bool in_lds = c <= RAND_LDS_KEYS;
    if (in_lds)
        for (int64_t i = tid; i < c; i += SEL_NT) keys[i] = list[i].key;
    if (tid == 0) { prefix_s = state[0]; need_s = state[1]; done_s = 0; }
    __syncthreads();
    // the 54 bits below the top digit: six digits of 8 bits, then one of 6
    for (int top = RAND_SHIFT; top > 0 && !done_s; top -= SEL_DIGIT_BITS) {
        const int shift = max(0, top - SEL_DIGIT_BITS), width = top - shift;
        for (int i = tid; i < SEL_BINS; i += SEL_NT) h[i] = 0;
        __syncthreads();
        const uint64_t prefix = prefix_s;
        for (int64_t i = tid; i < c; i += SEL_NT) {
            const uint64_t key = in_lds ? keys[i] : list[i].key;
            if ((key >> top) == (prefix >> top)) atomicAdd(&h[(uint32_t)(key >> shift) & ((1u << width) - 1u)], 1u);
        }
        __syncthreads();
        // pick by the first 256 threads, one bin each: inclusive scan over the four wavefronts
        uint32_t cb = 0, x = 0;
        if (tid < SEL_BINS) {
            cb = h[tid];
            x = cb;
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t y = __shfl_up(x, d, 64);
                if (lane >= d) x += y;
            }
            if (lane == 63) wtot[wave] = x;
        }
        __syncthreads();
        if (tid < SEL_BINS) {
            uint64_t incl = x;
            for (int w = 0; w < wave; ++w) incl += wtot[w];
            const uint64_t k = need_s, before = incl - cb;
            if (before < k && incl >= k) {                // exactly one bin
                uint64_t pre = prefix | ((uint64_t)tid << shift);
                if (k - before == cb) {                   // the whole bin: every key <= prefix | ones is taken
                    pre |= shift ? ((1ull << shift) - 1ull) : 0ull;
                    done_s = 1;
                }
                prefix_s = pre;
                need_s = k - before;
            }
        }
        __syncthreads();
    }
    if (done_s) {                                     // every listed key <= prefix_s is taken
        const uint64_t top_key = prefix_s;
        for (int64_t i = tid; i < c; i += SEL_NT)
            if (list[i].key <= top_key) sink.put(list[i].f, true);
        if (tid == 0) { state[0] = prefix_s; state[1] = need_s; state[2] = 1; }
        return;
    }
    // equal keys (cannot happen with distinct indices, kept for exactness): the need_s lowest indices.
    // The cut is the need_s-th smallest index among the items whose key is the threshold.
    __shared__ long long cut_s;
    if (tid == 0) {
        const uint64_t tau = prefix_s, need = need_s;
        long long lo = -1;
        for (uint64_t r = 0; r < need; ++r) {          // repeated minimum above lo: need is 1 unless keys collide
            long long best = -1;
            for (int64_t i = 0; i < c; ++i)
                if (list[i].key == tau && list[i].f > lo && (best < 0 || list[i].f < best)) best = list[i].f;
            lo = best;
        }
        state[0] = tau;
        state[1] = need;
        state[2] = 2;
        state[6] = (uint64_t)lo;
        cut_s = lo;
    }
    __syncthreads();
    const uint64_t tau = prefix_s;
    const long long cut = cut_s;
    for (int64_t i = tid; i < c; i += SEL_NT) {
        const RandItem it = list[i];
        if (it.key < tau || (it.key == tau && (long long)it.f <= cut)) sink.put(it.f, true);
    }
}

// start of an update: the three selection states
__global__ void k_update_init(uint64_t* __restrict__ state, uint64_t k0, uint64_t k1, uint64_t k2) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (int64_t)SEL_STATES * SEL_STATE_WORDS) {
        const int w = (int)(i % SEL_STATE_WORDS), which = (int)(i / SEL_STATE_WORDS);
        state[i] = (w == 1) ? (which == 0 ? k0 : which == 1 ? k1 : k2) : 0ull;
    }
}

// kept weights go to the dense scratch, pruned positions leave the mask (psel null: nothing is pruned)
// (zero_pruned: Wd is the layer's dense copy, whose inactive positions must read 0)
__global__ void k_apply_prune(const float* __restrict__ vals, const int* __restrict__ flat,
                              const uint8_t* __restrict__ psel, int64_t nnz, float* __restrict__ Wd,
                              uint8_t* __restrict__ mask, int zero_pruned) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    const int f = flat[k];
    if (psel && psel[k]) {
        mask[f] = 0;
        if (zero_pruned) Wd[f] = 0.f;
    } else {
        Wd[f] = vals[k];
    }
}

static unsigned digit_blocks(int64_t n) { return (unsigned)std::min<int64_t>(cdiv(n, SEL_NT * 4), 256); }
static unsigned rand_blocks(int64_t n) { return (unsigned)std::min<int64_t>(cdiv(n, SEL_NT * 8), 256); }

// prune set (over the nnz active weights) and gradient-growth set (over all N positions) of one
// update, side by side: 4 digit launches, one tie-count launch, one flag launch
template <typename PK>
static int select_prune_and_grad(PK pk, int64_t nnz, int64_t n_prune, GradKeys gk, int64_t N, int64_t n_grad,
                                 uint64_t* st_prune, uint64_t* st_grad, const Workspace& ws, uint8_t* mask, float* Wnew,
                                 hipStream_t s) {
    const bool do_p = n_prune > 0 && nnz > 0, do_g = n_grad > 0;
    if (!do_p && !do_g) return MST_OK;
    const int nb0 = do_p ? (int)digit_blocks(nnz) : 0, nb1 = do_g ? (int)digit_blocks(N) : 0;
    for (int top = 32; top > 0; top -= SEL_DIGIT_BITS) {
        const int shift = top - SEL_DIGIT_BITS;
        k_select_digit2<PK, GradKeys><<<(unsigned)(nb0 + nb1), SEL_NT, 0, s>>>(pk, nnz, st_prune, nb0, shift, SEL_DIGIT_BITS, gk, N,
                                                                             st_grad, nb1, shift, SEL_DIGIT_BITS, top == 32 ? 1 : 0);
        MST_LAUNCH_CHECK();
    }
    const int fb0 = do_p ? (int)cdiv(nnz, SELECT_BLOCK) : 0, fb1 = do_g ? (int)cdiv(N, SELECT_BLOCK) : 0;
    int* blk_g = reinterpret_cast<int*>(ws.blk);
    int* blk_p = reinterpret_cast<int*>(ws.blk) + cdiv(N, SELECT_BLOCK) + 1;
    k_select_ties2<PK, GradKeys><<<(unsigned)(fb0 + fb1), 256, 0, s>>>(pk, nnz, st_prune, blk_p, fb0, gk, N, st_grad, blk_g);
    MST_LAUNCH_CHECK();
    const FlagSink sink_p{ws.psel, 1, 1, nullptr, nullptr};
    const FlagSink sink_g{ws.sel, 2, 1, mask, Wnew};
    k_select_flag2<PK, GradKeys><<<(unsigned)(fb0 + fb1), 256, 0, s>>>(pk, nnz, st_prune, blk_p, sink_p, fb0, gk, N, st_grad, blk_g,
                                                                     sink_g);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int mask_update_device(mst_layer* L, const float* G, const mst_update_stats& st, uint64_t seed,
                       const Workspace& ws, hipStream_t s) {
    const int64_t N = L->N, nnz = L->nnz;
    int rc;
    // Where the new dense weights are formed.  A layer that stays on the dense contractions after
    // this update gets them straight into its dense copy (zero at every inactive position: kept
    // weights are rewritten, pruned and grown positions written 0) and only vals / flat / rowptr
    // are rebuilt; otherwise they go to the workspace and both index views are rebuilt from them.
    const int64_t nnz_before = L->nnz;
    L->nnz = st.nnz_after;
    const bool with_views = views_wanted(L);
    L->nnz = nnz_before;
    float* const Wnew = with_views ? ws.Wd : L->Wd;
    if (!with_views && !L->Wd_zeros && (rc = fill_u32(L->Wd, 0u, N, s)) != MST_OK) return rc;
    uint64_t* st0 = ws.sel_state;
    k_update_init<<<(unsigned)cdiv((int64_t)SEL_STATES * SEL_STATE_WORDS, 256), 256, 0, s>>>(
        st0, (uint64_t)st.n_prune, (uint64_t)st.n_grad, (uint64_t)st.n_rand);
    MST_LAUNCH_CHECK();

    // During the selections the mask still means "active before this update" for every position
    // a later selection looks at: positions grown by gradient become active at once (random
    // growth must skip them anyway), pruned positions leave the mask only at the very end.
    const GradKeys gk{G, L->mask};
    uint64_t* st_grad = st0 + SEL_STATE_WORDS;
    if (L->prune_lambda == 0.f)
        rc = select_prune_and_grad(PruneKeys{L->vals}, nnz, st.n_prune, gk, N, st.n_grad, st0, st_grad, ws, L->mask, Wnew, s);
    else
        rc = select_prune_and_grad(ScoredPruneKeys{L->vals, L->flat, G, L->prune_lambda}, nnz, st.n_prune, gk, N, st.n_grad,
                                   st0, st_grad, ws, L->mask, Wnew, s);
    if (rc != MST_OK) return rc;

    if (st.n_rand > 0) {
        if (st.n_grad <= 0 && (rc = fill_u32(ws.sel, 0u, cdiv(N, 4), s)) != MST_OK) return rc;   // no flag pass wrote sel
        const RandKeys rk{L->mask, ws.sel, seed};
        uint64_t* st_rand = st0 + 2 * SEL_STATE_WORDS;
        RandItem* list = reinterpret_cast<RandItem*>(ws.gemm);          // 2 N items fit: more than any candidate count
        k_rand_hist<<<rand_blocks(N), SEL_NT, 0, s>>>(rk, N, st_rand);
        MST_LAUNCH_CHECK();
        // selected positions become active (weight 0) where they are decided: below the picked bin in the
        // compaction pass, inside it by the finishing block; no separate flag pass
        const FlagSink sink_r{ws.sel, 3, 0, L->mask, Wnew};
        k_rand_compact<<<(unsigned)cdiv(N, COMPACT_PER_BLOCK), SEL_NT, 0, s>>>(rk, N, st_rand, list, sink_r);
        MST_LAUNCH_CHECK();
        k_rand_finish<<<1, SEL_NT, 0, s>>>(st_rand, list, sink_r);
        MST_LAUNCH_CHECK();
    }

    if (nnz > 0) {
        const bool pruned = st.n_prune > 0;
        k_apply_prune<<<(unsigned)cdiv(nnz, 256), 256, 0, s>>>(L->vals, L->flat, pruned ? ws.psel : nullptr, nnz, Wnew, L->mask,
                                                               with_views ? 0 : 1);
        MST_LAUNCH_CHECK();
    }
    L->nnz = st.nnz_after;
    if (with_views) return build_views(L, ws.Wd, ws, s);
    L->Wd_valid = L->Wd_zeros = true;
    return build_canonical(L, L->Wd, ws, s);
}

}  // namespace mst
