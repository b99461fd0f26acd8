// Layer object, storage format and its construction on the device.
//
// Storage (not prescribed by the paper, which only names the binary mask M of
// Sec. 3.2): the active weights are kept once in canonical order (ascending flat
// index o*I + i) as vals[] / flat[], plus two "views" that the product kernels walk:
//   row view  S = W    [O x I]  -> forward
//   col view  S = W^T  [I x O]  -> input gradient
// (the weight gradient walks whichever of the two is cheaper, see build_views).
// A view cuts the contraction index into chunks of KC and stores, per (chunk, block of
// 16 rows, quad), an ELL slice of four rows (see View in common.h).  perm[] maps an
// entry slot back to its canonical position, so that values can be refreshed after an
// optimiser step and weight gradients can be returned in canonical order.
#include "common.h"

namespace mst {

thread_local int g_last_hip_error = 0;

static int64_t nchunks(int K) { return cdiv(K, KC); }
static int64_t nblocks(int R) { return cdiv(R, RB); }
static int64_t nbpad(int R) { return nblocks(R) + MAX_WG_BLOCKS; }

// A quad segment holds max(len of its four rows) steps rounded up to even, which is at
// most (sum of the four lens) + 1; summed over all segments: steps <= nnz + #segments.
int64_t view_pair_capacity(int64_t cap, int64_t nchunk, int64_t R) {
    const int64_t nqs = nchunk * nblocks((int)R) * 4;
    return cdiv((cap + nqs) / 2 + 1 + PAIR_TAIL, 8) * 8;
}

// Measured cross-overs (GPT-2 small / medium / large layer shapes).  With fp32 activations the
// dense products run on the bf16 matrix cores (operands split hi + lo) at 250-360 TFLOP/s and
// cost the same at every density; the sparse kernels cost about in proportion to nnz.  At
// T >= 2048 the two meet at a density of 0.045-0.06 for Y and dX and at 0.03-0.04 for the
// weight gradient; short batches fill the matrix cores badly and meet at about 0.15 (there the
// one-call backward, both gradients from one walk, is also ahead of two separate products).
// With bfloat16 activations on whole 256 x 256 tiles Y and dX take two bf16 products per term
// (490 TFLOP/s at the GPT-2-medium shapes) and meet the sparse kernels at 0.042-0.05; other
// shapes run on the fp32 MFMA kernel (cross-over 0.30).  The bfloat16 weight gradient has both
// operands in bfloat16 (cross-over 0.045).
bool use_dense_path(const mst_layer* L, mst_dtype act, int T) {
    if (L->path == MST_PATH_DENSE) return true;
    if (L->path == MST_PATH_SPARSE) return false;
    double thr;
    if (act == MST_BF16) {
        const bool tiles = T % 256 == 0 && L->O % 256 == 0 && L->I % 256 == 0;
        thr = tiles && T >= 2048 ? 0.045 : 0.30;
    } else {
        // the split kernels need whole 128-tiles (and a depth that is a multiple of 64); other shapes
        // run on the fp32 MFMA kernel, a third as fast
        const bool tiles = T % 128 == 0 && L->O % 128 == 0 && L->I % 128 == 0;
        thr = !tiles ? 0.30 : T >= 2048 ? 0.055 : 0.15;
    }
    return (double)L->nnz > thr * (double)L->N;
}

// The one-call backward has a third choice, the shared walk, and it moves the cross-over: against the
// two dense contractions it wins up to densities of 0.065-0.11 with fp32 activations (GPT-2 small /
// large layer shapes, T >= 8192; a sparse dX beside a dense dW is never the fastest), and only up to
// 0.03 with bfloat16 activations, whose dense weight gradient is a single bf16 product.  Elsewhere the
// thresholds of the separate calls coincide and apply.
bool use_fused_backward(const mst_layer* L, mst_dtype act, int T) {
    if (L->path == MST_PATH_DENSE) return false;
    if (L->path == MST_PATH_SPARSE) return true;
    double thr;
    if (act == MST_BF16) {
        const bool tiles = T % 256 == 0 && L->O % 256 == 0 && L->I % 256 == 0;
        thr = tiles && T >= 2048 ? 0.03 : 0.30;
    } else {
        const bool tiles = T % 128 == 0 && L->O % 128 == 0 && L->I % 128 == 0;
        thr = !tiles ? 0.30 : T >= 2048 ? 0.07 : 0.15;
    }
    return (double)L->nnz <= thr * (double)L->N;
}

bool use_dense_weight_grad(const mst_layer* L, mst_dtype act, int T) {
    if (L->path == MST_PATH_DENSE) return true;
    if (L->path == MST_PATH_SPARSE) return false;
    const bool tiles = act == MST_BF16 || (T % 64 == 0 && L->O % 128 == 0 && L->I % 128 == 0);   // (the bf16 kernels take any shape)
    const double thr = act == MST_BF16 ? (T >= 2048 ? 0.045 : 0.30) : !tiles ? 0.30 : T >= 2048 ? 0.035 : 0.15;
    return (double)L->nnz > thr * (double)L->N;
}

struct LayerCarve {
    size_t mask, vals, flat, rowptr, Wd;
    size_t rptr, rent, rperm, rmap, rpos, cptr, cent, cperm, cmap, cpos, choice, heavy, Hd;
    size_t total;
};

static LayerCarve carve_layer(int O, int I, int64_t cap) {
    LayerCarve c{};
    const int64_t N = (int64_t)O * I;
    const int64_t nseg_r = nchunks(I) * nbpad(O) * 4, nseg_c = nchunks(O) * nbpad(I) * 4;
    const int64_t cp_r = view_pair_capacity(cap, nchunks(I), O), cp_c = view_pair_capacity(cap, nchunks(O), I);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    c.mask = take((size_t)N);
    c.vals = take((size_t)cap * 4);
    c.flat = take((size_t)cap * 4);
    c.rowptr = take((size_t)(O + 1) * 4);
    c.Wd = take((size_t)N * 4);
    c.rptr = take((size_t)(nseg_r + 1) * 4);
    c.rent = take((size_t)cp_r * 64);
    c.rperm = take((size_t)cp_r * 32);
    c.rmap = take((size_t)nbpad(O) * RB * 4);
    c.rpos = take((size_t)nbpad(O) * RB * 4);
    c.cptr = take((size_t)(nseg_c + 1) * 4);
    c.cent = take((size_t)cp_c * 64);
    c.cperm = take((size_t)cp_c * 32);
    c.cmap = take((size_t)nbpad(I) * RB * 4);
    c.cpos = take((size_t)nbpad(I) * RB * 4);
    c.choice = take(16);
    c.heavy = take((size_t)(HEAVY_MAX + 2) * 4);
    c.Hd = take((size_t)HEAVY_MAX * I * 4);
    c.total = off;
    return c;
}

static bool shape_ok(int O, int I, int64_t cap) {
    if (O < 1 || I < 1 || O > 65535 || I > 65535) return false;
    const int64_t N = (int64_t)O * I;
    if (N >= (int64_t)1 << 31) return false;
    if (cap < 0 || cap > N) return false;
    return true;
}

Workspace carve_workspace(void* base, int O, int I, int64_t cap, int T) {
    Workspace w{};
    const int64_t N = (int64_t)O * I;
    // per-row-per-chunk counts of either view, rows padded to whole blocks
    const int64_t cnt_r = nchunks(I) * nbpad(O) * RB, cnt_c = nchunks(O) * nbpad(I) * RB;
    const int64_t nseg_r = nchunks(I) * nbpad(O) * 4, nseg_c = nchunks(O) * nbpad(I) * 4;
    const int64_t ntile = cdiv(T > 0 ? T : 1, TT);
    char* b = static_cast<char*>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return b ? b + o : nullptr; };
    w.G = (float*)take((size_t)N * 4);
    w.Wd = (float*)take((size_t)N * 4);
    w.cidx = (int*)take((size_t)N * 4);
    w.sel = (uint8_t*)take((size_t)N);
    w.psel = (uint8_t*)take((size_t)(cap > 0 ? cap : 1));
    w.segcnt = (int*)take((size_t)(std::max(cnt_r, cnt_c) + 1) * 4);
    w.qlen = (int*)take((size_t)(std::max(nseg_r, nseg_c) + 1) * 4);
    w.rowcnt = (int*)take((size_t)(O + 1) * 4);
    w.blk = (uint32_t*)take((size_t)(cdiv(N, SELECT_BLOCK) + cdiv(cap > 0 ? cap : 1, SELECT_BLOCK) + 4) * 4);
    w.sel_state = (uint64_t*)take((size_t)SEL_STATES * SEL_STATE_WORDS * 8);
    w.gemm_floats = (size_t)GEMM_WS_SPLITS * (size_t)N;
    w.gemm = (float*)take(w.gemm_floats * 4);
    w.partial_floats = (size_t)ntile * 8 *
                       (size_t)std::max(view_pair_capacity(cap, nchunks(I), O), view_pair_capacity(cap, nchunks(O), I));
    w.partial = (float*)take(w.partial_floats * 4);
    w.total = off;
    return w;
}

// ------------------------------------------------------------------ kernels

// one block per row r of the mask: active count per chunk of columns and per row; blocks past
// the last row (the padding rows of the view) write zero counts
__global__ void k_count_row(const uint8_t* __restrict__ mask, int O, int I, int nchunk, int Rpad,
                            int* __restrict__ segcnt, int* __restrict__ rowcnt) {
    extern __shared__ int cnt[];   // [nchunk]
    const int r = blockIdx.x;
    if (r >= O) {
        for (int c = threadIdx.x; c < nchunk; c += blockDim.x) segcnt[(size_t)c * Rpad + r] = 0;
        return;
    }
    for (int c = threadIdx.x; c < nchunk; c += blockDim.x) cnt[c] = 0;
    __syncthreads();
    const uint8_t* m = mask + (size_t)r * I;
    int total = 0;
    for (int i = threadIdx.x; i < I; i += blockDim.x) {
        if (m[i]) { atomicAdd(&cnt[i / KC], 1); }
    }
    __syncthreads();
    if (segcnt)
        for (int c = threadIdx.x; c < nchunk; c += blockDim.x) segcnt[(size_t)c * Rpad + r] = cnt[c];
    if (threadIdx.x == 0) {
        for (int c = 0; c < nchunk; ++c) total += cnt[c];
        rowcnt[r] = total;
    }
}

// [KC rows x 64 columns] of the mask into LDS (rows beyond O and columns beyond I read as
// zero); 256 threads, 32 bytes each.  Row stride 68 bytes: the 64 lanes of a wavefront read
// one row's 64 bytes without bank conflicts.
constexpr int MT_COLS = 64, MT_LD = 68;
__device__ inline void load_mask_tile(const uint8_t* __restrict__ mask, int O, int I, int o0, int i0,
                                      uint8_t* __restrict__ m, int tid) {
    const int r = tid >> 1, half = tid & 1;
    const int o = o0 + r, ib = i0 + 32 * half;
    uint8_t* dst = m + r * MT_LD + 32 * half;
    const uint8_t* src = mask + (size_t)o * I + ib;
    if (o < O && ib + 32 <= I && ((reinterpret_cast<uintptr_t>(src) & 3) == 0)) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
            reinterpret_cast<uint32_t*>(dst)[u] = reinterpret_cast<const uint32_t*>(src)[u];
    } else {
        for (int u = 0; u < 32; ++u) dst[u] = (o < O && ib + u < I) ? src[u] : (uint8_t)0;
    }
}

// block = (64 columns, chunk c of KC rows): active count of every column inside the chunk.
// Thread (column j, row group rg of 32 rows) counts its rows from the LDS tile.
__global__ __launch_bounds__(256) void k_count_col(const uint8_t* __restrict__ mask, int O, int I, int Rpad,
                                                   int* __restrict__ segcnt) {
    __shared__ __attribute__((aligned(16))) uint8_t m[KC * MT_LD];
    __shared__ int part[4][MT_COLS];
    const int tid = threadIdx.x, j = tid & 63, rg = tid >> 6;
    const int i0 = blockIdx.x * MT_COLS, c = blockIdx.y;
    load_mask_tile(mask, O, I, c * KC, i0, m, tid);
    __syncthreads();
    int n = 0;
#pragma unroll
    for (int k = 0; k < 32; ++k) n += m[(32 * rg + k) * MT_LD + j] != 0;
    part[rg][j] = n;
    __syncthreads();
    // (columns past the matrix read as empty: the padding rows of the view get zero counts)
    if (rg == 0 && i0 + j < Rpad) segcnt[(size_t)c * Rpad + i0 + j] = part[0][j] + part[1][j] + part[2][j] + part[3][j];
}

// 16 lanes per row block (lane j = row j): order its 16 rows by total length over all
// chunks, longest first, lower row first on ties (the empty padding blocks keep the
// identity).  With h rows spread over whole quads (h <= #empty rows / 3) the quads cost about
//   sum_{j<h} ceil(len_j / 4)  +  sum over the quads of the other rows of their longest row,
// h is the value that minimises it (0 for every mask without empty rows).
__global__ __launch_bounds__(256) void k_block_rank(const int* __restrict__ segcnt, int nchunk, int Rpad, int NBpad,
                                                    int* __restrict__ rowmap, int* __restrict__ rowpos) {
    __shared__ int sorted_s[16][RB];
    __shared__ int h_s[16];
    const int tid = threadIdx.x, j = tid & 15, lb = tid >> 4;
    const int b = blockIdx.x * 16 + lb;
    const bool live = b < NBpad;
    int len = 0;
    if (live)
        for (int c = 0; c < nchunk; ++c) len += segcnt[(size_t)c * Rpad + b * RB + j];
    int rank = 0;
#pragma unroll
    for (int u = 0; u < RB; ++u) {
        const int lu = __shfl(len, u, 16);
        rank += (lu > len) || (lu == len && u < j);
    }
    sorted_s[lb][rank] = len;
    __syncthreads();
    if (j == 0) {
        const int* sorted = sorted_s[lb];
        int nzero = 0;
        for (int u = 0; u < RB; ++u) nzero += sorted[u] == 0;
        int h = 0, best = sorted[0] + sorted[4] + sorted[8] + sorted[12];
        for (int hh = 1; hh <= 4 && 3 * hh <= nzero; ++hh) {
            int cost = 0;
            for (int u = 0; u < hh; ++u) cost += (sorted[u] + 3) >> 2;
            for (int p = hh; p < RB - 3 * hh; p += 4) cost += sorted[p];
            if (cost < best) { best = cost; h = hh; }
        }
        h_s[lb] = h;
    }
    __syncthreads();
    if (!live) return;
    const int h = h_s[lb], p = rank;
    int slot, flag_row = 0;
    if (p < h) { slot = 4 * p; flag_row = SPREAD_FLAG; }                 // spread row: lane group 0 of quad p
    else if (p < RB - 3 * h) slot = 4 * h + (p - h);                     // ordinary rows fill the other quads
    else { const int e = p - (RB - 3 * h); slot = 4 * (e / 3) + 1 + e % 3; }   // empty rows own the rest
    const int flag_quad = (slot >> 2) < h ? SPREAD_FLAG : 0;
    rowmap[b * RB + slot] = (b * RB + j) | flag_quad;
    rowpos[b * RB + j] = slot | flag_row;
}

// pairs of one quad segment: longest of its four rows (a spread row: a quarter of it),
// rounded up to even, halved
__device__ inline int quad_pairs(const int* __restrict__ segcnt, const int* __restrict__ rowmap, int Rpad, int NBpad,
                                 int64_t sidx) {
    const int q = (int)(sidx & 3);
    const int64_t cb = sidx >> 2;
    const int b = (int)(cb % NBpad);
    const int64_t c = cb / NBpad;
    const int* cnt = segcnt + c * Rpad;
    const int* rm = rowmap + b * RB + 4 * q;          // the quad's four rows (one per lane group)
    int L;
    if (rm[0] & SPREAD_FLAG) L = (cnt[rm[0] & ~SPREAD_FLAG] + 3) >> 2;
    else L = max(max(cnt[rm[0]], cnt[rm[1]]), max(cnt[rm[2]], cnt[rm[3]]));
    return (L + 1) >> 1;
}

__global__ void k_quad_len(const int* __restrict__ segcnt, const int* __restrict__ rowmap, int Rpad, int NBpad,
                           int64_t nseg, int* __restrict__ qlen) {
    const int64_t sidx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (c*NBpad + b)*4 + q
    if (sidx < nseg) qlen[sidx] = quad_pairs(segcnt, rowmap, Rpad, NBpad, sidx);
}

// exclusive scan by ONE block of 1024 threads: out[j] = sum_{j' < j} in[j'], out[n] = total (in == out
// is allowed).  Each of the 16 wavefronts owns one contiguous segment and reads it with its 64
// lanes side by side (coalesced, several rows of 64 in flight): first the segment's sum, then,
// with the sums of the segments before it as carry, the running values (a 64-lane scan per row).
__device__ inline void block_scan_excl(const int* in, int* out, int64_t n, int* wsum) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwave = blockDim.x >> 6;
    const int64_t rows = (n + 63) / 64;                            // rows of 64 elements
    const int64_t rpw = (rows + nwave - 1) / nwave;                // rows per wavefront
    const int64_t r0 = (int64_t)wave * rpw, r1 = min(rows, r0 + rpw);
    int tot = 0;
#pragma unroll 4
    for (int64_t r = r0; r < r1; ++r) {
        const int64_t j = r * 64 + lane;
        tot += (j < n) ? in[j] : 0;
    }
    for (int d = 32; d >= 1; d >>= 1) tot += __shfl_xor(tot, d, 64);
    __syncthreads();                                 // wsum free again (an earlier scan of this block may still read it)
    if (lane == 0) wsum[wave] = tot;
    __syncthreads();
    int carry = 0;
    for (int w = 0; w < wave; ++w) carry += wsum[w];
    int v_next = (r0 < r1 && r0 * 64 + lane < n) ? in[r0 * 64 + lane] : 0;
    for (int64_t r = r0; r < r1; ++r) {
        const int64_t j = r * 64 + lane;
        const int v = v_next;
        if (r + 1 < r1) v_next = ((r + 1) * 64 + lane < n) ? in[(r + 1) * 64 + lane] : 0;   // read before the row is written: in may be out
        int x = v;
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(x, d, 64);
            if (lane >= d) x += y;
        }
        if (j < n) out[j] = carry + x - v;
        carry += __shfl(x, 63, 64);
    }
    if (wave == nwave - 1 && lane == 0) out[n] = carry;            // the last segment ends at n (or is empty): the total
}

__global__ __launch_bounds__(1024) void k_scan_excl(const int* in, int* out, int64_t n) {
    __shared__ int wsum[16];
    block_scan_excl(in, out, n, wsum);
}

// One block does what follows the segment lengths of a view: (row view only) the canonical row
// pointers from the per-row counts; the first pair of every quad segment; the view's cost
// for the weight gradient -- a workgroup of the SDDMM owns about 16 consecutive row blocks and
// waits at every chunk for its longest wavefront, so a view costs the sum over (chunk, group
// of 16 blocks) of the most pairs of a block -- and, when the other view's cost is known
// (`choice` not null), the view that drives the weight gradient: the one with the clearly
// smaller cost, else the one with more rows.
__global__ __launch_bounds__(1024) void k_view_ptr(const int* __restrict__ rowcnt, int* __restrict__ rowptr, int nrows,
                                                   const int* __restrict__ qlen, int NBpad, int NB, int nchunk,
                                                   int64_t nseg, int* __restrict__ ptr,
                                                   unsigned long long* __restrict__ cost_mine,
                                                   const unsigned long long* __restrict__ cost_row, int prefer_col,
                                                   int* __restrict__ choice, const int* __restrict__ heavy) {
    __shared__ int wsum[16];
    __shared__ unsigned long long cost_s;
    if (rowcnt) block_scan_excl(rowcnt, rowptr, nrows, wsum);
    block_scan_excl(qlen, ptr, nseg, wsum);
    // cost: per (chunk, group of 16 blocks) the most pairs of a block, summed.  Every thread takes
    // (chunk, block) items side by side and folds them into an LDS table of the groups.
    constexpr int MAXG = 4096;
    __shared__ int worst_s[MAXG];
    const int ngroup = (NB + 15) / 16;
    const int ngrp_all = nchunk * ngroup;
    if (threadIdx.x == 0) cost_s = 0ull;
    for (int i = threadIdx.x; i < min(ngrp_all, MAXG); i += blockDim.x) worst_s[i] = 0;
    __syncthreads();                                  // ptr[] written by this block is visible to it
    unsigned long long mine = 0ull;
    if (ngrp_all <= MAXG) {
        for (int idx = threadIdx.x; idx < nchunk * NB; idx += blockDim.x) {
            const int c = idx / NB, b = idx % NB;
            const int64_t sidx = ((int64_t)c * NBpad + b) * 4;
            atomicMax(&worst_s[c * ngroup + (b >> 4)], ptr[sidx + 4] - ptr[sidx]);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < ngrp_all; i += blockDim.x) mine += (unsigned long long)worst_s[i];
    } else {
        for (int idx = threadIdx.x; idx < ngrp_all; idx += blockDim.x) {
            const int c = idx / ngroup, grp = idx % ngroup;
            int worst = 0;
            for (int b = grp * 16; b < min(NB, grp * 16 + 16); ++b) {
                const int64_t sidx = ((int64_t)c * NBpad + b) * 4;
                worst = max(worst, ptr[sidx + 4] - ptr[sidx]);
            }
            mine += (unsigned long long)worst;
        }
    }
    if (mine) atomicAdd(&cost_s, mine);
    __syncthreads();
    if (threadIdx.x == 0) {
        // a row view that leaves heavy rows out cannot drive the weight gradient
        *cost_mine = (heavy && heavy[0] > 0) ? (1ull << 50) : cost_s;
        if (choice) {
            const unsigned long long pr = *cost_row, pc = cost_s;
            int ch = prefer_col;
            if (prefer_col && pr * 10 < pc * 9) ch = 0;
            if (!prefer_col && pc * 10 < pr * 9) ch = 1;
            *choice = ch;
        }
    }
}

// entry slot (as index into ent viewed as uint2[], and into perm) of step j of a row
__device__ inline int64_t entry_slot(int pair0, int g, int j) {
    return (((int64_t)pair0 + (j >> 1)) * 4 + g) * 2 + (j & 1);
}

// Slots of a row's lane group (of the whole quad for a spread row) past its `run` entries, up
// to the quad's length: zero-weight padding (offset 0, perm -1).  The three empty rows that
// share a spread quad own no slots.  `lanes` threads of the caller share the work.
__device__ inline void pad_row_slots(uint2* __restrict__ ent, int* __restrict__ perm, int pair0, int npairs, int g,
                                     bool spread, int run, int lane, int lanes) {
    const int total = spread ? 8 * npairs : 2 * npairs;
    for (int j = run + lane; j < total; j += lanes) {
        const int64_t e = spread ? entry_slot(pair0, j & 3, j >> 2) : entry_slot(pair0, g, j);
        ent[e] = make_uint2(0u, 0u);
        perm[e] = -1;
    }
}

// one wavefront per (row, part of its chunks) (incl. the padding rows of the last block, which
// only pad): ordered compaction of the row into canonical arrays and the row view.  A layer of
// few long rows gives every row `nparts` wavefronts of `cpp` chunks each (one per row would leave
// the 1280 rows of a 5120-wide layer on 320 workgroups); a part finds its first canonical index
// from the per-chunk counts of the chunks before it (a heavy row, whose counts were cleared, from
// the mask itself).
__global__ void k_fill_row(const uint8_t* __restrict__ mask, const float* __restrict__ W,
                           int O, int I, int nchunk, int NBpad, int NB,
                           const int* __restrict__ rowptr, const int* __restrict__ ptr,
                           const int* __restrict__ rowpos, const int* __restrict__ rowmap,
                           float* __restrict__ vals, int* __restrict__ flat, int* __restrict__ cidx,
                           uint2* __restrict__ ent, int* __restrict__ perm, const int* __restrict__ heavy,
                           int nparts, int cpp, const int* __restrict__ segcnt, int Rpad) {
    const int lane = threadIdx.x & 63;
    const int unit = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int r = unit / nparts, c0 = (unit % nparts) * cpp, c1 = min(nchunk, c0 + cpp);
    if (r >= NB * RB) return;
    // a heavy row (HEAVY_MAX = 64 list entries, one per lane) fills the canonical arrays only
    const bool hv = heavy != nullptr && __ballot(lane < heavy[0] && heavy[1 + lane] == r) != 0ull;
    const int b = r / RB, rp = rowpos[r], rank = rp & ~SPREAD_FLAG, g = rank & 3, q = rank >> 2;
    const bool spread = (rp & SPREAD_FLAG) != 0;
    // an empty row placed in a spread quad: the quad's slots belong to the spread row
    const bool guest = !spread && (rowmap[b * RB + 4 * q] & SPREAD_FLAG) != 0;
    const bool real = r < O;
    const uint8_t* m = mask + (size_t)r * I;
    const float* w = W + (size_t)r * I;
    int canon = real ? rowptr[r] : 0;
    if (real && c0 > 0) {                             // entries of this row in the chunks before c0
        int before = 0;
        if (hv) {                                     // (a heavy row's per-chunk counts were cleared: count the mask)
            for (int i = lane; i < c0 * KC; i += 64) before += m[i] != 0;
        } else {
            for (int c = lane; c < c0; c += 64) before += segcnt[(size_t)c * Rpad + r];
        }
        for (int d = 32; d >= 1; d >>= 1) before += __shfl_xor(before, d, 64);
        canon += before;
    }
    for (int c = c0; c < c1; ++c) {
        const size_t seg = ((size_t)c * NBpad + b) * 4 + q;
        const int pair0 = ptr[seg], npairs = ptr[seg + 1] - pair0;
        int run = 0;
        const int i1 = real ? min(I, (c + 1) * KC) : 0;
        for (int i0 = c * KC; i0 < i1; i0 += 64) {
            const int i = i0 + lane;
            const bool on = i < i1 && m[i] != 0;
            const unsigned long long bal = __ballot(on);
            if (on) {
                const int j = run + __popcll(bal & ((1ull << lane) - 1ull));
                const int k = canon + j;
                const float v = w[i];
                vals[k] = v;
                flat[k] = r * I + i;
                cidx[(size_t)r * I + i] = k;
                if (!hv) {
                    const int64_t e = spread ? entry_slot(pair0, j & 3, j >> 2) : entry_slot(pair0, g, j);
                    ent[e] = make_uint2(lds_off((uint32_t)(i - c * KC)), __float_as_uint(v));
                    perm[e] = k;
                }
            }
            run += __popcll(bal);
        }
        canon += run;
        if (!guest) pad_row_slots(ent, perm, pair0, npairs, g, spread, hv ? 0 : run, lane, 64);
    }
}

// ---- vals / flat / rowptr alone.  Canonical order is ascending flat index, so the arrays are
// the ordered compaction of the mask as ONE sequence of N positions: a wavefront owns a segment of
// CSEG consecutive positions whatever the layer's shape is (one wavefront per row leaves a
// layer of few long rows with a handful of workgroups).
constexpr int CSEG = 2048;

__device__ inline int nonzero_bytes(uint32_t x) {
    const uint32_t t = (((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x) & 0x80808080u;
    return __popc(t);
}

// active positions of every segment
__global__ __launch_bounds__(256) void k_count_seg(const uint8_t* __restrict__ mask, int64_t N, int nseg,
                                                   int* __restrict__ segcnt) {
    const int lane = threadIdx.x & 63;
    const int sg = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (sg >= nseg) return;
    const int64_t base = (int64_t)sg * CSEG;
    int c = 0;
#pragma unroll
    for (int j = 0; j < CSEG; j += 1024) {           // 16 bytes per lane and round
        const int64_t p = base + j + 16 * lane;
        if (p + 16 <= N) {
            const uint4 m = *reinterpret_cast<const uint4*>(mask + p);
            c += nonzero_bytes(m.x) + nonzero_bytes(m.y) + nonzero_bytes(m.z) + nonzero_bytes(m.w);
        } else {
            for (int u = 0; u < 16; ++u) c += (p + u < N && mask[p + u] != 0) ? 1 : 0;
        }
    }
    for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d, 64);
    if (lane == 0) segcnt[sg] = c;
}

// segptr[sg] = active positions before segment sg.  A lane takes four consecutive positions of a
// window of 256; the row pointers are written by the wavefront whose segment holds the row's
// first position (rowptr[O] by the last one).
__global__ __launch_bounds__(256) void k_fill_canonical(const uint8_t* __restrict__ mask, const float* __restrict__ W, int O, int I,
                                                        int64_t N, int nseg, const int* __restrict__ segptr,
                                                        int* __restrict__ rowptr, float* __restrict__ vals,
                                                        int* __restrict__ flat) {
    const int lane = threadIdx.x & 63;
    const int sg = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (sg >= nseg) return;
    const int64_t base = (int64_t)sg * CSEG, end = min(N, base + (int64_t)CSEG);
    const unsigned long long below = (1ull << lane) - 1ull;
    int canon = segptr[sg];
    int64_t row = (base + I - 1) / I;                 // first row that starts at or after base
    for (int64_t w0 = base; w0 < end; w0 += 256) {
        const int64_t p = w0 + 4 * lane;
        bool on[4] = {false, false, false, false};
        float w[4] = {0.f, 0.f, 0.f, 0.f};
        if (p + 4 <= end) {
            const uint32_t m4 = *reinterpret_cast<const uint32_t*>(mask + p);
            if (m4) {
                const float4 w4 = *reinterpret_cast<const float4*>(W + p);
                w[0] = w4.x; w[1] = w4.y; w[2] = w4.z; w[3] = w4.w;
            }
            on[0] = (m4 & 0xFFu) != 0; on[1] = (m4 & 0xFF00u) != 0; on[2] = (m4 & 0xFF0000u) != 0; on[3] = (m4 & 0xFF000000u) != 0;
        } else {
            for (int u = 0; u < 4; ++u)
                if (p + u < end && mask[p + u] != 0) { on[u] = true; w[u] = W[p + u]; }
        }
        unsigned long long bal[4];
        int before = 0, total = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            bal[u] = __ballot(on[u]);
            before += __popcll(bal[u] & below);
            total += __popcll(bal[u]);
        }
        int k = canon + before;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (on[u]) { vals[k] = w[u]; flat[k] = (int)(p + u); ++k; }
        const int64_t wend = min(end, w0 + 256);
        for (int64_t q = row * I; q < wend; q += I, ++row) {   // rows that start inside the window
            const int l = (int)(q - w0) >> 2, u0 = (int)(q - w0) & 3;
            const unsigned long long lt = (1ull << l) - 1ull;
            int cnt = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) cnt += __popcll(bal[u] & lt) + ((u < u0) ? (int)((bal[u] >> l) & 1ull) : 0);
            if (lane == 0) rowptr[row] = canon + cnt;
        }
        canon += total;
    }
    if (sg == nseg - 1 && lane == 0) rowptr[O] = canon;
}

// block = (64 columns, chunk c of KC rows): rows i0 .. i0+63 of the col view, chunk c.  The
// mask tile sits in LDS; thread (column j, row group rg of 32 rows) counts its rows, the
// counts of the row groups before it give the position of its first entry in the column's
// list, then it writes its entries in row order.
__global__ __launch_bounds__(256) void k_fill_col(const uint8_t* __restrict__ mask, const float* __restrict__ W,
                                                  int O, int I, int NBpad, int NB, const int* __restrict__ ptr,
                                                  const int* __restrict__ rowpos, const int* __restrict__ rowmap,
                                                  const int* __restrict__ cidx,
                                                  uint2* __restrict__ ent, int* __restrict__ perm) {
    __shared__ __attribute__((aligned(16))) uint8_t m[KC * MT_LD];
    __shared__ int part[4][MT_COLS];
    const int tid = threadIdx.x, j = tid & 63, rg = tid >> 6;
    const int i0 = blockIdx.x * MT_COLS, c = blockIdx.y, i = i0 + j;
    const int o0 = c * KC;
    load_mask_tile(mask, O, I, o0, i0, m, tid);
    __syncthreads();
    int n = 0;
#pragma unroll
    for (int k = 0; k < 32; ++k) n += m[(32 * rg + k) * MT_LD + j] != 0;
    part[rg][j] = n;
    __syncthreads();
    if (i >= NB * RB) return;                         // (columns past the matrix only pad)
    int jj = 0;
    for (int r = 0; r < rg; ++r) jj += part[r][j];
    const int b = i / RB, rp = rowpos[i], rank = rp & ~SPREAD_FLAG, g = rank & 3, q = rank >> 2;
    const bool spread = (rp & SPREAD_FLAG) != 0;
    const bool guest = !spread && (rowmap[b * RB + 4 * q] & SPREAD_FLAG) != 0;
    const size_t seg = ((size_t)c * NBpad + b) * 4 + q;
    const int pair0 = ptr[seg], npairs = ptr[seg + 1] - pair0;
    if (n > 0) {
        for (int k = 0; k < 32; ++k) {
            const int ol = 32 * rg + k;
            if (!m[ol * MT_LD + j]) continue;
            const size_t f = (size_t)(o0 + ol) * I + i;
            const int64_t e = spread ? entry_slot(pair0, jj & 3, jj >> 2) : entry_slot(pair0, g, jj);
            ent[e] = make_uint2(lds_off((uint32_t)ol), __float_as_uint(W[f]));
            perm[e] = cidx[f];
            ++jj;
        }
    }
    // the thread of the last row group knows the column's whole count in this chunk: it pads
    if (rg == 3 && !guest) pad_row_slots(ent, perm, pair0, npairs, g, spread, jj, 0, 1);
}

// Both views in one launch: the first `row_blocks` blocks refresh the row view's entries,
// the next `col_blocks` the col view's, the last HEAVY_MAX the dense matrix of the heavy rows.
__global__ void k_sync_views(const float* __restrict__ vals, unsigned row_blocks, unsigned col_blocks,
                             const int* __restrict__ ptr_r, int64_t nseg_r, const int* __restrict__ perm_r,
                             uint2* __restrict__ ent_r,
                             const int* __restrict__ ptr_c, int64_t nseg_c, const int* __restrict__ perm_c,
                             uint2* __restrict__ ent_c, const int* __restrict__ heavy, const int* __restrict__ rowptr,
                             const int* __restrict__ flat, int I, float* __restrict__ Hd) {
    if (blockIdx.x >= row_blocks + col_blocks) {
        heavy_fill_row((int)(blockIdx.x - row_blocks - col_blocks), heavy, rowptr, flat, vals, I, Hd);
        return;
    }
    const bool col = blockIdx.x >= row_blocks;
    const int* __restrict__ ptr = col ? ptr_c : ptr_r;
    const int* __restrict__ perm = col ? perm_c : perm_r;
    uint2* __restrict__ ent = col ? ent_c : ent_r;
    const int64_t nseg = col ? nseg_c : nseg_r;
    const int64_t e = (int64_t)(blockIdx.x - (col ? row_blocks : 0u)) * blockDim.x + threadIdx.x;
    if (e >= (int64_t)ptr[nseg] * 8) return;
    const int p = perm[e];
    if (p >= 0) ent[e].y = __float_as_uint(vals[p]);
}

__global__ void k_scatter_dense(const float* __restrict__ vals, const int* __restrict__ flat,
                                int64_t nnz, float* __restrict__ Wd) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < nnz) Wd[flat[k]] = vals[k];
}

__global__ void k_fill_u32(uint32_t* __restrict__ dst, uint32_t value, int64_t n) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n) dst[k] = value;
}

__global__ void k_copy_i32(const int* __restrict__ src, int* __restrict__ dst, int64_t n) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n) dst[k] = src[k];
}

// ------------------------------------------------------------------ build

// out[j] = sum of in[0 .. j), out[n] = total; in == out is allowed
int scan_excl_i32(const int* in, int* out, int64_t n, hipStream_t s) {
    k_scan_excl<<<1, 1024, 0, s>>>(in, out, n);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

// Clears device memory with a kernel (safe to record into a HIP graph, unlike a memset node).
int fill_u32(void* dst, uint32_t value, int64_t n_words, hipStream_t s) {
    if (n_words <= 0) return MST_OK;
    k_fill_u32<<<(unsigned)cdiv(n_words, 256), 256, 0, s>>>((uint32_t*)dst, value, n_words);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

// One view: count per (row, chunk) -> ranking of every block's rows -> pointers of the quad
// segments (with the view's cost for the weight gradient and, for the second view, the choice
// of the driving view) -> ordered compaction.  Five launches; nothing is cleared beforehand:
// the count kernels write the padding rows' zero counts and the fill kernels their own padding.
static int build_one_view(View& v, bool row_view, const mst_layer* L, const float* Wsrc,
                          const Workspace& ws, unsigned long long* cost, hipStream_t s) {
    const int O = L->O, I = L->I;
    const int Rpad = v.NBpad * RB;
    if (row_view) {
        k_count_row<<<Rpad, 256, (size_t)v.nchunk * 4, s>>>(L->mask, O, I, v.nchunk, Rpad, ws.segcnt, ws.rowcnt);
        if (L->heavy_on) {
            MST_LAUNCH_CHECK();
            const int rc = heavy_mark(L, ws, Rpad, s);  // heavy rows leave the view
            if (rc != MST_OK) return rc;
        }
    } else {
        dim3 gcnt((unsigned)cdiv(Rpad, 64), (unsigned)v.nchunk);
        k_count_col<<<gcnt, 256, 0, s>>>(L->mask, O, I, Rpad, ws.segcnt);
    }
    MST_LAUNCH_CHECK();
    k_block_rank<<<(unsigned)cdiv(v.NBpad, 16), 256, 0, s>>>(ws.segcnt, v.nchunk, Rpad, v.NBpad, v.rowmap, v.rowpos);
    MST_LAUNCH_CHECK();
    k_quad_len<<<(unsigned)cdiv(v.nseg, 256), 256, 0, s>>>(ws.segcnt, v.rowmap, Rpad, v.NBpad, v.nseg, ws.qlen);
    MST_LAUNCH_CHECK();
    k_view_ptr<<<1, 1024, 0, s>>>(row_view ? ws.rowcnt : nullptr, L->rowptr, O, ws.qlen, v.NBpad, v.NB, v.nchunk, v.nseg,
                                  v.ptr, cost + (row_view ? 0 : 1), cost, L->I > L->O ? 1 : 0,
                                  row_view ? nullptr : L->sddmm_view, row_view && L->heavy_on ? L->heavy : nullptr);
    MST_LAUNCH_CHECK();
    if (row_view) {
        const int nrows = v.NB * RB;
        const int nparts = std::max(1, std::min(v.nchunk, 8192 / nrows));
        const int cpp = (int)cdiv(v.nchunk, nparts);
        k_fill_row<<<(unsigned)cdiv((int64_t)nrows * nparts, 4), 256, 0, s>>>(
            L->mask, Wsrc, O, I, v.nchunk, v.NBpad, v.NB, L->rowptr, v.ptr, v.rowpos, v.rowmap, L->vals, L->flat, ws.cidx,
            reinterpret_cast<uint2*>(v.ent), v.perm, L->heavy_on ? L->heavy : nullptr, nparts, cpp, ws.segcnt, Rpad);
        if (L->heavy_on) {
            MST_LAUNCH_CHECK();
            const int rc = heavy_fill(L, s);
            if (rc != MST_OK) return rc;
        }
    } else {
        dim3 gcol((unsigned)cdiv(v.NB * RB, 64), (unsigned)v.nchunk);
        k_fill_col<<<gcol, 256, 0, s>>>(L->mask, Wsrc, O, I, v.NBpad, v.NB, v.ptr, v.rowpos, v.rowmap, ws.cidx,
                                        reinterpret_cast<uint2*>(v.ent), v.perm);
    }
    MST_LAUNCH_CHECK();
    return MST_OK;
}

// Rebuilds vals / flat / rowptr and both views from the layer's mask and a dense weight
// array (read at the active positions only).  The col view needs the canonical indices the
// row view pass writes to ws.cidx; its pointer kernel also names the view that drives the
// weight gradient (either can: the product is symmetric in its dense operands).
int build_views(mst_layer* L, const float* Wsrc, const Workspace& ws, hipStream_t s, bool keep_dense_copy) {
    unsigned long long* cost = reinterpret_cast<unsigned long long*>(ws.sel_state);
    L->views_valid = false;
    int rc = build_one_view(L->row, true, L, Wsrc, ws, cost, s);
    if (rc != MST_OK) return rc;
    rc = build_one_view(L->col, false, L, Wsrc, ws, cost, s);
    if (rc != MST_OK) return rc;
    L->views_valid = true;
    if (!keep_dense_copy) L->Wd_valid = L->Wd_zeros = false;
    return MST_OK;
}

// vals / flat / rowptr alone (three launches): what a layer served by the dense contractions needs
int build_canonical(mst_layer* L, const float* Wsrc, const Workspace& ws, hipStream_t s) {
    L->views_valid = false;
    const int nseg = (int)cdiv(L->N, CSEG);
    k_count_seg<<<(unsigned)cdiv(nseg, 4), 256, 0, s>>>(L->mask, L->N, nseg, ws.segcnt);
    MST_LAUNCH_CHECK();
    const int rc = scan_excl_i32(ws.segcnt, ws.segcnt, nseg, s);
    if (rc != MST_OK) return rc;
    k_fill_canonical<<<(unsigned)cdiv(nseg, 4), 256, 0, s>>>(L->mask, Wsrc, L->O, L->I, L->N, nseg, ws.segcnt, L->rowptr, L->vals,
                                                          L->flat);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int refresh_dense_copy(mst_layer* L, hipStream_t s) {
    if (!L->Wd_zeros) {                              // the active set is unchanged since the last fill: only values move
        const int rc = fill_u32(L->Wd, 0u, L->N, s);
        if (rc != MST_OK) return rc;
    }
    if (L->nnz > 0) {
        k_scatter_dense<<<(unsigned)cdiv(L->nnz, 256), 256, 0, s>>>(L->vals, L->flat, L->nnz, L->Wd);
        MST_LAUNCH_CHECK();
    }
    L->Wd_valid = L->Wd_zeros = true;
    return MST_OK;
}

// The views of a layer whose last update left them unbuilt, from the mask and the dense copy.
int ensure_views(const mst_layer* Lc, const Workspace& ws, hipStream_t s) {
    if (Lc->views_valid) return MST_OK;
    mst_layer* L = const_cast<mst_layer*>(Lc);       // a cache of (mask, vals), not layer state
    if (!L->Wd_valid) {
        const int rc = refresh_dense_copy(L, s);
        if (rc != MST_OK) return rc;
    }
    return build_views(L, L->Wd, ws, s, true);
}

// After an update: will a sparse kernel walk the views?  Judged at the batch size and type of
// the last product call; a layer that has seen none yet, or is pinned to the sparse kernels, says yes.
bool views_wanted(const mst_layer* L) {
    if (L->path == MST_PATH_SPARSE) return true;
    if (L->path == MST_PATH_DENSE) return false;
    if (L->hint_T <= 0) return true;
    return !(use_dense_path(L, (mst_dtype)L->hint_act, L->hint_T) && use_dense_weight_grad(L, (mst_dtype)L->hint_act, L->hint_T));
}

}  // namespace mst

using namespace mst;

extern "C" {

int mst_last_hip_error(void) { return g_last_hip_error; }

size_t mst_layer_device_bytes(int O, int I, int64_t nnz_capacity) {
    if (!shape_ok(O, I, nnz_capacity)) return 0;
    return carve_layer(O, I, nnz_capacity).total;
}

size_t mst_workspace_bytes(int O, int I, int64_t nnz_capacity, int T) {
    if (!shape_ok(O, I, nnz_capacity) || T < 1) return 0;
    return carve_workspace(nullptr, O, I, nnz_capacity, T).total;
}

int mst_layer_create(mst_layer_t** out, int O, int I, int64_t nnz_capacity, void* buf_dev,
                     size_t buf_bytes) {
    if (!out || !buf_dev || !aligned16(buf_dev)) return MST_ERR_ARG;
    if (!shape_ok(O, I, nnz_capacity)) return MST_ERR_SHAPE;
    const LayerCarve c = carve_layer(O, I, nnz_capacity);
    if (buf_bytes < c.total) return MST_ERR_WORKSPACE;
    mst_layer* L = new (std::nothrow) mst_layer();
    if (!L) return MST_ERR_STATE;
    char* b = static_cast<char*>(buf_dev);
    L->O = O; L->I = I; L->N = (int64_t)O * I; L->cap = nnz_capacity; L->nnz = 0;
    L->buf = buf_dev; L->buf_bytes = buf_bytes;
    L->mask = (uint8_t*)(b + c.mask);
    L->vals = (float*)(b + c.vals);
    L->flat = (int*)(b + c.flat);
    L->rowptr = (int*)(b + c.rowptr);
    L->Wd = (float*)(b + c.Wd);
    L->sddmm_view = (int*)(b + c.choice);
    L->heavy = (int*)(b + c.heavy);
    L->Hd = (float*)(b + c.Hd);
    auto init_view = [&](View& v, int R, int K, size_t optr, size_t oent, size_t operm, size_t omap, size_t opos) {
        v.R = R; v.K = K; v.nchunk = (int)nchunks(K); v.NB = (int)nblocks(R); v.NBpad = (int)nbpad(R);
        v.nseg = (int64_t)v.nchunk * v.NBpad * 4;
        v.cap_pairs = view_pair_capacity(nnz_capacity, v.nchunk, R);
        v.ptr = (int*)(b + optr); v.ent = (uint4*)(b + oent); v.perm = (int*)(b + operm);
        v.rowmap = (int*)(b + omap); v.rowpos = (int*)(b + opos);
    };
    init_view(L->row, O, I, c.rptr, c.rent, c.rperm, c.rmap, c.rpos);
    init_view(L->col, I, O, c.cptr, c.cent, c.cperm, c.cmap, c.cpos);
    *out = L;
    return MST_OK;
}

int mst_layer_destroy(mst_layer_t* layer) {
    delete layer;
    return MST_OK;
}

int mst_layer_load_dense(mst_layer_t* L, const float* W_dev, const uint8_t* M_dev, void* ws_dev,
                         size_t ws_bytes, mst_stream_t stream) {
    if (!L || !W_dev || !M_dev || !ws_dev || !aligned16(W_dev) || !aligned16(M_dev) || !aligned16(ws_dev))
        return MST_ERR_ARG;
    const Workspace ws = carve_workspace(ws_dev, L->O, L->I, L->cap, 1);
    if (ws_bytes < ws.total) return MST_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    // learn the active count first so that nothing is written when it does not fit
    k_count_row<<<L->O, 256, (size_t)L->row.nchunk * 4, s>>>(M_dev, L->O, L->I, L->row.nchunk, 0, nullptr, ws.rowcnt);
    MST_LAUNCH_CHECK();
    int rcs = scan_excl_i32(ws.rowcnt, L->rowptr, L->O, s);          // rebuilt below anyway
    if (rcs != MST_OK) return rcs;
    int total = 0;
    MST_HIP(hipMemcpyAsync(&total, L->rowptr + L->O, 4, hipMemcpyDeviceToHost, s));
    MST_HIP(hipStreamSynchronize(s));
    if ((int64_t)total > L->cap) return MST_ERR_STATE;
    MST_HIP(hipMemcpyAsync(L->mask, M_dev, (size_t)L->N, hipMemcpyDeviceToDevice, s));
    L->nnz = total;
    L->built = false;                                   // a failed rebuild leaves no usable layer
    // Heavy rows (heavy.hip).  The dense pass costs a launch after every sparse forward, a read of
    // X and T scattered stores per heavy row: a layer of less than 2^20 positions does not earn
    // that back (measured: 768 x 768 at T = 16384 loses 10 us, 768 x 2304 gains 19 us), and a layer
    // whose loaded mask has no heavy row (every uniformly random mask) should not pay the launch.
    // So the rule is tried on this first build of a large layer and kept for the layer's lifetime
    // only if it found rows; the forced mode of the hook keeps it for every layer.
    const int mode = heavy_rows_mode();
    L->heavy_on = mode == 2 || (mode == 1 && L->N >= ((int64_t)1 << 20));
    const int rc = build_views(L, W_dev, ws, s);
    if (rc != MST_OK) return rc;
    if (L->heavy_on && mode == 1) {
        int found = 0;
        MST_HIP(hipMemcpyAsync(&found, L->heavy, 4, hipMemcpyDeviceToHost, s));
        MST_HIP(hipStreamSynchronize(s));
        L->heavy_on = found > 0;
    }
    L->built = true;
    return MST_OK;
}

int mst_layer_export_dense(const mst_layer_t* L, float* W_dev, uint8_t* M_dev, mst_stream_t stream) {
    if (!L) return MST_ERR_ARG;
    if ((W_dev && !aligned16(W_dev)) || (M_dev && !aligned16(M_dev))) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    hipStream_t s = (hipStream_t)stream;
    if (W_dev) {
        int rc = fill_u32(W_dev, 0u, L->N, s);
        if (rc != MST_OK) return rc;
        if (L->nnz > 0) {
            k_scatter_dense<<<(unsigned)cdiv(L->nnz, 256), 256, 0, s>>>(L->vals, L->flat, L->nnz, W_dev);
            MST_LAUNCH_CHECK();
        }
    }
    if (M_dev) MST_HIP(hipMemcpyAsync(M_dev, L->mask, (size_t)L->N, hipMemcpyDeviceToDevice, s));
    return MST_OK;
}

int mst_layer_values(mst_layer_t* L, float** vals_dev, int64_t* nnz) {
    if (!L) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    if (vals_dev) *vals_dev = L->vals;
    if (nnz) *nnz = L->nnz;
    return MST_OK;
}

int mst_layer_sync_values(mst_layer_t* L, mst_stream_t stream) {
    if (!L) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    hipStream_t s = (hipStream_t)stream;
    // A dense copy that is in use (zero at every inactive position) takes the new values now rather
    // than at the next product, so that products recorded into a graph never see stale weights.
    if (L->Wd_zeros && L->nnz > 0) {
        k_scatter_dense<<<(unsigned)cdiv(L->nnz, 256), 256, 0, s>>>(L->vals, L->flat, L->nnz, L->Wd);
        MST_LAUNCH_CHECK();
        L->Wd_valid = true;
    } else {
        L->Wd_valid = false;
    }
    if (L->nnz == 0 || !L->views_valid) return MST_OK;     // unbuilt views take the values when they are built
    // every real entry slot lies below 4 * (nnz + #quad segments); the kernel stops at ptr[nseg] * 8
    const View &r = L->row, &c = L->col;
    const unsigned rb = (unsigned)cdiv(4 * (L->nnz + (int64_t)r.nchunk * r.NB * 4), 256);
    const unsigned cb = (unsigned)cdiv(4 * (L->nnz + (int64_t)c.nchunk * c.NB * 4), 256);
    k_sync_views<<<rb + cb + (L->heavy_on ? HEAVY_MAX : 0), 256, 0, s>>>(L->vals, rb, cb, r.ptr, r.nseg, r.perm, reinterpret_cast<uint2*>(r.ent),
                                                     c.ptr, c.nseg, c.perm, reinterpret_cast<uint2*>(c.ent), L->heavy,
                                                     L->rowptr, L->flat, L->I, L->Hd);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int mst_layer_indices(const mst_layer_t* L, int32_t* flat_dev, mst_stream_t stream) {
    if (!L || !flat_dev) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    if (L->nnz == 0) return MST_OK;
    k_copy_i32<<<(unsigned)cdiv(L->nnz, 256), 256, 0, (hipStream_t)stream>>>(L->flat, flat_dev, L->nnz);
    MST_LAUNCH_CHECK();
    return MST_OK;
}

int mst_layer_set_path(mst_layer_t* L, mst_path path) {
    if (!L || path < MST_PATH_AUTO || path > MST_PATH_DENSE) return MST_ERR_ARG;
    L->path = path;
    return MST_OK;
}

int mst_layer_set_prune_lambda(mst_layer_t* L, float lambda) {
    if (!L || !(lambda >= 0.f) || lambda > 3.4028234e38f) return MST_ERR_ARG;
    L->prune_lambda = lambda;
    return MST_OK;
}

int64_t mst_layer_nnz(const mst_layer_t* L) { return L ? L->nnz : -1; }

}  // extern "C"
