// Internal declarations shared by the translation units of libmst_hip.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mst.h"

namespace mst {

// ---- tiling constants shared by the format builder and the product kernels ----
// The contraction dimension of a view is cut into chunks of KC indices; one chunk of
// the dense operand for TT tokens is what a workgroup stages in LDS at a time.
constexpr int KC = 128;          // contraction indices per chunk
constexpr int TT = 128;          // tokens per LDS tile
constexpr int RB = 16;           // rows per row block: 4 lane groups x 4 quads
constexpr int MAX_WG_BLOCKS = 32;
constexpr int SPREAD_FLAG = 1 << 30;   // in rowmap / rowpos: the quad holds ONE row spread over its four lane groups   // most row blocks one workgroup may own
constexpr int HEAVY_MAX = 64;   // rows a layer may keep out of its row view as a small dense matrix (heavy.hip)
constexpr int PAIR_TAIL = 16;    // readable step pairs past the last one (a whole entry batch may be fetched there)

// LDS tile layout: row k (one contraction index) holds TT tokens = 512 bytes as 32
// 16-byte slots of four consecutive tokens; slot u of tokens 4u..4u+3 sits at byte
// (u >> 4) * 256 + ((u & 15) ^ ((k >> 2) & 15)) * 16.  Lane s (0..15) of a lane group
// owns tokens 4s..4s+3 and 64+4s..64+4s+3 and finds them at lds_off(k) ^ (s << 4) and
// 256 bytes further.  The XOR spreads the transposing stores of the tile loader over all
// banks while the 16 lanes of a group still read one contiguous 256 bytes.
__host__ __device__ inline uint32_t lds_off(uint32_t k) {
    return (k << 9) | (((k >> 2) & 15u) << 4);
}

// Sparse matrix S [R x K] as the product kernels walk it.  Rows are grouped in blocks of
// RB = 16 consecutive rows.  Inside a block the rows are ranked by their total length
// (longest first, lower index first on ties); the row of rank 4q + g belongs to quad q and
// lane group g, so the four rows of a quad have similar lengths (little ELL padding even
// when row lengths are very uneven).  rowmap[16b + rank] is that row.  For every
// (chunk c of K, block b, quad q) the four rows' entries inside the chunk are stored side
// by side, padded with zero-weight entries to the longest of the four and to an even
// count (an ELL slice of height 4): step j of the quad holds one entry per lane group.
// Two steps form a pair = uint4[4]: element g is {off_j, w_j, off_j+1, w_j+1} of lane
// group g, off = lds_off(k - c*KC), w = fp32 bits.
// A very long row can take a whole quad ("spread"): its entries are dealt to the four lane
// groups in turn (entry j of a chunk: lane group j & 3, step j >> 2), the kernels add the
// four lane groups' sums at the end.  The other three places of such a quad are given to
// three EMPTY rows of the block (they own the output positions, which receive zero), so a
// block spreads at most as many rows as it has triples of empty rows.  All four rowmap
// entries of a spread quad and the rowpos entry of the spread row carry SPREAD_FLAG.
struct View {
    int R = 0, K = 0, nchunk = 0;
    int NB = 0;            // row blocks: ceil(R / 16)
    int NBpad = 0;         // block stride of ptr: NB + MAX_WG_BLOCKS (the extra blocks stay empty)
    int64_t nseg = 0;      // nchunk * NBpad * 4 quad segments
    int64_t cap_pairs = 0; // pairs the arrays can hold (incl. tail)
    int* ptr = nullptr;    // [nseg + 1] first pair of segment (c*NBpad + b)*4 + q
    uint4* ent = nullptr;  // [cap_pairs * 4]
    int* perm = nullptr;   // [cap_pairs * 8] canonical index of entry slot (pair*4 + g)*2 + half, -1 = padding
    int* rowmap = nullptr; // [NBpad * 16] rank inside the block -> row (identity in the empty blocks)
    int* rowpos = nullptr; // [NBpad * 16] row -> rank inside its block
};

// Hd row j = row heavy[1 + j] of W . M, from the canonical arrays, by one block (heavy rows, heavy.hip).
// Every thread of the block must call it; j at or past the count does nothing.
__device__ inline void heavy_fill_row(int j, const int* __restrict__ heavy, const int* __restrict__ rowptr,
                                      const int* __restrict__ flat, const float* __restrict__ vals, int I,
                                      float* __restrict__ Hd) {
    if (j >= min(heavy[0], HEAVY_MAX)) return;
    const int h = heavy[1 + j];
    float* row = Hd + (int64_t)j * I;
    for (int i = threadIdx.x; i < I; i += blockDim.x) row[i] = 0.f;
    __syncthreads();
    const int k1 = rowptr[h + 1];
    for (int k = rowptr[h] + threadIdx.x; k < k1; k += blockDim.x) row[flat[k] - h * I] = vals[k];
}

}  // namespace mst

struct mst_layer {
    int O = 0, I = 0;
    int64_t N = 0, cap = 0, nnz = 0;
    bool built = false;        // the device arrays are meaningful only after mst_layer_load_dense has succeeded
    int path = MST_PATH_AUTO;
    float prune_lambda = 0.f;  // prune score |w| + prune_lambda |grad| (0: magnitude only)
    void* buf = nullptr;
    size_t buf_bytes = 0;
    uint8_t* mask = nullptr;   // [N]
    float* vals = nullptr;     // [cap] canonical (ascending flat index) values
    int* flat = nullptr;       // [cap] canonical flat indices
    int* rowptr = nullptr;     // [O + 1] canonical CSR row pointers
    float* Wd = nullptr;       // [N] dense W . M, maintained only while the dense path is in use
    bool Wd_valid = false;     // Wd equals W . M
    bool Wd_zeros = false;     // Wd is zero at every inactive position (survives a change of the values)
    // The index views are built lazily: an update of a layer that the dense contractions serve
    // (path choice at the batch size and type of the last product call) leaves them unbuilt; a
    // call that needs them and has a workspace builds them, one without runs the dense product.
    bool views_valid = false;
    int hint_T = 0;            // batch size and activation type of the last product call (0: none yet)
    int hint_act = 0;
    mst::View row;             // S = W   [O x I], used by fwd (and bwd_weight)
    mst::View col;             // S = W^T [I x O], used by bwd_input
    int* sddmm_view = nullptr; // device flag: view that drives bwd_weight (0 row, 1 col), set when the views are built
    // Heavy rows (see heavy.hip): device list [0] = count, [1 + j] = row; Hd [HEAVY_MAX x I] their dense weights.
    // Both follow the views: written when they are built, Hd again whenever the values change.
    int* heavy = nullptr;
    float* Hd = nullptr;
    bool heavy_on = false;     // the rule applies to this layer (decided when it is loaded)
};

namespace mst {

extern thread_local int g_last_hip_error;

#define MST_HIP(call)                                                     \
    do {                                                                  \
        hipError_t e__ = (call);                                          \
        if (e__ != hipSuccess) {                                          \
            mst::g_last_hip_error = (int)e__;                             \
            return MST_ERR_HIP;                                           \
        }                                                                 \
    } while (0)

#define MST_LAUNCH_CHECK() MST_HIP(hipGetLastError())

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// true when a layer of this density should run the masked dense MFMA kernels
bool use_dense_path(const mst_layer* L, mst_dtype act, int T);
bool use_dense_weight_grad(const mst_layer* L, mst_dtype act, int T);
bool use_fused_backward(const mst_layer* L, mst_dtype act, int T);

// ---- workspace carving (one place so that mst_workspace_bytes and the users agree) ----
struct Workspace {
    float* G = nullptr;        // [N] dense gradient (mst_mask_update)
    float* Wd = nullptr;       // [N] dense scratch of the weights during a rebuild
    int* cidx = nullptr;       // [N] canonical index of each active position
    uint8_t* sel = nullptr;    // [N] selection flags of the grow step
    uint8_t* psel = nullptr;   // [cap] selection flags of the prune step
    int* segcnt = nullptr;     // active count per (chunk, row) of the view being built
    int* qlen = nullptr;       // pairs per quad segment of the view being built
    int* rowcnt = nullptr;     // [O + 1]
    uint32_t* blk = nullptr;   // per-block tie counts: [blocks(N) + 1] of the growth selections, then [blocks(cap) + 1] of the prune selection
    uint64_t* sel_state = nullptr;   // [SEL_STATES][SEL_STATE_WORDS] radix-select state + histogram
    float* gemm = nullptr;     // [GEMM_WS_SPLITS * N] split-k partial outputs of the dense GEMM
    size_t gemm_floats = 0;
    float* partial = nullptr;  // SDDMM partial sums [ntile][entry slots of the row view]
    size_t partial_floats = 0;
    size_t total = 0;
};
Workspace carve_workspace(void* base, int O, int I, int64_t cap, int T);

constexpr int GEMM_WS_SPLITS = 8;
constexpr int SELECT_BLOCK = 2048;   // elements per block in the ordered tie pass
constexpr int SEL_DIGIT_BITS = 8;                        // radix-select digit
constexpr int SEL_BINS = 1 << SEL_DIGIT_BITS;
constexpr int SEL_STATE_WORDS = 8 + 4096 / 2;            // one selection: 8 control words + up to 4096 uint32 histogram bins
constexpr int SEL_STATES = 3;                            // prune, gradient growth, random growth

int64_t view_pair_capacity(int64_t cap, int64_t nchunk, int64_t R);
int fill_u32(void* dst, uint32_t value, int64_t n_words, hipStream_t s);

// ---- internal entry points implemented across the .hip files ----
int build_views(mst_layer* L, const float* Wsrc, const Workspace& ws, hipStream_t s, bool keep_dense_copy = false);
int build_canonical(mst_layer* L, const float* Wsrc, const Workspace& ws, hipStream_t s);
int ensure_views(const mst_layer* L, const Workspace& ws, hipStream_t s);
bool views_wanted(const mst_layer* L);
int spmm(const View& v, const void* A, float* out, int T, int64_t nnz, mst_dtype act, hipStream_t s);
int spmm_force_shape(int tokens_per_workgroup, int quads_per_wavefront);
int sddmm(const mst_layer* L, const void* dY, const void* X, float* dW, int T, mst_dtype act,
          const Workspace& ws, hipStream_t s);
// dX and dW from one walk of the col view; see bwd_fused.hip
int bwd_fused(const mst_layer* L, const void* dY, const void* X, float* dX, float* dW, int T, mst_dtype act,
              const Workspace& ws, hipStream_t s);
bool bwd_fused_pays(const mst_layer* L);
int bwd_fused_force_shape(int waves, int quads);
// C[M x N] (fp32) = op(A) op(B) on the matrix cores; see gemm_mfma.hip
enum GemmKind { GEMM_TN = 0, GEMM_NT = 1, GEMM_NN = 2 };
int gemm_mfma(GemmKind kind, const void* A, mst_dtype a_dt, const void* B, mst_dtype b_dt, float* C,
              int M, int N, int Kdim, float* split_ws, int64_t split_ws_floats, hipStream_t s, int* left_unsummed = nullptr);
int gemm_force_fp32_mfma(int on);
int gemm_last_tile();
int mask_update_device(mst_layer* L, const float* G, const mst_update_stats& st, uint64_t seed,
                       const Workspace& ws, hipStream_t s);
int dense_products_fwd(const mst_layer* L, const void* X, float* Y, int T, mst_dtype act, hipStream_t s,
                       float* split_ws = nullptr, int64_t split_ws_floats = 0);
int dense_products_bwd_input(const mst_layer* L, const void* dY, float* dX, int T, mst_dtype act, hipStream_t s,
                             float* split_ws = nullptr, int64_t split_ws_floats = 0);
int dense_products_bwd_weight(const mst_layer* L, const void* dY, const void* X, float* dW, int T,
                              mst_dtype act, const Workspace& ws, hipStream_t s);
int refresh_dense_copy(mst_layer* L, hipStream_t s);
// heavy rows of the forward product; see heavy.hip
int heavy_rows_enable(int on);
int heavy_rows_mode();
int heavy_mark(const mst_layer* L, const Workspace& ws, int Rpad, hipStream_t s);
int heavy_fill(const mst_layer* L, hipStream_t s);
int heavy_fwd(const mst_layer* L, const void* X, float* Y, int T, mst_dtype act, hipStream_t s);

}  // namespace mst
