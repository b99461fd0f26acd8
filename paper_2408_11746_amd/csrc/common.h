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
constexpr int TT = 128;          // tokens per LDS tile (two per lane of a wavefront)
constexpr int SEG_PAD = 4;       // every (chunk, row) segment holds a multiple of 4 entries
constexpr int ENT_TAIL = 16;     // readable entries past the last one (prefetch overrun)

// LDS tile layout: row k (one contraction index) holds TT tokens = 512 bytes as 64
// token pairs of 8 bytes.  Lane l owns tokens 2l, 2l+1 and finds them at byte
// lds_off(k) ^ (l << 3): the 5-bit swizzle (k >> 2) spreads the transposing stores of
// the tile loader over all banks while a wavefront's read of one row stays a
// permutation of that row (conflict-free).
__host__ __device__ inline uint32_t lds_off(uint32_t k) {
    return (k << 9) | (((k >> 2) & 31u) << 3);
}

constexpr int MAX_SLAB = 512;    // most rows one workgroup may own; views carry that many empty rows past R

struct View {          // sparse matrix S [R x K] stored by (chunk of K, row, k)
    int R = 0, K = 0, nchunk = 0;
    int Rpad = 0;          // row stride of ptr: >= R + MAX_SLAB; rows >= R have empty segments
    int64_t nseg = 0;      // nchunk * Rpad
    int64_t capv = 0;      // entries the arrays can hold (incl. padding and tail)
    int* ptr = nullptr;    // [nseg + 1] first entry of segment c*Rpad + r
    uint2* ent = nullptr;  // [capv] {lds_off(k - c*KC), fp32 bits of the weight}
    int* perm = nullptr;   // [capv] canonical index of the entry, -1 for padding
};

}  // namespace mst

struct mst_layer {
    int O = 0, I = 0;
    int64_t N = 0, cap = 0, nnz = 0;
    int path = MST_PATH_AUTO;
    void* buf = nullptr;
    size_t buf_bytes = 0;
    uint8_t* mask = nullptr;   // [N]
    float* vals = nullptr;     // [cap] canonical (ascending flat index) values
    int* flat = nullptr;       // [cap] canonical flat indices
    int* rowptr = nullptr;     // [O + 1] canonical CSR row pointers
    float* Wd = nullptr;       // [N] dense W . M, maintained only while the dense path is in use
    bool Wd_valid = false;
    mst::View row;             // S = W   [O x I], used by fwd and bwd_weight
    mst::View col;             // S = W^T [I x O], used by bwd_input
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
bool use_dense_path(const mst_layer* L);

// ---- workspace carving (one place so that mst_workspace_bytes and the users agree) ----
struct Workspace {
    float* G = nullptr;        // [N] dense gradient (mst_mask_update)
    float* Wd = nullptr;       // [N] dense scratch of the weights during a rebuild
    int* cidx = nullptr;       // [N] canonical index of each active position
    uint8_t* sel = nullptr;    // [N] selection flags of the grow step
    uint8_t* psel = nullptr;   // [cap] selection flags of the prune step
    int* segcnt = nullptr;     // [max(nseg_row, nseg_col) + 1]
    int* rowcnt = nullptr;     // [O + 1]
    uint32_t* blk = nullptr;   // [select_blocks(N) + 1] per-block tie counts
    uint64_t* sel_state = nullptr;   // radix-select state + histogram
    float* gemm = nullptr;     // [GEMM_WS_SPLITS * N] split-k partial outputs of the dense GEMM
    size_t gemm_floats = 0;
    float* partial = nullptr;  // SDDMM partial sums [ntile][capv_row]
    size_t partial_floats = 0;
    size_t total = 0;
};
Workspace carve_workspace(void* base, int O, int I, int64_t cap, int T);

constexpr int GEMM_WS_SPLITS = 4;
constexpr int SELECT_BLOCK = 2048;   // elements per block in the ordered tie pass
constexpr int SEL_STATE_WORDS = 8 + 256;

int64_t view_capacity(int64_t cap, int64_t nchunk, int64_t R);
int fill_u32(void* dst, uint32_t value, int64_t n_words, hipStream_t s);

// ---- internal entry points implemented across the .hip files ----
int build_views(mst_layer* L, const float* Wsrc, const Workspace& ws, hipStream_t s);
int spmm(const View& v, const void* A, float* out, int T, int64_t nnz, mst_dtype act, hipStream_t s);
int sddmm(const mst_layer* L, const void* dY, const void* X, float* dW, int T, mst_dtype act,
          const Workspace& ws, hipStream_t s);
// C[M x N] (fp32) = op(A) op(B) on the matrix cores; see gemm_mfma.hip
enum GemmKind { GEMM_TN = 0, GEMM_NT = 1, GEMM_NN = 2 };
int gemm_mfma(GemmKind kind, const void* A, mst_dtype a_dt, const void* B, mst_dtype b_dt, float* C,
              int M, int N, int Kdim, float* split_ws, int64_t split_ws_floats, hipStream_t s);
int mask_update_device(mst_layer* L, const float* G, const mst_update_stats& st, uint64_t seed,
                       const Workspace& ws, hipStream_t s);
int dense_products_fwd(const mst_layer* L, const void* X, float* Y, int T, mst_dtype act, hipStream_t s);
int dense_products_bwd_input(const mst_layer* L, const void* dY, float* dX, int T, mst_dtype act, hipStream_t s);
int dense_products_bwd_weight(const mst_layer* L, const void* dY, const void* X, float* dW, int T,
                              mst_dtype act, const Workspace& ws, hipStream_t s);
int refresh_dense_copy(mst_layer* L, hipStream_t s);

}  // namespace mst
