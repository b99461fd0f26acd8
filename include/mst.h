/*
 * mst.h -- C ABI of the MI355X (gfx950) library for the training step of the
 * dynamically sparse fully-connected layers of Mixed Sparsity Training.
 *
 * A layer is W [O x I] (row-major, flat index f = o*I + i) with a binary mask M of
 * the same shape (the mask M of Sec. 3.2).
 * Its effective weight is W (.) M (Algorithm 1, last line).  With X [T x I] the input
 * and dY [T x O] the gradient at the output:
 *
 *   mst_sparse_fc_fwd         Y  = X (W.M)^T                   (App. "FLOP Calculation", Eq. (1))
 *   mst_sparse_fc_bwd_input   dX = dY (W.M)                    (same App.: backward = 2 x forward)
 *   mst_sparse_fc_bwd_weight  dW = (dY^T X) at active positions only
 *   mst_mask_update           Algorithm 1 "Topology Evolution by MG"
 *   mst_schedule_density      Sec. 3.1 "Sparsity Variation" + Sec. 3.2 update fraction
 * and around them the per-layer density allocation of Sec. 3.2, the FLOP counts of
 * App. "FLOP Calculation" and the strided attention pattern of Sec. 3.3.
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory, owned by the caller, 16-byte aligned;
 *     everything else is host memory.  The library allocates no device memory: the
 *     caller hands it one backing buffer per layer (mst_layer_device_bytes) and a
 *     workspace (mst_workspace_bytes) that may be shared by all layers used on a stream.
 *   - Activations (X, dY) are row-major, fp32 or bfloat16 (mst_dtype); W, Y, dX, dW and
 *     the dense gradient are fp32; accumulation is fp32.
 *   - All device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  Calls return after enqueueing unless stated otherwise.
 *   - Outputs are overwritten, never accumulated into.  Results are deterministic:
 *     identical inputs give bit-identical outputs (no floating-point atomics).
 *   - Return value: MST_OK or a negative mst_status.  Arguments are validated on the
 *     host before anything is launched; on error nothing has been enqueued.
 *   - Inputs must be finite; NaN / Inf give unspecified selections in mst_mask_update.
 *   - Calls on the same layer or the same workspace must not overlap in time.
 */
#ifndef MST_H
#define MST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mst_layer mst_layer_t;   /* opaque host object */
typedef void* mst_stream_t;             /* hipStream_t */

typedef enum { MST_F32 = 0, MST_BF16 = 1 } mst_dtype;

typedef enum {
    MST_OK = 0,
    MST_ERR_ARG = -1,        /* null pointer, misaligned pointer, value out of range */
    MST_ERR_SHAPE = -2,      /* dimension not supported / inconsistent */
    MST_ERR_WORKSPACE = -3,  /* workspace or layer buffer too small */
    MST_ERR_STATE = -4,      /* layer not loaded yet, or the active count would exceed its capacity */
    MST_ERR_HIP = -5         /* a HIP runtime call failed; see mst_last_hip_error() */
} mst_status;

/* compute path of the three products: unstructured-sparse kernels, masked dense
 * MFMA kernels (for the dense end of the warm-up / restoration phases), or chosen
 * from the layer's density. */
typedef enum { MST_PATH_AUTO = 0, MST_PATH_SPARSE = 1, MST_PATH_DENSE = 2 } mst_path;

/* The index views that the sparse kernels walk are built when a sparse kernel will need them.
 * mst_layer_load_dense always builds them.  A topology update builds them unless the layer, at
 * its new density, is served by the dense contractions (judged by the path setting and by
 * the batch size and activation type of the layer's last product call; a layer that has seen
 * no product call yet, or is pinned to MST_PATH_SPARSE, always gets them); such an update
 * rebuilds only the value / index vectors and writes the layer's dense weight copy in place.
 * While the views are unbuilt: the calls that carry a workspace (mst_sparse_fc_bwd,
 * mst_sparse_fc_bwd_weight, mst_sparse_fc_bwd_weight_update) build them first whenever a sparse
 * kernel is due; mst_sparse_fc_fwd and mst_sparse_fc_bwd_input, which carry none, compute the
 * same product with the dense contraction whatever the density; mst_sparse_fc_bwd_weight_static
 * returns MST_ERR_STATE; mst_layer_format_stats reports zero stored entries. */

/* Hyper-parameters of Sec. 3.1 / 3.2 (Table "Private hyperparameters of MST"). */
typedef struct {
    double S_M;            /* maximum sparsity, in [0, 1] (paper: 0.96) */
    int32_t N;             /* number of sparsity stages (5) */
    int64_t Delta_W;       /* pruning frequency of the warm-up (2000); T_W = N * Delta_W */
    int64_t T_U;           /* ultra-sparsification duration (100000) */
    int64_t Delta_R;       /* growing frequency of the restoration (2000); T_R = N * Delta_R */
    const double* zeta;    /* zeta_1 .. zeta_{N+1}: magnitude of each cosine period (host) */
    int32_t n_zeta;        /* must equal N + 1 */
} mst_schedule_cfg;

/* What one mask update did (Algorithm 1, count lines). */
typedef struct {
    int64_t nnz_before, nnz_after;
    int64_t n_prune, n_grow, n_rand, n_grad;
} mst_update_stats;

const char* mst_version(void);
int mst_last_hip_error(void);           /* hipError_t of the last failing HIP call on this thread */

/* ------------------------------------------------------------------ layers */

/* Bytes of device memory a layer of shape [O x I] needs to hold up to nnz_capacity
 * active weights (mask, values, both index views).  0 on invalid arguments. */
size_t mst_layer_device_bytes(int O, int I, int64_t nnz_capacity);

/* Bytes of workspace sufficient for every call below on a layer of this shape with
 * up to T tokens.  0 on invalid arguments. */
size_t mst_workspace_bytes(int O, int I, int64_t nnz_capacity, int T);

/* Creates the host object over the caller's buffer (kept, not copied, never freed by
 * the library; its contents are not touched).  The layer has no weights until
 * mst_layer_load_dense has succeeded: until then every call that would read the layer's
 * device arrays (the products, the updates, export, values, indices, sync) returns
 * MST_ERR_STATE without launching anything.  1 <= O, I <= 65535. */
int mst_layer_create(mst_layer_t** out, int O, int I, int64_t nnz_capacity,
                     void* buf_dev, size_t buf_bytes);
int mst_layer_destroy(mst_layer_t* layer);   /* frees the host object only */

/* Loads W . M from dense arrays (W_dev [O*I] fp32, M_dev [O*I] bytes, non-zero = active)
 * and builds the index views.  Synchronises `stream` once to learn the active count.
 * MST_ERR_STATE if it exceeds the capacity. */
int mst_layer_load_dense(mst_layer_t* layer, const float* W_dev, const uint8_t* M_dev,
                         void* ws_dev, size_t ws_bytes, mst_stream_t stream);

/* Writes W . M (zeros at inactive positions) and / or M; either pointer may be NULL. */
int mst_layer_export_dense(const mst_layer_t* layer, float* W_dev, uint8_t* M_dev,
                           mst_stream_t stream);

/* The active weights as one fp32 vector in ascending flat-index order, for the caller's
 * optimiser to update in place.  After changing them call mst_layer_sync_values: it copies
 * the values into whatever the products read (the entries of built index views, a dense
 * weight copy that is in use) with one or two kernels on `stream`, nothing else; products
 * recorded into a HIP graph therefore see the new values on their next replay.  Every
 * mask update changes the set and therefore the meaning of position k of this vector. */
int mst_layer_values(mst_layer_t* layer, float** vals_dev, int64_t* nnz);
int mst_layer_sync_values(mst_layer_t* layer, mst_stream_t stream);

/* Flat indices (ascending, int32) of the active positions, same order as the values. */
int mst_layer_indices(const mst_layer_t* layer, int32_t* flat_dev, mst_stream_t stream);

int mst_layer_set_path(mst_layer_t* layer, mst_path path);

/* Which path a product call with these arguments takes on the layer as it stands: 1 = masked
 * dense MFMA contraction, 0 = sparse kernel; weight_gradient = 0 asks for Y and dX (Eq. (1) and
 * its input gradient), 1 for the gradient of the active weights, 2 for mst_sparse_fc_bwd (both
 * gradients from the shared walk, or both from dense contractions).  Host only, no device work;
 * MST_ERR_ARG on a null layer, an unknown type or T < 1. */
int mst_layer_uses_dense(const mst_layer_t* layer, mst_dtype act, int T, int weight_gradient);

/* Prune criterion of the following updates of this layer.  0 (the default) is the paper's:
 * the smallest |w|.  lambda > 0 selects the other criterion of the table of topology
 * evolution schemes in Sec. 3.2, the smallest |w| + lambda |grad|, with the same dense
 * gradient that scores growth (the score buffer of mst_mask_update_from_scores) and the
 * score formed in fp32 (product rounded, then the sum); ties go to the lower flat index as
 * always.  The paper gives no value for lambda.  MST_ERR_ARG unless lambda is finite and >= 0. */
int mst_layer_set_prune_lambda(mst_layer_t* layer, float lambda);
int64_t mst_layer_nnz(const mst_layer_t* layer);

/* Launch shape of the sparse products' SpMM kernel: tokens per workgroup (128 or 64) and
 * quads of four rows per wavefront (2, 3 or 4 with 128 tokens; 2, 3, 4, 6 or 8 with 64).  By
 * default the library chooses per call from T, the layer's shape and its density; every
 * shape gives bit-identical results.  This call pins one shape for all later calls of the
 * process (tests and tuning); (0, 0) returns to the automatic choice.  Not thread-safe.
 * MST_ERR_ARG for a combination that does not exist. */
int mst_spmm_force_shape(int tokens_per_workgroup, int quads_per_wavefront);

/* Heavy rows.  When the index views of a layer are built, rows of W . M that hold at least a
 * quarter of a row's positions AND at least four times the mean row (and at least 32 entries) --
 * the first 64 such rows in row order -- are kept out of the row view and stored as a small
 * dense matrix instead; mst_sparse_fc_fwd computes their outputs Y[:, row] with a dense
 * contraction on the matrix cores (fp32 operands split into bfloat16 hi + lo as described at
 * mst_gemm_force_fp32_mfma: within 2^-16 per term of the fp32 product) after the sparse kernel
 * has written the others.  Masks with power-law row lengths have such rows (a few dozen rows
 * holding most of the nonzeros); uniformly random masks have none, and nothing changes for
 * them.  The backward products and every index order are unaffected.  By default (1) the rule
 * applies to a layer of at least 2^20 positions whose mask, as mst_layer_load_dense received it,
 * has such rows, and then for the layer's lifetime (smaller layers do not earn the extra pass
 * back; the others are spared its launch); mst_heavy_rows(0) switches it off and
 * mst_heavy_rows(2) on for every layer, for the layers loaded from then on in this process.
 * Test and measurement aid, not thread-safe; MST_ERR_ARG for another value. */
int mst_heavy_rows(int on);

/* ------------------------------------------------------------- the products */

/* Y_dev [T*O] = X_dev [T*I] (W.M)^T.  T >= 1. */
int mst_sparse_fc_fwd(const mst_layer_t* layer, const void* X_dev, float* Y_dev, int T,
                      mst_dtype act, mst_stream_t stream);

/* dX_dev [T*I] = dY_dev [T*O] (W.M). */
int mst_sparse_fc_bwd_input(const mst_layer_t* layer, const void* dY_dev, float* dX_dev, int T,
                            mst_dtype act, mst_stream_t stream);

/* dW_dev [nnz] = sum_t dY[t, o] X[t, i] for the active (o, i), ascending flat index. */
int mst_sparse_fc_bwd_weight(const mst_layer_t* layer, const void* dY_dev, const void* X_dev,
                             float* dW_dev, int T, mst_dtype act,
                             void* ws_dev, size_t ws_bytes, mst_stream_t stream);

/* For callers that cannot allocate or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): mst_sparse_fc_bwd_weight with its scratch
 * -- the per-token-tile partial sums of the SDDMM -- in a device array that is part of the
 * library (mst_static_scratch_bytes() = 64 MiB, held by every GPU the library runs on until
 * the process ends).  Always runs the sparse kernels (never the dense-gradient variant), so
 * dW_dev equals mst_sparse_fc_bwd_weight's result exactly on the sparse path and up to the
 * order of the fp32 sums where that call would use a dense contraction.  Calls no allocating
 * routine.  MST_ERR_WORKSPACE when ceil(T / 128) planes of partial sums (8 floats per pair of
 * entry slots of the larger index view at the layer's CAPACITY) exceed the array: e.g. a
 * 768 x 3072 layer of capacity 177 k fits up to T = 2944.  All calls on one GPU share the
 * array: calls that overlap in time on one GPU (other streams, other threads) race.  The
 * first call on a device looks the array's address up (hipGetSymbolAddress); make that call
 * outside stream capture. */
int mst_sparse_fc_bwd_weight_static(const mst_layer_t* layer, const void* dY_dev, const void* X_dev,
                                    float* dW_dev, int T, mst_dtype act, mst_stream_t stream);
size_t mst_static_scratch_bytes(void);

/* Both gradients of the backward pass in one call: dX as mst_sparse_fc_bwd_input, dW_vals as
 * mst_sparse_fc_bwd_weight.  On the sparse path the two products share one walk of the
 * layer's transposed view (the staged dY tile, the entries and every LDS read serve both);
 * dX is bit-identical to mst_sparse_fc_bwd_input, dW_vals equals mst_sparse_fc_bwd_weight up
 * to the order of the fp32 sums.  (A short batch may split the contraction over several
 * workgroups; dX then equals mst_sparse_fc_bwd_input up to the order of its sums too.  The same
 * holds on the dense path: with the workspace at hand the dense product for dX may cut its
 * contraction range into two or three where the output has too few tiles to fill the chip.)
 * Workspace: mst_workspace_bytes(O, I, nnz_capacity, T). */
int mst_sparse_fc_bwd(const mst_layer_t* layer, const void* dY_dev, const void* X_dev,
                      float* dX_dev, float* dW_vals_dev, int T, mst_dtype act,
                      void* ws_dev, size_t ws_bytes, mst_stream_t stream);

/* Test hook like mst_spmm_force_shape for the shared walk of mst_sparse_fc_bwd:
 * (8, 3) .. (8, 5), (16, 1) or (16, 2) wavefronts per workgroup x quads per wavefront, (0, 0) = automatic.
 * Every shape gives the same results. */
int mst_bwd_force_shape(int wavefronts_per_workgroup, int quads_per_wavefront);

/* The dense fp32 products (the dense gradient below, and the three products of a layer on the
 * dense path) run on the bf16 matrix cores when their shapes are whole tiles: each fp32
 * operand element is split into two bfloat16 values (hi + lo, exact to 2^-17) while it is
 * staged, a product is hi*hi + hi*lo + lo*hi with fp32 accumulation; the result differs from
 * an fp32 product by less than 2^-16 per term.  This hook pins, for all later calls of the
 * process: 1 = the plain fp32 MFMA kernel; 128, 256, 160 or 192 = the split kernel with the
 * workgroup tile 128 x 128, 256 x 256, 256 x 160 or 256 x 192 (where the shape is a multiple of
 * it; the last two serve Y and dX only); 0 returns to the automatic choice.  All tiles add a
 * result's terms in the same order and give identical bits.  -52 / 52 switch off / on the
 * schedule that gives two 256 x 256 tiles five workgroups (used where plain k ranges would
 * leave a fifth of the CUs idle; other cut points of the k range, so another order of
 * additions); these two leave the other settings as they are.  Test and measurement aid,
 * not thread-safe. */
int mst_gemm_force_fp32_mfma(int on);
/* Workgroup tile (128, 256, 160 or 192 as above) of the last dense product that ran on a split
 * kernel in this process, 0 if it ran on another kernel.  Test aid, not thread-safe. */
int mst_gemm_last_tile(void);

/* G_dev [O*I] = dY^T X at every position (the score of gradient-based growth: the dense
 * gradient that Sec. 2 notes such growth needs now and then).  Runs on the matrix cores.  ws_dev may be
 * NULL; with a workspace small outputs split the token range over more workgroups. */
int mst_dense_grad(const void* dY_dev, const void* X_dev, float* G_dev, int T, int O, int I,
                   mst_dtype act, void* ws_dev, size_t ws_bytes, mst_stream_t stream);

/* dW_dev [nnz] = G_dev [O*I] read at the active positions (ascending flat index): the weight
 * gradient of a step whose dense gradient was formed anyway (mst_dense_grad on an update
 * step), the middle part of mst_sparse_fc_bwd_weight_update as a call of its own. */
int mst_gather_active(const mst_layer_t* layer, const float* G_dev, float* dW_dev, mst_stream_t stream);

/* What the index views of a layer store.  A view keeps, per chunk of 128 contraction indices
 * and quad of four rows, as many steps as the longest of the four rows needs, padded to an
 * even count; each step has one entry slot per row.  efficiency = nnz / slots is the share of
 * walk steps that do real work (for the row view: of the entries it holds, nnz minus those of
 * the heavy rows, see mst_heavy_rows).  Synchronises `stream` (reads a few counters back). */
typedef struct {
    int64_t nnz;
    int64_t row_view_slots, col_view_slots;     /* entry slots incl. zero-weight padding */
    double row_view_efficiency, col_view_efficiency;
    int64_t heavy_rows, heavy_entries;          /* rows kept as a dense matrix and their entries (0 if the rule is off) */
} mst_format_stats;
int mst_layer_format_stats(const mst_layer_t* layer, mst_format_stats* out, mst_stream_t stream);

/* Measurement aid: a kernel that only reads LDS, for the on-chip roofline of the sparse
 * products (every multiply-add of the walk needs its own 4-byte activation operand from
 * LDS).  `blocks` workgroups of 1024 threads each perform iters * 8 conflict-free reads of
 * `width` bytes (4, 8 or 16) per thread from a 64 KB tile and write one float per thread to
 * out_dev [blocks * 1024].  Bytes read = blocks * 1024 * iters * 8 * width; time it with
 * events on `stream`. */
int mst_probe_lds_read(float* out_dev, int width, int iters, int blocks, mst_stream_t stream);

/* ------------------------------------------------------------ topology update */

/* Host arithmetic of Algorithm 1's count lines for a layer of n_total positions with
 * nnz active: target count = floor(d*n_total + 0.5); N_prune = floor(zeta*nnz);
 * N_grow = N_prune + (target - nnz), clamped so that 0 <= N_grow <= n_total - nnz and the
 * layer lands exactly on the target; N_rand = floor(N_grow*R); N_grad = N_grow - N_rand. */
int mst_update_counts(int64_t n_total, int64_t nnz, double target_density, double zeta,
                      double rand_ratio, mst_update_stats* out);

/* One Mixed-Growing update given the score buffer G_dev [O*I] (fp32):
 *   prune  the N_prune active weights with the smallest (|w|, f);
 *   grow   the N_grad inactive positions with the largest |G| (lowest f on ties), then
 *          the N_rand inactive, not gradient-grown positions with the smallest
 *          (SplitMix64(rng_seed)[f], f), where SplitMix64(s)[f] is the (f+1)-th output of
 *          the SplitMix64 generator started at state s;
 *   apply  pruned and grown weights are 0; kept weights keep their value; the index
 *          views are rebuilt.  |.| compares fp32 bit patterns with the sign cleared.
 * The new active count is known on return (host arithmetic); the device work is
 * asynchronous.  stats_out (host) may be NULL. */
int mst_mask_update_from_scores(mst_layer_t* layer, const float* G_dev,
                                double target_density, double zeta, double rand_ratio,
                                uint64_t rng_seed, void* ws_dev, size_t ws_bytes,
                                mst_update_stats* stats_out, mst_stream_t stream);

/* mst_mask_update_from_scores for n_layers layers in one call: layer j with score buffer
 * G_dev[j], density target_density[j], seed rng_seed[j], workspace ws_dev[j] (ws_bytes[j]) on
 * stream streams[j]; zeta and rand_ratio are shared.  An update is a chain of about fifteen small
 * kernels that depend on one another; the chains of different layers are independent, so on
 * different streams they run side by side, and issued from one native call the host keeps up
 * with them (issued call by call from an interpreter the host is the bound).  The layers, their
 * workspaces and score buffers must be distinct; streams may repeat (those layers then follow
 * one another).  Every argument of every layer is checked before any device work; a failure of a
 * later step (MST_ERR_HIP) leaves the earlier layers updated.  stats_out (host, [n_layers]) may be
 * NULL.  Results per layer are those of the single-layer call, bit for bit. */
int mst_mask_update_from_scores_multi(int n_layers, mst_layer_t* const* layers, const float* const* G_dev,
                                      const double* target_density, double zeta, double rand_ratio,
                                      const uint64_t* rng_seed, void* const* ws_dev, const size_t* ws_bytes,
                                      mst_update_stats* stats_out, const mst_stream_t* streams);

/* The same with the score computed inside: G = dY^T X on the matrix cores. */
int mst_mask_update(mst_layer_t* layer, const void* dY_dev, const void* X_dev, int T,
                    mst_dtype act, double target_density, double zeta, double rand_ratio,
                    uint64_t rng_seed, void* ws_dev, size_t ws_bytes,
                    mst_update_stats* stats_out, mst_stream_t stream);

/* The weight gradient and the update of one step from ONE dense gradient.  On a step that
 * updates the topology the dense gradient G = dY^T X is needed anyway (Sec. 2, Algorithm 1's
 * gradient-based growth); this call forms it once on the matrix cores, writes
 * dW_vals_dev = G at the positions active BEFORE the update (canonical order, the result of
 * mst_sparse_fc_bwd_weight up to rounding order) and then performs mst_mask_update with it.
 * When the update needs no gradient (nothing grows by gradient and the prune score has no
 * gradient term) the weight gradient is computed as in mst_sparse_fc_bwd_weight.
 * ORDER CONTRACT: on return mst_layer_values / mst_layer_indices already describe the NEW
 * topology, while dW_vals_dev (nnz_before entries) is in the order of the OLD one.  A caller
 * that applies this gradient, or carries per-weight optimiser state across the update, must
 * save mst_layer_indices before the call and match flat indices afterwards (pruned positions
 * drop out, grown ones start from zero state); a caller that simply skips the optimiser step
 * on update steps needs nothing.
 * Workspace: mst_workspace_bytes(O, I, nnz_capacity, T). */
int mst_sparse_fc_bwd_weight_update(mst_layer_t* layer, const void* dY_dev, const void* X_dev,
                                    float* dW_vals_dev, int T, mst_dtype act,
                                    double target_density, double zeta, double rand_ratio,
                                    uint64_t rng_seed, void* ws_dev, size_t ws_bytes,
                                    mst_update_stats* stats_out, mst_stream_t stream);

/* ------------------------------------------------------------------ schedule */

/* Pure host.  Density d_t = 1 - S_t of Sec. 3.1 read with stage index
 * k = min(N, floor(t_phase / Delta)):
 *   warm-up      t <  T_W:            d = d_min + (1 - d_min)(1 - k/N)^3
 *   ultra        t <  T_W + T_U:      d = d_min = 1 - S_M
 *   restoration  t <  T_W + T_U + T_R: d = 1 + (d_min - 1)(1 - k/N)^3
 *   afterwards                        d = 1
 * and the update fraction of Sec. 3.2,
 *   zeta_t = zeta_i / 2 (1 + cos(pi (t - T_{i-1}) / (T_i - T_{i-1}))),  t in [T_{i-1}, T_i),
 *   T_0 = 0, T_1 = T_W + T_U, T_{j+1} = T_W + T_U + j Delta_R; 0 from T_{N+1} on.
 * Either output pointer may be NULL. */
int mst_schedule_density(const mst_schedule_cfg* cfg, int64_t step,
                         double* density_out, double* zeta_out);

/* Pure host.  Whether `step` carries a topology update: every Delta_t-th step after step 0
 * (Sec. 3.2; Table "Private hyperparameters of MST": Delta_t = 100).  1 = yes, 0 = no,
 * MST_ERR_ARG for step < 0 or delta_t < 1. */
int mst_update_due(int64_t step, int64_t delta_t);

/* Pure host.  The rng_seed of layer `layer` (0-based, of n_layers) at `step` for a run seeded
 * with run_seed: run_seed + step * n_layers + layer modulo 2^64, distinct per (step, layer). */
uint64_t mst_update_seed(uint64_t run_seed, int64_t step, int32_t n_layers, int32_t layer);

/* ------------------------------------------------------ per-layer densities */

/* Pure host.  Sec. 3.2: the network's density d is spread over the layers by the
 * Erdos-Renyi strategy,
 *   d_l = min(1, eps (I_l + O_l) / (I_l O_l)),   sum_l d_l I_l O_l = d sum_l I_l O_l,
 * a layer whose share would exceed 1 being dense and eps solved for the others.
 * O, I, density_out: host arrays of n_layers entries (the caller's list decides which
 * layers take part).  The densities feed the target_density argument of the update
 * calls, whose count rule turns them into integers.
 * MST_ERR_ARG: null pointer, n_layers < 1, a dimension < 1, d outside [0, 1]. */
int mst_erdos_renyi_density(int n_layers, const int* O, const int* I, double global_density,
                            double* density_out);

/* ------------------------------------------------------------- FLOP counts */

/* Pure host.  App. "FLOP Calculation", Eq. (1): forward FLOPs of the layers for one
 * token, sum_l (1 - S_l)(2 I_l - 1) O_l with S_l = 1 - density[l]. */
int mst_flops_fc_forward(int n_layers, const int* O, const int* I, const double* density,
                         double* flops_out);

typedef struct {
    int64_t L;             /* input sequence length */
    int64_t N_embd;        /* embedding dimensionality */
    int64_t D_ffw;         /* feed-forward size (commonly 4 N_embd) */
    int64_t D_vocab;       /* vocabulary size */
    int64_t n_layers;      /* model depth */
} mst_transformer_shape;

typedef struct {
    double kqv, scores, reduce, proj, ffw1, ffw2, lm;   /* one block's terms; lm once */
    double forward, backward, total;                    /* whole model, one sequence */
} mst_transformer_flops;

/* Pure host.  The seven terms of the same appendix for one sequence, with sparsity
 * S = 1 - density on every fully-connected term (the output layer included) and the
 * attention ratio q_atten on the two attention products; the second of them is read as
 * 2 L L N_embd (all heads together).  forward = n_layers (attention + MLP) + lm,
 * backward = 2 forward, total = forward + backward.
 * MST_ERR_ARG: null pointer, a size < 1, density or q_atten outside [0, 1]. */
int mst_flops_transformer(const mst_transformer_shape* shape, double density, double q_atten,
                          mst_transformer_flops* out);

/* --------------------------------------------- strided attention pattern */

/* Sec. 3.3, unfactorized strided sparse self-attention shared by all heads: output i
 * attends to the previous `stride` positions and to every stride-th position before it,
 *   S_i = { max(i - l + 1, 0), ..., i }  union  { j <= i : (i - j) mod l = 0 }
 * (the text's description; the printed intersection is taken to be a misprint).
 * Writes M_dev [L x L] bytes, row-major, M[i][j] = 1 iff j in S_i.  1 <= L <= 32768,
 * stride >= 1.  Asynchronous on `stream`. */
int mst_strided_attention_mask(uint8_t* M_dev, int L, int stride, mst_stream_t stream);

/* Pure host.  Number of (i, j) pairs the pattern keeps; Q_atten of the appendix's
 * pattern table is this count over L * L. */
int mst_strided_attention_count(int L, int stride, int64_t* count_out);

#ifdef __cplusplus
}
#endif
#endif /* MST_H */
