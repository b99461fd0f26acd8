// The C-ABI entry points that launch device work: argument checks on the host, then
// dispatch to the sparse kernels or, for dense layers, to the masked dense MFMA path.
#include <mutex>

#include "common.h"

namespace mst {

// ---- scratch of the entry point that allocates nothing (mst_sparse_fc_bwd_weight_static):
// the SDDMM's per-token-tile partial sums live in this file-scope device array instead of a
// caller workspace.  Each GPU the library runs on holds its own copy at its own address until
// the process ends; host code never uses the array's name as an address, only the pointer
// hipGetSymbolAddress returns for the current device.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES] = {};
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device, looked up once per device
static int static_scratch(void** out) {
    int dev = -1;
    MST_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return MST_ERR_STATE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        MST_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return MST_ERR_STATE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MST_OK;
}

// out[k] = sum over the nparts partial outputs (stride apart, added in ascending order) at
// the k-th active position: the split sum of the dense gradient is only formed where the
// weight gradient is wanted
// (a thread takes four consecutive active positions: one 16-byte read of their indices, the four
// gathers of a part in flight together, one 16-byte store; flat and out are 16-byte aligned)
__global__ void k_gather_flat(const float* __restrict__ G, int64_t stride, int nparts, const int* __restrict__ flat,
                              int64_t nnz, float* __restrict__ out) {
    const int64_t k = 4 * ((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
    if (k >= nnz) return;
    if (k + 4 <= nnz) {
        const int4 f = *reinterpret_cast<const int4*>(flat + k);
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int z = 0; z < nparts; ++z) {
            const float* g = G + (int64_t)z * stride;
            const float a = g[f.x], b = g[f.y], c = g[f.z], d = g[f.w];
            sum.x += a;
            sum.y += b;
            sum.z += c;
            sum.w += d;
        }
        *reinterpret_cast<float4*>(out + k) = sum;
        return;
    }
    for (int64_t i = k; i < nnz; ++i) {
        const float* g = G + flat[i];
        float sum = 0.f;
        for (int z = 0; z < nparts; ++z) sum += g[(int64_t)z * stride];
        out[i] = sum;
    }
}

static int ensure_dense_copy(const mst_layer* L, hipStream_t s) {
    if (L->Wd_valid) return MST_OK;
    return refresh_dense_copy(const_cast<mst_layer*>(L), s);   // cache of vals[], not layer state
}

// (split_ws: room for partial outputs of a split of the contraction range, used where the output
// has too few tiles to fill the chip; null: one workgroup per tile whatever their number)
int dense_products_fwd(const mst_layer* L, const void* X, float* Y, int T, mst_dtype act, hipStream_t s,
                       float* split_ws, int64_t split_ws_floats) {
    int rc = ensure_dense_copy(L, s);
    if (rc != MST_OK) return rc;
    return gemm_mfma(GEMM_NT, X, act, L->Wd, MST_F32, Y, T, L->O, L->I, split_ws, split_ws_floats, s);
}

int dense_products_bwd_input(const mst_layer* L, const void* dY, float* dX, int T, mst_dtype act, hipStream_t s,
                             float* split_ws, int64_t split_ws_floats) {
    int rc = ensure_dense_copy(L, s);
    if (rc != MST_OK) return rc;
    return gemm_mfma(GEMM_NN, dY, act, L->Wd, MST_F32, dX, T, L->I, L->O, split_ws, split_ws_floats, s);
}

int dense_products_bwd_weight(const mst_layer* L, const void* dY, const void* X, float* dW, int T,
                              mst_dtype act, const Workspace& ws, hipStream_t s) {
    int nparts = 1;
    int rc = gemm_mfma(GEMM_TN, dY, act, X, act, ws.G, L->O, L->I, T, ws.gemm, (int64_t)ws.gemm_floats, s, &nparts);
    if (rc != MST_OK) return rc;
    if (L->nnz > 0) {
        k_gather_flat<<<(unsigned)cdiv(L->nnz, 1024), 256, 0, s>>>(nparts > 1 ? ws.gemm : ws.G, L->N, nparts, L->flat,
                                                                  L->nnz, dW);
        MST_LAUNCH_CHECK();
    }
    return MST_OK;
}

static bool act_ok(mst_dtype a) { return a == MST_F32 || a == MST_BF16; }

// remembered for the next update's decision whether the index views will be walked
static void note_call(const mst_layer* L, mst_dtype act, int T) {
    mst_layer* m = const_cast<mst_layer*>(L);
    m->hint_T = T;
    m->hint_act = (int)act;
}

}  // namespace mst

using namespace mst;

extern "C" {

int mst_spmm_force_shape(int tokens_per_workgroup, int quads_per_wavefront) {
    return spmm_force_shape(tokens_per_workgroup, quads_per_wavefront);
}

int mst_gemm_force_fp32_mfma(int on) { return gemm_force_fp32_mfma(on); }

int mst_gemm_last_tile(void) { return gemm_last_tile(); }

int mst_heavy_rows(int on) { return heavy_rows_enable(on); }

int mst_bwd_force_shape(int wavefronts_per_workgroup, int quads_per_wavefront) {
    return bwd_fused_force_shape(wavefronts_per_workgroup, quads_per_wavefront);
}

int mst_sparse_fc_fwd(const mst_layer_t* L, const void* X_dev, float* Y_dev, int T, mst_dtype act,
                      mst_stream_t stream) {
    if (!L || !X_dev || !Y_dev || T < 1 || !act_ok(act) || !aligned16(X_dev) || !aligned16(Y_dev)) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    hipStream_t s = (hipStream_t)stream;
    note_call(L, act, T);
    // (unbuilt views and no workspace to build them with: the dense product, same result within tolerance)
    if (use_dense_path(L, act, T) || !L->views_valid) return dense_products_fwd(L, X_dev, Y_dev, T, act, s);
    const int rc = spmm(L->row, X_dev, Y_dev, T, L->nnz, act, s);
    if (rc != MST_OK || !L->heavy_on) return rc;
    return heavy_fwd(L, X_dev, Y_dev, T, act, s);        // the rows the view leaves out (returns at once without any)
}

int mst_sparse_fc_bwd_input(const mst_layer_t* L, const void* dY_dev, float* dX_dev, int T, mst_dtype act,
                            mst_stream_t stream) {
    if (!L || !dY_dev || !dX_dev || T < 1 || !act_ok(act) || !aligned16(dY_dev) || !aligned16(dX_dev)) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    hipStream_t s = (hipStream_t)stream;
    note_call(L, act, T);
    if (use_dense_path(L, act, T) || !L->views_valid) return dense_products_bwd_input(L, dY_dev, dX_dev, T, act, s);
    return spmm(L->col, dY_dev, dX_dev, T, L->nnz, act, s);
}

int mst_sparse_fc_bwd_weight(const mst_layer_t* L, const void* dY_dev, const void* X_dev, float* dW_dev, int T,
                             mst_dtype act, void* ws_dev, size_t ws_bytes, mst_stream_t stream) {
    if (!L || !dY_dev || !X_dev || !dW_dev || !ws_dev || T < 1 || !act_ok(act)) return MST_ERR_ARG;
    if (!aligned16(dY_dev) || !aligned16(X_dev) || !aligned16(dW_dev) || !aligned16(ws_dev)) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    const Workspace ws = carve_workspace(ws_dev, L->O, L->I, L->cap, T);
    if (ws_bytes < ws.total) return MST_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    note_call(L, act, T);
    if (use_dense_weight_grad(L, act, T)) return dense_products_bwd_weight(L, dY_dev, X_dev, dW_dev, T, act, ws, s);
    const int rc = ensure_views(L, ws, s);
    if (rc != MST_OK) return rc;
    return sddmm(L, dY_dev, X_dev, dW_dev, T, act, ws, s);
}

size_t mst_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int mst_sparse_fc_bwd_weight_static(const mst_layer_t* L, const void* dY_dev, const void* X_dev, float* dW_dev, int T,
                                    mst_dtype act, mst_stream_t stream) {
    if (!L || !dY_dev || !X_dev || !dW_dev || T < 1 || !act_ok(act)) return MST_ERR_ARG;
    if (!aligned16(dY_dev) || !aligned16(X_dev) || !aligned16(dW_dev)) return MST_ERR_ARG;
    if (!L->built || !L->views_valid) return MST_ERR_STATE;      // (it has no workspace to build unbuilt views with)
    // partial sums: one plane of entry slots per tile of TT tokens; the plane's stride is that of
    // the larger view because the view that drives the product is chosen on the device
    const size_t slots = (size_t)std::max(L->row.cap_pairs, L->col.cap_pairs) * 8;
    const size_t need = (size_t)cdiv(T, TT) * slots * sizeof(float);
    if (need > STATIC_SCRATCH_BYTES) return MST_ERR_WORKSPACE;
    void* base = nullptr;
    const int rc = static_scratch(&base);
    if (rc != MST_OK) return rc;
    Workspace ws{};
    ws.partial = static_cast<float*>(base);      // every slot the second kernel reads is written by the first
    ws.partial_floats = STATIC_SCRATCH_BYTES / sizeof(float);
    return sddmm(L, dY_dev, X_dev, dW_dev, T, act, ws, (hipStream_t)stream);
}

int mst_sparse_fc_bwd(const mst_layer_t* L, const void* dY_dev, const void* X_dev, float* dX_dev, float* dW_dev,
                      int T, mst_dtype act, void* ws_dev, size_t ws_bytes, mst_stream_t stream) {
    if (!L || !dY_dev || !X_dev || !dX_dev || !dW_dev || !ws_dev || T < 1 || !act_ok(act)) return MST_ERR_ARG;
    if (!aligned16(dY_dev) || !aligned16(X_dev) || !aligned16(dX_dev) || !aligned16(dW_dev) || !aligned16(ws_dev))
        return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    const Workspace ws = carve_workspace(ws_dev, L->O, L->I, L->cap, T);
    if (ws_bytes < ws.total) return MST_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    note_call(L, act, T);
    if (use_fused_backward(L, act, T) && bwd_fused_pays(L)) {
        const int rcv = ensure_views(L, ws, s);
        if (rcv != MST_OK) return rcv;
        return bwd_fused(L, dY_dev, X_dev, dX_dev, dW_dev, T, act, ws, s);
    }
    // the two dense contractions (the split area of the workspace serves dX first, then the weight
    // gradient: same stream)
    const int rc = dense_products_bwd_input(L, dY_dev, dX_dev, T, act, s, ws.gemm, (int64_t)ws.gemm_floats);
    if (rc != MST_OK) return rc;
    return dense_products_bwd_weight(L, dY_dev, X_dev, dW_dev, T, act, ws, s);
}

int mst_layer_uses_dense(const mst_layer_t* L, mst_dtype act, int T, int weight_gradient) {
    if (!L || !act_ok(act) || T < 1) return MST_ERR_ARG;
    // Y and dX have no workspace to build unbuilt views with: they then run dense whatever the density
    if (weight_gradient == 2) return use_fused_backward(L, act, T) ? 0 : 1;
    return (weight_gradient ? use_dense_weight_grad(L, act, T) : (use_dense_path(L, act, T) || !L->views_valid)) ? 1 : 0;
}

int mst_gather_active(const mst_layer_t* L, const float* G_dev, float* dW_dev, mst_stream_t stream) {
    if (!L || !G_dev || !dW_dev || !aligned16(G_dev) || !aligned16(dW_dev)) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    if (L->nnz > 0) {
        k_gather_flat<<<(unsigned)cdiv(L->nnz, 1024), 256, 0, (hipStream_t)stream>>>(G_dev, L->N, 1, L->flat, L->nnz, dW_dev);
        MST_LAUNCH_CHECK();
    }
    return MST_OK;
}

int mst_layer_format_stats(const mst_layer_t* L, mst_format_stats* out, mst_stream_t stream) {
    if (!L || !out) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    hipStream_t s = (hipStream_t)stream;
    if (!L->views_valid) {                            // unbuilt (layer on the dense contractions): nothing stored
        out->nnz = L->nnz;
        out->row_view_slots = out->col_view_slots = 0;
        out->row_view_efficiency = out->col_view_efficiency = 0.0;
        out->heavy_rows = out->heavy_entries = 0;
        return MST_OK;
    }
    int pr = 0, pc = 0, hv[2] = {0, 0};
    MST_HIP(hipMemcpyAsync(&pr, L->row.ptr + L->row.nseg, 4, hipMemcpyDeviceToHost, s));
    MST_HIP(hipMemcpyAsync(&pc, L->col.ptr + L->col.nseg, 4, hipMemcpyDeviceToHost, s));
    if (L->heavy_on) {
        MST_HIP(hipMemcpyAsync(&hv[0], L->heavy, 4, hipMemcpyDeviceToHost, s));
        MST_HIP(hipMemcpyAsync(&hv[1], L->heavy + HEAVY_MAX + 1, 4, hipMemcpyDeviceToHost, s));
    }
    MST_HIP(hipStreamSynchronize(s));
    out->nnz = L->nnz;
    out->heavy_rows = hv[0];
    out->heavy_entries = hv[1];
    out->row_view_slots = (int64_t)pr * 8;
    out->col_view_slots = (int64_t)pc * 8;
    out->row_view_efficiency = pr ? (double)(L->nnz - hv[1]) / (double)out->row_view_slots : 1.0;
    out->col_view_efficiency = pc ? (double)L->nnz / (double)out->col_view_slots : 1.0;
    return MST_OK;
}

int mst_dense_grad(const void* dY_dev, const void* X_dev, float* G_dev, int T, int O, int I, mst_dtype act,
                   void* ws_dev, size_t ws_bytes, mst_stream_t stream) {
    if (!dY_dev || !X_dev || !G_dev || T < 1 || O < 1 || I < 1 || !act_ok(act)) return MST_ERR_ARG;
    if (!aligned16(dY_dev) || !aligned16(X_dev) || !aligned16(G_dev) || (ws_dev && !aligned16(ws_dev))) return MST_ERR_ARG;
    return gemm_mfma(GEMM_TN, dY_dev, act, X_dev, act, G_dev, O, I, T, (float*)ws_dev,
                     ws_dev ? (int64_t)(ws_bytes / 4) : 0, (hipStream_t)stream);
}

// the dense gradient scores gradient growth and, with a prune score that has a gradient
// term, pruning; an update that does neither does not need it
static bool needs_gradient(const mst_layer* L, const mst_update_stats& st) {
    return st.n_grad > 0 || (L->prune_lambda != 0.f && st.n_prune > 0);
}

static int update_common(mst_layer_t* L, const float* G, uint64_t seed, const Workspace& ws,
                         mst_update_stats* stats_out, hipStream_t s, const mst_update_stats& st) {
    if (stats_out) *stats_out = st;
    if (st.n_prune == 0 && st.n_grow == 0) return MST_OK;     // nothing moves
    return mask_update_device(L, G, st, seed, ws, s);
}

int mst_mask_update_from_scores(mst_layer_t* L, const float* G_dev, double target_density, double zeta,
                                double rand_ratio, uint64_t rng_seed, void* ws_dev, size_t ws_bytes,
                                mst_update_stats* stats_out, mst_stream_t stream) {
    if (!L || !G_dev || !ws_dev || !aligned16(G_dev) || !aligned16(ws_dev)) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    mst_update_stats st;
    int rc = mst_update_counts(L->N, L->nnz, target_density, zeta, rand_ratio, &st);
    if (rc != MST_OK) return rc;
    if (st.nnz_after > L->cap) return MST_ERR_STATE;
    const Workspace ws = carve_workspace(ws_dev, L->O, L->I, L->cap, 1);
    if (ws_bytes < ws.total) return MST_ERR_WORKSPACE;
    return update_common(L, G_dev, rng_seed, ws, stats_out, (hipStream_t)stream, st);
}

int mst_mask_update_from_scores_multi(int n_layers, mst_layer_t* const* layers, const float* const* G_dev,
                                      const double* target_density, double zeta, double rand_ratio,
                                      const uint64_t* rng_seed, void* const* ws_dev, const size_t* ws_bytes,
                                      mst_update_stats* stats_out, const mst_stream_t* streams) {
    if (n_layers < 0 || (n_layers > 0 && (!layers || !G_dev || !target_density || !rng_seed || !ws_dev || !ws_bytes || !streams)))
        return MST_ERR_ARG;
    // everything that can be refused is refused before the first launch
    for (int j = 0; j < n_layers; ++j) {
        mst_layer_t* L = layers[j];
        if (!L || !G_dev[j] || !ws_dev[j] || !aligned16(G_dev[j]) || !aligned16(ws_dev[j])) return MST_ERR_ARG;
        for (int u = 0; u < j; ++u)
            if (layers[u] == L || ws_dev[u] == ws_dev[j] || G_dev[u] == G_dev[j]) return MST_ERR_ARG;
        if (!L->built) return MST_ERR_STATE;
        mst_update_stats st;
        const int rc = mst_update_counts(L->N, L->nnz, target_density[j], zeta, rand_ratio, &st);
        if (rc != MST_OK) return rc;
        if (st.nnz_after > L->cap) return MST_ERR_STATE;
        if (ws_bytes[j] < carve_workspace(nullptr, L->O, L->I, L->cap, 1).total) return MST_ERR_WORKSPACE;
    }
    for (int j = 0; j < n_layers; ++j) {
        const int rc = mst_mask_update_from_scores(layers[j], G_dev[j], target_density[j], zeta, rand_ratio, rng_seed[j],
                                                   ws_dev[j], ws_bytes[j], stats_out ? stats_out + j : nullptr, streams[j]);
        if (rc != MST_OK) return rc;
    }
    return MST_OK;
}

int mst_mask_update(mst_layer_t* L, const void* dY_dev, const void* X_dev, int T, mst_dtype act,
                    double target_density, double zeta, double rand_ratio, uint64_t rng_seed, void* ws_dev,
                    size_t ws_bytes, mst_update_stats* stats_out, mst_stream_t stream) {
    if (!L || !dY_dev || !X_dev || !ws_dev || T < 1 || !act_ok(act)) return MST_ERR_ARG;
    if (!aligned16(dY_dev) || !aligned16(X_dev) || !aligned16(ws_dev)) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    mst_update_stats st;
    int rc = mst_update_counts(L->N, L->nnz, target_density, zeta, rand_ratio, &st);
    if (rc != MST_OK) return rc;
    if (st.nnz_after > L->cap) return MST_ERR_STATE;
    const Workspace ws = carve_workspace(ws_dev, L->O, L->I, L->cap, 1);
    if (ws_bytes < ws.total) return MST_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    note_call(L, act, T);
    if (needs_gradient(L, st)) {
        rc = gemm_mfma(GEMM_TN, dY_dev, act, X_dev, act, ws.G, L->O, L->I, T, ws.gemm, (int64_t)ws.gemm_floats, s);
        if (rc != MST_OK) return rc;
    }
    return update_common(L, ws.G, rng_seed, ws, stats_out, s, st);
}

int mst_sparse_fc_bwd_weight_update(mst_layer_t* L, const void* dY_dev, const void* X_dev, float* dW_dev, int T,
                                    mst_dtype act, double target_density, double zeta, double rand_ratio,
                                    uint64_t rng_seed, void* ws_dev, size_t ws_bytes, mst_update_stats* stats_out,
                                    mst_stream_t stream) {
    if (!L || !dY_dev || !X_dev || !dW_dev || !ws_dev || T < 1 || !act_ok(act)) return MST_ERR_ARG;
    if (!aligned16(dY_dev) || !aligned16(X_dev) || !aligned16(dW_dev) || !aligned16(ws_dev)) return MST_ERR_ARG;
    if (!L->built) return MST_ERR_STATE;
    mst_update_stats st;
    int rc = mst_update_counts(L->N, L->nnz, target_density, zeta, rand_ratio, &st);
    if (rc != MST_OK) return rc;
    if (st.nnz_after > L->cap) return MST_ERR_STATE;
    const Workspace ws = carve_workspace(ws_dev, L->O, L->I, L->cap, T);
    if (ws_bytes < ws.total) return MST_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    note_call(L, act, T);
    if (needs_gradient(L, st)) {
        // one dense gradient serves both: the weight gradient is read from it at the positions
        // that are active now, then the update scores growth with it
        rc = gemm_mfma(GEMM_TN, dY_dev, act, X_dev, act, ws.G, L->O, L->I, T, ws.gemm, (int64_t)ws.gemm_floats, s);
        if (rc != MST_OK) return rc;
        if (L->nnz > 0) {
            k_gather_flat<<<(unsigned)cdiv(L->nnz, 1024), 256, 0, s>>>(ws.G, L->N, 1, L->flat, L->nnz, dW_dev);
            MST_LAUNCH_CHECK();
        }
    } else {
        if (use_dense_weight_grad(L, act, T)) {
            rc = dense_products_bwd_weight(L, dY_dev, X_dev, dW_dev, T, act, ws, s);
        } else {
            rc = ensure_views(L, ws, s);
            if (rc == MST_OK) rc = sddmm(L, dY_dev, X_dev, dW_dev, T, act, ws, s);
        }
        if (rc != MST_OK) return rc;
    }
    return update_common(L, ws.G, rng_seed, ws, stats_out, s, st);
}

}  // extern "C"
