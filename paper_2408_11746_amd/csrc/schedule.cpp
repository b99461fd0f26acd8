// Host-only parts of the C ABI: the Sparsity Variation density schedule (Sec. 3.1),
// the piecewise cosine update fraction (Sec. 3.2), the count lines of Algorithm 1, the
// per-layer density allocation (Sec. 3.2), the FLOP counts (App. "FLOP Calculation") and
// the size of the strided attention pattern (Sec. 3.3).
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "../../include/mst.h"

extern "C" {

const char* mst_version(void) { return "mst-hip 0.1 (gfx950)"; }

int mst_schedule_density(const mst_schedule_cfg* cfg, int64_t step, double* density_out,
                         double* zeta_out) {
    if (!cfg || step < 0) return MST_ERR_ARG;
    if (cfg->N < 1 || cfg->Delta_W < 1 || cfg->Delta_R < 1 || cfg->T_U < 0) return MST_ERR_ARG;
    if (!(cfg->S_M >= 0.0 && cfg->S_M <= 1.0)) return MST_ERR_ARG;
    const int64_t N = cfg->N;
    const int64_t T_W = N * cfg->Delta_W, T_R = N * cfg->Delta_R;
    const int64_t t_rest = T_W + cfg->T_U, t_dense = t_rest + T_R;
    const double d_min = 1.0 - cfg->S_M;

    if (density_out) {
        double d;
        if (step < T_W) {
            int64_t k = step / cfg->Delta_W;
            if (k > N) k = N;
            d = d_min + (1.0 - d_min) * std::pow(1.0 - (double)k / (double)N, 3.0);
        } else if (step < t_rest) {
            d = d_min;
        } else if (step < t_dense) {
            int64_t k = (step - t_rest) / cfg->Delta_R;
            if (k > N) k = N;
            d = 1.0 + (d_min - 1.0) * std::pow(1.0 - (double)k / (double)N, 3.0);
        } else {
            d = 1.0;
        }
        *density_out = d;
    }
    if (zeta_out) {
        if (!cfg->zeta || cfg->n_zeta != cfg->N + 1) return MST_ERR_ARG;
        double z = 0.0;
        if (step < t_dense) {
            // period i = 1 is [0, T_W + T_U); period j + 1 is one restoration stage
            int64_t lo, hi;
            int idx;
            if (step < t_rest) {
                lo = 0; hi = t_rest; idx = 0;
            } else {
                int64_t j = (step - t_rest) / cfg->Delta_R;       // 0 .. N-1
                lo = t_rest + j * cfg->Delta_R; hi = lo + cfg->Delta_R; idx = (int)j + 1;
            }
            const double pi = 3.14159265358979323846;
            z = 0.5 * cfg->zeta[idx] * (1.0 + std::cos(pi * (double)(step - lo) / (double)(hi - lo)));
        }
        *zeta_out = z;
    }
    return MST_OK;
}

// Sec. 3.2 / Table "Private hyperparameters of MST": the topology is updated every Delta_t
// steps (100); step 0 holds the initial topology and is no update step.
int mst_update_due(int64_t step, int64_t delta_t) {
    if (step < 0 || delta_t < 1) return MST_ERR_ARG;
    return (step > 0 && step % delta_t == 0) ? 1 : 0;
}

// one seed per (step, layer) for the random growth of Algorithm 1, arithmetic modulo 2^64
uint64_t mst_update_seed(uint64_t run_seed, int64_t step, int32_t n_layers, int32_t layer) {
    return run_seed + (uint64_t)step * (uint64_t)n_layers + (uint64_t)layer;
}

int mst_update_counts(int64_t n_total, int64_t nnz, double target_density, double zeta,
                      double rand_ratio, mst_update_stats* out) {
    if (!out || n_total < 1 || nnz < 0 || nnz > n_total) return MST_ERR_ARG;
    if (!(target_density >= 0.0 && target_density <= 1.0)) return MST_ERR_ARG;
    if (!(zeta >= 0.0 && zeta <= 1.0) || !(rand_ratio >= 0.0 && rand_ratio <= 1.0)) return MST_ERR_ARG;
    const int64_t target = (int64_t)std::floor(target_density * (double)n_total + 0.5);
    int64_t n_prune = (int64_t)std::floor(zeta * (double)nnz);
    int64_t n_grow = n_prune + (target - nnz);
    if (n_grow < 0) {                    // shrinking faster than zeta allows: prune only
        n_prune = nnz - target;
        n_grow = 0;
    }
    if (n_grow > n_total - nnz) {        // not enough empty positions: fill all of them
        n_grow = n_total - nnz;
        n_prune = n_grow - (target - nnz);
    }
    out->nnz_before = nnz;
    out->nnz_after = target;
    out->n_prune = n_prune;
    out->n_grow = n_grow;
    out->n_rand = (int64_t)std::floor((double)n_grow * rand_ratio);
    out->n_grad = n_grow - out->n_rand;
    return MST_OK;
}

// Erdos-Renyi allocation.  The kept budget sum_l min(1, eps r_l) N_l, r_l = (I_l + O_l) / N_l,
// grows with eps and the layers saturate in the order of decreasing r_l: walk that order,
// and with the first k layers dense take eps from the rest, until the next layer fits.
int mst_erdos_renyi_density(int n_layers, const int* O, const int* I, double global_density,
                            double* density_out) {
    if (n_layers < 1 || !O || !I || !density_out) return MST_ERR_ARG;
    if (!(global_density >= 0.0 && global_density <= 1.0)) return MST_ERR_ARG;
    for (int l = 0; l < n_layers; ++l)
        if (O[l] < 1 || I[l] < 1) return MST_ERR_ARG;
    std::vector<double> n(n_layers), r(n_layers);
    double total = 0.0, edges = 0.0;
    for (int l = 0; l < n_layers; ++l) {
        n[l] = (double)O[l] * (double)I[l];
        r[l] = ((double)O[l] + (double)I[l]) / n[l];
        total += n[l];
        edges += (double)O[l] + (double)I[l];
    }
    if (global_density == 1.0 || global_density == 0.0) {
        std::fill(density_out, density_out + n_layers, global_density);
        return MST_OK;
    }
    std::vector<int> order(n_layers);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return r[a] > r[b]; });
    double budget = global_density * total;
    int k = 0;
    double eps = 0.0;
    for (; k < n_layers; ++k) {
        eps = budget / edges;
        if (eps * r[order[k]] <= 1.0) break;     // the layer most eager to saturate fits
        budget -= n[order[k]];
        edges -= (double)O[order[k]] + (double)I[order[k]];
    }
    for (int j = 0; j < n_layers; ++j) {
        const int l = order[j];
        density_out[l] = (j < k) ? 1.0 : std::min(1.0, std::max(0.0, eps * r[l]));   // rounding guard
    }
    return MST_OK;
}

int mst_flops_fc_forward(int n_layers, const int* O, const int* I, const double* density,
                         double* flops_out) {
    if (n_layers < 1 || !O || !I || !density || !flops_out) return MST_ERR_ARG;
    double sum = 0.0;
    for (int l = 0; l < n_layers; ++l) {
        if (O[l] < 1 || I[l] < 1 || !(density[l] >= 0.0 && density[l] <= 1.0)) return MST_ERR_ARG;
        sum += density[l] * (2.0 * (double)I[l] - 1.0) * (double)O[l];
    }
    *flops_out = sum;
    return MST_OK;
}

int mst_flops_transformer(const mst_transformer_shape* shape, double density, double q_atten,
                          mst_transformer_flops* out) {
    if (!shape || !out) return MST_ERR_ARG;
    if (shape->L < 1 || shape->N_embd < 1 || shape->D_ffw < 1 || shape->D_vocab < 1 || shape->n_layers < 1)
        return MST_ERR_ARG;
    if (!(density >= 0.0 && density <= 1.0) || !(q_atten >= 0.0 && q_atten <= 1.0)) return MST_ERR_ARG;
    const double L = (double)shape->L, E = (double)shape->N_embd, F = (double)shape->D_ffw;
    const double V = (double)shape->D_vocab, depth = (double)shape->n_layers;
    const double row_e = density * L * (2.0 * E - 1.0);      // (1 - S) L (2 N_embd - 1): one output of width N_embd
    out->kqv = row_e * 3.0 * E;
    out->proj = row_e * E;
    out->ffw1 = row_e * F;
    out->ffw2 = density * L * (2.0 * F - 1.0) * E;
    out->lm = row_e * V;
    out->scores = q_atten * 2.0 * L * L * E;
    out->reduce = out->scores;
    out->forward = depth * (out->kqv + out->scores + out->reduce + out->proj + out->ffw1 + out->ffw2) + out->lm;
    out->backward = 2.0 * out->forward;
    out->total = out->forward + out->backward;
    return MST_OK;
}

// Row i keeps its window, min(i + 1, l) positions, and the positions i - l, i - 2l, ... >= 0
// outside it: floor(i / l) of them.  Summed over the rows in closed form.
int mst_strided_attention_count(int L, int stride, int64_t* count_out) {
    if (L < 1 || stride < 1 || !count_out) return MST_ERR_ARG;
    const int64_t n = L, l = stride;
    const int64_t ramp = std::min(n, l);                     // rows 0 .. ramp-1 see i + 1 positions
    int64_t window = ramp * (ramp + 1) / 2 + (n - ramp) * l;
    const int64_t q = (n - 1) / l;                           // floor(i / l) takes 0 .. q
    // every value v < q is taken by l rows, v = q by the last n - q l rows
    int64_t strided = l * (q * (q - 1) / 2) + q * (n - q * l);
    *count_out = window + strided;
    return MST_OK;
}

}  // extern "C"
