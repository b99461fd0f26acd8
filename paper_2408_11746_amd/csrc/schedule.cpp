// Host-only parts of the C ABI: the Sparsity Variation density schedule (Sec. 3.1),
// the piecewise cosine update fraction (Sec. 3.2) and the count lines of Algorithm 1.
#include <cmath>

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

}  // extern "C"
