// Load-balancing placement of experts on devices (paper Sec. 7).  Host logic only -- no HIP call.
//
// Historical activation A[m][b] = fraction of batch b's tokens that went to expert m.  Every device
// gets E / D experts.  Experts are walked in descending order of their average load (equal loads:
// lower id first); each goes to the device that offers the smallest load (equal: lower device id),
// and a device that is full leaves the candidates.
//   greedy (Sec. 7.1):           load of device n = sum over its experts m of mean[m]
//   anti-correlation (Sec. 7.2): load of device n for expert a = sum over its experts m of
//                                mean[m] + w * S[a][m],  S = Pearson correlation of the historical
//                                activations, w = 0.5 in the paper
// The objective as printed in the paper is garbled; what its text describes is implemented: keep
// every device's share  sum_m P[m][n] A[m][b]  of every batch near 1 / D.
// Sums run in index order in double precision.
#include <algorithm>
#include <cmath>
#include <vector>

#include "moe_internal.h"

namespace moe355 {

static void mean_rows(const float *A, int E, int B, std::vector<double> &mu)
{
    mu.assign(E, 0.0);
    for (int m = 0; m < E; ++m) {
        double s = 0.0;
        for (int b = 0; b < B; ++b) s += (double)A[(size_t)m * B + b];
        mu[m] = B > 0 ? s / B : 0.0;
    }
}

static int place(const float *A, int E, int B, int D, double w, int32_t *device_of)
{
    if (!A || !device_of || E < 1 || B < 1 || D < 1 || E % D != 0) {
        set_error("placement: NULL argument, or E = %d does not split evenly over %d devices, or B = %d < 1", E, D, B);
        return MOE_ERR_INVALID_ARG;
    }
    const int cap = E / D;
    std::vector<double> mu;
    mean_rows(A, E, B, mu);
    std::vector<double> S;  // [E][E], only with a correlation weight
    if (w != 0.0) {
        std::vector<double> dev((size_t)E * B), ss(E, 0.0);
        for (int m = 0; m < E; ++m)
            for (int b = 0; b < B; ++b) dev[(size_t)m * B + b] = (double)A[(size_t)m * B + b] - mu[m];
        for (int m = 0; m < E; ++m) {
            double s = 0.0;
            for (int b = 0; b < B; ++b) s += dev[(size_t)m * B + b] * dev[(size_t)m * B + b];
            ss[m] = s;
        }
        S.assign((size_t)E * E, 0.0);
        for (int a = 0; a < E; ++a)
            for (int m = 0; m < E; ++m)
                if (ss[a] > 0.0 && ss[m] > 0.0) {
                    double c = 0.0;
                    for (int b = 0; b < B; ++b) c += dev[(size_t)a * B + b] * dev[(size_t)m * B + b];
                    S[(size_t)a * E + m] = c / std::sqrt(ss[a] * ss[m]);
                }
    }
    std::vector<int> order(E);
    for (int m = 0; m < E; ++m) order[m] = m;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return mu[x] > mu[y]; });
    std::vector<std::vector<int>> members(D);
    for (int a : order) {
        int best = -1;
        double best_load = 0.0;
        for (int n = 0; n < D; ++n) {
            if ((int)members[n].size() >= cap) continue;
            double load = 0.0;
            for (int m : members[n]) load += mu[m] + (w != 0.0 ? w * S[(size_t)a * E + m] : 0.0);
            if (best < 0 || load < best_load) {
                best = n;
                best_load = load;
            }
        }
        members[best].push_back(a);
        device_of[a] = best;
    }
    return MOE_OK;
}

}  // namespace moe355

extern "C" {

int moe_placement_greedy(const float *A, int32_t E, int32_t B, int32_t n_devices, int32_t *device_of)
{
    return moe355::place(A, E, B, n_devices, 0.0, device_of);
}

int moe_placement_anticorrelation(const float *A, int32_t E, int32_t B, int32_t n_devices, double corr_weight,
                                  int32_t *device_of)
{
    return moe355::place(A, E, B, n_devices, corr_weight, device_of);
}

int moe_placement_loads(const float *A, int32_t E, int32_t B, const int32_t *device_of, int32_t n_devices,
                        double *max_load, double *avg_max_load)
{
    if (!A || !device_of || E < 1 || B < 1 || n_devices < 1) {
        moe355::set_error("placement loads: NULL argument or a size below 1");
        return MOE_ERR_INVALID_ARG;
    }
    for (int m = 0; m < E; ++m)
        if (device_of[m] < 0 || device_of[m] >= n_devices) {
            moe355::set_error("placement loads: device_of[%d] = %d outside [0,%d)", m, device_of[m], n_devices);
            return MOE_ERR_INVALID_ARG;
        }
    std::vector<double> dev(n_devices);
    double worst = 0.0, acc = 0.0;
    for (int b = 0; b < B; ++b) {
        std::fill(dev.begin(), dev.end(), 0.0);
        for (int m = 0; m < E; ++m) dev[device_of[m]] += (double)A[(size_t)m * B + b];
        const double mx = *std::max_element(dev.begin(), dev.end());
        worst = std::max(worst, mx);
        acc += mx;
    }
    if (max_load) *max_load = worst;
    if (avg_max_load) *avg_max_load = acc / B;
    return MOE_OK;
}

}  // extern "C"
