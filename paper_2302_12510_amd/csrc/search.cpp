// Layer-wise bitwidth search (Sec. III-C: Eq. 3, Eq. 4 and the search flow of Alg. 1), host only.
//
// The search works on tables: the latency of every layer in each of the nine (W, A) modes and the
// quantization error (Eq. 2) of every layer's weight and activation tensor at each width.  Where
// the paper consults a cycle-accurate simulator of its accelerator, the caller fills the latency
// table with times measured on the device.
#include <algorithm>
#include <cmath>
#include <vector>

#include "dybit_host.h"

namespace {

constexpr int kLevels = 3;                      // 8, 4, 2 bits (Sec. III-C)
constexpr int kBits[kLevels] = {8, 4, 2};

struct Tables {
    int n;
    const double *lat, *err_w, *err_a;
    double latency(int l, int w, int a) const { return lat[(l * kLevels + w) * kLevels + a]; }
    double error(int l, int w, int a) const { return err_w[l * kLevels + w] + err_a[l * kLevels + a]; }
};

struct Assignment {
    std::vector<int> w, a;                      // level index per layer
    std::vector<int> &table(int which) { return which == 0 ? w : a; }
};

double sum_latency(const Tables &t, const Assignment &s)
{
    double acc = 0.0;
    for (int l = 0; l < t.n; ++l) acc += t.latency(l, s.w[l], s.a[l]);
    return acc;
}

double sum_error(const Tables &t, const Assignment &s)
{
    double acc = 0.0;
    for (int l = 0; l < t.n; ++l) acc += t.error(l, s.w[l], s.a[l]);
    return acc;
}

bool tables_valid(const Tables &t)
{
    for (int i = 0; i < t.n * kLevels * kLevels; ++i)
        if (!(t.lat[i] > 0.0) || !std::isfinite(t.lat[i])) return false;
    for (int i = 0; i < t.n * kLevels; ++i)
        if (!(t.err_w[i] >= 0.0) || !(t.err_a[i] >= 0.0) || !std::isfinite(t.err_w[i]) || !std::isfinite(t.err_a[i]))
            return false;
    return true;
}

}  // namespace

extern "C" dybit_status dybit_search(int32_t n_layers, const double *lat, const double *rmse_w, const double *rmse_a,
                                     int32_t strategy, double constraint, int32_t k,
                                     int32_t *w_bits_out, int32_t *a_bits_out, double *ratio_out, int32_t *met_out)
{
    if (!lat || !rmse_w || !rmse_a || !w_bits_out || !a_bits_out) return DYBIT_ERR_NULL;
    if (n_layers < 1 || n_layers > (1 << 20) || k < 1 || (strategy != DYBIT_SEARCH_SPEEDUP && strategy != DYBIT_SEARCH_RMSE) ||
        std::isnan(constraint))
        return DYBIT_ERR_INVALID_ARG;
    const Tables t{n_layers, lat, rmse_w, rmse_a};
    if (!tables_valid(t)) return DYBIT_ERR_INVALID_ARG;
    const bool by_speed = strategy == DYBIT_SEARCH_SPEEDUP;

    Assignment s{std::vector<int>(n_layers, 0), std::vector<int>(n_layers, 0)};      // everything at 8 bits
    const double base = by_speed ? sum_latency(t, s) : sum_error(t, s);
    if (!(base > 0.0)) return DYBIT_ERR_INVALID_ARG;
    double ratio = 1.0;
    bool finished = by_speed && ratio >= constraint;

    std::vector<int> open, order;
    while (!finished) {
        // layers with something left to lower, and their metrics under the current assignment
        open.clear();
        for (int l = 0; l < n_layers; ++l)
            if (s.w[l] < kLevels - 1 || s.a[l] < kLevels - 1) open.push_back(l);
        if (open.empty()) break;
        auto slower = [&](int x, int y) { return t.latency(x, s.w[x], s.a[x]) > t.latency(y, s.w[y], s.a[y]); };
        auto smaller_error = [&](int x, int y) { return t.error(x, s.w[x], s.a[x]) < t.error(y, s.w[y], s.a[y]); };
        // rank by the constrained quantity, keep k, re-rank those by the other one; `open` is in
        // index order and both sorts are stable, so equal metrics leave the lower index in front
        order = open;
        if (by_speed) std::stable_sort(order.begin(), order.end(), slower);
        else          std::stable_sort(order.begin(), order.end(), smaller_error);
        if ((size_t)k < order.size()) order.resize(k);
        std::sort(order.begin(), order.end());
        if (by_speed) std::stable_sort(order.begin(), order.end(), smaller_error);
        else          std::stable_sort(order.begin(), order.end(), slower);
        // lower the weights of the listed layers one step each, then their activations
        for (int which = 0; which < 2 && !finished; ++which) {
            std::vector<int> &level = s.table(which);
            for (int l : order) {
                if (level[l] == kLevels - 1) continue;
                ++level[l];
                if (by_speed) {
                    ratio = base / sum_latency(t, s);
                    if (ratio >= constraint) { finished = true; break; }
                } else {
                    const double r = sum_error(t, s) / base;
                    if (r > constraint) { --level[l]; finished = true; break; }     // over the budget: undone
                    ratio = r;
                }
            }
        }
    }
    for (int l = 0; l < n_layers; ++l) {
        w_bits_out[l] = kBits[s.w[l]];
        a_bits_out[l] = kBits[s.a[l]];
    }
    if (ratio_out) *ratio_out = ratio;
    if (met_out) *met_out = by_speed ? ratio >= constraint : ratio <= constraint;
    return DYBIT_OK;
}
