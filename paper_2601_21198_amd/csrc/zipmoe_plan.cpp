// Cache-pool planning for the expert cache: how much of a memory budget each of the pools F, C, S, E
// should get.  Follows ZipMoE (arXiv 2601.21198) Sec. 3.4 "Hierarchical Cache Planning", App. C
// (hit-count distribution of a rank interval, makespan estimate, grid search over memory ratios) and
// App. D (modified iterative proportional fitting that turns rank-based inclusion probabilities into
// independent selection probabilities).  Host only, double precision.
#include "zipmoe.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

namespace {

// p(x) *= (a + b x), coefficients above degree deg dropped
void poly_times(std::vector<double> &p, double a, double b, int deg)
{
    for (int j = deg; j >= 1; --j) p[j] = a * p[j] + b * p[j - 1];
    p[0] *= a;
}

// p(x) *= (1 + w x): the generating polynomial of the weights' elementary symmetric polynomials (App. D)
void poly_times(std::vector<double> &p, double w, int deg) { poly_times(p, 1.0, w, deg); }

// f_i implied by the weights: w_i * R(k-1, all but i) / R(k, all), with the leave-one-out symmetric
// polynomials taken from prefix and suffix products (no division).
void implied_inclusion(const std::vector<double> &w, int k, std::vector<double> &out)
{
    const int n = static_cast<int>(w.size());
    const int deg = k;
    std::vector<std::vector<double>> suffix(n + 1, std::vector<double>(deg + 1, 0.0));
    suffix[n][0] = 1.0;
    for (int i = n - 1; i >= 0; --i) { suffix[i] = suffix[i + 1]; poly_times(suffix[i], w[i], deg); }
    const double total = suffix[0][k];
    std::vector<double> prefix(deg + 1, 0.0);
    prefix[0] = 1.0;
    out.assign(n, 0.0);
    for (int i = 0; i < n; ++i) {
        double r = 0.0;                                    // R(k-1, all but i)
        for (int a = 0; a <= k - 1; ++a) r += prefix[a] * suffix[i + 1][k - 1 - a];
        out[i] = total > 0 ? w[i] * r / total : 0.0;
        poly_times(prefix, w[i], deg);
    }
}

// App. C: the number of selected ranks among n independent draws with probabilities q has the generating
// polynomial prod_r ((1 - q_r) + q_r x); phi[h] is its coefficient of x^h.
void hit_distribution(const double *q, int n, double *phi)
{
    std::vector<double> poly(n + 1, 0.0);
    poly[0] = 1.0;
    for (int r = 0; r < n; ++r) poly_times(poly, 1.0 - q[r], q[r], std::min(r + 1, n));
    std::copy(poly.begin(), poly.end(), phi);
}

// What an expert found in each state still needs (App. C; Sec. 3.2): {SM-chunks read, E-chunks read, decompression}.
// States: the pools F, C, S, E and, last, cached nowhere.
constexpr int kNeeds[5][3] = {{0, 0, 0}, {0, 0, 1}, {0, 1, 1}, {1, 0, 1}, {1, 1, 1}};

// App. C: the I/O thread reads everything that is missing one after the other; the L workers share the E-chunk
// reads they wait for and the decompressions; the layer takes the longer of the two.
double makespan(int k, const int32_t hits[4], const zm_plan_costs &p)
{
    int in_state[5] = {hits[0], hits[1], hits[2], hits[3], k - hits[0] - hits[1] - hits[2] - hits[3]};
    double experts[3] = {0.0, 0.0, 0.0};                   // experts that need each of the three things
    for (int s = 0; s < 5; ++s)
        for (int part = 0; part < 3; ++part) experts[part] += in_state[s] * kNeeds[s][part];
    const double tensors = p.tensors_per_expert, shards = tensors * p.shards_per_tensor;
    const double sm_reads = experts[0] * tensors * p.sm_read_delay;
    const double e_reads = experts[1] * shards * p.e_read_delay;
    const double decompressions = experts[2] * shards * p.decompress_delay;
    return std::max(sm_reads + e_reads, (e_reads + decompressions) / p.threads);
}

bool costs_ok(const zm_plan_costs *p)
{
    return p && p->threads >= 1 && p->shards_per_tensor >= 1 && p->tensors_per_expert >= 1 &&
           p->decompress_delay >= 0 && p->e_read_delay >= 0 && p->sm_read_delay >= 0;
}

double expected_cost(const double *q, int n, const int32_t slots[4], int k, const zm_plan_costs &costs,
                     const std::vector<double> &phi_all)
{
    std::vector<double> phi[4], phi_miss;
    int at = 0;
    for (int p = 0; p < 4; ++p) { phi[p].assign(slots[p] + 1, 0.0); hit_distribution(q + at, slots[p], phi[p].data()); at += slots[p]; }
    phi_miss.assign(n - at + 1, 0.0);
    hit_distribution(q + at, n - at, phi_miss.data());
    double cost = 0.0;
    int32_t h[4];
    for (h[0] = 0; h[0] <= slots[0] && h[0] <= k; ++h[0])
        for (h[1] = 0; h[1] <= slots[1] && h[0] + h[1] <= k; ++h[1])
            for (h[2] = 0; h[2] <= slots[2] && h[0] + h[1] + h[2] <= k; ++h[2])
                for (h[3] = 0; h[3] <= slots[3]; ++h[3]) {
                    const int rem = k - h[0] - h[1] - h[2] - h[3];
                    if (rem < 0) break;
                    if (rem > n - at) continue;
                    const double pr = phi_miss[rem] / phi_all[k] * phi[0][h[0]] * phi[1][h[1]] * phi[2][h[2]] * phi[3][h[3]];
                    cost += makespan(k, h, costs) * pr;
                }
    return cost;
}

}  // namespace

extern "C" {

int zm_plan_selection_probabilities(const double *f, int n, int k, int max_iters, double tol, double *q_out, int *iters_out)
{
    if (!f || !q_out || n <= 0 || k <= 0 || k > n || max_iters <= 0 || !(tol > 0)) return ZM_E_ARG;
    for (int i = 0; i < n; ++i) if (!(f[i] >= 0) || f[i] > 1) return ZM_E_ARG;
    try {
        std::vector<double> w(f, f + n), cur;
        int used = 0;
        for (used = 1; used <= max_iters; ++used) {
            implied_inclusion(w, k, cur);
            double worst = 0.0;
            for (int i = 0; i < n; ++i) worst = std::max(worst, std::fabs(cur[i] - f[i]));
            if (worst < tol) break;
            for (int i = 0; i < n; ++i) w[i] = cur[i] > 0 ? w[i] * f[i] / cur[i] : 0.0;
        }
        if (used > max_iters) used = max_iters;
        for (int i = 0; i < n; ++i) q_out[i] = w[i] / (1.0 + w[i]);
        if (iters_out) *iters_out = used;
    } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    return ZM_OK;
}

int zm_plan_hit_distribution(const double *q, int n, double *phi_out)
{
    if ((!q && n > 0) || !phi_out || n < 0) return ZM_E_ARG;
    try {
        hit_distribution(q, n, phi_out);
    } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    return ZM_OK;
}

int zm_plan_makespan(int k, const int32_t hits[4], const zm_plan_costs *costs, double *makespan_out)
{
    if (!hits || !costs_ok(costs) || !makespan_out || k < 0) return ZM_E_ARG;
    if (hits[0] < 0 || hits[1] < 0 || hits[2] < 0 || hits[3] < 0 || hits[0] + hits[1] + hits[2] + hits[3] > k) return ZM_E_ARG;
    *makespan_out = makespan(k, hits, *costs);
    return ZM_OK;
}

int zm_plan_expected_makespan(const double *q, int n_experts, const int32_t slots[4], int k, const zm_plan_costs *costs,
                              double *cost_out)
{
    if (!q || !slots || !costs_ok(costs) || !cost_out || n_experts <= 0 || k <= 0 || k > n_experts) return ZM_E_ARG;
    long sum = 0;
    for (int p = 0; p < 4; ++p) { if (slots[p] < 0) return ZM_E_ARG; sum += slots[p]; }
    if (sum > n_experts) return ZM_E_ARG;
    try {
        std::vector<double> phi_all(n_experts + 1);
        hit_distribution(q, n_experts, phi_all.data());
        if (!(phi_all[k] > 0)) return ZM_E_ARG;
        *cost_out = expected_cost(q, n_experts, slots, k, *costs, phi_all);
    } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    return ZM_OK;
}

int zm_plan_pools(const double *f, int n_experts, int k, const zm_plan_costs *costs, double memory_bytes,
                  const double bytes_per_expert[4], int grid, int pool_mask,
                  double ratios_out[4], int32_t slots_out[4], double *cost_out)
{
    if (!f || !costs_ok(costs) || !bytes_per_expert || !ratios_out || !slots_out || !cost_out) return ZM_E_ARG;
    if (n_experts <= 0 || k <= 0 || k > n_experts || grid < 1 || grid > 1000 || !(memory_bytes >= 0)) return ZM_E_ARG;
    if ((pool_mask & 15) == 0) return ZM_E_ARG;
    for (int p = 0; p < 4; ++p) if (!(bytes_per_expert[p] > 0)) return ZM_E_ARG;
    try {
        std::vector<double> q(n_experts);
        int rc = zm_plan_selection_probabilities(f, n_experts, k, 5000, 1e-12, q.data(), nullptr);
        if (rc != ZM_OK) return rc;
        std::vector<double> phi_all(n_experts + 1);
        hit_distribution(q.data(), n_experts, phi_all.data());
        if (!(phi_all[k] > 0)) return ZM_E_ARG;
        bool have = false;
        double best = 0.0;
        for (int gF = 0; gF <= grid; ++gF)
            for (int gC = 0; gC + gF <= grid; ++gC)
                for (int gS = 0; gS + gC + gF <= grid; ++gS) {
                    const int g[4] = {gF, gC, gS, grid - gF - gC - gS};
                    bool allowed = true;
                    for (int p = 0; p < 4; ++p) if (g[p] > 0 && !((pool_mask >> p) & 1)) allowed = false;
                    if (!allowed) continue;
                    int32_t slots[4];
                    int left = n_experts;
                    for (int p = 0; p < 4; ++p) {
                        const double ratio = static_cast<double>(g[p]) / grid;
                        long s = g[p] > 0 ? static_cast<long>(std::floor(ratio * memory_bytes / bytes_per_expert[p] + 1e-9)) : 0;
                        s = std::min<long>(s, left);
                        left -= static_cast<int>(s);
                        slots[p] = static_cast<int32_t>(s);
                    }
                    const double cost = expected_cost(q.data(), n_experts, slots, k, *costs, phi_all);
                    if (!have || cost < best) {
                        have = true; best = cost;
                        for (int p = 0; p < 4; ++p) { ratios_out[p] = static_cast<double>(g[p]) / grid; slots_out[p] = slots[p]; }
                    }
                }
        *cost_out = best;
    } catch (const std::bad_alloc &) { return ZM_E_NOMEM; }
    return ZM_OK;
}

}  // extern "C"
