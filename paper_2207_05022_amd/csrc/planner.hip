// Two-stage planning (Section "Compute Planning", Section "IO Planning"): host code, no
// device work.  Given the profiled delays it picks the submodel size for a deadline and then
// the fidelity version of every shard, keeping every layer's accumulated IO budget
// non-negative so that the load || compute pipeline never waits for IO.
#include <vector>

#include "api_internal.hpp"

namespace sti {
namespace {

constexpr int kVersions[6] = {2, 3, 4, 5, 6, 32};
constexpr double kSlack = 1e-12;   // seconds; absorbs rounding of sums of profiled delays

inline int version_slot(int bits)
{
    for (int v = 0; v < 6; ++v)
        if (kVersions[v] == bits) return v;
    return -1;
}

bool tables_ok(const sti_plan_tables *t)
{
    if (!t || !t->t_comp) return false;
    if (t->n_layers <= 0 || t->n_shards <= 0 || t->n_shards > kMaxShardsPerLayer) return false;
    for (int v = 0; v < 6; ++v)
        if (!(t->t_io[v] >= 0.0)) return false;
    for (int m = 0; m < t->n_shards; ++m)
        if (!(t->t_comp[m] > 0.0)) return false;
    return true;
}

}  // namespace
}  // namespace sti

using namespace sti;

extern "C" {

sti_status sti_plan_submodel(const sti_plan_tables *tables, double deadline_s, int32_t *n_out, int32_t *m_out)
{
    if (!tables || !n_out || !m_out) return STI_ERR_NULL;
    if (!tables_ok(tables) || !(deadline_s >= 0.0)) return STI_ERR_DIMS;
    int best_n = 0, best_m = 0;
    for (int n = 1; n <= tables->n_layers; ++n)
        for (int m = 1; m <= tables->n_shards; ++m) {
            if ((double)n * tables->t_comp[m - 1] > deadline_s) continue;
            const long shards = (long)n * m, best = (long)best_n * best_m;
            if (shards > best || (shards == best && n > best_n)) { best_n = n; best_m = m; }
        }
    *n_out = best_n;
    *m_out = best_m;
    return STI_OK;
}

sti_status sti_plan_bitwidths(const sti_plan_tables *tables, int32_t n, int32_t m, const int8_t *preloaded,
                              const int32_t *importance, int8_t *plan, double *aib_out)
{
    if (!tables || !plan) return STI_ERR_NULL;
    if (!tables_ok(tables)) return STI_ERR_DIMS;
    const int N = tables->n_layers, M = tables->n_shards;
    if (n < 0 || n > N || m < 0 || m > M) return STI_ERR_DIMS;
    if ((n == 0) != (m == 0)) return STI_ERR_DIMS;
    if (n > 0 && !importance) return STI_ERR_NULL;
    std::vector<double> aib;
    std::vector<int8_t> out;
    std::vector<char> seen;
    try {
        aib.assign(n, 0.0);
        out.assign((size_t)N * M, 0);
        seen.assign((size_t)N * M, 0);
    } catch (const std::bad_alloc &) {
        return STI_ERR_HIP;
    }
    for (int s = 0; s < N * M && n > 0; ++s) {
        const int id = importance[s];
        if (id < 0 || id >= N * M || seen[id]) return STI_ERR_DIMS;   // a permutation of the shard ids
        seen[id] = 1;
    }
    if (preloaded) {
        for (int s = 0; s < N * M; ++s)
            if (preloaded[s] != 0 && version_slot(preloaded[s]) < 0) return STI_ERR_BITWIDTH;
    }
    if (n > 0) {
        const double t_comp = tables->t_comp[m - 1];
        // AIB(0): the IO that filled the preload buffer ("bonus IO"); AIB(k) = AIB(k-1) + T_comp
        double bonus = 0.0;
        for (int l = 0; l < n; ++l)
            for (int i = 0; i < m; ++i) {
                const int b = preloaded ? preloaded[l * M + i] : 0;
                if (b) bonus += tables->t_io[version_slot(b)];
            }
        for (int k = 0; k < n; ++k) aib[k] = bonus + k * t_comp;
        // a shard selected at layer l is charged to layer l and to every later layer
        auto charge = [&](int layer, double seconds) {
            for (int k = layer; k < n; ++k) aib[k] -= seconds;
        };
        auto fits = [&](int layer, double seconds) {
            for (int k = layer; k < n; ++k)
                if (aib[k] - seconds < -kSlack) return false;
            return true;
        };
        std::vector<int> free_per_layer(n, 0);
        for (int l = 0; l < n; ++l)
            for (int i = 0; i < m; ++i) {
                const int b = preloaded ? preloaded[l * M + i] : 0;
                if (b) {
                    out[l * M + i] = (int8_t)b;
                    charge(l, tables->t_io[version_slot(b)]);
                } else {
                    free_per_layer[l] += 1;
                }
            }
        // pass 1: the highest uniform version of all shards that are not preloaded
        int uniform = -1;
        for (int v = 0; v < 6; ++v) {
            std::vector<double> trial(aib);
            bool ok = true;
            for (int l = 0; l < n; ++l) {
                const double cost = free_per_layer[l] * tables->t_io[v];
                for (int k = l; k < n; ++k) trial[k] -= cost;
            }
            for (int k = 0; k < n; ++k) ok = ok && trial[k] >= -kSlack;
            if (ok) uniform = v;
        }
        const bool starved = uniform < 0;   // not even 2 bits fit: take them anyway, allocate nothing more
        if (starved) uniform = 0;
        for (int l = 0; l < n; ++l)
            for (int i = 0; i < m; ++i)
                if (!out[l * M + i]) {
                    out[l * M + i] = (int8_t)kVersions[uniform];
                    charge(l, tables->t_io[uniform]);
                }
        // pass 2: full fidelity for the most important shards while the budgets last
        if (!starved) {
            for (int s = 0; s < N * M; ++s) {
                const int id = importance[s], l = id / M, i = id - l * M;
                if (l >= n || i >= m) continue;
                if (preloaded && preloaded[id]) continue;
                if (out[id] == 32) continue;
                const double extra = tables->t_io[5] - tables->t_io[version_slot(out[id])];
                if (fits(l, extra)) {
                    charge(l, extra);
                    out[id] = 32;
                }
            }
        }
    }
    for (int s = 0; s < N * M; ++s) plan[s] = out[s];
    if (aib_out)
        for (int k = 0; k < n; ++k) aib_out[k] = aib[k];
    return STI_OK;
}

}  // extern "C"
