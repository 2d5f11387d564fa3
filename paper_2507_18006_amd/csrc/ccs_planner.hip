// Scale-up planning on the host (Section 4.1): the speed-up model of layer replication (Eq. 1-4)
// and the greedy scale-up of Algorithm 1 with its continuity ordering.  No GPU work happens
// here; the functions are part of the same C ABI so that a serving loop can decide where the
// next replica goes and then call ccs_module_replicate.
#include <cstdint>
#include <vector>

#include "../../include/cocoserve_mi.h"

namespace {

// sum_i 1 / p_i: the L1 norm of the element-wise quotient 1 / P in Algorithm 1
double inv_sum(const int32_t *p, int32_t n)
{
    double s = 0.0;
    for (int32_t i = 0; i < n; ++i) s += 1.0 / (double)p[i];
    return s;
}

// Length of the run of consecutive layers around `layer` that node g would hold with it.
int run_with(const uint8_t *on_g, int32_t n, int32_t layer)
{
    int len = 1;
    for (int32_t i = layer - 1; i >= 0 && on_g[i]; --i) ++len;
    for (int32_t i = layer + 1; i < n && on_g[i]; ++i) ++len;
    return len;
}

}  // namespace

extern "C" {

double ccs_speedup_homo(const int32_t *p, int32_t n, double gamma)
{
    if (!p || n < 1) return 0.0;
    for (int32_t i = 0; i < n; ++i)
        if (p[i] < 1) return 0.0;
    return 1.0 / (gamma + (1.0 - gamma) / (double)n * inv_sum(p, n));
}

double ccs_speedup(const int32_t *p, int32_t n, const double *bs, const double *capacity, const double *bandwidth,
                   double d, double l, double delta)
{
    if (!p || !bs || !capacity || !bandwidth || n < 1) return 0.0;
    double w = 0.0, t = 0.0, w0 = 0.0;
    int64_t o = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (p[i] < 1) return 0.0;
        double slowest = 0.0, batch = 0.0;
        for (int32_t j = 0; j < p[i]; ++j) {
            const double c = d * d * bs[o + j] * l / capacity[o + j];      // Eq. 1: replica j's compute
            if (c > slowest) slowest = c;
            batch += bs[o + j];
            if (j >= 1) t += d * bs[o + j] * l / bandwidth[o + j];         // Eq. 2: what travels to a replica
        }
        w += slowest;
        w0 += d * d * batch * l / capacity[o];                            // P0: the whole batch on the original
        o += p[i];
    }
    return w0 / (w + delta * t);                                          // Eq. 3
}

int ccs_shares_from_capacity(int64_t n, int32_t k, const double *capacity, int32_t *counts_out)
{
    if (!capacity || !counts_out || k < 1 || k > CCS_MAX_REPLICAS || n < 0 || n > 0x7fffffffLL) return CCS_EINVAL;
    double total = 0.0;
    for (int32_t j = 0; j < k; ++j) {
        if (!(capacity[j] > 0.0) || capacity[j] > 1e300) return CCS_EINVAL;
        total += capacity[j];
    }
    // capacity-weighted contiguous split: boundary j = floor(n * (C_0 + .. + C_{j-1}) / C_total)
    double before = 0.0;
    int64_t lo = 0;
    for (int32_t j = 0; j < k; ++j) {
        before += capacity[j];
        int64_t hi = j == k - 1 ? n : (int64_t)__builtin_floor((double)n * before / total);
        if (hi < lo) hi = lo;
        if (hi > n) hi = n;
        counts_out[j] = (int32_t)(hi - lo);
        lo = hi;
    }
    // hand units from a slowest instance to the one that stays fastest, while that helps
    for (;;) {
        int32_t worst = 0, taker = 0;
        for (int32_t j = 1; j < k; ++j) {
            if (counts_out[j] / capacity[j] > counts_out[worst] / capacity[worst]) worst = j;
            if ((counts_out[j] + 1) / capacity[j] < (counts_out[taker] + 1) / capacity[taker]) taker = j;
        }
        if (counts_out[worst] == 0 || (counts_out[taker] + 1) / capacity[taker] >= counts_out[worst] / capacity[worst]) break;
        counts_out[worst] -= 1;
        counts_out[taker] += 1;
    }
    return CCS_OK;
}

int ccs_plan_scale_up(const int32_t *p_in, int32_t n, double gamma, const int64_t *node_available, int32_t n_nodes,
                      int64_t replica_size, const uint8_t *placed_in, int32_t *p_out, uint8_t *placed_out,
                      double *speedup_out)
{
    if (!p_in || !p_out || !placed_out || n < 1 || n_nodes < 0 || replica_size < 1 || (n_nodes > 0 && !node_available))
        return CCS_EINVAL;
    for (int32_t i = 0; i < n; ++i) {
        if (p_in[i] < 1) return CCS_EINVAL;
        p_out[i] = p_in[i];
    }
    for (int64_t i = 0; i < (int64_t)n_nodes * n; ++i) placed_out[i] = placed_in ? (placed_in[i] ? 1 : 0) : 0;
    double best = ccs_speedup_homo(p_out, n, gamma);
    std::vector<int32_t> cand;
    std::vector<uint8_t> sim(n);
    for (int32_t g = 0; g < n_nodes; ++g) {
        const int64_t max_replicas = node_available[g] / replica_size;
        if (max_replicas < 1) continue;   // not eligible: no room for one replica
        uint8_t *on_g = placed_out + (int64_t)g * n;
        // candidates in continuity order: repeatedly the free layer that gives node g its longest
        // run of consecutive layers (ties: the lower layer index), at most max_replicas of them
        cand.clear();
        for (int32_t i = 0; i < n; ++i) sim[i] = on_g[i];
        for (int64_t c = 0; c < max_replicas; ++c) {
            int32_t pick = -1;
            int pick_run = 0;
            for (int32_t i = 0; i < n; ++i) {
                if (sim[i]) continue;
                const int r = run_with(sim.data(), n, i);
                if (r > pick_run) { pick_run = r; pick = i; }
            }
            if (pick < 0) break;
            sim[pick] = 1;
            cand.push_back(pick);
        }
        for (int32_t layer : cand) {
            p_out[layer] += 1;
            const double sp = ccs_speedup_homo(p_out, n, gamma);
            if (sp > best) {
                best = sp;
                on_g[layer] = 1;
            } else {
                p_out[layer] -= 1;
            }
        }
    }
    if (speedup_out) *speedup_out = best;
    return CCS_OK;
}

}  // extern "C"
