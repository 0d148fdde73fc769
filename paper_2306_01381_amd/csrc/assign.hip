// Bit-width assignment for the next period (Sec. 4.2): host code, no GPU work.
//
// The paper builds a bi-objective problem from the traced beta values - Eq. 8, the variance a message adds to the
// weight gradients, against Eq. 7, the time of the slowest device pair - scalarises it with a weight lambda
// (Eq. 9) and hands it to a MILP solver, with the messages of a pair sorted by beta and cut into groups that
// share a width.  Here the solver is replaced by a greedy search that needs no library: every group starts at
// 2 bits; per pair the upgrades 2->4 and 4->8 are ordered by variance removed per extra transferred bit (the
// order in which the relaxed problem would take them); for every pair time that such a prefix can reach, each
// pair takes the longest prefix that fits under it, and the time with the smallest Eq. 9 value wins.  With one
// pair this is the exact optimum; with several, a pair misses its best packing by less than one upgrade.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <vector>

#include "adaqp.h"

namespace {

struct Upgrade {
    double efficiency;      // variance removed per extra bit on the wire
    int32_t group;
    int32_t step;           // 0: 2 -> 4 bits, 1: 4 -> 8 bits
    double gain;
    int64_t cost;           // extra bits on the wire
};

struct PairPath {
    std::vector<std::vector<int64_t>> groups;   // slot numbers, descending beta
    std::vector<Upgrade> upgrades;              // in the order they are taken
    std::vector<double> time;                   // [m]: pair time with the first m upgrades applied
    std::vector<double> variance;               // [m]: Eq. 8 share of this pair
};

double inv_levels_sq(int b)
{
    const double levels = (double)((1 << b) - 1);
    return 1.0 / (levels * levels);
}

}  // namespace

extern "C" int adaqp_assign_bits(int64_t n, const float *beta_host, const int32_t *peer_of_slot_host,
                                 int32_t n_peers, int32_t dim, int32_t group_size, double lambda,
                                 const double *theta_host, const double *gamma_host, uint8_t *bits_out,
                                 double *objective_out)
{
    if (n < 0 || n_peers <= 0 || dim <= 0 || group_size <= 0 || !(lambda >= 0.0 && lambda <= 1.0))
        return ADAQP_EINVAL;
    if (!theta_host || !gamma_host) return ADAQP_EINVAL;
    if (n > 0 && (!beta_host || !peer_of_slot_host || !bits_out)) return ADAQP_EINVAL;
    if (n > ((int64_t)1 << 40) / dim) return ADAQP_ESIZE;           // bit counts stay far inside int64
    for (int32_t i = 0; i < n_peers; ++i)
        if (!(theta_host[i] >= 0.0) || !std::isfinite(theta_host[i]) || !std::isfinite(gamma_host[i]))
            return ADAQP_EINVAL;
    for (int64_t k = 0; k < n; ++k) {
        if (peer_of_slot_host[k] < 0 || peer_of_slot_host[k] >= n_peers) return ADAQP_EINVAL;
        if (!(beta_host[k] >= 0.0f) || !std::isfinite(beta_host[k])) return ADAQP_EINVAL;
    }

    const double w2 = inv_levels_sq(2), w4 = inv_levels_sq(4), w8 = inv_levels_sq(8);
    const double step_weight[2] = {w2 - w4, w4 - w8};
    const int64_t step_bits[2] = {2, 4};

    // ---- per pair: groups, upgrade order, reachable (time, variance) points ----
    std::vector<std::vector<int64_t>> members((size_t)n_peers);
    for (int64_t k = 0; k < n; ++k) members[(size_t)peer_of_slot_host[k]].push_back(k);
    std::vector<PairPath> pairs;
    std::vector<int32_t> pair_id;
    for (int32_t i = 0; i < n_peers; ++i) {
        std::vector<int64_t> &slots = members[(size_t)i];
        if (slots.empty()) continue;                                // a pair that exchanges nothing takes no time
        std::stable_sort(slots.begin(), slots.end(),
                         [&](int64_t a, int64_t b) { return beta_host[a] > beta_host[b]; });
        PairPath path;
        double variance_at_2 = 0.0;
        for (size_t s = 0; s < slots.size(); s += (size_t)group_size) {
            const size_t e = std::min(slots.size(), s + (size_t)group_size);
            path.groups.emplace_back(slots.begin() + (std::ptrdiff_t)s, slots.begin() + (std::ptrdiff_t)e);
            double group_beta = 0.0;
            for (size_t q = s; q < e; ++q) group_beta += (double)beta_host[slots[q]];
            variance_at_2 += group_beta * w2;
            const int32_t g = (int32_t)path.groups.size() - 1;
            for (int32_t step = 0; step < 2; ++step) {
                Upgrade u;
                u.group = g;
                u.step = step;
                u.gain = group_beta * step_weight[step];
                u.cost = step_bits[step] * (int64_t)(e - s) * dim;
                u.efficiency = u.gain / (double)u.cost;
                path.upgrades.push_back(u);
            }
        }
        std::sort(path.upgrades.begin(), path.upgrades.end(), [](const Upgrade &a, const Upgrade &b) {
            if (a.efficiency != b.efficiency) return a.efficiency > b.efficiency;
            if (a.group != b.group) return a.group < b.group;
            return a.step < b.step;
        });
        const int64_t base_bits = 2 * (int64_t)dim * (int64_t)slots.size();
        path.time.push_back(theta_host[i] * (double)base_bits + gamma_host[i]);
        path.variance.push_back(variance_at_2);
        int64_t cost = 0;
        double gain = 0.0;
        for (const Upgrade &u : path.upgrades) {
            cost += u.cost;
            gain += u.gain;
            path.time.push_back(theta_host[i] * (double)(base_bits + cost) + gamma_host[i]);
            path.variance.push_back(variance_at_2 - gain);
        }
        pairs.push_back(std::move(path));
        pair_id.push_back(i);
    }

    // ---- the candidate times: every point any pair can reach, not below the all-2-bit time of the slowest ----
    std::vector<size_t> taken(pairs.size(), 0);
    if (!pairs.empty()) {
        double z_min = pairs[0].time[0];
        for (const PairPath &p : pairs) z_min = std::max(z_min, p.time[0]);
        std::vector<double> candidates;
        for (const PairPath &p : pairs)
            for (double t : p.time)
                if (t >= z_min) candidates.push_back(t);
        std::sort(candidates.begin(), candidates.end());
        candidates.erase(std::unique(candidates.begin(), candidates.end()), candidates.end());
        bool have = false;
        double best = 0.0;
        std::vector<size_t> m(pairs.size());
        for (double z : candidates) {
            double variance = 0.0, worst = 0.0;
            for (size_t q = 0; q < pairs.size(); ++q) {
                const std::vector<double> &t = pairs[q].time;           // non-decreasing (theta >= 0)
                m[q] = (size_t)(std::upper_bound(t.begin(), t.end(), z) - t.begin()) - 1;
                variance += pairs[q].variance[m[q]];
                worst = q == 0 ? t[m[q]] : std::max(worst, t[m[q]]);
            }
            const double f = lambda * variance + (1.0 - lambda) * worst;
            if (!have || f < best) {
                have = true;
                best = f;
                taken = m;
            }
        }
    }

    // ---- widths per slot, and the objective of the result from its definition ----
    double variance = 0.0, worst = 0.0;
    for (size_t q = 0; q < pairs.size(); ++q) {
        const PairPath &p = pairs[q];
        std::vector<int> width(p.groups.size(), 2);
        for (size_t j = 0; j < taken[q]; ++j) width[(size_t)p.upgrades[j].group] += p.upgrades[j].step == 0 ? 2 : 4;
        int64_t payload = 0;
        for (size_t g = 0; g < p.groups.size(); ++g)
            for (int64_t k : p.groups[g]) {
                bits_out[k] = (uint8_t)width[g];
                payload += (int64_t)dim * width[g];
            }
        const double t = theta_host[pair_id[q]] * (double)payload + gamma_host[pair_id[q]];
        worst = q == 0 ? t : std::max(worst, t);
    }
    if (objective_out) {
        for (int64_t k = 0; k < n; ++k) variance += (double)beta_host[k] * inv_levels_sq(bits_out[k]);
        objective_out[0] = lambda * variance + (1.0 - lambda) * worst;
        objective_out[1] = variance;
        objective_out[2] = worst;
    }
    return ADAQP_OK;
}
