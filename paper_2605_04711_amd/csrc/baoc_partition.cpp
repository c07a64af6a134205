// baoc_partition: structure-guided, statistic-refined block partitioning (App. C.2, Algorithm 2).
// Host code over per-unit diagnostic vectors; O(m^2 K) for the pairwise differences.
//
// Readings where the algorithm is loose: a temporary block's statistics are the
// parameter-weighted mean of its units' vectors (accumulated in unit order); tau is the
// upper quartile (linear interpolation) of Delta over all unit pairs; an undersized block is
// merged into the adjacent block with the smaller Delta (tie: the smaller neighbour, then the
// left one), always handling the first undersized block; a boundary between adjacent
// temporary blocks survives when Delta > tau and both sides reach n_min; a formed block is
// split at the internal boundary with the largest difference of the two sides' statistics if
// that exceeds tau and both sides reach n_min, recursively; undersized results are merged again.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "baoc.h"

namespace {

struct Ctx {
    const uint64_t* numel; const double* z; uint32_t K; std::vector<double> w; double n_min;
};

typedef std::vector<uint32_t> Units;              // contiguous unit indices of one (temporary) block

void stats(const Ctx& c, const Units* parts, size_t n_parts, std::vector<double>& mean, double& size)
{
    mean.assign(c.K, 0.0);
    uint64_t total = 0;
    for (size_t p = 0; p < n_parts; ++p)
        for (uint32_t j : parts[p]) {
            total += c.numel[j];
            for (uint32_t k = 0; k < c.K; ++k) mean[k] += (double)c.numel[j] * c.z[(size_t)j * c.K + k];
        }
    size = (double)total;
    for (uint32_t k = 0; k < c.K; ++k) mean[k] /= size;
}

double delta(const Ctx& c, const std::vector<double>& a, const std::vector<double>& b)
{
    double d = 0.0;
    for (uint32_t k = 0; k < c.K; ++k) {
        const double x = c.w[k] * std::fabs(a[k] - b[k]);
        if (x > d) d = x;
    }
    return d;
}

void merge_small(const Ctx& c, std::vector<Units>& blocks)
{
    std::vector<double> zs, zn;
    double ss, sn;
    while (blocks.size() > 1) {
        size_t small = blocks.size();
        for (size_t i = 0; i < blocks.size(); ++i) {
            stats(c, &blocks[i], 1, zs, ss);
            if (ss < c.n_min) { small = i; break; }
        }
        if (small == blocks.size()) break;
        stats(c, &blocks[small], 1, zs, ss);
        bool have = false; double bd = 0, bs = 0; size_t bn = 0;
        for (int side = 0; side < 2; ++side) {
            if (side == 0 && small == 0) continue;
            if (side == 1 && small + 1 >= blocks.size()) continue;
            const size_t nb = side == 0 ? small - 1 : small + 1;
            stats(c, &blocks[nb], 1, zn, sn);
            const double d = delta(c, zs, zn);
            if (!have || d < bd || (d == bd && sn < bs)) { have = true; bd = d; bs = sn; bn = nb; }
        }
        const size_t lo = std::min(small, bn), hi = std::max(small, bn);
        blocks[lo].insert(blocks[lo].end(), blocks[hi].begin(), blocks[hi].end());
        blocks.erase(blocks.begin() + hi);
    }
}

void split(const Ctx& c, const std::vector<Units>& temp, size_t lo, size_t hi, double tau, std::vector<Units>& out)
{
    std::vector<double> zl, zr;
    double sl, sr, best = -1.0; size_t at = 0; bool have = false;
    for (size_t p = lo + 1; p < hi; ++p) {
        stats(c, &temp[lo], p - lo, zl, sl);
        stats(c, &temp[p], hi - p, zr, sr);
        if (sl < c.n_min || sr < c.n_min) continue;
        const double d = delta(c, zl, zr);
        if (d > best) { best = d; at = p; have = true; }
    }
    if (!have || !(best > tau)) {
        Units u;
        for (size_t p = lo; p < hi; ++p) u.insert(u.end(), temp[p].begin(), temp[p].end());
        out.push_back(u);
        return;
    }
    split(c, temp, lo, at, tau, out);
    split(c, temp, at, hi, tau, out);
}

}  // namespace

static int partition(const uint64_t* unit_numel, const double* z, uint32_t n_units, uint32_t n_stats,
                     const double* weights, double alpha,
                     uint32_t* out_block_of_unit, uint32_t* out_n_blocks, double* out_tau)
{
    if (!unit_numel || !z || !out_block_of_unit || n_units == 0 || n_stats == 0) return BAOC_ERR_INVALID;
    if (!(alpha >= 0.0) || !(alpha <= 1.0)) return BAOC_ERR_INVALID;
    if (n_units > 32768) return BAOC_ERR_UNSUPPORTED;             // tau looks at all unit pairs (8 bytes each)
    Ctx c{unit_numel, z, n_stats, std::vector<double>(n_stats, 1.0), 0.0};
    uint64_t total = 0;
    for (uint32_t j = 0; j < n_units; ++j) {
        if (unit_numel[j] == 0 || total + unit_numel[j] < total) return BAOC_ERR_INVALID;
        total += unit_numel[j];
        for (uint32_t k = 0; k < n_stats; ++k)
            if (!std::isfinite(z[(size_t)j * n_stats + k])) return BAOC_ERR_INVALID;
    }
    for (uint32_t k = 0; k < n_stats && weights; ++k) {
        if (!(weights[k] >= 0.0) || !std::isfinite(weights[k])) return BAOC_ERR_INVALID;
        c.w[k] = weights[k];
    }
    c.n_min = alpha * (double)total;

    // tau: upper quartile of Delta over all pairs of candidate units
    std::vector<double> pair;
    pair.reserve((size_t)n_units * (n_units - 1) / 2);
    {
        std::vector<double> a(n_stats), b(n_stats);
        for (uint32_t i = 0; i < n_units; ++i)
            for (uint32_t j = i + 1; j < n_units; ++j) {
                for (uint32_t k = 0; k < n_stats; ++k) { a[k] = z[(size_t)i * n_stats + k]; b[k] = z[(size_t)j * n_stats + k]; }
                pair.push_back(delta(c, a, b));
            }
    }
    double tau = 0.0;
    if (!pair.empty()) {
        // the two order statistics that bracket position 0.75 (n - 1), by selection instead of a full sort
        const double pos = 0.75 * (double)(pair.size() - 1);
        const size_t lo = (size_t)pos;
        std::nth_element(pair.begin(), pair.begin() + (std::ptrdiff_t)lo, pair.end());
        const double at_lo = pair[lo];
        const double at_hi = lo + 1 < pair.size() ? *std::min_element(pair.begin() + (std::ptrdiff_t)lo + 1, pair.end()) : at_lo;
        tau = at_lo + (pos - (double)lo) * (at_hi - at_lo);
    }

    std::vector<Units> temp(n_units);
    for (uint32_t j = 0; j < n_units; ++j) temp[j] = Units{j};
    merge_small(c, temp);                                         // minimum-size filtering

    std::vector<std::pair<size_t, size_t>> formed;                // runs [lo, hi) of temporary blocks
    {
        std::vector<double> za, zb; double sa, sb;
        size_t lo = 0;
        for (size_t i = 1; i < temp.size(); ++i) {
            stats(c, &temp[i - 1], 1, za, sa);
            stats(c, &temp[i], 1, zb, sb);
            if (delta(c, za, zb) > tau && sa >= c.n_min && sb >= c.n_min) { formed.push_back({lo, i}); lo = i; }
        }
        formed.push_back({lo, temp.size()});
    }
    std::vector<Units> fin;
    for (const auto& f : formed) split(c, temp, f.first, f.second, tau, fin);
    merge_small(c, fin);

    for (size_t b = 0; b < fin.size(); ++b)
        for (uint32_t u : fin[b]) out_block_of_unit[u] = (uint32_t)b;
    if (out_n_blocks) *out_n_blocks = (uint32_t)fin.size();
    if (out_tau) *out_tau = tau;
    return BAOC_OK;
}

// No exception crosses the C boundary: running out of host memory (the pair table of a call near the unit
// limit takes about 4 GB) is reported like a size this build does not handle.
extern "C" int baoc_partition(const uint64_t* unit_numel, const double* z, uint32_t n_units, uint32_t n_stats,
                              const double* weights, double alpha,
                              uint32_t* out_block_of_unit, uint32_t* out_n_blocks, double* out_tau)
{
    try {
        return partition(unit_numel, z, n_units, n_stats, weights, alpha, out_block_of_unit, out_n_blocks, out_tau);
    } catch (const std::bad_alloc&) {
        return BAOC_ERR_UNSUPPORTED;
    }
}
