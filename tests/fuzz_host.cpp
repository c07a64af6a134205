// Memory-safety fuzz of the host-only entry points under ASan/UBSan (no GPU code).
#include <cstdio>
#include <cstdint>
#include <random>
#include <vector>
#include <cmath>
#include "baoc.h"
int main()
{
    std::mt19937_64 rng(123);
    auto U = [&](double a, double b) { return a + (b - a) * (rng() >> 11) * (1.0 / 9007199254740992.0); };
    long ok = 0, inf = 0, lim = 0, inv = 0;
    for (int trial = 0; trial < 600; ++trial) {
        const uint32_t N = 1 + rng() % 60, K = 1 + rng() % 21;
        std::vector<double> risk(N * K), tc(N * K); std::vector<int64_t> mem(N * K); std::vector<uint8_t> fb(N * K);
        int64_t lo = 0, hi = 0; double tlo = 0, thi = 0;
        for (uint32_t i = 0; i < N; ++i) {
            int64_t mn = INT64_MAX, mx = 0; double tn = 1e300, tx = 0;
            for (uint32_t c = 0; c < K; ++c) {
                const size_t q = (size_t)i * K + c;
                risk[q] = (trial % 5 == 0) ? (double)(rng() % 4) : U(-1, 3);
                if (rng() % 97 == 0) risk[q] = NAN; if (rng() % 131 == 0) risk[q] = INFINITY;
                mem[q] = (int64_t)(rng() % 1000000) * (trial % 7 == 0 ? 1000003 : 1);
                tc[q] = U(0.2, 2.0); fb[q] = rng() % 11 == 0;
                mn = std::min(mn, mem[q]); mx = std::max(mx, mem[q]); tn = std::min(tn, tc[q]); tx = std::max(tx, tc[q]);
            }
            lo += mn; hi += mx; tlo += tn; thi += tx;
        }
        const int64_t bm = lo + (int64_t)(U(-0.05, 1.0) * (double)(hi - lo));
        const double bt = tlo + U(-0.05, 1.0) * (thi - tlo);
        std::vector<uint32_t> choice(N); double obj; int64_t om; double ot;
        baoc_allocate_set_node_limit(trial % 3 == 0 ? 20000 : 0);
        if (trial % 4 == 1) baoc_allocate_set_exact_work(1, 1 + trial % 7); else baoc_allocate_set_exact_work(0, 0);   // thinned forward pass
        const int rc = baoc_allocate(risk.data(), mem.data(), tc.data(), N, K, bm, bt, trial % 2 ? fb.data() : nullptr, choice.data(), &obj, &om, &ot);
        if (rc == BAOC_OK) { ++ok; for (uint32_t i = 0; i < N; ++i) if (choice[i] >= K) { printf("bad choice\n"); return 1; } if (om > bm) { printf("budget violated\n"); return 1; } }
        else if (rc == BAOC_ERR_INFEASIBLE) ++inf; else if (rc == BAOC_ERR_LIMIT) ++lim; else ++inv;
    }
    printf("allocate: ok %ld infeasible %ld limit %ld other %ld\n", ok, inf, lim, inv);
    long pok = 0;
    for (int trial = 0; trial < 400; ++trial) {
        const uint32_t m = 1 + rng() % 120, K = 1 + rng() % 6;
        std::vector<uint64_t> numel(m); std::vector<double> z((size_t)m * K), w(K);
        for (auto& x : numel) x = 1 + rng() % 1000000; for (auto& x : z) x = (trial % 3 == 0) ? (double)(rng() % 3) : U(0, 1); for (auto& x : w) x = U(0, 2);
        std::vector<uint32_t> ids(m); uint32_t nb; double tau;
        const double alphas[] = {0.0, 0.001, 0.01, 0.1, 0.5, 1.0};
        const int rc = baoc_partition(numel.data(), z.data(), m, K, trial % 2 ? w.data() : nullptr, alphas[trial % 6], ids.data(), &nb, &tau);
        if (rc != BAOC_OK) { printf("partition rc %d\n", rc); return 1; }
        uint32_t prev = 0; for (uint32_t j = 0; j < m; ++j) { if (ids[j] < prev || ids[j] > prev + 1 || ids[j] >= nb) { printf("bad ids\n"); return 1; } prev = ids[j]; }
        ++pok;
    }
    printf("partition: ok %ld\n", pok);
    return 0;
}
