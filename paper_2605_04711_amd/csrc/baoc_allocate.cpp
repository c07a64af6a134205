// baoc_allocate: exact solver of the allocation problem of Eq. 2 -- one
// configuration per block, a memory row and a time row -- with the hard
// exclusions of Sec. 3.2 and a canonical answer (lexicographically smallest
// optimum of the integer image of the instance).
//
// Method: blocks are taken in index order and partial assignments are kept as
// a list of states (objective Z, memory W, time T).  A state is dropped when
//   - it cannot be completed within the budgets (suffix minima),
//   - a Lagrangian bound of the remaining blocks shows it cannot reach the
//     incumbent (weak duality, evaluated exactly in 128-bit integers for a few
//     fixed multiplier pairs found on the LP dual of the whole instance), or
//   - another state of the same level uses no more of either resource and is
//     better in (Z, lexicographic rank) -- any completion of the worse one is
//     beaten by the same completion of the better one.
// States of a level are generated in lexicographic order of their prefix, so
// "lexicographic rank" is just the generation index.  The best final state is
// the answer.  The list is capped by a node limit: when it is hit the call
// fails rather than return a guess.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

#include "baoc_internal.h"

namespace {

typedef __int128 i128;
constexpr double kPhiScale = 1e9, kPhiClamp = 1e6, kTauScale = 1e6;
constexpr int64_t kInf64 = std::numeric_limits<int64_t>::max() / 4;

struct Item { int64_t phi, w, t; uint32_t cfg; };

struct Instance {
    uint32_t N = 0;
    std::vector<std::vector<Item>> items;   // per block, ascending configuration index
    int64_t B1 = 0, B2 = 0;
};

thread_local uint64_t g_node_limit = 0;
constexpr uint64_t kDefaultNodeLimit = 40'000'000ull;

inline double clampd(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

// Remove configurations that can never be part of the canonical optimum: c is removed when some c'
// needs no more memory and time and is strictly better, or equally good with a smaller index.
void drop_dominated(std::vector<Item>& v)
{
    std::vector<Item> keep;
    for (size_t a = 0; a < v.size(); ++a) {
        bool dead = false;
        for (size_t b = 0; b < v.size() && !dead; ++b) {
            if (a == b) continue;
            if (v[b].w <= v[a].w && v[b].t <= v[a].t &&
                (v[b].phi < v[a].phi || (v[b].phi == v[a].phi && v[b].cfg < v[a].cfg)))
                dead = true;
        }
        if (!dead) keep.push_back(v[a]);
    }
    v.swap(keep);
}

struct Multiplier { i128 L1, L2, S; };          // lambda = L / S

// value and minimiser statistics of the Lagrangian for real multipliers
struct LagEval { double value; double W, T, Z; };

LagEval eval_lagrangian(const Instance& I, double l1, double l2, std::vector<uint32_t>* pick = nullptr)
{
    LagEval r{0, 0, 0, 0};
    if (pick) pick->resize(I.N);
    for (uint32_t i = 0; i < I.N; ++i) {
        double best = 0; size_t bi = 0; bool first = true;
        for (size_t k = 0; k < I.items[i].size(); ++k) {
            const Item& it = I.items[i][k];
            const double rc = (double)it.phi + l1 * (double)it.w + l2 * (double)it.t;
            // ties: lighter item first, so that a multiplier just above a breakpoint is feasible
            if (first || rc < best || (rc == best && (it.w < I.items[i][bi].w))) { best = rc; bi = k; first = false; }
        }
        const Item& it = I.items[i][bi];
        r.value += best; r.W += (double)it.w; r.T += (double)it.t; r.Z += (double)it.phi;
        if (pick) (*pick)[i] = (uint32_t)bi;
    }
    r.value -= l1 * (double)I.B1 + l2 * (double)I.B2;
    return r;
}

struct Heuristic {
    bool have = false; int64_t Z = 0;
    std::vector<uint32_t> pick;
};

void consider(const Instance& I, const std::vector<uint32_t>& pick, Heuristic& H)
{
    int64_t Z = 0, W = 0, T = 0;
    for (uint32_t i = 0; i < I.N; ++i) { const Item& it = I.items[i][pick[i]]; Z += it.phi; W += it.w; T += it.t; }
    if (W > I.B1 || T > I.B2) return;
    if (!H.have || Z < H.Z) { H.have = true; H.Z = Z; H.pick = pick; }
}

// Best single swap that lowers the objective and stays within both budgets, repeated.
void improve(const Instance& I, Heuristic& H)
{
    if (!H.have) return;
    int64_t W = 0, T = 0;
    for (uint32_t i = 0; i < I.N; ++i) { const Item& it = I.items[i][H.pick[i]]; W += it.w; T += it.t; }
    for (uint32_t round = 0; round < 4 * I.N + 16; ++round) {
        int64_t best = 0; uint32_t bi = 0, bk = 0;
        for (uint32_t i = 0; i < I.N; ++i) {
            const Item& cur = I.items[i][H.pick[i]];
            for (uint32_t k = 0; k < I.items[i].size(); ++k) {
                const Item& it = I.items[i][k];
                const int64_t d = it.phi - cur.phi;
                if (d < best && W - cur.w + it.w <= I.B1 && T - cur.t + it.t <= I.B2) { best = d; bi = i; bk = k; }
            }
        }
        if (best == 0) break;
        const Item& cur = I.items[bi][H.pick[bi]]; const Item& it = I.items[bi][bk];
        W += it.w - cur.w; T += it.t - cur.t; H.Z += best; H.pick[bi] = bk;
    }
}

// Greedy descent from the unconstrained optimum: start from the least-risk configuration of every
// block and, while a budget is exceeded, take the swap that buys the most relief per unit of added
// risk (relief = reduction of the excess over both rows, each in units of its budget).
void greedy_descent(const Instance& I, Heuristic& H)
{
    std::vector<uint32_t> pick(I.N);
    int64_t W = 0, T = 0;
    for (uint32_t i = 0; i < I.N; ++i) {
        uint32_t b = 0;
        for (uint32_t k = 1; k < I.items[i].size(); ++k)
            if (I.items[i][k].phi < I.items[i][b].phi) b = k;
        pick[i] = b; W += I.items[i][b].w; T += I.items[i][b].t;
    }
    const double n1 = 1.0 / std::max<double>(1.0, (double)I.B1), n2 = 1.0 / std::max<double>(1.0, (double)I.B2);
    for (uint64_t guard = 0; (W > I.B1 || T > I.B2) && guard < (uint64_t)I.N * 64; ++guard) {
        double best = -1.0; uint32_t bi = 0, bk = 0; bool any = false;
        for (uint32_t i = 0; i < I.N; ++i) {
            const Item& cur = I.items[i][pick[i]];
            for (uint32_t k = 0; k < I.items[i].size(); ++k) {
                const Item& it = I.items[i][k];
                double relief = 0.0;
                if (W > I.B1) relief += (double)std::min<int64_t>(cur.w - it.w, W - I.B1) * n1;
                if (T > I.B2) relief += (double)std::min<int64_t>(cur.t - it.t, T - I.B2) * n2;
                if (!(relief > 0.0)) continue;
                const double cost = (double)std::max<int64_t>(it.phi - cur.phi, 0) + 1.0;
                const double score = relief / cost;
                if (!any || score > best) { any = true; best = score; bi = i; bk = k; }
            }
        }
        if (!any) return;
        const Item& cur = I.items[bi][pick[bi]]; const Item& it = I.items[bi][bk];
        W += it.w - cur.w; T += it.t - cur.t; pick[bi] = bk;
    }
    Heuristic G;
    consider(I, pick, G);
    improve(I, G);
    if (G.have && (!H.have || G.Z < H.Z)) H = G;
}

// Concave maximisation of the dual in one multiplier by bisection on the sign of the subgradient.
double bisect(const Instance& I, bool first_row, double other, Heuristic& H)
{
    auto over = [&](double l) {
        std::vector<uint32_t> pick;
        LagEval e = first_row ? eval_lagrangian(I, l, other, &pick) : eval_lagrangian(I, other, l, &pick);
        consider(I, pick, H);
        return first_row ? e.W > (double)I.B1 : e.T > (double)I.B2;
    };
    if (!over(0.0)) return 0.0;
    double hi = 1.0;
    while (over(hi) && hi < 1e30) hi *= 4.0;
    if (hi >= 1e30) return hi;
    double lo = 0.0;
    for (int it = 0; it < 90; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (over(mid)) lo = mid; else hi = mid;
    }
    return hi;
}

Multiplier to_integer(double l1, double l2)
{
    const double mx = std::max(l1, l2);
    int k = 0;
    if (mx > 0) { k = 40 - (int)std::ceil(std::log2(mx)); k = std::max(0, std::min(40, k)); }
    const double S = std::ldexp(1.0, k);
    Multiplier m;
    m.S = (i128)1 << k;
    m.L1 = (i128)std::min(std::llround(std::min(l1 * S, 4e18)), (long long)4e18);
    m.L2 = (i128)std::min(std::llround(std::min(l2 * S, 4e18)), (long long)4e18);
    return m;
}

struct State { int64_t Z, W, T; uint32_t node; float slack; };   // node: arena index (parent, cfg); slack: cutoff - bound, scaled
struct Node { uint32_t parent; uint32_t item; };

struct Key { int64_t Z; uint32_t seq; };
inline bool operator<(const Key& a, const Key& b) { return a.Z < b.Z || (a.Z == b.Z && a.seq < b.seq); }

int solve(const Instance& I, std::vector<uint32_t>& answer)
{
    const uint32_t N = I.N;
    // suffix minima of each resource, for feasibility
    std::vector<int64_t> sufW(N + 1, 0), sufT(N + 1, 0);
    for (int i = (int)N - 1; i >= 0; --i) {
        int64_t mw = kInf64, mt = kInf64;
        for (const Item& it : I.items[i]) { mw = std::min(mw, it.w); mt = std::min(mt, it.t); }
        sufW[i] = sufW[i + 1] + mw; sufT[i] = sufT[i + 1] + mt;
    }
    if (sufW[0] > I.B1 || sufT[0] > I.B2) return BAOC_ERR_INFEASIBLE;

    // multipliers: alternate the two one-dimensional dual maximisations a few times
    Heuristic H;
    double l1 = 0.0, l2 = 0.0;
    for (int round = 0; round < 3; ++round) {
        const double n1 = bisect(I, true, l2, H);
        const double n2 = bisect(I, false, n1, H);
        const bool same = (n1 == l1 && n2 == l2);
        l1 = n1; l2 = n2;
        if (same) break;
    }
    improve(I, H);
    greedy_descent(I, H);

    std::vector<Multiplier> mult;
    mult.push_back(to_integer(l1, l2));
    mult.push_back(to_integer(0.0, 0.0));
    if (l1 > 0) { mult.push_back(to_integer(l1 * 0.5, l2)); mult.push_back(to_integer(l1 * 2.0, l2)); mult.push_back(to_integer(l1, 0.0)); }
    if (l2 > 0) { mult.push_back(to_integer(l1, l2 * 0.5)); mult.push_back(to_integer(l1, l2 * 2.0)); mult.push_back(to_integer(0.0, l2)); }
    const size_t M = mult.size();
    // sufRC[m][k] = sum over blocks >= k of the least reduced cost, minus the budget terms
    std::vector<std::vector<i128>> sufRC(M, std::vector<i128>(N + 1));
    for (size_t m = 0; m < M; ++m) {
        sufRC[m][N] = -(mult[m].L1 * (i128)I.B1 + mult[m].L2 * (i128)I.B2);
        for (int i = (int)N - 1; i >= 0; --i) {
            i128 best = 0; bool first = true;
            for (const Item& it : I.items[i]) {
                const i128 rc = (i128)it.phi * mult[m].S + mult[m].L1 * (i128)it.w + mult[m].L2 * (i128)it.t;
                if (first || rc < best) { best = rc; first = false; }
            }
            sufRC[m][i] = sufRC[m][i + 1] + best;
        }
    }
    // double images of the multipliers: a bound far from the cutoff is decided in floating point,
    // only a near miss is evaluated exactly
    std::vector<double> Sd(M), L1d(M), L2d(M);
    std::vector<std::vector<double>> sufRCd(M, std::vector<double>(N + 1));
    for (size_t m = 0; m < M; ++m) {
        Sd[m] = (double)mult[m].S; L1d[m] = (double)mult[m].L1; L2d[m] = (double)mult[m].L2;
        for (uint32_t i = 0; i <= N; ++i) sufRCd[m][i] = (double)sufRC[m][i];
    }
    int64_t z_max = 0;                                 // no assignment costs more than this
    for (uint32_t i = 0; i < N; ++i) {
        int64_t mx = I.items[i][0].phi;
        for (const Item& it : I.items[i]) mx = std::max(mx, it.phi);
        z_max += mx;
    }
    const int64_t ub = H.have ? H.Z : z_max;

    const uint64_t limit = g_node_limit ? g_node_limit : kDefaultNodeLimit;
    std::vector<Node> arena;
    std::vector<State> cur, nxt;
    std::vector<uint32_t> order;
    std::vector<uint8_t> dead;
    std::vector<std::pair<int64_t, Key>> stair;        // (T, best key among kept states with time <= T), T ascending

    // run(cutoff, level_cap): build the state lists for this cutoff.  A run that ends with states
    // has kept every prefix of every assignment of value <= cutoff that is not dominated.
    enum { kRunOk = 0, kRunEmpty = 1, kRunCapped = 2, kRunLimit = 3 };
    std::vector<float> slacks;
    auto run = [&](int64_t cutoff, size_t level_cap, size_t beam) -> int {
        arena.clear();
        arena.push_back({0xffffffffu, 0});
        cur.assign(1, State{0, 0, 0, 0, 0.f});
        bool empty = false;
        for (uint32_t i = 0; i < N && !empty; ++i) {
            nxt.clear();
            for (const State& s : cur) {
                for (uint32_t k = 0; k < I.items[i].size(); ++k) {
                    const Item& it = I.items[i][k];
                    State c{s.Z + it.phi, s.W + it.w, s.T + it.t, 0, 0.f};
                    if (c.W + sufW[i + 1] > I.B1 || c.T + sufT[i + 1] > I.B2) continue;
                    bool cut = false;
                    for (size_t m = 0; m < M && !cut; ++m) {
                        const double a = (double)c.Z * Sd[m], b = L1d[m] * (double)c.W, d = L2d[m] * (double)c.T;
                        const double lhs_d = a + b + d + sufRCd[m][i + 1], rhs_d = (double)cutoff * Sd[m];
                        if (m == 0) c.slack = (float)((rhs_d - lhs_d) / Sd[0]);
                        const double tol = 1e-9 * (std::fabs(a) + b + std::fabs(d) + std::fabs(sufRCd[m][i + 1]) + std::fabs(rhs_d));
                        if (lhs_d > rhs_d + tol) { cut = true; break; }
                        if (lhs_d < rhs_d - tol) continue;
                        const i128 lhs = (i128)c.Z * mult[m].S + mult[m].L1 * (i128)c.W + mult[m].L2 * (i128)c.T + sufRC[m][i + 1];
                        cut = lhs > (i128)cutoff * mult[m].S;
                    }
                    if (cut) continue;
                    if (arena.size() >= limit || arena.size() >= 0xfffffff0ull) return kRunLimit;
                    c.node = (uint32_t)arena.size();
                    arena.push_back({s.node, k});
                    nxt.push_back(c);
                }
            }
            if (nxt.empty()) { empty = true; break; }
            // dominance: sweep by (W, T, key); staircase over T of the best key seen
            const size_t n = nxt.size();
            if (n > 1) {
                order.resize(n);
                for (size_t j = 0; j < n; ++j) order[j] = (uint32_t)j;
                std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
                    const State &x = nxt[a], &y = nxt[b];
                    if (x.W != y.W) return x.W < y.W;
                    if (x.T != y.T) return x.T < y.T;
                    if (x.Z != y.Z) return x.Z < y.Z;
                    return a < b;
                });
                dead.assign(n, 0);
                stair.clear();
                for (uint32_t j : order) {
                    const State& s = nxt[j];
                    const Key key{s.Z, j};
                    // first entry with T > s.T; the one before it holds the best key with time <= s.T
                    auto it = std::upper_bound(stair.begin(), stair.end(), s.T,
                                               [](int64_t t, const std::pair<int64_t, Key>& e) { return t < e.first; });
                    if (it != stair.begin() && std::prev(it)->second < key) { dead[j] = 1; continue; }
                    if (it != stair.begin() && std::prev(it)->first == s.T) {
                        --it;
                        it->second = key;
                    } else {
                        it = stair.insert(it, std::make_pair(s.T, key));
                    }
                    auto nx = std::next(it), e = nx;
                    while (e != stair.end() && !(e->second < key)) ++e;   // entries to the right that are no better
                    stair.erase(nx, e);
                }
                size_t o = 0;
                for (size_t j = 0; j < n; ++j)
                    if (!dead[j]) nxt[o++] = nxt[j];
                nxt.resize(o);
            }
            if (beam && nxt.size() > beam) {              // heuristic mode: keep the most promising states
                slacks.resize(nxt.size());
                for (size_t j = 0; j < nxt.size(); ++j) slacks[j] = nxt[j].slack;
                std::nth_element(slacks.begin(), slacks.begin() + (nxt.size() - beam), slacks.end());
                const float thr = slacks[nxt.size() - beam];
                size_t o = 0;
                for (size_t j = 0; j < nxt.size() && o < beam; ++j)
                    if (nxt[j].slack >= thr) nxt[o++] = nxt[j];
                nxt.resize(o);
            }
            cur.swap(nxt);
            if (cur.size() > level_cap) return kRunCapped;
        }
        return empty ? kRunEmpty : kRunOk;
    };
    // First try the incumbent itself as cutoff: the heuristics usually land within 1e-4 of the
    // optimum and then one pass is all there is.  If the lists grow large the incumbent was poor:
    // a beam-limited pass of the same recursion finds a better one, then the exact pass is repeated.
    const size_t no_cap = std::numeric_limits<size_t>::max();
    int64_t cut = ub;
    int rc = run(cut, 20000, 0);
    if (rc == kRunCapped) {
        rc = run(cut, no_cap, 1024);
        if (rc == kRunOk)
            for (const State& st : cur) cut = std::min(cut, st.Z);
        rc = run(cut, no_cap, 0);
    }
    if (rc == kRunLimit) return BAOC_ERR_LIMIT;
    if (rc == kRunEmpty) return BAOC_ERR_INFEASIBLE;
    // best final state: least Z, then earliest in lexicographic order
    size_t best = 0;
    for (size_t j = 1; j < cur.size(); ++j)
        if (cur[j].Z < cur[best].Z) best = j;
    answer.assign(N, 0);
    uint32_t node = cur[best].node;
    for (int i = (int)N - 1; i >= 0; --i) { answer[i] = I.items[i][arena[node].item].cfg; node = arena[node].parent; }
    return BAOC_OK;
}

}  // namespace

extern "C" void baoc_allocate_set_node_limit(uint64_t max_nodes) { g_node_limit = max_nodes; }

extern "C" int baoc_allocate(const double* risk, const int64_t* mem, const double* time_cost,
                             uint32_t N, uint32_t K, int64_t mem_budget, double time_budget_sum,
                             const uint8_t* forbidden,
                             uint32_t* out_choice, double* out_objective, int64_t* out_mem, double* out_time)
{
    if (!risk || !mem || !time_cost || !out_choice || N == 0 || K == 0) return BAOC_ERR_INVALID;
    if (time_budget_sum != time_budget_sum) return BAOC_ERR_INVALID;
    Instance I;
    I.N = N; I.items.resize(N);
    I.B1 = mem_budget;
    I.B2 = std::llround(clampd(time_budget_sum, -9e12, 9e12) * kTauScale);
    i128 sum_phi = 0, sum_w = 0, sum_t = 0;
    std::vector<int64_t> phi_all((size_t)N * K), tau_all((size_t)N * K);
    for (uint32_t i = 0; i < N; ++i) {
        i128 mp = 0, mw = 0, mt = 0;
        for (uint32_t c = 0; c < K; ++c) {
            const size_t k = (size_t)i * K + c;
            if (mem[k] < 0) return BAOC_ERR_INVALID;
            const bool ok = !(forbidden && forbidden[k]) && std::isfinite(risk[k]) && std::isfinite(time_cost[k]);
            if (!ok) continue;
            Item it;
            it.phi = std::llround(clampd(risk[k], -kPhiClamp, kPhiClamp) * kPhiScale);
            it.t = std::llround(clampd(time_cost[k], -kPhiClamp, kPhiClamp) * kTauScale);
            it.w = mem[k]; it.cfg = c;
            phi_all[k] = it.phi; tau_all[k] = it.t;
            I.items[i].push_back(it);
            mp = std::max<i128>(mp, it.phi < 0 ? -(i128)it.phi : (i128)it.phi);
            mw = std::max<i128>(mw, it.w); mt = std::max<i128>(mt, it.t < 0 ? -(i128)it.t : (i128)it.t);
        }
        if (I.items[i].empty()) return BAOC_ERR_INFEASIBLE;
        sum_phi += mp; sum_w += mw; sum_t += mt;
    }
    const i128 cap = (i128)4000000000000000000ll;
    if (sum_phi > cap || sum_w > cap || sum_t > cap) return BAOC_ERR_UNSUPPORTED;
    for (uint32_t i = 0; i < N; ++i) drop_dominated(I.items[i]);

    std::vector<uint32_t> x;
    const int rc = solve(I, x);
    if (rc) return rc;
    int64_t Z = 0, W = 0, T = 0;
    for (uint32_t i = 0; i < N; ++i) {
        const size_t k = (size_t)i * K + x[i];
        Z += phi_all[k]; W += mem[k]; T += tau_all[k];
    }
    for (uint32_t i = 0; i < N; ++i) out_choice[i] = x[i];
    if (out_objective) *out_objective = (double)Z / kPhiScale;
    if (out_mem) *out_mem = W;
    if (out_time) *out_time = (double)T / kTauScale;
    return BAOC_OK;
}
