// baoc_allocate: exact solver of the allocation problem of Eq. 2 -- one
// configuration per block, a memory row and a time row -- with the hard
// exclusions of Sec. 3.2 and a canonical answer (lexicographically smallest
// optimum of the integer image of the instance).
//
// Method: list recursions over the blocks, three in a row.
//   Lists.  For one ordering of the blocks ("levels"), lists[i] holds states (Z, W, T) = sums of
//   (phi, mem, tau) over some choice for the levels i..N-1.  A state is dropped when
//     - no choice for the levels before i can complete it within the budgets (least use of each row),
//     - a Lagrangian bound of the levels before i shows that no completion reaches the cutoff (weak
//       duality, decided in floating point and, on a near miss, exactly in 128-bit integers, for a small
//       grid of multiplier pairs around the maximiser of the dual of the whole instance), or
//     - another state of the same level is no larger in all of Z, W and T: whatever completes the worse
//       one completes the better one too, with a total no larger.
//   A row that no earlier level can push over its budget any more does not constrain a state: its use is
//   raised to that threshold, so that more states undercut each other.
//   1. The optimal value Z*.  Levels ordered by how firmly the multipliers decide a block (undecided blocks
//      first, i.e. processed last).  Cutoffs rise from the smallest lattice value the bound of the whole
//      instance allows (all totals lie on base + g Z, g the gcd of the phi differences inside the blocks): a
//      run that ends empty proves that the optimum lies above its cutoff; the first run that reaches level 0
//      holds Z*.
//   2. The configurations that occur in optimal assignments at all: a forward pass over the same levels keeps
//      a state of the levels before i, extended by a configuration of level i, when a state of lists[i+1]
//      completes it to Z* within both rows.
//   3. The canonical optimum.  The recursion once more in index order, over those configurations only, with
//      Z* as cutoff.  Its lists hold, for every optimal assignment and every i, a state that undercuts the
//      assignment's part on the blocks i..N-1, so the lexicographically smallest optimum is read off in
//      index order: block i takes the smallest configuration for which some state of lists[i+1] completes
//      the prefix to Z* within both rows.
// The lists are capped by a node limit: when it is hit the call fails rather than return a guess.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <new>
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

thread_local uint64_t g_node_limit = 0, g_exact_work = 0;
thread_local uint32_t g_front_cap = 0;
constexpr uint64_t kDefaultNodeLimit = 32'000'000ull;      // states kept over all levels (24 bytes each)

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

// Best single swap that lowers the objective and stays within both budgets, repeated (at most 64 times:
// the incumbent only ends the rising cutoffs of solve(), it does not have to be good).
void improve(const Instance& I, Heuristic& H)
{
    if (!H.have) return;
    int64_t W = 0, T = 0;
    for (uint32_t i = 0; i < I.N; ++i) { const Item& it = I.items[i][H.pick[i]]; W += it.w; T += it.t; }
    for (uint32_t round = 0; round < 64; ++round) {
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

// A partial state: sums of (phi, mem, tau) over some choice for a run of consecutive levels.
struct State { int64_t Z, W, T; };

int64_t gcd64(int64_t a, int64_t b)
{
    if (a < 0) a = -a;
    if (b < 0) b = -b;
    while (b) { const int64_t t = a % b; a = b; b = t; }
    return a;
}

// For states added in any order: the least Z among those added with time <= t.
struct Stair {
    std::vector<std::pair<int64_t, int64_t>> e;        // (T, least Z among the added states with time <= T), T ascending, Z descending
    void clear() { e.clear(); }
    int64_t least(int64_t t) const
    {
        auto it = std::upper_bound(e.begin(), e.end(), t, [](int64_t x, const std::pair<int64_t, int64_t>& y) { return x < y.first; });
        return it == e.begin() ? kInf64 : std::prev(it)->second;
    }
    void add(int64_t t, int64_t z)
    {
        auto it = std::upper_bound(e.begin(), e.end(), t, [](int64_t x, const std::pair<int64_t, int64_t>& y) { return x < y.first; });
        if (it != e.begin() && std::prev(it)->second <= z) return;
        if (it != e.begin() && std::prev(it)->first == t) { --it; it->second = z; }
        else it = e.insert(it, std::make_pair(t, z));
        auto nx = std::next(it), r = nx;
        while (r != e.end() && r->second >= z) ++r;      // entries to the right that are no better
        e.erase(nx, r);
    }
};

// Keep the states that no other one undercuts (no larger in all of Z, W, T; of equal states one stays), in the
// order (W, T, Z) ascending.
void keep_undercut_free(std::vector<State>& cand, std::vector<State>& out, std::vector<uint32_t>& order, Stair& stair)
{
    const size_t n = cand.size();
    out.clear();
    order.resize(n);
    for (size_t j = 0; j < n; ++j) order[j] = (uint32_t)j;
    std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        const State &x = cand[a], &y = cand[b];
        if (x.W != y.W) return x.W < y.W;
        if (x.T != y.T) return x.T < y.T;
        return x.Z < y.Z;
    });
    stair.clear();
    for (uint32_t j : order) {
        const State& s = cand[j];
        if (stair.least(s.T) <= s.Z) continue;             // undercut (or equalled) by a state swept before
        stair.add(s.T, s.Z);
        out.push_back(s);
    }
}

enum { kRunOk = 0, kRunEmpty = 1, kRunLimit = 3 };
// The forward pass of Levels::viable is exact while it is cheap: after this many extended states (by default), fronts are cut
// down to a few hundred states per level (still marking every configuration it must, and then some more).
constexpr uint64_t kDefaultExactWork = 16'000'000ull;
constexpr size_t kDefaultFrontCap = 256;

// The list recursion over one ordering of the blocks ("levels"): lists[i] holds states of the levels i..N-1.
struct Levels {
    const Instance& I;
    const std::vector<Multiplier>& mult;
    uint32_t N;
    size_t M;
    // least and largest use of each row by the levels before i, for feasibility and for the clamp
    std::vector<int64_t> preMinW, preMinT, preMaxW, preMaxT;
    // preRC[m][i] = sum over the levels before i of the least reduced cost, minus the budget terms; and the
    // double images of the multipliers: a bound far from the cutoff is decided in floating point, only a near
    // miss is evaluated exactly
    std::vector<std::vector<i128>> preRC;
    std::vector<double> Sd, L1d, L2d;
    std::vector<std::vector<double>> preRCd;
    std::vector<std::vector<State>> lists;
    std::vector<State> cand;
    std::vector<uint32_t> order;
    Stair stair;

    Levels(const Instance& inst, const std::vector<Multiplier>& m)
        : I(inst), mult(m), N(inst.N), M(m.size()), preMinW(N + 1, 0), preMinT(N + 1, 0), preMaxW(N + 1, 0), preMaxT(N + 1, 0),
          preRC(M, std::vector<i128>(N + 1)), Sd(M), L1d(M), L2d(M), preRCd(M, std::vector<double>(N + 1)), lists(N + 1)
    {
        for (uint32_t i = 0; i < N; ++i) {
            int64_t lw = kInf64, lt = kInf64, hw = -kInf64, ht = -kInf64;
            for (const Item& it : I.items[i]) {
                lw = std::min(lw, it.w); lt = std::min(lt, it.t); hw = std::max(hw, it.w); ht = std::max(ht, it.t);
            }
            preMinW[i + 1] = preMinW[i] + lw; preMinT[i + 1] = preMinT[i] + lt;
            preMaxW[i + 1] = preMaxW[i] + hw; preMaxT[i + 1] = preMaxT[i] + ht;
        }
        for (size_t k = 0; k < M; ++k) {
            preRC[k][0] = -(mult[k].L1 * (i128)I.B1 + mult[k].L2 * (i128)I.B2);
            for (uint32_t i = 0; i < N; ++i) {
                i128 best = 0; bool first = true;
                for (const Item& it : I.items[i]) {
                    const i128 rc = (i128)it.phi * mult[k].S + mult[k].L1 * (i128)it.w + mult[k].L2 * (i128)it.t;
                    if (first || rc < best) { best = rc; first = false; }
                }
                preRC[k][i + 1] = preRC[k][i] + best;
            }
            Sd[k] = (double)mult[k].S; L1d[k] = (double)mult[k].L1; L2d[k] = (double)mult[k].L2;
            for (uint32_t i = 0; i <= N; ++i) preRCd[k][i] = (double)preRC[k][i];
        }
    }

    // Build the lists from the last level backwards.  A run that ends with states at level 0 has kept, for every
    // feasible assignment of value <= cutoff and every i, a state of lists[i] that undercuts (or equals) the part
    // of the assignment on the levels i..N-1.
    int run(int64_t cutoff, uint64_t limit)
    {
        uint64_t total = 1;
        lists[N].assign(1, State{0, 0, 0});
        for (int i = (int)N - 1; i >= 0; --i) {
            // A row that no choice for the levels before i can push over its budget any more is not a constraint
            // for the state: below the threshold every value is as good as the threshold itself, which lets more
            // states undercut others.
            const int64_t floorW = I.B1 - preMaxW[i], floorT = I.B2 - preMaxT[i];
            cand.clear();
            for (const State& s : lists[i + 1]) {
                for (const Item& it : I.items[i]) {
                    State c{s.Z + it.phi, std::max(s.W + it.w, floorW), std::max(s.T + it.t, floorT)};
                    if (c.W + preMinW[i] > I.B1 || c.T + preMinT[i] > I.B2) continue;
                    bool cut = false;
                    for (size_t m = 0; m < M && !cut; ++m) {
                        const double a = (double)c.Z * Sd[m], b = L1d[m] * (double)c.W, d = L2d[m] * (double)c.T;
                        const double lhs_d = a + b + d + preRCd[m][i], rhs_d = (double)cutoff * Sd[m];
                        const double tol = 1e-9 * (std::fabs(a) + std::fabs(b) + std::fabs(d) + std::fabs(preRCd[m][i]) + std::fabs(rhs_d));
                        if (lhs_d > rhs_d + tol) { cut = true; break; }
                        if (lhs_d < rhs_d - tol) continue;
                        const i128 lhs = (i128)c.Z * mult[m].S + mult[m].L1 * (i128)c.W + mult[m].L2 * (i128)c.T + preRC[m][i];
                        cut = lhs > (i128)cutoff * mult[m].S;
                    }
                    if (cut) continue;
                    cand.push_back(c);
                }
            }
            if (cand.empty()) return kRunEmpty;
            keep_undercut_free(cand, lists[i], order, stair);
            total += lists[i].size();
            if (total > limit) return kRunLimit;
        }
        return kRunOk;
    }

    // A long front is replaced by fewer, more optimistic states: runs of neighbours in (Z, W) order collapse to
    // their least Z, W and T (within one value of Z the times fall as the memory rises, so a run is a short piece
    // of that staircase and its stand-in the corner below it).  Whatever completes a member completes its
    // stand-in.  Runs stop at a change of Z unless the values of Z alone outnumber the cap.
    void thin(std::vector<State>& front, std::vector<State>& tmp, size_t cap)
    {
        std::sort(front.begin(), front.end(), [](const State& a, const State& b) { return a.Z != b.Z ? a.Z < b.Z : a.W < b.W; });
        const size_t n = front.size(), len = (n + cap - 1) / cap;
        size_t values = 1;
        for (size_t a = 1; a < n; ++a) values += front[a].Z != front[a - 1].Z;
        const bool across = values > cap;
        tmp.clear();
        for (size_t a = 0; a < n;) {
            State m = front[a];
            size_t b = a + 1;
            for (; b < std::min(n, a + len) && (across || front[b].Z == front[a].Z); ++b) {
                m.Z = std::min(m.Z, front[b].Z); m.W = std::min(m.W, front[b].W); m.T = std::min(m.T, front[b].T);
            }
            tmp.push_back(m);
            a = b;
        }
        keep_undercut_free(tmp, front, order, stair);
    }

    // After a run that reached level 0 with a cutoff >= z: marks every configuration that occurs in some feasible
    // assignment of value <= z (and, once the fronts are thinned, possibly some that do not).  Forward over the
    // levels: front holds states of the levels before i; a state extended by a configuration is kept
    // when some state of lists[i+1] completes it within z and both budgets, and the configuration is marked.
    // Nothing is missed: the parts of any assignment of value <= z before and after level i are undercut by a state
    // of front and of lists[i+1].  Until the fronts are thinned the marks are exact: a kept pair is an
    // assignment.
    int viable(int64_t z, std::vector<std::vector<uint8_t>>& mark)
    {
        struct Ext { State s; uint32_t k; };
        std::vector<Ext> ext;
        std::vector<State> front(1, State{0, 0, 0}), kept;
        uint64_t work = 0;
        const uint64_t exact_work = g_exact_work ? g_exact_work : kDefaultExactWork;
        const size_t front_cap = g_front_cap ? g_front_cap : kDefaultFrontCap;
        mark.assign(N, std::vector<uint8_t>());
        for (uint32_t i = 0; i < N; ++i) {
            mark[i].assign(I.items[i].size(), 0);
            // The clamp of run(), mirrored: a row that the levels after i cannot push over its budget any more does
            // not tell states of the levels 0..i apart (the second term keeps a clamped state within what those
            // levels can use at all, so that it still fits the clamped states of lists[i+1]).
            const int64_t floorW = std::min(I.B1 - (preMaxW[N] - preMaxW[i + 1]), preMaxW[i + 1]);
            const int64_t floorT = std::min(I.B2 - (preMaxT[N] - preMaxT[i + 1]), preMaxT[i + 1]);
            ext.clear();
            for (const State& p : front)
                for (uint32_t k = 0; k < I.items[i].size(); ++k) {
                    const Item& it = I.items[i][k];
                    ext.push_back(Ext{State{p.Z + it.phi, std::max(p.W + it.w, floorW), std::max(p.T + it.t, floorT)}, k});
                }
            work += ext.size();
            // most room in the memory row last: the states of lists[i+1] come in ascending W and enter the staircase as they fit
            std::sort(ext.begin(), ext.end(), [](const Ext& a, const Ext& b) { return a.s.W > b.s.W; });
            stair.clear();
            const std::vector<State>& next = lists[i + 1];
            size_t at = 0;
            kept.clear();
            for (const Ext& q : ext) {
                const int64_t roomW = I.B1 - q.s.W, roomT = I.B2 - q.s.T;
                while (at < next.size() && next[at].W <= roomW) { stair.add(next[at].T, next[at].Z); ++at; }
                if (stair.least(roomT) <= z - q.s.Z) { mark[i][q.k] = 1; kept.push_back(q.s); }
            }
            if (kept.empty()) return kRunEmpty;
            keep_undercut_free(kept, front, order, stair);
            if (work > exact_work && front.size() > front_cap) thin(front, kept, front_cap);
        }
        return kRunOk;
    }
};

int solve(const Instance& I, std::vector<uint32_t>& answer)
{
    const uint32_t N = I.N;
    int64_t g = 0;                                     // all totals lie on one lattice base + g Z
    {
        int64_t minW = 0, minT = 0;
        for (uint32_t i = 0; i < N; ++i) {
            int64_t lw = kInf64, lt = kInf64;
            for (const Item& it : I.items[i]) {
                lw = std::min(lw, it.w); lt = std::min(lt, it.t);
                g = gcd64(g, it.phi - I.items[i][0].phi);
            }
            minW += lw; minT += lt;
        }
        if (minW > I.B1 || minT > I.B2) return BAOC_ERR_INFEASIBLE;
    }
    if (g == 0) g = 1;

    // multipliers: alternate the two one-dimensional dual maximisations a few times, then polish the pair by a
    // pattern search on the dual value (alternation alone can stall at a kink of the piecewise linear dual)
    Heuristic H;
    double l1 = 0.0, l2 = 0.0;
    for (int round = 0; round < 3; ++round) {
        const double n1 = bisect(I, true, l2, H);
        const double n2 = bisect(I, false, n1, H);
        const bool same = (n1 == l1 && n2 == l2);
        l1 = n1; l2 = n2;
        if (same) break;
    }
    if (l1 < 1e29 && l2 < 1e29) {
        double best = eval_lagrangian(I, l1, l2).value;
        double r = 1.25;
        for (int it = 0; it < 60 && r > 1.0005; ++it) {
            double c1 = l1, c2 = l2, cv = best;
            for (int a = -1; a <= 1; ++a)
                for (int b = -1; b <= 1; ++b) {
                    if ((a == 0 && b == 0) || (a && l1 == 0.0) || (b && l2 == 0.0)) continue;
                    const double m1 = a == 0 ? l1 : (a > 0 ? l1 * r : l1 / r), m2 = b == 0 ? l2 : (b > 0 ? l2 * r : l2 / r);
                    std::vector<uint32_t> pick;
                    const double v = eval_lagrangian(I, m1, m2, &pick).value;
                    consider(I, pick, H);
                    if (v > cv) { cv = v; c1 = m1; c2 = m2; }
                }
            if (cv > best) { best = cv; l1 = c1; l2 = c2; }
            else r = std::sqrt(r);
        }
    }
    improve(I, H);

    // Bounds are taken under a small grid of multiplier pairs around the best pair (steps of 5 %): deeper in the
    // recursion the pair that bounds a state best drifts with the budgets the state has left.
    std::vector<Multiplier> mult;
    mult.push_back(to_integer(l1, l2));
    mult.push_back(to_integer(0.0, 0.0));
    for (int a = -2; a <= 2; ++a)
        for (int b = -2; b <= 2; ++b) {
            if ((a == 0 && b == 0) || (a && l1 == 0.0) || (b && l2 == 0.0)) continue;
            mult.push_back(to_integer(l1 * std::pow(1.05, a), l2 * std::pow(1.05, b)));
        }
    if (l1 > 0 && l2 > 0) { mult.push_back(to_integer(l1, 0.0)); mult.push_back(to_integer(0.0, l2)); }

    int64_t z_max = 0;                                 // no assignment costs more than this
    for (uint32_t i = 0; i < N; ++i) {
        int64_t mx = I.items[i][0].phi;
        for (const Item& it : I.items[i]) mx = std::max(mx, it.phi);
        z_max += mx;
    }
    const int64_t ub = H.have ? H.Z : z_max;           // some feasible assignment has a total <= ub (or none exists)
    const uint64_t limit = g_node_limit ? g_node_limit : kDefaultNodeLimit;

    // Step 1, the optimal value.  The order of the levels is free here, and it decides how long the lists get: blocks
    // whose best configuration under the multipliers leads the second best by a wide margin come last (they are
    // processed first and hardly branch, since any other choice fails the bound at once), the undecided blocks come
    // first, where the levels still to come are few and their bound is sharp.
    std::vector<uint32_t> perm(N);
    {
        const double m1 = l1 < 1e29 ? l1 : 0.0, m2 = l2 < 1e29 ? l2 : 0.0;
        std::vector<double> lead(N);
        for (uint32_t i = 0; i < N; ++i) {
            double lo = std::numeric_limits<double>::infinity(), lo2 = lo;
            for (const Item& it : I.items[i]) {
                const double rc = (double)it.phi + m1 * (double)it.w + m2 * (double)it.t;
                if (rc < lo) { lo2 = lo; lo = rc; } else if (rc < lo2) lo2 = rc;
            }
            lead[i] = lo2 - lo;                        // infinite for a block with one configuration
            perm[i] = i;
        }
        std::stable_sort(perm.begin(), perm.end(), [&](uint32_t a, uint32_t b) { return lead[a] < lead[b]; });
    }
    Instance J;
    J.N = N; J.B1 = I.B1; J.B2 = I.B2; J.items.resize(N);
    for (uint32_t j = 0; j < N; ++j) J.items[j] = I.items[perm[j]];
    Levels LJ(J, mult);

    // Cutoffs rise from the smallest lattice value that the bound of the whole instance allows towards the
    // incumbent: a run that ends empty proves that the optimum lies above its cutoff, the first run that reaches
    // level 0 holds the optimum.  The distance from the bound grows by half each time, so the last run looks at a
    // window at most 1.5 times wider than the one the optimum needs, however poor the incumbent is (the number of
    // surviving states grows steeply with that width), and the empty runs before it are cheap.
    int64_t low = ub;
    {
        const i128 room = (i128)ub * mult[0].S - LJ.preRC[0][N];               // S (ub - bound of the whole instance)
        if (room > 0) low = ub - (int64_t)(room / (mult[0].S * (i128)g)) * g;
    }
    int rc;
    {
        const int64_t span = (ub - low) / g;               // lattice steps from low to the incumbent
        int64_t at = 0, step = std::max<int64_t>(1, span >> 20);
        for (;;) {
            rc = LJ.run(low + at * g, limit);
            if (rc != kRunEmpty || at >= span) break;
            at = std::min(span, at + step);
            step = std::max(step + 1, step + step / 2);
        }
    }
    if (rc == kRunLimit) return BAOC_ERR_LIMIT;
    if (rc == kRunEmpty) return BAOC_ERR_INFEASIBLE;
    int64_t z_star = kInf64;                           // least Z among the states of level 0 (all of them are feasible)
    for (const State& s : LJ.lists[0]) z_star = std::min(z_star, s.Z);

    // Step 2, the configurations that occur in optimal assignments at all (usually one per block, or a few).
    std::vector<std::vector<uint8_t>> mark;
    rc = LJ.viable(z_star, mark);
    if (rc != kRunOk) return BAOC_ERR_LIMIT;           // cannot happen: an optimal assignment exists
    Instance R;
    R.N = N; R.B1 = I.B1; R.B2 = I.B2; R.items.resize(N);
    for (uint32_t j = 0; j < N; ++j)
        for (size_t k = 0; k < J.items[j].size(); ++k)
            if (mark[j][k]) R.items[perm[j]].push_back(J.items[j][k]);          // ascending configuration index, as in I
    LJ.lists.clear(); LJ.lists.shrink_to_fit();

    // Step 3, the canonical optimum: the recursion once more, in index order, over those configurations only and
    // with the optimal value as cutoff; then block by block the smallest configuration index for which some kept
    // state of the next list still completes the prefix to the optimal value within both budgets.
    Levels LR(R, mult);
    rc = LR.run(z_star, limit);
    if (rc != kRunOk) return BAOC_ERR_LIMIT;
    answer.assign(N, 0);
    int64_t Zp = 0, Wp = 0, Tp = 0;
    for (uint32_t i = 0; i < N; ++i) {
        bool placed = false;
        for (const Item& it : R.items[i]) {
            const int64_t z = Zp + it.phi, w = Wp + it.w, t = Tp + it.t;
            for (const State& s : LR.lists[i + 1])
                if (z + s.Z <= z_star && w + s.W <= I.B1 && t + s.T <= I.B2) { placed = true; break; }
            if (placed) { answer[i] = it.cfg; Zp = z; Wp = w; Tp = t; break; }
        }
        if (!placed) return BAOC_ERR_LIMIT;            // cannot happen: the lists hold a witness for every step
    }
    return BAOC_OK;
}

}  // namespace

extern "C" void baoc_allocate_set_node_limit(uint64_t max_nodes) { g_node_limit = max_nodes; }
extern "C" void baoc_allocate_set_exact_work(uint64_t max_states, uint32_t front_cap) { g_exact_work = max_states; g_front_cap = front_cap; }

static int allocate(const double* risk, const int64_t* mem, const double* time_cost,
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

// No exception crosses the C boundary: running out of host memory for the state lists is the same event as
// reaching the state limit.
extern "C" int baoc_allocate(const double* risk, const int64_t* mem, const double* time_cost,
                             uint32_t N, uint32_t K, int64_t mem_budget, double time_budget_sum,
                             const uint8_t* forbidden,
                             uint32_t* out_choice, double* out_objective, int64_t* out_mem, double* out_time)
{
    try {
        return allocate(risk, mem, time_cost, N, K, mem_budget, time_budget_sum, forbidden, out_choice, out_objective, out_mem, out_time);
    } catch (const std::bad_alloc&) {
        return BAOC_ERR_LIMIT;
    }
}
