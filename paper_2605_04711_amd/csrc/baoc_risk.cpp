// Host side of baoc_profile_finalize: raw sums of one block -> metrics of
// Sec. 3.3 -> normalised signals of App. A -> risk entries (Eq. 9, Eq. 1).
// O(N K) work on a few dozen doubles per block.
#include <cmath>
#include <cstring>

#include "baoc_internal.h"

namespace baoc {

static inline double clip(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

// Eq. 8 from the accumulated sums.  U1 = <u32,u^b> is available twice: summed
// directly, and as (|u32|^2 + |u^b|^2 - |u^b - u32|^2) / 2.  The second form
// keeps 1 - Q accurate when the two directions nearly coincide (fp32 partial
// sums cannot resolve 1 - Q ~ 1e-6 directly); the first is the accurate one
// when they differ a lot.  NaN -> 0, then the clip of Eq. 10.
static double cosine_Q(double U0, double U1, double U2, double D, double eps)
{
    if (D <= 0.0625 * (U0 + U2)) U1 = 0.5 * (U0 + U2 - D);
    double q = U1 / (std::sqrt(U0) * std::sqrt(U2) + eps);
    if (q != q) q = 0.0;
    return clip(q, eps, 1.0);
}

void block_metrics(const RawBlock& r, double eps, const baoc_risk_params& rp,
                   double C_raw, double F_raw, baoc_block_stats* o)
{
    std::memset(o, 0, sizeof(*o));
    const double* s = r.sums;
    o->numel = r.numel; o->steps = r.steps; o->n_cos = r.n_cos;
    o->rho_bar = r.n_cos ? r.rho_bar : 0.0;
    o->cos_last = r.cos_last;
    o->m_sq = s[S_MM]; o->v_l1 = s[S_V1]; o->g_sq_last = s[S_GG];

    o->snr = s[S_MM] / (s[S_V1] + eps);                                   // Eq. 5 right

    // Eq. 4: quantiles by linear interpolation between bracketing order statistics
    const double a0 = r.order_stat[0], a1 = r.order_stat[1], b0 = r.order_stat[2], b1 = r.order_stat[3];
    o->q10 = a0 + r.frac10 * (a1 - a0);
    o->q90 = b0 + r.frac90 * (b1 - b0);
    o->A = std::log((o->q90 + eps) / (o->q10 + eps));

    const double Q32 = cosine_Q(s[U0], s[U0], s[U0], 0.0, eps);
    o->Q16 = cosine_Q(s[U0], s[U1_16], s[U2_16], s[D_16], eps);
    o->Q8 = cosine_Q(s[U0], s[U1_8], s[U2_8], s[D_8], eps);
    o->lQ32 = -std::log(Q32 + eps);                                       // Eq. 20
    o->lQ16 = -std::log(o->Q16 + eps);
    o->lQ8 = -std::log(o->Q8 + eps);

    const double nm = std::sqrt(s[S_MM]) + eps, nv = std::sqrt(s[S_VV]) + eps;
    o->err_m16 = std::sqrt(s[EM_16]) / nm; o->err_v16 = std::sqrt(s[EV_16]) / nv;
    o->err_m8 = std::sqrt(s[EM_8]) / nm;   o->err_v8 = std::sqrt(s[EV_8]) / nv;

    o->s_A = clip((o->A - rp.A_low) / (rp.A_high - rp.A_low), 0.0, 1.0);                          // Eq. 12
    o->s_rho = clip((o->rho_bar - rp.rho_low) / (rp.rho_high - rp.rho_low), 0.0, 1.0);            // Eq. 14
    o->s_snr = clip((std::log(1.0 + o->snr) - rp.eta_low) / (rp.eta_high - rp.eta_low), 0.0, 1.0); // Eq. 16
    o->s_M = rp.use_snr_gate ? o->s_rho * o->s_snr : o->s_rho;                                    // Eq. 17
    o->C = C_raw; o->F = F_raw;
    o->C_tilde = std::log(1.0 + C_raw);                                                           // Eq. 18
    o->s_F = clip(F_raw, 0.0, 1.0);                                                               // Eq. 19
}

double config_phi(const baoc_block_stats& z, const baoc_config& c, bool preferred,
                  const baoc_risk_params& rp)
{
    const double lQ = c.bits == 32 ? z.lQ32 : (c.bits == 16 ? z.lQ16 : z.lQ8);
    double R = z.s_A * (1 - c.y_a) + z.s_M * (1 - c.y_m) + z.C_tilde * (1 - c.y_d) + z.s_F * c.y_f + lQ;
    if (preferred) R -= rp.lambda_pref;
    const double agg = (1 - c.y_a) + (1 - c.y_m) + (1 - c.y_d) + c.y_f + 32.0 / c.bits - 1.0;  // Eq. 1
    return R + rp.gamma * agg;
}

}  // namespace baoc

extern "C" void baoc_risk_params_default(baoc_risk_params* p)
{
    if (!p) return;
    p->gamma = 0.1;
    p->A_low = std::log(2.0); p->A_high = std::log(10.0);
    p->rho_low = 0.2; p->rho_high = 0.6;
    p->eta_low = 0.0; p->eta_high = 2.0;
    p->use_snr_gate = 1;
    p->lambda_pref = 0.0;
    p->pref_mask = nullptr; p->C_raw = nullptr; p->F_raw = nullptr;
    p->compute_F = 1; p->d_theta_flat = nullptr; p->theta_numel = 0; p->theta_dtype = BAOC_GRAD_F32;
}
