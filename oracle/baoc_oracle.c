/*
 * CPU oracle for the BAOC gradient-stream profiler, risk table and allocation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, sequential, obviously
 * correct statement of what the method computes.  It shares no code with the
 * HIP library; only tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it.  The product path never does.
 *
 * Precision.  The per-coordinate EMA states m, v are 32-bit floats (the
 * "32-bit" state of Eq. 8 / the fp32 Adam state of the StateMem definition)
 * and are advanced with one fixed sequence of fp32 operations, so that every
 * decision a quantiser takes (a bf16 rounding, an 8-bit code) is a function
 * of bit-identical inputs on both sides.  Everything that is derived from the
 * states (sums, update directions, cosines, errors, quantiles, risk) is
 * evaluated in fp64.  Build with -ffp-contract=off and without -ffast-math
 * so that each fp32 operation below is rounded exactly once, as written.
 *
 * Pins (tests/test_oracle_*.py): closed forms of the EMA, cosine special
 * cases, exactly representable values under both quantisers, error bounds of
 * the quantisers, quantiles against a sort-based library routine, chi-square
 * anisotropy of isotropic noise, the normalisation constants of App. A,
 * Agg(c) of Eq. 1, the order of NaN and +inf in the quantile against a library
 * sort, the distance of the fp32 state sequence from the same definitions in
 * fp64 throughout, and for the allocation exhaustive enumeration, a dense
 * dynamic programme and a depth-first branch and bound checked against both.
 * The end-to-end trajectory on a workload is parity unpinned against the
 * paper: it prints no statistic, risk or allocation.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Profiler state of one parameter block B_i (Sec. 3.1, Sec. 3.3)      */
/* ------------------------------------------------------------------ */

typedef struct {
    uint64_t d;          /* d_i, coordinates in the block (Omega_i = all)   */
    uint32_t t;          /* sampled steps seen                              */
    uint32_t n_cos;      /* cosines folded into rho_bar                     */
    uint32_t qb;         /* coordinates per 8-bit quantisation group        */
    float beta_m, beta_v;
    double beta_rho, eps;
    float eps_u;
    float *m, *v, *p;    /* m-hat, v-hat, previous gradient g_{t-1}         */
    double rho_bar, cos_last;
    double S_gg, S_pp, S_gp;      /* |g_t|^2, |g_{t-1}|^2, <g_t, g_{t-1}>   */
    double S_mm, S_v1, S_vv;      /* |m|^2, |v|_1, |v|^2                     */
    double U0;                    /* |u32|^2                                */
    double U1[2], U2[2];          /* <u32,u^b>, |u^b|^2 ; index 0: b=16, 1: b=8 */
    double Em[2], Ev[2];          /* |m^b - m|^2, |v^b - v|^2               */
} orc_block;

orc_block *orc_block_new(uint64_t d, float beta_m, float beta_v, double beta_rho,
                         double eps, float eps_u, uint32_t qb)
{
    orc_block *b = (orc_block *)calloc(1, sizeof(orc_block));
    if (!b) return NULL;
    b->d = d; b->qb = qb;
    b->beta_m = beta_m; b->beta_v = beta_v; b->beta_rho = beta_rho;
    b->eps = eps; b->eps_u = eps_u;
    b->m = (float *)calloc(d ? d : 1, sizeof(float));
    b->v = (float *)calloc(d ? d : 1, sizeof(float));
    b->p = (float *)calloc(d ? d : 1, sizeof(float));
    if (!b->m || !b->v || !b->p) { free(b->m); free(b->v); free(b->p); free(b); return NULL; }
    return b;
}

void orc_block_free(orc_block *b)
{
    if (!b) return;
    free(b->m); free(b->v); free(b->p); free(b);
}

const float *orc_block_m(const orc_block *b) { return b->m; }
const float *orc_block_v(const orc_block *b) { return b->v; }
const float *orc_block_p(const orc_block *b) { return b->p; }

/* bf16 storage: the upper 16 bits of an IEEE binary32. Widening is exact. */
static float bf16_widen(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16; float f; memcpy(&f, &u, 4); return f;
}

/* Round-to-nearest-even of a binary32 to the bf16 grid, returned as binary32. */
static float bf16_round(float x)
{
    uint32_t u; memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) {        /* NaN stays NaN */
        u |= 0x00400000u; u &= 0xffff0000u;
    } else {
        u += 0x7fffu + ((u >> 16) & 1u);
        u &= 0xffff0000u;
    }
    float r; memcpy(&r, &u, 4); return r;
}

float orc_bf16_round(float x) { return bf16_round(x); }

/*
 * Block-wise absmax linear 8-bit quantiser (the reading of the "standard
 * quantizer" of Eq. 8 for b = 8).  a = the group's absmax, L = 127 for the
 * signed first moment, 255 for the non-negative second moment.  The integer
 * code is decided in fp32:  k = rint_fp32( x (*) (L (/) a) ), ties to even,
 * with (*) and (/) the correctly rounded binary32 operations; when L/a is not
 * finite (a == 0, or so small that the scale overflows) every code is 0.
 * The de-quantised value a*k/L is formed in fp64.
 */
static double q8_dequant(float x, float a, float L)
{
    float s = L / a;
    if (!(s < INFINITY)) return 0.0;
    float k = rintf(x * s);
    return (double)a * (double)k / (double)L;
}

float orc_q8_code(float x, float a, float L)
{
    float s = L / a;
    if (!(s < INFINITY)) return 0.0f;
    return rintf(x * s);
}

/* One sampled step for one block; g widened exactly to binary32 beforehand. */
static void block_step(orc_block *b, const float *g)
{
    const uint64_t d = b->d;
    const float bm = b->beta_m, bv = b->beta_v;
    const float om_m = 1.0f - bm, om_v = 1.0f - bv;      /* 1 - beta, in fp32 */
    b->t += 1;

    /* Eq. 3: m <- beta_m m + (1-beta_m) g ; v <- beta_v v + (1-beta_v) g*g.
       fp32: the new term is rounded, then one fused multiply-add. */
    for (uint64_t j = 0; j < d; ++j) {
        float tm = om_m * g[j];
        float tv = (om_v * g[j]) * g[j];
        b->m[j] = fmaf(bm, b->m[j], tm);
        b->v[j] = fmaf(bv, b->v[j], tv);
    }

    /* Eq. 5 (left): cosine of consecutive gradients, EMA with beta_rho.
       The first step has no predecessor and leaves rho_bar untouched; the
       first cosine initialises it. NaN cosines count as 0 (App. A.1). */
    double S_gg = 0.0, S_gp = 0.0;
    for (uint64_t j = 0; j < d; ++j) {
        S_gg += (double)g[j] * (double)g[j];
        S_gp += (double)g[j] * (double)b->p[j];
    }
    b->S_gg = S_gg; b->S_gp = (b->t >= 2) ? S_gp : 0.0;
    if (b->t >= 2) {
        double c = S_gp / (sqrt(S_gg) * sqrt(b->S_pp) + b->eps);
        if (isnan(c)) c = 0.0;
        b->cos_last = c;
        if (b->n_cos == 0) b->rho_bar = c;
        else b->rho_bar = b->beta_rho * b->rho_bar + (1.0 - b->beta_rho) * c;
        b->n_cos += 1;
    }
    memcpy(b->p, g, d * sizeof(float));
    b->S_pp = S_gg;

    /* Eq. 5 (right): the sums behind rho_snr = |m|^2 / (|v|_1 + eps). */
    double S_mm = 0.0, S_v1 = 0.0, S_vv = 0.0;
    for (uint64_t j = 0; j < d; ++j) {
        double m = b->m[j], v = b->v[j];
        S_mm += m * m; S_v1 += v; S_vv += v * v;
    }
    b->S_mm = S_mm; b->S_v1 = S_v1; b->S_vv = S_vv;

    /* Eq. 8: update direction u = m / (sqrt(v) + eps_u) from the 32-bit state
       and from the state after a one-shot quantise/de-quantise to b bits. */
    double U0 = 0.0, U1[2] = {0, 0}, U2[2] = {0, 0}, Em[2] = {0, 0}, Ev[2] = {0, 0};
    const double eu = (double)b->eps_u;
    for (uint64_t s = 0; s < d; s += b->qb) {
        uint64_t e = s + b->qb < d ? s + b->qb : d;
        float a_m = 0.0f, a_v = 0.0f;              /* group absmax (NaN ignored) */
        for (uint64_t j = s; j < e; ++j) {
            a_m = fmaxf(a_m, fabsf(b->m[j]));
            a_v = fmaxf(a_v, b->v[j]);
        }
        for (uint64_t j = s; j < e; ++j) {
            double m = b->m[j], v = b->v[j];
            double u32 = m / (sqrt(v) + eu);
            double mq[2], vq[2];
            mq[0] = bf16_round(b->m[j]);          vq[0] = bf16_round(b->v[j]);
            mq[1] = q8_dequant(b->m[j], a_m, 127.0f);
            vq[1] = q8_dequant(b->v[j], a_v, 255.0f);
            U0 += u32 * u32;
            for (int k = 0; k < 2; ++k) {
                double ub = mq[k] / (sqrt(vq[k]) + eu);
                U1[k] += u32 * ub;
                U2[k] += ub * ub;
                Em[k] += (mq[k] - m) * (mq[k] - m);
                Ev[k] += (vq[k] - v) * (vq[k] - v);
            }
        }
    }
    b->U0 = U0;
    for (int k = 0; k < 2; ++k) { b->U1[k] = U1[k]; b->U2[k] = U2[k]; b->Em[k] = Em[k]; b->Ev[k] = Ev[k]; }
}

int orc_block_step_f32(orc_block *b, const float *g) { block_step(b, g); return 0; }

int orc_block_step_bf16(orc_block *b, const uint16_t *g)
{
    float *w = (float *)malloc((b->d ? b->d : 1) * sizeof(float));
    if (!w) return -1;
    for (uint64_t j = 0; j < b->d; ++j) w[j] = bf16_widen(g[j]);
    block_step(b, w);
    free(w);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Sparse coordinate sampling (Sec. 3.1)                               */
/* ------------------------------------------------------------------ */

/* |Omega_i| = ceil(s d_i), at least 1 and at most d_i. */
uint64_t orc_sample_count(uint64_t d, double s)
{
    double k = ceil(s * (double)d);
    if (!(k >= 1.0)) k = 1.0;
    if (k > (double)d) k = (double)d;
    return (uint64_t)k;
}

static uint64_t mix64(uint64_t x)
{
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

/* Omega_i is drawn once and then fixed.  Reading of "sample a subset of coordinates":
   a stratified uniform draw -- cut {0..d-1} into k = |Omega_i| strata
   [floor(j d / k), floor((j+1) d / k)) and take one coordinate of each, chosen by a
   64-bit mix of (seed, block, j).  Indices come out ascending; s = 1 gives every coordinate. */
void orc_sample_indices(uint64_t d, uint64_t k, uint64_t seed, uint32_t block, uint64_t *out)
{
    const uint64_t key = mix64(mix64(seed) + block);
    for (uint64_t j = 0; j < k; ++j) {
        uint64_t lo = (uint64_t)(((unsigned __int128)j * d) / k);
        uint64_t hi = (uint64_t)(((unsigned __int128)(j + 1) * d) / k);
        uint64_t h = mix64(key + (j + 1) * 0x9E3779B97F4A7C15ull);
        out[j] = lo + h % (hi - lo);
    }
}

/* Matrix form of the sampled coordinates.  Eq. 7 is stated on "the matrix form of the sampled gradients"
   while Sec. 3.1 fixes only the count.  Reading: for a rows x cols block Omega is a product set of r rows
   and c columns, so that the sampled coordinates are a sub-matrix (row-major in the compact buffer):
   r = round(rows sqrt(s)) within [1, rows], c = the least count with r c >= ceil(s d), at most cols.
   Returns 1 and the shape when both r and c are at least 2; 0 when the block has no matrix shape or the
   sample is too thin for one (then the flat draw above applies and F = 0). */
int orc_sample_matrix_shape(uint32_t rows, uint32_t cols, double s, uint32_t *r_out, uint32_t *c_out)
{
    if (rows < 2 || cols < 2) return 0;
    uint64_t target = orc_sample_count((uint64_t)rows * cols, s);
    double rr = floor((double)rows * sqrt(s) + 0.5);
    if (!(rr >= 1.0)) rr = 1.0;
    if (rr > (double)rows) rr = (double)rows;
    uint64_t r = (uint64_t)rr, c = (target + r - 1) / r;
    if (c > cols) c = cols;
    if (r < 2 || c < 2) return 0;
    *r_out = (uint32_t)r; *c_out = (uint32_t)c;
    return 1;
}

/* The r rows and c columns are drawn like the coordinates of the flat draw: one out of each of r (c) equal
   strata of the row (column) range, by a 64-bit mix of (seed, block, axis, stratum).  out[a c + b] is the
   position of (row a, column b) inside the block, ascending. */
void orc_sample_indices_matrix(uint32_t rows, uint32_t cols, uint32_t r, uint32_t c, uint64_t seed, uint32_t block,
                               uint64_t *out)
{
    const uint64_t key = mix64(mix64(seed) + block);
    const uint64_t key_r = mix64(key + 0x52), key_c = mix64(key + 0x43);
    uint64_t *col = (uint64_t *)malloc((size_t)c * 8);
    for (uint64_t b = 0; b < c; ++b) {
        uint64_t lo = b * cols / c, hi = (b + 1) * cols / c;
        col[b] = lo + mix64(key_c + (b + 1) * 0x9E3779B97F4A7C15ull) % (hi - lo);
    }
    for (uint64_t a = 0; a < r; ++a) {
        uint64_t lo = a * rows / r, hi = (a + 1) * rows / r;
        uint64_t row = lo + mix64(key_r + (a + 1) * 0x9E3779B97F4A7C15ull) % (hi - lo);
        for (uint64_t b = 0; b < c; ++b) out[a * c + b] = row * cols + col[b];
    }
    free(col);
}

/* ------------------------------------------------------------------ */
/* Finalize: raw metrics, normalisation (App. A) and risk (Eq. 9)      */
/* ------------------------------------------------------------------ */

typedef struct {
    uint64_t numel; uint32_t steps; uint32_t n_cos;
    double rho_bar, cos_last, snr, A, q10, q90;
    double Q16, Q8, lQ32, lQ16, lQ8;
    double err_m16, err_v16, err_m8, err_v8;
    double s_A, s_rho, s_snr, s_M, C_tilde, s_F;
    double m_sq, v_l1, g_sq_last;
    double C, F;                  /* raw Eq. 6 / Eq. 7 values that produced C_tilde and s_F */
} orc_stats;

typedef struct {
    double gamma, A_low, A_high, rho_low, rho_high, eta_low, eta_high;
    int use_snr_gate;
    double lambda_pref;
} orc_risk_params;

/* ascending; a NaN (only possible after a non-finite gradient) ranks above +inf */
static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    int nx = isnan(x), ny = isnan(y);
    if (nx || ny) return nx - ny;
    return (x > y) - (x < y);
}

/* q-th quantile: linear interpolation between the order statistics that
   bracket position q (d-1) of the ascending sort. */
static double quantile_sorted(const double *s, uint64_t d, double q)
{
    double pos = q * (double)(d - 1);
    uint64_t lo = (uint64_t)floor(pos);
    uint64_t hi = lo + 1 < d ? lo + 1 : d - 1;
    return s[lo] + (pos - (double)lo) * (s[hi] - s[lo]);
}

double orc_quantile(const float *x, uint64_t d, double q)
{
    double *s = (double *)malloc(d * sizeof(double));
    for (uint64_t j = 0; j < d; ++j) s[j] = x[j];
    qsort(s, d, sizeof(double), cmp_double);
    double r = quantile_sorted(s, d, q);
    free(s);
    return r;
}

/* Eq. 7: structure residual of a matrix block.  S = EMA(G*G) is the second moment v-hat
   viewed as a rows x cols matrix (row-major).  S~ is the rank-1 matrix built from the
   row means r, the column means c and the grand mean mu: S~_ij = r_i c_j / mu
   (S~ = 0 when mu = 0).  F = |S - S~|_F / (|S|_F + eps).  Blocks that are not matrices
   have nothing to factor: F = 0. */
double orc_block_structure_residual(const orc_block *b, uint32_t rows, uint32_t cols)
{
    if (rows == 0 || cols == 0 || (uint64_t)rows * cols != b->d) return 0.0;
    double *r = (double *)calloc(rows, sizeof(double)), *c = (double *)calloc(cols, sizeof(double));
    double mu = 0.0;
    for (uint32_t i = 0; i < rows; ++i)
        for (uint32_t j = 0; j < cols; ++j) {
            double s = b->v[(uint64_t)i * cols + j];
            r[i] += s; c[j] += s; mu += s;
        }
    for (uint32_t i = 0; i < rows; ++i) r[i] /= (double)cols;
    for (uint32_t j = 0; j < cols; ++j) c[j] /= (double)rows;
    mu /= (double)rows * (double)cols;
    double num = 0.0, den = 0.0;
    for (uint32_t i = 0; i < rows; ++i)
        for (uint32_t j = 0; j < cols; ++j) {
            double s = b->v[(uint64_t)i * cols + j];
            double st = mu != 0.0 ? r[i] * c[j] / mu : 0.0;
            num += (s - st) * (s - st);
            den += s * s;
        }
    free(r); free(c);
    return sqrt(num) / (sqrt(den) + b->eps);
}

/* Eq. 6: distortion of the weight-decay direction by the preconditioner
   p = 1 / (sqrt(v-hat) + eps), p-bar its mean over the block:
   C = |(p / p-bar - 1) * theta| / (|theta| + eps).  theta: the block's parameters. */
double orc_block_distortion(const orc_block *b, const float *theta)
{
    double pbar = 0.0;
    for (uint64_t j = 0; j < b->d; ++j) pbar += 1.0 / (sqrt((double)b->v[j]) + b->eps);
    pbar /= (double)b->d;
    double num = 0.0, den = 0.0;
    for (uint64_t j = 0; j < b->d; ++j) {
        double p = 1.0 / (sqrt((double)b->v[j]) + b->eps);
        double t = theta[j];
        double x = (p / pbar - 1.0) * t;
        num += x * x; den += t * t;
    }
    return sqrt(num) / (sqrt(den) + b->eps);
}

static double clip(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

/* Eq. 8 then the clip of Eq. 10 (to [eps,1]; NaN -> 0 first) */
static double cosine_Q(double U1, double U0, double U2, double eps)
{
    double q = U1 / (sqrt(U0) * sqrt(U2) + eps);
    if (isnan(q)) q = 0.0;
    return clip(q, eps, 1.0);
}

int orc_block_finalize(const orc_block *b, const orc_risk_params *rp, double C_raw, double F_raw,
                       orc_stats *o)
{
    const double eps = b->eps;
    memset(o, 0, sizeof(*o));
    o->numel = b->d; o->steps = b->t; o->n_cos = b->n_cos;
    o->rho_bar = b->n_cos ? b->rho_bar : 0.0;
    o->cos_last = b->cos_last;
    o->m_sq = b->S_mm; o->v_l1 = b->S_v1; o->g_sq_last = b->S_gg;

    /* Eq. 5 right */
    o->snr = b->S_mm / (b->S_v1 + eps);

    /* Eq. 4: quantile ratio of v-hat */
    {
        double *s = (double *)malloc(b->d * sizeof(double));
        if (!s) return -1;
        for (uint64_t j = 0; j < b->d; ++j) s[j] = b->v[j];
        qsort(s, b->d, sizeof(double), cmp_double);
        o->q10 = quantile_sorted(s, b->d, 0.1);
        o->q90 = quantile_sorted(s, b->d, 0.9);
        free(s);
        o->A = log((o->q90 + eps) / (o->q10 + eps));
    }

    /* Eq. 8, Eq. 10 (clip), Eq. 20 (l_Q = -log(Q + eps)) */
    double Q32 = cosine_Q(b->U0, b->U0, b->U0, eps);
    o->Q16 = cosine_Q(b->U1[0], b->U0, b->U2[0], eps);
    o->Q8  = cosine_Q(b->U1[1], b->U0, b->U2[1], eps);
    o->lQ32 = -log(Q32 + eps);
    o->lQ16 = -log(o->Q16 + eps);
    o->lQ8  = -log(o->Q8 + eps);

    /* relative L2 error of the states themselves in the cheaper precisions */
    o->err_m16 = sqrt(b->Em[0]) / (sqrt(b->S_mm) + eps);
    o->err_m8  = sqrt(b->Em[1]) / (sqrt(b->S_mm) + eps);
    o->err_v16 = sqrt(b->Ev[0]) / (sqrt(b->S_vv) + eps);
    o->err_v8  = sqrt(b->Ev[1]) / (sqrt(b->S_vv) + eps);

    /* App. A: Eq. 12 (s_A), Eq. 14 (s_rho), Eq. 16 (s_snr), Eq. 17 (s_M),
       Eq. 18 (C-tilde), Eq. 19 (s_F) */
    o->s_A   = clip((o->A - rp->A_low) / (rp->A_high - rp->A_low), 0.0, 1.0);
    o->s_rho = clip((o->rho_bar - rp->rho_low) / (rp->rho_high - rp->rho_low), 0.0, 1.0);
    o->s_snr = clip((log(1.0 + o->snr) - rp->eta_low) / (rp->eta_high - rp->eta_low), 0.0, 1.0);
    o->s_M   = rp->use_snr_gate ? o->s_rho * o->s_snr : o->s_rho;
    o->C = C_raw; o->F = F_raw;
    o->C_tilde = log(1.0 + C_raw);
    o->s_F   = clip(F_raw, 0.0, 1.0);
    return 0;
}

/* Eq. 1: Agg(c) = (1-y_a)+(1-y_m)+(1-y_d)+y_f+32/b-1 */
double orc_agg(int y_a, int y_m, int y_d, int y_f, int bits)
{
    return (1 - y_a) + (1 - y_m) + (1 - y_d) + y_f + 32.0 / (double)bits - 1.0;
}

/* Eq. 9 (= Eq. 21) with the soft preference of Sec. 3.2 and the regulariser of Eq. 1:
   Phi = R - lambda_pref [c in C_pref] + gamma Agg(c). cfg = (y_a,y_m,y_d,y_f,bits). */
double orc_phi(const orc_stats *z, const uint8_t cfg[5], int preferred, const orc_risk_params *rp)
{
    int y_a = cfg[0], y_m = cfg[1], y_d = cfg[2], y_f = cfg[3], bits = cfg[4];
    double lQ = bits == 32 ? z->lQ32 : (bits == 16 ? z->lQ16 : z->lQ8);
    double R = z->s_A * (1 - y_a) + z->s_M * (1 - y_m) + z->C_tilde * (1 - y_d) + z->s_F * y_f + lQ;
    if (preferred) R -= rp->lambda_pref;
    return R + rp->gamma * orc_agg(y_a, y_m, y_d, y_f, bits);
}

/* ------------------------------------------------------------------ */
/* Allocation (Eq. 2): exact reference solvers                          */
/* ------------------------------------------------------------------ */

#define ORC_OK 0
#define ORC_INFEASIBLE (-5)
#define ORC_TOO_BIG (-6)
#define ORC_INVALID (-1)

#define PHI_SCALE 1e9
#define PHI_CLAMP 1e6
#define TAU_SCALE 1e6

/* Integer instance: phi = llround(Phi 1e9) with |Phi| clamped to 1e6,
   tau = llround(r 1e6); a pair is excluded when forbidden (hard constraint of
   Sec. 3.2) or when its risk or time is not finite. */
typedef struct {
    uint32_t N, K;
    int64_t *phi, *mem, *tau;
    uint8_t *ok;
    int64_t B_mem, B_tau;
} int_instance;

static int integerise(const double *risk, const int64_t *mem, const double *time,
                      uint32_t N, uint32_t K, int64_t B_mem, double time_budget_sum,
                      const uint8_t *forbidden, int_instance *I)
{
    size_t n = (size_t)N * K;
    I->N = N; I->K = K;
    I->phi = (int64_t *)malloc(n * 8); I->mem = (int64_t *)malloc(n * 8);
    I->tau = (int64_t *)malloc(n * 8); I->ok = (uint8_t *)malloc(n);
    I->B_mem = B_mem;
    double tb = time_budget_sum;
    if (isnan(tb)) return ORC_INVALID;
    if (tb > 9e12) tb = 9e12;           /* "no limit": beyond any sum of clamped tau */
    if (tb < -9e12) tb = -9e12;
    I->B_tau = llround(tb * TAU_SCALE);
    for (size_t k = 0; k < n; ++k) {
        int ok = !(forbidden && forbidden[k]) && isfinite(risk[k]) && isfinite(time[k]);
        if (mem[k] < 0) return ORC_INVALID;
        I->ok[k] = (uint8_t)ok;
        double r = ok ? clip(risk[k], -PHI_CLAMP, PHI_CLAMP) : 0.0;
        double t = ok ? clip(time[k], -PHI_CLAMP, PHI_CLAMP) : 0.0;
        I->phi[k] = llround(r * PHI_SCALE);
        I->tau[k] = llround(t * TAU_SCALE);
        I->mem[k] = mem[k];
    }
    return ORC_OK;
}

static void inst_free(int_instance *I) { free(I->phi); free(I->mem); free(I->tau); free(I->ok); }

static void report(const int_instance *I, const uint32_t *x, double *obj, int64_t *omem, double *otime)
{
    int64_t z = 0, m = 0, t = 0;
    for (uint32_t i = 0; i < I->N; ++i) {
        size_t k = (size_t)i * I->K + x[i];
        z += I->phi[k]; m += I->mem[k]; t += I->tau[k];
    }
    if (obj) *obj = (double)z / PHI_SCALE;
    if (omem) *omem = m;
    if (otime) *otime = (double)t / TAU_SCALE;
}

/* Exhaustive enumeration of all K^N assignments in lexicographic order
   (block 1 most significant); a later assignment replaces the incumbent only
   when strictly better, so ties resolve to the lexicographically smallest. */
int orc_allocate_brute(const double *risk, const int64_t *mem, const double *time,
                       uint32_t N, uint32_t K, int64_t B_mem, double time_budget_sum,
                       const uint8_t *forbidden, uint32_t *out_choice,
                       double *out_obj, int64_t *out_mem, double *out_time)
{
    if (pow((double)K, (double)N) > 2e8) return ORC_TOO_BIG;
    int_instance I;
    int rc = integerise(risk, mem, time, N, K, B_mem, time_budget_sum, forbidden, &I);
    if (rc) { inst_free(&I); return rc; }
    uint32_t *x = (uint32_t *)calloc(N, 4), *best = (uint32_t *)calloc(N, 4);
    int found = 0; int64_t zbest = 0;
    for (;;) {
        int64_t z = 0, m = 0, t = 0; int ok = 1;
        for (uint32_t i = 0; i < N; ++i) {
            size_t k = (size_t)i * K + x[i];
            if (!I.ok[k]) { ok = 0; break; }
            z += I.phi[k]; m += I.mem[k]; t += I.tau[k];
        }
        if (ok && m <= I.B_mem && t <= I.B_tau && (!found || z < zbest)) {
            found = 1; zbest = z; memcpy(best, x, N * 4);
        }
        int i = (int)N - 1;                       /* odometer, last block fastest */
        while (i >= 0 && ++x[i] == K) { x[i] = 0; --i; }
        if (i < 0) break;
    }
    if (found) { memcpy(out_choice, best, N * 4); report(&I, best, out_obj, out_mem, out_time); }
    free(x); free(best); inst_free(&I);
    return found ? ORC_OK : ORC_INFEASIBLE;
}

static int64_t gcd64(int64_t a, int64_t b) { while (b) { int64_t t = a % b; a = b; b = t; } return a < 0 ? -a : a; }

/* Textbook multiple-choice-knapsack dynamic programme over the two resource
   rows.  f_i(w,t) = least objective of blocks i..N-1 within remaining
   capacities (w,t) (in units of the gcd of each row).  The forward
   reconstruction takes, block by block, the smallest configuration index
   that still reaches the optimum: the lexicographically smallest optimum. */
int orc_allocate_dp(const double *risk, const int64_t *mem, const double *time,
                    uint32_t N, uint32_t K, int64_t B_mem, double time_budget_sum,
                    const uint8_t *forbidden, uint32_t *out_choice,
                    double *out_obj, int64_t *out_mem, double *out_time)
{
    int_instance I;
    int rc = integerise(risk, mem, time, N, K, B_mem, time_budget_sum, forbidden, &I);
    if (rc) { inst_free(&I); return rc; }
    size_t n = (size_t)N * K;
    int64_t gm = 0, gt = 0, summ = 0, sumt = 0;
    for (uint32_t i = 0; i < N; ++i) {
        int64_t mm = 0, mt = 0;
        for (uint32_t c = 0; c < K; ++c) {
            size_t k = (size_t)i * K + c;
            if (!I.ok[k]) continue;
            if (I.tau[k] < 0) { inst_free(&I); return ORC_INVALID; }
            gm = gcd64(gm, I.mem[k]); gt = gcd64(gt, I.tau[k]);
            if (I.mem[k] > mm) mm = I.mem[k];
            if (I.tau[k] > mt) mt = I.tau[k];
        }
        summ += mm; sumt += mt;
    }
    if (gm == 0) gm = 1;
    if (gt == 0) gt = 1;
    if (I.B_mem < 0 || I.B_tau < 0) { inst_free(&I); return ORC_INFEASIBLE; }
    int64_t W = (I.B_mem < summ ? I.B_mem : summ) / gm;   /* capacities beyond the max sum are slack */
    int64_t T = (I.B_tau < sumt ? I.B_tau : sumt) / gt;
    if ((double)(W + 1) * (double)(T + 1) * (double)(N + 1) > 3e8) { inst_free(&I); return ORC_TOO_BIG; }
    size_t plane = (size_t)(W + 1) * (size_t)(T + 1);
    const int64_t INF = INT64_MAX / 4;
    int64_t *f = (int64_t *)malloc((size_t)(N + 1) * plane * 8);
    for (size_t s = 0; s < plane; ++s) f[(size_t)N * plane + s] = 0;
    for (int i = (int)N - 1; i >= 0; --i)
        for (int64_t w = 0; w <= W; ++w)
            for (int64_t t = 0; t <= T; ++t) {
                int64_t best = INF;
                for (uint32_t c = 0; c < K; ++c) {
                    size_t k = (size_t)i * K + c;
                    if (!I.ok[k]) continue;
                    int64_t dw = I.mem[k] / gm, dt = I.tau[k] / gt;
                    if (dw > w || dt > t) continue;
                    int64_t r = f[(size_t)(i + 1) * plane + (size_t)(w - dw) * (T + 1) + (size_t)(t - dt)];
                    if (r >= INF) continue;
                    if (I.phi[k] + r < best) best = I.phi[k] + r;
                }
                f[(size_t)i * plane + (size_t)w * (T + 1) + (size_t)t] = best;
            }
    int found = f[(size_t)0 * plane + (size_t)W * (T + 1) + (size_t)T] < INF;
    if (found) {
        int64_t w = W, t = T;
        for (uint32_t i = 0; i < N; ++i) {
            int64_t target = f[(size_t)i * plane + (size_t)w * (T + 1) + (size_t)t];
            for (uint32_t c = 0; c < K; ++c) {
                size_t k = (size_t)i * K + c;
                if (!I.ok[k]) continue;
                int64_t dw = I.mem[k] / gm, dt = I.tau[k] / gt;
                if (dw > w || dt > t) continue;
                int64_t r = f[(size_t)(i + 1) * plane + (size_t)(w - dw) * (T + 1) + (size_t)(t - dt)];
                if (r < INF && I.phi[k] + r == target) { out_choice[i] = c; w -= dw; t -= dt; break; }
            }
        }
        report(&I, out_choice, out_obj, out_mem, out_time);
    }
    (void)n;
    free(f); inst_free(&I);
    return found ? ORC_OK : ORC_INFEASIBLE;
}

/* Integer image of an instance, for tests that want to see phi / tau. */
int orc_integerise(const double *risk, const int64_t *mem, const double *time,
                   uint32_t N, uint32_t K, int64_t B_mem, double time_budget_sum,
                   const uint8_t *forbidden, int64_t *phi, int64_t *tau, uint8_t *ok, int64_t *B_tau)
{
    int_instance I;
    int rc = integerise(risk, mem, time, N, K, B_mem, time_budget_sum, forbidden, &I);
    if (!rc) {
        size_t n = (size_t)N * K;
        memcpy(phi, I.phi, n * 8); memcpy(tau, I.tau, n * 8); memcpy(ok, I.ok, n);
        *B_tau = I.B_tau;
    }
    inst_free(&I);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Allocation (Eq. 2): depth-first branch and bound                     */
/* ------------------------------------------------------------------ */

/*
 * The third exact method, for instances that neither the enumeration nor the
 * dynamic programme reaches.  Blocks are fixed in index order and, inside a
 * block, configurations are tried in index order, so complete assignments are
 * met in lexicographic order.  A complete assignment replaces the incumbent
 * only when it is strictly better; the first optimum met is therefore the
 * lexicographically smallest one and stays.
 *
 * Before the search, a configuration is struck from its block when another
 * allowed one needs no more of either row and has less risk, or the same risk
 * and a smaller index: exchanging it keeps an assignment feasible and makes it
 * better or lexicographically smaller, so the answer never contains it.
 *
 * A partial assignment (a prefix) is abandoned when
 *   - a row cannot be met any more (its use so far plus the least use of the
 *     open blocks exceeds the budget), or
 *   - weak duality shows that no completion reaches the cutoff: for any
 *     multipliers l1, l2 >= 0 every feasible completion has
 *       Z >= Z_fixed + l1 W_fixed + l2 T_fixed
 *            + sum over open blocks of min_c (phi + l1 mem + l2 tau) - l1 B_mem - l2 B_tau.
 *     The test is made in exact integers (multipliers are fractions L / S with
 *     S a power of two) for a fixed ladder of multiplier pairs around the pair
 *     that maximises the bound of the whole instance (found by alternating
 *     bisections; any pair >= 0 is valid, a good one only saves time).
 *     Pairs with S = 0 bound the rows alone: l1 W + l2 T of any completion
 *     against l1 B_mem + l2 B_tau, which abandons prefixes that no completion
 *     can bring inside both budgets at once; or
 *   - a prefix of the same depth with Z_fixed, W_fixed and T_fixed all no
 *     larger has been left before in this search: the open blocks are the
 *     same, whatever completes this prefix within the budgets completed that
 *     one too, with a total no larger; every such completion was abandoned or
 *     met then, and the cutoff can only have fallen since.  Left states are
 *     kept per depth (a list that is full simply stops growing).
 *
 * Cutoff.  All objective values lie on one lattice base + g Z (g = gcd of the
 * differences of phi inside the blocks), so "strictly better" means "better by
 * at least g": once a complete assignment of value z has been met, only totals
 * <= z - g are of interest.  Until then totals <= `cut` are accepted, and
 * cut = U works, U being the value of a feasible assignment (Lagrangian
 * minimisers that happen to be feasible, improved by single exchanges; the sum
 * of the largest risks when none is known).  On a coarse lattice (at most 64
 * values between the bound of the whole instance and U) the search is instead
 * run with the rising starting cutoffs low, low + g, ...: a search that meets
 * nothing proves that the optimum lies above its starting cutoff, the first
 * search that meets something returns the answer, and the searched window
 * stays narrow even when U is poor.
 *
 * A node limit over all searches ends the call with ORC_TOO_BIG and no answer.
 */
typedef __int128 i128;

static uint64_t bnb_node_limit = 2000000000ull;
static uint64_t bnb_last_nodes = 0;

void orc_allocate_bnb_set_node_limit(uint64_t n) { bnb_node_limit = n ? n : 2000000000ull; }
uint64_t orc_allocate_bnb_last_nodes(void) { return bnb_last_nodes; }

/* Minimiser of phi + l1 mem + l2 tau in every block (ties: less memory, then less time, then
   the smaller index); returns its exact sums. */
static void lagrangian_pick(const int_instance *I, double l1, double l2, uint32_t *pick,
                            int64_t *Z, int64_t *W, int64_t *T)
{
    *Z = *W = *T = 0;
    for (uint32_t i = 0; i < I->N; ++i) {
        int have = 0; double best = 0.0; size_t bk = 0;
        for (uint32_t c = 0; c < I->K; ++c) {
            size_t k = (size_t)i * I->K + c;
            if (!I->ok[k]) continue;
            double v = (double)I->phi[k] + l1 * (double)I->mem[k] + l2 * (double)I->tau[k];
            int better = !have || v < best ||
                         (v == best && (I->mem[k] < I->mem[bk] || (I->mem[k] == I->mem[bk] && I->tau[k] < I->tau[bk])));
            if (better) { have = 1; best = v; bk = k; }
        }
        pick[i] = (uint32_t)(bk - (size_t)i * I->K);
        *Z += I->phi[bk]; *W += I->mem[bk]; *T += I->tau[bk];
    }
}

typedef struct { const int_instance *I; uint32_t *pick, *best; int have; int64_t U; } bnb_start;

/* Does the minimiser at (l1, l2) exceed row `row`?  A minimiser inside both budgets is a
   feasible assignment: its value is an upper bound on the optimum. */
static int row_exceeded(bnb_start *s, double l1, double l2, int row)
{
    int64_t Z, W, T;
    lagrangian_pick(s->I, l1, l2, s->pick, &Z, &W, &T);
    if (W <= s->I->B_mem && T <= s->I->B_tau && (!s->have || Z < s->U)) {
        s->have = 1; s->U = Z; memcpy(s->best, s->pick, s->I->N * 4);
    }
    return row == 0 ? W > s->I->B_mem : T > s->I->B_tau;
}

/* Least multiplier of one row (the other fixed) at which the minimiser meets that row. */
static double bisect_row(bnb_start *s, int row, double other)
{
    double lo = 0.0, hi = 1.0;
    if (!(row == 0 ? row_exceeded(s, 0.0, other, 0) : row_exceeded(s, other, 0.0, 1))) return 0.0;
    while ((row == 0 ? row_exceeded(s, hi, other, 0) : row_exceeded(s, other, hi, 1)) && hi < 1e18) hi *= 4.0;
    if (hi >= 1e18) return 1e18;
    for (int it = 0; it < 80; ++it) {
        double mid = 0.5 * (lo + hi);
        if (row == 0 ? row_exceeded(s, mid, other, 0) : row_exceeded(s, other, mid, 1)) lo = mid; else hi = mid;
    }
    return hi;
}

/* Lower the upper bound by single exchanges: while some block can move to another allowed
   configuration with less risk and both rows still hold, take the exchange that gains most. */
static void exchange_descent(bnb_start *s)
{
    const int_instance *I = s->I;
    if (!s->have) return;
    int64_t W = 0, T = 0;
    for (uint32_t i = 0; i < I->N; ++i) { size_t k = (size_t)i * I->K + s->best[i]; W += I->mem[k]; T += I->tau[k]; }
    for (;;) {
        int64_t gain = 0; uint32_t bi = 0, bc = 0;
        for (uint32_t i = 0; i < I->N; ++i) {
            size_t cur = (size_t)i * I->K + s->best[i];
            for (uint32_t c = 0; c < I->K; ++c) {
                size_t k = (size_t)i * I->K + c;
                if (!I->ok[k]) continue;
                if (I->phi[cur] - I->phi[k] > gain && W - I->mem[cur] + I->mem[k] <= I->B_mem &&
                    T - I->tau[cur] + I->tau[k] <= I->B_tau) { gain = I->phi[cur] - I->phi[k]; bi = i; bc = c; }
            }
        }
        if (gain == 0) return;
        size_t cur = (size_t)bi * I->K + s->best[bi], k = (size_t)bi * I->K + bc;
        W += I->mem[k] - I->mem[cur]; T += I->tau[k] - I->tau[cur];
        s->U -= gain; s->best[bi] = bc;
    }
}

/* States (Z, W, T) of one depth whose subtree has been searched to the end; only those that no
   other one undercuts in all three are kept. */
typedef struct { int64_t *Z, *W, *T; uint32_t n, cap; } left_list;
enum { LEFT_MAX = 1024 };                /* a list that is full simply stops growing */

/* Has a state been left at this depth that had fixed no more risk and used no more of either row? */
static int left_covers(const left_list *l, int64_t Z, int64_t W, int64_t T)
{
    for (uint32_t j = 0; j < l->n; ++j)
        if (l->Z[j] <= Z && l->W[j] <= W && l->T[j] <= T) return 1;
    return 0;
}

static void left_add(left_list *l, int64_t Z, int64_t W, int64_t T)
{
    uint32_t o = 0;
    for (uint32_t j = 0; j < l->n; ++j)               /* drop what the new state makes redundant */
        if (!(Z <= l->Z[j] && W <= l->W[j] && T <= l->T[j])) { l->Z[o] = l->Z[j]; l->W[o] = l->W[j]; l->T[o] = l->T[j]; ++o; }
    l->n = o;
    if (l->n >= LEFT_MAX) return;
    if (l->n == l->cap) {
        uint32_t cap = l->cap ? 2 * l->cap : 16;
        int64_t *z = (int64_t *)realloc(l->Z, cap * 8), *w = (int64_t *)realloc(l->W, cap * 8), *t = (int64_t *)realloc(l->T, cap * 8);
        if (z) l->Z = z;
        if (w) l->W = w;
        if (t) l->T = t;
        if (!z || !w || !t) return;                   /* no room: the state is simply not recorded */
        l->cap = cap;
    }
    l->Z[l->n] = Z; l->W[l->n] = W; l->T[l->n] = T; l->n += 1;
}

enum { BNB_MAXM = 26 + 7 };

typedef struct {
    const int_instance *I;
    int64_t *sufW, *sufT;                /* least use of each row by the blocks i..N-1           */
    int64_t g;                           /* lattice step of the objective                        */
    int M;                               /* multiplier pairs                                     */
    i128 S[BNB_MAXM], L1[BNB_MAXM], L2[BNB_MAXM], bud[BNB_MAXM];
    i128 *rcst;                          /* [m][i*K+c]: S phi + L1 mem + L2 tau                  */
    i128 *suf;                           /* [m][i]: sum over blocks >= i of the least rcst       */
    i128 *pre;                           /* [m][depth]: sum of rcst over the fixed blocks        */
    uint32_t *x, *best, *next;
    int64_t *Zp, *Wp, *Tp;
    left_list *left;                     /* [depth] */
    uint64_t nodes;
} bnb_ctx;

/* One lexicographic depth-first search that accepts totals <= cut.  Returns 1 when a complete
   assignment was met (c->best then holds the lexicographically smallest optimum), 0 when none
   has a total <= cut, -1 when the node limit was reached. */
static int bnb_search(bnb_ctx *c, int64_t cut)
{
    const int_instance *I = c->I;
    const uint32_t N = I->N, K = I->K;
    const size_t NK = (size_t)N * K, N1 = (size_t)N + 1;
    int found = 0;
    for (uint32_t d = 0; d <= N; ++d) c->left[d].n = 0;
    int i = 0;
    c->next[0] = 0; c->Zp[0] = c->Wp[0] = c->Tp[0] = 0;
    for (int m = 0; m < c->M; ++m) c->pre[(size_t)m * N1] = 0;
    while (i >= 0) {
        if ((uint32_t)i == N) {                    /* complete, inside both rows, total <= cut */
            found = 1; memcpy(c->best, c->x, N * 4);
            cut = c->Zp[N] - c->g;
            --i;
            continue;
        }
        int went_down = 0;
        for (uint32_t cfg = c->next[i]; cfg < K; ++cfg) {
            size_t k = (size_t)i * K + cfg;
            if (!I->ok[k]) continue;
            if (++c->nodes > bnb_node_limit) return -1;
            int64_t W = c->Wp[i] + I->mem[k], T = c->Tp[i] + I->tau[k];
            if (W + c->sufW[i + 1] > I->B_mem || T + c->sufT[i + 1] > I->B_tau) continue;
            int hopeless = 0;
            for (int m = 0; m < c->M && !hopeless; ++m) {
                i128 lhs = c->pre[(size_t)m * N1 + i] + c->rcst[(size_t)m * NK + k] + c->suf[(size_t)m * N1 + i + 1] - c->bud[m];
                hopeless = lhs > c->S[m] * (i128)cut;
            }
            if (hopeless) continue;
            if (left_covers(&c->left[i + 1], c->Zp[i] + I->phi[k], W, T)) continue;
            c->x[i] = cfg; c->next[i] = cfg + 1;
            c->Zp[i + 1] = c->Zp[i] + I->phi[k]; c->Wp[i + 1] = W; c->Tp[i + 1] = T;
            for (int m = 0; m < c->M; ++m)
                c->pre[(size_t)m * N1 + i + 1] = c->pre[(size_t)m * N1 + i] + c->rcst[(size_t)m * NK + k];
            ++i; c->next[i] = 0;
            went_down = 1;
            break;
        }
        if (!went_down) {                          /* every completion of this prefix has been dealt with */
            left_add(&c->left[i], c->Zp[i], c->Wp[i], c->Tp[i]);
            --i;
        }
    }
    return found;
}

static int64_t clamp_mult(double x) { return llround(x < 4e18 ? x : 4e18); }

int orc_allocate_bnb(const double *risk, const int64_t *mem, const double *time,
                     uint32_t N, uint32_t K, int64_t B_mem, double time_budget_sum,
                     const uint8_t *forbidden, uint32_t *out_choice,
                     double *out_obj, int64_t *out_mem, double *out_time)
{
    int_instance I;
    int rc = integerise(risk, mem, time, N, K, B_mem, time_budget_sum, forbidden, &I);
    if (rc) { inst_free(&I); return rc; }
    bnb_last_nodes = 0;
    const size_t NK = (size_t)N * K, N1 = (size_t)N + 1;

    /* strike configurations that another one of the same block makes pointless (see above) */
    for (uint32_t b = 0; b < N; ++b)
        for (uint32_t c = 0; c < K; ++c) {
            size_t k = (size_t)b * K + c;
            if (!I.ok[k]) continue;
            for (uint32_t e = 0; e < K; ++e) {
                size_t q = (size_t)b * K + e;
                if (e == c || !I.ok[q]) continue;   /* a struck one (ok == 2) still shows that k is pointless */
                if (I.mem[q] <= I.mem[k] && I.tau[q] <= I.tau[k] &&
                    (I.phi[q] < I.phi[k] || (I.phi[q] == I.phi[k] && e < c))) { I.ok[k] = 2; break; }
            }
        }
    for (size_t k = 0; k < NK; ++k)
        if (I.ok[k] == 2) I.ok[k] = 0;

    bnb_ctx C;
    memset(&C, 0, sizeof(C));
    C.I = &I;
    C.sufW = (int64_t *)calloc(N1, 8); C.sufT = (int64_t *)calloc(N1, 8);
    int64_t zmax = 0;
    int dead_block = 0;
    double sum_mem = 0.0, spreadW = 1.0, spreadT = 1.0;
    for (int i = (int)N - 1; i >= 0; --i) {
        int have = 0; int64_t lw = 0, hw = 0, lt = 0, ht = 0, first_phi = 0, hphi = 0;
        for (uint32_t c = 0; c < K; ++c) {
            size_t k = (size_t)i * K + c;
            if (!I.ok[k]) continue;
            if (!have) { have = 1; lw = hw = I.mem[k]; lt = ht = I.tau[k]; first_phi = hphi = I.phi[k]; }
            if (I.mem[k] < lw) lw = I.mem[k];
            if (I.mem[k] > hw) hw = I.mem[k];
            if (I.tau[k] < lt) lt = I.tau[k];
            if (I.tau[k] > ht) ht = I.tau[k];
            if (I.phi[k] > hphi) hphi = I.phi[k];
            C.g = gcd64(C.g, I.phi[k] - first_phi);
        }
        if (!have) dead_block = 1;
        C.sufW[i] = C.sufW[i + 1] + lw; C.sufT[i] = C.sufT[i + 1] + lt;
        zmax += hphi; sum_mem += (double)hw;
        spreadW += (double)(hw - lw); spreadT += (double)(ht - lt);
    }
    if (C.g == 0) C.g = 1;
    if (sum_mem > 4e18) rc = ORC_TOO_BIG;
    else if (dead_block || C.sufW[0] > I.B_mem || C.sufT[0] > I.B_tau) rc = ORC_INFEASIBLE;
    if (rc) { free(C.sufW); free(C.sufT); inst_free(&I); return rc; }

    /* multipliers of the whole instance, and an upper bound from the minimisers seen on the way */
    bnb_start st; st.I = &I; st.pick = (uint32_t *)calloc(N, 4); st.best = (uint32_t *)calloc(N, 4); st.have = 0; st.U = 0;
    double l1 = 0.0, l2 = 0.0;
    for (int round = 0; round < 3; ++round) {
        l1 = bisect_row(&st, 0, l2);
        l2 = bisect_row(&st, 1, l1);
    }
    exchange_descent(&st);
    const int64_t U = st.have ? st.U : zmax;      /* some assignment inside both rows has a total <= U */

    /* ladder of multiplier pairs (steps of 5 % on either axis) as exact fractions L / S; pair 0 is (l1, l2) itself */
    static const double step[5] = {1.0, 1.0 / 1.05, 1.05, 1.0 / 1.1025, 1.1025};
    for (int a = 0; a < 5; ++a)
        for (int b = 0; b < 5; ++b) {
            if ((a > 0 && l1 == 0.0) || (b > 0 && l2 == 0.0)) continue;
            double m1 = l1 * step[a], m2 = l2 * step[b];
            double mx = m1 > m2 ? m1 : m2;
            int k = 40;
            while (k > 0 && ldexp(mx, k) > 4e18) --k;
            C.S[C.M] = (i128)1 << k;
            C.L1[C.M] = (i128)clamp_mult(ldexp(m1, k));
            C.L2[C.M] = (i128)clamp_mult(ldexp(m2, k));
            ++C.M;
        }
    C.S[C.M] = 1; C.L1[C.M] = 0; C.L2[C.M] = 0; ++C.M;          /* (0,0): the plain objective bound */
    {   /* the rows alone (S = 0): weights theta / spread of the memory row, (1 - theta) / spread of the time row */
        static const double theta[7] = {0.5, 0.25, 0.75, 0.1, 0.9, 0.02, 0.98};
        for (int a = 0; a < 7; ++a) {
            C.S[C.M] = 0;
            C.L1[C.M] = (i128)clamp_mult(ldexp(theta[a] / spreadW, 62));
            C.L2[C.M] = (i128)clamp_mult(ldexp((1.0 - theta[a]) / spreadT, 62));
            ++C.M;
        }
    }

    /* reduced costs, their least value per block summed over the open blocks, the budget terms */
    C.rcst = (i128 *)malloc((size_t)C.M * NK * sizeof(i128));
    C.suf = (i128 *)malloc((size_t)C.M * N1 * sizeof(i128));
    C.pre = (i128 *)malloc((size_t)C.M * N1 * sizeof(i128));
    for (int m = 0; m < C.M; ++m) {
        C.bud[m] = C.L1[m] * (i128)I.B_mem + C.L2[m] * (i128)I.B_tau;
        C.suf[(size_t)m * N1 + N] = 0;
        for (int i = (int)N - 1; i >= 0; --i) {
            int have = 0; i128 least = 0;
            for (uint32_t c = 0; c < K; ++c) {
                size_t k = (size_t)i * K + c;
                i128 v = C.S[m] * (i128)I.phi[k] + C.L1[m] * (i128)I.mem[k] + C.L2[m] * (i128)I.tau[k];
                C.rcst[(size_t)m * NK + k] = v;
                if (!I.ok[k]) continue;
                if (!have || v < least) { have = 1; least = v; }
            }
            C.suf[(size_t)m * N1 + i] = C.suf[(size_t)m * N1 + i + 1] + least;
        }
    }
    C.x = (uint32_t *)calloc(N, 4); C.best = (uint32_t *)calloc(N, 4); C.next = (uint32_t *)calloc(N1, 4);
    C.Zp = (int64_t *)calloc(N1, 8); C.Wp = (int64_t *)calloc(N1, 8); C.Tp = (int64_t *)calloc(N1, 8);
    C.left = (left_list *)calloc(N1, sizeof(left_list));

    /* Smallest lattice value the bound of the whole instance allows: the optimum Z* satisfies
       S Z* >= suf[0][0] - bud[0], and Z* = U - j g for some j >= 0. */
    int64_t low = U;
    {
        i128 lb = C.suf[0] - C.bud[0];                         /* scaled by S[0] */
        i128 room = (i128)U * C.S[0] - lb;                     /* S (U - LB) */
        if (room > 0) {
            i128 j = room / (C.S[0] * (i128)C.g);              /* floor((U - LB) / g) */
            low = U - (int64_t)j * C.g;
        }
    }
    /* rising starting cutoffs low, low + g, ... up to U while only a few lattice values lie between
       (a coarse lattice: ties are everywhere and a poor U costs most); otherwise U at once */
    int found = 0;
    int64_t cut = (U - low) / C.g <= 64 ? low : U;
    for (;;) {
        found = bnb_search(&C, cut);
        if (found || cut >= U) break;
        cut += C.g;
    }
    bnb_last_nodes = C.nodes;
    if (found == 1) { memcpy(out_choice, C.best, N * 4); report(&I, C.best, out_obj, out_mem, out_time); }
    free(C.x); free(C.best); free(C.next); free(C.Zp); free(C.Wp); free(C.Tp);
    for (uint32_t d = 0; d <= N; ++d) { free(C.left[d].Z); free(C.left[d].W); free(C.left[d].T); }
    free(C.left);
    free(C.rcst); free(C.suf); free(C.pre); free(st.pick); free(st.best); free(C.sufW); free(C.sufT); inst_free(&I);
    if (found < 0) return ORC_TOO_BIG;
    return found ? ORC_OK : ORC_INFEASIBLE;
}
