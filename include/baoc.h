/*
 * baoc.h -- C ABI of the BAOC gradient-stream profiler and allocator for
 * AMD Instinct MI355X (gfx950).
 *
 * BAOC (Budget-Aware Optimizer Configurator) assigns one optimizer
 * configuration to every parameter block under a memory and a time budget
 * (Sec. 3, Algorithm 1).  This library is the data-parallel part of it:
 *
 *   baoc_profile_begin     describe the blocks B_i of a flat gradient buffer
 *   baoc_profile_step      feed one sampled gradient g_t (one fused HBM pass)
 *   baoc_profile_finalize  per-block metrics z_i and the risk table Phi[i][c]
 *   baoc_allocate          exact solution of the allocation problem (Eq. 2)
 *   baoc_sample_*          optional front end: fixed index sets Omega_i and a gather (Sec. 3.1)
 *   baoc_partition         block partitioning over structural units (App. C.2, Algorithm 2)
 *
 * Conventions
 *   - Every function returns a status (BAOC_OK = 0, errors negative).  On an
 *     error no out-parameter has been written.
 *   - "d_" arguments are DEVICE pointers (HIP, current device); all other
 *     pointers are HOST pointers.
 *   - The caller owns every buffer it passes in, including the device
 *     workspace; the library owns only the opaque handle.
 *   - A handle is not thread safe; different handles are independent.
 *   - The profiler takes every coordinate of the blocks it is given (Omega_i = all of B_i);
 *     to profile a subset, gather it first (baoc_sample_*) and describe the compact buffer.
 */
#ifndef BAOC_H
#define BAOC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BAOC_OK                0
#define BAOC_ERR_INVALID      (-1)  /* null pointer, empty or overlapping blocks, bad parameter */
#define BAOC_ERR_WORKSPACE    (-2)  /* workspace too small or not 256-byte aligned */
#define BAOC_ERR_UNSUPPORTED  (-3)  /* parameter value this build has no kernel for */
#define BAOC_ERR_HIP          (-4)  /* HIP runtime error; sticky for the handle */
#define BAOC_ERR_INFEASIBLE   (-5)  /* no assignment satisfies the budgets */
#define BAOC_ERR_LIMIT        (-6)  /* solver node limit reached; no answer rather than a sub-optimal one */
#define BAOC_ERR_STATE        (-7)  /* call out of order (finalize before any step, ...) */

#define BAOC_GRAD_F32  0u
#define BAOC_GRAD_BF16 1u

/* One parameter block B_i (Sec. 3.1): numel = d_i coordinates starting `offset`
 * elements into the flat gradient buffer.  Blocks may come in any order and
 * leave gaps but must not overlap.  rows*cols == numel marks a matrix block
 * (its v-hat, viewed as rows x cols row-major, enters the structure residual of Eq. 7);
 * otherwise both are 0. */
typedef struct {
    uint64_t offset;
    uint64_t numel;
    uint32_t rows, cols;
} baoc_block;

/* Profiler parameters.  baoc_profile_params_default() fills the defaults. */
typedef struct {
    float    beta_m;       /* EMA rate of the first moment, Eq. 3             (0.9)   */
    float    beta_v;       /* EMA rate of the second moment, Eq. 3            (0.999) */
    double   beta_rho;     /* smoothing of the direction stability, Eq. 5     (0.9)   */
    double   eps;          /* epsilon of Sec. 3.3 / App. A.1                  (1e-12) */
    float    eps_update;   /* epsilon inside u = m / (sqrt(v) + eps_update), Eq. 8 (1e-8); > 0 */
    uint32_t quant_block;  /* coordinates per 8-bit absmax group; only 256 is built     */
    uint32_t grad_dtype;   /* BAOC_GRAD_F32 | BAOC_GRAD_BF16 (states are always fp32)   */
    /* Launch shape of the per-step kernel; 0 = the default measured best for the gradient type
     * (fp32 layouts of fewer than 2^26 coordinates: 4 wavefronts x 1 group, 4 resident).
     * None of the five changes any result bit except through the order of the partial sums. */
    uint32_t chunk_groups;        /* quantisation groups per chunk, the unit of the tables and of the
                                   * finalize passes (default 8 for bf16 gradients, 4 for fp32)       */
    uint32_t chunk_slices;        /* workgroups of the step kernel per chunk (default: as many as
                                   * make a slice one round, chunk_groups / (waves * groups_per_wave)) */
    uint32_t groups_per_wave;     /* adjacent groups a wavefront loads together: 1 or 2 (default 2)   */
    uint32_t waves_per_workgroup; /* 1, 2 or 4 (default 4 for bf16 gradients, 1 for fp32)             */
    uint32_t resident_workgroups; /* workgroups of the steady-state step kernel resident per compute
                                   * unit, 3..32, held by launching with unused LDS (default 3 for
                                   * bf16 gradients, 10 for fp32)                                     */
} baoc_profile_params;

/* A candidate configuration c = (y_a, y_m, y_d, y_f, b) of Def. 3.1:
 * adaptive scaling, momentum, decoupled weight decay, factored state, bits. */
typedef struct {
    uint8_t y_a, y_m, y_d, y_f;
    uint8_t bits;          /* 32 | 16 | 8 */
} baoc_config;

/* Normalisation anchors of App. A and the weights of Eq. 1 / Sec. 3.2. */
typedef struct {
    double gamma;                 /* weight of Agg(c), Eq. 1                  (0.1)      */
    double A_low, A_high;         /* anisotropy anchors, Eq. 11               (ln 2, ln 10) */
    double rho_low, rho_high;     /* direction anchors, Eq. 13                (0.2, 0.6) */
    double eta_low, eta_high;     /* log(1+snr) anchors, Eq. 15               (0, 2)     */
    int32_t use_snr_gate;         /* 1: s_M = s_rho * s_snr (Eq. 17); 0: s_M = s_rho     */
    double lambda_pref;           /* soft preference strength, Sec. 3.2       (0)        */
    const uint8_t* pref_mask;     /* n_configs flags marking C_pref, or NULL             */
    const double*  C_raw;         /* n_blocks raw distortions C_i (Eq. 6) supplied by the caller, or NULL */
    const double*  F_raw;         /* n_blocks raw structure residuals F_i (Eq. 7) supplied by the caller, or NULL */
    int32_t compute_F;            /* F_raw == NULL: 1 = compute F from v-hat for matrix blocks
                                     (rows*cols == numel; other blocks get 0), 0 = F = 0   (1)   */
    const void* d_theta_flat;     /* C_raw == NULL: DEVICE buffer of the parameters theta, laid out
                                     like the gradient buffer; C is then computed from it (Eq. 6).
                                     NULL = C = 0                                                */
    uint64_t theta_numel;         /* elements in d_theta_flat (must cover every block)           */
    uint32_t theta_dtype;         /* BAOC_GRAD_F32 | BAOC_GRAD_BF16                              */
} baoc_risk_params;

/* Per-block result of baoc_profile_finalize: raw metrics of Sec. 3.3 after the
 * last step, their normalised signals (App. A), and the relative L2 error of
 * storing the moment states in bf16 / block-wise 8 bit. */
typedef struct {
    uint64_t numel;
    uint32_t steps;               /* sampled steps seen                                   */
    uint32_t n_cos;               /* cosines folded into rho_bar (= steps - 1)            */
    double rho_bar, cos_last;     /* Eq. 5 left: EMA of cos(g_t, g_{t-1}); the last cosine */
    double snr;                   /* Eq. 5 right: |m|^2 / (|v|_1 + eps)                   */
    double A, q10, q90;           /* Eq. 4 and the two quantiles of v it is built from    */
    double Q16, Q8;               /* Eq. 8 after the clip of Eq. 10                       */
    double lQ32, lQ16, lQ8;       /* Eq. 20: -log(Q + eps)                                */
    double err_m16, err_v16, err_m8, err_v8;  /* |x^b - x|_2 / (|x|_2 + eps), x = m, v   */
    double s_A, s_rho, s_snr, s_M, C_tilde, s_F;   /* App. A signals                      */
    double m_sq, v_l1, g_sq_last; /* |m|^2, |v|_1, |g_T|^2                                */
    double C, F;                  /* raw distortion (Eq. 6) and structure residual (Eq. 7) behind C_tilde, s_F */
} baoc_block_stats;

typedef struct baoc_profiler baoc_profiler;

/* Defaults named in the paper (Sec. 3.2, Sec. 3.3, App. A) or, where it is
 * silent, the values listed next to each field above. */
void baoc_profile_params_default(baoc_profile_params* p);
void baoc_risk_params_default(baoc_risk_params* p);

/* Device workspace needed for this block layout: the fp32 states m, v (Eq. 3),
 * the previous gradient (Eq. 5) in the gradient's dtype, per-workgroup partial
 * sums, tables and the quantile scratch (for matrix blocks: candidate lists of
 * 4 bytes per 8 coordinates); roughly 12.7 (fp32 gradients) or 10.6 (bf16) bytes
 * per profiled coordinate.  blocks: HOST array of n_blocks. */
int baoc_profile_workspace_bytes(const baoc_block* blocks, uint32_t n_blocks,
                                 const baoc_profile_params* params, uint64_t* out_bytes);

/* Validate the layout, carve `d_workspace` (DEVICE, 256-byte aligned, at least
 * workspace_bytes long, owned by the caller and kept alive until
 * baoc_profile_end) and upload the layout tables.  The states start at zero: the
 * first step does not read them, it writes them.  Synchronous on the null stream.
 * *out receives the handle.  Errors: INVALID, WORKSPACE, UNSUPPORTED, HIP. */
int baoc_profile_begin(const baoc_block* blocks, uint32_t n_blocks,
                       const baoc_profile_params* params,
                       void* d_workspace, uint64_t workspace_bytes, baoc_profiler** out);

/* baoc_profile_begin for callers that cannot allocate device memory (code between the begin and the
 * end of a HIP graph capture, serving loops, harnesses that forbid hipMalloc): the workspace is an
 * array of BAOC_STATIC_WORKSPACE_BYTES that the library holds on every GPU it is loaded on, from load
 * until the process ends.  The call, and the step / finalize / end calls on its handle, allocate no
 * device memory.  Everything else is as in baoc_profile_begin: the same kernels, bit-identical results.
 * The array keeps what the last handle left in it (begin clears what must start at zero), and all
 * handles begun this way on one GPU share it: only one may be alive per GPU at a time (a second begin
 * before baoc_profile_end returns STATE), and work still queued on a stream for an ended handle races
 * with the next one.  Errors: WORKSPACE when baoc_profile_workspace_bytes of the layout exceeds
 * BAOC_STATIC_WORKSPACE_BYTES (about 12 M coordinates with bf16 gradients, 10 M with fp32);
 * UNSUPPORTED for a device ordinal above 63; otherwise as baoc_profile_begin. */
#define BAOC_STATIC_WORKSPACE_BYTES (128ull << 20)
int baoc_profile_begin_static(const baoc_block* blocks, uint32_t n_blocks,
                              const baoc_profile_params* params, baoc_profiler** out);

/* One sampled step (Eq. 3, Eq. 5, Eq. 8): enqueue, on `hip_stream`
 * (a hipStream_t, NULL = null stream), one fused pass over the flat gradient
 * buffer `d_grad_flat` (DEVICE, grad_numel elements of the dtype given at
 * begin) and the per-block reduction.  Returns without waiting.  The gradient
 * buffer must stay valid until that stream work has run; afterwards the
 * caller may overwrite it (the library keeps its own copy of g_t as g_{t-1}).
 * Consecutive calls are consecutive samples.  The first call after begin launches another
 * kernel than the later ones (the states are known to be zero); from the second call on
 * the launches are the same for every step (the step count is kept on the device), so a HIP
 * graph captured from a later call may be replayed once per further step, with the next
 * gradient in the same buffer.
 * Range: the sums of squares of a
 * chunk are kept in fp32 before the fp64 stage, so gradient magnitudes up to about
 * 1e8 give finite statistics (beyond, sums of v^2 overflow and the error and noise
 * terms of that block come out inf or NaN); small magnitudes are safe down to the
 * point where v underflows to zero.  A NaN or inf in a gradient makes the
 * statistics of its block NaN and leaves the other blocks alone.
 * Errors: INVALID (a block reaches beyond grad_numel, null pointer), HIP. */
int baoc_profile_step(baoc_profiler* p, const void* d_grad_flat, uint64_t grad_numel,
                      void* hip_stream);

/* Metrics and risk table after the steps seen so far (Sec. 3.3, App. A, Eq. 9,
 * Eq. 1): runs the quantile selection of Eq. 4 on `hip_stream`, waits for it,
 * then fills out_stats (HOST, n_blocks entries, in the order given at begin)
 * and out_risk (HOST, n_blocks x n_configs row-major,
 * Phi[i][c] = R_i(c) - lambda_pref [c in C_pref] + gamma Agg(c)).
 * The structure residual F (Eq. 7: v-hat of a matrix block against the rank-1
 * matrix of its row and column means) and, when risk_params->d_theta_flat is
 * given, the distortion C (Eq. 6) are computed on the device in the same call.
 * Either output may be NULL.  The state is kept: more steps may follow and
 * finalize may be called again with other configurations.
 * Errors: INVALID (bits not in {8,16,32}, null configs with out_risk, theta
 * buffer shorter than the layout), STATE
 * (no step yet), HIP. */
int baoc_profile_finalize(baoc_profiler* p, const baoc_config* configs, uint32_t n_configs,
                          const baoc_risk_params* risk_params,
                          baoc_block_stats* out_stats, double* out_risk, void* hip_stream);

/* Device views of one block's state inside the caller's workspace (for
 * checkpoints and bit-level tests): d_m, d_v are fp32[numel]; d_g_prev holds
 * numel elements of the gradient dtype.  Pointers are valid until
 * baoc_profile_end; their contents are defined once the first step has run. */
int baoc_profile_state(const baoc_profiler* p, uint32_t block,
                       const float** d_m, const float** d_v, const void** d_g_prev);

/* Release the handle (host memory only; the workspace stays the caller's). */
int baoc_profile_end(baoc_profiler* p);

/* ---- Sparse coordinate sampling (Sec. 3.1) --------------------------------
 * The paper profiles a fixed subset Omega_i of each block, |Omega_i| =
 * ceil(ratio * d_i) (at least 1), drawn once.  Here: a stratified uniform draw
 * (one coordinate out of each of |Omega_i| equal strata, by a 64-bit mix of
 * (seed, block, stratum)), indices ascending.  The sampler packs g[Omega] of all
 * blocks into a compact buffer; the profiler then runs on that buffer with the
 * compact block layout.
 * Matrix blocks (rows, cols >= 2) keep a matrix form, which the structure residual of Eq. 7 needs:
 * their Omega is a product of r = round(rows sqrt(ratio)) rows and c columns, c the least count with
 * r c >= ceil(ratio d_i), each axis drawn by the same stratified rule, and the compact block is that
 * r x c sub-matrix, row-major (so |Omega_i| may exceed ceil(ratio d_i) by less than r).  When r or c would
 * be below 2 the block is sampled as a plain vector and its compact block carries no shape (F = 0). */
typedef struct baoc_sampler baoc_sampler;

/* Compact layout for this ratio (0 < ratio <= 1): out_compact (HOST, n_blocks, may
 * be NULL) receives offset/numel and the sub-matrix shape of each block in the compact buffer (starts on
 * multiples of 64 elements), out_compact_numel its length, out_workspace_bytes the
 * device bytes the sampler needs (tables + 8 bytes per sampled coordinate). */
int baoc_sample_layout(const baoc_block* blocks, uint32_t n_blocks, double ratio,
                       baoc_block* out_compact, uint64_t* out_compact_numel,
                       uint64_t* out_workspace_bytes);

/* Draw Omega on the device into d_workspace (DEVICE, 256-byte aligned, caller
 * owned, kept until baoc_sample_end).  Synchronous on the null stream.
 * Errors: INVALID, WORKSPACE, UNSUPPORTED, HIP. */
int baoc_sample_begin(const baoc_block* blocks, uint32_t n_blocks, double ratio, uint64_t seed,
                      void* d_workspace, uint64_t workspace_bytes, baoc_sampler** out);

/* d_compact[compact offset of block i + j] = d_grad_flat[Omega_i[j]] for every block,
 * enqueued on hip_stream.  Both buffers DEVICE, of dtype grad_dtype; gaps of the
 * compact buffer are left untouched.  Errors: INVALID (buffers too short), HIP. */
int baoc_sample_gather(baoc_sampler* s, const void* d_grad_flat, uint64_t grad_numel,
                       uint32_t grad_dtype, void* d_compact, uint64_t compact_numel,
                       void* hip_stream);

/* Device view of Omega_i as absolute element positions in the flat buffer. */
int baoc_sample_indices(const baoc_sampler* s, uint32_t block,
                        const uint64_t** d_indices, uint64_t* count);

int baoc_sample_end(baoc_sampler* s);

/* Exact solution of the allocation problem of Eq. 2 (a multiple-choice knapsack
 * with a memory row and a time row) on the integer image of the instance:
 *   phi = llround(1e9 * clamp(risk, -1e6, 1e6)),  tau = llround(1e6 * time_cost),
 *   tau_budget = llround(1e6 * time_budget_sum).
 * A pair (i,c) is excluded when forbidden[i*K+c] != 0 (hard constraint of
 * Sec. 3.2) or when its risk or time cost is not finite.  Among the feasible
 * assignments of least sum(phi) the lexicographically smallest choice vector
 * is returned.  time_budget_sum bounds the SUM of r_{i,c_i}; the paper's
 * mean form is B_time * n_blocks.  All pointers HOST; risk, mem_cost_bytes,
 * time_cost, forbidden are n_blocks x n_configs row-major; out_choice has
 * n_blocks entries; out_objective / out_mem / out_time may be NULL and receive
 * sum(phi)/1e9, sum(mem) and sum(tau)/1e6 of the answer.
 * Errors: INVALID (null, zero sizes, negative memory, NaN budget),
 * INFEASIBLE, LIMIT (state limit of the search, or host memory exhausted). */
int baoc_allocate(const double* risk, const int64_t* mem_cost_bytes, const double* time_cost,
                  uint32_t n_blocks, uint32_t n_configs,
                  int64_t mem_budget_bytes, double time_budget_sum,
                  const uint8_t* forbidden,
                  uint32_t* out_choice, double* out_objective, int64_t* out_mem, double* out_time);

/* Block partitioning (App. C.2, Algorithm 2), host code.  Units are the structural
 * candidates in forward order: unit j has unit_numel[j] > 0 parameters and a normalised
 * diagnostic vector z[j*n_stats .. ] (e.g. the App. A signals that a profile of the units
 * returned).  Delta(U_a,U_b) = max_k w_k |z_a,k - z_b,k| (weights NULL = all 1); tau = upper
 * quartile of Delta over all unit pairs; n_min = alpha * total parameters (0 <= alpha <= 1).
 * Undersized candidates are merged into their statistically closest neighbour, adjacent
 * candidates stay separate only when Delta > tau and both reach n_min, formed blocks are
 * split where their two sides differ by more than tau, and what is still undersized is
 * merged again.  out_block_of_unit (n_units) receives ascending block ids from 0; a
 * block's statistics are the parameter-weighted mean of its units.  All pointers HOST;
 * out_n_blocks and out_tau may be NULL.  Errors: INVALID (null, zero sizes, non-finite z,
 * negative weights, alpha outside [0,1]), UNSUPPORTED (more than 32,768 units, or not enough host memory
 * for the pair table: tau is a quantile over all unit pairs, so time and memory grow with n_units^2). */
int baoc_partition(const uint64_t* unit_numel, const double* z, uint32_t n_units, uint32_t n_stats,
                   const double* weights, double alpha,
                   uint32_t* out_block_of_unit, uint32_t* out_n_blocks, double* out_tau);

/* Cap on the states baoc_allocate keeps over all levels of any one of its recursions (24 bytes each), for
 * this thread's later calls; 0 = default (32 M).  Beyond it the call returns BAOC_ERR_LIMIT. */
void baoc_allocate_set_node_limit(uint64_t max_nodes);

/* Work the solver spends on finding exactly which configurations occur in optimal assignments (max_states:
 * states extended by its forward pass), for this thread's later calls; 0 = default (16 M, about a second).
 * Beyond it the pass goes on with at most front_cap coarser, optimistic states per level (0 = default, 256):
 * the answer is the same, only the last recursion of the call has more configurations to carry.  Tuning
 * knobs (Eq. 2 does not know them); max_states = 1 switches the exact phase off. */
void baoc_allocate_set_exact_work(uint64_t max_states, uint32_t front_cap);

const char* baoc_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* BAOC_H */
