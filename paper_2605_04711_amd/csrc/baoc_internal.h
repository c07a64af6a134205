// Internal declarations shared by the translation units of libbaoc.
#pragma once
#include <cstdint>
#include <vector>

#include "baoc.h"

namespace baoc {

constexpr uint32_t kQB = 256;            // coordinates per 8-bit absmax group = one wavefront x 4
constexpr uint32_t kNumSums = 16;        // floats in one partial-sum row

// Launch shape of the step kernel, per gradient type (fp32, bf16).  Measured: a DRAM stream of 4 reads
// and 3 writes per coordinate runs fastest with few, fat requesters; more resident wavefronts only add
// row conflicts.  fp32 gradients: single-wavefront workgroups of two adjacent groups, about 10 resident
// per compute unit; bf16: 4 wavefronts x 2 groups, 3 resident.  A chunk (the unit of the tables and of
// the finalize passes) is cut into slices of one round each.
struct LaunchShape { uint32_t chunk_groups, groups_per_wave, waves_per_workgroup, resident_workgroups; };
constexpr LaunchShape kDefaultShape[2] = {{4, 2, 1, 10}, {8, 2, 4, 3}};
constexpr LaunchShape kSmallF32Shape = {4, 1, 4, 4};          // fp32 layouts below kSmallLayout coordinates
constexpr uint64_t kSmallLayout = 1ull << 26;
constexpr uint32_t kLdsBytesPerCU = 160 * 1024;   // gfx950

// order of the sums in a partial row and in the per-block raw record
enum Sum : int {
    S_GG = 0, S_GP, S_MM, S_V1, S_VV, U0,
    U1_16, D_16, U2_16, EM_16, EV_16,
    U1_8, D_8, U2_8, EM_8, EV_8
};

// per-block record kept on the device, doubles
enum Rec : int {
    R_SPP = 16, R_RHO, R_COS, R_NCOS, R_STEPS, R_Q0, R_Q1, R_Q2, R_Q3,
    R_PSUM, R_CNUM, R_CDEN, R_FRES, R_FS2, kRecDoubles = 32
};

// Raw per-block numbers handed from the device path to the host-side metrics.
struct RawBlock {
    uint64_t numel;
    double sums[kNumSums];
    double rho_bar, cos_last;
    uint32_t n_cos, steps;
    float order_stat[4];                 // v at ranks lo(0.1), lo+1, lo(0.9), lo+1
    double frac10, frac90;               // interpolation weights of the two quantiles
};

// Sec. 3.3 metrics + App. A signals of one block from its raw sums.
void block_metrics(const RawBlock& r, double eps, const baoc_risk_params& rp,
                   double C_raw, double F_raw, baoc_block_stats* out);

// Phi_{i,c} = R_i(c) - lambda_pref [c in C_pref] + gamma Agg(c)   (Eq. 9, Sec. 3.2, Eq. 1)
double config_phi(const baoc_block_stats& z, const baoc_config& c, bool preferred,
                  const baoc_risk_params& rp);

}  // namespace baoc
