// Gradient-stream profiler of BAOC for gfx950 (MI355X): kernels and the
// baoc_profile_* entry points.
//
// One sampled step is one streaming pass: every coordinate's gradient, previous
// gradient and fp32 EMA states are read once and written once (28 B per
// coordinate with fp32 gradients, 22 B with bf16), and everything Sec. 3.3 needs
// from that coordinate is accumulated in registers on the way:
//   Eq. 3  m <- beta_m m + (1-beta_m) g,  v <- beta_v v + (1-beta_v) g*g
//   Eq. 5  <g_t, g_{t-1}>, |g_t|^2, |m|^2, |v|_1
//   Eq. 8  update directions u = m/(sqrt(v)+eps_u) from the fp32 state and from
//          the state after a bf16 or a block-wise absmax 8-bit round trip.
// Work is cut into chunks that never straddle a parameter block; the step kernel cuts a chunk into
// slices, one workgroup (1, 2 or 4 wavefronts, a launch-shape parameter) and one partial row each.  A
// wavefront owns whole 256-coordinate quantisation groups (4 coordinates per lane, one or two groups
// next to each other), so a group's absmax is a DPP reduction inside the wavefront.  Sums go wavefront
// (DPP) -> workgroup (LDS) -> one partial row per workgroup -> per parameter block in fp64 (second kernel).
// No float atomics anywhere: two runs give identical bits.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "baoc_internal.h"

namespace baoc {

struct alignas(8) Chunk {
    uint64_t grad_start;    // element index into the caller's flat gradient buffer
    uint64_t state_start;   // element index into m / v / g_prev (multiple of 256)
    uint32_t count;         // coordinates in the chunk (only a block's last chunk may end off a multiple of 256)
    uint32_t block;
};

struct alignas(8) BlockRow {
    uint64_t grad_start;    // the block's offset in the caller's flat gradient buffer
    uint64_t state_start;
    uint64_t numel;
    uint32_t first_chunk, n_chunks;
    uint32_t groups_per_chunk;
    uint32_t vec_first;     // first entry of the block in the list of chunks finalize walks chunk-wise; kNoVec when tiled
    uint32_t first_slab, n_slabs;   // the block's slabs of partial rows (first stage of the per-block sum)
    uint32_t first_prow, n_prows;   // the block's partial rows of the step kernel (one per workgroup: chunk x slice)
    uint64_t rank[4];       // order statistics wanted from v: lo(0.1), lo+1, lo(0.9), lo+1
};

struct StepConsts {
    float beta_m, beta_v, om_m, om_v, eps_u;
};

constexpr uint32_t kNoVec = 0xffffffffu;

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------
// wavefront reductions on the DPP crossbar (64 lanes = 4 rows of 16)
// ---------------------------------------------------------------------------

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp(float old, float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
        __builtin_bit_cast(int, old), __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xf, false));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t old, uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)x, CTRL, ROW_MASK, 0xf, false);
}

// quad_perm[1,0,3,2]=0xB1, quad_perm[2,3,0,1]=0x4E, row_ror:4=0x124, row_ror:8=0x128 leave every
// lane of a row with the row's total; row_bcast:15 (0x142, rows 1 and 3) and row_bcast:31
// (0x143, rows 2 and 3) carry the totals upwards so that lane 63 ends with the wavefront's.
//
// Largest of the lanes' non-negative binary32 values.  Among non-negative values the order of the
// bit patterns as unsigned integers is the order of the values, so the reduction runs on integers
// (one v_max_u32 with a DPP operand per level).  A NaN pattern ranks above +inf, so a NaN anywhere
// in the group comes out as the maximum; such a group's sums are NaN whatever its scale is.
__device__ __forceinline__ float wave_max_nonneg(float v)
{
    uint32_t x = __builtin_bit_cast(uint32_t, v);
    x = max(x, dpp_u32<0xB1, 0xf>(0u, x));
    x = max(x, dpp_u32<0x4E, 0xf>(0u, x));
    x = max(x, dpp_u32<0x124, 0xf>(0u, x));
    x = max(x, dpp_u32<0x128, 0xf>(0u, x));
    x = max(x, dpp_u32<0x142, 0xa>(0u, x));
    x = max(x, dpp_u32<0x143, 0xc>(0u, x));
    return __builtin_bit_cast(float, (uint32_t)__builtin_amdgcn_readlane((int)x, 63));
}

__device__ __forceinline__ float wave_sum(float x)
{
    x += dpp<0xB1, 0xf>(0.f, x);
    x += dpp<0x4E, 0xf>(0.f, x);
    x += dpp<0x124, 0xf>(0.f, x);
    x += dpp<0x128, 0xf>(0.f, x);
    x += dpp<0x142, 0xa>(0.f, x);
    x += dpp<0x143, 0xc>(0.f, x);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

// ---------------------------------------------------------------------------
// element helpers
// ---------------------------------------------------------------------------

__device__ __forceinline__ float bf16_widen(uint32_t h) { return __builtin_bit_cast(float, h << 16); }

// Round-to-nearest-even of two binary32 values to the bf16 grid, widened back.  One
// v_cvt_pk_bf16_f32 (gfx950) converts both; the halves are then moved back to the top of a word.
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void bf16_round2(float a, float b, float& ra, float& rb)
{
    const f2 x = {a, b};
    const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf2));
    ra = __builtin_bit_cast(float, w << 16);
    rb = __builtin_bit_cast(float, w & 0xffff0000u);
}

// u = m / (sqrt(v) + eps_u) with the hardware's 1-ulp square root and reciprocal
__device__ __forceinline__ float direction(float m, float v, float eps_u)
{
    return m * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v) + eps_u);
}

// Preconditioner of Eq. 6, p = 1 / (sqrt(v) + eps), with one transcendental instead of two where eps is small
// against sqrt(v): with r = 1/sqrt(v), p = r / (1 + eps r) = r (1 - eps r) up to (eps r)^2 < 1e-6.  Elsewhere
// (v tiny, zero, sub-normal or NaN) the plain form.
__device__ __forceinline__ float preconditioner(float v, float eps)
{
    const float r = __builtin_amdgcn_rsqf(v);
    const float er = eps * r;
    float p = __builtin_fmaf(-er, r, r);
    if (!(er < 1e-3f)) p = __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v) + eps);
    return p;
}

// Every array is touched exactly once per pass: load and store with the nontemporal hint so the
// stream does not displace anything in L2 / MALL on its way through.
template <typename T> __device__ __forceinline__ T ld_stream(const void* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
}
template <typename T> __device__ __forceinline__ void st_stream(void* p, T val)
{
    __builtin_nontemporal_store(val, reinterpret_cast<T*>(p));
}

template <int GT> struct GradIO;

template <> struct GradIO<BAOC_GRAD_F32> {
    typedef float elem;
    typedef f4 vec4;                                      // four elements as loaded
    __device__ static __forceinline__ vec4 loadv(const elem* p) { return ld_stream<f4>(p); }
    __device__ static __forceinline__ void unpack(vec4 t, float g[4]) { g[0] = t.x; g[1] = t.y; g[2] = t.z; g[3] = t.w; }
    __device__ static __forceinline__ void load4(const elem* p, float g[4]) { unpack(loadv(p), g); }
    __device__ static __forceinline__ float load1(const elem* p) { return *p; }
    __device__ static __forceinline__ void store4(elem* p, const float g[4])
    {
        f4 t = {g[0], g[1], g[2], g[3]};
        st_stream<f4>(p, t);
    }
    static constexpr uintptr_t kAlignMask = 15;
};

template <> struct GradIO<BAOC_GRAD_BF16> {
    typedef uint16_t elem;
    typedef u2 vec4;
    __device__ static __forceinline__ vec4 loadv(const elem* p) { return ld_stream<u2>(p); }
    __device__ static __forceinline__ void unpack(vec4 t, float g[4])
    {
        g[0] = __builtin_bit_cast(float, t.x << 16); g[1] = __builtin_bit_cast(float, t.x & 0xffff0000u);
        g[2] = __builtin_bit_cast(float, t.y << 16); g[3] = __builtin_bit_cast(float, t.y & 0xffff0000u);
    }
    __device__ static __forceinline__ void load4(const elem* p, float g[4]) { unpack(loadv(p), g); }
    __device__ static __forceinline__ float load1(const elem* p) { return bf16_widen(*p); }
    // g holds exact bf16 values: the upper half of each word is the stored pattern
    __device__ static __forceinline__ void store4(elem* p, const float g[4])
    {
        u2 t;
        t.x = (__builtin_bit_cast(uint32_t, g[0]) >> 16) | (__builtin_bit_cast(uint32_t, g[1]) & 0xffff0000u);
        t.y = (__builtin_bit_cast(uint32_t, g[2]) >> 16) | (__builtin_bit_cast(uint32_t, g[3]) & 0xffff0000u);
        st_stream<u2>(p, t);
    }
    static constexpr uintptr_t kAlignMask = 7;
};

// ---------------------------------------------------------------------------
// the fused per-step pass
// ---------------------------------------------------------------------------

// FIRST: the states are known to be zero (first step after begin), so they are not read.
// A workgroup of NW wavefronts takes one slice of a chunk (`slice_groups` quantisation groups, `slices`
// slices per chunk) and writes one partial row.  G: groups a wavefront takes per round, next to each
// other (G * 1 KB of m and of v per wavefront and round); the workgroup covers NW * G groups per round.
// The loads of a round are issued together, one round ahead of their use.  With the default shapes a
// slice is a single round, so no wavefront ever waits on its own stores.
template <int GT, bool FIRST, int G, int NW>
__global__ __launch_bounds__(64 * NW) void k_step(
    const typename GradIO<GT>::elem* __restrict__ grad,
    float* __restrict__ m_all, float* __restrict__ v_all,
    typename GradIO<GT>::elem* __restrict__ gp_all,
    const Chunk* __restrict__ chunks, float* __restrict__ partials, StepConsts k,
    uint32_t slices, uint32_t slice_groups)
{
    typedef GradIO<GT> IO;
    const uint32_t chunk = blockIdx.x / slices, slice = blockIdx.x - chunk * slices;
    const Chunk ck = chunks[chunk];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    // this workgroup's groups of the chunk: [g_begin, ngroups)
    const uint32_t g_begin = slice * slice_groups;
    const uint32_t ngroups = min((ck.count + (kQB - 1)) / kQB, g_begin + slice_groups);
    const typename IO::elem* gsrc = grad + ck.grad_start;
    const bool vec_ok = (reinterpret_cast<uintptr_t>(gsrc) & IO::kAlignMask) == 0;

    float acc[kNumSums];
#pragma unroll
    for (int i = 0; i < (int)kNumSums; ++i) acc[i] = 0.f;

    typedef typename IO::vec4 GV;
    f4 nm[G], nv[G];
    GV np[G], ng[G];
#pragma unroll
    for (int i = 0; i < G; ++i) { nm[i] = f4{0.f, 0.f, 0.f, 0.f}; nv[i] = nm[i]; np[i] = GV{}; ng[i] = GV{}; }
    auto issue = [&](uint32_t first) {                    // first: the wavefront's first group of a round
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const uint32_t grp = first + i;
            if (grp < ngroups) {
                const uint32_t e = grp * kQB + lane * 4;
                const uint64_t si = ck.state_start + e;   // states are padded to whole groups
                if (!FIRST) { nm[i] = ld_stream<f4>(m_all + si); nv[i] = ld_stream<f4>(v_all + si); np[i] = IO::loadv(gp_all + si); }
                if (vec_ok && e + 4 <= ck.count) ng[i] = IO::loadv(gsrc + e);
            }
        }
    };
    if (g_begin + wave * G < ngroups) issue(g_begin + wave * G);

    for (uint32_t first = g_begin + wave * G; first < ngroups; first += NW * G) {
        f4 cm[G], cv[G];
        GV cp[G], cg[G];
#pragma unroll
        for (int i = 0; i < G; ++i) { cm[i] = nm[i]; cv[i] = nv[i]; cp[i] = np[i]; cg[i] = ng[i]; }
        if (first + NW * G < ngroups) issue(first + NW * G);
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const uint32_t grp = first + i;
            if (grp >= ngroups) break;
            const uint32_t e = grp * kQB + lane * 4;          // first of this lane's 4 coordinates
            const uint64_t si = ck.state_start + e;
            float* m_dst = m_all + si;                        // store addresses formed early: the stores then
            float* v_dst = v_all + si;                        // leave as soon as the updated states exist
            float g[4], p[4], m[4], v[4];
            if (FIRST) {
#pragma unroll
                for (int j = 0; j < 4; ++j) m[j] = v[j] = p[j] = 0.f;
            } else {
                m[0] = cm[i].x; m[1] = cm[i].y; m[2] = cm[i].z; m[3] = cm[i].w;
                v[0] = cv[i].x; v[1] = cv[i].y; v[2] = cv[i].z; v[3] = cv[i].w;
                IO::unpack(cp[i], p);
            }
            if (vec_ok && e + 4 <= ck.count) {
                IO::unpack(cg[i], g);
            } else {                                          // ragged tail or unaligned block start
#pragma unroll
                for (int j = 0; j < 4; ++j) g[j] = (e + j < ck.count) ? IO::load1(gsrc + e + j) : 0.f;
            }

            // Eq. 3 in fp32: the new term is rounded, then one fused multiply-add
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float tm = k.om_m * g[j];
                const float tv = (k.om_v * g[j]) * g[j];
                m[j] = __builtin_fmaf(k.beta_m, m[j], tm);
                v[j] = __builtin_fmaf(k.beta_v, v[j], tv);
            }
            {
                f4 t = {m[0], m[1], m[2], m[3]};
                st_stream<f4>(m_dst, t);
                f4 s = {v[0], v[1], v[2], v[3]};
                st_stream<f4>(v_dst, s);
            }
            IO::store4(gp_all + si, g);

            // group absmax of the 256 coordinates this wavefront holds
            const float a_m = wave_max_nonneg(fmaxf(fmaxf(fabsf(m[0]), fabsf(m[1])), fmaxf(fabsf(m[2]), fabsf(m[3]))));
            const float a_v = wave_max_nonneg(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])));
            // 8-bit code = rint(x * (L / a)) decided in fp32 with a correctly rounded quotient;
            // an infinite scale (a == 0 or tiny) means all codes are 0
            float s_m = 127.0f / a_m, s_v = 255.0f / a_v;
            s_m = s_m < INFINITY ? s_m : 0.f;
            s_v = s_v < INFINITY ? s_v : 0.f;
            const float d_m = a_m * (1.0f / 127.0f), d_v = a_v * (1.0f / 255.0f);

#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float mj = m[j], vj = v[j];
                acc[S_GG] = __builtin_fmaf(g[j], g[j], acc[S_GG]);
                acc[S_GP] = __builtin_fmaf(g[j], p[j], acc[S_GP]);
                acc[S_MM] = __builtin_fmaf(mj, mj, acc[S_MM]);
                acc[S_V1] += vj;
                acc[S_VV] = __builtin_fmaf(vj, vj, acc[S_VV]);
                const float u32 = direction(mj, vj, k.eps_u);
                acc[U0] = __builtin_fmaf(u32, u32, acc[U0]);
                {   // bf16 round trip
                    float mb, vb;
                    bf16_round2(mj, vj, mb, vb);
                    const float ub = direction(mb, vb, k.eps_u);
                    const float du = ub - u32, dm = mb - mj, dv = vb - vj;
                    acc[U1_16] = __builtin_fmaf(u32, ub, acc[U1_16]);
                    acc[D_16] = __builtin_fmaf(du, du, acc[D_16]);
                    acc[U2_16] = __builtin_fmaf(ub, ub, acc[U2_16]);
                    acc[EM_16] = __builtin_fmaf(dm, dm, acc[EM_16]);
                    acc[EV_16] = __builtin_fmaf(dv, dv, acc[EV_16]);
                }
                {   // block-wise absmax 8-bit round trip
                    const float mb = __builtin_rintf(mj * s_m) * d_m;
                    const float vb = __builtin_rintf(vj * s_v) * d_v;
                    const float ub = direction(mb, vb, k.eps_u);
                    const float du = ub - u32, dm = mb - mj, dv = vb - vj;
                    acc[U1_8] = __builtin_fmaf(u32, ub, acc[U1_8]);
                    acc[D_8] = __builtin_fmaf(du, du, acc[D_8]);
                    acc[U2_8] = __builtin_fmaf(ub, ub, acc[U2_8]);
                    acc[EM_8] = __builtin_fmaf(dm, dm, acc[EM_8]);
                    acc[EV_8] = __builtin_fmaf(dv, dv, acc[EV_8]);
                }
            }
        }
    }

    // Sixteen sums held by sixteen lanes: a halving exchange inside each row of 16 lanes (after the
    // level that pairs lanes differing in bit b, a lane keeps only the sums whose index has its own
    // bit b) leaves lane l of a row with that row's total of sum l & 15, in 8+4+2+1 DPP additions.
    // Then LDS (4 wavefronts x 4 rows) -> one partial row per chunk, in a fixed order.
    static_assert(kNumSums == 16, "the exchange below is written for 16 sums");
    {
        const bool b3 = lane & 8u, b2 = lane & 4u, b1 = lane & 2u, b0 = lane & 1u;
#pragma unroll
        for (int i = 0; i < 8; ++i) {                     // partner lane ^ 8 (row_ror:8)
            const float keep = b3 ? acc[i + 8] : acc[i], send = b3 ? acc[i] : acc[i + 8];
            acc[i] = keep + dpp<0x128, 0xf>(0.f, send);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {                     // partner 7 - (lane & 7) in the same half (row_half_mirror)
            const float keep = b2 ? acc[i + 4] : acc[i], send = b2 ? acc[i] : acc[i + 4];
            acc[i] = keep + dpp<0x141, 0xf>(0.f, send);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {                     // partner lane ^ 2
            const float keep = b1 ? acc[i + 2] : acc[i], send = b1 ? acc[i] : acc[i + 2];
            acc[i] = keep + dpp<0x4E, 0xf>(0.f, send);
        }
        const float keep = b0 ? acc[1] : acc[0], send = b0 ? acc[0] : acc[1];
        acc[0] = keep + dpp<0xB1, 0xf>(0.f, send);       // partner lane ^ 1
    }
    __shared__ float red[NW * 4 * kNumSums];              // [wavefront * 4 + row][sum]
    red[threadIdx.x] = acc[0];
    __syncthreads();
    if (threadIdx.x < kNumSums) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < NW * 4; ++q) s += red[q * kNumSums + threadIdx.x];
        partials[(uint64_t)blockIdx.x * kNumSums + threadIdx.x] = s;
    }
}

// Per-block sums of the partial rows, in fp64.  Blocks with more than kSlabRows chunks are summed in
// two stages (slabs of kSlabRows rows by k_slab_reduce, then k_block_reduce); smaller ones directly.
constexpr uint32_t kSlabRows = 4096;      // partial rows summed by one workgroup of the first stage

struct alignas(8) Slab { uint32_t first_row, n_rows; };

// First stage for large blocks: one workgroup adds a slab of partial rows in fp64.
__global__ __launch_bounds__(256) void k_slab_reduce(const float* __restrict__ partials, const Slab* __restrict__ slabs,
                                                     double* __restrict__ slab_sums)
{
    const Slab sl = slabs[blockIdx.x];
    double acc[kNumSums];
#pragma unroll
    for (int i = 0; i < (int)kNumSums; ++i) acc[i] = 0.0;
    for (uint32_t c = threadIdx.x; c < sl.n_rows; c += 256) {
        const f4* row = reinterpret_cast<const f4*>(partials + (uint64_t)(sl.first_row + c) * kNumSums);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f4 t = row[q];
            acc[4 * q + 0] += (double)t.x; acc[4 * q + 1] += (double)t.y;
            acc[4 * q + 2] += (double)t.z; acc[4 * q + 3] += (double)t.w;
        }
    }
    __shared__ double sh[256];
#pragma unroll 1
    for (int i = 0; i < (int)kNumSums; ++i) {
        sh[threadIdx.x] = acc[i];
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) slab_sums[(uint64_t)blockIdx.x * kNumSums + i] = sh[0];
        __syncthreads();
    }
}

// Second stage, one workgroup per parameter block: the block's slab sums -- or, for a block of at
// most one slab (n_slabs == 0), its partial rows directly -- are added in fp64, then the step is
// folded into the running direction stability (Eq. 5, left):
//   cos_t = <g_t,g_{t-1}> / (|g_t| |g_{t-1}| + eps), NaN -> 0 (App. A.1);
//   the first cosine initialises rho_bar, later ones enter with weight 1 - beta_rho.
__global__ __launch_bounds__(256) void k_block_reduce(
    const float* __restrict__ partials, const double* __restrict__ slab_sums, const BlockRow* __restrict__ rows,
    double* __restrict__ rec_all, double beta_rho, double eps)
{
    const BlockRow br = rows[blockIdx.x];
    double* rec = rec_all + (uint64_t)blockIdx.x * kRecDoubles;
    if (br.n_slabs) {
        if (threadIdx.x < kNumSums) {
            double a = 0.0;
            for (uint32_t t = 0; t < br.n_slabs; ++t) a += slab_sums[(uint64_t)(br.first_slab + t) * kNumSums + threadIdx.x];
            rec[threadIdx.x] = a;
        }
    } else {
        double acc[kNumSums];
#pragma unroll
        for (int i = 0; i < (int)kNumSums; ++i) acc[i] = 0.0;
        for (uint32_t c = threadIdx.x; c < br.n_prows; c += 256) {
            const f4* row = reinterpret_cast<const f4*>(partials + (uint64_t)(br.first_prow + c) * kNumSums);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4 t = row[q];
                acc[4 * q + 0] += (double)t.x; acc[4 * q + 1] += (double)t.y;
                acc[4 * q + 2] += (double)t.z; acc[4 * q + 3] += (double)t.w;
            }
        }
        __shared__ double sh[256];
#pragma unroll 1
        for (int i = 0; i < (int)kNumSums; ++i) {
            sh[threadIdx.x] = acc[i];
            __syncthreads();
            for (int w = 128; w > 0; w >>= 1) {
                if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
                __syncthreads();
            }
            if (threadIdx.x == 0) rec[i] = sh[0];
            __syncthreads();
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        // The step index lives in the block's record, not in a launch argument: a captured launch of a
        // steady-state step can be replayed for later steps.
        const uint32_t step = (uint32_t)rec[R_STEPS] + 1u;
        const double S_gg = rec[S_GG], S_gp = rec[S_GP];
        if (step >= 2) {
            double c = S_gp / (sqrt(S_gg) * sqrt(rec[R_SPP]) + eps);
            if (c != c) c = 0.0;
            const double n = rec[R_NCOS];
            rec[R_RHO] = (n == 0.0) ? c : beta_rho * rec[R_RHO] + (1.0 - beta_rho) * c;
            rec[R_COS] = c;
            rec[R_NCOS] = n + 1.0;
        }
        rec[R_SPP] = S_gg;
        rec[R_STEPS] = (double)step;
    }
}

// ---------------------------------------------------------------------------
// Eq. 4: exact order statistics of v per block by a three-digit radix selection
// on the bit patterns (v >= 0, so the pattern order is the value order).
// Digits: bits 30..19, 18..8, 7..0.  Four ranks per block share every pass.
// Matrix blocks read v twice only: the pass that counts the second digit also
// writes the few coordinates that carry a selected first digit into a candidate
// list, and the third digit is counted on that list.
// ---------------------------------------------------------------------------

// Chunk table from the block rows (one thread per chunk; the owning block by bisection on
// first_chunk).  A block's groups are split evenly over its chunks, whole groups each.
__global__ __launch_bounds__(256) void k_build_chunks(const BlockRow* __restrict__ rows, uint32_t n_blocks,
                                                      Chunk* __restrict__ chunks, uint32_t n_chunks,
                                                      uint32_t* __restrict__ vec_list)
{
    const uint32_t c = blockIdx.x * 256 + threadIdx.x;
    if (c >= n_chunks) return;
    uint32_t lo = 0, hi = n_blocks - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (rows[mid].first_chunk <= c) lo = mid; else hi = mid - 1;
    }
    const BlockRow r = rows[lo];
    const uint64_t g0 = (uint64_t)(c - r.first_chunk) * r.groups_per_chunk;
    const uint64_t groups = (r.numel + kQB - 1) / kQB;
    const uint64_t g1 = min(groups, g0 + r.groups_per_chunk);
    Chunk ck;
    ck.grad_start = r.grad_start + g0 * kQB;
    ck.state_start = r.state_start + g0 * kQB;
    ck.count = (uint32_t)(min(r.numel, g1 * kQB) - g0 * kQB);
    ck.block = lo;
    chunks[c] = ck;
    if (r.vec_first != kNoVec) vec_list[r.vec_first + (c - r.first_chunk)] = c;
}

__global__ void k_fill_u32(uint32_t* p, uint64_t n, uint32_t val)
{
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) p[i] = val;
}

constexpr uint32_t kBins = 2048;          // words of one rank's histogram; a block owns four of them
constexpr uint32_t kBits2 = 11, kBits3 = 8;                       // 12 + 11 + 8 bits of the 31-bit key
constexpr uint32_t kShift1 = kBits2 + kBits3, kShift2 = kBits3;   // key >> kShift1: first digit; key >> kShift2: first two
constexpr uint32_t kBins1 = 1u << (31 - kShift1), kBins2 = 1u << kBits2, kBins3 = 1u << kBits3;
static_assert(kBins1 == 2 * kBins && kBins2 == kBins, "the first-digit histogram fills two of a block's four slots");

// The four ranks of a block usually share their key prefix pairwise (lo and lo+1 of a quantile fall
// into one bin).  Elements are matched against the distinct prefixes only; slot_of[t] names the LDS
// histogram that serves rank t, and the flush adds it to every rank that shares it.
struct Prefixes { uint32_t pre[4]; uint32_t slot_of[4]; uint32_t n; };
constexpr uint32_t kNoPrefix = 0xffffffffu;             // never equals a key prefix (at most 23 bits)
__device__ __forceinline__ Prefixes distinct_prefixes(const uint32_t* __restrict__ sel_prefix, uint32_t block)
{
    // fully unrolled with static indices so that everything stays in (scalar) registers
    Prefixes d;
    d.n = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) d.pre[j] = kNoPrefix;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const uint32_t p = sel_prefix[block * 4 + t];
        uint32_t slot = 4;
#pragma unroll
        for (int j = 3; j >= 0; --j)
            if (d.pre[j] == p) slot = j;
        const bool fresh = slot == 4;
        if (fresh) slot = d.n;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (fresh && (uint32_t)j == d.n) d.pre[j] = p;
        if (fresh) d.n += 1;
        d.slot_of[t] = slot;
    }
    return d;
}

// h[u * nb + bin] += 1 for the slot u whose prefix equals hi (the prefixes are distinct, so at most
// one does): the slot is selected first and a single LDS atomic follows.  Slots 2 and 3 are rarely in use.
__device__ __forceinline__ void count_match(uint32_t* h, const Prefixes& d, uint32_t nb, uint32_t hi, uint32_t bin)
{
    bool hit = hi == d.pre[0];
    uint32_t at = bin;
    if (hi == d.pre[1]) { at = nb + bin; hit = true; }
    if (d.n > 2) {
        if (hi == d.pre[2]) { at = 2 * nb + bin; hit = true; }
        if (hi == d.pre[3]) { at = 3 * nb + bin; hit = true; }
    }
    if (hit) atomicAdd(&h[at], 1u);
}

constexpr uint32_t kHistGrid = 2048;     // persistent workgroups of the histogram passes (8 per CU)

// Each workgroup walks a contiguous run of chunks and keeps the histogram of the parameter block it
// is in in LDS; the LDS copy is added to the block's global histogram (integer atomics) only when
// the run crosses into another block and at its end.
template <int PASS>
__global__ __launch_bounds__(256) void k_hist(
    const float* __restrict__ v_all, const Chunk* __restrict__ chunks, const uint32_t* __restrict__ list,
    uint32_t n_chunks, const uint32_t* __restrict__ sel_prefix, uint32_t* __restrict__ hist_all,
    const BlockRow* __restrict__ rows, const uint32_t* __restrict__ scan3)
{
    // list == nullptr: every chunk; otherwise the chunks named by list[0 .. n_chunks).
    // scan3 (third pass over every chunk only): blocks whose flag is 0 have had their last digit counted on
    // their candidate lists and are skipped, a whole block per iteration.
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    constexpr int NT = PASS == 1 ? 1 : 4;
    constexpr uint32_t NB = PASS == 1 ? kBins1 : (PASS == 2 ? kBins2 : kBins3);
    __shared__ uint32_t h[NT * NB];
    const uint32_t per = (n_chunks + gridDim.x - 1) / gridDim.x;
    const uint32_t c0 = blockIdx.x * per, c1 = min(n_chunks, c0 + per);
    if (c0 >= c1) return;
    for (uint32_t i = threadIdx.x; i < NT * NB; i += 256) h[i] = 0;
    uint32_t cur = chunks[list ? list[c0] : c0].block;
    Prefixes d;
    d.n = 0;
    auto load_prefixes = [&]() {
        if (PASS > 1) d = distinct_prefixes(sel_prefix, cur);
    };
    auto flush = [&]() {
        __syncthreads();
        uint32_t* out = hist_all + (uint64_t)cur * 4 * kBins;
        if (PASS == 1) {
            for (uint32_t i = threadIdx.x; i < NB; i += 256) {
                const uint32_t c = h[i];
                if (c) { atomicAdd(&out[i], c); h[i] = 0; }
            }
        } else {
            for (uint32_t i = threadIdx.x; i < NB; i += 256) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {                 // static t: slot_of stays in registers
                    const uint32_t c = h[d.slot_of[t] * NB + i];
                    if (c) atomicAdd(&out[t * kBins + i], c);
                }
            }
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < NT * NB; i += 256) h[i] = 0;
        }
        __syncthreads();
    };
    load_prefixes();
    __syncthreads();
    for (uint32_t c = c0; c < c1;) {
        const Chunk ck = chunks[list ? list[c] : c];
        if (PASS == 3 && scan3 && !scan3[ck.block]) {        // chunk ids of a block are consecutive (list == nullptr here)
            c = rows[ck.block].first_chunk + rows[ck.block].n_chunks;
            continue;
        }
        if (ck.block != cur) { flush(); cur = ck.block; load_prefixes(); }
        const uint32_t* bits = reinterpret_cast<const uint32_t*>(v_all + ck.state_start);
        for (uint32_t e0 = threadIdx.x * 4; e0 < ck.count; e0 += 4096) {
            u4 w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)                              // padded state: e < count is in bounds
                if (e0 + q * 1024 < ck.count) w[q] = ld_stream<u4>(bits + e0 + q * 1024);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t e = e0 + q * 1024;
                if (e >= ck.count) break;
                const uint32_t key[4] = {w[q].x & 0x7fffffffu, w[q].y & 0x7fffffffu, w[q].z & 0x7fffffffu, w[q].w & 0x7fffffffu};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (e + j >= ck.count) break;
                    if (PASS == 1) {
                        atomicAdd(&h[key[j] >> kShift1], 1u);
                    } else {
                        const uint32_t hi = PASS == 2 ? key[j] >> kShift1 : key[j] >> kShift2;
                        const uint32_t bin = PASS == 2 ? (key[j] >> kShift2) & (kBins2 - 1) : key[j] & (kBins3 - 1);
                        count_match(h, d, NB, hi, bin);
                    }
                }
            }
        }
        ++c;
    }
    flush();
}

// One wavefront per (block, rank): every lane sums a run of consecutive bins, a wavefront scan
// finds the lane whose run holds the rank, and that lane walks its run.  The key prefix grows by
// the digit found and the rank is made relative to that bin.  Counts fit 32 bits (numel < 2^32).
template <int PASS>
__global__ __launch_bounds__(64) void k_pick(const uint32_t* __restrict__ hist_all, const BlockRow* __restrict__ rows,
                                             uint32_t* __restrict__ sel_prefix, uint32_t* __restrict__ sel_rank,
                                             float* __restrict__ order_stat, uint32_t* __restrict__ scan3)
{
    constexpr uint32_t NB = PASS == 1 ? kBins1 : (PASS == 2 ? kBins2 : kBins3), PER = NB / 64;
    const uint32_t id = blockIdx.x, b = id >> 2, t = id & 3, lane = threadIdx.x;
    // the first-digit histogram is shared by the four ranks and fills the block's first two slots
    const uint32_t* h = hist_all + ((uint64_t)b * 4 + (PASS == 1 ? 0 : t)) * kBins + lane * PER;
    const uint32_t r = PASS == 1 ? (uint32_t)rows[b].rank[t] : sel_rank[id];
    // Blocks walked chunk-wise have their last digit counted by a third scan; matrix blocks only if
    // a candidate list overflows (set by the second tile pass).
    if (PASS == 1 && t == 0 && lane == 0) scan3[b] = rows[b].vec_first != kNoVec;
    uint32_t cnt[PER], mine = 0;
#pragma unroll
    for (uint32_t i = 0; i < PER; ++i) { cnt[i] = h[i]; mine += cnt[i]; }
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d);
        if ((int)lane >= d) incl += o;
    }
    const uint32_t excl = incl - mine;
    const uint64_t holders = __ballot(r >= excl && r < incl);
    const uint32_t owner = holders ? (uint32_t)__builtin_ctzll(holders) : 63u;
    if (lane == owner) {
        uint32_t rr = r - excl, bin = PER - 1;
        bool found = false;
#pragma unroll
        for (uint32_t i = 0; i < PER; ++i) {
            if (!found) {
                if (rr < cnt[i] || i == PER - 1) { bin = i; found = true; }
                else rr -= cnt[i];
            }
        }
        bin += lane * PER;
        const uint32_t prefix = PASS == 1 ? bin : ((sel_prefix[id] << (PASS == 2 ? kBits2 : kBits3)) | bin);
        sel_prefix[id] = prefix;
        sel_rank[id] = rr;
        if (PASS == 3) order_stat[id] = __builtin_bit_cast(float, prefix);
    }
}

// ---------------------------------------------------------------------------
// Finalize over matrix blocks, tiled.  A task is a tile of up to 256 rows x 256 columns
// of v (viewed as rows x cols) owned by one wavefront; a workgroup takes four consecutive
// tasks of one block.  Two passes over v serve three consumers at once:
//   pass 1: row / column partial sums (Eq. 7), sum of p = 1/(sqrt(v)+eps) (Eq. 6), first
//           radix digit histogram (Eq. 4)
//   pass 2: |S - r c^T / mu|^2 and |S|^2 (Eq. 7), ((p/p-bar - 1) theta)^2 and theta^2 (Eq. 6),
//           second digit histogram, and the keys that carry a selected first digit appended to the
//           task's candidate list (the last digit is then counted on the lists, k_cand_hist3)
// Full tiles on the vector path load their rows one round ahead of their use.
// Blocks without a matrix shape are walked chunk-wise by k_hist / k_distortion instead.
// ---------------------------------------------------------------------------

constexpr uint32_t kTileRows = 256, kTileCols = 256;

struct alignas(8) MatRow {
    uint64_t state_start;                 // first coordinate of the block in v
    uint64_t grad_start;                  // the block's offset in the caller's flat buffers (theta)
    uint64_t off_r, off_c;                // into the r / c vectors (floats)
    uint64_t off_rowpart, off_colpart;    // into the partial-sum arrays (floats)
    uint64_t cand_base;                   // the block's first candidate list (words into the candidate buffer)
    uint32_t rows, cols, n_tiles, n_segs;
    uint32_t first_task, first_quad, block;
    uint32_t cand_cap;                    // words per candidate list (one list per task)
};

struct MatTask { uint32_t mat, task, row0, row1, col0, ncols, tile, seg; bool vec, valid; };

// Workgroup `quad` -> its block and this wavefront's task (tile index fastest).
// `wave` must be uniform over the wavefront (callers pass it through readfirstlane), so that the task and
// every address derived from it live in scalar registers.
__device__ __forceinline__ MatTask decode_quad(const MatRow* __restrict__ mats, uint32_t n_mats, uint32_t quad, uint32_t wave)
{
    uint32_t lo = 0, hi = n_mats - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (mats[mid].first_quad <= quad) lo = mid; else hi = mid - 1;
    }
    const MatRow& m = mats[lo];
    const uint32_t local = (quad - m.first_quad) * 4 + wave;
    MatTask t;
    t.mat = lo; t.valid = local < m.n_tiles * m.n_segs;
    t.task = m.first_task + local;
    t.seg = local / m.n_tiles; t.tile = local % m.n_tiles;
    t.row0 = t.seg * kTileRows; t.row1 = t.valid ? min(m.rows, t.row0 + kTileRows) : t.row0;
    t.col0 = t.tile * kTileCols; t.ncols = t.valid ? min(kTileCols, m.cols - t.col0) : 0;
    t.vec = (m.cols & 3u) == 0;           // rows start 16-byte aligned (blocks start on 1 KB)
    return t;
}

// Column owned by slot k of a lane: 4 consecutive columns on the vector path, stride 64 otherwise.
__device__ __forceinline__ uint32_t tile_col(bool vec, uint32_t lane, int k) { return vec ? 4 * lane + k : lane + 64 * k; }

__device__ __forceinline__ void load_tile_row(const float* __restrict__ row, bool vec, uint32_t lane, uint32_t ncols, float x[4])
{
    if (vec) {
        if (4 * lane < ncols) {
            const f4 t = ld_stream<f4>(row + 4 * lane);
            x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
        } else {
            x[0] = x[1] = x[2] = x[3] = 0.f;
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = (lane + 64 * k < ncols) ? row[lane + 64 * k] : 0.f;
    }
}

template <int TT>
__device__ __forceinline__ void load_tile_theta(const typename GradIO<TT>::elem* __restrict__ row, bool vec, bool aligned,
                                                uint32_t lane, uint32_t ncols, float x[4])
{
    // column ownership follows v's (vec: 4 consecutive columns per lane); `aligned` only picks the load width
    typedef GradIO<TT> IO;
    if (vec) {
        if (4 * lane < ncols) {
            if (aligned) IO::load4(row + 4 * lane, x);
            else {
#pragma unroll
                for (int k = 0; k < 4; ++k) x[k] = IO::load1(row + 4 * lane + k);
            }
        } else {
            x[0] = x[1] = x[2] = x[3] = 0.f;
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = (lane + 64 * k < ncols) ? IO::load1(row + lane + 64 * k) : 0.f;
    }
}

__device__ __forceinline__ uint32_t scalar_wave_index()
{
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}

constexpr int kRowsAhead = 2;             // rows of a full tile loaded per round, one round ahead of their use

__global__ __launch_bounds__(256) void k_tile_pass1(
    const float* __restrict__ v_all, const MatRow* __restrict__ mats, uint32_t n_mats,
    float* __restrict__ rowpart, float* __restrict__ colpart, float* __restrict__ psumpart,
    uint32_t* __restrict__ hist_all, float eps, bool want_p)
{
    __shared__ uint32_t h[kBins1];
    __shared__ float rowsum[4][kTileRows];                // a tile's row sums, written out together at the end
    const uint32_t lane = threadIdx.x & 63u, wave = scalar_wave_index();
    for (uint32_t i = threadIdx.x; i < kBins1; i += 256) h[i] = 0;
    const MatTask t = decode_quad(mats, n_mats, blockIdx.x, wave);
    const MatRow& m = mats[t.mat];
    __syncthreads();
    if (t.valid) {
        const float* row = v_all + m.state_start + (uint64_t)t.row0 * m.cols + t.col0;
        bool ok[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) ok[k] = tile_col(t.vec, lane, k) < t.ncols;
        // Column sums and the sum of p run over up to 256 rows per lane: kept in fp64 so that a constant
        // v (rank one, p constant) comes out as such to ~1e-7 instead of the ~1e-5 of a long fp32 chain.
        double cs[4] = {0.0, 0.0, 0.0, 0.0}, psum = 0.0;
        float* rs_out = rowsum[wave];
        auto consume = [&](auto full, const float x[4]) {
            constexpr bool FULL = decltype(full)::value;     // every column of the lane is inside the tile
            float prow = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                cs[k] += (double)x[k];
                if (FULL || ok[k]) {
                    atomicAdd(&h[(__builtin_bit_cast(uint32_t, x[k]) & 0x7fffffffu) >> kShift1], 1u);
                    if (want_p) prow += preconditioner(x[k], eps);
                }
            }
            psum += (double)prow;
            return wave_sum((x[0] + x[1]) + (x[2] + x[3]));
        };
        uint32_t r = t.row0;
        if (t.vec && t.ncols == kTileCols) {
            const float* vp = row + 4 * lane;
            f4 nx[kRowsAhead];
#pragma unroll
            for (int q = 0; q < kRowsAhead; ++q) nx[q] = f4{0.f, 0.f, 0.f, 0.f};
            auto issue = [&](uint32_t r0) {
#pragma unroll
                for (int q = 0; q < kRowsAhead; ++q)
                    if (r0 + q < t.row1) nx[q] = ld_stream<f4>(vp + (uint64_t)(r0 + q - t.row0) * m.cols);
            };
            issue(r);
            for (; r < t.row1; r += kRowsAhead) {
                f4 cx[kRowsAhead];
#pragma unroll
                for (int q = 0; q < kRowsAhead; ++q) cx[q] = nx[q];
                if (r + kRowsAhead < t.row1) issue(r + kRowsAhead);
#pragma unroll
                for (int q = 0; q < kRowsAhead; ++q) {
                    if (r + q >= t.row1) break;
                    const float x[4] = {cx[q].x, cx[q].y, cx[q].z, cx[q].w};
                    const float rs = consume(std::true_type(), x);
                    if (lane == 0) rs_out[r + q - t.row0] = rs;
                }
            }
        } else {
            for (; r < t.row1; ++r) {
                float x[4];
                load_tile_row(row, t.vec, lane, t.ncols, x);
                const float rs = consume(std::false_type(), x);
                if (lane == 0) rs_out[r - t.row0] = rs;
                row += m.cols;
            }
        }
        // row sums of this tile: rowpart is tile-major ([tile][row]), so the wavefront writes one run
        {
            float* rp = rowpart + m.off_rowpart + (uint64_t)t.tile * m.rows + t.row0;
            const uint32_t nr = t.row1 - t.row0;
#pragma unroll
            for (uint32_t j = 0; j < kTileRows / 64; ++j)
                if (lane + 64 * j < nr) rp[lane + 64 * j] = rs_out[lane + 64 * j];
        }
        float* cp = colpart + m.off_colpart + (uint64_t)t.seg * m.cols + t.col0;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (ok[k]) cp[tile_col(t.vec, lane, k)] = (float)cs[k];
        const float ptile = wave_sum((float)psum);
        if (lane == 0) psumpart[t.task] = ptile;
    }
    __syncthreads();
    uint32_t* out = hist_all + (uint64_t)m.block * 4 * kBins;
    for (uint32_t i = threadIdx.x; i < kBins1; i += 256)
        if (h[i]) atomicAdd(&out[i], h[i]);
}

// r_i, c_j (fp32 for pass 2) and, per slice, the sums behind mu and the block's sum of p, from the pass-1
// partial sums.  A matrix block is cut into kFinSlices slices of rows, of columns and of tasks (grid.y).
constexpr uint32_t kFinSlices = 32;

__global__ __launch_bounds__(256) void k_tile_finish1(const MatRow* __restrict__ mats, const float* __restrict__ rowpart,
                                                      const float* __restrict__ colpart, const float* __restrict__ psumpart,
                                                      float* __restrict__ rvec, float* __restrict__ cvec,
                                                      double* __restrict__ finpart)
{
    const MatRow m = mats[blockIdx.x];
    const uint32_t y = blockIdx.y;
    double local = 0.0, lp = 0.0;
    const uint32_t rper = (m.rows + kFinSlices - 1) / kFinSlices, i1 = min(m.rows, (y + 1) * rper);
    for (uint32_t i = y * rper + threadIdx.x; i < i1; i += 256) {
        const float* rp = rowpart + m.off_rowpart + i;                       // tile-major: [tile][row]
        double s = 0.0;
        for (uint32_t t = 0; t < m.n_tiles; ++t) s += (double)rp[(uint64_t)t * m.rows];
        const double r = s / (double)m.cols;
        rvec[m.off_r + i] = (float)r;
        local += r;
    }
    const uint32_t cper = (m.cols + kFinSlices - 1) / kFinSlices, j1 = min(m.cols, (y + 1) * cper);
    for (uint32_t j = y * cper + threadIdx.x; j < j1; j += 256) {
        const float* cp = colpart + m.off_colpart + j;
        double s = 0.0;
        for (uint32_t g = 0; g < m.n_segs; ++g) s += (double)cp[(uint64_t)g * m.cols];
        cvec[m.off_c + j] = (float)(s / (double)m.rows);
    }
    const uint32_t n_tasks = m.n_tiles * m.n_segs, tper = (n_tasks + kFinSlices - 1) / kFinSlices, k1 = min(n_tasks, (y + 1) * tper);
    for (uint32_t i = y * tper + threadIdx.x; i < k1; i += 256) lp += (double)psumpart[m.first_task + i];
    __shared__ double sh[256], sp[256];
    sh[threadIdx.x] = local; sp[threadIdx.x] = lp;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) { sh[threadIdx.x] += sh[threadIdx.x + w]; sp[threadIdx.x] += sp[threadIdx.x + w]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        double* o = finpart + ((uint64_t)blockIdx.x * kFinSlices + y) * 2;
        o[0] = sh[0]; o[1] = sp[0];
    }
}

// mu (fp64) and the block's sum of p: the slices of k_tile_finish1 added in a fixed order.
__global__ __launch_bounds__(64) void k_tile_finish1_sum(const MatRow* __restrict__ mats, const double* __restrict__ finpart,
                                                         double* __restrict__ mu_out, double* __restrict__ rec_all)
{
    if (threadIdx.x != 0) return;
    const MatRow& m = mats[blockIdx.x];
    const double* in = finpart + (uint64_t)blockIdx.x * kFinSlices * 2;
    double a = 0.0, p = 0.0;
    for (uint32_t y = 0; y < kFinSlices; ++y) { a += in[2 * y]; p += in[2 * y + 1]; }
    mu_out[blockIdx.x] = a / (double)m.rows;
    rec_all[(uint64_t)m.block * kRecDoubles + R_PSUM] = p;
}

template <int TT>
__global__ __launch_bounds__(256) void k_tile_pass2(
    const float* __restrict__ v_all, const typename GradIO<TT>::elem* __restrict__ theta,
    const MatRow* __restrict__ mats, uint32_t n_mats,
    const float* __restrict__ rvec, const float* __restrict__ cvec, const double* __restrict__ mu_all,
    const double* __restrict__ rec_all, const uint32_t* __restrict__ sel_prefix,
    float* __restrict__ residpart, uint32_t* __restrict__ hist_all,
    uint32_t* __restrict__ cand, uint32_t* __restrict__ cand_count, uint32_t* __restrict__ scan3,
    float eps, bool want_F, bool want_C)
{
    typedef GradIO<TT> IO;
    typedef typename IO::vec4 TV;
    // LDS histograms for the first two distinct prefixes (lo and lo+1 of a quantile almost always share
    // theirs); a third or fourth distinct prefix is rare and counts straight into global memory.
    constexpr uint32_t NSLOT = 2;
    __shared__ uint32_t h[NSLOT * kBins2];
    const uint32_t lane = threadIdx.x & 63u, wave = scalar_wave_index();
    for (uint32_t i = threadIdx.x; i < NSLOT * kBins2; i += 256) h[i] = 0;
    const MatTask t = decode_quad(mats, n_mats, blockIdx.x, wave);
    const MatRow& m = mats[t.mat];
    const Prefixes d = distinct_prefixes(sel_prefix, m.block);
    uint32_t* hist_out = hist_all + (uint64_t)m.block * 4 * kBins;
    __syncthreads();
    if (t.valid) {
        const double mu = mu_all[t.mat];
        // c_j / mu is formed in fp64 (mu may lie below the fp32 normal range); S~ = 0 when mu = 0
        float inv_pbar = 0.f;
        if (want_C) inv_pbar = (float)((double)((uint64_t)m.rows * m.cols) / rec_all[(uint64_t)m.block * kRecDoubles + R_PSUM]);
        bool ok[4]; float cm[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t c = tile_col(t.vec, lane, k);
            ok[k] = c < t.ncols;
            cm[k] = (ok[k] && mu != 0.0) ? (float)((double)cvec[m.off_c + t.col0 + c] / mu) : 0.f;
        }
        const uint64_t first = (uint64_t)t.row0 * m.cols + t.col0;
        const float* row = v_all + m.state_start + first;
        const typename IO::elem* trow = theta + m.grad_start + first;
        const bool talign = (reinterpret_cast<uintptr_t>(trow) & IO::kAlignMask) == 0;   // cols % 4 == 0: same for all rows
        const float* rr = rvec + m.off_r + t.row0;
        uint32_t* list = cand + m.cand_base + (uint64_t)(t.task - m.first_task) * m.cand_cap;
        uint32_t n_cand = 0;                                  // uniform over the wavefront
        float res = 0.f, s2 = 0.f, cn = 0.f, cd = 0.f;
        auto consume = [&](auto full, const float x[4], const float th[4], float ri) {
            constexpr bool FULL = decltype(full)::value;     // every column of the lane is inside the tile
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool in = FULL || ok[k];
                const uint32_t key = __builtin_bit_cast(uint32_t, x[k]) & 0x7fffffffu;
                const uint32_t hi = key >> kShift1, bin = (key >> kShift2) & (kBins2 - 1);
                bool hit = false;
                if (in) {
                    if (hi == d.pre[0]) { atomicAdd(&h[bin], 1u); hit = true; }
                    else if (hi == d.pre[1]) { atomicAdd(&h[kBins2 + bin], 1u); hit = true; }
                    else if (d.n > 2 && (hi == d.pre[2] || hi == d.pre[3])) {
                        const uint32_t slot = hi == d.pre[2] ? 2u : 3u;
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            if (d.slot_of[q] == slot) atomicAdd(&hist_out[q * kBins + bin], 1u);
                        hit = true;
                    }
                }
                // candidates: the keys that carry a selected first digit, in the task's own list
                const uint64_t hits = __builtin_amdgcn_ballot_w64(hit);
                if (hits) {
                    const uint32_t at = n_cand + __builtin_amdgcn_mbcnt_hi((uint32_t)(hits >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)hits, 0u));
                    if (hit && at < m.cand_cap) list[at] = key;
                    n_cand += (uint32_t)__builtin_popcountll(hits);
                }
                if (in) {
                    if (want_F) {
                        const float dd = x[k] - ri * cm[k];
                        res = __builtin_fmaf(dd, dd, res);
                        s2 = __builtin_fmaf(x[k], x[k], s2);
                    }
                    if (want_C) {
                        const float p = preconditioner(x[k], eps);
                        const float y = (p * inv_pbar - 1.0f) * th[k];
                        cn = __builtin_fmaf(y, y, cn);
                        cd = __builtin_fmaf(th[k], th[k], cd);
                    }
                }
            }
        };
        uint32_t r = t.row0;
        if (t.vec && talign && t.ncols == kTileCols) {
            const float* vp = row + 4 * lane;
            const typename IO::elem* tp = trow + 4 * lane;
            f4 nx[kRowsAhead]; TV nt[kRowsAhead]; float nr[kRowsAhead];
#pragma unroll
            for (int q = 0; q < kRowsAhead; ++q) { nx[q] = f4{0.f, 0.f, 0.f, 0.f}; nt[q] = TV{}; nr[q] = 0.f; }
            auto issue = [&](uint32_t r0) {
#pragma unroll
                for (int q = 0; q < kRowsAhead; ++q)
                    if (r0 + q < t.row1) {
                        const uint64_t o = (uint64_t)(r0 + q - t.row0) * m.cols;
                        nx[q] = ld_stream<f4>(vp + o);
                        if (want_C) nt[q] = IO::loadv(tp + o);
                        nr[q] = rr[r0 + q - t.row0];
                    }
            };
            issue(r);
            for (; r < t.row1; r += kRowsAhead) {
                f4 cx[kRowsAhead]; TV ct[kRowsAhead]; float cr[kRowsAhead];
#pragma unroll
                for (int q = 0; q < kRowsAhead; ++q) { cx[q] = nx[q]; ct[q] = nt[q]; cr[q] = nr[q]; }
                if (r + kRowsAhead < t.row1) issue(r + kRowsAhead);
#pragma unroll
                for (int q = 0; q < kRowsAhead; ++q) {
                    if (r + q >= t.row1) break;
                    const float x[4] = {cx[q].x, cx[q].y, cx[q].z, cx[q].w};
                    float th[4] = {0.f, 0.f, 0.f, 0.f};
                    if (want_C) IO::unpack(ct[q], th);
                    consume(std::true_type(), x, th, cr[q]);
                }
            }
        } else {
            for (; r < t.row1; ++r) {
                float x[4], th[4] = {0.f, 0.f, 0.f, 0.f};
                load_tile_row(row, t.vec, lane, t.ncols, x);
                if (want_C) load_tile_theta<TT>(trow, t.vec, talign, lane, t.ncols, th);
                consume(std::false_type(), x, th, *rr);
                row += m.cols; trow += m.cols; ++rr;
            }
        }
        res = wave_sum(res); s2 = wave_sum(s2); cn = wave_sum(cn); cd = wave_sum(cd);
        if (lane == 0) {
            float* o = residpart + (uint64_t)t.task * 4;
            o[0] = res; o[1] = s2; o[2] = cn; o[3] = cd;
            cand_count[t.task] = n_cand;
            if (n_cand > m.cand_cap) scan3[m.block] = 1u;    // list too short: the block's last digit takes a third scan
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < kBins2; i += 256) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (d.slot_of[q] >= NSLOT) continue;
            const uint32_t c = h[d.slot_of[q] * kBins2 + i];
            if (c) atomicAdd(&hist_out[q * kBins + i], c);
        }
    }
}

// Third digit of the matrix blocks, counted on the candidate lists that the second tile pass wrote (a few
// per cent of the coordinates).  Blocks flagged in scan3 are left to the third scan of v.
__global__ __launch_bounds__(256) void k_cand_hist3(
    const MatRow* __restrict__ mats, uint32_t n_mats, const uint32_t* __restrict__ cand,
    const uint32_t* __restrict__ cand_count, const uint32_t* __restrict__ sel_prefix,
    const uint32_t* __restrict__ scan3, uint32_t* __restrict__ hist_all)
{
    __shared__ uint32_t h[4 * kBins3];
    const uint32_t lane = threadIdx.x & 63u, wave = scalar_wave_index();
    const MatTask t = decode_quad(mats, n_mats, blockIdx.x, wave);
    const MatRow& m = mats[t.mat];
    if (scan3[m.block]) return;                              // the same for the whole workgroup (one block per quad)
    for (uint32_t i = threadIdx.x; i < 4 * kBins3; i += 256) h[i] = 0;
    const Prefixes d = distinct_prefixes(sel_prefix, m.block);
    __syncthreads();
    if (t.valid) {
        const uint32_t n = min(cand_count[t.task], m.cand_cap);
        const uint32_t* list = cand + m.cand_base + (uint64_t)(t.task - m.first_task) * m.cand_cap;
        for (uint32_t i = lane; i < n; i += 64) {
            const uint32_t key = list[i];
            count_match(h, d, kBins3, key >> kShift2, key & (kBins3 - 1));
        }
    }
    __syncthreads();
    uint32_t* out = hist_all + (uint64_t)m.block * 4 * kBins;
    for (uint32_t i = threadIdx.x; i < kBins3; i += 256) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t c = h[d.slot_of[q] * kBins3 + i];
            if (c) atomicAdd(&out[q * kBins + i], c);
        }
    }
}

__global__ __launch_bounds__(256) void k_tile_finish2(const MatRow* __restrict__ mats, const float* __restrict__ residpart,
                                                      double* __restrict__ rec_all)
{
    const MatRow m = mats[blockIdx.x];
    const uint32_t n = m.n_tiles * m.n_segs;
    double a[4] = {0.0, 0.0, 0.0, 0.0};
    for (uint32_t i = threadIdx.x; i < n; i += 256) {
        const f4 t = *reinterpret_cast<const f4*>(residpart + (uint64_t)(m.first_task + i) * 4);
        a[0] += (double)t.x; a[1] += (double)t.y; a[2] += (double)t.z; a[3] += (double)t.w;
    }
    __shared__ double sh[4][256];
#pragma unroll
    for (int q = 0; q < 4; ++q) sh[q][threadIdx.x] = a[q];
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
#pragma unroll
            for (int q = 0; q < 4; ++q) sh[q][threadIdx.x] += sh[q][threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        double* rec = rec_all + (uint64_t)m.block * kRecDoubles;
        rec[R_FRES] = sh[0][0]; rec[R_FS2] = sh[1][0]; rec[R_CNUM] = sh[2][0]; rec[R_CDEN] = sh[3][0];
    }
}

// ---------------------------------------------------------------------------
// Eq. 6 on the chunks of blocks without a matrix shape.  p = 1/(sqrt(v) + eps).
// Pass 1: sum of p per chunk (-> p-bar per block).  Pass 2: sum of
// ((p/p-bar - 1) theta)^2 and of theta^2 per chunk.  theta is laid out like the
// gradient buffer.  Partial rows reuse the step's partial-sum buffer.
// ---------------------------------------------------------------------------

template <int TT, int PASS>
__global__ __launch_bounds__(256) void k_distortion(
    const float* __restrict__ v_all, const typename GradIO<TT>::elem* __restrict__ theta,
    const Chunk* __restrict__ chunks, const uint32_t* __restrict__ list, const BlockRow* __restrict__ rows,
    const double* __restrict__ rec_all, float* __restrict__ partials, float eps)
{
    typedef GradIO<TT> IO;
    const uint32_t cid = list[blockIdx.x];
    const Chunk ck = chunks[cid];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const typename IO::elem* tsrc = theta + ck.grad_start;
    const bool vec_ok = (reinterpret_cast<uintptr_t>(tsrc) & IO::kAlignMask) == 0;
    float inv_pbar = 0.f;
    if (PASS == 2) inv_pbar = (float)((double)rows[ck.block].numel / rec_all[(uint64_t)ck.block * kRecDoubles + R_PSUM]);
    float a0 = 0.f, a1 = 0.f;
    for (uint32_t e = threadIdx.x * 4; e < ck.count; e += 1024) {
        const f4 vv = ld_stream<f4>(v_all + ck.state_start + e);
        const float v[4] = {vv.x, vv.y, vv.z, vv.w};
        float th[4] = {0.f, 0.f, 0.f, 0.f};
        if (PASS == 2) {
            if (vec_ok && e + 4 <= ck.count) IO::load4(tsrc + e, th);
            else {
#pragma unroll
                for (int j = 0; j < 4; ++j) th[j] = (e + j < ck.count) ? IO::load1(tsrc + e + j) : 0.f;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (e + j < ck.count) {                          // padding coordinates are not part of the block
                const float p = preconditioner(v[j], eps);
                if (PASS == 1) a0 += p;
                else {
                    const float x = (p * inv_pbar - 1.0f) * th[j];
                    a0 = __builtin_fmaf(x, x, a0);
                    a1 = __builtin_fmaf(th[j], th[j], a1);
                }
            }
        }
    }
    __shared__ float red[4][2];
    a0 = wave_sum(a0); a1 = wave_sum(a1);
    if (lane == 0) { red[wave][0] = a0; red[wave][1] = a1; }
    __syncthreads();
    if (threadIdx.x < 2)
        partials[(uint64_t)cid * kNumSums + threadIdx.x] =
            (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// Per chunk-walked block: fp64 sum of the first `ncols` entries of its partial rows into rec[dst .. dst+ncols).
__global__ __launch_bounds__(256) void k_reduce_partials(const float* __restrict__ partials, const BlockRow* __restrict__ rows,
                                                         double* __restrict__ rec_all, uint32_t ncols, uint32_t dst)
{
    const BlockRow br = rows[blockIdx.x];
    if (br.vec_first == kNoVec) return;                      // tiled block: its sums come from k_tile_finish*
    __shared__ double sh[256];
    for (uint32_t col = 0; col < ncols; ++col) {
        double a = 0.0;
        for (uint32_t c = threadIdx.x; c < br.n_chunks; c += 256) a += (double)partials[(uint64_t)(br.first_chunk + c) * kNumSums + col];
        sh[threadIdx.x] = a;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) rec_all[(uint64_t)blockIdx.x * kRecDoubles + dst + col] = sh[0];
        __syncthreads();
    }
}

}  // namespace baoc

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

using namespace baoc;

// Workspace of baoc_profile_begin_static: one array per GPU, resident from the moment the code object is
// loaded until the process ends.  In host code the name below is only a handle for hipGetSymbolAddress;
// the device address is looked up once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[BAOC_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each GPU
static bool g_scratch_busy[kMaxDevices] = {};      // a handle begun with baoc_profile_begin_static is alive

struct Plan {
    uint64_t n_chunks = 0;
    uint32_t gpw = 1, nw = 4, slices = 1, slice_groups = 4, resident = 8;   // launch shape of the step kernel
    uint64_t n_prows = 0;         // partial rows of the step kernel = n_chunks * slices
    std::vector<BlockRow> rows;
    std::vector<MatRow> mats;     // matrix blocks (rows*cols == numel), for Eq. 7
    uint64_t n_tasks = 0, n_quads = 0, n_vec_chunks = 0;
    std::vector<Slab> slabs;
    uint64_t off_slabs = 0, off_slabsums = 0;
    uint64_t off_mats = 0, off_rvec = 0, off_cvec = 0, off_rowpart = 0, off_colpart = 0, off_residpart = 0, off_mu = 0,
             off_psumpart = 0, off_veclist = 0, off_cand = 0, off_candcount = 0, off_scan3 = 0, off_finpart = 0;
    uint64_t padded = 0;          // coordinates in m / v / g_prev
    uint64_t off_m = 0, off_v = 0, off_gp = 0, off_partials = 0, off_chunks = 0, off_rows = 0,
             off_rec = 0, off_hist = 0, off_selp = 0, off_selr = 0, off_ostat = 0, total = 0;
};

struct baoc_profiler {
    baoc_profile_params params;
    Plan plan;
    std::vector<baoc_block> blocks;
    char* ws = nullptr;
    int static_device = -1;       // >= 0: the workspace is that device's `scratch` array
    uint32_t steps = 0;
    uint64_t max_end = 0;         // largest offset + numel over the blocks
    int sticky = BAOC_OK;
    std::vector<double> h_rec;
    std::vector<float> h_ostat;
};

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

static int check_params(const baoc_profile_params* p)
{
    if (!p) return BAOC_ERR_INVALID;
    if (!(p->beta_m > 0.f && p->beta_m < 1.f) || !(p->beta_v > 0.f && p->beta_v < 1.f)) return BAOC_ERR_INVALID;
    if (!(p->beta_rho >= 0.0 && p->beta_rho < 1.0)) return BAOC_ERR_INVALID;
    if (!(p->eps >= 0.0) || !(p->eps_update > 0.f)) return BAOC_ERR_INVALID;   // u = m / (sqrt(v) + eps_update) must exist where v = 0
    if (p->grad_dtype != BAOC_GRAD_F32 && p->grad_dtype != BAOC_GRAD_BF16) return BAOC_ERR_INVALID;
    if (p->quant_block != kQB) return BAOC_ERR_UNSUPPORTED;
    if (p->chunk_groups > 4096 || p->groups_per_wave > 2 || p->chunk_slices > 64) return BAOC_ERR_INVALID;
    if (p->waves_per_workgroup != 0 && p->waves_per_workgroup != 1 && p->waves_per_workgroup != 2 && p->waves_per_workgroup != 4)
        return BAOC_ERR_INVALID;
    if (p->resident_workgroups != 0 && (p->resident_workgroups < 3 || p->resident_workgroups > 32)) return BAOC_ERR_INVALID;
    return BAOC_OK;
}

static int make_plan(const baoc_block* blocks, uint32_t n, const baoc_profile_params* prm, Plan* out, uint64_t* max_end)
{
    if (!blocks || n == 0) return BAOC_ERR_INVALID;
    int rc = check_params(prm);
    if (rc) return rc;
    // no overlap: sort a copy by offset
    std::vector<std::pair<uint64_t, uint64_t>> iv(n);
    uint64_t end_max = 0;
    for (uint32_t i = 0; i < n; ++i) {
        const baoc_block& b = blocks[i];
        if (b.numel == 0) return BAOC_ERR_INVALID;
        if (b.numel > 0xffffffffull) return BAOC_ERR_UNSUPPORTED;      // 32-bit histogram counters
        if (b.offset + b.numel < b.offset) return BAOC_ERR_INVALID;
        if ((b.rows || b.cols) && (uint64_t)b.rows * b.cols != b.numel) return BAOC_ERR_INVALID;
        iv[i] = {b.offset, b.numel};
        end_max = std::max(end_max, b.offset + b.numel);
    }
    std::sort(iv.begin(), iv.end());
    for (uint32_t i = 1; i < n; ++i)
        if (iv[i - 1].first + iv[i - 1].second > iv[i].first) return BAOC_ERR_INVALID;
    if (max_end) *max_end = end_max;

    Plan& P = *out;
    uint64_t total = 0;
    for (uint32_t i = 0; i < n; ++i) total += blocks[i].numel;
    // fp32 layouts too small to keep the chip busy for long (ResNet-50-sized) run faster with the 4-wavefront shape
    const LaunchShape& ds = (prm->grad_dtype == BAOC_GRAD_F32 && total < kSmallLayout) ? kSmallF32Shape : kDefaultShape[prm->grad_dtype];
    P.gpw = prm->groups_per_wave ? prm->groups_per_wave : ds.groups_per_wave;
    P.nw = prm->waves_per_workgroup ? prm->waves_per_workgroup : ds.waves_per_workgroup;
    P.resident = prm->resident_workgroups ? prm->resident_workgroups : ds.resident_workgroups;
    const uint32_t round = P.gpw * P.nw;                            // groups a workgroup takes per round
    const uint32_t cg = prm->chunk_groups ? prm->chunk_groups : std::max(ds.chunk_groups, round);
    P.slices = prm->chunk_slices ? std::min(prm->chunk_slices, cg) : std::max(1u, cg / round);   // default: one round per slice
    P.slice_groups = (cg + P.slices - 1) / P.slices;
    P.n_chunks = 0; P.rows.resize(n); P.slabs.clear();
    uint64_t state = 0;
    for (uint32_t i = 0; i < n; ++i) {
        const baoc_block& b = blocks[i];
        const uint64_t groups = (b.numel + kQB - 1) / kQB;
        const uint64_t nch = (groups + cg - 1) / cg;
        const uint64_t per = (groups + nch - 1) / nch;               // balanced, whole groups
        BlockRow& r = P.rows[i];
        r.grad_start = b.offset; r.state_start = state; r.numel = b.numel;
        r.first_chunk = (uint32_t)P.n_chunks;
        r.n_chunks = (uint32_t)((groups + per - 1) / per);
        r.groups_per_chunk = (uint32_t)per; r.vec_first = 0;
        const uint64_t prows = (uint64_t)r.n_chunks * P.slices, first_prow = P.n_chunks * P.slices;
        if (first_prow + prows > 0x7fffffffull) return BAOC_ERR_UNSUPPORTED;
        r.first_prow = (uint32_t)first_prow; r.n_prows = (uint32_t)prows;
        r.first_slab = (uint32_t)P.slabs.size();
        if (r.n_prows > kSlabRows)                                   // small blocks are summed directly
            for (uint32_t c = 0; c < r.n_prows; c += kSlabRows)
                P.slabs.push_back(Slab{r.first_prow + c, std::min(kSlabRows, r.n_prows - c)});
        r.n_slabs = (uint32_t)P.slabs.size() - r.first_slab;
        P.n_chunks += r.n_chunks;
        for (int q = 0; q < 2; ++q) {                                // ranks bracketing position q (d-1)
            const double pos = (q == 0 ? 0.1 : 0.9) * (double)(b.numel - 1);
            const uint64_t lo = (uint64_t)std::floor(pos);
            r.rank[2 * q] = lo;
            r.rank[2 * q + 1] = std::min<uint64_t>(lo + 1, b.numel - 1);
        }
        state += groups * kQB;
        if (P.n_chunks > 0x7fffffffull) return BAOC_ERR_UNSUPPORTED;
    }
    P.padded = state;
    P.n_prows = P.n_chunks * P.slices;
    // Finalize walks blocks with a real matrix shape tile-wise and the rest chunk-wise.  A shape with a
    // single row or column is rank one by construction (F = 0 exactly) and stays on the chunk path.
    P.mats.clear(); P.n_tasks = 0; P.n_quads = 0; P.n_vec_chunks = 0;
    uint64_t n_r = 0, n_c = 0, n_rowpart = 0, n_colpart = 0, n_cand = 0;
    for (uint32_t i = 0; i < n; ++i) {
        const baoc_block& b = blocks[i];
        if (b.rows < 2 || b.cols < 2) {
            P.rows[i].vec_first = (uint32_t)P.n_vec_chunks;
            P.n_vec_chunks += P.rows[i].n_chunks;
            continue;
        }
        P.rows[i].vec_first = kNoVec;
        MatRow m;
        m.state_start = P.rows[i].state_start; m.grad_start = b.offset;
        m.rows = b.rows; m.cols = b.cols;
        m.n_tiles = (b.cols + kTileCols - 1) / kTileCols; m.n_segs = (b.rows + kTileRows - 1) / kTileRows;
        m.off_r = n_r; m.off_c = n_c; m.off_rowpart = n_rowpart; m.off_colpart = n_colpart;
        m.first_task = (uint32_t)P.n_tasks; m.first_quad = (uint32_t)P.n_quads; m.block = i;
        n_r += b.rows; n_c += b.cols;
        n_rowpart += (uint64_t)b.rows * m.n_tiles; n_colpart += (uint64_t)m.n_segs * b.cols;
        const uint64_t tasks = (uint64_t)m.n_tiles * m.n_segs;
        // one candidate list per task, an eighth of a tile long (the keys that share a selected first digit
        // are a few per cent of a block unless its v is nearly constant; then the list overflows and the
        // block takes the third scan)
        const uint64_t tile_elems = (uint64_t)std::min(b.rows, kTileRows) * std::min(b.cols, kTileCols);
        m.cand_cap = (uint32_t)align_up(std::max<uint64_t>(64, tile_elems / 8), 64);
        m.cand_base = n_cand;
        n_cand += tasks * m.cand_cap;
        P.n_tasks += tasks; P.n_quads += (tasks + 3) / 4;
        if (P.n_tasks > 0x7fffffffull) return BAOC_ERR_UNSUPPORTED;
        P.mats.push_back(m);
    }
    const uint64_t gsz = prm->grad_dtype == BAOC_GRAD_F32 ? 4 : 2;
    uint64_t o = 0;
    P.off_m = o;        o = align_up(o + P.padded * 4, 256);
    P.off_v = o;        o = align_up(o + P.padded * 4, 256);
    P.off_gp = o;       o = align_up(o + P.padded * gsz, 256);
    P.off_partials = o; o = align_up(o + P.n_prows * kNumSums * 4, 256);   // also holds the per-chunk sums of Eq. 6
    P.off_chunks = o;   o = align_up(o + P.n_chunks * sizeof(Chunk), 256);
    P.off_rows = o;     o = align_up(o + (uint64_t)n * sizeof(BlockRow), 256);
    P.off_rec = o;      o = align_up(o + (uint64_t)n * kRecDoubles * 8, 256);
    P.off_hist = o;     o = align_up(o + (uint64_t)n * 4 * kBins * 4, 256);
    P.off_selp = o;     o = align_up(o + (uint64_t)n * 4 * 4, 256);
    P.off_selr = o;     o = align_up(o + (uint64_t)n * 4 * 4, 256);
    P.off_ostat = o;    o = align_up(o + (uint64_t)n * 4 * 4, 256);
    P.off_mats = o;     o = align_up(o + P.mats.size() * sizeof(MatRow), 256);
    P.off_mu = o;       o = align_up(o + P.mats.size() * 8, 256);
    P.off_rvec = o;     o = align_up(o + n_r * 4, 256);
    P.off_cvec = o;     o = align_up(o + n_c * 4, 256);
    P.off_rowpart = o;  o = align_up(o + n_rowpart * 4, 256);
    P.off_colpart = o;  o = align_up(o + n_colpart * 4, 256);
    P.off_residpart = o; o = align_up(o + P.n_tasks * 4 * 4, 256);
    P.off_psumpart = o; o = align_up(o + P.n_tasks * 4, 256);
    P.off_veclist = o;  o = align_up(o + P.n_vec_chunks * 4, 256);
    P.off_slabs = o;    o = align_up(o + P.slabs.size() * sizeof(Slab), 256);
    P.off_slabsums = o; o = align_up(o + P.slabs.size() * kNumSums * 8, 256);
    P.off_candcount = o; o = align_up(o + P.n_tasks * 4, 256);
    P.off_scan3 = o;    o = align_up(o + (uint64_t)n * 4, 256);
    P.off_finpart = o;  o = align_up(o + P.mats.size() * kFinSlices * 2 * 8, 256);
    P.off_cand = o;     o = align_up(o + n_cand * 4, 256);
    P.total = o;
    return BAOC_OK;
}

template <int GT, bool FIRST, int G, int NW>
static void launch_step_as(uint32_t grid, uint32_t lds, hipStream_t st, const typename GradIO<GT>::elem* g, float* m, float* v,
                           typename GradIO<GT>::elem* gp, const Chunk* ch, float* part, StepConsts k, uint32_t slices, uint32_t slice_groups)
{
    hipLaunchKernelGGL((k_step<GT, FIRST, G, NW>), dim3(grid), dim3(64 * NW), lds, st, g, m, v, gp, ch, part, k, slices, slice_groups);
}

// The instantiation for (first step?, groups per wavefront, wavefronts per workgroup); the values were validated at begin.
template <int GT, typename... Args>
static void launch_step(bool first, uint32_t gpw, uint32_t nw, Args... a)
{
#define BAOC_STEP_CASE(GG, NN) \
    if (gpw == GG && nw == NN) { if (first) launch_step_as<GT, true, GG, NN>(a...); else launch_step_as<GT, false, GG, NN>(a...); return; }
    BAOC_STEP_CASE(1, 1) BAOC_STEP_CASE(2, 1) BAOC_STEP_CASE(1, 2) BAOC_STEP_CASE(2, 2) BAOC_STEP_CASE(1, 4) BAOC_STEP_CASE(2, 4)
#undef BAOC_STEP_CASE
}

extern "C" void baoc_profile_params_default(baoc_profile_params* p)
{
    if (!p) return;
    p->beta_m = 0.9f; p->beta_v = 0.999f; p->beta_rho = 0.9; p->eps = 1e-12; p->eps_update = 1e-8f;
    p->quant_block = kQB; p->grad_dtype = BAOC_GRAD_F32;
    p->chunk_groups = 0; p->chunk_slices = 0; p->groups_per_wave = 0; p->waves_per_workgroup = 0; p->resident_workgroups = 0;
}

extern "C" int baoc_profile_workspace_bytes(const baoc_block* blocks, uint32_t n_blocks,
                                            const baoc_profile_params* params, uint64_t* out_bytes)
{
    if (!out_bytes) return BAOC_ERR_INVALID;
    Plan P;
    int rc = make_plan(blocks, n_blocks, params, &P, nullptr);
    if (rc) return rc;
    *out_bytes = P.total;
    return BAOC_OK;
}

// Shared by the two begin calls: plan, carve `d_workspace`, clear what must start at zero, upload the tables.
static int begin_on(const baoc_block* blocks, uint32_t n_blocks, const baoc_profile_params* params,
                    void* d_workspace, uint64_t workspace_bytes, baoc_profiler** out)
{
    baoc_profiler* h = new (std::nothrow) baoc_profiler();
    if (!h) return BAOC_ERR_INVALID;
    int rc = make_plan(blocks, n_blocks, params, &h->plan, &h->max_end);
    if (rc) { delete h; return rc; }
    if (workspace_bytes < h->plan.total || (reinterpret_cast<uintptr_t>(d_workspace) & 255)) { delete h; return BAOC_ERR_WORKSPACE; }
    h->params = *params;
    h->blocks.assign(blocks, blocks + n_blocks);
    h->ws = static_cast<char*>(d_workspace);
    const Plan& P = h->plan;
    // The first step treats m, v and g_prev as zero without reading them and writes all of them
    // (padding included), so only the small tail of the workspace is cleared here.
    hipError_t e = hipMemset(h->ws + P.off_rec, 0, P.off_mats - P.off_rec);
    if (e == hipSuccess) e = hipMemcpy(h->ws + P.off_rows, P.rows.data(), P.rows.size() * sizeof(BlockRow), hipMemcpyHostToDevice);
    if (e == hipSuccess && !P.slabs.empty())
        e = hipMemcpy(h->ws + P.off_slabs, P.slabs.data(), P.slabs.size() * sizeof(Slab), hipMemcpyHostToDevice);
    if (e == hipSuccess && !P.mats.empty())
        e = hipMemcpy(h->ws + P.off_mats, P.mats.data(), P.mats.size() * sizeof(MatRow), hipMemcpyHostToDevice);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(k_build_chunks, dim3((uint32_t)((P.n_chunks + 255) / 256)), dim3(256), 0, nullptr,
                           reinterpret_cast<const BlockRow*>(h->ws + P.off_rows), n_blocks,
                           reinterpret_cast<Chunk*>(h->ws + P.off_chunks), (uint32_t)P.n_chunks,
                           reinterpret_cast<uint32_t*>(h->ws + P.off_veclist));
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) { (void)hipGetLastError(); delete h; return BAOC_ERR_HIP; }
    h->h_rec.resize((size_t)n_blocks * kRecDoubles);
    h->h_ostat.resize((size_t)n_blocks * 4);
    *out = h;
    return BAOC_OK;
}

extern "C" int baoc_profile_begin(const baoc_block* blocks, uint32_t n_blocks,
                                  const baoc_profile_params* params,
                                  void* d_workspace, uint64_t workspace_bytes, baoc_profiler** out)
{
    if (!out || !d_workspace) return BAOC_ERR_INVALID;
    return begin_on(blocks, n_blocks, params, d_workspace, workspace_bytes, out);
}

extern "C" int baoc_profile_begin_static(const baoc_block* blocks, uint32_t n_blocks,
                                         const baoc_profile_params* params, baoc_profiler** out)
{
    if (!out) return BAOC_ERR_INVALID;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return BAOC_ERR_HIP; }
    if (dev < 0 || dev >= kMaxDevices) return BAOC_ERR_UNSUPPORTED;
    if (g_scratch_busy[dev]) return BAOC_ERR_STATE;            // one handle at a time shares the array
    if (!g_scratch_ptr[dev]) {                                 // first use on this device: where its copy of the array lives
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return BAOC_ERR_HIP; }
        g_scratch_ptr[dev] = ptr;
    }
    const int rc = begin_on(blocks, n_blocks, params, g_scratch_ptr[dev], BAOC_STATIC_WORKSPACE_BYTES, out);
    if (rc == BAOC_OK) { (*out)->static_device = dev; g_scratch_busy[dev] = true; }
    return rc;
}

extern "C" int baoc_profile_step(baoc_profiler* h, const void* d_grad_flat, uint64_t grad_numel, void* hip_stream)
{
    if (!h || !d_grad_flat) return BAOC_ERR_INVALID;
    if (h->sticky) return h->sticky;
    if (grad_numel < h->max_end) return BAOC_ERR_INVALID;
    const Plan& P = h->plan;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const baoc_profile_params& q = h->params;
    StepConsts k{q.beta_m, q.beta_v, 1.0f - q.beta_m, 1.0f - q.beta_v, q.eps_update};
    float* m = reinterpret_cast<float*>(h->ws + P.off_m);
    float* v = reinterpret_cast<float*>(h->ws + P.off_v);
    const Chunk* ch = reinterpret_cast<const Chunk*>(h->ws + P.off_chunks);
    float* part = reinterpret_cast<float*>(h->ws + P.off_partials);
    const bool first = h->steps == 0;
    // The first launch is bound by its arithmetic and runs at full residency.  Later launches are bound
    // by DRAM and run with fewer resident workgroups: each is given so much unused LDS that only about
    // `resident` of them fit a compute unit (allocations are counted in multiples of 2 KB here).
    const uint32_t static_lds = P.nw * 4 * kNumSums * 4;
    uint32_t lds = 0;
    if (!first && P.resident * P.nw < 32) lds = kLdsBytesPerCU / P.resident / 2048 * 2048 - static_lds;
    const uint32_t grid = (uint32_t)P.n_prows;
    if (q.grad_dtype == BAOC_GRAD_F32)
        launch_step<BAOC_GRAD_F32>(first, P.gpw, P.nw, grid, lds, st, static_cast<const float*>(d_grad_flat), m, v,
                                   reinterpret_cast<float*>(h->ws + P.off_gp), ch, part, k, P.slices, P.slice_groups);
    else
        launch_step<BAOC_GRAD_BF16>(first, P.gpw, P.nw, grid, lds, st, static_cast<const uint16_t*>(d_grad_flat), m, v,
                                    reinterpret_cast<uint16_t*>(h->ws + P.off_gp), ch, part, k, P.slices, P.slice_groups);
    h->steps += 1;
    double* slab_sums = reinterpret_cast<double*>(h->ws + P.off_slabsums);
    if (!P.slabs.empty())
        hipLaunchKernelGGL(k_slab_reduce, dim3((uint32_t)P.slabs.size()), dim3(256), 0, st,
                           part, reinterpret_cast<const Slab*>(h->ws + P.off_slabs), slab_sums);
    hipLaunchKernelGGL(k_block_reduce, dim3((uint32_t)P.rows.size()), dim3(256), 0, st,
                       part, slab_sums, reinterpret_cast<const BlockRow*>(h->ws + P.off_rows),
                       reinterpret_cast<double*>(h->ws + P.off_rec), q.beta_rho, q.eps);
    if (hipGetLastError() != hipSuccess) { h->sticky = BAOC_ERR_HIP; return BAOC_ERR_HIP; }
    return BAOC_OK;
}

extern "C" int baoc_profile_finalize(baoc_profiler* h, const baoc_config* configs, uint32_t n_configs,
                                     const baoc_risk_params* risk_params,
                                     baoc_block_stats* out_stats, double* out_risk, void* hip_stream)
{
    if (!h) return BAOC_ERR_INVALID;
    if (h->sticky) return h->sticky;
    if (h->steps == 0) return BAOC_ERR_STATE;
    if (out_risk && (!configs || n_configs == 0)) return BAOC_ERR_INVALID;
    for (uint32_t c = 0; out_risk && c < n_configs; ++c) {
        const baoc_config& k = configs[c];
        if ((k.bits != 32 && k.bits != 16 && k.bits != 8) || k.y_a > 1 || k.y_m > 1 || k.y_d > 1 || k.y_f > 1) return BAOC_ERR_INVALID;
    }
    baoc_risk_params rp;
    if (risk_params) rp = *risk_params; else baoc_risk_params_default(&rp);
    if (!(rp.A_high != rp.A_low) || !(rp.rho_high != rp.rho_low) || !(rp.eta_high != rp.eta_low)) return BAOC_ERR_INVALID;

    const bool want_F = !rp.F_raw && rp.compute_F && !h->plan.mats.empty();
    const bool want_C = !rp.C_raw && rp.d_theta_flat;
    if (want_C && (rp.theta_numel < h->max_end || (rp.theta_dtype != BAOC_GRAD_F32 && rp.theta_dtype != BAOC_GRAD_BF16)))
        return BAOC_ERR_INVALID;

    const Plan& P = h->plan;
    const uint32_t N = (uint32_t)P.rows.size(), nch = (uint32_t)P.n_chunks;
    const uint32_t n_vec = (uint32_t)P.n_vec_chunks, n_mats = (uint32_t)P.mats.size(), n_quads = (uint32_t)P.n_quads;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const float* v = reinterpret_cast<const float*>(h->ws + P.off_v);
    const Chunk* ch = reinterpret_cast<const Chunk*>(h->ws + P.off_chunks);
    const BlockRow* rows = reinterpret_cast<const BlockRow*>(h->ws + P.off_rows);
    const uint32_t* vec_list = reinterpret_cast<const uint32_t*>(h->ws + P.off_veclist);
    const MatRow* mats = reinterpret_cast<const MatRow*>(h->ws + P.off_mats);
    uint32_t* hist = reinterpret_cast<uint32_t*>(h->ws + P.off_hist);
    uint32_t* selp = reinterpret_cast<uint32_t*>(h->ws + P.off_selp);
    uint32_t* selr = reinterpret_cast<uint32_t*>(h->ws + P.off_selr);
    float* ostat = reinterpret_cast<float*>(h->ws + P.off_ostat);
    float* rvec = reinterpret_cast<float*>(h->ws + P.off_rvec);
    float* cvec = reinterpret_cast<float*>(h->ws + P.off_cvec);
    float* rowpart = reinterpret_cast<float*>(h->ws + P.off_rowpart);
    float* colpart = reinterpret_cast<float*>(h->ws + P.off_colpart);
    float* residpart = reinterpret_cast<float*>(h->ws + P.off_residpart);
    float* psumpart = reinterpret_cast<float*>(h->ws + P.off_psumpart);
    double* mu = reinterpret_cast<double*>(h->ws + P.off_mu);
    float* part = reinterpret_cast<float*>(h->ws + P.off_partials);
    double* rec = reinterpret_cast<double*>(h->ws + P.off_rec);
    const float epsf = (float)h->params.eps;
    const bool th32 = rp.theta_dtype == BAOC_GRAD_F32;
    const float* th_f = static_cast<const float*>(rp.d_theta_flat);
    const uint16_t* th_h = static_cast<const uint16_t*>(rp.d_theta_flat);
    const uint64_t hist_words = (uint64_t)N * 4 * kBins;
    const uint32_t fill_grid = (uint32_t)std::min<uint64_t>((hist_words + 255) / 256, 4096);

    uint32_t* cand = reinterpret_cast<uint32_t*>(h->ws + P.off_cand);
    uint32_t* cand_count = reinterpret_cast<uint32_t*>(h->ws + P.off_candcount);
    uint32_t* scan3 = reinterpret_cast<uint32_t*>(h->ws + P.off_scan3);
    const uint32_t* no_list = nullptr;
    const uint32_t* no_flags = nullptr;

    // pass 1 over v: first digit everywhere; row/column sums and the sum of p on the way
    hipLaunchKernelGGL(k_fill_u32, dim3(fill_grid), dim3(256), 0, st, hist, hist_words, 0u);
    if (n_quads)
        hipLaunchKernelGGL(k_tile_pass1, dim3(n_quads), dim3(256), 0, st, v, mats, n_mats, rowpart, colpart, psumpart, hist, epsf, want_C);
    if (n_vec) {
        hipLaunchKernelGGL(k_hist<1>, dim3(std::min(n_vec, kHistGrid)), dim3(256), 0, st, v, ch, vec_list, n_vec, selp, hist, rows, no_flags);
        if (want_C) {
            if (th32) hipLaunchKernelGGL((k_distortion<BAOC_GRAD_F32, 1>), dim3(n_vec), dim3(256), 0, st, v, th_f, ch, vec_list, rows, rec, part, epsf);
            else hipLaunchKernelGGL((k_distortion<BAOC_GRAD_BF16, 1>), dim3(n_vec), dim3(256), 0, st, v, th_h, ch, vec_list, rows, rec, part, epsf);
            hipLaunchKernelGGL(k_reduce_partials, dim3(N), dim3(256), 0, st, part, rows, rec, 1u, (uint32_t)R_PSUM);
        }
    }
    if (n_quads) {
        double* finpart = reinterpret_cast<double*>(h->ws + P.off_finpart);
        hipLaunchKernelGGL(k_tile_finish1, dim3(n_mats, kFinSlices), dim3(256), 0, st, mats, rowpart, colpart, psumpart, rvec, cvec, finpart);
        hipLaunchKernelGGL(k_tile_finish1_sum, dim3(n_mats), dim3(64), 0, st, mats, finpart, mu, rec);
    }
    hipLaunchKernelGGL(k_pick<1>, dim3(N * 4), dim3(64), 0, st, hist, rows, selp, selr, ostat, scan3);

    // pass 2 over v (and theta): second digit; rank-1 residual and distortion on the way; matrix blocks
    // also set aside the keys that carry a selected first digit
    hipLaunchKernelGGL(k_fill_u32, dim3(fill_grid), dim3(256), 0, st, hist, hist_words, 0u);
    if (n_quads) {
        if (th32) hipLaunchKernelGGL(k_tile_pass2<BAOC_GRAD_F32>, dim3(n_quads), dim3(256), 0, st, v, th_f, mats, n_mats, rvec, cvec, mu, rec, selp, residpart, hist, cand, cand_count, scan3, epsf, want_F, want_C);
        else hipLaunchKernelGGL(k_tile_pass2<BAOC_GRAD_BF16>, dim3(n_quads), dim3(256), 0, st, v, th_h, mats, n_mats, rvec, cvec, mu, rec, selp, residpart, hist, cand, cand_count, scan3, epsf, want_F, want_C);
        hipLaunchKernelGGL(k_tile_finish2, dim3(n_mats), dim3(256), 0, st, mats, residpart, rec);
    }
    if (n_vec) {
        hipLaunchKernelGGL(k_hist<2>, dim3(std::min(n_vec, kHistGrid)), dim3(256), 0, st, v, ch, vec_list, n_vec, selp, hist, rows, no_flags);
        if (want_C) {
            if (th32) hipLaunchKernelGGL((k_distortion<BAOC_GRAD_F32, 2>), dim3(n_vec), dim3(256), 0, st, v, th_f, ch, vec_list, rows, rec, part, epsf);
            else hipLaunchKernelGGL((k_distortion<BAOC_GRAD_BF16, 2>), dim3(n_vec), dim3(256), 0, st, v, th_h, ch, vec_list, rows, rec, part, epsf);
            hipLaunchKernelGGL(k_reduce_partials, dim3(N), dim3(256), 0, st, part, rows, rec, 2u, (uint32_t)R_CNUM);
        }
    }
    hipLaunchKernelGGL(k_pick<2>, dim3(N * 4), dim3(64), 0, st, hist, rows, selp, selr, ostat, scan3);

    // last digit: on the candidate lists of the matrix blocks; by a third scan of v for the blocks walked
    // chunk-wise and for matrix blocks whose lists overflowed (scan3 flags, skipped a block at a time otherwise)
    hipLaunchKernelGGL(k_fill_u32, dim3(fill_grid), dim3(256), 0, st, hist, hist_words, 0u);
    if (n_quads)
        hipLaunchKernelGGL(k_cand_hist3, dim3(n_quads), dim3(256), 0, st, mats, n_mats, cand, cand_count, selp, scan3, hist);
    hipLaunchKernelGGL(k_hist<3>, dim3(std::min(nch, kHistGrid)), dim3(256), 0, st, v, ch, no_list, nch, selp, hist, rows, static_cast<const uint32_t*>(scan3));
    hipLaunchKernelGGL(k_pick<3>, dim3(N * 4), dim3(64), 0, st, hist, rows, selp, selr, ostat, scan3);

    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(h->h_rec.data(), h->ws + P.off_rec, h->h_rec.size() * 8, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipMemcpyAsync(h->h_ostat.data(), ostat, h->h_ostat.size() * 4, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { (void)hipGetLastError(); h->sticky = BAOC_ERR_HIP; return BAOC_ERR_HIP; }

    std::vector<baoc_block_stats> stats(N);
    for (uint32_t i = 0; i < N; ++i) {
        RawBlock r;
        const double* rec = &h->h_rec[(size_t)i * kRecDoubles];
        r.numel = P.rows[i].numel;
        for (int s = 0; s < (int)kNumSums; ++s) r.sums[s] = rec[s];
        r.rho_bar = rec[R_RHO]; r.cos_last = rec[R_COS];
        r.n_cos = (uint32_t)rec[R_NCOS]; r.steps = (uint32_t)rec[R_STEPS];
        for (int t = 0; t < 4; ++t) r.order_stat[t] = h->h_ostat[(size_t)i * 4 + t];
        const double p10 = 0.1 * (double)(r.numel - 1), p90 = 0.9 * (double)(r.numel - 1);
        r.frac10 = p10 - std::floor(p10); r.frac90 = p90 - std::floor(p90);
        const double eps = h->params.eps;
        double C_raw = rp.C_raw ? rp.C_raw[i] : 0.0, F_raw = rp.F_raw ? rp.F_raw[i] : 0.0;
        if (want_C) C_raw = std::sqrt(rec[R_CNUM]) / (std::sqrt(rec[R_CDEN]) + eps);                  // Eq. 6
        if (want_F && P.rows[i].vec_first == kNoVec) F_raw = std::sqrt(rec[R_FRES]) / (std::sqrt(rec[R_FS2]) + eps);   // Eq. 7
        block_metrics(r, eps, rp, C_raw, F_raw, &stats[i]);
    }
    if (out_stats) std::memcpy(out_stats, stats.data(), sizeof(baoc_block_stats) * N);
    if (out_risk)
        for (uint32_t i = 0; i < N; ++i)
            for (uint32_t c = 0; c < n_configs; ++c)
                out_risk[(size_t)i * n_configs + c] =
                    config_phi(stats[i], configs[c], rp.pref_mask && rp.pref_mask[c], rp);
    return BAOC_OK;
}

extern "C" int baoc_profile_state(const baoc_profiler* h, uint32_t block,
                                  const float** d_m, const float** d_v, const void** d_g_prev)
{
    if (!h || block >= h->plan.rows.size()) return BAOC_ERR_INVALID;
    const Plan& P = h->plan;
    const uint64_t s = P.rows[block].state_start;
    const uint64_t gsz = h->params.grad_dtype == BAOC_GRAD_F32 ? 4 : 2;
    if (d_m) *d_m = reinterpret_cast<const float*>(h->ws + P.off_m) + s;
    if (d_v) *d_v = reinterpret_cast<const float*>(h->ws + P.off_v) + s;
    if (d_g_prev) *d_g_prev = h->ws + P.off_gp + s * gsz;
    return BAOC_OK;
}

extern "C" int baoc_profile_end(baoc_profiler* h)
{
    if (!h) return BAOC_ERR_INVALID;
    if (h->static_device >= 0) g_scratch_busy[h->static_device] = false;
    delete h;
    return BAOC_OK;
}

extern "C" const char* baoc_status_string(int s)
{
    switch (s) {
    case BAOC_OK: return "ok";
    case BAOC_ERR_INVALID: return "invalid argument";
    case BAOC_ERR_WORKSPACE: return "workspace too small or misaligned";
    case BAOC_ERR_UNSUPPORTED: return "unsupported parameter";
    case BAOC_ERR_HIP: return "HIP runtime error";
    case BAOC_ERR_INFEASIBLE: return "no assignment satisfies the budgets";
    case BAOC_ERR_LIMIT: return "solver node limit reached";
    case BAOC_ERR_STATE: return "call out of order";
    default: return "unknown status";
    }
}
