// Pure stream with the bf16 step kernel's bytes (harness code, not part of libbaoc): per coordinate 4 reads
// (m, v fp32; g_prev, g bf16) and 3 writes (m, v, g_prev), 22 bytes, and no arithmetic to speak of.  It shows what
// this HBM system delivers for that mix -- the practical ceiling next to which the benchmark reports the step kernel.
// Launch shape: single-wavefront workgroups that each move two groups of 256 coordinates, all loads issued before the
// first store, and so much unused LDS per workgroup that 4 of them are resident per compute unit (the fastest of the
// shapes tried: fewer, fatter requesters keep DRAM rows open).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

constexpr int kGroups = 2;                          // groups of 256 coordinates per wavefront
constexpr uint32_t kLdsBytes = 160 * 1024 / 4;      // per workgroup: 4 resident per compute unit

__global__ __launch_bounds__(64) void k_mix(float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ gp,
                                            const uint16_t* __restrict__ g, uint64_t n)
{
    const uint64_t base = (uint64_t)blockIdx.x * (256ull * kGroups) + threadIdx.x * 4;
    if (base + 256ull * (kGroups - 1) + 4 > n) return;
    f4 a[kGroups], b[kGroups]; u2 c[kGroups], d[kGroups];
#pragma unroll
    for (int i = 0; i < kGroups; ++i) {
        const uint64_t e = base + 256ull * i;
        a[i] = __builtin_nontemporal_load((const f4*)(m + e)); b[i] = __builtin_nontemporal_load((const f4*)(v + e));
        c[i] = __builtin_nontemporal_load((const u2*)(gp + e)); d[i] = __builtin_nontemporal_load((const u2*)(g + e));
    }
#pragma unroll
    for (int i = 0; i < kGroups; ++i) {
        const uint64_t e = base + 256ull * i;
        const f4 x = a[i] * 0.9f + b[i], y = b[i] * 0.999f + a[i];
        const u2 z = {c[i].x ^ d[i].x, c[i].y + d[i].y};
        __builtin_nontemporal_store(x, (f4*)(m + e)); __builtin_nontemporal_store(y, (f4*)(v + e)); __builtin_nontemporal_store(z, (u2*)(gp + e));
    }
}

}  // namespace

// One launch over n coordinates (n a multiple of 512, at most 2^31 workgroups); the four buffers hold n elements each.
// Returns 0, -1 (bad argument) or a hipError_t.
extern "C" int synth_mix_stream(uint64_t n, float* d_m, float* d_v, uint16_t* d_gp, const uint16_t* d_g, void* stream)
{
    const uint64_t per = 256ull * kGroups;
    if (n == 0 || n % per || n / per > 0x7fffffffull || !d_m || !d_v || !d_gp || !d_g) return -1;
    hipLaunchKernelGGL(k_mix, dim3((uint32_t)(n / per)), dim3(64), kLdsBytes, static_cast<hipStream_t>(stream), d_m, d_v, d_gp, d_g, n);
    return (int)hipGetLastError();
}
