// Memory-system probe (harness code, not part of libbaoc): kernels that move the step kernel's bytes --
// per coordinate 4 reads (m, v fp32; g_prev, g bf16) and 3 writes (m, v, g_prev), 22 bytes -- with no
// arithmetic to speak of, plus a read-only and a write-only stream.  Used to find what this HBM system
// delivers for that mix as a function of how many wavefronts request at the same time.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

// One workgroup of NW wavefronts covers NW * G groups of 256 coordinates; every load is issued before the first store.
template <int G>
__global__ void k_mix(float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ gp,
                      const uint16_t* __restrict__ g, uint64_t n)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint64_t base = ((uint64_t)blockIdx.x * nw + wave) * (256ull * G) + lane * 4;
    if (base + 256ull * (G - 1) + 4 > n) return;
    f4 a[G], b[G]; u2 c[G], d[G];
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const uint64_t e = base + 256ull * i;
        a[i] = __builtin_nontemporal_load((const f4*)(m + e)); b[i] = __builtin_nontemporal_load((const f4*)(v + e));
        c[i] = __builtin_nontemporal_load((const u2*)(gp + e)); d[i] = __builtin_nontemporal_load((const u2*)(g + e));
    }
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const uint64_t e = base + 256ull * i;
        const f4 x = a[i] * 0.9f + b[i], y = b[i] * 0.999f + a[i];
        const u2 z = {c[i].x ^ d[i].x, c[i].y + d[i].y};
        __builtin_nontemporal_store(x, (f4*)(m + e)); __builtin_nontemporal_store(y, (f4*)(v + e)); __builtin_nontemporal_store(z, (u2*)(gp + e));
    }
}

template <int G>
__global__ void k_read(const float* __restrict__ m, float* __restrict__ sink, uint64_t n)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint64_t base = ((uint64_t)blockIdx.x * nw + wave) * (256ull * G) + lane * 4;
    if (base + 256ull * (G - 1) + 4 > n) return;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < G; ++i) { const f4 a = __builtin_nontemporal_load((const f4*)(m + base + 256ull * i)); s += (a.x + a.y) + (a.z + a.w); }
    if (s == 1234.5678f) sink[threadIdx.x] = s;           // never true for the probe's data; keeps the loads alive
}

template <int G>
__global__ void k_write(float* __restrict__ m, uint64_t n)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint64_t base = ((uint64_t)blockIdx.x * nw + wave) * (256ull * G) + lane * 4;
    if (base + 256ull * (G - 1) + 4 > n) return;
    const f4 x = {1.f, 2.f, 3.f, (float)lane};
#pragma unroll
    for (int i = 0; i < G; ++i) __builtin_nontemporal_store(x, (f4*)(m + base + 256ull * i));
}

}  // namespace

// kind: 0 = mix (22 B/coordinate), 1 = read m (4 B), 2 = write m (4 B).  waves: 1, 2 or 4 per workgroup; groups: 1, 2 or 4
// per wavefront; lds_bytes of unused dynamic LDS limit the residency (0 = no limit, at most 64 KB).  n must be a multiple
// of 256 * waves * groups; the buffers hold n elements each (d_sink: 256 floats).  Returns 0, -1 (bad argument) or a hipError_t.
extern "C" int synth_mem_probe(int kind, int waves, int groups, uint32_t lds_bytes, uint64_t n,
                               float* d_m, float* d_v, uint16_t* d_gp, const uint16_t* d_g, float* d_sink, void* stream)
{
    if ((waves != 1 && waves != 2 && waves != 4) || (groups != 1 && groups != 2 && groups != 4) || lds_bytes > 65536) return -1;
    const uint64_t per = 256ull * waves * groups;
    if (n == 0 || n % per || n / per > 0x7fffffffull) return -1;
    const dim3 grid((uint32_t)(n / per)), block(64 * waves);
    hipStream_t st = static_cast<hipStream_t>(stream);
#define LAUNCH(G) \
    if (groups == G) { \
        if (kind == 0) hipLaunchKernelGGL(k_mix<G>, grid, block, lds_bytes, st, d_m, d_v, d_gp, d_g, n); \
        else if (kind == 1) hipLaunchKernelGGL(k_read<G>, grid, block, lds_bytes, st, d_m, d_sink, n); \
        else if (kind == 2) hipLaunchKernelGGL(k_write<G>, grid, block, lds_bytes, st, d_m, n); \
        else return -1; \
    }
    LAUNCH(1) LAUNCH(2) LAUNCH(4)
#undef LAUNCH
    return (int)hipGetLastError();
}
