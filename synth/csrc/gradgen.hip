// Device twin of synth/gradgen.py: counter-based synthetic gradient streams written
// straight into a flat fp32 or bf16 buffer.  Input recipe only -- nothing of the
// profiler's arithmetic lives here, and libbaoc does not link against this file.
//
//   g[j] = kappa_j * (delta * n_j / sqrt(d) + sigma * xi_j),  kappa_j = exp(s * zeta_j)
// zeta, n: fixed normals of stream 0; xi: unit-variance noise of the step (Gaussian,
// or Student-t(3)/sqrt(3)).  Normals are Box-Muller transforms of a 64-bit mix of
// (seed, block, stream, step, j).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__host__ __device__ inline uint64_t mix64(uint64_t x)
{
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

inline uint64_t stream_key(uint64_t seed, uint32_t block, uint32_t stream, uint32_t step)
{
    uint64_t k = mix64(seed) + block;
    k = mix64(k) + (((uint64_t)stream << 32) | step);
    return mix64(k);
}

__device__ inline void normal_pair(uint64_t key, uint64_t j, float& z0, float& z1)
{
    const uint64_t h = mix64(key + (j + 1) * 0x9E3779B97F4A7C15ull);
    const float u1 = ((float)(uint32_t)(h >> 40) + 0.5f) * 5.9604644775390625e-8f;
    const float u2 = ((float)(uint32_t)((h >> 16) & 0xFFFFFFu) + 0.5f) * 5.9604644775390625e-8f;
    const float r = sqrtf(-2.0f * logf(u1));
    float s, c;
    sincosf(6.283185307179586f * u2, &s, &c);
    z0 = r * c; z1 = r * s;
}

__device__ inline uint16_t to_bf16(float x)
{
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

template <typename T> __device__ inline void put(T* p, float x);
template <> __device__ inline void put<float>(float* p, float x) { *p = x; }
template <> __device__ inline void put<uint16_t>(uint16_t* p, float x) { *p = to_bf16(x); }

template <typename T>
__global__ __launch_bounds__(256) void k_fill(T* out, uint64_t numel, uint64_t key0, uint64_t key1, uint64_t key2,
                                              float delta_over_sqrt_d, float sigma, float s, uint32_t noise)
{
    for (uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x; j < numel; j += (uint64_t)gridDim.x * 256) {
        float zeta, n, z0, z1;
        normal_pair(key0, j, zeta, n);
        normal_pair(key1, j, z0, z1);
        float xi = z0;
        if (noise == 1) {
            float z2, z3;
            normal_pair(key2, j, z2, z3);
            xi = z0 / sqrtf(z1 * z1 + z2 * z2 + z3 * z3);
        }
        put<T>(out + j, expf(s * zeta) * (delta_over_sqrt_d * n + sigma * xi));
    }
}

}  // namespace

// dtype: 0 = fp32, 1 = bf16.  d_out points at the block's first element. Returns 0 or a hipError_t.
extern "C" int synth_fill_block(void* d_out, uint32_t dtype, uint64_t numel, uint64_t seed, uint32_t block,
                                uint32_t step, float delta, float sigma, float s, uint32_t noise, void* stream)
{
    if (numel == 0) return 0;
    const uint64_t k0 = stream_key(seed, block, 0, 0), k1 = stream_key(seed, block, 1, step), k2 = stream_key(seed, block, 2, step);
    const float dd = (float)((double)delta / sqrt((double)numel));
    uint64_t grid = (numel + 255) / 256;
    if (grid > 65536) grid = 65536;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == 0)
        hipLaunchKernelGGL(k_fill<float>, dim3((uint32_t)grid), dim3(256), 0, st, static_cast<float*>(d_out), numel, k0, k1, k2, dd, sigma, s, noise);
    else
        hipLaunchKernelGGL(k_fill<uint16_t>, dim3((uint32_t)grid), dim3(256), 0, st, static_cast<uint16_t*>(d_out), numel, k0, k1, k2, dd, sigma, s, noise);
    return (int)hipGetLastError();
}
