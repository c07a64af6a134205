// Sparse coordinate sampling front end (Sec. 3.1): a fixed index set Omega_i with
// |Omega_i| = ceil(s d_i) per block, drawn once on the device, and a gather kernel that
// packs g[Omega] of every block into a compact buffer the profiler then runs on
// unchanged (its blocks are the compact ones).
//
// Draw: stratified uniform -- stratum j of block i is [floor(j d/k), floor((j+1) d/k)),
// one coordinate of each by a 64-bit mix of (seed, block, j); indices ascend.
// A matrix block (rows x cols, both >= 2) keeps a matrix form, which Eq. 7 needs: Omega is a product of
// r rows and c columns, r = round(rows sqrt(s)), c the least count with r c >= ceil(s d), each axis drawn
// by the same stratified rule; the compact block is the r x c sub-matrix, row-major.  A sample too thin for
// that (r < 2 or c < 2) falls back to the flat draw and carries no shape.
#include <hip/hip_runtime.h>

#include <cmath>
#include <new>
#include <vector>

#include "baoc.h"

namespace {

struct alignas(8) SampleRow {
    uint64_t src_offset;      // block start in the flat gradient buffer
    uint64_t dst_offset;      // block start in the compact buffer
    uint64_t numel;           // d_i
    uint64_t count;           // k_i = |Omega_i|
    uint64_t idx_start;       // first entry of the block in the index table
    uint32_t first_tile;
    uint32_t rows, cols;      // matrix shape of the block, or 0, 0
    uint32_t sub_rows, sub_cols;   // shape of the sampled sub-matrix (product form), or 0, 0 for the flat draw
    uint32_t pad_;
};

constexpr uint32_t kTile = 1024;    // samples per workgroup

__host__ __device__ inline uint64_t mix64(uint64_t x)
{
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

__device__ inline uint32_t find_row(const SampleRow* __restrict__ rows, uint32_t n, uint32_t tile)
{
    uint32_t lo = 0, hi = n - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (rows[mid].first_tile <= tile) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// idx[idx_start + j] = src_offset + lo_j + mix(...) % (hi_j - lo_j): absolute positions in the flat buffer
__global__ __launch_bounds__(256) void k_draw(const SampleRow* __restrict__ rows, uint32_t n_rows, uint64_t seed,
                                              uint64_t* __restrict__ idx)
{
    const uint32_t b = find_row(rows, n_rows, blockIdx.x);
    const SampleRow r = rows[b];
    const uint64_t key = mix64(mix64(seed) + b);
    const uint64_t j0 = (uint64_t)(blockIdx.x - r.first_tile) * kTile;
    if (r.sub_rows) {                                      // product form: sample j is (row a, column c) of the sub-matrix
        const uint64_t key_r = mix64(key + 0x52), key_c = mix64(key + 0x43);
        for (uint64_t j = j0 + threadIdx.x; j < min(r.count, j0 + kTile); j += 256) {
            const uint64_t a = j / r.sub_cols, c = j - a * r.sub_cols;
            const uint64_t rlo = a * r.rows / r.sub_rows, rhi = (a + 1) * r.rows / r.sub_rows;
            const uint64_t clo = c * r.cols / r.sub_cols, chi = (c + 1) * r.cols / r.sub_cols;
            const uint64_t row = rlo + mix64(key_r + (a + 1) * 0x9E3779B97F4A7C15ull) % (rhi - rlo);
            const uint64_t col = clo + mix64(key_c + (c + 1) * 0x9E3779B97F4A7C15ull) % (chi - clo);
            idx[r.idx_start + j] = r.src_offset + row * r.cols + col;
        }
        return;
    }
    for (uint64_t j = j0 + threadIdx.x; j < min(r.count, j0 + kTile); j += 256) {
        const uint64_t lo = (uint64_t)(((unsigned __int128)j * r.numel) / r.count);
        const uint64_t hi = (uint64_t)(((unsigned __int128)(j + 1) * r.numel) / r.count);
        const uint64_t h = mix64(key + (j + 1) * 0x9E3779B97F4A7C15ull);
        idx[r.idx_start + j] = r.src_offset + lo + h % (hi - lo);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_gather(const SampleRow* __restrict__ rows, uint32_t n_rows,
                                                const uint64_t* __restrict__ idx, const T* __restrict__ src,
                                                T* __restrict__ dst)
{
    const uint32_t b = find_row(rows, n_rows, blockIdx.x);
    const SampleRow r = rows[b];
    const uint64_t j0 = (uint64_t)(blockIdx.x - r.first_tile) * kTile;
    const uint64_t j1 = min(r.count, j0 + kTile);
#pragma unroll 4
    for (uint64_t j = j0 + threadIdx.x; j < j1; j += 256) dst[r.dst_offset + j] = src[idx[r.idx_start + j]];
}

int make_rows(const baoc_block* blocks, uint32_t n, double ratio, std::vector<SampleRow>* rows,
              uint64_t* compact_numel, uint64_t* total_samples, uint64_t* n_tiles, uint64_t* max_end)
{
    if (!blocks || n == 0 || !(ratio > 0.0) || !(ratio <= 1.0)) return BAOC_ERR_INVALID;
    rows->resize(n);
    uint64_t dst = 0, idx = 0, tiles = 0, end = 0;
    for (uint32_t i = 0; i < n; ++i) {
        const baoc_block& b = blocks[i];
        if (b.numel == 0 || b.offset + b.numel < b.offset) return BAOC_ERR_INVALID;
        if ((b.rows || b.cols) && (uint64_t)b.rows * b.cols != b.numel) return BAOC_ERR_INVALID;
        double k = std::ceil(ratio * (double)b.numel);                // |Omega_i| = ceil(s d_i), in [1, d_i]
        if (!(k >= 1.0)) k = 1.0;
        if (k > (double)b.numel) k = (double)b.numel;
        SampleRow& r = (*rows)[i];
        dst = (dst + 63) / 64 * 64;                                    // compact blocks start on 64 elements
        r.src_offset = b.offset; r.dst_offset = dst; r.numel = b.numel; r.count = (uint64_t)k;
        r.rows = b.rows; r.cols = b.cols; r.sub_rows = r.sub_cols = 0;
        if (b.rows >= 2 && b.cols >= 2) {                              // matrix form of the sample (Eq. 7)
            double rr = std::floor((double)b.rows * std::sqrt(ratio) + 0.5);
            if (!(rr >= 1.0)) rr = 1.0;
            if (rr > (double)b.rows) rr = (double)b.rows;
            const uint64_t sr = (uint64_t)rr, sc = std::min<uint64_t>(b.cols, (r.count + sr - 1) / sr);
            if (sr >= 2 && sc >= 2) { r.sub_rows = (uint32_t)sr; r.sub_cols = (uint32_t)sc; r.count = sr * sc; }
        }
        r.idx_start = idx; r.first_tile = (uint32_t)tiles; r.pad_ = 0;
        dst += r.count; idx += r.count; tiles += (r.count + kTile - 1) / kTile;
        if (tiles > 0x7fffffffull) return BAOC_ERR_UNSUPPORTED;
        end = std::max(end, b.offset + b.numel);
    }
    *compact_numel = (dst + 63) / 64 * 64; *total_samples = idx; *n_tiles = tiles; *max_end = end;
    return BAOC_OK;
}

}  // namespace

struct baoc_sampler {
    std::vector<SampleRow> rows;
    uint64_t compact_numel = 0, total = 0, n_tiles = 0, max_end = 0;
    char* ws = nullptr;
    uint64_t off_idx = 0;
};

static uint64_t rows_bytes(uint32_t n) { return ((uint64_t)n * sizeof(SampleRow) + 255) / 256 * 256; }

extern "C" int baoc_sample_layout(const baoc_block* blocks, uint32_t n_blocks, double ratio,
                                  baoc_block* out_compact, uint64_t* out_compact_numel, uint64_t* out_workspace_bytes)
{
    std::vector<SampleRow> rows;
    uint64_t cn, tot, tiles, end;
    const int rc = make_rows(blocks, n_blocks, ratio, &rows, &cn, &tot, &tiles, &end);
    if (rc) return rc;
    if (out_compact)
        for (uint32_t i = 0; i < n_blocks; ++i) out_compact[i] = baoc_block{rows[i].dst_offset, rows[i].count, rows[i].sub_rows, rows[i].sub_cols};
    if (out_compact_numel) *out_compact_numel = cn;
    if (out_workspace_bytes) *out_workspace_bytes = rows_bytes(n_blocks) + tot * 8;
    return BAOC_OK;
}

extern "C" int baoc_sample_begin(const baoc_block* blocks, uint32_t n_blocks, double ratio, uint64_t seed,
                                 void* d_workspace, uint64_t workspace_bytes, baoc_sampler** out)
{
    if (!out || !d_workspace) return BAOC_ERR_INVALID;
    baoc_sampler* h = new (std::nothrow) baoc_sampler();
    if (!h) return BAOC_ERR_INVALID;
    int rc = make_rows(blocks, n_blocks, ratio, &h->rows, &h->compact_numel, &h->total, &h->n_tiles, &h->max_end);
    if (rc) { delete h; return rc; }
    h->off_idx = rows_bytes(n_blocks);
    if (workspace_bytes < h->off_idx + h->total * 8 || (reinterpret_cast<uintptr_t>(d_workspace) & 255)) { delete h; return BAOC_ERR_WORKSPACE; }
    h->ws = static_cast<char*>(d_workspace);
    hipError_t e = hipMemcpy(h->ws, h->rows.data(), h->rows.size() * sizeof(SampleRow), hipMemcpyHostToDevice);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(k_draw, dim3((uint32_t)h->n_tiles), dim3(256), 0, nullptr,
                           reinterpret_cast<const SampleRow*>(h->ws), n_blocks, seed,
                           reinterpret_cast<uint64_t*>(h->ws + h->off_idx));
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) { (void)hipGetLastError(); delete h; return BAOC_ERR_HIP; }
    *out = h;
    return BAOC_OK;
}

extern "C" int baoc_sample_gather(baoc_sampler* h, const void* d_grad_flat, uint64_t grad_numel, uint32_t grad_dtype,
                                  void* d_compact, uint64_t compact_numel, void* hip_stream)
{
    if (!h || !d_grad_flat || !d_compact) return BAOC_ERR_INVALID;
    if (grad_numel < h->max_end || compact_numel < h->compact_numel) return BAOC_ERR_INVALID;
    if (grad_dtype != BAOC_GRAD_F32 && grad_dtype != BAOC_GRAD_BF16) return BAOC_ERR_INVALID;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const SampleRow* rows = reinterpret_cast<const SampleRow*>(h->ws);
    const uint64_t* idx = reinterpret_cast<const uint64_t*>(h->ws + h->off_idx);
    const uint32_t n = (uint32_t)h->rows.size();
    if (grad_dtype == BAOC_GRAD_F32)
        hipLaunchKernelGGL(k_gather<float>, dim3((uint32_t)h->n_tiles), dim3(256), 0, st, rows, n, idx,
                           static_cast<const float*>(d_grad_flat), static_cast<float*>(d_compact));
    else
        hipLaunchKernelGGL(k_gather<uint16_t>, dim3((uint32_t)h->n_tiles), dim3(256), 0, st, rows, n, idx,
                           static_cast<const uint16_t*>(d_grad_flat), static_cast<uint16_t*>(d_compact));
    return hipGetLastError() == hipSuccess ? BAOC_OK : BAOC_ERR_HIP;
}

extern "C" int baoc_sample_indices(const baoc_sampler* h, uint32_t block, const uint64_t** d_indices, uint64_t* count)
{
    if (!h || block >= h->rows.size()) return BAOC_ERR_INVALID;
    if (d_indices) *d_indices = reinterpret_cast<const uint64_t*>(h->ws + h->off_idx) + h->rows[block].idx_start;
    if (count) *count = h->rows[block].count;
    return BAOC_OK;
}

extern "C" int baoc_sample_end(baoc_sampler* h)
{
    if (!h) return BAOC_ERR_INVALID;
    delete h;
    return BAOC_OK;
}
