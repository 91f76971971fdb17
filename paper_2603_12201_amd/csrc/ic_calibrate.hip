// Calibration kernels: what this chip sustains on the access and issue patterns the hot path is made of,
// measured through the same library the benchmark times (a plain stream read, a copy, a gather of KV rows
// in the attention kernels' access shape, and back-to-back matrix instructions).  Measurement aids, not
// part of the computation.
#include "ic_common.hpp"

namespace ic {

namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;

// Every thread reads 16-byte vectors, grid-strided, and folds them; one word per workgroup leaves the chip.
__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4 *src, int64_t n_vec, uint32_t *out)
{
    uint32_t acc = 0;
    const int64_t stride = (int64_t)gridDim.x * 256 * 4;
    for (int64_t i = (int64_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n_vec; i += stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = (i + 256 * u < n_vec) ? src[i + 256 * u] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;          // practically never: keeps the loads alive
}

__global__ __launch_bounds__(256) void calib_copy_kernel(const u32x4 *src, u32x4 *dst, int64_t n_vec)
{
    const int64_t stride = (int64_t)gridDim.x * 256 * 4;
    for (int64_t i = (int64_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n_vec; i += stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = (i + 256 * u < n_vec) ? src[i + 256 * u] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + 256 * u < n_vec) dst[i + 256 * u] = v[u];
    }
}

// Gather of whole rows of `row_bytes` (a multiple of 128): eight lanes fetch one 128-byte line, a wave 8 rows
// per round, every load of a row group in flight before any is consumed.  idx entries are clamped to the table.
template <int LINES>
__global__ __launch_bounds__(256) void calib_gather_kernel(const unsigned char *src, const int32_t *idx, int64_t n_rows,
                                                           int64_t table_rows, uint32_t *out)
{
    const int lane = threadIdx.x & 63, gr = lane >> 3, gp = lane & 7;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (int64_t)gridDim.x * 4;
    uint32_t acc = 0;
    for (int64_t r0 = wave * 8; r0 < n_rows; r0 += n_waves * 8) {
        const int64_t r = r0 + gr;
        int64_t row = r < n_rows ? idx[r] : 0;
        row = row < 0 ? 0 : (row >= table_rows ? table_rows - 1 : row);
        const u32x4 *p = (const u32x4 *)(src + row * (int64_t)(LINES * 128)) + gp;
        u32x4 v[LINES];
#pragma unroll
        for (int l = 0; l < LINES; ++l) v[l] = p[8 * l];
#pragma unroll
        for (int l = 0; l < LINES; ++l) acc ^= v[l][0] ^ v[l][1] ^ v[l][2] ^ v[l][3];
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;
}

// Back-to-back matrix instructions on four independent accumulators per wave (no memory traffic).
template <bool FP8>
__global__ __launch_bounds__(256) void calib_mfma_kernel(int iters, float *out)
{
    f32x16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    const int lane = threadIdx.x & 63;
    if constexpr (FP8) {
        i32x8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[i] = 0x38383838 + lane;                      // e4m3 bytes near 1.0
            b[i] = 0x30303030 + i;
        }
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[c], 0, 0, 0, 0, 0, 0);
    } else {
        bf16x8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[i] = (__bf16)(0.001f * (lane + i));
            b[i] = (__bf16)(0.002f * (lane - i));
        }
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[c][i];
    if (s == 12345.678f) out[blockIdx.x * 256 + threadIdx.x] = s;
}

} // namespace

hipError_t launch_calib(int kind, const void *src, void *dst, const int32_t *idx, int64_t n, int64_t table_rows, int row_bytes,
                        int wgs, hipStream_t st)
{
    dim3 grid((unsigned)wgs), block(256);
    switch (kind) {
    case IC_CALIB_READ:
        hipLaunchKernelGGL(calib_read_kernel, grid, block, 0, st, (const u32x4 *)src, n / 16, (uint32_t *)dst);
        break;
    case IC_CALIB_COPY:
        hipLaunchKernelGGL(calib_copy_kernel, grid, block, 0, st, (const u32x4 *)src, (u32x4 *)dst, n / 16);
        break;
    case IC_CALIB_GATHER:
        if (row_bytes == 1152)
            hipLaunchKernelGGL((calib_gather_kernel<9>), grid, block, 0, st, (const unsigned char *)src, idx, n, table_rows, (uint32_t *)dst);
        else if (row_bytes == 256)
            hipLaunchKernelGGL((calib_gather_kernel<2>), grid, block, 0, st, (const unsigned char *)src, idx, n, table_rows, (uint32_t *)dst);
        else
            return hipErrorInvalidValue;
        break;
    case IC_CALIB_MFMA_BF16:
        hipLaunchKernelGGL((calib_mfma_kernel<false>), grid, block, 0, st, (int)n, (float *)dst);
        break;
    case IC_CALIB_MFMA_FP8:
        hipLaunchKernelGGL((calib_mfma_kernel<true>), grid, block, 0, st, (int)n, (float *)dst);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace ic
