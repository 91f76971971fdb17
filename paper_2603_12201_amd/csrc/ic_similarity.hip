// Output similarity between a layer's attention under its own indices and under reused ones
// (paper App. C: the matrix S the similarity-based pattern search is built on).
//
// cosine_kernel: one wave per row (one query token's output over all heads, bf16); products
// and squares are exact in fp32, a lane sums a few dozen of them in fp32 and everything across
// lanes and rows is combined in fp64.  The mean over the rows goes through one fp64 atomic per
// workgroup.  HBM-bound: both tensors are read once.
#include "ic_common.hpp"

namespace ic {

namespace {

__device__ __forceinline__ float bf16_to_f32(unsigned short h) { return __uint_as_float((uint32_t)h << 16); }

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// One wave per row, rows dealt round-robin to the waves of a grid that fills the chip once: no barrier and no LDS
// inside a row, eight 16-byte vectors per tensor and lane in flight, and one fp64 atomic per workgroup at the end
// (one per row would queue tens of thousands of them on a single address).
template <bool VEC>
__global__ __launch_bounds__(256) void cosine_kernel(const unsigned short *A, const unsigned short *B, int64_t n_rows,
                                                     int64_t row_len, float *per_row, double *acc)
{
    __shared__ double part[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    double mine = 0.0;                                         // sum of this wave's rows (lane 0)
    for (int64_t r = (int64_t)blockIdx.x * 4 + wave; r < n_rows; r += n_waves) {
        const unsigned short *a = A + r * row_len, *b = B + r * row_len;
        double ab = 0.0, aa = 0.0, bb = 0.0;
        if (VEC) {
            constexpr int U = 8;
            for (int64_t c0 = 0; c0 < row_len; c0 += 64 * 8 * U) {
                u32x4 va[U], vb[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t c = c0 + ((int64_t)u * 64 + lane) * 8;
                    va[u] = u32x4{0u, 0u, 0u, 0u};
                    vb[u] = u32x4{0u, 0u, 0u, 0u};
                    if (c < row_len) {
                        va[u] = *(const u32x4 *)(a + c);
                        vb[u] = *(const u32x4 *)(b + c);
                    }
                }
                float sab = 0.f, saa = 0.f, sbb = 0.f;
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float x0 = __uint_as_float(va[u][e] << 16), x1 = __uint_as_float(va[u][e] & 0xFFFF0000u);
                        const float y0 = __uint_as_float(vb[u][e] << 16), y1 = __uint_as_float(vb[u][e] & 0xFFFF0000u);
                        sab += x0 * y0 + x1 * y1;
                        saa += x0 * x0 + x1 * x1;
                        sbb += y0 * y0 + y1 * y1;
                    }
                ab += (double)sab;
                aa += (double)saa;
                bb += (double)sbb;
            }
        } else {
            for (int64_t c0 = 0; c0 < row_len; c0 += 64 * 16) {
                float sab = 0.f, saa = 0.f, sbb = 0.f;
                for (int u = 0; u < 16; ++u) {
                    const int64_t c = c0 + (int64_t)u * 64 + lane;
                    if (c < row_len) {
                        const float x = bf16_to_f32(a[c]), y = bf16_to_f32(b[c]);
                        sab += x * y;
                        saa += x * x;
                        sbb += y * y;
                    }
                }
                ab += (double)sab;
                aa += (double)saa;
                bb += (double)sbb;
            }
        }
        ab = wave_sum(ab);
        aa = wave_sum(aa);
        bb = wave_sum(bb);
        double cs;
        if (aa == 0.0 && bb == 0.0) cs = 1.0;                  // two all-zero rows agree
        else if (aa == 0.0 || bb == 0.0) cs = 0.0;
        else cs = ab / (sqrt(aa) * sqrt(bb));
        if (lane == 0 && per_row) per_row[r] = (float)cs;
        mine += cs;
    }
    if (lane == 0) part[wave] = mine;
    __syncthreads();
    if (tid == 0) atomicAdd(acc, part[0] + part[1] + part[2] + part[3]);
}

__global__ void cosine_zero_kernel(double *acc) { *acc = 0.0; }

__global__ void cosine_finish_kernel(const double *acc, int64_t n_rows, double *mean) { *mean = *acc / (double)n_rows; }

// loss = 1/n * sum_l (1 - sims[l]): the attention-output error of a pattern against the all-Full stack
__global__ void loss_finish_kernel(const double *sims, int n, double *loss)
{
    double t = 0.0;
    for (int l = 0; l < n; ++l) t += 1.0 - sims[l];
    *loss = t / (double)n;
}

// S starts as the identity: the diagonal is 1 by definition, the upper triangle is not defined (0)
__global__ void sim_init_kernel(double *S, int n)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n * n) S[e] = (e / n == e % n) ? 1.0 : 0.0;
}

} // namespace

hipError_t launch_cosine(const void *A, const void *B, int64_t n_rows, int64_t row_len, double *mean, float *per_row,
                         double *acc, hipStream_t st)
{
    hipLaunchKernelGGL(cosine_zero_kernel, dim3(1), dim3(1), 0, st, acc);
    const bool vec = row_len % 8 == 0 && (uintptr_t)A % 16 == 0 && (uintptr_t)B % 16 == 0;
    const int64_t want = (n_rows + 3) / 4;                    // workgroups if every wave took one row
    const unsigned grid = (unsigned)(want < 2048 ? (want < 1 ? 1 : want) : 2048);   // 8 workgroups per CU at most
    if (vec)
        hipLaunchKernelGGL(cosine_kernel<true>, dim3(grid), dim3(256), 0, st, (const unsigned short *)A,
                           (const unsigned short *)B, n_rows, row_len, per_row, acc);
    else
        hipLaunchKernelGGL(cosine_kernel<false>, dim3(grid), dim3(256), 0, st, (const unsigned short *)A,
                           (const unsigned short *)B, n_rows, row_len, per_row, acc);
    hipLaunchKernelGGL(cosine_finish_kernel, dim3(1), dim3(1), 0, st, (const double *)acc, n_rows, mean);
    return hipGetLastError();
}

hipError_t launch_loss_finish(const double *sims, int n, double *loss, hipStream_t st)
{
    hipLaunchKernelGGL(loss_finish_kernel, dim3(1), dim3(1), 0, st, sims, n, loss);
    return hipGetLastError();
}

hipError_t launch_sim_init(double *S, int n, hipStream_t st)
{
    hipLaunchKernelGGL(sim_init_kernel, dim3((unsigned)((n * n + 255) / 256)), dim3(256), 0, st, S, n);
    return hipGetLastError();
}

} // namespace ic
