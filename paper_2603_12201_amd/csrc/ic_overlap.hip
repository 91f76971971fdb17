// Pairwise cross-layer overlap of the top-k index sets (paper App. A: |T(i) ^ T(j)| / k for every
// pair of layers, averaged over the queries).
//
// A workgroup owns one layer i and a block of kQB query rows.  Per query it marks layer i's
// selected positions in an LDS bitmap of Lk bits, then tests the rows of every layer j >= i against
// it (the intersection count is symmetric); hits are counted with a wave ballot + popcount and
// summed per j in LDS; one 64-bit global atomic per (workgroup, j) at the end.  The workgroups
// that share a block of query rows (all layers i) are mapped to one XCD and to neighbouring
// positions in dispatch order, so the index rows they all read come out of that XCD's L2; with
// the layers dealt over all eight L2s every pair's rows came from memory (315 GB of fetches for
// 48 layers at 32K queries) and the kernel ran at the memory rate instead of the LDS rate.
#include "ic_common.hpp"

namespace ic {

namespace {

constexpr int kQB = 16;          // query rows per workgroup

struct OverlapArgs {
    const int32_t *idx[IC_MAX_OVERLAP_LAYERS];
    unsigned long long *inter;   // [n_layers, n_layers], only j >= i written
    unsigned long long *sizes;   // [n_layers]
    int64_t nq;
    int32_t n_layers, k_sel, Lk, bm_words;
};

// VEC: rows are read as 16-byte vectors (k_sel % 4 == 0, 16-byte aligned tensors); the rows of kJU
// layers are requested together so that their latencies overlap.
template <bool VEC>
__global__ __launch_bounds__(256) void overlap_kernel(OverlapArgs a)
{
    constexpr int kJU = 4;                     // layers j tested per round
    constexpr int kNV = IC_MAX_K / (256 * 4);  // 16-byte vectors per thread and row
    extern __shared__ __attribute__((aligned(16))) uint32_t osm[];
    uint32_t *bm = osm;                        // [bm_words]
    uint32_t *cnt = osm + a.bm_words;          // [n_layers] hits per layer j, + [1] members of layer i
    const int tid = threadIdx.x, lane = tid & 63;
    // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2: id % 8 picks the
    // query block's residue, so that all layers i of one query block run on the same XCD, next to
    // each other in dispatch order, and find each other's index rows in that L2.
    const unsigned xcd = blockIdx.x & 7u, rest = blockIdx.x >> 3;
    const int i = (int)(rest % (unsigned)a.n_layers);
    const int64_t q0 = ((int64_t)(rest / (unsigned)a.n_layers) * 8 + xcd) * kQB;
    if (q0 >= a.nq) return;                    // the grid is padded to a multiple of 8 query blocks
    const int64_t q1 = q0 + kQB < a.nq ? q0 + kQB : a.nq;

    auto member = [&](int32_t v) -> bool {
        const bool ok = v >= 0 && v < a.Lk;
        return ok && ((bm[ok ? (v >> 5) : 0] >> (v & 31)) & 1u);
    };

    for (int e = tid; e <= a.n_layers; e += 256) cnt[e] = 0;
    for (int64_t q = q0; q < q1; ++q) {
        for (int e = tid; e < a.bm_words; e += 256) bm[e] = 0;
        __syncthreads();
        const int32_t *ri = a.idx[i] + q * a.k_sel;
        uint32_t members = 0;                  // wave-uniform
        for (int m0 = 0; m0 < a.k_sel; m0 += 256) {
            const int m = m0 + tid;
            const int32_t v = m < a.k_sel ? ri[m] : -1;
            const bool ok = v >= 0 && v < a.Lk;
            if (ok) atomicOr(&bm[v >> 5], 1u << (v & 31));
            members += (uint32_t)__popcll(__ballot(ok));
        }
        if (lane == 0 && members) atomicAdd(&cnt[a.n_layers], members);
        __syncthreads();
        if (VEC) {
            for (int j0 = i; j0 < a.n_layers; j0 += kJU) {
                i32x4 v[kJU][kNV];
#pragma unroll
                for (int u = 0; u < kJU; ++u) {
                    const int j = j0 + u < a.n_layers ? j0 + u : a.n_layers - 1;     // clamped: loads stay unconditional
                    const int32_t *rj = a.idx[j] + q * a.k_sel;
#pragma unroll
                    for (int c = 0; c < kNV; ++c) {
                        const int m = (c * 256 + tid) * 4;
                        v[u][c] = *(const i32x4 *)(rj + (m < a.k_sel ? m : 0));
                    }
                }
#pragma unroll
                for (int u = 0; u < kJU; ++u) {
                    if (j0 + u >= a.n_layers) break;                               // uniform
                    uint32_t hits = 0;         // wave-uniform
#pragma unroll
                    for (int c = 0; c < kNV; ++c) {
                        const bool in_row = (c * 256 + tid) * 4 < a.k_sel;
#pragma unroll
                        for (int e = 0; e < 4; ++e) hits += (uint32_t)__popcll(__ballot(in_row && member(v[u][c][e])));
                    }
                    if (lane == 0 && hits) atomicAdd(&cnt[j0 + u], hits);
                }
            }
        } else {
            for (int j = i; j < a.n_layers; ++j) {
                const int32_t *rj = a.idx[j] + q * a.k_sel;
                uint32_t hits = 0;             // wave-uniform
                for (int m0 = 0; m0 < a.k_sel; m0 += 256) {
                    const int m = m0 + tid;
                    hits += (uint32_t)__popcll(__ballot(member(m < a.k_sel ? rj[m] : -1)));
                }
                if (lane == 0 && hits) atomicAdd(&cnt[j], hits);
            }
        }
        __syncthreads();                       // everyone is done with the bitmap
    }
    __syncthreads();
    for (int j = i + tid; j < a.n_layers; j += 256)
        if (cnt[j]) atomicAdd(&a.inter[(int64_t)i * a.n_layers + j], (unsigned long long)cnt[j]);
    if (tid == 0 && cnt[a.n_layers]) atomicAdd(&a.sizes[i], (unsigned long long)cnt[a.n_layers]);
}

__global__ void overlap_zero_kernel(unsigned long long *p, int n)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) p[e] = 0ull;
}

// overlap(i,j) = inter(min,max) / sizes(i); also mirrors the counts into the caller's buffers
__global__ void overlap_finish_kernel(const unsigned long long *inter, const unsigned long long *sizes, int n,
                                      double *overlap, unsigned long long *inter_out, unsigned long long *sizes_out)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n * n) return;
    const int i = e / n, j = e % n;
    const unsigned long long c = inter[i <= j ? (int64_t)i * n + j : (int64_t)j * n + i];
    const unsigned long long s = sizes[i];
    if (overlap) overlap[e] = s ? (double)c / (double)s : 0.0;
    if (inter_out) inter_out[e] = c;
    if (sizes_out && j == 0) sizes_out[i] = s;
}

} // namespace

size_t overlap_ws_bytes(int n_layers) { return ((size_t)n_layers * n_layers + n_layers) * sizeof(unsigned long long); }

size_t overlap_lds_bytes(int n_layers, int Lk) { return ((size_t)(Lk + 31) / 32 + n_layers + 1) * sizeof(uint32_t); }

hipError_t launch_overlap(const int32_t *const *idx_layers, int n_layers, int64_t nq, int k_sel, int Lk, double *overlap,
                          unsigned long long *inter_out, unsigned long long *sizes_out, void *ws, hipStream_t st)
{
    OverlapArgs a;
    for (int l = 0; l < IC_MAX_OVERLAP_LAYERS; ++l) a.idx[l] = l < n_layers ? idx_layers[l] : nullptr;
    a.inter = (unsigned long long *)ws;
    a.sizes = a.inter + (size_t)n_layers * n_layers;
    a.nq = nq;
    a.n_layers = n_layers;
    a.k_sel = k_sel;
    a.Lk = Lk;
    a.bm_words = (Lk + 31) / 32;
    const int nz = n_layers * n_layers + n_layers;
    hipLaunchKernelGGL(overlap_zero_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st, a.inter, nz);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (nq > 0) {
        const size_t lds = overlap_lds_bytes(n_layers, Lk);
        bool vec = k_sel % 4 == 0 && k_sel <= IC_MAX_K;
        for (int l = 0; l < n_layers; ++l) vec = vec && ((uintptr_t)idx_layers[l] % 16 == 0);
        static size_t lds_opt_in[2] = {0, 0};  // largest footprint opted in so far (per process and variant)
        const void *fn = vec ? (const void *)overlap_kernel<true> : (const void *)overlap_kernel<false>;
        if (lds > lds_opt_in[vec]) {
            e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            lds_opt_in[vec] = lds;
        }
        dim3 grid((unsigned)(((nq + kQB - 1) / kQB + 7) / 8 * 8 * n_layers));
        if (vec)
            hipLaunchKernelGGL(overlap_kernel<true>, grid, dim3(256), lds, st, a);
        else
            hipLaunchKernelGGL(overlap_kernel<false>, grid, dim3(256), lds, st, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const int nn = n_layers * n_layers;
    hipLaunchKernelGGL(overlap_finish_kernel, dim3((unsigned)((nn + 255) / 256)), dim3(256), 0, st, a.inter, a.sizes, n_layers,
                       overlap, inter_out, sizes_out);
    return hipGetLastError();
}

} // namespace ic
