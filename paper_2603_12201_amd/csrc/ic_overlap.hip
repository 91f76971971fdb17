// Pairwise cross-layer overlap of the top-k index sets (paper App. A: |T(i) ^ T(j)| / k for every
// pair of layers, averaged over the queries).  Two forms.
//
// Bitmap form (position ranges up to 256 k: the usual case).  One workgroup of 16 waves per CU walks
// over query rows.  Per query and per chunk of the position range it turns the row of every layer into
// a bitmap in LDS (one LDS atomic OR per member), and then every pair of layers i <= j costs one AND
// and one population count per 32 positions: a wave takes a tile of 4 x 4 layers, every lane four
// consecutive words of the eight bitmaps (16-byte LDS reads, no bank conflicts), 16 counters per
// lane, a transposing butterfly over the lanes at the end of the tile, sums per pair in LDS for all the
// queries of the workgroup, one 64-bit global atomic per pair and workgroup at the very end.  The
// members of a row are distinct (the contract of the entry point), so a layer's set size is the
// diagonal count.  The index rows are read once per chunk, nothing else touches memory.
//
// Membership form (very long position ranges with few members, where whole bitmaps would be mostly
// zeros).  A workgroup owns one layer i and a block of kQB query rows.  Per query it marks layer i's
// selected positions in an LDS bitmap of Lk bits, then tests the rows of every layer j >= i against
// it (the intersection count is symmetric); hits are counted with a wave ballot + popcount and
// summed per j in LDS; one 64-bit global atomic per (workgroup, j) at the end.  The workgroups
// that share a block of query rows (all layers i) are mapped to one XCD and to neighbouring
// positions in dispatch order, so the index rows they all read come out of that XCD's L2.
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

// ---------------------------------------- bitmap form ----------------------------------------
constexpr int kBitsThreads = 1024;
constexpr int kBitsLdsBudget = 150 * 1024;

struct BitsPlan { int W, logW, n_chunks; size_t lds; };

// words per layer and chunk: a power of two such that the bitmaps of all layers, the pair counters and
// the pointer table fit the LDS budget, and no larger than a whole row
BitsPlan bits_plan(int n_layers, int Lk)
{
    BitsPlan p;
    const int words = (Lk + 31) / 32;
    const size_t fixed = (size_t)n_layers * n_layers * 4 + (size_t)n_layers * 8;
    int W = 4, logW = 2;
    while (W < 4096 && W < words && fixed + (size_t)n_layers * (2 * W) * 4 <= (size_t)kBitsLdsBudget) {
        W *= 2;
        ++logW;
    }
    p.W = W;
    p.logW = logW;
    p.n_chunks = (words + W - 1) / W;
    p.lds = fixed + (size_t)n_layers * W * 4;
    return p;
}

// VEC: rows are read as 16-byte vectors (k_sel % 4 == 0, 16-byte aligned tensors)
template <bool VEC>
__global__ __launch_bounds__(kBitsThreads) void overlap_bits_kernel(OverlapArgs a, int W, int logW, int n_chunks)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t osm[];
    const int N = a.n_layers;
    uint32_t *bm = osm;                                        // [N][W]
    const int32_t **ptrs = (const int32_t **)(bm + (size_t)N * W);    // [N] (an LDS copy: lanes index it by layer)
    uint32_t *cnt = (uint32_t *)(ptrs + N);                    // [N][N], only j >= i used
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int e = tid; e < N * N; e += kBitsThreads) cnt[e] = 0;
    for (int l = tid; l < N; l += kBitsThreads) ptrs[l] = a.idx[l];
    // the flat space of a query's members: layer-major, EV entries per item
    constexpr int EV = VEC ? 4 : 1;
    const int per_row = a.k_sel / EV;                          // items per layer row
    const int dq = kBitsThreads / per_row, dr = kBitsThreads % per_row;
    const int l_first = tid / per_row, m_first = tid % per_row;
    // tiles of 4 x 4 layers over the upper triangle, dealt to the 16 waves
    const int NB = (N + 3) / 4;
    const int n_tiles = NB * (NB + 1) / 2;
    // the workgroup's sums go out at the end, and before a 32-bit counter could wrap (a pair gains at most k_sel
    // per query); a layer's set size is its diagonal count (distinct members)
    auto flush = [&]() {
        for (int e = tid; e < N * N; e += kBitsThreads) {
            const int i = e / N, j = e % N;
            const uint32_t cv = cnt[e];
            if (j >= i && cv) {
                atomicAdd(&a.inter[(int64_t)i * N + j], (unsigned long long)cv);
                if (i == j) atomicAdd(&a.sizes[i], (unsigned long long)cv);
            }
            cnt[e] = 0;
        }
    };
    const int64_t flush_every = (int64_t)(0x7fffffff / a.k_sel) > 0 ? (int64_t)(0x7fffffff / a.k_sel) : 1;
    int64_t done = 0;
    __syncthreads();
    for (int64_t q = blockIdx.x; q < a.nq; q += gridDim.x) {
        if (++done % flush_every == 0) {                       // (uniform; the last barrier of the chunk loop precedes it)
            flush();
            __syncthreads();
        }
        for (int c = 0; c < n_chunks; ++c) {
            // positions of this chunk
            const uint32_t lo = (uint32_t)c << (5 + logW);
            const uint32_t span = min((uint32_t)a.Lk - lo, 32u << logW);
            // (A) clear the bitmaps
            for (int e = tid * 4; e < N * W; e += kBitsThreads * 4) *(u32x4 *)(bm + e) = u32x4{0u, 0u, 0u, 0u};
            __syncthreads();
            // (B) one bit per member whose position falls into this chunk
            // (eight loads in flight per thread: the rows come from memory, one load at a time would leave the
            // workgroup waiting for most of this phase)
            for (int l = l_first, m = m_first; l < N;) {
                constexpr int kInFlight = 8;
                int ll[kInFlight];
                int32_t v[kInFlight][EV];
#pragma unroll
                for (int b = 0; b < kInFlight; ++b) {
                    ll[b] = l;
                    const int32_t *row = ptrs[min(l, N - 1)] + q * a.k_sel;
                    if constexpr (VEC) {
                        const i32x4 x = *(const i32x4 *)(row + 4 * m);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[b][e] = x[e];
                    } else {
                        v[b][0] = row[m];
                    }
                    l += dq;
                    m += dr;
                    if (m >= per_row) {
                        m -= per_row;
                        ++l;
                    }
                }
#pragma unroll
                for (int b = 0; b < kInFlight; ++b)
#pragma unroll
                    for (int e = 0; e < EV; ++e) {
                        // (negative and out-of-range entries fall outside every chunk's [lo, lo + span))
                        const uint32_t u = (uint32_t)v[b][e] - lo;
                        if (ll[b] < N && u < span) atomicOr(&bm[ll[b] * W + (u >> 5)], 1u << (u & 31u));
                    }
            }
            __syncthreads();
            // (C) AND + population count, a tile of 4 x 4 pairs at a time
            for (int t = wave; t < n_tiles; t += kBitsThreads / 64) {
                // tile number -> (bi <= bj): row bi of the triangle starts at bi * NB - bi (bi - 1) / 2
                int bi = 0, rem = t;
                while (rem >= NB - bi) {
                    rem -= NB - bi;
                    ++bi;
                }
                const int bj = bi + rem;
                const uint32_t *ri[4], *rj[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    ri[x] = bm + (size_t)min(4 * bi + x, N - 1) * W;
                    rj[x] = bm + (size_t)min(4 * bj + x, N - 1) * W;
                }
                uint32_t s[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) s[e] = 0;
                for (int w0 = lane * 4; w0 < W; w0 += 256) {
                    u32x4 wi[4], wj[4];
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        wi[x] = *(const u32x4 *)(ri[x] + w0);
                        wj[x] = *(const u32x4 *)(rj[x] + w0);
                    }
#pragma unroll
                    for (int x = 0; x < 4; ++x)
#pragma unroll
                        for (int y = 0; y < 4; ++y)
#pragma unroll
                            for (int e = 0; e < 4; ++e) s[4 * x + y] += (uint32_t)__popc(wi[x][e] & wj[y][e]);
                }
                // transposing butterfly: afterwards lane 4 p holds the wave's sum of counter p
                uint32_t d8[8], d4[4], d2[2];
                const bool b5 = lane & 32, b4 = lane & 16, b3 = lane & 8, b2 = lane & 4;
#pragma unroll
                for (int e = 0; e < 8; ++e) d8[e] = (b5 ? s[e + 8] : s[e]) + (uint32_t)__shfl_xor((int)(b5 ? s[e] : s[e + 8]), 32);
#pragma unroll
                for (int e = 0; e < 4; ++e) d4[e] = (b4 ? d8[e + 4] : d8[e]) + (uint32_t)__shfl_xor((int)(b4 ? d8[e] : d8[e + 4]), 16);
#pragma unroll
                for (int e = 0; e < 2; ++e) d2[e] = (b3 ? d4[e + 2] : d4[e]) + (uint32_t)__shfl_xor((int)(b3 ? d4[e] : d4[e + 2]), 8);
                uint32_t d1 = (b2 ? d2[1] : d2[0]) + (uint32_t)__shfl_xor((int)(b2 ? d2[0] : d2[1]), 4);
                d1 += (uint32_t)__shfl_xor((int)d1, 2);
                d1 += (uint32_t)__shfl_xor((int)d1, 1);
                const int pr = lane >> 2;                      // counter 4 x + y
                const int i = 4 * bi + (pr >> 2), j = 4 * bj + (pr & 3);
                if ((lane & 3) == 0 && i < N && j < N && i <= j && d1) atomicAdd(&cnt[i * N + j], d1);
            }
            __syncthreads();                                   // the bitmaps are free again
        }
    }
    flush();
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
    bool vec = k_sel % 4 == 0;
    for (int l = 0; l < n_layers; ++l) vec = vec && ((uintptr_t)idx_layers[l] % 16 == 0);
    if (nq > 0 && (int64_t)Lk <= 256 * (int64_t)k_sel) {
        // bitmap form: an AND per 32 positions costs less than a membership test per member up to about here
        const BitsPlan bp = bits_plan(n_layers, Lk);
        static int n_cu = 0;
        if (n_cu == 0) {
            int dev = 0, v = 0;
            if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
                return hipErrorInvalidDevice;
            n_cu = v;
        }
        static size_t lds_opt_in[2] = {0, 0};  // largest footprint opted in so far (per process and variant)
        const void *fn = vec ? (const void *)overlap_bits_kernel<true> : (const void *)overlap_bits_kernel<false>;
        if (bp.lds > lds_opt_in[vec]) {
            e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bp.lds);
            if (e != hipSuccess) return e;
            lds_opt_in[vec] = bp.lds;
        }
        dim3 grid((unsigned)(nq < n_cu ? nq : n_cu));
        if (vec)
            hipLaunchKernelGGL(overlap_bits_kernel<true>, grid, dim3(kBitsThreads), bp.lds, st, a, bp.W, bp.logW, bp.n_chunks);
        else
            hipLaunchKernelGGL(overlap_bits_kernel<false>, grid, dim3(kBitsThreads), bp.lds, st, a, bp.W, bp.logW, bp.n_chunks);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else if (nq > 0) {
        const size_t lds = overlap_lds_bytes(n_layers, Lk);
        vec = vec && k_sel <= IC_MAX_K;
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
