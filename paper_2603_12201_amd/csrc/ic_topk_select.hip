// Per-query top-k over a strip of indexer scores (T_t = Top-k(I_t), paper Sec. 3 Notation).
//
// One workgroup per query row.  Scores become order-preserving 32-bit keys; an MSB-first
// radix select (four 8-bit digits, LDS histograms) finds the exact key of the k-th largest
// score and how many entries equal to it belong to the result; one ordered pass then emits
// every position whose key is larger, plus the first (lowest-position) entries that tie with
// it, in ascending position order.  Rows of up to `cache_elems` scores are read from HBM once
// and kept in LDS for all passes.
#include "ic_common.hpp"

namespace ic {

namespace {

__device__ __forceinline__ uint32_t score_key(float x)
{
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;                      // -0 and +0 are the same score
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u); // larger float <=> larger key
}

__device__ __forceinline__ float key_score(uint32_t key)
{
    const uint32_t u = (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;
    return __uint_as_float(u);
}

constexpr int kCopies = 8; // histogram copies per digit (lanes spread over them)

template <int NT>
__global__ __launch_bounds__(NT) void select_kernel(SelectArgs a)
{
    constexpr int NW = NT / 64;
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    uint32_t *hist = smem;                     // [256][kCopies]
    uint32_t *cnt = hist + 256 * kCopies;      // [256]
    uint32_t *wtot = cnt + 256;                // [2][NW] packed per-wave totals (double buffered)
    uint32_t *bc = wtot + 2 * NW;              // [2] broadcast: chosen digit, remaining need
    uint32_t *cache = bc + 4;                  // [cache_elems] keys of the row

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = blockIdx.x;
    const int b = a.b0 + r / a.Ri;
    const int i = a.i0 + r % a.Ri;
    if (i >= a.Tq) return;
    int64_t nv64 = a.q_pos0 + (int64_t)i + 1;
    nv64 = nv64 < 0 ? 0 : (nv64 > a.Lk ? a.Lk : nv64);
    const int nv = (int)nv64;
    const float *row = a.strip + (int64_t)r * a.ld;
    int32_t *oidx = a.idx + ((int64_t)b * a.Tq + i) * a.k_sel;
    float *osel = a.sel ? a.sel + ((int64_t)b * a.Tq + i) * a.k_sel : nullptr;

    if (nv <= a.k_sel) {                       // every visible key is selected
        for (int m = tid; m < a.k_sel; m += NT) {
            oidx[m] = m < nv ? m : -1;
            if (osel) osel[m] = m < nv ? row[m] : -INFINITY;
        }
        return;
    }

    const bool cached = nv <= a.cache_elems;   // workgroup-uniform
    if (cached) {
        for (int p = tid; p < nv; p += NT) cache[p] = score_key(row[p]);
        __syncthreads();
    }
    auto get_key = [&](int p) -> uint32_t { return cached ? cache[p] : score_key(row[p]); };

    // ---- radix select: exact key of the k-th largest score ----
    uint32_t prefix = 0, prefix_mask = 0;
    uint32_t need = (uint32_t)a.k_sel;         // entries still to take among keys matching prefix
#pragma unroll 1
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int e = tid; e < 256 * kCopies; e += NT) hist[e] = 0;
        __syncthreads();
        for (int p = tid; p < nv; p += NT) {
            const uint32_t key = get_key(p);
            if ((key & prefix_mask) == prefix)
                atomicAdd(&hist[((key >> shift) & 255u) * kCopies + (lane & (kCopies - 1))], 1u);
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t s = 0;
#pragma unroll
            for (int c = 0; c < kCopies; ++c) s += hist[tid * kCopies + c];
            cnt[tid] = s;
        }
        __syncthreads();
        if (wave == 0) {
            // lane L owns digits 255-4L .. 252-4L (descending); find where the running count reaches need
            uint32_t c4[4];
            uint32_t mine = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c4[j] = cnt[255 - 4 * lane - j];
                mine += c4[j];
            }
            uint32_t incl = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            const uint32_t excl = incl - mine;
            if (excl < need && need <= incl) {           // exactly one lane
                uint32_t run = excl;
                int digit = 255 - 4 * lane;
                uint32_t left = need;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (run < need && need <= run + c4[j]) {
                        digit = 255 - 4 * lane - j;
                        left = need - run;
                    }
                    run += c4[j];
                }
                bc[0] = (uint32_t)digit;
                bc[1] = left;
            }
        }
        __syncthreads();
        prefix |= bc[0] << shift;
        prefix_mask |= 255u << shift;
        need = bc[1];
        __syncthreads();
    }
    const uint32_t tau = prefix;               // key of the k-th largest score
    const uint32_t need_eq = need;             // how many entries equal to tau are selected

    // ---- ordered emit: slot = #greater before + min(#equal before, need_eq) ----
    uint32_t run_g = 0, run_e = 0;
    const int nchunks = (nv + NT - 1) / NT;
#pragma unroll 1
    for (int c = 0; c < nchunks; ++c) {
        const int p = c * NT + tid;
        uint32_t key = 0;
        bool g = false, e = false;
        if (p < nv) {
            key = get_key(p);
            g = key > tau;
            e = key == tau;
        }
        const unsigned long long mg = __ballot(g), me = __ballot(e);
        const unsigned long long below = (1ull << lane) - 1ull;
        const uint32_t g_in = (uint32_t)__popcll(mg & below), e_in = (uint32_t)__popcll(me & below);
        uint32_t *wt = wtot + (c & 1) * NW;
        if (lane == 0) wt[wave] = ((uint32_t)__popcll(me) << 16) | (uint32_t)__popcll(mg);
        __syncthreads();
        uint32_t g_before = run_g, e_before = run_e, g_all = 0, e_all = 0;
#pragma unroll
        for (int wv = 0; wv < NW; ++wv) {
            const uint32_t t = wt[wv];
            const uint32_t tg = t & 0xFFFFu, te = t >> 16;
            if (wv < wave) {
                g_before += tg;
                e_before += te;
            }
            g_all += tg;
            e_all += te;
        }
        g_before += g_in;
        e_before += e_in;
        if (g || (e && e_before < need_eq)) {
            const uint32_t slot = g_before + (e_before < need_eq ? e_before : need_eq);
            if (slot < (uint32_t)a.k_sel) {            // always true for a consistent select
                oidx[slot] = p;
                if (osel) osel[slot] = key_score(key);
            }
        }
        run_g += g_all;
        run_e += e_all;
    }
}

size_t select_lds_bytes(int cache_elems)
{
    return (size_t)(256 * kCopies + 256 + 2 * 16 + 4 + cache_elems) * sizeof(uint32_t);
}

} // namespace

int select_cache_limit() { return 32768; }

hipError_t launch_select(const SelectArgs &a_in, int n_rows, int max_row_len, hipStream_t st)
{
    if (n_rows <= 0) return hipSuccess;
    SelectArgs a = a_in;
    int cache = max_row_len <= select_cache_limit() ? (max_row_len + 63) / 64 * 64 : select_cache_limit();
    if (max_row_len <= a.k_sel) cache = 0;     // short rows never reach the radix path
    a.cache_elems = cache;
    const size_t lds = select_lds_bytes(cache);
    // opt in once per process to the largest LDS footprint either variant can ask for
    static hipError_t attr256 = hipFuncSetAttribute((const void *)select_kernel<256>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                                    (int)select_lds_bytes(8192));
    static hipError_t attr1024 = hipFuncSetAttribute((const void *)select_kernel<1024>,
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     (int)select_lds_bytes(select_cache_limit()));
    if (attr256 != hipSuccess) return attr256;
    if (attr1024 != hipSuccess) return attr1024;
    if (max_row_len <= 8192)
        hipLaunchKernelGGL((select_kernel<256>), dim3((unsigned)n_rows), dim3(256), lds, st, a);
    else
        hipLaunchKernelGGL((select_kernel<1024>), dim3((unsigned)n_rows), dim3(1024), lds, st, a);
    return hipGetLastError();
}

} // namespace ic
