// Per-query top-k over a strip of indexer scores (T_t = Top-k(I_t), paper Sec. 3 Notation).
//
// One workgroup per query row.  Scores become order-preserving 32-bit keys.  An MSB-first
// radix select finds the exact key of the k-th largest score and how many entries equal to it
// belong to the result; one ordered pass then emits every position whose key is larger, plus
// the first (lowest-position) entries that tie with it, in ascending position order.
//
//   pass 1   12-bit digit (sign, exponent, 3 mantissa bits) over the whole row, fused with the
//            single read of the row from HBM; rows of up to `cache_elems` keys stay in LDS
//   pass 2,3 12 + 8 bits; only entries that match the prefix found so far touch the histogram,
//            so these are read-mostly sweeps over the cached row.  The sweeps stop as soon as the
//            boundary bin holds exactly the entries still needed (with distinct scores: after
//            pass 2), because then every entry with key >= prefix is selected
//   emit     a thread owns 4 consecutive positions in every sweep.  When every entry equal to the
//            k-th key is selected (the usual case: known from the last histogram) "selected" is
//            the single test key >= tau: per-thread counts of two sweeps packed in one word, one
//            wave scan per word on the DPP path, one scan over the (sweep, wave) cells, two
//            barriers in all.  When ties are cut at the boundary: per-sweep scans of packed
//            greater / equal counts.
// Forms by row length: the radix select with the keys cached in LDS (launches whose rows have up to 8192 keys; up to
// 32768 when k exceeds a quarter of the row), the candidate form further down (8193 to 131072 keys; two instances, the
// one for rows of up to 32768 keys sized so that two rows are in flight per CU), and the radix select re-reading the
// row on every sweep (whatever is longer).
#include "ic_common.hpp"

namespace ic {

namespace {

__device__ __forceinline__ uint32_t score_key(float x)
{
    uint32_t u = __float_as_uint(x);
    u = (u == 0x80000000u) ? 0u : u;                   // -0 and +0 are the same score
    const uint32_t flip = (uint32_t)((int32_t)u >> 31) | 0x80000000u;   // all ones for negatives, else the sign bit
    return u ^ flip;                                   // larger float <=> larger key
}

__device__ __forceinline__ float key_score(uint32_t key)
{
    const uint32_t u = (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;
    return __uint_as_float(u);
}

constexpr int kBins1 = 4096;   // histogram bins: digits of 12, 12 and 8 key bits

// Inclusive prefix sum over the 64 lanes of a wave on the data-parallel-primitive path of the
// vector ALU (no LDS traffic): shifts by 1, 2, 4, 8 lanes inside each row of 16 lanes, then the
// last lane of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.  Lanes
// without a source add zero.  Packed fields are summed independently as long as none overflows.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);   // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);   // row_shr:8
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1, 3
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2, 3
    return x;
}

// Workgroup-wide descending scan over `nbins` counters: finds the digit d with
// count(bins > d) < need <= count(bins >= d) and writes {d, need - count(bins > d), count(bin d)} to bc.
// Every thread owns BPT consecutive bins, highest bins first.  A bin is the sum of R adjacent
// counters (R > 1: the histogram was spread over R copies against same-address collisions).
template <int NT, int BPT, int R = 1>
__device__ __forceinline__ void find_digit(const uint32_t *cnt, uint32_t need, uint32_t *wsum, uint32_t *bc,
                                           int tid, int lane, int wave)
{
    constexpr int NW = NT / 64;
    const int top = NT * BPT - 1 - BPT * tid;          // highest bin of this thread
    uint32_t c[BPT];
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        if constexpr (R == 1) {
            c[j] = cnt[top - j];
        } else {
            static_assert(R % 4 == 0, "copies are read as 16-byte vectors");
            c[j] = 0;
#pragma unroll
            for (int q = 0; q < R / 4; ++q) {
                const u32x4 v = *(const u32x4 *)(cnt + (top - j) * R + 4 * q);
                c[j] += v[0] + v[1] + v[2] + v[3];
            }
        }
        mine += c[j];
    }
    uint32_t incl = wave_incl_scan(mine);
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
#pragma unroll
    for (int wv = 0; wv < NW; ++wv)
        if (wv < wave) before += wsum[wv];
    incl += before;
    const uint32_t excl = incl - mine;
    if (excl < need && need <= incl) {                 // exactly one thread
        uint32_t run = excl;
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            if (run < need && need <= run + c[j]) {
                bc[0] = (uint32_t)(top - j);
                bc[1] = need - run;
                bc[2] = c[j];
            }
            run += c[j];
        }
    }
    __syncthreads();
}

// The radix select of one row (workgroup-wide; smem: kBins1 + 2 NW + 4 + a.cache_elems words).
template <int NT>
__device__ __forceinline__ void select_row_generic(const SelectArgs &a, uint32_t *smem)
{
    constexpr int NW = NT / 64;
    uint32_t *hist1 = smem;                    // [kBins1]
    uint32_t *wsum = hist1 + kBins1;           // [2][NW] (scan partials / emit totals, double buffered)
    uint32_t *bc = wsum + 2 * NW;              // [4] broadcast: digit, remaining need
    uint32_t *cache = bc + 4;                  // [cache_elems] keys of the row

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = blockIdx.x;
    const int b = a.b0 + r / a.Ri;
    const int i = a.i0 + r % a.Ri;
    if (i >= a.Tq) return;
    // ragged cache: the sequence holds Lk_b keys and its Tq query rows are its last Tq positions
    const int Lk_b = a.seq_lens ? max(0, min(a.seq_lens[b], a.Lk)) : a.Lk;
    int64_t nv64 = (a.seq_lens ? (int64_t)Lk_b - a.Tq : a.q_pos0) + (int64_t)i + 1;
    nv64 = nv64 < 0 ? 0 : (nv64 > Lk_b ? Lk_b : nv64);
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
    // four consecutive keys starting at p (p % 4 == 0); entries at or beyond nv are unspecified
    auto get_key4 = [&](int p) -> u32x4 {
        u32x4 k4 = u32x4{0u, 0u, 0u, 0u};
        if (p < nv) {
            if (cached) {
                k4 = *(const u32x4 *)(cache + p);
            } else {
                const f32x4 v = *(const f32x4 *)(row + p);
#pragma unroll
                for (int e = 0; e < 4; ++e) k4[e] = score_key(v[e]);
            }
        }
        return k4;
    };

    // ---- pass 1: 12-bit digit, fused with the read of the row ----
    for (int e = tid; e < kBins1; e += NT) hist1[e] = 0;
    __syncthreads();
    {
        // 16-byte loads, kLoadBatch of them in flight per thread: the strip lives in HBM and one
        // workgroup per CU has to cover the whole memory latency by itself.  Rows start 256-byte
        // aligned and are padded to a multiple of 64 floats, so the last vector may run past nv
        // (never past the row); those lanes are masked.
        constexpr int kLoadBatch = 4;
        for (int base = 0; base < nv; base += NT * 4 * kLoadBatch) {
            f32x4 v[kLoadBatch];
#pragma unroll
            for (int u = 0; u < kLoadBatch; ++u) {
                const int p = base + (u * NT + tid) * 4;
                v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (p < nv) v[u] = *(const f32x4 *)(row + p);
            }
#pragma unroll
            for (int u = 0; u < kLoadBatch; ++u) {
                const int p = base + (u * NT + tid) * 4;
                if (p < nv) {
                    u32x4 k4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        k4[e] = score_key(v[u][e]);
                        if (p + e < nv) atomicAdd(&hist1[k4[e] >> 20], 1u);
                    }
                    if (cached) *(u32x4 *)(cache + p) = k4;   // cache is 16-byte aligned, p % 4 == 0
                }
            }
        }
    }
    __syncthreads();
    find_digit<NT, kBins1 / NT>(hist1, (uint32_t)a.k_sel, wsum, bc, tid, lane, wave);
    uint32_t prefix = bc[0] << 20, prefix_mask = 0xFFF00000u;
    uint32_t need = bc[1];
    // Once the boundary bin holds exactly as many entries as are still needed, all of them are
    // selected and the remaining digits do not matter: "selected" is key >= prefix (rest zero).
    // With distinct scores that happens after the second digit, which saves the third sweep.
    bool all_sel = bc[2] == need;              // workgroup-uniform
    uint32_t total_eq = bc[2];
    __syncthreads();

    // ---- passes 2 and 3: bits [19:8] and [7:0] of the entries that match the prefix so far ----
#pragma unroll 1
    for (int pass = 0; pass < 2 && !all_sel; ++pass) {
        const int shift = pass == 0 ? 8 : 0;
        const uint32_t dmask = pass == 0 ? 4095u : 255u;
        for (int e = tid; e < kBins1; e += NT) hist1[e] = 0;
        __syncthreads();
        for (int p0 = 0; p0 < nv; p0 += 4 * NT) {
            const int p = p0 + 4 * tid;
            const u32x4 k4 = get_key4(p);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (p + e < nv && (k4[e] & prefix_mask) == prefix) atomicAdd(&hist1[(k4[e] >> shift) & dmask], 1u);
        }
        __syncthreads();
        find_digit<NT, kBins1 / NT>(hist1, need, wsum, bc, tid, lane, wave);
        prefix |= bc[0] << shift;
        prefix_mask |= dmask << shift;
        need = bc[1];
        total_eq = bc[2];
        all_sel = total_eq == need;
        __syncthreads();
    }
    // tau: key of the k-th largest score, or (all_sel) a lower bound of it that no unselected entry
    // reaches.  need_eq: how many of the total_eq entries equal to tau are selected.
    const uint32_t tau = prefix;
    const uint32_t need_eq = need;

    // ---- ordered emit, common case: the row is cached, has at most kFastChunks sweeps, and every
    // entry equal to tau is selected (the k-th score is unique, or all of its ties fit).  Then
    // "selected" is the single test key >= tau and the slot of an entry is the number of selected
    // entries ahead of it in (chunk, wave, lane, element) order: one packed wave scan per chunk
    // pair, one scan over the (chunk, wave) cells, two barriers in all. ----
    constexpr int kFastChunks = 8;
    const int nchunks = (nv + 4 * NT - 1) / (4 * NT);
    if (cached && nchunks <= kFastChunks && all_sel) {
        uint32_t *cellsum = hist1;                     // [kFastChunks / 2][NW]  (the histogram is dead: its barrier is behind us)
        uint32_t *cellbase = cellsum + kFastChunks / 2 * NW;   // [kFastChunks * NW]
        uint32_t cw[kFastChunks / 2], inc[kFastChunks / 2];
#pragma unroll
        for (int j = 0; j < kFastChunks / 2; ++j) {
            uint32_t n2[2] = {0u, 0u};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int p = (2 * j + h) * 4 * NT + 4 * tid;
                if (2 * j + h < nchunks) {             // workgroup-uniform
                    const u32x4 k4 = get_key4(p);
#pragma unroll
                    for (int e = 0; e < 4; ++e) n2[h] += (p + e < nv && k4[e] >= tau) ? 1u : 0u;
                }
            }
            cw[j] = n2[0] | (n2[1] << 16);
            inc[j] = wave_incl_scan(cw[j]);
        }
        if (lane == 63) {
#pragma unroll
            for (int j = 0; j < kFastChunks / 2; ++j) cellsum[j * NW + wave] = inc[j];
        }
        __syncthreads();
        if (wave == 0) {
            // cells in (chunk, wave) order, 64 at a time
            uint32_t carry = 0;
#pragma unroll
            for (int base = 0; base < kFastChunks * NW; base += 64) {
                const int cell = base + lane, c = cell / NW, w = cell % NW;
                const bool real = cell < kFastChunks * NW;
                const uint32_t v = real ? (cellsum[(c >> 1) * NW + w] >> (16 * (c & 1))) & 0xFFFFu : 0u;
                const uint32_t in = wave_incl_scan(v);
                if (real) cellbase[cell] = carry + in - v;
                carry += __shfl(in, 63);
            }
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < kFastChunks; ++c) {
            if (c >= nchunks) continue;                // workgroup-uniform
            const int p = c * 4 * NT + 4 * tid;
            const u32x4 k4 = get_key4(p);
            uint32_t slot = cellbase[c * NW + wave] + (((inc[c >> 1] - cw[c >> 1]) >> (16 * (c & 1))) & 0xFFFFu);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (p + e < nv && k4[e] >= tau) {
                    if (slot < (uint32_t)a.k_sel) {    // always true for a consistent select
                        oidx[slot] = p + e;
                        if (osel) osel[slot] = key_score(k4[e]);
                    }
                    ++slot;
                }
            }
        }
        return;
    }

    // ---- ordered emit, general case: slot = #greater before + min(#equal before, need_eq) ----
    // A thread owns 4 consecutive positions; the counts of greater / equal entries of ONE chunk
    // (at most 4 * NT of each) travel packed in one word (equal << 16 | greater) through a wave scan
    // and a 16-entry scan of the wave totals.  The totals over all previous chunks are kept in two
    // full words: a row longer than 65535 keys may tie with the k-th score in more than 65535 places.
    static_assert(4 * NT < 65536, "per-chunk counts must fit 16 bits");
    uint32_t run_g = 0, run_e = 0;                     // greater / equal entries of all previous chunks
#pragma unroll 1
    for (int c = 0; c < nchunks; ++c) {
        const int p = c * 4 * NT + 4 * tid;
        const u32x4 k4 = get_key4(p);
        uint32_t gm = 0, em = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (p + e < nv) {
                gm |= ((all_sel ? k4[e] >= tau : k4[e] > tau) ? 1u : 0u) << e;
                em |= ((!all_sel && k4[e] == tau) ? 1u : 0u) << e;
            }
        }
        const uint32_t mine = ((uint32_t)__popc(em) << 16) | (uint32_t)__popc(gm);
        uint32_t incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        uint32_t *wt = wsum + (c & 1) * NW;
        if (lane == 63) wt[wave] = incl;
        __syncthreads();
        uint32_t ws = lane < NW ? wt[lane] : 0u;       // scan of the wave totals (NW <= 16)
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            const uint32_t up = __shfl_up(ws, off);
            if (lane >= off) ws += up;
        }
        const uint32_t waves_before = wave == 0 ? 0u : __shfl(ws, wave - 1);
        const uint32_t chunk_total = __shfl(ws, NW - 1);
        const uint32_t before = waves_before + incl - mine;   // inside this chunk: both fields < 65536
        uint32_t g_before = run_g + (before & 0xFFFFu), e_before = run_e + (before >> 16);
        if ((gm | em) != 0u) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool g = (gm >> e) & 1u, q = (em >> e) & 1u;
                if (g || (q && e_before < need_eq)) {
                    const uint32_t slot = g_before + (e_before < need_eq ? e_before : need_eq);
                    if (slot < (uint32_t)a.k_sel) {    // always true for a consistent select
                        oidx[slot] = p + e;
                        if (osel) osel[slot] = key_score(k4[e]);
                    }
                }
                g_before += g ? 1u : 0u;
                e_before += q ? 1u : 0u;
            }
        }
        run_g += chunk_total & 0xFFFFu;
        run_e += chunk_total >> 16;
    }
}

template <int NT>
__global__ __launch_bounds__(NT) void select_kernel(SelectArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    select_row_generic<NT>(a, smem);
}

// ---- candidate form (long rows) ------------------------------------------------------------------
// For rows much longer than k almost every key is far below the k-th score, and pushing all of them through
// the digit histograms (LDS atomics into the few dozen bins a row's exponents fall into) is what the generic
// form spends its time on.  Here the row is read ONCE:
//   sample    4096 keys in 32 contiguous blocks spread over the row -> a histogram of 4096 linear bins between
//             the smallest and the largest sampled key -> a threshold T0 that about 2k keys of the row should reach
//   sweep     one pass over the row: every wave appends its keys >= T0 to a candidate list of its own in LDS (no
//             atomics: a wave scan places the entries), their maximum is tracked
//   select    one histogram over the candidates with 4096 LINEAR bins between T0 and that maximum (candidates
//             spread over all of them), a scan for the bin of the k-th largest, and an exact ranking
//             (key descending, position ascending) of the few members of that bin
//   emit      selected positions set bits in a bitmap of the row; a prefix count over the bitmap words gives
//             every selected candidate its slot, so positions come out ascending with their scores
// Exact for every input: whenever a step cannot proceed (fewer than k candidates, more than the list holds,
// too many ties in the boundary bin) the workgroup falls back to the generic radix select on the same row.
constexpr int kCandCap = 12288;          // candidate list entries (6 k for k = 2048)
constexpr int kCandMinLen = 8192;        // shorter rows of a launch take the generic form at once
constexpr int kCandFrom = 8192;          // launches whose longest row exceeds this use the candidate form (measured: with
                                         // two rows in flight per CU it beats the LDS-cached generic form from here on;
                                         // with one it did so only from 16384)
constexpr int kCandMaxLen = 131072;      // bitmap capacity
constexpr int kCandSample = 4096;
constexpr int kBoundaryCap = 1024;       // boundary-bin members ranked exactly
// A second instance for rows of up to kCandSmallLen keys: half the threads and half the LDS, so that two rows are in
// flight per CU (a row's phases are chains of latencies; a second workgroup fills them)
constexpr int kCandSmallLen = 32768;
constexpr int kCandSmallCap = 6144;
constexpr int cand_aux_words(int maxlen) { return maxlen / 32 > 2 * kBoundaryCap ? maxlen / 32 : 2 * kBoundaryCap; }
constexpr int cand_lds_words(int nt, int maxlen, int cap)
{
    return kBins1 + 2 * (nt / 64) + 4 + 16 + 2 * cap + maxlen / 32 + cand_aux_words(maxlen);
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x = max(x, (uint32_t)__shfl_xor((int)x, off));
    return x;
}

// RES: every row of the launch has at most 16 vectors per thread, and all of them are requested before anything is
// waited for (the row sits in registers while the sample is worked on).  Used by the half-size instance, where it
// is worth 4 % of a strip; for the 64K-key rows of a decode step it changed nothing (their sweep is bound by the
// vector ALU of the one CU a row has, not by the loads).
template <int NT, int MAXLEN, int CAP, bool RES>
__global__ __launch_bounds__(NT) void select_cand_kernel(SelectArgs a)
{
    static_assert(kCandSample % (4 * NT) == 0 && (MAXLEN / 32) % NT == 0, "whole sample vectors and bitmap words per thread");
    constexpr int NW = NT / 64;
    constexpr int SV = kCandSample / (4 * NT); // sample vectors per thread
    constexpr int BW = MAXLEN / 32 / NT;       // bitmap words per thread
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    uint32_t *hist = smem;                     // [kBins1]  (the generic form's layout starts the same way)
    uint32_t *wsum = hist + kBins1;            // [2 NW]
    uint32_t *bc = wsum + 2 * NW;              // [4]
    uint32_t *misc = bc + 4;                   // [16]: 0 candidate count, 1 largest candidate key, 2 boundary-list count, 3 a list overflowed
    uint32_t *ckey = misc + 16;                // [CAP]
    uint32_t *cpos = ckey + CAP;               // [CAP]
    uint32_t *bitmap = cpos + CAP;             // [MAXLEN / 32]
    uint32_t *wpre = bitmap + MAXLEN / 32;     // [max(MAXLEN / 32, 2 kBoundaryCap)] selected entries ahead of each bitmap
                                               // word; before that: the boundary bin's members (key, position)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = blockIdx.x;
    const int b = a.b0 + r / a.Ri;
    const int i = a.i0 + r % a.Ri;
    if (i >= a.Tq) return;
    const int Lk_b = a.seq_lens ? max(0, min(a.seq_lens[b], a.Lk)) : a.Lk;
    int64_t nv64 = (a.seq_lens ? (int64_t)Lk_b - a.Tq : a.q_pos0) + (int64_t)i + 1;
    nv64 = nv64 < 0 ? 0 : (nv64 > Lk_b ? Lk_b : nv64);
    const int nv = (int)nv64;
    // The candidate form proper; false = this row takes the generic form (one call site below: a fallback reached
    // through several calls is not inlined, and a kernel argument captured by a real function is copied to scratch
    // memory by every thread of every row).
    auto candidate_form = [&]() -> bool {
    if (nv < kCandMinLen || nv < 4 * a.k_sel || nv > MAXLEN) return false;   // workgroup-uniform
    if (RES && nv > 16 * 4 * NT) return false;
    const float *row = a.strip + (int64_t)r * a.ld;
    int32_t *oidx = a.idx + ((int64_t)b * a.Tq + i) * a.k_sel;
    float *osel = a.sel ? a.sel + ((int64_t)b * a.Tq + i) * a.k_sel : nullptr;
    const uint32_t k = (uint32_t)a.k_sel;

    // The row arrives in groups of kGroup vectors per thread, two groups in flight: a single workgroup has to
    // cover the whole memory latency by itself.  The sample and the first group are requested before anything else.
    constexpr int kGroup = 4;
    constexpr int WCAP = CAP / NW;             // every wave keeps its candidates in a list of its own
    const int nsteps = (nv + 4 * NT - 1) / (4 * NT);
    auto load_group = [&](int c0, f32x4 (&dst)[kGroup]) {
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            const int p = ((c0 + j) * NT + tid) * 4;
            dst[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (p < nv) dst[j] = *(const f32x4 *)(row + p);   // may run past nv inside the row's padding; masked below
        }
    };
    constexpr int NG = RES ? 4 : 2;
    f32x4 rv[NG][kGroup];
    f32x4 (&ga)[kGroup] = rv[0], (&gb)[kGroup] = rv[1];
    f32x4 sv[SV];
#pragma unroll
    for (int u = 0; u < SV; ++u) {
        const int blk = (tid >> 5) + (NT / 32) * u;
        const int p = (int)(((int64_t)blk * nv / 32) & ~(int64_t)3) + (tid & 31) * 4;   // p + 3 < nv: blocks are nv / 32 >= 256 apart
        sv[u] = *(const f32x4 *)(row + p);
    }
    if constexpr (RES) {
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) load_group(gi * kGroup, rv[gi]);
    } else {
        load_group(0, ga);
    }

    // ---- sample: 32 blocks of 128 keys, a histogram of 4096 linear bins between the smallest and the largest of
    //      them (the scores of a row share a few exponents: bins of a key digit would be hit a hundred times each,
    //      and LDS atomics on one address take turns) ----
    for (int e = tid; e < kBins1; e += NT) hist[e] = 0;
#pragma unroll
    for (int q = 0; q < BW; ++q) bitmap[BW * tid + q] = 0;
    if (tid < 16) misc[tid] = 0;
    uint32_t skey[4 * SV];
    uint32_t kmx = 0u, kmn = 0xFFFFFFFFu;
#pragma unroll
    for (int e = 0; e < 4 * SV; ++e) {
        skey[e] = score_key(sv[e >> 2][e & 3]);
        kmx = max(kmx, skey[e]);
        kmn = min(kmn, skey[e]);
    }
    {
        const uint32_t mx = wave_max_u32(kmx);
        const uint32_t mn = ~wave_max_u32(~kmn);
        if (lane == 0) {                       // (wpre is free until the boundary list is built)
            wpre[wave] = mn;
            wpre[NW + wave] = mx;
        }
    }
    __syncthreads();
    const uint32_t smin = ~wave_max_u32(~(lane < NW ? wpre[lane] : 0xFFFFFFFFu));
    const uint32_t smax = wave_max_u32(lane < NW ? wpre[NW + lane] : 0u);
    const uint32_t srange = smax - smin;
    const int sbits = srange ? 32 - __clz((int)srange) : 0;
    const int ssh = sbits > 12 ? sbits - 12 : 0;
#pragma unroll
    for (int e = 0; e < 4 * SV; ++e) atomicAdd(&hist[(skey[e] - smin) >> ssh], 1u);
    __syncthreads();
    uint32_t want = (uint32_t)(((int64_t)kCandSample * 2 * k) / nv) + 32u;
    want = want > (uint32_t)kCandSample ? (uint32_t)kCandSample : want;
    find_digit<NT, kBins1 / NT>(hist, want, wsum, bc, tid, lane, wave);
    const uint32_t T0 = smin + (bc[0] << ssh); // a bin's lower edge: at least `want` sampled keys reach it
    __syncthreads();

    // ---- sweep: the row once, the positions of the candidates to the wave's list ----
    // The sweep is bound by vector-ALU instructions (sixteen keys per thread and group), so it does the least per
    // key: one float comparison against the threshold (the key order is the float order) into a bit mask; only the
    // set bits are visited afterwards, and only positions are stored -- the few candidates' keys are read back
    // from the row (still in L2) once the sweep is over.
    uint32_t my_cnt = 0;                       // entries in this wave's list (uniform)
    uint32_t *wkey = ckey + wave * WCAP, *wpos = cpos + wave * WCAP;
    // (rows of up to 65536 keys: a workgroup's row is still in L2 when its candidates are read back; longer rows of
    // a full grid push one another out, there the keys are stored during the sweep)
    const bool reread = nv <= 65536;           // workgroup-uniform
    {
        const float T0f = key_score(T0);
        auto sweep_group = [&](int c0, const f32x4 (&v)[kGroup]) {
            uint32_t m = 0;
#pragma unroll
            for (int j = 0; j < kGroup; ++j) {
                const int p = ((c0 + j) * NT + tid) * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e) m |= (uint32_t)((int)(p + e < nv) & (int)(v[j][e] >= T0f)) << (4 * j + e);
            }
            const uint32_t n_t = (uint32_t)__popc(m);
            const uint32_t incl = wave_incl_scan(n_t);
            const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            if (total == 0u) return;               // wave-uniform
            uint32_t off = my_cnt + incl - n_t;
            my_cnt += total;
            if (reread) {
                while (m) {
                    const int bit = __builtin_ctz(m);
                    m &= m - 1u;
                    if (off < (uint32_t)WCAP) wpos[off] = (uint32_t)(((c0 + (bit >> 2)) * NT + tid) * 4 + (bit & 3));
                    ++off;
                }
            } else {
#pragma unroll
                for (int j = 0; j < kGroup; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if ((m >> (4 * j + e)) & 1u) {
                            if (off < (uint32_t)WCAP) {
                                wpos[off] = (uint32_t)(((c0 + j) * NT + tid) * 4 + e);
                                wkey[off] = max(score_key(v[j][e]), T0);
                            }
                            ++off;
                        }
            }
        };
        if constexpr (RES) {
#pragma unroll
            for (int gi = 0; gi < NG; ++gi)
                if (gi * kGroup < nsteps) sweep_group(gi * kGroup, rv[gi]);
        } else {
#pragma unroll 1
            for (int c0 = 0; c0 < nsteps; c0 += 2 * kGroup) {
                if (c0 + kGroup < nsteps) load_group(c0 + kGroup, gb);
                sweep_group(c0, ga);
                if (c0 + kGroup >= nsteps) break;
                if (c0 + 2 * kGroup < nsteps) load_group(c0 + 2 * kGroup, ga);
                sweep_group(c0 + kGroup, gb);
            }
        }
        if (lane == 0) {
            atomicAdd(&misc[0], my_cnt);
            if (my_cnt > (uint32_t)WCAP) misc[3] = 1u;     // this wave's list overflowed
        }
    }
    __syncthreads();
    const uint32_t n_cand = misc[0];
    if (n_cand < k || misc[3] != 0u) {             // workgroup-uniform
        __syncthreads();
        return false;
    }
    // the candidates' keys and their maximum
    {
        uint32_t tmax = 0;
        for (uint32_t j = lane; j < my_cnt; j += 64) {
            uint32_t key;
            if (reread) {
                key = max(score_key(row[wpos[j]]), T0);   // (>= T0 by construction; the bins below rely on it)
                wkey[j] = key;
            } else {
                key = wkey[j];
            }
            tmax = max(tmax, key);
        }
        tmax = wave_max_u32(tmax);
        if (lane == 0 && tmax != 0u) atomicMax(&misc[1], tmax);
    }

    // ---- one histogram over the candidates: 4096 linear bins over [T0, kmax] ----
    for (int e = tid; e < kBins1; e += NT) hist[e] = 0;
    __syncthreads();
    const uint32_t kmax = misc[1];
    const uint32_t range = kmax - T0;
    const int nbits = range ? 32 - __clz((int)range) : 0;
    const int sh = nbits > 12 ? nbits - 12 : 0;
    for (uint32_t j = lane; j < my_cnt; j += 64) atomicAdd(&hist[(wkey[j] - T0) >> sh], 1u);
    __syncthreads();
    find_digit<NT, kBins1 / NT>(hist, k, wsum, bc, tid, lane, wave);
    const uint32_t bstar = bc[0], need = bc[1], n_b = bc[2];
    __syncthreads();
    const bool ranked = need < n_b;            // the boundary bin is cut: rank its members exactly
    if (ranked && n_b > (uint32_t)kBoundaryCap) return false;

    // ---- mark the selected positions ----
    uint32_t *bl_key = wpre, *bl_pos = wpre + kBoundaryCap;
    for (uint32_t j = lane; j < my_cnt; j += 64) {
        const uint32_t bin = (wkey[j] - T0) >> sh;
        if (bin > bstar || (bin == bstar && !ranked)) {
            atomicOr(&bitmap[wpos[j] >> 5], 1u << (wpos[j] & 31u));
        } else if (bin == bstar) {
            const uint32_t s = atomicAdd(&misc[2], 1u);
            bl_key[s] = wkey[j];
            bl_pos[s] = wpos[j];
        }
    }
    __syncthreads();
    if (ranked) {
        for (uint32_t m = tid; m < n_b; m += NT) {
            const uint32_t km = bl_key[m], pm = bl_pos[m];
            uint32_t ahead = 0;                // members that beat this one: larger key, or equal key at a lower position
            for (uint32_t x = 0; x < n_b; ++x) ahead += (bl_key[x] > km || (bl_key[x] == km && bl_pos[x] < pm)) ? 1u : 0u;
            if (ahead < need) atomicOr(&bitmap[pm >> 5], 1u << (pm & 31u));
        }
        __syncthreads();
    }

    // ---- slots: selected entries ahead of every bitmap word ----
    {
        uint32_t wcnt[BW], mine = 0;
#pragma unroll
        for (int q = 0; q < BW; ++q) {
            wcnt[q] = (uint32_t)__popc(bitmap[BW * tid + q]);
            mine += wcnt[q];
        }
        const uint32_t incl = wave_incl_scan(mine);
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();                       // also: every read of the boundary list is over, wpre may be overwritten
        uint32_t before = 0;
#pragma unroll
        for (int wv = 0; wv < NW; ++wv)
            if (wv < wave) before += wsum[wv];
        uint32_t run = before + incl - mine;
#pragma unroll
        for (int q = 0; q < BW; ++q) {
            wpre[BW * tid + q] = run;
            run += wcnt[q];
        }
    }
    __syncthreads();
    for (uint32_t j = lane; j < my_cnt; j += 64) {
        const uint32_t pos = wpos[j], word = bitmap[pos >> 5], bit = pos & 31u;
        if ((word >> bit) & 1u) {
            const uint32_t slot = wpre[pos >> 5] + (uint32_t)__popc(word & ((1u << bit) - 1u));
            if (slot < k) {                    // always true for a consistent select
                oidx[slot] = (int32_t)pos;
                if (osel) osel[slot] = key_score(wkey[j]);
            }
        }
    }
    return true;
    };
    if (!candidate_form()) {
        SelectArgs ga = a;
        // the candidate arrays' space serves as the row cache (rows that do not fit it are streamed)
        constexpr int kSpace = 16 + 2 * CAP + MAXLEN / 32 + cand_aux_words(MAXLEN);
        ga.cache_elems = kSpace >= 32768 ? 32768 : kSpace / 64 * 64;
        select_row_generic<NT>(ga, smem);
    }
}

size_t select_lds_bytes(int cache_elems)
{
    return (size_t)(kBins1 + 2 * 16 + 4 + cache_elems) * sizeof(uint32_t);
}

} // namespace

int select_cache_limit() { return 32768; }

hipError_t launch_select(const SelectArgs &a_in, int n_rows, int max_row_len, hipStream_t st)
{
    if (n_rows <= 0) return hipSuccess;
    SelectArgs a = a_in;
    int cache = max_row_len <= select_cache_limit() ? (max_row_len + 63) / 64 * 64 : 0;
    if (max_row_len <= a.k_sel) cache = 0;     // short rows never reach the radix path
    a.cache_elems = cache;
    const size_t lds = select_lds_bytes(cache);
    // opt in once per process to the largest LDS footprint either cached variant can ask for
    static hipError_t attr256 = hipFuncSetAttribute((const void *)select_kernel<256>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                                    (int)select_lds_bytes(8192));
    static hipError_t attr1024 = hipFuncSetAttribute((const void *)select_kernel<1024>,
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     (int)select_lds_bytes(select_cache_limit()));
    if (attr256 != hipSuccess) return attr256;
    if (attr1024 != hipSuccess) return attr1024;
    constexpr int lds_big = cand_lds_words(1024, kCandMaxLen, kCandCap) * (int)sizeof(uint32_t);
    constexpr int lds_small = cand_lds_words(512, kCandSmallLen, kCandSmallCap) * (int)sizeof(uint32_t);
    static hipError_t attr_cand = hipFuncSetAttribute((const void *)select_cand_kernel<1024, kCandMaxLen, kCandCap, false>,
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds_big);
    static hipError_t attr_cand_s = hipFuncSetAttribute((const void *)select_cand_kernel<512, kCandSmallLen, kCandSmallCap, true>,
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, lds_small);
    if (attr_cand != hipSuccess) return attr_cand;
    if (attr_cand_s != hipSuccess) return attr_cand_s;
    if (max_row_len > kCandFrom && max_row_len <= kCandMaxLen && max_row_len >= 4 * a.k_sel) {
        // one read of the row, a sampled threshold and a candidate list (falls back row by row)
        if (max_row_len <= kCandSmallLen)
            hipLaunchKernelGGL((select_cand_kernel<512, kCandSmallLen, kCandSmallCap, true>), dim3((unsigned)n_rows), dim3(512), lds_small, st, a);
        else
            hipLaunchKernelGGL((select_cand_kernel<1024, kCandMaxLen, kCandCap, false>), dim3((unsigned)n_rows), dim3(1024), lds_big, st, a);
        return hipGetLastError();
    }
    if (max_row_len <= 8192)
        hipLaunchKernelGGL((select_kernel<256>), dim3((unsigned)n_rows), dim3(256), lds, st, a);
    else
        // rows up to the cache limit stay in LDS after one read; longer ones (beyond the candidate form's range, or
        // with k above a quarter of the row) are streamed on every sweep
        hipLaunchKernelGGL((select_kernel<1024>), dim3((unsigned)n_rows), dim3(1024), lds, st, a);
    return hipGetLastError();
}

} // namespace ic
