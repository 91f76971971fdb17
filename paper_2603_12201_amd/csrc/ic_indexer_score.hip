// Lightning-indexer score kernel for gfx950 (CDNA4).
//
//   I[t,s] = sum_j w[t,j] * ReLU( q[t,j,:] . k[s,:] )        (paper Sec. 2.1, Sec. 3 Notation)
//
// Mapping.  The contraction runs on v_mfma_f32_32x32x16_bf16 with the indexer HEADS of one
// query token as the 32 rows of the A operand and 32 KEYS as the columns of the B operand,
// so one accumulator tile holds dot(q[t,j], k[s]) for 32 heads x 32 keys.  In that result
// layout a lane owns one key column and 16 of the 32 head rows: the ReLU, the weighting by
// w[t,j] and the sum over heads are 16 in-lane max/fma pairs plus one exchange between the
// two half-waves.  The q rows of the tokens a wave owns stay in registers for the whole key
// loop; key tiles (64 keys) are staged through LDS, double buffered, one barrier per tile,
// and shared by the four waves of the workgroup (each wave owns TPW tokens).
//
// Occupancy.  A wave cannot overlap its own MFMAs with its own VALU epilogue (both issue through
// the same port), and the epilogue costs about as many cycles as the MFMAs.  Two workgroups per
// CU (two waves per SIMD, <= 256 registers each) let one wave's epilogue run under the other's
// MFMAs; that caps a wave at 3 tokens (96 q + 48 w registers), which still reuses every B
// operand read from LDS three times (LDS return bandwidth, ~64 B/clk/CU, is the next limit).
//
// The kernel writes scores of the query rows in flight into a strip (rows x Lk fp32); it
// never holds more rows than the caller's workspace allows.  Keys hidden by the causal mask
// are not written.
#include "ic_common.hpp"

namespace ic {

namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;

// The two operand formats.  bf16: v_mfma_f32_32x32x16_bf16, 16 contraction elements per step,
// a lane holds 8 of them (16 bytes).  fp8 (OCP e4m3): v_mfma_f32_32x32x64_f8f6f4, 64 elements per
// step, a lane holds 32 of them (32 bytes) -- twice the matrix rate per instruction cycle.
template <bool FP8> struct Fmt;
template <> struct Fmt<false> {
    typedef bf16x8 Op;
    static constexpr int kStep = 16, kElemBytes = 2;
    static __device__ __forceinline__ Op load(const unsigned char *p) { return *(const Op *)p; }
    static __device__ __forceinline__ Op zero() { return __builtin_bit_cast(Op, u32x4{0u, 0u, 0u, 0u}); }
    static __device__ __forceinline__ f32x16 mma(Op x, Op y, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, c, 0, 0, 0);
    }
};
template <> struct Fmt<true> {
    typedef i32x8 Op;
    static constexpr int kStep = 64, kElemBytes = 1;
    static __device__ __forceinline__ Op load(const unsigned char *p)
    {
        const u32x4 lo = *(const u32x4 *)p, hi = *(const u32x4 *)(p + 16);
        return Op{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
    }
    static __device__ __forceinline__ Op zero() { return Op{0, 0, 0, 0, 0, 0, 0, 0}; }
    static __device__ __forceinline__ f32x16 mma(Op x, Op y, f32x16 c)
    {
        // formats 0/0 = e4m3 x e4m3; constant zero scale operands select the unscaled instruction
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(x, y, c, 0, 0, 0, 0, 0, 0);
    }
};

// Global -> register -> LDS staging of one tile of 64 key rows (16-byte chunks, coalesced).
// RB = bytes per key row.
// tile: address of the tile's first key row; rows_valid >= 1 of its 64 rows exist.
template <int RB, int LPT, int NT>
__device__ __forceinline__ void tile_gload(u32x4 (&pre)[LPT], const unsigned char *tile, int rows_valid, int tid)
{
    constexpr int CPR = RB / 16;
#pragma unroll
    for (int r = 0; r < LPT; ++r) {
        const int c = tid + NT * r;
        const int row = c / CPR, col = c % CPR;
        const int s = min(row, rows_valid - 1);             // clamp: rows past the end are masked later
        pre[r] = *(const u32x4 *)(tile + (s * RB + col * 16));
    }
}

template <int RB, int LPT, int ROWB, int NT>
__device__ __forceinline__ void tile_lstore(const u32x4 (&pre)[LPT], unsigned char *buf, int tid)
{
    constexpr int CPR = RB / 16;
#pragma unroll
    for (int r = 0; r < LPT; ++r) {
        const int c = tid + NT * r;
        const int row = c / CPR, col = c % CPR;
        *(u32x4 *)(buf + row * ROWB + col * 16) = pre[r];
    }
}

// ReLU on the bit pattern: a non-positive float (including -0) is a non-positive integer.
__device__ __forceinline__ float relu(float x)
{
    const int xi = __float_as_int(x);
    return __int_as_float(xi > 0 ? xi : 0);
}

// STREAM = true is the few-query-rows form (decode): the workgroup owns ONE token, every wave
// keeps its q rows, and the waves take turns on the key subtiles (wave w multiplies subtile
// w & 1 of the tiles with parity w >> 1) so that all four SIMDs share the little matrix work
// while the kernel streams the key cache.
// PG: the key cache may be ragged and / or paged (a.pv); false compiles the dense layout only.
template <int HT, int DI, int TPW, int NW, int PD, int MINB, bool STREAM, bool FP8, bool PG>
__global__ __launch_bounds__(64 * NW, MINB) void score_kernel(ScoreArgs a)
{
    static_assert(!STREAM || (TPW == 1 && NW == 4), "the streaming form is one token, four waves");
    typedef Fmt<FP8> F;
    typedef typename F::Op Op;
    constexpr int NT = 64 * NW;                 // threads per workgroup
    constexpr int KS = DI / F::kStep;           // MFMA k-steps over the head dim
    constexpr int OPB = F::kStep / 2 * F::kElemBytes;   // operand bytes per lane per k-step
    constexpr int BT = STREAM ? 1 : NW * TPW;   // tokens per workgroup
    constexpr int RB = DI * F::kElemBytes;      // bytes per key row
    constexpr int ROWB = RB + 16;               // LDS row stride (bytes), padded against bank conflicts
    constexpr int TILE = 64;                    // keys per LDS tile
    constexpr int CPR = RB / 16;                // 16-byte chunks per key row
    constexpr int LPT = (TILE * CPR + NT - 1) / NT;     // 16-byte loads per thread per tile
    static_assert(TILE * CPR % NT == 0, "tile chunks must divide evenly over the threads");
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][TILE * ROWB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, half = lane >> 5;
    const int qb = a.n_qblocks - 1 - (int)blockIdx.x;      // longest rows first
    const int b = a.b0 + (int)blockIdx.z;
    const int i_end = min(a.i0 + a.Ri, a.Tq);
    const int t_blk = a.i0 + qb * BT;
    if (t_blk >= i_end) return;
    const int t_blk_last = min(t_blk + BT, i_end) - 1;
    // ragged cache: this sequence holds Lk_b keys and its Tq query rows are its last Tq positions
    const bool ragged = PG && a.pv.seq_lens, paged = PG && a.pv.page_table;
    const int Lk_b = ragged ? max(0, min(a.pv.seq_lens[b], a.Lk)) : a.Lk;
    const int64_t q_pos0 = ragged ? (int64_t)Lk_b - a.Tq : a.q_pos0;

    int64_t vis64 = q_pos0 + (int64_t)t_blk_last + 1;      // keys visible to the block's last token
    vis64 = vis64 < 0 ? 0 : (vis64 > Lk_b ? Lk_b : vis64);
    const int kc0 = (int)blockIdx.y * a.KC;
    const int kend = min(kc0 + a.KC, (int)vis64);
    if (kc0 >= kend) return;                               // whole workgroup: nothing visible here

    const int t_w0 = STREAM ? t_blk : t_blk + wave * TPW;  // this wave's first token
    int64_t wv64 = q_pos0 + (int64_t)min(t_w0 + TPW, i_end);
    wv64 = wv64 < 0 ? 0 : (wv64 > Lk_b ? Lk_b : wv64);
    const int wave_vis = (t_w0 < i_end) ? (int)wv64 : 0;   // keys >= wave_vis matter to none of its tokens

    // ---- stationary operands: q rows (A operand) and head weights of the wave's tokens ----
    Op qa[TPW][HT][KS];
    float wr[TPW][HT][16];
    float sqr[TPW];                                        // fp8: per-token scale of q
    const unsigned char *qp = (const unsigned char *)a.q;
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        const int t = t_w0 + j;
        const bool tv = t < i_end;
        const int64_t trow = (int64_t)b * a.Tq + (tv ? t : 0);
        sqr[j] = (FP8 && tv) ? a.q_scale[trow] : 1.f;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            const int head = ht * 32 + r32;
            const bool hv = tv && head < a.H_I;
            const unsigned char *src = qp + ((trow * a.H_I + (hv ? head : 0)) * DI) * F::kElemBytes + half * OPB;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                qa[j][ht][ks] = F::zero();
                if (hv) qa[j][ht][ks] = F::load(src + ks * 2 * OPB);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int hrow = ht * 32 + 8 * (i / 4) + 4 * half + (i % 4);
                wr[j][ht][i] = (tv && hrow < a.H_I) ? a.w[trow * a.H_I + hrow] : 0.f;
            }
        }
    }

    // ---- key tile pipeline: global -> registers -> LDS, double buffered, one barrier per tile ----
    const unsigned char *kp = (const unsigned char *)a.k + (paged ? 0 : (int64_t)b * a.Lk * RB);
    const float *ksc = FP8 ? a.k_scale + (int64_t)b * a.Lk : nullptr;
    // first row of the 64-key tile at kt (tiles never straddle a page: pages hold a multiple of 64 positions)
    auto tile_ptr = [&](int kt) -> const unsigned char * {
        return kp + (paged ? paged_row(a.pv, b, kt) : (int64_t)kt) * RB;
    };
    // PD register sets keep PD tiles in flight from HBM/L2 (set t % PD holds tile t); a tile is
    // copied to LDS one iteration before it is multiplied.
    u32x4 pre[PD][LPT];
    const int ntiles = (kend - kc0 + TILE - 1) / TILE;
    tile_gload<RB, LPT, NT>(pre[0], tile_ptr(kc0), Lk_b - kc0, tid);
#pragma unroll
    for (int d = 1; d < PD; ++d)
        if (d < ntiles) tile_gload<RB, LPT, NT>(pre[d], tile_ptr(kc0 + d * TILE), Lk_b - (kc0 + d * TILE), tid);
    tile_lstore<RB, LPT, ROWB, NT>(pre[0], &lds[0][0], tid);
    __syncthreads();

    // Combine the two half-wave partial sums of a token pair (or of one token with itself) and
    // store 32 scores per row.  permlane32_swap(x, y) returns {[x.lo, y.lo], [x.hi, y.hi]}: their
    // sum is token A's total in lanes 0-31 and token B's in lanes 32-63.
    auto emit = [&](float pa, float pb, bool pair, int j, int s0, bool interior) {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(pa), __float_as_uint(pb), false, false);
        float v = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
        const int t = t_w0 + j + half;
        const int s = s0 + r32;
        const bool lane_on = pair || half == 0;
        if (FP8) {
            // positive per-token scales commute with the ReLU gate: I = sq[t] sk[s] sum_j w_j ReLU(q8_j . k8)
            const float sq = (pair && half) ? sqr[(j + 1) % TPW] : sqr[j];
            v *= sq * ksc[min(s, Lk_b - 1)];
        }
        if (lane_on && (interior || (t < i_end && s < Lk_b && (int64_t)s <= q_pos0 + t))) {
            const int64_t srow = (int64_t)blockIdx.z * a.Ri + (t - a.i0);
            a.strip[srow * a.ld + s] = v;
        }
    };

    for (int it0 = 0; it0 < ntiles; it0 += PD) {
#pragma unroll
      for (int ph = 0; ph < PD; ++ph) {
        const int it = it0 + ph;
        if (it >= ntiles) break;                            // workgroup-uniform
        const int kt = kc0 + it * TILE;
        const int buf = it & 1;
        if (it + PD < ntiles) tile_gload<RB, LPT, NT>(pre[ph], tile_ptr(kt + PD * TILE), Lk_b - (kt + PD * TILE), tid);

        // Interior tile: all 64 keys are visible to every token of this wave and every token is a
        // real row, so nothing needs masking and the whole tile is one straight-line block.
        const bool interior = (t_w0 + TPW <= i_end) && (kt + TILE <= Lk_b) &&
                              ((int64_t)(kt + TILE - 1) <= q_pos0 + t_w0);
        if (interior && !STREAM) {
            // Software pipeline over the units (key subtile, token, head tile): the MFMA chain of unit
            // c+1 is issued before the ReLU/weight/sum epilogue of unit c, so the matrix pipe works
            // under this wave's own VALU epilogue as well as under the other wave's.
            Op kb[KS];                                      // B operands of the subtile being multiplied
            auto load_kb = [&](int sub) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    kb[ks] = F::load(&lds[buf][(sub * 32 + r32) * ROWB + (ks * 2 + half) * OPB]);
            };
            constexpr int NCH = 2 * TPW * HT;
            f32x16 acc[2];
            float part[TPW];
            auto chain = [&](int c) -> f32x16 {
                const int x = c / HT, ht = c % HT, j = x % TPW;
                if (c % (TPW * HT) == 0) load_kb(x / TPW);  // first unit of a subtile
                f32x16 r;
#pragma unroll
                for (int i = 0; i < 16; ++i) r[i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    r = F::mma(qa[j][ht][ks], kb[ks], r);
                return r;
            };
            acc[0] = chain(0);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                if (c + 1 < NCH) acc[(c + 1) & 1] = chain(c + 1);
                const int x = c / HT, ht = c % HT, sub = x / TPW, j = x % TPW;
                float s_acc = (ht == 0) ? 0.f : part[j];
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    s_acc = fmaf(relu(acc[c & 1][i]), wr[j][ht][i], s_acc);
                part[j] = s_acc;
                if (ht == HT - 1) {
                    if (j & 1) emit(part[j - 1], part[j], true, j - 1, kt + sub * 32, true);
                    else if (j == TPW - 1) emit(part[j], part[j], false, j, kt + sub * 32, true);
                }
            }
        } else {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const int s0 = kt + sub * 32;
                if (s0 >= wave_vis) continue;               // wave-uniform: hidden from all its tokens
                if (STREAM && (sub != (wave & 1) || (it & 1) != (wave >> 1))) continue;   // another wave's turn
                Op kb[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    kb[ks] = F::load(&lds[buf][(sub * 32 + r32) * ROWB + (ks * 2 + half) * OPB]);
                float part[TPW];
#pragma unroll
                for (int j = 0; j < TPW; ++j) {
                    float s_acc = 0.f;
#pragma unroll
                    for (int ht = 0; ht < HT; ++ht) {
                        f32x16 acc;
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks)
                            acc = F::mma(qa[j][ht][ks], kb[ks], acc);
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            s_acc = fmaf(relu(acc[i]), wr[j][ht][i], s_acc);
                    }
                    part[j] = s_acc;
                }
#pragma unroll
                for (int j = 0; j < TPW; j += 2) {
                    const bool pair = j + 1 < TPW;
                    emit(part[j], pair ? part[j + 1] : part[j], pair, j, s0, false);
                }
            }
        }

        if (it + 1 < ntiles) tile_lstore<RB, LPT, ROWB, NT>(pre[(ph + 1) % PD], &lds[buf ^ 1][0], tid);
        __syncthreads();
      }
    }
}

__global__ void fill_kernel(float *p, int64_t n, float v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

template <int HT, int DI, int TPW, int NW, int PD, int MINB, bool STREAM, bool FP8>
hipError_t launch_t(const ScoreArgs &a, int Bc, int64_t max_vis, hipStream_t st)
{
    const int n_kc = (int)((max_vis + a.KC - 1) / a.KC);
    if (n_kc <= 0 || a.n_qblocks <= 0 || Bc <= 0) return hipSuccess;
    dim3 grid((unsigned)a.n_qblocks, (unsigned)n_kc, (unsigned)Bc);
    if (a.pv.seq_lens || a.pv.page_table)
        hipLaunchKernelGGL((score_kernel<HT, DI, TPW, NW, PD, MINB, STREAM, FP8, true>), grid, dim3(64 * NW), 0, st, a);
    else
        hipLaunchKernelGGL((score_kernel<HT, DI, TPW, NW, PD, MINB, STREAM, FP8, false>), grid, dim3(64 * NW), 0, st, a);
    return hipGetLastError();
}

} // namespace

bool score_shape_supported(int dtype, int H_I, int d_I)
{
    if (H_I < 1 || H_I > IC_MAX_HEADS_I) return false;
    if (dtype == IC_FP8_E4M3) return d_I == 128;
    if (dtype != IC_BF16) return false;
    return d_I == 64 || d_I == 128;
}

hipError_t launch_score(const ScoreArgs &a_in, int dtype, int d_I, int Bc, hipStream_t st)
{
    ScoreArgs a = a_in;
    // Few query rows per sequence (decode, short chunks): one token per workgroup, three workgroups
    // per CU and three key tiles in flight per workgroup, because the kernel then only streams keys.
    // Otherwise 3 tokens per wave (2 for 64 heads) and the matrix pipe is the limit.
    const bool few_rows = a.Ri <= 4;
    const int BT = few_rows ? 1 : (a.H_I <= 32 ? 12 : 8);   // 4 waves x tokens per wave of the chosen form
    a.n_qblocks = (a.Ri + BT - 1) / BT;
    const int i_last = min(a.i0 + a.Ri, a.Tq) - 1;
    int64_t max_vis = a.q_pos0 + i_last + 1;
    max_vis = max_vis < 0 ? 0 : (max_vis > a.Lk ? a.Lk : max_vis);
    if (a.pv.seq_lens) max_vis = a.Lk;          // ragged: the lengths live on the device, Lk is their bound
    if (max_vis == 0) return hipSuccess;
    // keys per workgroup (tiles of 64 keys): prefill wants enough workgroups to fill 256 CUs
    // several times; the streaming variant wants exactly one resident round (3 per CU).
    const int64_t want_wgs = few_rows ? 768 : 2048;
    int64_t kc = (max_vis * a.n_qblocks * Bc / want_wgs + 63) / 64 * 64;
    kc = kc < 512 ? 512 : (kc > 4096 ? 4096 : kc);
    a.KC = (int)kc;
    const bool fp8 = dtype == IC_FP8_E4M3;
    if (!fp8) {
        if (a.H_I <= 32) {
            if (d_I == 128) return few_rows ? launch_t<1, 128, 1, 4, 3, 3, true, false>(a, Bc, max_vis, st) : launch_t<1, 128, 3, 4, 1, 2, false, false>(a, Bc, max_vis, st);
            if (d_I == 64) return few_rows ? launch_t<1, 64, 1, 4, 3, 3, true, false>(a, Bc, max_vis, st) : launch_t<1, 64, 3, 4, 1, 2, false, false>(a, Bc, max_vis, st);
        } else {
            if (d_I == 128) return few_rows ? launch_t<2, 128, 1, 4, 3, 2, true, false>(a, Bc, max_vis, st) : launch_t<2, 128, 2, 4, 1, 1, false, false>(a, Bc, max_vis, st);
            if (d_I == 64) return few_rows ? launch_t<2, 64, 1, 4, 3, 2, true, false>(a, Bc, max_vis, st) : launch_t<2, 64, 2, 4, 1, 1, false, false>(a, Bc, max_vis, st);
        }
    } else {
        if (a.H_I <= 32) {
            if (d_I == 128) return few_rows ? launch_t<1, 128, 1, 4, 3, 3, true, true>(a, Bc, max_vis, st) : launch_t<1, 128, 3, 4, 1, 2, false, true>(a, Bc, max_vis, st);
        } else {
            if (d_I == 128) return few_rows ? launch_t<2, 128, 1, 4, 3, 2, true, true>(a, Bc, max_vis, st) : launch_t<2, 128, 2, 4, 1, 2, false, true>(a, Bc, max_vis, st);
        }
    }
    return hipErrorInvalidValue;
}

hipError_t launch_fill(float *p, int64_t n, float v, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 65535) blocks = 65535;
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

} // namespace ic
