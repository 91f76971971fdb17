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
// Schedule.  A wave's work is a stream of units (32 keys x one token x one head tile): a chain of
// KS MFMAs into a fresh accumulator, then 16 max/fma pairs on the result.  The chain of unit c + 1
// is issued one MFMA at a time between the epilogue steps of unit c, one step ahead so that it ends
// before the epilogue that reads it begins (a scheduling barrier after each MFMA + its share of the
// epilogue pins that order), and the stream runs on across key tiles: the
// first chain of the next tile is issued under the last epilogue of this one.  For that the tile
// hand-over sits in the middle of a tile -- after the wave's last LDS read of the tile the other
// buffer is refilled, and the barrier that publishes it comes two units later, just before the first
// read of the next tile.  Tiles on the causal diagonal or at a ragged end take a plain, checked path.
// Two workgroups per CU (two waves per SIMD, <= 256 registers each) cover what bubbles remain (LDS
// read latency at the start of a subtile, the barrier); that caps a wave at 3 tokens (96 q + 48 w
// registers), which still reuses every B operand read from LDS three times.
// fp8 halves the MFMA time per unit but not the 32 VALU operations of its epilogue, so that form is
// bound by VALU issue at about half of the fp8 matrix peak.
//
// The kernel writes scores of the query rows in flight into a strip (rows x Lk fp32); it
// never holds more rows than the caller's workspace allows.  Keys hidden by the causal mask
// are not written.
#include "ic_common.hpp"

#include <type_traits>

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
    static_assert(NT % CPR == 0, "a thread keeps its chunk column over the tile");
    unsigned char *p = buf + (tid / CPR) * ROWB + (tid % CPR) * 16;
#pragma unroll
    for (int r = 0; r < LPT; ++r) *(u32x4 *)(p + r * (NT / CPR) * ROWB) = pre[r];
}

// The same load for a tile whose 64 rows all exist: one lane offset, constant strides.
template <int LPT, int NT>
__device__ __forceinline__ void tile_gload_full(u32x4 (&pre)[LPT], const unsigned char *tile, int tid)
{
    const unsigned off = (unsigned)tid * 16u;
#pragma unroll
    for (int r = 0; r < LPT; ++r) pre[r] = *(const u32x4 *)(tile + r * NT * 16 + off);
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
    __shared__ float lds_ks[2][TILE];                       // fp8: the key scales of the two tiles

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
    if (FP8 && !STREAM) lds_ks[0][lane] = ksc[min(kc0 + lane, Lk_b - 1)];
    __syncthreads();

    // Combine the two half-wave partial sums of a token pair (or of one token with itself) and
    // store 32 scores per row.  permlane32_swap(x, y) returns {[x.lo, y.lo], [x.hi, y.hi]}: their
    // sum is token A's total in lanes 0-31 and token B's in lanes 32-63.
    auto emit = [&](float pa, float pb, bool pair, int j, int s0, int r32_x, int half_x) {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(pa), __float_as_uint(pb), false, false);
        float v = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
        const int t = t_w0 + j + half_x;
        const int s = s0 + r32_x;
        const bool lane_on = pair || half_x == 0;
        if (FP8) {
            // positive per-token scales commute with the ReLU gate: I = sq[t] sk[s] sum_j w_j ReLU(q8_j . k8)
            const float sq = (pair && half_x) ? sqr[(j + 1) % TPW] : sqr[j];
            v *= sq * ksc[min(s, Lk_b - 1)];
        }
        if (lane_on && t < i_end && s < Lk_b && (int64_t)s <= q_pos0 + t) {
            const int64_t srow = (int64_t)blockIdx.z * a.Ri + (t - a.i0);
            a.strip[srow * a.ld + s] = v;
        }
    };

    if constexpr (STREAM) {
        for (int it0 = 0; it0 < ntiles; it0 += PD) {
#pragma unroll
          for (int ph = 0; ph < PD; ++ph) {
            const int it = it0 + ph;
            if (it >= ntiles) break;                        // workgroup-uniform
            const int kt = kc0 + it * TILE;
            const int buf = it & 1;
            if (it + PD < ntiles) tile_gload<RB, LPT, NT>(pre[ph], tile_ptr(kt + PD * TILE), Lk_b - (kt + PD * TILE), tid);
            const int sub = wave & 1;                       // this wave's subtile; tiles alternate between wave pairs
            const int s0 = kt + sub * 32;
            if (s0 < wave_vis && (it & 1) == (wave >> 1)) {
                Op kb[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    kb[ks] = F::load(&lds[buf][(sub * 32 + r32) * ROWB + (ks * 2 + half) * OPB]);
                float s_acc = 0.f;
#pragma unroll
                for (int ht = 0; ht < HT; ++ht) {
                    f32x16 acc;
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        acc = F::mma(qa[0][ht][ks], kb[ks], acc);
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        s_acc = fmaf(relu(acc[i]), wr[0][ht][i], s_acc);
                }
                emit(s_acc, s_acc, false, 0, s0, r32, half);
            }
            if (it + 1 < ntiles) tile_lstore<RB, LPT, ROWB, NT>(pre[(ph + 1) % PD], &lds[buf ^ 1][0], tid);
            __syncthreads();
          }
        }
    } else {
        static_assert(STREAM || PD == 1, "the tiled form keeps one key tile in flight");
        static_assert(16 % KS == 0, "epilogue elements per MFMA step");
        constexpr int NCH = 2 * TPW * HT;                   // units (key subtile, token, head tile) per key tile
        constexpr int HALF = TPW * HT;                      // units per key subtile
        constexpr int EPC = 16 / KS;                        // epilogue elements that ride under one MFMA
        constexpr int LEAD = 1;

        // Leading tiles in which all 64 keys are visible to every token of this wave and every token is
        // a real row: nothing needs masking there.  The remaining tiles (the causal diagonal, a ragged
        // end) take the checked path.
        int n_int = 0;
        if (t_w0 + TPW <= i_end) {
            const int64_t lim = min((int64_t)Lk_b, q_pos0 + t_w0 + 1);
            const int64_t n = (lim - kc0) / TILE;
            n_int = (int)(n < 0 ? 0 : (n > ntiles ? ntiles : n));
        }

        float pre_s = 1.f;                                  // fp8: a key scale of the tile in flight
        if (FP8 && ntiles > 1) pre_s = ksc[min(kc0 + TILE + lane, Lk_b - 1)];
        // Hand-over of a tile: once every LDS read of tile `it` has been issued by this wave, the other
        // buffer (last read for tile it - 1, before the previous barrier) takes tile it + 1 and the
        // registers take tile it + 2.  The barrier that publishes the buffer follows later in the tile,
        // before the first read of tile it + 1, so the four waves rarely wait for one another.
        auto stage = [&](int it, int tid_x, auto steady_c) {
            if (decltype(steady_c)::value) {
                // tile it + 1 follows for certain and tile it + 2, if there is one, has all its 64 rows;
                // past the end the load repeats tile it + 1 instead of being skipped, which keeps the
                // steady-state loop body free of branches
                tile_lstore<RB, LPT, ROWB, NT>(pre[0], &lds[(it + 1) & 1][0], tid_x);
                if (FP8) lds_ks[(it + 1) & 1][tid_x & 63] = pre_s;
                const int kn = kc0 + (it + 2 < ntiles ? it + 2 : it + 1) * TILE;
                if (FP8) pre_s = ksc[kn + (tid_x & 63)];
                tile_gload_full<LPT, NT>(pre[0], tile_ptr(kn), tid_x);
            } else {
                if (it + 1 < ntiles) tile_lstore<RB, LPT, ROWB, NT>(pre[0], &lds[(it + 1) & 1][0], tid_x);
                if (it + 2 < ntiles) {
                    const int kn = kc0 + (it + 2) * TILE;
                    tile_gload<RB, LPT, NT>(pre[0], tile_ptr(kn), Lk_b - kn, tid_x);
                }
            }
        };
        if (ntiles > 1) tile_gload<RB, LPT, NT>(pre[0], tile_ptr(kc0 + TILE), Lk_b - (kc0 + TILE), tid);

        // fp8: the 64 key scales of a tile travel with the tile (register -> lds_ks at the hand-over, every
        // wave writing the same values) and are read back at the start of the tile (ks0 / ks1: the lane's
        // key in either subtile); the query scales of a lane's two possible rows are folded into one
        // value per emit (sq_l0: tokens 0 / 1, sq_l1: tokens 2 / 3)
        static_assert(TPW <= 4, "two emits per key subtile at most");
        float ks0 = 1.f, ks1 = 1.f;
        const float sq_l0 = (half && TPW > 1) ? sqr[1 % TPW] : sqr[0];
        const float sq_l1 = (half && TPW > 3) ? sqr[3 % TPW] : sqr[2 % TPW];
        // Unmasked store of two 32-score runs of tile kt: lanes 0-31 write token ja at the keys of subtile
        // suba, lanes 32-63 token jb at those of subtile subb (pa / pb: the half-wave partial sums of the
        // two runs; sc: the lane's fp8 scale product).
        float *const srow0 = a.strip + ((int64_t)blockIdx.z * a.Ri + (t_w0 - a.i0)) * a.ld + r32;
        auto emit_full = [&](float pa, float pb, int ja, int suba, int jb, int subb, int kt, float sc) {
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(pa), __float_as_uint(pb), false, false);
            float v = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
            const int j = half ? jb : ja, s = kt + 32 * (half ? subb : suba);
            if (FP8) v *= sc;
            srow0[(int64_t)j * a.ld + s] = v;
        };

        Op kb[KS];
        f32x16 acc[2];
        float part[TPW];
        float held = 0.f;                                   // odd TPW: the last token's sum over subtile 0
        auto load_kb = [&](int buf, int sub) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kb[ks] = F::load(&lds[buf][(sub * 32 + r32) * ROWB + (ks * 2 + half) * OPB]);
        };
        auto mma_step = [&](int u, int ks) {                // MFMA ks of unit u's chain
            const int x = u / HT, ht = u % HT, j = x % TPW;
            f32x16 c0;
#pragma unroll
            for (int i = 0; i < 16; ++i) c0[i] = 0.f;
            acc[u & 1] = F::mma(qa[j][ht][ks], kb[ks], ks == 0 ? c0 : acc[u & 1]);
        };
        // One interior tile, software pipelined over its units and into the next tile: the MFMA chain of
        // unit c + 1 is issued one instruction at a time between the ReLU/weight/sum steps of unit c, so
        // the matrix pipe never waits for this wave's VALU work.  On entry the chain of unit 0 is in
        // flight and kb holds subtile 0; NEXT: another interior tile follows.
        auto tile_body = [&](const int it, const int tid_x, auto next_c) {
            constexpr bool NEXT = decltype(next_c)::value;
            const int kt = kc0 + it * TILE, buf = it & 1;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int x = c / HT, ht = c % HT, sub = x / TPW, j = x % TPW;
                if (FP8 && c == 0) {
                    ks0 = lds_ks[buf][r32];
                    ks1 = lds_ks[buf][32 + r32];
                }
                if (c + 1 == HALF) load_kb(buf, 1);
                if (c + 1 == NCH && NEXT) load_kb(buf ^ 1, 0);
                float s_acc = (ht == 0) ? 0.f : part[j];
                // MFMA ks + LEAD of the next chain goes out with epilogue step ks: the chain ends LEAD steps
                // before the epilogue that reads its result begins
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if (c + 1 < NCH || NEXT) {
                        if (ks == 0) {
#pragma unroll
                            for (int m = 0; m < LEAD; ++m) mma_step((c + 1) % NCH, m);
                        }
                        if (ks + LEAD < KS) mma_step((c + 1) % NCH, ks + LEAD);
                    }
#pragma unroll
                    for (int i = ks * EPC; i < (ks + 1) * EPC; ++i)
                        s_acc = fmaf(relu(acc[c & 1][i]), wr[j][ht][i], s_acc);
                    __builtin_amdgcn_sched_barrier(0);
                }
                part[j] = s_acc;
                if (ht == HT - 1) {
                    const float sq = (j / 2 == 0) ? sq_l0 : sq_l1;
                    if (j & 1) emit_full(part[j - 1], part[j], j - 1, sub, j, sub, kt, sq * (sub ? ks1 : ks0));
                    else if (j == TPW - 1) {
                        if (sub == 0) held = part[j];
                        else emit_full(held, part[j], j, 0, j, 1, kt, sq * (half ? ks1 : ks0));
                    }
                }
                if (c + 1 == HALF) stage(it, tid_x, next_c);
                if (c + 2 == NCH) __syncthreads();
            }
        };

        int it = 0;
        if (n_int > 0) {
            load_kb(0, 0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) mma_step(0, ks);
        }
        // steady state: the next tile is interior too and the one after it is not a ragged last tile
        const int n_steady = min(n_int - 1, kc0 + ntiles * TILE <= Lk_b ? ntiles : ntiles - 3);
        for (; it < n_steady; ++it) tile_body(it, tid, std::true_type{});
        // What the remaining tiles need of the lane's position is rebuilt from the thread id behind a
        // compiler barrier, so that none of it occupies registers during the steady-state loop.
        int tid_c = tid;
        asm volatile("" : "+v"(tid_c));
        if (it < n_int) {
            tile_body(it, tid_c, std::false_type{});
            ++it;
        }
        const int r32_c = tid_c & 31, half_c = (tid_c >> 5) & 1;
        for (; it < ntiles; ++it) {
            const int kt = kc0 + it * TILE, buf = it & 1;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const int s0 = kt + sub * 32;
                if (s0 >= wave_vis) continue;               // wave-uniform: hidden from all its tokens
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    kb[ks] = F::load(&lds[buf][(sub * 32 + r32_c) * ROWB + (ks * 2 + half_c) * OPB]);
                float ps[TPW];
#pragma unroll
                for (int j = 0; j < TPW; ++j) {
                    float s_acc = 0.f;
#pragma unroll
                    for (int ht = 0; ht < HT; ++ht) {
                        f32x16 r;
#pragma unroll
                        for (int i = 0; i < 16; ++i) r[i] = 0.f;
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks)
                            r = F::mma(qa[j][ht][ks], kb[ks], r);
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            s_acc = fmaf(relu(r[i]), wr[j][ht][i], s_acc);
                    }
                    ps[j] = s_acc;
                }
#pragma unroll
                for (int j = 0; j < TPW; j += 2) {
                    const bool pair = j + 1 < TPW;
                    emit(ps[j], pair ? ps[j + 1] : ps[j], pair, j, s0, r32_c, half_c);
                }
            }
            stage(it, tid_c, std::false_type{});
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

// ---------------------------------------------------------------------------------------------------------
// Few query rows, bf16, d_I = 128 (decode): the kernel is a stream over the index-key cache, so what matters is
// how the keys travel and in which order the chip walks the cache.
// Travel.  Every wave owns a ring of R slots in LDS (one slot = 32 rows of 256 B = 8 KB) that it fills with loads
// that write LDS directly: 64 lanes x 16 bytes = 1 KB = four whole rows per instruction, no registers, no LDS
// stores, and -- the ring being private to the wave -- no barrier: the wave waits for its own oldest slot with the
// vector-memory counter (loads return in order) and multiplies it while R - 1 slots are in flight.  A lane
// fetches the 16-byte piece (lane & 15) ^ (row & 15) of its row, so that the operand reads (one row per lane, the
// same piece for all lanes) spread over all banks.  The q rows of a token (32 heads x 256 B = one slot per head
// tile) travel through the same ring as items of their own, ahead of the token's keys.
// Order.  Reading the cache as a few wide windows that slide is faster than many narrow streams (measured: 32
// concurrent per-token windows 100 us, 8 windows 90 us, one window 87 us for 537 MB).  So only G tokens are in
// flight, each with the workgroups of one residue mod G (for G = 8 that is one XCD: workgroup ids are dealt
// round-robin over the eight XCDs; the kernel itself is a little faster with G = 16, two tokens per XCD); all waves
// of those workgroups interleave slot by slot over the token's keys, then move to the token G further on together.
// ---------------------------------------------------------------------------------------------------------
__device__ __forceinline__ void dma_lanes(const void *lane_addr, unsigned lds_addr /*uniform*/)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(lane_addr), "s"(lds_addr) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vm_le()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Small read-only operands (head weights, lengths, page table) are read through the constant address space: with a
// uniform address that is a scalar load, which does not enter the vector-memory queue the ring's waits count on.
// (An ordinary load inside the loop would make the compiler wait for "all its loads", i.e. drain the ring.)
template <typename T> __device__ __forceinline__ T load_uniform(const T *p)
{
    return *(const __attribute__((address_space(4))) T *)(uintptr_t)p;
}

template <int HT, int NW, int R, bool PG>
__global__ __launch_bounds__(64 * NW, 1) void score_stream_kernel(ScoreArgs a, int T, int G)
{
    constexpr int RB = 256;                     // bytes per key row (and per q row)
    constexpr int SUB = 32;                     // rows per slot
    constexpr int SLOT = SUB * RB;              // 8 KB
    constexpr int NI = SLOT / 1024;             // loads per slot
    constexpr int KS = 8;                       // MFMA steps over d_I = 128
    static_assert(R >= 2 && NI * (R - 1) < 64, "the vector-memory counter holds 63");
    extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];   // [NW][R][SLOT]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, half = lane >> 5;
    const int wdw = (int)blockIdx.x % G;                    // this workgroup's tokens: wdw, wdw + G, ...
    const int wstride = NW * ((int)gridDim.x / G);          // waves that share a token
    const int wfirst = ((int)blockIdx.x / G) * NW + wave;   // this wave's slots of a token: wfirst, wfirst + wstride, ...
    const bool ragged = PG && a.pv.seq_lens, paged = PG && a.pv.page_table;
    const int i_end = min(a.i0 + a.Ri, a.Tq);

    // A cursor walks the wave's items: per token HT q items (jj = -HT .. -1), then its key slots (jj = 0 .. n_w - 1).
    // Two cursors run over the same sequence: the one that issues loads stays R - 1 items ahead of the one that
    // computes.
    struct Cur {
        int tk, jj, n_w;
        int bz, t, Lk_b, vis;                   // sequence within the launch, query row, visible keys
    };
    auto enter = [&](Cur &c) {                  // first item of token c.tk or of the next token that has work
        for (; c.tk < T; c.tk += G) {
            c.bz = c.tk / a.Ri;
            c.t = a.i0 + c.tk % a.Ri;
            if (c.t >= i_end) continue;
            const int b = a.b0 + c.bz;
            c.Lk_b = ragged ? max(0, min(load_uniform(a.pv.seq_lens + b), a.Lk)) : a.Lk;
            const int64_t q_pos0 = ragged ? (int64_t)c.Lk_b - a.Tq : a.q_pos0;
            int64_t vis64 = q_pos0 + (int64_t)c.t + 1;
            vis64 = vis64 < 0 ? 0 : (vis64 > c.Lk_b ? c.Lk_b : vis64);
            c.vis = (int)vis64;
            const int nsub = (c.vis + SUB - 1) / SUB;
            c.n_w = nsub > wfirst ? (nsub - wfirst + wstride - 1) / wstride : 0;
            if (c.n_w > 0) {
                c.jj = -HT;
                return;
            }
        }
    };
    auto next = [&](Cur &c) {
        if (++c.jj >= c.n_w) {
            c.tk += G;
            enter(c);
        }
    };

    const unsigned ring_w = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)ring + (unsigned)wave * (R * SLOT);
    // rows a lane fetches within a slot: 4 i + (lane >> 4), i = 0..7; its piece of the row (lane & 15) ^ (row & 15)
    const int lrow = lane >> 4, lpiece = lane & 15;
    auto issue = [&](const Cur &c, int slot_i) {
        const int b = a.b0 + c.bz;
        const unsigned char *base;
        int last;                               // rows past this one re-read it (their results are masked or weigh 0)
        if (c.jj < 0) {
            const int h0 = (c.jj + HT) * 32;    // head tile
            base = (const unsigned char *)a.q + (((int64_t)b * a.Tq + c.t) * a.H_I + min(h0, a.H_I - 1)) * RB;
            last = max(a.H_I - 1 - h0, 0);
        } else {
            const int s0 = (wfirst + c.jj * wstride) * SUB;             // < vis <= Lk_b
            int64_t krow = (int64_t)b * a.Lk + s0;
            if (paged) {                        // a slot never straddles a page: pages hold a multiple of 64 positions
                const int32_t page = load_uniform(a.pv.page_table + (int64_t)b * a.pv.max_pages + (s0 >> a.pv.page_shift));
                krow = ((int64_t)page << a.pv.page_shift) + (s0 & ((1 << a.pv.page_shift) - 1));
            }
            base = (const unsigned char *)a.k + krow * RB;
            last = c.Lk_b - 1 - s0;
        }
        const unsigned slot = ring_w + (unsigned)slot_i * SLOT;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = 4 * i + lrow;
            const int off = min(row, last) * RB + ((lpiece ^ (row & 15)) << 4);
            dma_lanes(base + off, slot + i * 1024);
        }
    };

    Cur pc, cc;                                 // producer, consumer
    pc.tk = wdw;
    enter(pc);
    if (pc.tk >= T) return;                     // nothing for this wave (no barrier in this kernel)
    cc = pc;
    int p_slot = 0, c_slot = 0;
#pragma unroll
    for (int d = 0; d < R - 1; ++d)
        if (pc.tk < T) {
            issue(pc, p_slot);
            p_slot = p_slot + 1 == R ? 0 : p_slot + 1;
            next(pc);
        }

    bf16x8 qa[HT][KS];
    float wr[HT][16];
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qa[ht][ks] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
#pragma unroll
        for (int i = 0; i < 16; ++i) wr[ht][i] = 0.f;
    }
    const unsigned char *my = ring + wave * (R * SLOT) + r32 * RB;       // this lane's row within a slot

    while (cc.tk < T) {
        if (pc.tk < T) {
            issue(pc, p_slot);                                           // the slot consumed in the previous iteration
            p_slot = p_slot + 1 == R ? 0 : p_slot + 1;
            next(pc);
            wait_vm_le<NI * (R - 1)>();                                  // the consumer's slot has landed
        } else {
            wait_vm_le<0>();
        }
        const unsigned char *sp = my + c_slot * SLOT;
        c_slot = c_slot + 1 == R ? 0 : c_slot + 1;
        bf16x8 kb[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            kb[ks] = *(const bf16x8 *)(sp + (((ks * 2 + half) ^ (r32 & 15)) << 4));
        if (cc.jj < 0) {
            // a q item: the token's rows of one head tile become the stationary operand; its head weights follow
            // (uniform addresses: scalar loads)
            const int ht_in = cc.jj + HT;
            const float *wrow = a.w + ((int64_t)(a.b0 + cc.bz) * a.Tq + cc.t) * a.H_I;
#pragma unroll
            for (int ht = 0; ht < HT; ++ht) {
                if (ht != ht_in) continue;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) qa[ht][ks] = kb[ks];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int h_lo = ht * 32 + 8 * (i / 4) + (i % 4), h_hi = h_lo + 4;
                    const float w_lo = h_lo < a.H_I ? load_uniform(wrow + h_lo) : 0.f;
                    const float w_hi = h_hi < a.H_I ? load_uniform(wrow + h_hi) : 0.f;
                    wr[ht][i] = half ? w_hi : w_lo;
                }
            }
            asm volatile("" ::: "memory");
            next(cc);
            continue;
        }
        float s_acc = 0.f;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ht][ks], kb[ks], acc, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 16; ++i)
                s_acc = fmaf(relu(acc[i]), wr[ht][i], s_acc);
        }
        // the reads of this slot have returned (the MFMAs consumed them) before the next iteration's loads
        // overwrite it; the statement below keeps the compiler from moving them
        asm volatile("" ::: "memory");
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(s_acc), __float_as_uint(s_acc), false, false);
        const float v = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
        const int s = (wfirst + cc.jj * wstride) * SUB + r32;
        if (half == 0 && s < cc.vis) a.strip[((int64_t)cc.bz * a.Ri + (cc.t - a.i0)) * a.ld + s] = v;
        next(cc);
    }
}

template <int HT, int NW, int R>
hipError_t launch_stream(const ScoreArgs &a, int Bc, hipStream_t st)
{
    const int T = Bc * a.Ri;                    // tokens of the launch
    if (T <= 0) return hipSuccess;
    const int G = T < 16 ? T : 16;              // tokens in flight (measured at 32 tokens: 2 -> 99.2, 4 -> 97.7, 8 -> 98.4, 16 -> 97.1, 32 -> 102.1 us)
    const int W = G * (256 / G);                // one workgroup per CU (the ring takes most of a CU's LDS)
    constexpr int lds = NW * R * 32 * 256;
    static hipError_t attr = hipFuncSetAttribute((const void *)score_stream_kernel<HT, NW, R, false>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    static hipError_t attr_pg = hipFuncSetAttribute((const void *)score_stream_kernel<HT, NW, R, true>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return attr;
    if (attr_pg != hipSuccess) return attr_pg;
    if (a.pv.seq_lens || a.pv.page_table)
        hipLaunchKernelGGL((score_stream_kernel<HT, NW, R, true>), dim3(W), dim3(64 * NW), lds, st, a, T, G);
    else
        hipLaunchKernelGGL((score_stream_kernel<HT, NW, R, false>), dim3(W), dim3(64 * NW), lds, st, a, T, G);
    return hipGetLastError();
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
    // Few query rows per sequence (decode, short chunks): the kernel only streams keys.  bf16 keys of 128
    // take the ring form (score_stream_kernel); the other formats one token per workgroup, three workgroups
    // per CU and three key tiles in flight per workgroup.
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
    kc = kc < 512 ? 512 : (kc > 8192 ? 8192 : kc);
    a.KC = (int)kc;
    const bool fp8 = dtype == IC_FP8_E4M3;
    if (few_rows && !fp8 && d_I == 128)
        return a.H_I <= 32 ? launch_stream<1, 4, 4>(a, Bc, st) : launch_stream<2, 4, 4>(a, Bc, st);
    if (!fp8) {
        if (a.H_I <= 32) {
            if (d_I == 128) return launch_t<1, 128, 3, 4, 1, 2, false, false>(a, Bc, max_vis, st);
            if (d_I == 64) return few_rows ? launch_t<1, 64, 1, 4, 3, 3, true, false>(a, Bc, max_vis, st) : launch_t<1, 64, 3, 4, 1, 2, false, false>(a, Bc, max_vis, st);
        } else {
            if (d_I == 128) return launch_t<2, 128, 2, 4, 1, 1, false, false>(a, Bc, max_vis, st);
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
