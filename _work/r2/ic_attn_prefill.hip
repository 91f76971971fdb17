// Sparse MQA core attention, prefill form for MLA rows (576 logit features, the first 512 of them the values;
// paper Sec. 2.1: the main attention runs over the selected top-k rows only).
//
// One workgroup of EIGHT waves per CU (two per SIMD, 256 registers each) walks a chain of queries; a query's
// selected rows pass through LDS in tiles of 64 rows, two tiles resident.
//
//   gather   loads that write LDS directly (global_load_lds_dwordx4): no trip through registers, no LDS store
//            instruction.  Wave w brings rows 8w..8w+7 of a tile: one instruction per row for the 1024 value
//            bytes (64 lanes x 16 bytes, the row's base in scalar registers), one for the 128 rope bytes of all
//            eight rows.  Such a load writes 64 consecutive 16-byte slots, so the bank swizzle is applied on
//            the global side: the lane that writes slot c fetches chunk c ^ x(row).
//   S^T      wave (rb, hb) = (w & 3, w >> 2) multiplies tile rows 16rb..16rb+15 with heads 16hb..16hb+15:
//            S^T = K Q^T on v_mfma_f32_16x16x32_bf16, K rows as the A operand (16-byte LDS reads), Q in
//            registers for the whole query.
//   softmax  against a lazily updated reference maximum per (wave, head); P (bf16) and the reference go to LDS
//   barrier  one per tile
//   P V      wave w owns value columns 64w..64w+63 for all 32 heads: O += P V on v_mfma_f32_32x32x16_bf16,
//            V out of the same row-major tile through the transposing LDS read (ds_read_b64_tr_b16), fetched
//            BEFORE the barrier so that the tile's buffer can be refilled right after it.
// Pipeline: iteration i = { start the gather of tile i+2 into the buffer tile i just left; P V of tile i;
// S^T, V fetch and softmax of tile i+1; wait for the gather; barrier }.  A gather has one whole iteration to land.
// With two waves per SIMD the matrix pipe runs one wave's MFMAs under the other's LDS and vector work.
//
// LDS layout of a tile: value part [64 rows][1024 B] and rope part [64 rows][128 B], kept apart so that every
// direct load covers whole rows.  Swizzles (16-byte slots): value part slot' = slot ^ x(row) on the low four
// bits, x(r) = ((r & 3) << 2) | h[(r >> 2) & 3], h = {2, 0, 1, 3}; rope part slot' = slot ^ ((row >> 1) & 7).
// Both make the A-operand reads (a 128-bit LDS read is served in groups of lanes {0-3, 12-15, 20-23, 24-27},
// {4-7, 8-11, 16-19, 28-31} and the same + 32) and the transposing reads (groups of 32 lanes) conflict-free.
#include "ic_common.hpp"

namespace ic {

namespace {

constexpr int kT = 64;                       // rows per tile
constexpr int kDQK = 576, kDV = 512;
constexpr int kVRow = 1024, kRRow = 128;     // bytes of a row's value / rope part in LDS
constexpr int kVBuf = kT * kVRow, kRBuf = kT * kRRow;
constexpr int kPStr = kT * 2 + 16;           // bytes per head row of the P tile: 64 probabilities + 4 references
constexpr int kPBuf = 32 * kPStr;
constexpr int kOffV = 0, kOffR = 2 * kVBuf, kOffP = kOffR + 2 * kRBuf, kOffL = kOffP + 2 * kPBuf, kOffA = kOffL + 4 * 32 * 4;
constexpr int kLdsBytes = kOffA + 8 * 32 * 4;
constexpr int kKS = kDQK / 32;               // contraction steps of S^T
constexpr float kLazyLog2 = 8.f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ int vswz(int r) { return ((r & 3) << 2) | ((0xD2 >> (2 * ((r >> 2) & 3))) & 3); }
__device__ __forceinline__ int rswz(int r) { return (r >> 1) & 7; }

__device__ __forceinline__ float xmax16_32(float x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ __forceinline__ float xsum16_32(float x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Loads that write LDS: 64 lanes x 16 bytes land in 1024 consecutive bytes starting at the LDS address in M0.
// The compiler does not see them as memory operations of its own; every use of their data follows an explicit
// wait (wait_vm) and a barrier.
// dma_row: lane l fetches 16 bytes at row_base + (lane16 ^ swz16), lane16 = 16 l, swz16 = 16 x(row) (uniform).  The
// exclusive-or sits inside the statement so that the eight per-row offsets are not kept in registers.
__device__ __forceinline__ void dma_row(const void *row_base /*uniform*/, unsigned lane16, unsigned swz16 /*uniform*/,
                                        unsigned lds_addr /*uniform*/)
{
    unsigned off;
    asm volatile("v_xor_b32 %0, %3, %1\n\ts_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2"
                 : "=&v"(off)
                 : "v"(lane16), "s"(row_base), "s"(swz16), "s"(lds_addr)
                 : "memory");
}
__device__ __forceinline__ void dma_lanes(const void *lane_addr, unsigned lds_addr /*uniform*/)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(lane_addr), "s"(lds_addr) : "memory");
}
// A 4-byte load the compiler does not track either (its result is used only behind wait_vm).
__device__ __forceinline__ int load_i32_async(const int32_t *p)
{
    int v;
    asm volatile("global_load_dword %0, %1, off" : "=v"(v) : "v"(p) : "memory");
    return v;
}
__device__ __forceinline__ void wait_vm(int &a, int &b)
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b)::"memory");
}

__device__ __forceinline__ unsigned lds_addr_of(const void *p)
{
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

__global__ __launch_bounds__(512, 1) void attn_prefill_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *lbuf = (float *)(smem + kOffL);                // [4][32] row sums of the four row-block waves
    float *abuf = (float *)(smem + kOffA);                // [8][32] per-wave rescale factors

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rb = w & 3, hb = w >> 2;
    const int l16 = lane & 15, g = lane >> 4, l32 = lane & 31, hh = lane >> 5;
    const int ntiles = (a.k_sel + kT - 1) / kT;           // >= 3 (launcher)
    const int64_t nq = (int64_t)a.B * a.Tq;
    const int rowbytes = a.row_elems * 2;

    int qrow = (int)blockIdx.x;                           // B * Tq < 2^30 (checked by the caller)
    if ((gridDim.x & 7u) == 0 && (int64_t)gridDim.x < nq) {
        // workgroup ids go round-robin over the 8 XCDs (one L2 each): give an XCD contiguous queries,
        // which select largely the same rows
        const unsigned per = gridDim.x >> 3;
        qrow = (int)((blockIdx.x & 7u) * per + (blockIdx.x >> 3));
    }
    int qnext = qrow + (int)gridDim.x;
    // a query past the end still names valid memory (the workgroup's first query); its rows are masked
    auto safe_q = [&](int q) { return (int64_t)q < nq ? q : (int)blockIdx.x; };
    int b_cur = safe_q(qrow) / a.Tq, b_next = safe_q(qnext) / a.Tq;
    const int64_t seq_bytes = (int64_t)a.Lk * rowbytes;

    // ---- per-lane LDS offsets (inside one tile buffer) ----
    const int st_row = 16 * rb + l16;                     // S^T role: the lane's tile row
    int a_v[4], a_r[2];
#pragma unroll
    for (int m = 0; m < 4; ++m) a_v[m] = st_row * kVRow + (((4 * m + g) ^ vswz(l16)) << 4);
#pragma unroll
    for (int m = 0; m < 2; ++m) a_r[m] = st_row * kRRow + (((4 * m + g) ^ rswz(l16)) << 4);
    int t_v[2][2];                                        // [first / second four rows][column block]
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
        const int r15 = 8 * hh + 4 * h2 + (l16 >> 2);
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const int c_low = 8 * (w & 1) + 4 * nb + 2 * (g & 1) + ((l16 & 3) >> 1);
            t_v[h2][nb] = r15 * kVRow + 256 * (w >> 1) + ((c_low ^ vswz(r15)) << 4) + 8 * (l16 & 1);
        }
    }
    const unsigned lane16 = (unsigned)lane << 4;

    // ---- state of the current query ----
    bf16x8 qreg[kKS];                                     // Q, heads 16hb + l16, as the B operand of S^T
    f32x16 oacc[2];
    s16x4 vq[4][2][2];                                    // V operands of the tile whose P V comes next
    float m_all = -INFINITY, m_ref = -INFINITY, m_c = -INFINITY, l_own = 0.f;
    int g0 = 0;                                           // buffer parity of the query's tile 0

    auto load_q = [&](int q) {
        const int head = 16 * hb + l16;
        const bool ok = head < a.H_q;
        const unsigned short *qp = (const unsigned short *)a.Q + ((int64_t)q * a.H_q + (ok ? head : 0)) * kDQK + 8 * g;
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) {
            u32x4 raw = u32x4{0u, 0u, 0u, 0u};
            if (ok) raw = *(const u32x4 *)(qp + 32 * ks);
            qreg[ks] = __builtin_bit_cast(bf16x8, raw);
        }
    };
    auto reset_acc = [&]() {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[nb][i] = 0.f;
        m_all = m_ref = m_c = -INFINITY;
        l_own = 0.f;
    };

    // The lane's tile row in the gather role (8w + lane / 8) and in the S^T role (16rb + lane % 16), rebuilt from
    // the thread id behind a compiler barrier wherever they are needed: cheaper than keeping them (a spilled
    // register's reload would bring a wait for everything in flight into the tile loop).
    auto row_dma = [&]() {
        int t = tid;
        asm volatile("" : "+v"(t));
        return ((t >> 6) << 3) + ((t & 63) >> 3);
    };
    auto row_st = [&]() {
        int t = tid;
        asm volatile("" : "+v"(t));
        return (((t >> 6) & 3) << 4) + (t & 15);
    };
    // Stream tile j of the current query; tiles at or beyond ntiles are the next query's first tiles.
    // row: the lane's tile row.  Address of its id / whether a loaded id names a row to attend to.
    auto id_addr = [&](int j, int row) {
        const bool nx = j >= ntiles;
        const int q = safe_q(nx ? qnext : qrow);
        const int slot = (nx ? j - ntiles : j) * kT + row;
        return a.idx + (int64_t)q * a.k_sel + min(slot, a.k_sel - 1);
    };
    auto valid_id = [&](int id, int j, int row) {
        const bool nx = j >= ntiles;
        const int live = (int)((int64_t)(nx ? qnext : qrow) < nq);
        const int slot = (nx ? j - ntiles : j) * kT + row;
        return live & (int)(slot < a.k_sel) & (int)(id >= 0) & (int)(id < a.Lk);
    };

    // The gather of stream tile j into its buffer, in nine pieces (one load instruction each) so that they can be
    // spread over an iteration: the CU's one address unit takes 16 clocks per 1 KiB instruction, and a wave that
    // issues its nine at once waits behind the other seven waves' for over a thousand clocks.
    // gather_begin: id = the lane's row id as loaded (row 8w + lane / 8); piece 0..7 = one row each, 8 = the rope bytes.
    struct Gather { const unsigned char *kv; unsigned ldsV, ldsR; int vrow; };
    auto gather_begin = [&](int j, int id) {
        Gather c;
        c.kv = (const unsigned char *)a.KV + (int64_t)(j >= ntiles ? b_next : b_cur) * seq_bytes;
        const int par = (g0 + j) & 1;
        c.vrow = valid_id(id, j, row_dma()) ? id : 0;     // empty slots fetch row 0, masked later
        c.ldsV = lds_addr_of(smem + kOffV) + (unsigned)(par * kVBuf + 8 * w * kVRow);
        c.ldsR = lds_addr_of(smem + kOffR) + (unsigned)(par * kRBuf + 8 * w * kRRow);
        return c;
    };
    auto gather_piece = [&](const Gather &c, int r) {
        if (r < 8) {
            const int rid = __builtin_amdgcn_readlane(c.vrow, 8 * r);
            const unsigned char *base = c.kv + (int64_t)rid * rowbytes;
            const unsigned sw = (unsigned)vswz((8 * (w & 1) + r) & 15) << 4;
            dma_row(base, lane16, sw, c.ldsV + r * kVRow);
        } else {
            const unsigned char *rp = c.kv + (int64_t)c.vrow * rowbytes + kVRow + (((tid & 7) ^ rswz(row_dma())) << 4);
            dma_lanes(rp, c.ldsR);
        }
    };
    auto gather = [&](int j, int id) {
        const Gather c = gather_begin(j, id);
#pragma unroll
        for (int r = 0; r < 9; ++r) gather_piece(c, r);
    };

    // V operands of tile j (published) for the P V that follows the next barrier
    auto vfetch = [&](int j) {
        const unsigned char *tbV = smem + kOffV + ((g0 + j) & 1) * kVBuf;
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                vq[jj][nb][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tbV + t_v[0][nb] + 16 * jj * kVRow));
                vq[jj][nb][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tbV + t_v[1][nb] + 16 * jj * kVRow));
            }
    };

    // S^T, V fetch and softmax of tile j (already in LDS and published); idv = the lane's row id for validity
    auto produce = [&](int j, int idv, const Gather *gc, bool with_v) {
        const int par = (g0 + j) & 1;
        const unsigned char *tbV = smem + kOffV + par * kVBuf;
        const unsigned char *tbR = smem + kOffR + par * kRBuf;
        unsigned char *pb = smem + kOffP + par * kPBuf;
        const unsigned vm = (unsigned)__ballot(valid_id(idv, j, row_st()) != 0) & 0xFFFFu;   // lanes 0..15: rows 0..15

        f32x4 s4[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
        constexpr int kRing = 6;                          // A-operand reads in flight ahead of the MFMAs
        bf16x8 ka[kRing];
        auto ka_read = [&](int ks) {
            return ks < 16 ? *(const bf16x8 *)(tbV + a_v[ks & 3] + 256 * (ks >> 2)) : *(const bf16x8 *)(tbR + a_r[ks - 16]);
        };
#pragma unroll
        for (int r = 0; r < kRing; ++r) ka[r] = ka_read(r);
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) {
            s4[ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks % kRing], qreg[ks], s4[ks & 1], 0, 0, 0);
            if (ks + kRing < kKS) ka[ks % kRing] = ka_read(ks + kRing);
            if (gc && ks % 3 == 2 && ks < 15) {           // pieces 4..8 behind MFMAs 2, 5, 8, 11, 14
                __builtin_amdgcn_sched_barrier(0);
                gather_piece(*gc, 4 + ks / 3);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (with_v) vfetch(j);

        float z[4], mx = -INFINITY;
        const bool all_rows = vm == 0xFFFFu;              // wave-uniform: no empty slot among the wave's 16 rows
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            z[i] = (s4[0][i] + s4[1][i]) * a.scale_log2e;
            if (!all_rows) z[i] = ((vm >> (4 * g + i)) & 1u) ? z[i] : -INFINITY;
            mx = fmaxf(mx, z[i]);
        }
        mx = xmax16_32(mx);
        // lazy reference: keep the common reference until this tile exceeds it by more than 2^kLazyLog2.  m_all may
        // lag one tile behind (the waves that produce before they consume): the consumer side never lowers its reference.
        const float m_base = fmaxf(m_all, m_ref);         // a wave never lowers its own reference either
        const float m_new = (mx > m_base + kLazyLog2) ? mx : m_base;
        const float resc = (m_new == -INFINITY) ? 1.f : fast_exp2(m_ref - m_new);
        float psum = 0.f;
        s16x4 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float p = fast_exp2(z[i] - m_new);            // z = -inf gives 0 unless m_new is -inf too
            if (!all_rows) p = (z[i] == -INFINITY) ? 0.f : p;
            psum += p;
            pk[i] = __builtin_bit_cast(short, (__bf16)p);
        }
        l_own = l_own * resc + psum;
        m_ref = m_new;
        unsigned char *prow = pb + (16 * hb + l16) * kPStr;
        *(s16x4 *)(prow + (16 * rb + 4 * g) * 2) = pk;
        if (g == 0) *(float *)(prow + kT * 2 + 4 * rb) = m_new;
    };

    // O += P V for tile j (P and the references published by the last barrier, V in vq)
    auto consume = [&](int j, const Gather *gc) {
        const int par = (g0 + j) & 1;
        const unsigned char *pp = smem + kOffP + par * kPBuf + l32 * kPStr;
        const f32x4 mjc = *(const f32x4 *)(pp + kT * 2);
        bf16x8 pa[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) pa[jj] = *(const bf16x8 *)(pp + (16 * jj + 8 * hh) * 2);
        // common case: all four row-block waves kept the common reference: nothing to rescale
        const bool same = (mjc[0] == m_c) & (mjc[1] == m_c) & (mjc[2] == m_c) & (mjc[3] == m_c);
        if (__ballot(!same) != 0ull) {
            // the reference never goes down (a producer's reference may lag one tile behind the common one)
            const float m_new_c = fmaxf(m_c, fmaxf(fmaxf(mjc[0], mjc[1]), fmaxf(mjc[2], mjc[3])));
            const float alpha = (m_new_c == -INFINITY) ? 1.f : fast_exp2(m_c - m_new_c);
            m_c = m_new_c;
            float fj[4];
            bool any_f = false;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                fj[jj] = (m_new_c == -INFINITY) ? 1.f : fast_exp2(mjc[jj] - m_new_c);
                any_f |= (fj[jj] != 1.f);
            }
            if (__ballot(alpha != 1.f) != 0ull) {
                // rescale factors of the 16 heads a lane accumulates, through a per-wave LDS row (LDS serves a wave in order)
                float *ab = abuf + w * 32;
                if (hh == 0) ab[l32] = alpha;
                f32x4 ar[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) ar[q] = *(const f32x4 *)(ab + 8 * q + 4 * hh);
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[nb][i] *= ar[i >> 2][i & 3];
            }
            if (__ballot(any_f) != 0ull) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pa[jj][e] = (__bf16)((float)pa[jj][e] * fj[jj]);
            }
        }
        // the producer role needs the common reference of head 16hb + l16, which lives in another 16-lane group
        {
            const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(m_c), __float_as_uint(m_c), false, false);
            m_all = __uint_as_float(hb ? sw[1] : sw[0]);
        }
        typedef __attribute__((ext_vector_type(8))) short s16x8;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const s16x4 v0 = vq[jj][nb][0], v1 = vq[jj][nb][1];
                const s16x8 vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa[jj], __builtin_bit_cast(bf16x8, vv), oacc[nb], 0, 0, 0);
                if (gc && nb == 1) {                      // pieces 0..3 behind MFMAs 1, 3, 5, 7
                    __builtin_amdgcn_sched_barrier(0);
                    gather_piece(*gc, jj);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
    };

    // epilogue of a query: combine the row-block waves' sums, normalise, store
    auto finish = [&]() {
        const float l = xsum16_32(l_own);
        const float f = (m_all == -INFINITY) ? 0.f : fast_exp2(m_ref - m_all);   // to the common reference
        if (g == 0) lbuf[rb * 32 + 16 * hb + l16] = l * f;
        __syncthreads();
        if (w == 0 && hh == 0 && l32 < a.H_q && a.lse) {
            const float l_head = lbuf[l32] + lbuf[32 + l32] + lbuf[64 + l32] + lbuf[96 + l32];
            a.lse[(int64_t)qrow * a.H_q + l32] = (l_head > 0.f) ? (m_c + __builtin_log2f(l_head)) * 0.6931471805599453f : -INFINITY;
        }
        f32x4 inv4[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f32x4 l4 = *(const f32x4 *)(lbuf + 8 * q + 4 * hh);
#pragma unroll
            for (int r = 1; r < 4; ++r) l4 += *(const f32x4 *)(lbuf + 32 * r + 8 * q + 4 * hh);
#pragma unroll
            for (int r = 0; r < 4; ++r) inv4[q][r] = (l4[r] > 0.f) ? __builtin_amdgcn_rcpf(l4[r]) : 0.f;
        }
        __bf16 *o_row = (__bf16 *)a.O + (int64_t)qrow * a.H_q * kDV + 64 * w + l32;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int hq = 8 * (i >> 2) + 4 * hh + (i & 3);              // head of accumulator element i
            if (hq < a.H_q) {
                const float inv = inv4[i >> 2][i & 3];
                o_row[hq * kDV] = (__bf16)(oacc[0][i] * inv);
                o_row[hq * kDV + 32] = (__bf16)(oacc[1][i] * inv);
            }
        }
    };

#ifdef IC_ATTN_TIMING
    long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    long long tprev = __builtin_readcyclecounter();
#define TSTAMP(k) do { const long long tn = __builtin_readcyclecounter(); tacc[k] += tn - tprev; tprev = tn; } while (0)
#else
#define TSTAMP(k) do { } while (0)
#endif
    // ---- prologue: tiles 0 and 1 of the first query in flight, Q in registers ----
    int id_dma = load_i32_async(id_addr(0, row_dma()));         // ids for the gather of the next tile to start
    int id_st = load_i32_async(id_addr(0, row_st()));           // ids for the validity mask of the next tile to produce
    int id_dma1 = load_i32_async(id_addr(1, row_dma()));
    load_q(qrow);
    reset_acc();
    wait_vm(id_dma, id_dma1);
    {
        int x = id_st, y = id_st;
        wait_vm(x, y);
        id_st = x;
    }
    gather(0, id_dma);
    gather(1, id_dma1);
    id_dma = load_i32_async(id_addr(2, row_dma()));
    int id_st_next = load_i32_async(id_addr(1, row_st()));
    wait_vm(id_dma, id_st_next);
    __syncthreads();
    produce(0, id_st, nullptr, true);
    id_st = id_st_next;
    __syncthreads();

    for (;;) {
#pragma unroll 1
        for (int i = 0; i + 1 < ntiles; ++i) {
            TSTAMP(0);
            // the gather of tile i + 2 goes into the buffer tile i has left (its reads ended before the barrier),
            // piece by piece under the MFMAs of this iteration
            const Gather gc = gather_begin(i + 2, id_dma);
            int nd = load_i32_async(id_addr(i + 3, row_dma()));
            int nv = load_i32_async(id_addr(i + 2, row_st()));
            TSTAMP(1);
            // the two waves of a SIMD take the two halves in opposite order, so that one's MFMAs run under
            // the other's softmax arithmetic
            if (w < 4) {
                consume(i, &gc);
                TSTAMP(2);
                produce(i + 1, id_st, &gc, true);
            } else {
                produce(i + 1, id_st, &gc, false);
                TSTAMP(2);
                consume(i, &gc);
                vfetch(i + 1);
            }
            TSTAMP(3);
            wait_vm(nd, nv);
            TSTAMP(4);
            id_dma = nd;
            id_st = nv;
            __syncthreads();
            TSTAMP(5);
        }
        // last tile of the query
        const bool more = (int64_t)qnext < nq;
        const Gather gl = gather_begin(ntiles + 1, id_dma);   // tile 1 of the next query (dead queries: row 0, masked)
        int nd = load_i32_async(id_addr(ntiles + 2, row_dma()));
        int nv = load_i32_async(id_addr(ntiles + 1, row_st()));
        consume(ntiles - 1, &gl);
#pragma unroll
        for (int r = 4; r < 9; ++r) gather_piece(gl, r);
        if (more) load_q(qnext);                          // Q is free: the query's last S^T ran in the previous iteration
        finish();
        if (!more) {
            wait_vm(nd, nv);                              // nothing may still be writing LDS when the workgroup ends
#ifdef IC_ATTN_TIMING
            if (blockIdx.x == 0 && lane == 0 && a.lse)
                for (int k = 0; k < 8; ++k) a.lse[w * 8 + k] = (float)tacc[k];
#endif
            break;
        }
        // the next query becomes the current one: its tile 0 sits where stream tile `ntiles` went
        g0 = (g0 + ntiles) & 1;
        qrow = qnext;
        qnext += (int)gridDim.x;
        b_cur = b_next;
        b_next = safe_q(qnext) / a.Tq;
        reset_acc();
        wait_vm(nd, nv);
        __syncthreads();
        produce(0, id_st, nullptr, true);
        id_dma = nd;
        id_st = nv;
        __syncthreads();
    }
}

} // namespace

bool attn_prefill_supported(const AttnArgs &a, int d_qk, int d_v)
{
    return d_qk == kDQK && d_v == kDV && a.v_off == 0 && a.n_splits <= 1 && a.k_sel > 2 * kT && !a.pv.seq_lens &&
           !a.pv.page_table && a.H_q <= 32;
}

hipError_t launch_attn_prefill(const AttnArgs &a, hipStream_t st)
{
    static hipError_t attr = hipFuncSetAttribute((const void *)attn_prefill_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr != hipSuccess) return attr;
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
            return hipErrorInvalidDevice;
        n_cu = v;
    }
    int64_t wgs = (int64_t)a.B * a.Tq;
    if (wgs > n_cu) wgs = n_cu;
    hipLaunchKernelGGL(attn_prefill_kernel, dim3((unsigned)wgs), dim3(512), kLdsBytes, st, a);
    return hipGetLastError();
}

} // namespace ic
