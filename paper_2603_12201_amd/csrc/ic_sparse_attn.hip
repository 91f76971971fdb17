// Sparse MQA core attention over the selected KV rows (paper Sec. 2.1: the main attention is
// computed only over the top-k subset; MLA form, one shared KV row per position).
//
// One workgroup (4 waves) per query token and key-slot split; two workgroups fit a CU (75 KB of
// LDS, <= 256 VGPRs each) so that one computes while the other waits for its gather.  Tiles of
// 32 selected rows are gathered with 16-byte coalesced loads (each row is contiguous) into a
// double-buffered LDS tile, row-major.  A wave owns 16 of the 32 heads and half of the value
// columns, and runs its own online softmax over every row of the tile:
//   S^T = K Q^T   v_mfma_f32_16x16x32_bf16, A = tile rows (16-byte LDS reads), B = Q (registers)
//   P   = exp2(S^T * scale*log2e - m)   in the result layout: a lane owns one head, 8 keys
//   O  += P V     same MFMA; P is already an A operand (its contraction slots are whatever keys
//                 the lane holds), and V comes out of the SAME row-major tile through the LDS
//                 transpose read ds_read_b64_tr_b16, which hands a lane one value column of four
//                 consecutive tile rows.  No transposed copy of V is ever made.
// The two waves of a head group compute the same S^T (cheap next to the gather) and therefore
// the same softmax statistics, so no exchange between waves is ever needed.  With several
// splits per query the unnormalised partials go to the workspace and a small kernel merges them.
#include "ic_common.hpp"
#include <stdlib.h>
#include <type_traits>

namespace ic {

namespace {

constexpr int kTile = 32;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Tile staging.  A thread owns tile row tid / 8 and the 16-byte chunks (tid % 8) + 8 r of that
// row: eight neighbouring lanes read one full 128-byte line, and no index needs a division.
template <int ROW_F, int LPT>
__device__ __forceinline__ void attn_gload(u32x4 (&pre)[LPT], const unsigned short *kv_seq, const int32_t *ti,
                                           int row_elems, int tid)
{
    constexpr int CPR = ROW_F / 8;
    const int row = tid >> 3, c0 = tid & 7;
    const int32_t v = ti[row];
    const unsigned short *src = kv_seq + (int64_t)(v < 0 ? 0 : v) * row_elems + c0 * 8;
#pragma unroll
    for (int r = 0; r < LPT; ++r)
        if (c0 + 8 * r < CPR) pre[r] = *(const u32x4 *)(src + 64 * r);
}

template <int ROW_F, int LPT, int ROWB>
__device__ __forceinline__ void attn_lstore(const u32x4 (&pre)[LPT], unsigned char *tile, int tid)
{
    constexpr int CPR = ROW_F / 8;
    const int row = tid >> 3, c0 = tid & 7;
    unsigned char *dst = tile + row * ROWB + c0 * 16;
#pragma unroll
    for (int r = 0; r < LPT; ++r)
        if (c0 + 8 * r < CPR) *(u32x4 *)(dst + 128 * r) = pre[r];
}

template <int D_QK, int D_V, int ROW_F>
__global__ __launch_bounds__(256, 2) void attn_kernel(AttnArgs a)
{
    constexpr int ROWB = ROW_F * 2 + 16;                  // LDS row stride in bytes
    constexpr int CPR = ROW_F / 8;                        // 16-byte chunks staged per row
    constexpr int LPT = (CPR + 7) / 8;                    // chunk loads per thread per tile (one row per 8 lanes)
    static_assert(kTile * 8 == 256, "256 threads cover the tile rows, 8 lanes per row");
    constexpr int KSTEPS = D_QK / 32;
    constexpr int DVW = D_V / 2;                          // value columns per wave
    constexpr int NB = DVW / 16;
    constexpr int TILEB = kTile * ROWB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *tile0 = smem;                          // [2][kTile][ROWB]
    int32_t *tidx = (int32_t *)(smem + 2 * TILEB);        // [3][kTile] validated row ids of a tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int mh = wave & 1, vh = wave >> 1;
    const int64_t qrow = blockIdx.x;                      // flattened (b, t)
    const int b = (int)(qrow / a.Tq);
    const int sp = blockIdx.y;
    const int slot0 = sp * a.split_len;
    const int slot1 = min(slot0 + a.split_len, a.k_sel);
    const int ntiles = (slot1 - slot0 + kTile - 1) / kTile;

    const int32_t *idx_row = a.idx + qrow * a.k_sel;
    const unsigned short *kv_seq = (const unsigned short *)a.KV + (int64_t)b * a.Lk * a.row_elems;

    auto fetch_idx = [&](int it) -> int32_t {             // threads 0..31: validated row id of a slot
        const int slot = slot0 + it * kTile + tid;
        int32_t v = -1;
        if (it < ntiles && slot < slot1) v = idx_row[slot];
        return (v >= 0 && v < a.Lk) ? v : -1;
    };

    // ---- Q as the B operand of S^T = K Q^T: lane (head l16, k-group g) ----
    const int head = 16 * mh + l16;
    const bool head_ok = head < a.H_q;
    const bool wave_ok = 16 * mh < a.H_q;                 // wave-uniform: any valid head at all
    bf16x8 qreg[KSTEPS];
    {
        const unsigned short *qp = (const unsigned short *)a.Q + (qrow * a.H_q + (head_ok ? head : 0)) * D_QK + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            u32x4 raw = u32x4{0u, 0u, 0u, 0u};
            if (head_ok) raw = *(const u32x4 *)(qp + 32 * ks);
            qreg[ks] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    // ---- prologue ----
    if (tid < kTile) {
        tidx[0 * kTile + tid] = fetch_idx(0);
        tidx[1 * kTile + tid] = fetch_idx(1);
    }
    __syncthreads();
    u32x4 pre[LPT];
    if (ntiles > 0) {
        attn_gload<ROW_F, LPT>(pre, kv_seq, tidx, a.row_elems, tid);
        attn_lstore<ROW_F, LPT, ROWB>(pre, tile0, tid);
    }
    __syncthreads();

    f32x4 oacc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) oacc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;                              // running max (log2 units) of head l16
    float l_run = 0.f;                                    // this lane's share of the running sum

#pragma unroll 1
    for (int it = 0; it < ntiles; ++it) {
        const int buf = it & 1;
        int32_t nxt_idx = -1;
        if (tid < kTile) nxt_idx = fetch_idx(it + 2);
        if (it + 1 < ntiles) attn_gload<ROW_F, LPT>(pre, kv_seq, tidx + ((it + 1) % 3) * kTile, a.row_elems, tid);

        if (wave_ok) {
            const unsigned char *tb = tile0 + buf * TILEB;
            // S^T for the tile's 32 rows (two 16-row blocks) x this wave's 16 heads
            f32x4 sacc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
                for (int blk = 0; blk < 2; ++blk) {
                    const bf16x8 ka = *(const bf16x8 *)(tb + (16 * blk + l16) * ROWB + (32 * ks + 8 * g) * 2);
                    sacc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qreg[ks], sacc[blk], 0, 0, 0);
                }
            }
            // validity of the lane's 8 key slots: rows 16blk + 4g + i
            const int32_t *ti = tidx + (it % 3) * kTile;
            float z[8];
            bool ok[8];
            float mx = -INFINITY;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const i32x4 rv = *(const i32x4 *)(ti + 16 * blk + 4 * g);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ok[4 * blk + i] = rv[i] >= 0;
                    z[4 * blk + i] = sacc[blk][i] * a.scale_log2e;
                    if (ok[4 * blk + i]) mx = fmaxf(mx, z[4 * blk + i]);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m_run - m_new);
            float psum = 0.f;
            float pv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pv[j] = ok[j] ? fast_exp2(z[j] - m_new) : 0.f;
                psum += pv[j];
            }
            l_run = l_run * alpha + psum;
            m_run = m_new;
            // rescale O only when some head's max moved (wave-uniform test)
            if (__ballot(alpha != 1.f) != 0ull) {
                float ar[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) ar[i] = __shfl(alpha, 4 * g + i);   // alpha of head row 4g+i
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) oacc[nb][i] *= ar[i];
            }
            bf16x8 pa;
#pragma unroll
            for (int j = 0; j < 8; ++j) pa[j] = (__bf16)pv[j];
            // O += P V : V columns of 4 consecutive tile rows through the LDS transpose read
            const unsigned char *vb0 = tb + (4 * g + (l16 >> 2)) * ROWB + (a.v_off + DVW * vh + 4 * (l16 & 3)) * 2;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(vb0 + nb * 32));
                const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(vb0 + 16 * ROWB + nb * 32));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                const s16x8 vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                oacc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, __builtin_bit_cast(bf16x8, vv), oacc[nb], 0, 0, 0);
            }
        }

        if (it + 1 < ntiles) attn_lstore<ROW_F, LPT, ROWB>(pre, tile0 + (buf ^ 1) * TILEB, tid);
        if (tid < kTile) tidx[((it + 2) % 3) * kTile + tid] = nxt_idx;
        __syncthreads();
    }
    if (!wave_ok) return;

    // ---- epilogue: this wave's heads x its value columns ----
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);                       // every lane: full sum of head l16
    const bool split = a.n_splits > 1;
    if (vh == 0 && g == 0 && head_ok) {
        if (split) {
            float *ml = a.part_ml + ((qrow * a.n_splits + sp) * a.H_q + head) * 2;
            ml[0] = m_run;
            ml[1] = l_tot;
        } else if (a.lse) {
            a.lse[qrow * a.H_q + head] =
                (l_tot > 0.f) ? (m_run + __builtin_log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int hr = 4 * g + i;                         // O row of this lane
        const int hq = 16 * mh + hr;
        const float l = __shfl(l_tot, hr);                // the sum lives in the lanes with l16 == hr
        if (hq >= a.H_q) continue;
        if (split) {
            float *po = a.part_o + ((qrow * a.n_splits + sp) * a.H_q + hq) * D_V + DVW * vh;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) po[16 * nb + l16] = oacc[nb][i];
        } else {
            const float inv = (l > 0.f) ? 1.f / l : 0.f;
            __bf16 *po = (__bf16 *)a.O + (qrow * a.H_q + hq) * D_V + DVW * vh;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) po[16 * nb + l16] = (__bf16)(oacc[nb][i] * inv);
        }
    }
}

// ---- row-slab form (576/512 MLA rows) --------------------------------------------------
// One workgroup (4 waves, one per SIMD, the whole register file) per query and key-slot split;
// tiles of 64 selected rows.  Wave w owns rows 16w..16w+15 of a tile and gathers them straight
// into registers in the A-operand layout of v_mfma_f32_16x16x32_bf16 (lane = row l%16, eight
// features 32 ks + 8 (l/16)): the key side of S^T = K Q^T never passes through LDS, and Q for all
// 32 heads stays in registers.  Only the value columns go to LDS (written from the same registers,
// read back once through the transpose read), and the 64x32 probabilities.
//   producer role (rows of the wave):  S^T, p = 2^(z - m_w) against the wave's own reference
//       maximum m_w = max(running maximum of all waves up to the previous tile, this tile's own)
//   one barrier per tile
//   consumer role (value columns 32w + 128nb + 0..31, all heads):  M = max over the four m_w, the
//       probabilities of wave j are rescaled by 2^(m_j - M) when some m_j differs, O += P V on
//       v_mfma_f32_32x32x16_bf16 whose contraction steps are exactly the four waves' row groups.
// Row sums stay with the producers in their own reference and are combined once at the end.
constexpr int kSlabTile = 64;
constexpr float kLazyLog2 = 8.f;

// Byte offset of value column byte `b` of tile row `row` in the LDS value tile (row stride
// D_V*2, no padding).  The 32-byte unit is xored with the row's low two bits and the 16-byte half
// with bit 2 of the row, so that the four rows of a transpose read and the eight rows of a
// 16-byte store pass fall into distinct banks.
template <int VROWB>
__device__ __forceinline__ int vswz(int row, int b)
{
    return row * VROWB + ((((b >> 5) ^ (row & 3)) << 5) | ((((b >> 4) & 1) ^ ((row >> 2) & 1)) << 4) | (b & 15));
}

// Reductions over the four 16-lane groups of a wave with the row-swap instructions (plain VALU
// latency, no trip through the LDS crossbar).  permlane16_swap(x, x) yields {[r0,r0,r2,r2],
// [r1,r1,r3,r3]} and permlane32_swap(y, y) yields {[lo,lo],[hi,hi]} in units of 16-lane rows.
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

template <int D_QK, int D_V, int V0S>                     // V0S: first 32-feature chunk of a row that holds value columns
__global__ __launch_bounds__(256, 1) void attn_slab_kernel(AttnArgs a)
{
    constexpr int KS = D_QK / 32;                         // contraction steps of S^T
    constexpr int VS = D_V / 32;                          // slab chunks that hold value columns
    constexpr int VROWB = D_V * 2;
    constexpr int VBUFB = kSlabTile * VROWB;
    constexpr int PSTR = kSlabTile * 2 + 16;              // bytes per head row of the P tile
    constexpr int PBUFB = 32 * PSTR;
    constexpr int NBW = D_V / 4 / 32;                     // 32-column blocks per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *vbuf = smem;                           // [2][64][VROWB]
    unsigned char *pbuf = smem + 2 * VBUFB;               // [2][32][PSTR]
    float *mbuf = (float *)(pbuf + 2 * PBUFB);            // [2][4][32] reference maxima of the waves
    float *lbuf = mbuf + 2 * 4 * 32;                      // [4][32] final row sums
    float *abuf = lbuf + 4 * 32;                          // [4][32] per-wave rescale factors

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int l32 = lane & 31, hh = lane >> 5;
    const int64_t qrow = blockIdx.x;
    const int b = (int)(qrow / a.Tq);
    const int sp = blockIdx.y;
    const int slot0 = sp * a.split_len;
    const int slot1 = min(slot0 + a.split_len, a.k_sel);
    const int ntiles = (slot1 - slot0 + kSlabTile - 1) / kSlabTile;

    const int32_t *idx_row = a.idx + qrow * a.k_sel;
    const unsigned short *kv_seq = (const unsigned short *)a.KV + (int64_t)b * a.Lk * a.row_elems;

    // Loads inside the tile loop are unconditional (clamped addresses, result discarded when out
    // of range): the wait counters are positional, and a load that may or may not have been
    // issued would force every later wait down to "everything has landed".
    auto fetch_idx = [&](int it) -> int32_t {             // validated id of the lane's row in tile it
        const int slot = slot0 + it * kSlabTile + 16 * wave + l16;
        const int32_t v = idx_row[min(slot, a.k_sel - 1)];
        return (slot < slot1 && v >= 0 && v < a.Lk) ? v : -1;
    };
    auto gload = [&](u32x4 (&s)[KS], int32_t v) {
        const unsigned short *src = kv_seq + (int64_t)(v < 0 ? 0 : v) * a.row_elems + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s[ks] = *(const u32x4 *)(src + 32 * ks);
    };

    // Q as the B operand: lane (head 16 hb + l16, features 8 g..) for both head blocks
    bf16x8 qreg[2][KS];
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
        const int head = 16 * hb + l16;
        const bool ok = head < a.H_q;
        const unsigned short *qp = (const unsigned short *)a.Q + (qrow * a.H_q + (ok ? head : 0)) * D_QK + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = u32x4{0u, 0u, 0u, 0u};
            if (ok) raw = *(const u32x4 *)(qp + 32 * ks);
            qreg[hb][ks] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    f32x16 oacc[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[nb][i] = 0.f;
    float m_all[2] = {-INFINITY, -INFINITY};              // running maximum over all waves, heads 16hb+l16
    float m_ref[2] = {-INFINITY, -INFINITY};              // this wave's current reference
    float m_c = -INFINITY;                                // running maximum over all waves, head l32
    float l_own[2] = {0.f, 0.f};                          // this lane's share of the wave's row sums (ref m_ref)

    // The slab is one register array that is refilled chunk by chunk: as soon as chunk ks of the
    // current tile has fed its two MFMAs and its LDS store, the same registers receive chunk ks of
    // the next tile, so every load has a whole tile period to land and only one slab is live.
    u32x4 cur[KS];
    int32_t idx_cur = fetch_idx(0);
    int32_t idx_nxt = fetch_idx(1);
    if (ntiles > 0) gload(cur, idx_cur);

    auto step = [&](int it, auto prefetch) {
        const int buf = it & 1;
        const int32_t idx_n2 = fetch_idx(it + 2);
        const unsigned short *nsrc = kv_seq + (int64_t)(idx_nxt < 0 ? 0 : idx_nxt) * a.row_elems + 8 * g;
        // chunk c of the value part holds bytes 64 c + 16 g of the row; the swizzle only touches
        // the low two bits of the 32-byte unit index, so even and odd chunks each sit at a
        // constant stride from one lane-dependent base
        unsigned char *we, *wo;
        {
            unsigned char *vb = vbuf + buf * VBUFB;
            const int row = 16 * wave + l16;
            we = vb + vswz<VROWB>(row, 16 * g);
            wo = vb + vswz<VROWB>(row, 64 + 16 * g);
        }
        // S^T for the wave's 16 rows x 32 heads (one accumulation chain per head block)
        f32x4 s2[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 ka = __builtin_bit_cast(bf16x8, cur[ks]);
            s2[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qreg[0][ks], s2[0], 0, 0, 0);
            s2[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qreg[1][ks], s2[1], 0, 0, 0);
            if (ks >= V0S && ks < V0S + VS) {
                const int c = ks - V0S;
                *(u32x4 *)(((c & 1) ? wo : we) + 128 * (c >> 1)) = cur[ks];
            }
            if constexpr (decltype(prefetch)::value) cur[ks] = *(const u32x4 *)(nsrc + 32 * ks);
        }
        // rows of the lane: 4 g + i; their validity from the row ids held by lanes 0..15
        const unsigned vmask = (unsigned)(__ballot(idx_cur >= 0) & 0xFFFFull);
        unsigned char *pb = pbuf + buf * PBUFB;
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            float z[4];
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool ok = (vmask >> (4 * g + i)) & 1u;
                z[i] = ok ? s2[hb][i] * a.scale_log2e : -INFINITY;
                mx = fmaxf(mx, z[i]);
            }
            mx = xmax16_32(mx);
            // lazy reference: keep the common reference until this tile exceeds it by more than
            // 2^kLazyLog2 (probabilities up to that factor are harmless in bf16/fp32), so that the
            // rescaling paths below run only on real jumps of the maximum
            const float m_new = (mx > m_all[hb] + kLazyLog2) ? mx : m_all[hb];   // m_all >= m_ref always
            const float resc = (m_new == -INFINITY) ? 1.f : fast_exp2(m_ref[hb] - m_new);
            float psum = 0.f;
            s16x4 pk;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = (z[i] == -INFINITY) ? 0.f : fast_exp2(z[i] - m_new);
                psum += p;
                pk[i] = __builtin_bit_cast(short, (__bf16)p);
            }
            l_own[hb] = l_own[hb] * resc + psum;
            m_ref[hb] = m_new;
            *(s16x4 *)(pb + (16 * hb + l16) * PSTR + (16 * wave + 4 * g) * 2) = pk;
            if (g == 0) mbuf[(buf * 4 + wave) * 32 + 16 * hb + l16] = m_new;
        }
        __syncthreads();

        // transpose reads: the wave's value columns are 32 w + 128 nb + (0..31), so that nb only
        // moves address bits above the swizzled ones; rows 16 j + 8 hh + (l16>>2) and + 4
        const unsigned char *vb = vbuf + buf * VBUFB;
        const int trow = 8 * hh + (l16 >> 2);
        const int tcb = (32 * wave + 16 * (g & 1) + 4 * (l16 & 3)) * 2;
        const unsigned char *vr0 = vb + vswz<VROWB>(trow, tcb);
        const unsigned char *vr1 = vb + vswz<VROWB>(trow + 4, tcb);
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        bf16x8 pa[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) pa[j] = *(const bf16x8 *)(pb + l32 * PSTR + (16 * j + 8 * hh) * 2);
        // the value operands of row group j+1 are requested before the MFMAs of group j issue
        s16x4 vq[2][NBW][2];
        auto vload = [&](int j) {
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                vq[j & 1][nb][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vr0 + 16 * j * VROWB + 256 * nb));
                vq[j & 1][nb][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vr1 + 16 * j * VROWB + 256 * nb));
            }
        };
        vload(0);

        // maxima of the four row groups: for the producer heads 16hb + l16 (next tile's reference)
        // and for the head l32 whose probabilities the lane feeds to the MFMA as the A operand
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            const float *mp = mbuf + buf * 128 + 16 * hb + l16;
            m_all[hb] = fmaxf(fmaxf(mp[0], mp[32]), fmaxf(mp[64], mp[96]));
        }
        float mjc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) mjc[j] = mbuf[buf * 128 + 32 * j + l32];
        const float m_new_c = fmaxf(fmaxf(mjc[0], mjc[1]), fmaxf(mjc[2], mjc[3]));
        const float alpha = (m_new_c == -INFINITY) ? 1.f : fast_exp2(m_c - m_new_c);
        m_c = m_new_c;
        float fj[4];
        bool any_f = false;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            fj[j] = (m_new_c == -INFINITY) ? 1.f : fast_exp2(mjc[j] - m_new_c);
            any_f |= (fj[j] != 1.f);
        }
        if (__ballot(alpha != 1.f) != 0ull) {
            // the rescale factors of the 16 heads a lane accumulates, through a per-wave LDS row
            float *ab = abuf + wave * 32;
            if (hh == 0) ab[l32] = alpha;
            f32x4 ar[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) ar[q] = *(const f32x4 *)(ab + 8 * q + 4 * hh);
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[nb][i] *= ar[i >> 2][i & 3];
        }
        const bool scale_p = __ballot(any_f) != 0ull;
        if (scale_p) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) pa[j][e] = (__bf16)((float)pa[j][e] * fj[j]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j + 1 < 4) vload(j + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                const s16x4 v0 = vq[j & 1][nb][0], v1 = vq[j & 1][nb][1];
                const s16x8 vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa[j], __builtin_bit_cast(bf16x8, vv), oacc[nb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        idx_cur = idx_nxt;
        idx_nxt = idx_n2;
    };

    {
        int it = 0;
#pragma unroll 1
        for (; it + 1 < ntiles; ++it) step(it, std::true_type{});
        if (it < ntiles) step(it, std::false_type{});
    }

    // ---- epilogue: combine the producers' row sums, normalise, store ----
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
        const float l = xsum16_32(l_own[hb]);
        // bring the wave's sum to the common maximum before publishing it
        const float f = (m_all[hb] == -INFINITY) ? 0.f : fast_exp2(m_ref[hb] - m_all[hb]);
        if (g == 0) lbuf[wave * 32 + 16 * hb + l16] = l * f;
    }
    __syncthreads();
    const float l_head = lbuf[l32] + lbuf[32 + l32] + lbuf[64 + l32] + lbuf[96 + l32];   // head l32
    const float m_head = m_c;
    const bool split = a.n_splits > 1;
    if (wave == 0 && hh == 0 && l32 < a.H_q) {
        if (split) {
            float *ml = a.part_ml + ((qrow * a.n_splits + sp) * a.H_q + l32) * 2;
            ml[0] = m_head;
            ml[1] = l_head;
        } else if (a.lse) {
            a.lse[qrow * a.H_q + l32] =
                (l_head > 0.f) ? (m_head + __builtin_log2f(l_head)) * 0.6931471805599453f : -INFINITY;
        }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int hq = 8 * (i >> 2) + 4 * hh + (i & 3);   // O row (head) of accumulator element i
        const float l = __shfl(l_head, hq);
        if (hq >= a.H_q) continue;
        if (split) {
            float *po = a.part_o + ((qrow * a.n_splits + sp) * a.H_q + hq) * D_V + 32 * wave + l32;
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) po[128 * nb] = oacc[nb][i];
        } else {
            const float inv = (l > 0.f) ? 1.f / l : 0.f;
            __bf16 *po = (__bf16 *)a.O + (qrow * a.H_q + hq) * D_V + 32 * wave + l32;
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) po[128 * nb] = (__bf16)(oacc[nb][i] * inv);
        }
    }
}

// Combine the per-split partials of one (query, head): O = sum_s O_s 2^(m_s-m) / sum_s l_s 2^(m_s-m).
// One workgroup per (query, head); a thread owns 4 consecutive value columns.
template <int D_V>
__global__ __launch_bounds__(D_V / 4) void attn_merge_kernel(AttnArgs a)
{
    const int64_t qrow = blockIdx.x;
    const int h = blockIdx.y;
    const int v = threadIdx.x * 4;
    const float *ml = a.part_ml + ((qrow * a.n_splits) * a.H_q + h) * 2;
    const int64_t ml_stride = (int64_t)a.H_q * 2;
    float m = -INFINITY;
    for (int s = 0; s < a.n_splits; ++s) m = fmaxf(m, ml[s * ml_stride]);
    float l = 0.f;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    const float *po = a.part_o + ((qrow * a.n_splits) * a.H_q + h) * D_V + v;
    for (int s = 0; s < a.n_splits; ++s) {
        const float ms = ml[s * ml_stride], ls = ml[s * ml_stride + 1];
        const float sc = (ms == -INFINITY) ? 0.f : fast_exp2(ms - m);
        l += ls * sc;
        const f32x4 x = *(const f32x4 *)(po + (int64_t)s * a.H_q * D_V);
        o += x * sc;
    }
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    __bf16 *out = (__bf16 *)a.O + (qrow * a.H_q + h) * D_V + v;
#pragma unroll
    for (int j = 0; j < 4; ++j) out[j] = (__bf16)(o[j] * inv);
    if (threadIdx.x == 0 && a.lse)
        a.lse[qrow * a.H_q + h] = (l > 0.f) ? (m + __builtin_log2f(l)) * 0.6931471805599453f : -INFINITY;
}

template <int D_QK, int D_V, int ROW_F>
hipError_t launch_t(const AttnArgs &a, hipStream_t st)
{
    constexpr int ROWB = ROW_F * 2 + 16;
    const size_t lds = (size_t)2 * kTile * ROWB + 3 * kTile * sizeof(int32_t);
    static hipError_t attr = hipFuncSetAttribute((const void *)attn_kernel<D_QK, D_V, ROW_F>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return attr;
    dim3 grid((unsigned)((int64_t)a.B * a.Tq), (unsigned)a.n_splits);
    hipLaunchKernelGGL((attn_kernel<D_QK, D_V, ROW_F>), grid, dim3(256), lds, st, a);
    return hipGetLastError();
}

template <int D_QK, int D_V, int V0S>
hipError_t launch_slab(const AttnArgs &a, hipStream_t st)
{
    const size_t lds = (size_t)2 * kSlabTile * D_V * 2 + 2 * 32 * (kSlabTile * 2 + 16) + (2 * 4 * 32 + 4 * 32 + 4 * 32) * sizeof(float);
    static hipError_t attr = hipFuncSetAttribute((const void *)attn_slab_kernel<D_QK, D_V, V0S>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return attr;
    dim3 grid((unsigned)((int64_t)a.B * a.Tq), (unsigned)a.n_splits);
    hipLaunchKernelGGL((attn_slab_kernel<D_QK, D_V, V0S>), grid, dim3(256), lds, st, a);
    return hipGetLastError();
}

} // namespace

bool attn_shape_supported(int d_qk, int d_v)
{
    return (d_qk == 576 && d_v == 512) || (d_qk == 64 && d_v == 64);
}

hipError_t launch_attn(const AttnArgs &a, int d_qk, int d_v, hipStream_t st)
{
    if ((int64_t)a.B * a.Tq <= 0) return hipSuccess;
    if (d_qk == 576 && d_v == 512) {
        static const bool tile_form = getenv("IC_ATTN_TILE") != nullptr;
        if (!tile_form && a.v_off == 0) return launch_slab<576, 512, 0>(a, st);
        return launch_t<576, 512, 576>(a, st);
    }
    if (d_qk == 64 && d_v == 64) return launch_t<64, 64, 128>(a, st);
    return hipErrorInvalidValue;
}

hipError_t launch_attn_merge(const AttnArgs &a, int d_v, hipStream_t st)
{
    if ((int64_t)a.B * a.Tq <= 0) return hipSuccess;
    dim3 grid((unsigned)((int64_t)a.B * a.Tq), (unsigned)a.H_q);
    if (d_v == 512)
        hipLaunchKernelGGL((attn_merge_kernel<512>), grid, dim3(128), 0, st, a);
    else if (d_v == 64)
        hipLaunchKernelGGL((attn_merge_kernel<64>), grid, dim3(16), 0, st, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

} // namespace ic
