// Sparse MQA core attention over the selected KV rows (paper Sec. 2.1: the main attention is
// computed only over the top-k subset; MLA form, one shared KV row per position).
//
// Two kernels.  MLA rows whose values are their first features (576 / 512) take the row-slab
// form further down: one workgroup per CU, 64-row tiles, walking a chain of queries when there are
// more queries than CUs, or one (query, split) each when there are fewer (decode).  Every other
// supported layout takes the small-tile form described here.
//
// Small-tile form: one workgroup (4 waves) per query token and key-slot split; two workgroups
// fit a CU (75 KB of LDS, <= 256 VGPRs each) so that one computes while the other waits for its
// gather.  Tiles of 32 selected rows are gathered with 16-byte coalesced loads (each row is
// contiguous) into a double-buffered LDS tile, row-major.  A wave owns 16 of the 32 heads and half
// of the value columns, and runs its own online softmax over every row of the tile:
//   S^T = K Q^T   v_mfma_f32_16x16x32_bf16, A = tile rows (16-byte LDS reads), B = Q (registers)
//   P   = exp2(S^T * scale*log2e - m)   in the result layout: a lane owns one head, 8 keys
//   O  += P V     same MFMA; P is already an A operand (its contraction slots are whatever keys
//                 the lane holds), and V comes out of the SAME row-major tile through the LDS
//                 transpose read ds_read_b64_tr_b16, which hands a lane one value column of four
//                 consecutive tile rows.  No transposed copy of V is ever made.
// The two waves of a head group compute the same S^T (cheap next to the gather) and therefore
// the same softmax statistics, so no exchange between waves is ever needed.
//
// Splits (both forms): a split stores its own normalised output in bf16 together with its
// reference maximum and row sum; attn_merge_kernel weighs the splits by their share of the total
// row sum.
#include "ic_common.hpp"
#include <type_traits>

namespace ic {

namespace {

constexpr int kTile = 32;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Tile staging.  A thread owns tile row tid / 8 and the 16-byte chunks (tid % 8) + 8 r of that
// row: eight neighbouring lanes read one full 128-byte line, and no index needs a division.
template <int ROW_F, int LPT, bool PG>
__device__ __forceinline__ void attn_gload(u32x4 (&pre)[LPT], const unsigned short *kv_seq, const int32_t *ti,
                                           int row_elems, int tid, const PagedView &pv, int b)
{
    constexpr int CPR = ROW_F / 8;
    const int row = tid >> 3, c0 = tid & 7;
    const int32_t v = ti[row];                             // empty slots read row 0 (never a page-table entry)
    const int64_t prow = v < 0 ? 0 : (PG && pv.page_table ? paged_row(pv, b, v) : (int64_t)v);
    const unsigned short *src = kv_seq + prow * row_elems + c0 * 8;
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

// PG: the KV cache may be ragged and / or paged (a.pv); false compiles the dense layout only.
template <int D_QK, int D_V, int ROW_F, bool PG>
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
    const unsigned short *kv_seq = (const unsigned short *)a.KV + (PG && a.pv.page_table ? 0 : (int64_t)b * a.Lk * a.row_elems);
    const int Lk_b = PG && a.pv.seq_lens ? min(a.pv.seq_lens[b], a.Lk) : a.Lk;     // ragged cache: rows of this sequence

    auto fetch_idx = [&](int it) -> int32_t {             // threads 0..31: validated row id of a slot
        const int slot = slot0 + it * kTile + tid;
        int32_t v = -1;
        if (it < ntiles && slot < slot1) v = idx_row[slot];
        return (v >= 0 && v < Lk_b) ? v : -1;
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
        attn_gload<ROW_F, LPT, PG>(pre, kv_seq, tidx, a.row_elems, tid, a.pv, b);
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
        if (it + 1 < ntiles) attn_gload<ROW_F, LPT, PG>(pre, kv_seq, tidx + ((it + 1) % 3) * kTile, a.row_elems, tid, a.pv, b);

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
        // a split stores its own normalised output (bf16, like the final one); the merge weighs the
        // splits by their share of the total row sum
        const float inv = (l > 0.f) ? 1.f / l : 0.f;
        __bf16 *po = (split ? a.part_o + ((qrow * a.n_splits + sp) * a.H_q + hq) * D_V
                            : (__bf16 *)a.O + (qrow * a.H_q + hq) * D_V) + DVW * vh;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) po[16 * nb + l16] = (__bf16)(oacc[nb][i] * inv);
    }
}

// ---- row-slab form (576/512 MLA rows) --------------------------------------------------
// One workgroup (4 waves, one per SIMD, the whole register file) per CU; tiles of 64 selected
// rows, two tiles resident in LDS.  Wave w owns rows 16w..16w+15 of a tile in the producer role
// and value columns 32w + 128nb + (0..31) in the consumer role:
//   gather    eight lanes fetch one 128-byte line of a row (the access shape the vector memory
//             path serves fastest), 18 loads per lane and tile, refilled in place one tile ahead
//   stage     the wave stores its own 16 rows to the LDS tile (after the barrier of the previous
//             tile, so nobody still reads that buffer) and reads them back in the A-operand
//             layout of v_mfma_f32_16x16x32_bf16: every key byte is written and read once
//   produce   S^T = K Q^T for 16 rows x 32 heads (Q stays in registers), p = 2^(z - m_w) against
//             a lazily updated reference maximum, P and m_w to LDS
//   one barrier per tile
//   consume   M = max over the four m_w; probabilities of wave j are rescaled by 2^(m_j - M) when
//             some m_j differs; O += P V on v_mfma_f32_32x32x16_bf16, whose four contraction
//             steps are exactly the four waves' row groups; V comes out of the same row-major
//             tile through the LDS transpose read, once per element.
// Row sums stay with the producers in their own reference and are combined once at the end.
// The consumer role lags the producer role by one tile (a step = produce tile it, consume tile
// it-1), so the previous tile's operand reads run under the softmax arithmetic and the staging
// stores under the PV MFMAs.
// Between two queries of a chain: the last two steps already gather and stage the next query's
// first tiles; one wave loads the next Q straight into the accumulation registers while the
// outputs are stored and hands it to the other waves through the tile buffer that is idle at
// that moment (see the driver at the end of the kernel).
constexpr int kSlabTile = 64;
constexpr float kLazyLog2 = 8.f;

// Tile rows in LDS are padded by 32 bytes (row stride 1184 for rows of 1152) and not swizzled.  Measured on this part
// with every wave of a CU reading: the 16-byte A-operand read of 16 rows (lane = row, same piece in every lane) takes
// 2.3 ticks per instruction with rows 1152 + an odd multiple of 32 bytes apart, as a contiguous read does, and 3.8
// with rows 1152 apart under either of two XOR swizzles; an 8-byte transpose read serves 32 lanes per pass out of 64
// banks of 4 bytes, i.e. 64 contiguous bytes of four rows, and rows 2 x 1184 apart start 64 bytes apart modulo 256:
// conflict-free when the four rows of a pass are two apart (even rows, then odd rows).
constexpr int kSlabPad = 32;

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

// Validity of the 16 rows of a wave from the two ballots over the gather lanes (lane 8r' + piece
// holds row r' of the first / second eight rows): bit r of the result is row r.
__device__ __forceinline__ unsigned rows_mask(unsigned long long ba, unsigned long long bb)
{
    // byte r of a ballot is 0x00 or 0xFF; keep bit 0 of each byte and gather the eight bits in the
    // top byte of a product whose partial sums never collide
    const unsigned long long ones = 0x0101010101010101ull, pack = 0x0102040810204080ull;
    const unsigned lo = (unsigned)(((ba & ones) * pack) >> 56);
    const unsigned hi = (unsigned)(((bb & ones) * pack) >> 56);
    return lo | (hi << 8);
}

// SPLIT: blockIdx.y selects a.split_len key slots of the query and the result is a partial
// (unnormalised accumulators, reference maximum, row sum) for the merge kernel.
template <int D_QK, int D_V, bool PG, bool SPLIT>         // value columns = the first D_V features of a row; PG as above
__global__ __launch_bounds__(256, 1) void attn_slab_kernel(AttnArgs a)
{
    constexpr int KS = D_QK / 32;                         // contraction steps of S^T = 16-byte chunks per gather lane
    constexpr int ROWB = D_QK * 2 + kSlabPad;             // LDS row stride
    static_assert((D_QK * 2) % 128 == 0 && D_V % 128 == 0 && KS % 2 == 0, "row = whole 128-byte windows");
    constexpr int TBUFB = kSlabTile * ROWB;
    constexpr int PSTR = kSlabTile * 2 + 16;              // bytes per head row of the P tile
    constexpr int PBUFB = 32 * PSTR;
    constexpr int NBW = D_V / 4 / 32;                     // 32-column blocks per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *tbuf = smem;                           // [2][64][ROWB]
    unsigned char *pbuf = smem + 2 * TBUFB;               // [2][32][PSTR]
    float *lbuf = (float *)(pbuf + 2 * PBUFB);            // [4][32] final row sums
    float *abuf = lbuf + 4 * 32;                          // [4][32] per-wave rescale factors

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int l32 = lane & 31, hh = lane >> 5;
    const int gr = lane >> 3, gp = lane & 7;              // gather role: row (and row + 8), 16-byte piece
    const int sp = SPLIT ? (int)blockIdx.y : 0;
    const int slot0 = SPLIT ? sp * a.split_len : 0;
    const int slot1 = SPLIT ? min(slot0 + a.split_len, a.k_sel) : a.k_sel;
    const int ntiles = (slot1 - slot0 + kSlabTile - 1) / kSlabTile;
    // Chained form (whole selections of at least three tiles, grid smaller than the number of
    // queries): the workgroup walks queries blockIdx.x, + gridDim.x, ... and treats their tiles as
    // one stream, so that the gather and staging of the next query's first tiles and the load of
    // its Q run under the last steps and the output stores of the current one.
    const int64_t nq = (int64_t)a.B * a.Tq;
    const bool chain = !SPLIT && ntiles >= 3 && (int64_t)gridDim.x < nq;   // workgroup-uniform
    int64_t qrow = blockIdx.x;
    if (chain && (gridDim.x & 7u) == 0) {
        // Workgroup ids are dealt round-robin over the 8 XCDs, each with its own L2.  Give XCD x the
        // contiguous queries x * grid/8 .. of every round of `grid` queries: neighbouring queries
        // select largely the same rows, which then meet in one L2.
        const unsigned per = gridDim.x >> 3;
        qrow = (int64_t)(blockIdx.x & 7u) * per + (blockIdx.x >> 3);
    }
    int64_t qnext = chain ? qrow + gridDim.x : nq;        // >= nq: this is the workgroup's last query

    // what the gather needs to know about a query: its index row, its cache and its length
    // nt: tiles of the query in the chained stream.  When the selection is known to be a causal top-k, a row near the
    // start of a sequence holds fewer than k_sel entries and ends in -1s: its tiles behind the last entry are left
    // out (never fewer than three per query: the stream looks three tiles ahead and knows two queries at a time).
    struct Src { const int32_t *idx_row; const unsigned short *kv; int b, len, nt; bool live; };
    auto src_of = [&](int64_t q) {
        Src r;
        r.live = q < nq;
        const int64_t qq = r.live ? q : (int64_t)blockIdx.x;          // a dead source still reads valid memory
        r.b = (int)(qq / a.Tq);
        r.nt = ntiles;
        if (!SPLIT && a.causal_pos0 >= 0) {
            const int64_t held = a.causal_pos0 + qq % a.Tq + 1;       // entries the row can hold
            if (held < a.k_sel) r.nt = max(3, (int)((held + kSlabTile - 1) / kSlabTile));
            r.nt = min(r.nt, ntiles);
        }
        r.idx_row = a.idx + qq * a.k_sel;
        r.kv = (const unsigned short *)a.KV + (PG && a.pv.page_table ? 0 : (int64_t)r.b * a.Lk * a.row_elems);
        r.len = PG && a.pv.seq_lens ? min(a.pv.seq_lens[r.b], a.Lk) : a.Lk;   // ragged cache: rows of this sequence
        return r;
    };
    Src cs = src_of(qrow), ns = src_of(qnext);            // current and next query

    // Loads inside the tile loop are unconditional (clamped addresses, result discarded when out
    // of range): the wait counters are positional, and a load that may or may not have been
    // issued would force every later wait down to "everything has landed".
    struct Ids { int32_t lo, hi; };                       // validated ids of tile rows 16w+gr and 16w+gr+8
    // tile `it` of the stream: tiles at or beyond ntiles are the first tiles of the next query
    auto fetch_ids = [&](int it) -> Ids {
        const bool nx = !SPLIT && it >= cs.nt;
        const Src &q = nx ? ns : cs;
        const int s_lo = slot0 + (nx ? it - cs.nt : it) * kSlabTile + 16 * wave + gr, s_hi = s_lo + 8;
        const int32_t v_lo = q.idx_row[min(s_lo, a.k_sel - 1)], v_hi = q.idx_row[min(s_hi, a.k_sel - 1)];
        Ids r;
        // no short-circuit: one basic block, so the loaded ids are not waited for before their use
        r.lo = ((int)q.live & (int)(s_lo < slot1) & (int)(v_lo >= 0) & (int)(v_lo < q.len)) ? v_lo : -1;
        r.hi = ((int)q.live & (int)(s_hi < slot1) & (int)(v_hi >= 0) & (int)(v_hi < q.len)) ? v_hi : -1;
        return r;
    };
    auto row_ptr = [&](int32_t v, int it) {
        const Src &q = (!SPLIT && it >= cs.nt) ? ns : cs;
        // empty slots read row 0 of the cache (never a page-table entry: the sequence may own no page)
        const int64_t prow = v < 0 ? 0 : (PG && a.pv.page_table ? paged_row(a.pv, q.b, v) : (int64_t)v);
        return q.kv + prow * a.row_elems + 8 * gp;
    };
    auto ids_mask = [&](const Ids &d) { return rows_mask(__ballot(d.lo >= 0), __ballot(d.hi >= 0)); };

    // Q as the B operand: lane (head 16 hb + l16, features 8 g..) for both head blocks.  All of its
    // loads are issued before anything waits for one of them, and the ids and rows of the first
    // tile are requested in their shadow.
    u32x4 qraw[2][KS];
    auto load_q = [&](int64_t q) {
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            const int head = 16 * hb + l16;
            const bool ok = head < a.H_q;
            const unsigned short *qp = (const unsigned short *)a.Q + (q * a.H_q + (ok ? head : 0)) * D_QK + 8 * g;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                qraw[hb][ks] = u32x4{0u, 0u, 0u, 0u};
                if (ok) qraw[hb][ks] = *(const u32x4 *)(qp + 32 * ks);
            }
        }
    };
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    f32x16 oacc[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[nb][i] = 0.f;
    float m_all[2] = {-INFINITY, -INFINITY};              // common reference of all waves, heads 16hb+l16
    float m_ref[2] = {-INFINITY, -INFINITY};              // this wave's current reference
    float m_c = -INFINITY;                                // common reference, head l32
    float l_own[2] = {0.f, 0.f};                          // this lane's share of the wave's row sums (ref m_ref)

    // LDS addresses of the lane in its three roles (byte offsets inside one tile buffer)
    const int st_off = (16 * wave + gr) * ROWB + (gp << 4);                           // + 8 rows for odd chunks
    const int ka_row = (16 * wave + l16) * ROWB;
    const int ka_e = ka_row + (g << 4);                                               // even contraction steps
    const int ka_o = ka_row + ((4 + g) << 4);                                         // odd ones
    // transpose reads: the four rows of a read are two apart; within a group of eight rows the first read takes the
    // even rows (contraction positions 0-3), the second the odd ones (positions 4-7), and P is written in that order
    const int tr_row = 8 * hh + 2 * (l16 >> 2);
    const int tr_slot = 4 * (wave & 1) + 2 * (g & 1) + ((l16 & 3) >> 1);
    const int tr0 = tr_row * ROWB + 128 * (wave >> 1) + (tr_slot << 4) + 8 * (l16 & 1);
    const int tr1 = tr0 + ROWB;

    // The gather registers are refilled chunk by chunk: as soon as chunk ks of tile t+1 has been
    // stored to LDS, the same registers receive chunk ks of tile t+2.
    u32x4 cur[KS];
    auto gload = [&](const Ids &d, int it) {
        const unsigned short *pl = row_ptr(d.lo, it), *ph = row_ptr(d.hi, it);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cur[ks] = *(const u32x4 *)(((ks & 1) ? ph : pl) + 64 * (ks >> 1));
    };
    unsigned vm_cur, vm_n1;
    Ids ids_n2;
    bf16x8 qreg[2][KS];
    // pin Q to the accumulation half of the register file (MFMA reads B operands from there
    // directly): the vector half is needed for the gather and the LDS operands
    auto pin_q = [&]() {
#pragma unroll
        for (int hb = 0; hb < 2; ++hb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u32x4 raw = qraw[hb][ks];
                asm volatile("" : "+a"(raw));
                qreg[hb][ks] = __builtin_bit_cast(bf16x8, raw);
            }
    };
    // Chained form: Q of the next query is loaded while the outputs of the current one are stored.  Its
    // only use is pinned to the accumulation registers (settle_q), so the loads target those registers
    // directly and take no vector registers; they are issued before the epilogue and waited for in
    // settle_q.  (With fewer than 32 heads the loads sit under a lane mask; there they are inline loads
    // the compiler does not count, which only makes its own waits conservative, and settle_q's explicit
    // wait ties every later use to them.)
    // Only wave 0 loads (each load touches 16 rows of Q, so four waves loading the same 36 KB keep the
    // CU's one address unit busy for 2.8 us); it then hands Q to the other waves through the tile
    // buffer that is free between two queries, in the very lane order the operand has.
    auto load_q_direct = [&](int64_t q) {
        if (wave_u != 0) return;
        // the lane's offset into Q is recomputed from the lane id here: kept live across the tile
        // loop it would be spilled, and its reload would wait behind the gathers in flight
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int hd = ln & 15, gq = ln >> 4;
        const unsigned short *q0 = (const unsigned short *)a.Q + q * a.H_q * D_QK + 8 * gq;
        if (a.H_q >= 32) {                                // workgroup-uniform: every lane has a head
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const unsigned short *src = q0 + (16 * hb + hd) * D_QK + 32 * ks;
                    qreg[hb][ks] = __builtin_bit_cast(bf16x8, *(const u32x4 *)src);
                }
        } else {
#pragma unroll
            for (int hb = 0; hb < 2; ++hb) {
                const int head = 16 * hb + hd;
                const bool ok = head < a.H_q;
                u32x4 raw[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) raw[ks] = u32x4{0u, 0u, 0u, 0u};
                if (ok) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        const unsigned short *src = q0 + head * D_QK + 32 * ks;
                        asm volatile("global_load_dwordx4 %0, %1, off" : "+a"(raw[ks]) : "v"(src));
                    }
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) qreg[hb][ks] = __builtin_bit_cast(bf16x8, raw[ks]);
            }
        }
    };
    auto settle_q = [&](unsigned char *qx) {              // qx: 2 * KS KiB of free LDS
        unsigned char *mine = qx + lane * 16;
        if (wave_u == 0) {
            asm volatile("s_waitcnt vmcnt(0)");
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    u32x4 raw = __builtin_bit_cast(u32x4, qreg[hb][ks]);
                    asm volatile("" : "+a"(raw));
                    qreg[hb][ks] = __builtin_bit_cast(bf16x8, raw);
                    *(u32x4 *)(mine + (hb * KS + ks) * 1024) = raw;
                }
        }
        __syncthreads();
        if (wave_u != 0) {
            u32x4 raw[2][KS];
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) raw[hb][ks] = *(const u32x4 *)(mine + (hb * KS + ks) * 1024);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    asm volatile("" : "+a"(raw[hb][ks]));
                    qreg[hb][ks] = __builtin_bit_cast(bf16x8, raw[hb][ks]);
                }
        }
    };
    int g0 = 0;                                           // stream position of the query's tile 0 (buffer parity)
    {
        const Ids d0 = fetch_ids(0), d1 = fetch_ids(1);
        ids_n2 = fetch_ids(2);
        __builtin_amdgcn_sched_barrier(0);
        // one wave loads Q (see load_q_direct above) and hands it over; its loads go out behind the
        // id fetches, so that the ids, and with them the first gather, do not wait for Q
        if (wave_u == 0) load_q(qrow);
        gload(d0, 0);
        __builtin_amdgcn_sched_barrier(0);
        {   // Q from wave 0 to the others through the second tile buffer (unused until step 0 stages tile 1)
            unsigned char *mine = tbuf + TBUFB + lane * 16;
            if (wave_u == 0) {
#pragma unroll
                for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) *(u32x4 *)(mine + (hb * KS + ks) * 1024) = qraw[hb][ks];
            }
            __syncthreads();
            if (wave_u != 0) {
#pragma unroll
                for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) qraw[hb][ks] = *(const u32x4 *)(mine + (hb * KS + ks) * 1024);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        pin_q();
        vm_cur = ids_mask(d0);
        vm_n1 = ids_mask(d1);
        const unsigned short *pl = row_ptr(d1.lo, 1), *ph = row_ptr(d1.hi, 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            *(u32x4 *)(tbuf + st_off + (ks & 1) * 8 * ROWB + 128 * (ks >> 1)) = cur[ks];
            cur[ks] = *(const u32x4 *)(((ks & 1) ? ph : pl) + 64 * (ks >> 1));
        }
    }

    // One step = the producer role for tile `it` and the consumer role for tile it-1 (have_prev).
    // stage_next: tile it+1 exists (store it);  load_next2: tile it+2 exists (refill the gather
    // registers).  The LDS pipeline is the busiest unit of this kernel (it spends about as long on
    // a 4-byte access as on a 16-byte one), so everything that crosses it is packed into wide
    // instructions and spread over the step: A-operand reads under the S^T MFMAs, the previous
    // tile's P/V operand reads under the softmax arithmetic, the staging stores under the PV MFMAs.
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    auto step = [&](int it, auto have_prev, auto have_cur, auto stage_next, auto load_next2) {
        constexpr bool kPrev = decltype(have_prev)::value, kCur = decltype(have_cur)::value;
        constexpr bool kStage = decltype(stage_next)::value, kLoad = decltype(load_next2)::value;
        const int buf = (g0 + it) & 1;
        Ids ids_n3 = ids_n2;
        if constexpr (kCur) ids_n3 = fetch_ids(it + 3);
        const unsigned char *tb = tbuf + buf * TBUFB;                 // tile it
        const unsigned char *tp = tbuf + (buf ^ 1) * TBUFB;           // tile it-1
        unsigned char *pb = pbuf + buf * PBUFB;                       // P of tile it
        const unsigned char *pp = pbuf + (buf ^ 1) * PBUFB;           // P of tile it-1

        // reference maxima of tile it-1 first: the softmax of tile it builds on them
        f32x4 mjc = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if constexpr (kPrev) mjc = *(const f32x4 *)(pp + l32 * PSTR + kSlabTile * 2);

        // consumer operands of tile it-1: probabilities of head l32 and every value operand.  The first of these
        // reads go out under the last S^T MFMAs (kConsPer per contraction step from step kConsFrom on: measured, 3
        // from step 10 on is 2.6 % faster than all of them behind the MFMAs and 2 % faster than all of them under
        // the MFMAs), the rest stream in while the softmax below keeps the vector ALU busy.
        bf16x8 pa[4];
        s16x4 vq[4][NBW][2];
        constexpr int NCR = 4 + 8 * NBW;                  // consumer reads of a step
        constexpr int kConsFrom = KS > 10 ? 10 : KS, kConsPer = 3;
        static_assert((KS - kConsFrom) * kConsPer <= NCR, "no more early reads than there are reads");
        auto cons_read = [&](int n) __attribute__((always_inline)) {
            if constexpr (kPrev) {
                if (n < 4) {
                    pa[n] = *(const bf16x8 *)(pp + l32 * PSTR + (16 * n + 8 * hh) * 2);
                } else if (n < NCR) {
                    const int m = n - 4, j = m / (2 * NBW), nb = (m >> 1) % NBW;
                    vq[j][nb][m & 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4 *)(tp + ((m & 1) ? tr1 : tr0) + 16 * j * ROWB + 256 * nb));
                }
            }
        };

        // S^T for the wave's 16 rows x 32 heads: two accumulation chains per head block
        f32x4 s4[2][2];
        if constexpr (kCur) {
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                for (int par = 0; par < 2; ++par) s4[hb][par] = f32x4{0.f, 0.f, 0.f, 0.f};
            constexpr int KRING = 4;                      // A-operand reads in flight ahead of the MFMAs
            bf16x8 ka[KRING];
            auto ka_read = [&](int ks) { return *(const bf16x8 *)(tb + ((ks & 1) ? ka_o : ka_e) + 128 * (ks >> 1)); };
#pragma unroll
            for (int r = 0; r < KRING; ++r) ka[r] = ka_read(r);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s4[0][ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks % KRING], qreg[0][ks], s4[0][ks & 1], 0, 0, 0);
                s4[1][ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks % KRING], qreg[1][ks], s4[1][ks & 1], 0, 0, 0);
                if (ks + KRING < KS) ka[ks % KRING] = ka_read(ks + KRING);
                if (ks >= kConsFrom) {
#pragma unroll
                    for (int n = (ks - kConsFrom) * kConsPer; n < (ks - kConsFrom + 1) * kConsPer; ++n) cons_read(n);
                }
            }
        }
        {
            constexpr int n0 = kCur ? (KS - kConsFrom) * kConsPer : 0;
#pragma unroll
            for (int n = n0; n < NCR; ++n) cons_read(n);
        }

        float alpha = 1.f, fj[4] = {1.f, 1.f, 1.f, 1.f};
        bool any_f = false;
        if constexpr (kPrev) {
            // new common reference of head l32 (= 16 (g&1) + l16); the producer role needs it for
            // heads l16 and 16 + l16, one of which lives in the neighbouring 16-lane group
            const float m_new_c = fmaxf(fmaxf(mjc[0], mjc[1]), fmaxf(mjc[2], mjc[3]));
            const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(m_new_c), __float_as_uint(m_new_c), false, false);
            m_all[0] = __uint_as_float(sw[0]);            // groups [0,0,2,2]: head l16
            m_all[1] = __uint_as_float(sw[1]);            // groups [1,1,3,3]: head 16 + l16
            alpha = (m_new_c == -INFINITY) ? 1.f : fast_exp2(m_c - m_new_c);
            m_c = m_new_c;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                fj[j] = (m_new_c == -INFINITY) ? 1.f : fast_exp2(mjc[j] - m_new_c);
                any_f |= (fj[j] != 1.f);
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        // producer role: rows 4 g + i of the wave.  A head row of the P tile is 128 bytes of
        // probabilities followed by the four waves' reference maxima in its 16 bytes of padding.
        if constexpr (kCur) {
#pragma unroll
            for (int hb = 0; hb < 2; ++hb) {
                float z[4];
                float mx = -INFINITY;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool ok = (vm_cur >> (4 * g + i)) & 1u;
                    z[i] = ok ? (s4[hb][0][i] + s4[hb][1][i]) * a.scale_log2e : -INFINITY;
                    mx = fmaxf(mx, z[i]);
                }
                mx = xmax16_32(mx);
                // lazy reference: keep the common reference until this tile exceeds it by more than
                // 2^kLazyLog2 (probabilities up to that factor are harmless in bf16/fp32), so that
                // the rescaling paths below run only on real jumps of the maximum
                const float m_new = (mx > m_all[hb] + kLazyLog2) ? mx : m_all[hb];   // m_all >= m_ref always
                const float resc = (m_new == -INFINITY) ? 1.f : fast_exp2(m_ref[hb] - m_new);
                float psum = 0.f;
                short pk[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p = (z[i] == -INFINITY) ? 0.f : fast_exp2(z[i] - m_new);
                    psum += p;
                    pk[i] = __builtin_bit_cast(short, (__bf16)p);
                }
                l_own[hb] = l_own[hb] * resc + psum;
                m_ref[hb] = m_new;
                unsigned char *prow = pb + (16 * hb + l16) * PSTR;
                // row e of a group of eight sits at contraction position e / 2 + 4 (e % 2) (see the transpose reads):
                // the lane's rows 4 (g & 1) + {0, 2} are neighbours there, and so are its rows 4 (g & 1) + {1, 3}
                typedef __attribute__((ext_vector_type(2))) short s16x2;
                unsigned char *pg = prow + (16 * wave + 8 * (g >> 1) + 2 * (g & 1)) * 2;
                *(s16x2 *)pg = s16x2{pk[0], pk[2]};
                *(s16x2 *)(pg + 8) = s16x2{pk[1], pk[3]};
                if (g == 0) *(float *)(prow + kSlabTile * 2 + 4 * wave) = m_new;
            }
        }
        // P of tile it is written; every wave has all its reads of tile it-1 back
        __syncthreads();

        if constexpr (kPrev) {
            if (__ballot(alpha != 1.f) != 0ull) {
                // the rescale factors of the 16 heads a lane accumulates, through a per-wave LDS row
                float *ab = abuf + wave * 32;
                if (hh == 0) ab[l32] = alpha;
                f32x4 ar[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) ar[q] = *(const f32x4 *)(ab + 8 * q + 4 * hh);
                // The accumulators live in accumulation registers; move each value out and back
                // right here (opaque to the compiler), otherwise it copies all 64 of them to vector
                // registers ahead of the branch in every tile.  The MFMAs that wrote them retired
                // a tile ago and the next MFMA that reads them is far behind the trailing no-ops.
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float t;
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(t) : "a"(oacc[nb][i]));
                        t *= ar[i >> 2][i & 3];
                        asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(oacc[nb][i]) : "v"(t));
                    }
                asm volatile("s_nop 7\n\ts_nop 7");
            }
            if (__ballot(any_f) != 0ull) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pa[j][e] = (__bf16)((float)pa[j][e] * fj[j]);
            }
        }
        const unsigned vm_n2 = ids_mask(ids_n2);

        // O += P V for tile it-1, with the staging of tile it+1 (nobody reads that buffer any more)
        // and the gather of tile it+2 issued in the shadow of the MFMAs
        unsigned char *tn = tbuf + (buf ^ 1) * TBUFB + st_off;
        const unsigned short *pl = row_ptr(ids_n2.lo, it + 2), *ph = row_ptr(ids_n2.hi, it + 2);
        auto stage = [&](int ks) {
            if constexpr (kStage) {
                if (ks < KS) {
                    *(u32x4 *)(tn + (ks & 1) * 8 * ROWB + 128 * (ks >> 1)) = cur[ks];
                    if constexpr (kLoad) cur[ks] = *(const u32x4 *)(((ks & 1) ? ph : pl) + 64 * (ks >> 1));
                }
            }
        };
        if constexpr (kPrev) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) {
                    const s16x4 v0 = vq[j][nb][0], v1 = vq[j][nb][1];
                    const s16x8 vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                    oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa[j], __builtin_bit_cast(bf16x8, vv), oacc[nb], 0, 0, 0);
                    stage(4 * j + nb);
                }
#pragma unroll
            for (int ks = 4 * NBW; ks < KS; ++ks) stage(ks);
            if constexpr (kStage) {
                // keep the order: one MFMA, then one LDS store and (when there is one) one gather load
#pragma unroll
                for (int k = 0; k < 4 * NBW; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                    if constexpr (kLoad) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) stage(ks);
        }
        if constexpr (kCur) {                             // the drain step leaves the stream where it is
            vm_cur = vm_n1;
            vm_n1 = vm_n2;
            ids_n2 = ids_n3;
        }
    };

    // ---- epilogue of a query: combine the producers' row sums, normalise, store ----
    auto finish = [&]() {
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            const float l = xsum16_32(l_own[hb]);
            // bring the wave's sum to the common reference before publishing it
            const float f = (m_all[hb] == -INFINITY) ? 0.f : fast_exp2(m_ref[hb] - m_all[hb]);
            if (g == 0) lbuf[wave * 32 + 16 * hb + l16] = l * f;
        }
        __syncthreads();
        const float l_head = lbuf[l32] + lbuf[32 + l32] + lbuf[64 + l32] + lbuf[96 + l32];   // head l32
        const float m_head = m_c;
        {
            if constexpr (SPLIT) {
                // partial of this split: its reference maximum and row sum (the output below is
                // normalised by that sum; the merge weighs the splits by their share of the total)
                if (wave == 0 && hh == 0 && l32 < a.H_q) {
                    float *ml = a.part_ml + ((qrow * a.n_splits + sp) * a.H_q + l32) * 2;
                    ml[0] = m_head;
                    ml[1] = l_head;
                }
            } else {
                if (wave == 0 && hh == 0 && l32 < a.H_q && a.lse)
                    a.lse[qrow * a.H_q + l32] =
                        (l_head > 0.f) ? (m_head + __builtin_log2f(l_head)) * 0.6931471805599453f : -INFINITY;
            }
            // accumulator element i belongs to head 8 (i / 4) + 4 hh + i % 4: the sums of the lane's
            // 16 heads come straight from the four waves' partials (independent 16-byte reads; a
            // lane-to-lane shuffle per head would be sixteen dependent trips through the crossbar)
            f32x4 inv4[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 l4 = *(const f32x4 *)(lbuf + 8 * q + 4 * hh);
#pragma unroll
                for (int w = 1; w < 4; ++w) l4 += *(const f32x4 *)(lbuf + 32 * w + 8 * q + 4 * hh);
#pragma unroll
                for (int r = 0; r < 4; ++r) inv4[q][r] = (l4[r] > 0.f) ? __builtin_amdgcn_rcpf(l4[r]) : 0.f;
            }
            const bool all_heads = a.H_q >= 32;               // workgroup-uniform
            // the lane's offset into O is recomputed from the thread id here: kept live across the
            // tile loop it is spilled, and its reload waits behind every gather in flight
            int tx = tid;
            asm volatile("" : "+v"(tx));
            const int o_lane = 32 * (tx >> 6) + (tx & 31), o_hh = (tx >> 5) & 1;
            __bf16 *o_row = (SPLIT ? a.part_o + (qrow * a.n_splits + sp) * a.H_q * D_V : (__bf16 *)a.O + qrow * a.H_q * D_V) + o_lane;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int hq = 8 * (i >> 2) + 4 * o_hh + (i & 3); // O row (head) of accumulator element i
                const float inv = inv4[i >> 2][i & 3];
                __bf16 *po = o_row + hq * D_V;
                if (all_heads) {
#pragma unroll
                    for (int nb = 0; nb < NBW; ++nb) po[128 * nb] = (__bf16)(oacc[nb][i] * inv);
                } else if (hq < a.H_q) {
#pragma unroll
                    for (int nb = 0; nb < NBW; ++nb) po[128 * nb] = (__bf16)(oacc[nb][i] * inv);
                }
            }
        }
    };

    constexpr std::true_type T{};
    constexpr std::false_type F{};
    if (!chain) {
        // one query (or one split of it): step 0 has no previous tile, step ntiles has no current one
        if (ntiles == 1) {
            step(0, F, T, F, F);
        } else if (ntiles == 2) {
            step(0, F, T, T, F);
            step(1, T, T, F, F);
        } else {
            step(0, F, T, T, T);
            int it = 1;
#pragma unroll 1
            for (; it + 2 < ntiles; ++it) step(it, T, T, T, T);
            step(it, T, T, T, F);
            ++it;
            step(it, T, T, F, F);
        }
        step(ntiles, T, F, F, F);
        finish();
        return;
    }
    if constexpr (!SPLIT) {
        // Chained queries.  The last two steps of a query stage and gather the first tiles of the
        // next one (dead tiles after the workgroup's last query: row 0, masked), so a query ends
        // in exactly the state the prologue sets up: tile 0 in LDS, tile 1 in the gather
        // registers, ids of tile 2 at hand.
        for (;;) {
            step(0, F, T, T, T);
#pragma unroll 1
            for (int it = 1; it < cs.nt; ++it) step(it, T, T, T, T);
            step(cs.nt, T, F, F, F);
            const bool more = qnext < nq;
            if (more) load_q_direct(qnext);               // lands while the outputs are stored
            finish();
            if (!more) break;
            qrow = qnext;
            qnext += gridDim.x;
            g0 = (g0 + cs.nt) & 1;
            cs = ns;
            ns = src_of(qnext);
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[nb][i] = 0.f;
#pragma unroll
            for (int hb = 0; hb < 2; ++hb) {
                m_all[hb] = -INFINITY;
                m_ref[hb] = -INFINITY;
                l_own[hb] = 0.f;
            }
            m_c = -INFINITY;
            settle_q(tbuf + ((g0 ^ 1) & 1) * TBUFB);      // the drained tile's buffer: nobody touches it before step 0's barrier
        }
    }
}

// Combine the per-split partials of one (query, head): O = sum_s w_s O_s / sum_s w_s with O_s the split's own
// normalised output and w_s = l_s 2^(m_s-m) its share of the row sum.
// One workgroup per (query, head); a thread owns 4 consecutive value columns.
template <int D_V>
__global__ __launch_bounds__(D_V / 4) void attn_merge_kernel(AttnArgs a)
{
    const int64_t qrow = blockIdx.x;
    const int h = blockIdx.y;
    const int v = threadIdx.x * 4;
    const float *ml = a.part_ml + ((qrow * a.n_splits) * a.H_q + h) * 2;
    const int64_t ml_stride = (int64_t)a.H_q * 2;
    // The partial outputs do not depend on the weights: the first batch of them is requested together with the
    // (maximum, sum) pairs, so that the launch waits for memory once, not twice.
    constexpr int kBatch = 8;
    const __bf16 *po = a.part_o + ((qrow * a.n_splits) * a.H_q + h) * D_V + v;
    const int64_t po_stride = (int64_t)a.H_q * D_V;
    s16x4 x[kBatch];
    auto load_x = [&](int s0) {
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            x[j] = s16x4{0, 0, 0, 0};
            if (s0 + j < a.n_splits) x[j] = *(const s16x4 *)(po + (s0 + j) * po_stride);
        }
    };
    load_x(0);
    float m = -INFINITY;
    for (int s = 0; s < a.n_splits; ++s) m = fmaxf(m, ml[s * ml_stride]);
    float l = 0.f;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < a.n_splits; s0 += kBatch) {
        if (s0 > 0) load_x(s0);
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            if (s0 + j < a.n_splits) {
                const float ms = ml[(s0 + j) * ml_stride], ls = ml[(s0 + j) * ml_stride + 1];
                const float sc = (ms == -INFINITY) ? 0.f : ls * fast_exp2(ms - m);   // the split's share of the row sum
                l += sc;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] += __uint_as_float((uint32_t)(uint16_t)x[j][e] << 16) * sc;   // bf16 -> fp32 is a shift
            }
        }
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
    static hipError_t attr = hipFuncSetAttribute((const void *)attn_kernel<D_QK, D_V, ROW_F, false>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    static hipError_t attr_pg = hipFuncSetAttribute((const void *)attn_kernel<D_QK, D_V, ROW_F, true>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return attr;
    if (attr_pg != hipSuccess) return attr_pg;
    dim3 grid((unsigned)((int64_t)a.B * a.Tq), (unsigned)a.n_splits);
    if (a.pv.seq_lens || a.pv.page_table)
        hipLaunchKernelGGL((attn_kernel<D_QK, D_V, ROW_F, true>), grid, dim3(256), lds, st, a);
    else
        hipLaunchKernelGGL((attn_kernel<D_QK, D_V, ROW_F, false>), grid, dim3(256), lds, st, a);
    return hipGetLastError();
}

template <int D_QK, int D_V, bool PG, bool SPLIT>
hipError_t launch_slab_t(const AttnArgs &a, size_t lds, hipStream_t st)
{
    static hipError_t attr = hipFuncSetAttribute((const void *)attn_slab_kernel<D_QK, D_V, PG, SPLIT>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return attr;
    int64_t wgs = (int64_t)a.B * a.Tq;
    if (!SPLIT && a.k_sel > 2 * kSlabTile) {
        // whole selections of three or more tiles: one workgroup per CU walks a chain of queries
        static int n_cu = 0;
        if (n_cu == 0) {
            int dev = 0, v = 0;
            if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
                return hipErrorInvalidDevice;
            n_cu = v;
        }
        if (wgs > n_cu) wgs = n_cu;
    }
    dim3 grid((unsigned)wgs, (unsigned)(SPLIT ? a.n_splits : 1));
    hipLaunchKernelGGL((attn_slab_kernel<D_QK, D_V, PG, SPLIT>), grid, dim3(256), lds, st, a);
    return hipGetLastError();
}

template <int D_QK, int D_V>
hipError_t launch_slab(const AttnArgs &a, hipStream_t st)
{
    const size_t lds = (size_t)2 * kSlabTile * (D_QK * 2 + kSlabPad) + 2 * 32 * (kSlabTile * 2 + 16) + (4 * 32 + 4 * 32) * sizeof(float);
    const bool pg = a.pv.seq_lens || a.pv.page_table;
    if (a.n_splits > 1) return pg ? launch_slab_t<D_QK, D_V, true, true>(a, lds, st) : launch_slab_t<D_QK, D_V, false, true>(a, lds, st);
    return pg ? launch_slab_t<D_QK, D_V, true, false>(a, lds, st) : launch_slab_t<D_QK, D_V, false, false>(a, lds, st);
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
        // the row-slab form: one workgroup per query, or per split of a query's selection when
        // there are too few queries to fill the chip (decode); rows with the values elsewhere than
        // in their first features take the small-tile form
        if (a.v_off == 0) return launch_slab<576, 512>(a, st);
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
