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

} // namespace

bool attn_shape_supported(int d_qk, int d_v)
{
    return (d_qk == 576 && d_v == 512) || (d_qk == 64 && d_v == 64);
}

hipError_t launch_attn(const AttnArgs &a, int d_qk, int d_v, hipStream_t st)
{
    if ((int64_t)a.B * a.Tq <= 0) return hipSuccess;
    if (d_qk == 576 && d_v == 512) return launch_t<576, 512, 576>(a, st);
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
