// Forward of the indexer's distillation loss (paper Sec. 3.3: Eq. 1 multi-layer loss, Eq. 2 loss
// against the averaged target, Prop. 1), in the form the sparse training phase uses: both
// distributions live on the k selected positions of a query.
//
//   attn_probs_kernel   p_bar_t(s) = 1/H sum_h softmax_s(sm_scale Q[t,h] . K[s]) over the selected
//                       rows: the layer's attention distribution aggregated over its heads, the
//                       indexer's training target (Sec. 2.1).  S^T = K Q^T on
//                       v_mfma_f32_16x16x32_bf16 with Q in registers and the gathered rows turned
//                       into the A-operand layout through a per-wave LDS tile; the per-head
//                       normalisers are the log-sum-exps the attention kernel already produced;
//                       the head sum is a 16-lane row reduction.
//   distill_row_kernel  (and its register-resident form for k <= 2048, which reads every input once)
//                       per query: q = Softmax(I) over the selected scores (in the log domain),
//                       sum_j 1/(m+1) KL(p_j || q), KL(p_bar || q), and q * |p_bar| - p_bar, the
//                       gradient with respect to the indexer's logits that both losses share.
//   distill_sum_kernel  fixed-order sum of the per-row values (one workgroup: deterministic).
#include "ic_common.hpp"

namespace ic {

namespace {

constexpr int kProbRows = 16;                 // selected rows per wave and step

// LDS rows are padded by 32 bytes and not swizzled: with rows 1152 + 32 bytes apart the 16-byte A-operand read of 16
// rows (lane = row, same piece in every lane) runs at the rate of a contiguous read (measured; with rows 1152 apart
// and an XOR swizzle it took 1.65 times as long).
constexpr int kProbPad = 32;

// Validity of a wave's 16 rows from the two ballots over the gather lanes (lane 8r' + piece holds
// row r' of the first / second eight rows): bit r of the result is row r.
__device__ __forceinline__ unsigned rows_mask(unsigned long long ba, unsigned long long bb)
{
    const unsigned long long ones = 0x0101010101010101ull, pack = 0x0102040810204080ull;
    const unsigned lo = (unsigned)(((ba & ones) * pack) >> 56);
    const unsigned hi = (unsigned)(((bb & ones) * pack) >> 56);
    return lo | (hi << 8);
}

// One workgroup per query, every wave on its own: wave w takes the selected rows 16 w .. 16 w + 15,
// then 64 further on.  Eight lanes fetch one 128-byte line of a row (the gather shape the memory
// system serves fastest); the 16 rows turn into the A-operand layout (lane = row, 8 features) through
// the wave's private 16-row LDS tile: LDS executes a wave's accesses in order, so the stores of the
// next rows simply follow the reads of the current ones and the workgroup never meets at a barrier.
// The next 16 rows are in flight while the current ones are multiplied.
template <int D_QK>
__global__ __launch_bounds__(256, 2) void attn_probs_kernel(ProbsArgs a)
{
    constexpr int KS = D_QK / 32;             // contraction steps = 16-byte chunks per gather lane
    constexpr int ROWB = D_QK * 2 + kProbPad; // bytes per LDS row
    static_assert((D_QK * 2) % 128 == 0 && KS % 2 == 0, "a row is a whole number of 128-byte windows");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [4 waves][16 rows][ROWB]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int gr = lane >> 3, gp = lane & 7;  // gather role: row (and row + 8), 16-byte piece of the window
    const int64_t qrow = blockIdx.x;
    const int b = (int)(qrow / a.Tq);
    const int32_t *idx_row = a.idx + qrow * a.k_sel;
    const unsigned short *kv_seq = (const unsigned short *)a.KV + (int64_t)b * a.Lk * a.row_elems;
    float *out = a.probs + qrow * a.k_sel;
    unsigned char *tb = smem + wave * kProbRows * ROWB;

    // Q as the B operand (head 16 hb + l16, features 8 g + 32 ks ..), and the heads' log-sum-exps
    bf16x8 qreg[2][KS];
    float lse2[2];
    bool head_ok[2];
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
        const int head = 16 * hb + l16;
        head_ok[hb] = head < a.H_q;
        const unsigned short *qp = (const unsigned short *)a.Q + (qrow * a.H_q + (head_ok[hb] ? head : 0)) * D_QK + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = u32x4{0u, 0u, 0u, 0u};
            if (head_ok[hb]) raw = *(const u32x4 *)(qp + 32 * ks);
            qreg[hb][ks] = __builtin_bit_cast(bf16x8, raw);
        }
        lse2[hb] = head_ok[hb] ? a.lse[qrow * a.H_q + head] * 1.4426950408889634f : INFINITY;
    }
    const float inv_h = 1.f / (float)a.H_q;

    // LDS offsets of the lane in its two roles
    const int st_off = gr * ROWB + (gp << 4);                             // + 8 rows for odd chunks
    const int ka_row = l16 * ROWB;
    const int ka_e = ka_row + (g << 4);                                   // even contraction steps
    const int ka_o = ka_row + ((4 + g) << 4);                             // odd ones

    struct Ids { int32_t lo, hi; };           // validated ids of rows gr and gr + 8 of a group, -1: empty slot
    auto fetch_ids = [&](int grp) -> Ids {
        const int s_lo = kProbRows * grp + gr, s_hi = s_lo + 8;
        const int32_t v_lo = idx_row[min(s_lo, a.k_sel - 1)], v_hi = idx_row[min(s_hi, a.k_sel - 1)];
        Ids r;
        r.lo = ((int)(s_lo < a.k_sel) & (int)(v_lo >= 0) & (int)(v_lo < a.Lk)) ? v_lo : -1;
        r.hi = ((int)(s_hi < a.k_sel) & (int)(v_hi >= 0) & (int)(v_hi < a.Lk)) ? v_hi : -1;
        return r;
    };
    // loads are unconditional (an empty slot reads row 0 and is masked later): the wait counters stay positional
    u32x4 cur[KS];
    auto gather = [&](const Ids &d) {
        const unsigned short *pl = kv_seq + (int64_t)(d.lo < 0 ? 0 : d.lo) * a.row_elems + 8 * gp;
        const unsigned short *ph = kv_seq + (int64_t)(d.hi < 0 ? 0 : d.hi) * a.row_elems + 8 * gp;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cur[ks] = *(const u32x4 *)(((ks & 1) ? ph : pl) + 64 * (ks >> 1));
    };

    const int ngroups = (a.k_sel + kProbRows - 1) / kProbRows;
    Ids d_cur = fetch_ids(wave), d_nxt = fetch_ids(wave + 4);
    gather(d_cur);
#pragma unroll 1
    for (int grp = wave; grp < ngroups; grp += 4) {                       // wave-uniform
        const unsigned rows_ok = rows_mask(__ballot(d_cur.lo >= 0), __ballot(d_cur.hi >= 0));
        const Ids d_n2 = fetch_ids(grp + 8);
        // the rows of this group go to the tile, their registers take the next group
        {
            const unsigned short *pl = kv_seq + (int64_t)(d_nxt.lo < 0 ? 0 : d_nxt.lo) * a.row_elems + 8 * gp;
            const unsigned short *ph = kv_seq + (int64_t)(d_nxt.hi < 0 ? 0 : d_nxt.hi) * a.row_elems + 8 * gp;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                *(u32x4 *)(tb + st_off + (ks & 1) * 8 * ROWB + 128 * (ks >> 1)) = cur[ks];
                cur[ks] = *(const u32x4 *)(((ks & 1) ? ph : pl) + 64 * (ks >> 1));
            }
        }
        // S^T for 16 rows x 32 heads: two accumulation chains per head block
        f32x4 s4[2][2];
#pragma unroll
        for (int hb = 0; hb < 2; ++hb)
#pragma unroll
            for (int par = 0; par < 2; ++par) s4[hb][par] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 ka = *(const bf16x8 *)(tb + ((ks & 1) ? ka_o : ka_e) + 128 * (ks >> 1));
            s4[0][ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qreg[0][ks], s4[0][ks & 1], 0, 0, 0);
            s4[1][ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qreg[1][ks], s4[1][ks & 1], 0, 0, 0);
        }
        // lane (head l16, g) holds rows 4 g + i: probabilities of its two heads, summed over the heads
        float ps[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = (rows_ok >> (4 * g + i)) & 1u;
            float p = 0.f;
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
                if (ok && head_ok[hb])
                    p += __builtin_amdgcn_exp2f((s4[hb][0][i] + s4[hb][1][i]) * a.scale_log2e - lse2[hb]);
            ps[i] = row16_sum(p);                         // lane l16 == 15: the sum over the 16 head lanes
        }
        if (l16 == 15) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int s = kProbRows * grp + 4 * g + i;
                if (s < a.k_sel) out[s] = ps[i] * inv_h;
            }
        }
        d_cur = d_nxt;
        d_nxt = d_n2;
    }
}

// Block-wide reductions (256 threads): a butterfly inside each wave, then the four wave results
// through LDS.  The sum runs in a fixed order, so a row's value does not depend on timing.
__device__ __forceinline__ double block_sum(double x, double *red, int tid)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    if ((tid & 63) == 0) red[tid >> 6] = x;
    __syncthreads();
    const double r = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ float block_max(float x, float *red, int tid)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    if ((tid & 63) == 0) red[tid >> 6] = x;
    __syncthreads();
    const float r = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    return r;
}

__global__ __launch_bounds__(256) void distill_row_kernel(DistillArgs a)
{
    __shared__ double redd[256];
    __shared__ float redf[256];
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    const float *sc = a.scores + row * a.k_sel;
    const float w = 1.f / (float)a.n_targets;

    // log q(s) = (I_s - max) - log sum exp(I - max), over the finite entries
    float mx = -INFINITY;
    for (int s = tid; s < a.k_sel; s += 256) {
        const float x = sc[s];
        if (x > -INFINITY && x < INFINITY) mx = fmaxf(mx, x);
    }
    mx = block_max(mx, redf, tid);
    double z = 0.0;
    for (int s = tid; s < a.k_sel; s += 256) {
        const float x = sc[s];
        if (x > -INFINITY && x < INFINITY) z += (double)expf(x - mx);
    }
    z = block_sum(z, redd, tid);
    const float log_z = z > 0.0 ? (float)log(z) : 0.f;

    // mass of the averaged target (1 for a row with selected entries, 0 for an empty one)
    double mass = 0.0;
    for (int s = tid; s < a.k_sel; s += 256) {
        float pb = 0.f;
        for (int j = 0; j < a.n_targets; ++j) pb += a.probs[j][row * a.k_sel + s];
        mass += (double)(pb * w);
    }
    mass = block_sum(mass, redd, tid);

    double multi = 0.0, avg = 0.0;
    for (int s = tid; s < a.k_sel; s += 256) {
        const float x = sc[s];
        const bool fin = x > -INFINITY && x < INFINITY;
        const float lq = fin ? (x - mx) - log_z : -INFINITY;
        float pb = 0.f;
        for (int j = 0; j < a.n_targets; ++j) {
            const float p = a.probs[j][row * a.k_sel + s];
            pb += p;
            if (p > 0.f) multi += (double)(w * p * (logf(p) - lq));
        }
        pb *= w;
        if (pb > 0.f) avg += (double)(pb * (logf(pb) - lq));
        if (a.grad) a.grad[row * a.k_sel + s] = (fin ? expf(lq) : 0.f) * (float)mass - pb;
    }
    multi = block_sum(multi, redd, tid);
    avg = block_sum(avg, redd, tid);
    if (tid == 0) {
        a.row_multi[row] = multi;
        a.row_avg[row] = avg;
    }
}

// The same per-row values for rows of up to 256 * EPT selected positions, every input read exactly
// once: the thread keeps its EPT logits (as log q) and the running sum of the targets in registers;
// the targets are visited one after the other, each adding its own term of Eq. 1.
template <int EPT>
__global__ __launch_bounds__(256) void distill_row_reg_kernel(DistillArgs a)
{
    __shared__ double redd[4];
    __shared__ float redf[4];
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    const float *sc = a.scores + row * a.k_sel;
    const float w = 1.f / (float)a.n_targets;

    float lq[EPT];                             // logits, then log q
    bool fin[EPT];
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int s = tid + 256 * e;
        lq[e] = s < a.k_sel ? sc[s] : -INFINITY;
        fin[e] = lq[e] > -INFINITY && lq[e] < INFINITY;
        if (fin[e]) mx = fmaxf(mx, lq[e]);
    }
    mx = block_max(mx, redf, tid);
    double z = 0.0;
#pragma unroll
    for (int e = 0; e < EPT; ++e)
        if (fin[e]) z += (double)expf(lq[e] - mx);
    z = block_sum(z, redd, tid);
    const float log_z = z > 0.0 ? (float)log(z) : 0.f;
#pragma unroll
    for (int e = 0; e < EPT; ++e) lq[e] = fin[e] ? (lq[e] - mx) - log_z : -INFINITY;

    float pb[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) pb[e] = 0.f;
    double multi = 0.0;
    for (int j = 0; j < a.n_targets; ++j) {
        const float *pj = a.probs[j] + row * a.k_sel;
        float p[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int s = tid + 256 * e;
            p[e] = s < a.k_sel ? pj[s] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            pb[e] += p[e];
            if (p[e] > 0.f) multi += (double)(w * p[e] * (logf(p[e]) - lq[e]));
        }
    }
    double avg = 0.0, mass = 0.0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        mass += (double)(pb[e] * w);           // 1 for a row with selected entries, 0 for an empty one
        pb[e] *= w;
        if (pb[e] > 0.f) avg += (double)(pb[e] * (logf(pb[e]) - lq[e]));
    }
    mass = block_sum(mass, redd, tid);
    if (a.grad) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int s = tid + 256 * e;
            if (s < a.k_sel) a.grad[row * a.k_sel + s] = (fin[e] ? expf(lq[e]) : 0.f) * (float)mass - pb[e];
        }
    }
    multi = block_sum(multi, redd, tid);
    avg = block_sum(avg, redd, tid);
    if (tid == 0) {
        a.row_multi[row] = multi;
        a.row_avg[row] = avg;
    }
}

__global__ __launch_bounds__(256) void distill_sum_kernel(const double *row_multi, const double *row_avg, int64_t n,
                                                          double *loss_multi, double *loss_avg)
{
    __shared__ double red[256];
    const int tid = threadIdx.x;
    double m = 0.0, v = 0.0;
    for (int64_t r = tid; r < n; r += 256) {
        m += row_multi[r];
        v += row_avg[r];
    }
    m = block_sum(m, red, tid);
    v = block_sum(v, red, tid);
    if (tid == 0) {
        if (loss_multi) *loss_multi = m;
        if (loss_avg) *loss_avg = v;
    }
}

} // namespace

hipError_t launch_attn_probs(const ProbsArgs &a, int d_qk, hipStream_t st)
{
    const int64_t nq = (int64_t)a.B * a.Tq;
    if (nq <= 0) return hipSuccess;
    if (d_qk == 576) {
        constexpr int lds = 4 * kProbRows * (576 * 2 + kProbPad);      // above the default limit of dynamic LDS: opt in once
        static hipError_t attr = hipFuncSetAttribute((const void *)attn_probs_kernel<576>,
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(attn_probs_kernel<576>, dim3((unsigned)nq), dim3(256), lds, st, a);
    } else if (d_qk == 64) {
        hipLaunchKernelGGL(attn_probs_kernel<64>, dim3((unsigned)nq), dim3(256), 4 * kProbRows * (64 * 2 + kProbPad), st, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_distill(const DistillArgs &a, int64_t nq, double *loss_multi, double *loss_avg, hipStream_t st)
{
    if (nq > 0) {
        if (a.k_sel <= 256 * 8)
            hipLaunchKernelGGL(distill_row_reg_kernel<8>, dim3((unsigned)nq), dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL(distill_row_kernel, dim3((unsigned)nq), dim3(256), 0, st, a);
    }
    hipLaunchKernelGGL(distill_sum_kernel, dim3(1), dim3(256), 0, st, (const double *)a.row_multi, (const double *)a.row_avg, nq,
                       loss_multi, loss_avg);
    return hipGetLastError();
}

} // namespace ic
