// Shared device/host declarations of the gfx950 IndexCache library (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "indexcache.h"

namespace ic {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // one 16-byte chunk
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kWave = 64;

// ---- kernel argument blocks ---------------------------------------------------------

// Ragged and paged caches (decode with a full KV cache, paper Sec. 4.3 setting): per-sequence
// lengths and a page table from logical to physical pages.  All-zero = the dense layout.
struct PagedView {
    const int32_t *seq_lens;    // [B] visible length of each sequence (nullptr: every sequence has Lk)
    const int32_t *page_table;  // [B, max_pages] physical page of a logical page (nullptr: not paged)
    int32_t page_shift;         // log2(positions per page), pages hold a power of two >= 64 positions
    int32_t max_pages;
};

// physical row of logical position s of sequence b (paged layout only)
__device__ __forceinline__ int64_t paged_row(const PagedView &pv, int b, int s)
{
    const int32_t page = pv.page_table[(int64_t)b * pv.max_pages + (s >> pv.page_shift)];
    return ((int64_t)page << pv.page_shift) + (s & ((1 << pv.page_shift) - 1));
}


// Indexer scoring of query rows [i0, i0+Ri) of sequences [b0, b0+Bc) against their keys.
// Scores land in a strip: row (b-b0)*Ri + (i-i0), element s, row stride ld floats.
struct ScoreArgs {
    const void *q;        // [B,Tq,H_I,d_I]
    const void *k;        // [B,Lk,d_I]
    const float *w;       // [B,Tq,H_I]
    const float *q_scale; // fp8 only
    const float *k_scale; // fp8 only
    float *strip;
    int64_t ld;
    int64_t q_pos0;
    int32_t Tq, Lk, H_I;
    int32_t b0, i0, Ri;   // chunk origin and rows per sequence in the strip
    int32_t n_qblocks;    // ceil(Ri / tokens per workgroup)
    int32_t KC;           // keys per workgroup along grid.y (multiple of 64)
    PagedView pv;         // ragged / paged key cache (the Tq query rows are the LAST Tq positions of a sequence)
};

// Per-row top-k over a strip of scores.
struct SelectArgs {
    const float *strip;
    int64_t ld;
    int64_t q_pos0;
    int32_t Tq, Lk, k_sel;
    int32_t b0, i0, Ri;
    int32_t cache_elems;  // row elements the workgroup may cache in LDS (0 = none)
    int32_t *idx;         // [B,Tq,k_sel]
    float *sel;           // [B,Tq,k_sel] or nullptr
    const int32_t *seq_lens;  // ragged: [B] visible lengths (nullptr: q_pos0 rule)
};

struct AttnArgs {
    const void *Q;        // [B,Tq,H_q,d_qk] bf16
    const void *KV;       // [B,Lk,row_elems] bf16
    const int32_t *idx;   // [B,Tq,k_sel]
    void *O;              // [B,Tq,H_q,d_v] bf16
    float *lse;           // [B,Tq,H_q] or nullptr
    __bf16 *part_o;       // split partials: [B*Tq, n_splits, H_q, d_v] bf16, each normalised by its own row sum
    float *part_ml;       // [B*Tq, n_splits, H_q, 2] fp32 (running max in log2 units, sum)
    int32_t B, Tq, Lk, H_q, v_off, row_elems, k_sel;
    int32_t n_splits, split_len; // key slots per split (multiple of 64)
    float scale_log2e;    // sm_scale * log2(e)
    PagedView pv;         // ragged / paged KV cache (KV is then the page pool [n_pages << page_shift, row_elems])
    // >= 0: idx comes from the causal top-k of this library with query row t at position causal_pos0 + t, so row t
    // holds min(k_sel, causal_pos0 + t + 1) entries followed by -1 only, and the tiles behind them need no work;
    // < 0: nothing is known about idx
    int64_t causal_pos0;
};

// Head-aggregated attention probabilities over the selected rows (the indexer's training target).
struct ProbsArgs {
    const void *Q;        // [B,Tq,H_q,d_qk] bf16
    const void *KV;       // [B,Lk,row_elems] bf16; K = the first d_qk features of a row
    const int32_t *idx;   // [B,Tq,k_sel]
    const float *lse;     // [B,Tq,H_q] natural-log sum-exp of each head over the same rows
    float *probs;         // [B,Tq,k_sel] out, slot order, 0 on empty slots
    int32_t B, Tq, Lk, H_q, row_elems, k_sel;
    float scale_log2e;
};

// Distillation losses of one Full layer's indexer against the layers it serves.
struct DistillArgs {
    const float *probs[IC_MAX_DISTILL_TARGETS];   // m+1 targets, each [nq, k_sel]
    int32_t n_targets, k_sel;
    const float *scores;  // [nq, k_sel] indexer logits at the selected positions (-inf on empty slots)
    double *row_multi;    // [nq] per-row Eq. 1 terms
    double *row_avg;      // [nq] per-row Eq. 2 terms
    float *grad;          // [nq, k_sel] or nullptr
};

// Sum over the 16 lanes of a row (lanes with equal lane / 16) on the data-parallel-primitive path:
// shifts by 1, 2, 4, 8 lanes inside the row; lanes without a source add zero.  Lane 15 of the row
// holds the total.
__device__ __forceinline__ float row16_sum(float x)
{
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x111, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x112, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x114, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x118, 0xf, 0xf, false));
    return x;
}

// ---- launchers (defined next to their kernels) ----------------------------------------

hipError_t launch_score(const ScoreArgs &a, int dtype, int d_I, int Bc, hipStream_t st);
hipError_t launch_fill(float *p, int64_t n, float v, hipStream_t st);
hipError_t launch_select(const SelectArgs &a, int n_rows, int max_row_len, hipStream_t st);
int select_cache_limit();
hipError_t launch_attn(const AttnArgs &a, int d_qk, int d_v, hipStream_t st);
hipError_t launch_attn_merge(const AttnArgs &a, int d_v, hipStream_t st);
size_t overlap_ws_bytes(int n_layers);
size_t overlap_lds_bytes(int n_layers, int Lk);
hipError_t launch_overlap(const int32_t *const *idx_layers, int n_layers, int64_t nq, int k_sel, int Lk, double *overlap,
                          unsigned long long *inter_out, unsigned long long *sizes_out, void *ws, hipStream_t st);
hipError_t launch_cosine(const void *A, const void *B, int64_t n_rows, int64_t row_len, double *mean, float *per_row,
                         double *acc, hipStream_t st);
hipError_t launch_sim_init(double *S, int n, hipStream_t st);
hipError_t launch_loss_finish(const double *sims, int n, double *loss, hipStream_t st);
hipError_t launch_attn_probs(const ProbsArgs &a, int d_qk, hipStream_t st);
hipError_t launch_distill(const DistillArgs &a, int64_t nq, double *loss_multi, double *loss_avg, hipStream_t st);
hipError_t launch_calib(int kind, const void *src, void *dst, const int32_t *idx, int64_t n, int64_t table_rows, int row_bytes,
                        int wgs, hipStream_t st);
bool score_shape_supported(int dtype, int H_I, int d_I);
bool attn_shape_supported(int d_qk, int d_v);

} // namespace ic
