// C ABI of the library: argument validation, workspace planning, the Full/Shared layer loop
// (paper Fig. 2b) and optional per-kernel event timing.  All device work is enqueued on the
// caller's stream; nothing here allocates device memory or synchronises in the hot path.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "ic_common.hpp"

// Scratch for ic_sparse_attn_static: part of the code object, one copy per GPU at its own address.
// In host code this name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[IC_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

ic_status fail(ic_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return s;
}

std::atomic<uint64_t> g_indexer_launches{0};

// ---- per-kernel event timing -------------------------------------------------------------
constexpr int kProfClasses = 4;
constexpr size_t kProfPool = 8192;
struct ProfRec {
    hipEvent_t e0, e1;
    int which;
};
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRec> g_prof_recs;
int64_t g_prof_n[kProfClasses] = {0, 0, 0, 0};
double g_prof_ms[kProfClasses] = {0, 0, 0, 0};

struct ProfScope {
    hipStream_t st;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int which;
    bool live = false;
    ProfScope(int which_, hipStream_t st_) : st(st_), which(which_)
    {
        if (!g_prof_on) return;
        std::lock_guard<std::mutex> lk(g_prof_mu);
        if (g_prof_recs.size() >= kProfPool) return;
        if (hipEventCreate(&e0) != hipSuccess) return;
        if (hipEventCreate(&e1) != hipSuccess) {
            (void)hipEventDestroy(e0);
            return;
        }
        live = true;
        (void)hipEventRecord(e0, st);
    }
    ~ProfScope()
    {
        if (!live) return;
        (void)hipEventRecord(e1, st);
        std::lock_guard<std::mutex> lk(g_prof_mu);
        g_prof_recs.push_back(ProfRec{e0, e1, which});
    }
};

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Default strip budget when the caller asks how much workspace to bring.
constexpr size_t kStripBudget = (size_t)1 << 30;   // 1 GiB of score rows in flight
constexpr size_t kSmallStrip = (size_t)64 << 20;    // problems whose whole score matrix is below this keep it in one strip
constexpr int kMinStripRows = 16;

ic_status check_indexer(const ic_indexer_desc *d)
{
    if (!d) return fail(IC_ERR_NULL, "indexer descriptor is NULL");
    if (d->B <= 0 || d->Tq <= 0 || d->Lk <= 0 || d->H_I <= 0 || d->d_I <= 0 || d->k_sel <= 0)
        return fail(IC_ERR_SHAPE, "indexer sizes must be positive (B=%d Tq=%d Lk=%d H_I=%d d_I=%d k_sel=%d)",
                    d->B, d->Tq, d->Lk, d->H_I, d->d_I, d->k_sel);
    if (d->k_sel > IC_MAX_K) return fail(IC_ERR_UNSUPPORTED, "k_sel=%d exceeds IC_MAX_K=%d", d->k_sel, IC_MAX_K);
    if (d->flags != 0) return fail(IC_ERR_UNSUPPORTED, "indexer flags must be 0");
    if (d->dtype != IC_BF16 && d->dtype != IC_FP8_E4M3) return fail(IC_ERR_UNSUPPORTED, "unknown dtype %d", d->dtype);
    if (!ic::score_shape_supported(d->dtype, d->H_I, d->d_I))
        return fail(IC_ERR_UNSUPPORTED, "indexer shape not covered: dtype=%d H_I=%d d_I=%d (H_I<=64; bf16: d_I in {64,128}; fp8: d_I = 128)",
                    d->dtype, d->H_I, d->d_I);
    if ((int64_t)d->B * d->Tq > INT32_MAX / 2 || (int64_t)d->B * d->Tq * d->k_sel > ((int64_t)1 << 40))
        return fail(IC_ERR_SHAPE, "B*Tq too large");
    if (d->q_pos0 < -(int64_t)d->Tq || d->q_pos0 > ((int64_t)1 << 40))
        return fail(IC_ERR_SHAPE, "q_pos0 out of range");
    if (d->dtype == IC_FP8_E4M3 && (!d->q_scale || !d->k_scale))
        return fail(IC_ERR_NULL, "fp8 indexer needs q_scale and k_scale");
    return IC_OK;
}

size_t strip_ld(const ic_indexer_desc *d) { return ((size_t)d->Lk + 63) / 64 * 64; }

// Rows of the strip a workspace of `bytes` can hold.
int64_t strip_rows(const ic_indexer_desc *d, size_t bytes) { return (int64_t)(bytes / (strip_ld(d) * sizeof(float))); }

ic_status check_attn(const ic_attn_desc *d)
{
    if (!d) return fail(IC_ERR_NULL, "attention descriptor is NULL");
    if (d->B <= 0 || d->Tq <= 0 || d->Lk <= 0 || d->H_q <= 0 || d->d_qk <= 0 || d->d_v <= 0 || d->k_sel <= 0 ||
        d->row_elems <= 0 || d->v_off < 0)
        return fail(IC_ERR_SHAPE, "attention sizes must be positive");
    if (d->H_q > IC_MAX_HEADS_Q) return fail(IC_ERR_UNSUPPORTED, "H_q=%d exceeds %d", d->H_q, IC_MAX_HEADS_Q);
    if (!ic::attn_shape_supported(d->d_qk, d->d_v))
        return fail(IC_ERR_UNSUPPORTED, "attention head dims not covered: d_qk=%d d_v=%d ((576,512) or (64,64))", d->d_qk, d->d_v);
    if (d->v_off % 8 != 0 || d->row_elems % 8 != 0)
        return fail(IC_ERR_SHAPE, "v_off and row_elems must be multiples of 8");
    const int staged = d->d_qk == 576 ? 576 : 128;   // features of a row the kernel stages
    if (d->v_off + d->d_v > staged || d->row_elems < staged)
        return fail(IC_ERR_UNSUPPORTED, "KV row layout not covered: need v_off+d_v <= %d <= row_elems", staged);
    if ((int64_t)d->B * d->Tq > INT32_MAX / 2) return fail(IC_ERR_SHAPE, "B*Tq too large");
    if (!(d->sm_scale > 0.f) || d->sm_scale > 1e6f) return fail(IC_ERR_SHAPE, "sm_scale must be positive and finite");
    return IC_OK;
}

// Key-slot splits per query.  MLA rows with the values in front run one workgroup per CU: one per
// query when there are at least 256 queries, otherwise the k_sel slots are split so that about 256
// workgroups exist.  The other layouts run two workgroups per CU and aim for 512.
void attn_splits(const ic_attn_desc *d, int *n_splits, int *split_len)
{
    const int64_t nq = (int64_t)d->B * d->Tq;
    const int tiles = (d->k_sel + 63) / 64;
    const int64_t wgs = (d->d_qk == 576 && d->v_off == 0) ? 256 : 512;
    int64_t want = nq >= wgs ? 1 : (wgs + nq - 1) / nq;
    if (want > tiles) want = tiles;
    const int tiles_per = (int)((tiles + want - 1) / want);
    *split_len = tiles_per * 64;
    *n_splits = (tiles + tiles_per - 1) / tiles_per;
}

size_t attn_ws_bytes(const ic_attn_desc *d)
{
    int ns, sl;
    attn_splits(d, &ns, &sl);
    if (ns <= 1) return 0;
    const size_t nq = (size_t)d->B * d->Tq;
    return align_up(nq * ns * d->H_q * d->d_v * 2) + align_up(nq * ns * d->H_q * 2 * sizeof(float));   // bf16 partial outputs, fp32 (max, sum)
}

// ragged / paged cache description -> the kernels' view (all-zero when pc is NULL)
ic::PagedView paged_view(const ic_paged_cache *pc)
{
    ic::PagedView v;
    memset(&v, 0, sizeof v);
    if (pc) {
        v.seq_lens = pc->seq_lens;
        v.page_table = pc->page_table;
        v.max_pages = pc->max_pages;
        int sh = 0;
        while ((1 << sh) < pc->page_size) ++sh;
        v.page_shift = sh;
    }
    return v;
}

ic_status check_paged(const ic_paged_cache *pc, int32_t Lk)
{
    if (!pc) return fail(IC_ERR_NULL, "paged cache descriptor is NULL");
    if (!pc->seq_lens && !pc->page_table) return fail(IC_ERR_NULL, "paged cache: seq_lens and page_table are both NULL");
    if (pc->page_table) {
        if (pc->page_size < 64 || (pc->page_size & (pc->page_size - 1)) != 0)
            return fail(IC_ERR_SHAPE, "page_size=%d must be a power of two >= 64", pc->page_size);
        if (pc->max_pages <= 0 || (int64_t)pc->max_pages * pc->page_size < Lk)
            return fail(IC_ERR_SHAPE, "page table rows of %d pages x %d positions do not cover Lk=%d", pc->max_pages, pc->page_size, Lk);
    }
    return IC_OK;
}

ic_status run_indexer(const ic_indexer_desc *d, const void *q, const void *k, const float *w, int32_t *idx,
                      float *sel, void *ws, size_t ws_bytes, hipStream_t st, const ic_paged_cache *pc = nullptr)
{
    const int64_t rows_cap = strip_rows(d, ws_bytes);
    const int Ri = (int)(d->Tq < rows_cap ? d->Tq : rows_cap);
    int64_t bc64 = rows_cap / Ri;
    const int Bc = (int)(bc64 < 1 ? 1 : (bc64 > d->B ? d->B : bc64));
    ic::ScoreArgs sa;
    memset(&sa, 0, sizeof sa);
    sa.q = q;
    sa.k = k;
    sa.w = w;
    sa.q_scale = d->q_scale;
    sa.k_scale = d->k_scale;
    sa.strip = (float *)ws;
    sa.ld = (int64_t)strip_ld(d);
    sa.q_pos0 = d->q_pos0;
    sa.Tq = d->Tq;
    sa.Lk = d->Lk;
    sa.H_I = d->H_I;
    sa.pv = paged_view(pc);
    ic::SelectArgs se;
    memset(&se, 0, sizeof se);
    se.strip = (const float *)ws;
    se.ld = sa.ld;
    se.q_pos0 = d->q_pos0;
    se.Tq = d->Tq;
    se.Lk = d->Lk;
    se.k_sel = d->k_sel;
    se.idx = idx;
    se.sel = sel;
    se.seq_lens = pc ? pc->seq_lens : nullptr;
    for (int b0 = 0; b0 < d->B; b0 += Bc) {
        const int bc = d->B - b0 < Bc ? d->B - b0 : Bc;
        for (int i0 = 0; i0 < d->Tq; i0 += Ri) {
            const int ri = d->Tq - i0 < Ri ? d->Tq - i0 : Ri;
            sa.b0 = b0;
            sa.i0 = i0;
            sa.Ri = ri;
            int64_t max_vis = d->q_pos0 + i0 + ri;
            max_vis = max_vis < 0 ? 0 : (max_vis > d->Lk ? d->Lk : max_vis);
            if (pc && pc->seq_lens) max_vis = d->Lk;   // ragged: lengths are device data, Lk bounds them
            if (max_vis > d->k_sel || sel) {   // rows with <= k_sel visible keys need no scores
                ProfScope ps(0, st);
                hipError_t e = ic::launch_score(sa, d->dtype, d->d_I, bc, st);
                if (e != hipSuccess) return fail(IC_ERR_HIP, "indexer score launch failed: %s", hipGetErrorString(e));
            }
            se.b0 = b0;
            se.i0 = i0;
            se.Ri = ri;
            {
                ProfScope ps(1, st);
                hipError_t e = ic::launch_select(se, bc * ri, (int)max_vis, st);
                if (e != hipSuccess) return fail(IC_ERR_HIP, "top-k select launch failed: %s", hipGetErrorString(e));
            }
        }
    }
    g_indexer_launches.fetch_add(1);
    return IC_OK;
}

ic_status check_ws(void *ws, size_t have, size_t need)
{
    if (need == 0) return IC_OK;
    if (!ws) return fail(IC_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    if (((uintptr_t)ws) % kAlign != 0) return fail(IC_ERR_WORKSPACE, "workspace must be %zu-byte aligned", kAlign);
    if (have < need) return fail(IC_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", have, need);
    return IC_OK;
}

size_t indexer_min_ws(const ic_indexer_desc *d)
{
    // at least kMinStripRows rows (or every row of one sequence when there are fewer)
    const int64_t rows = d->Tq < kMinStripRows ? d->Tq : kMinStripRows;
    return align_up((size_t)rows * strip_ld(d) * sizeof(float));
}

// causal_pos0 >= 0: idx is this library's causal top-k for query rows at positions causal_pos0 + t (rows that can hold
// fewer than k_sel entries end in -1s, and the kernel leaves their empty tiles out); -1: idx is the caller's own
ic_status run_attn(const ic_attn_desc *d, const void *Q, const void *KV, const int32_t *idx, void *O, float *lse,
                   void *ws, hipStream_t st, const ic_paged_cache *pc = nullptr, int64_t causal_pos0 = -1)
{
    ic::AttnArgs a;
    memset(&a, 0, sizeof a);
    a.Q = Q;
    a.KV = KV;
    a.idx = idx;
    a.O = O;
    a.lse = lse;
    a.B = d->B;
    a.Tq = d->Tq;
    a.Lk = d->Lk;
    a.H_q = d->H_q;
    a.v_off = d->v_off;
    a.row_elems = d->row_elems;
    a.k_sel = d->k_sel;
    attn_splits(d, &a.n_splits, &a.split_len);
    a.scale_log2e = d->sm_scale * 1.4426950408889634f;
    a.pv = paged_view(pc);
    a.causal_pos0 = causal_pos0;
    if (a.n_splits > 1) {
        const size_t nq = (size_t)d->B * d->Tq;
        a.part_o = (__bf16 *)ws;
        a.part_ml = (float *)((char *)ws + align_up(nq * a.n_splits * d->H_q * d->d_v * 2));
    }
    {
        ProfScope ps(2, st);
        hipError_t e = ic::launch_attn(a, d->d_qk, d->d_v, st);
        if (e != hipSuccess) return fail(IC_ERR_HIP, "sparse attention launch failed: %s", hipGetErrorString(e));
    }
    if (a.n_splits > 1) {
        ProfScope ps(3, st);
        hipError_t e = ic::launch_attn_merge(a, d->d_v, st);
        if (e != hipSuccess) return fail(IC_ERR_HIP, "attention merge launch failed: %s", hipGetErrorString(e));
    }
    return IC_OK;
}

} // namespace

extern "C" {

const char *ic_last_error(void) { return g_err; }

size_t ic_indexer_topk_workspace(const ic_indexer_desc *d)
{
    if (check_indexer(d) != IC_OK) return 0;
    const size_t row_bytes = strip_ld(d) * sizeof(float);
    const size_t all = (size_t)d->B * d->Tq * row_bytes;
    // small problems keep every row in flight; larger ones at most a quarter of their rows and at most the budget,
    // so that the scores of a long sequence are never all resident at once
    size_t want = all;
    if (all > kSmallStrip) {
        want = all / 4 > kSmallStrip ? all / 4 : kSmallStrip;
        if (want > kStripBudget) want = kStripBudget;
    }
    const size_t min_b = indexer_min_ws(d);
    if (want < min_b) want = min_b;
    return align_up(want / row_bytes * row_bytes);
}

ic_status ic_indexer_topk(const ic_indexer_desc *d, const void *q, const void *k, const float *w, int32_t *idx,
                          float *sel_scores, void *workspace, size_t workspace_bytes, void *stream)
{
    ic_status s = check_indexer(d);
    if (s != IC_OK) return s;
    if (!q || !k || !w || !idx) return fail(IC_ERR_NULL, "q, k, w and idx must not be NULL");
    s = check_ws(workspace, workspace_bytes, indexer_min_ws(d));
    if (s != IC_OK) return s;
    return run_indexer(d, q, k, w, idx, sel_scores, workspace, workspace_bytes, (hipStream_t)stream);
}

size_t ic_sparse_attn_workspace(const ic_attn_desc *d)
{
    if (check_attn(d) != IC_OK) return 0;
    return attn_ws_bytes(d);
}

ic_status ic_sparse_attn(const ic_attn_desc *d, const void *Q, const void *KV, const int32_t *idx, void *O,
                         float *lse, void *workspace, size_t workspace_bytes, void *stream)
{
    ic_status s = check_attn(d);
    if (s != IC_OK) return s;
    if (!Q || !KV || !idx || !O) return fail(IC_ERR_NULL, "Q, KV, idx and O must not be NULL");
    s = check_ws(workspace, workspace_bytes, attn_ws_bytes(d));
    if (s != IC_OK) return s;
    return run_attn(d, Q, KV, idx, O, lse, workspace, (hipStream_t)stream);
}

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of the current GPU's copy of `scratch`, looked up once per device.
ic_status static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(IC_ERR_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(IC_ERR_HIP, "address of the static scratch on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return IC_OK;
}
} // namespace

ic_status ic_sparse_attn_static(const ic_attn_desc *d, const void *Q, const void *KV, const int32_t *idx, void *O,
                                float *lse, void *stream)
{
    ic_status s = check_attn(d);
    if (s != IC_OK) return s;
    if (!Q || !KV || !idx || !O) return fail(IC_ERR_NULL, "Q, KV, idx and O must not be NULL");
    const size_t need = attn_ws_bytes(d);
    if (need > (size_t)IC_STATIC_SCRATCH_BYTES)
        return fail(IC_ERR_WORKSPACE, "this shape needs %zu bytes of split-attention scratch, the static scratch holds %zu",
                    need, (size_t)IC_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    if (need > 0) {
        s = static_scratch(&ws);
        if (s != IC_OK) return s;
    }
    return run_attn(d, Q, KV, idx, O, lse, ws, (hipStream_t)stream);
}

static ic_status check_stack(const ic_layer *layers, int32_t n, const uint8_t *full_mask)
{
    if (!layers) return fail(IC_ERR_NULL, "layers is NULL");
    if (n <= 0) return fail(IC_ERR_SHAPE, "n_layers must be positive");
    if (full_mask) {
        if (!full_mask[0]) return fail(IC_ERR_PATTERN, "the first layer must be Full: there are no indices to reuse yet");
    }
    int32_t idx_lk = 0;                        // key range the cached indices were drawn from (the last Full layer's)
    for (int l = 0; l < n; ++l) {
        const ic_layer *L = &layers[l];
        const bool full = !full_mask || full_mask[l];
        ic_status s = check_attn(&L->at);
        if (s != IC_OK) return s;
        if (!L->Q || !L->KV || !L->O) return fail(IC_ERR_NULL, "layer %d: Q, KV and O must not be NULL", l);
        if (full) {
            s = check_indexer(&L->ix);
            if (s != IC_OK) return s;
            if (!L->q || !L->k || !L->w) return fail(IC_ERR_NULL, "Full layer %d: q, k and w must not be NULL", l);
            if (L->ix.B != L->at.B || L->ix.Tq != L->at.Tq || L->ix.k_sel != L->at.k_sel)
                return fail(IC_ERR_SHAPE, "layer %d: indexer and attention disagree on B, Tq or k_sel", l);
            if (L->ix.Lk != L->at.Lk)
                return fail(IC_ERR_SHAPE, "layer %d: indexer scores %d keys but the KV cache holds %d rows", l, L->ix.Lk, L->at.Lk);
            idx_lk = L->ix.Lk;
        } else if (L->at.Lk < idx_lk) {
            // a Shared layer reads positions selected among idx_lk keys: its own cache must hold them all
            return fail(IC_ERR_SHAPE, "Shared layer %d: its KV cache holds %d rows, the inherited indices cover %d", l, L->at.Lk, idx_lk);
        }
        if (L->at.B != layers[0].at.B || L->at.Tq != layers[0].at.Tq || L->at.k_sel != layers[0].at.k_sel)
            return fail(IC_ERR_SHAPE, "layer %d: all layers must share B, Tq and k_sel (one index buffer)", l);
    }
    return IC_OK;
}

size_t ic_forward_stack_workspace(const ic_layer *layers, int32_t n_layers)
{
    if (!layers || n_layers <= 0) return 0;
    size_t need = 0;
    for (int l = 0; l < n_layers; ++l) {
        size_t a = ic_sparse_attn_workspace(&layers[l].at);
        size_t b = layers[l].q ? ic_indexer_topk_workspace(&layers[l].ix) : 0;
        if (a > need) need = a;
        if (b > need) need = b;
    }
    return need;
}

static ic_status forward_stack_impl(const ic_layer *layers, int32_t n_layers, const uint8_t *full_mask, const ic_paged_cache *pc,
                                    int32_t *idx_cache, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!full_mask) return fail(IC_ERR_NULL, "full_mask is NULL");
    if (!idx_cache) return fail(IC_ERR_NULL, "idx_cache is NULL");
    ic_status s = check_stack(layers, n_layers, full_mask);
    if (s != IC_OK) return s;
    if (pc) {
        for (int l = 0; l < n_layers; ++l) {
            s = check_paged(pc, layers[l].at.Lk);
            if (s != IC_OK) return s;
            if (full_mask[l] && pc->page_table && layers[l].ix.dtype != IC_BF16)
                return fail(IC_ERR_UNSUPPORTED, "layer %d: a paged index-key cache must be bf16", l);
        }
    }
    size_t need = 0;
    for (int l = 0; l < n_layers; ++l) {
        size_t a = attn_ws_bytes(&layers[l].at);
        size_t b = full_mask[l] ? indexer_min_ws(&layers[l].ix) : 0;
        if (a > need) need = a;
        if (b > need) need = b;
    }
    s = check_ws(workspace, workspace_bytes, need);
    if (s != IC_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    int64_t idx_pos0 = -1;                     // position of query row 0 when the cached indices were selected
    for (int l = 0; l < n_layers; ++l) {
        const ic_layer *L = &layers[l];
        if (full_mask[l]) {   // Full: fresh indices overwrite the cache; Shared: cache left as it is
            s = run_indexer(&L->ix, L->q, L->k, L->w, idx_cache, nullptr, workspace, workspace_bytes, st, pc);
            if (s != IC_OK) return s;
            idx_pos0 = (pc && pc->seq_lens) ? -1 : (L->ix.q_pos0 >= 0 ? (int64_t)L->ix.q_pos0 : -1);
        }
        s = run_attn(&L->at, L->Q, L->KV, idx_cache, L->O, nullptr, workspace, st, pc, idx_pos0);
        if (s != IC_OK) return s;
    }
    return IC_OK;
}

ic_status ic_forward_stack(const ic_layer *layers, int32_t n_layers, const uint8_t *full_mask, int32_t *idx_cache,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    return forward_stack_impl(layers, n_layers, full_mask, nullptr, idx_cache, workspace, workspace_bytes, stream);
}

ic_status ic_forward_stack_paged(const ic_layer *layers, int32_t n_layers, const uint8_t *full_mask, const ic_paged_cache *pc,
                                 int32_t *idx_cache, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!pc) return fail(IC_ERR_NULL, "paged cache descriptor is NULL");
    return forward_stack_impl(layers, n_layers, full_mask, pc, idx_cache, workspace, workspace_bytes, stream);
}

ic_status ic_indexer_topk_paged(const ic_indexer_desc *d, const ic_paged_cache *pc, const void *q, const void *k_pool,
                                const float *w, int32_t *idx, float *sel_scores, void *workspace, size_t workspace_bytes,
                                void *stream)
{
    ic_status s = check_indexer(d);
    if (s != IC_OK) return s;
    s = check_paged(pc, d->Lk);
    if (s != IC_OK) return s;
    if (pc->page_table && d->dtype != IC_BF16) return fail(IC_ERR_UNSUPPORTED, "a paged index-key cache must be bf16");
    if (!q || !k_pool || !w || !idx) return fail(IC_ERR_NULL, "q, k_pool, w and idx must not be NULL");
    s = check_ws(workspace, workspace_bytes, indexer_min_ws(d));
    if (s != IC_OK) return s;
    return run_indexer(d, q, k_pool, w, idx, sel_scores, workspace, workspace_bytes, (hipStream_t)stream, pc);
}

ic_status ic_sparse_attn_paged(const ic_attn_desc *d, const ic_paged_cache *pc, const void *Q, const void *KV_pool,
                               const int32_t *idx, void *O, float *lse, void *workspace, size_t workspace_bytes, void *stream)
{
    ic_status s = check_attn(d);
    if (s != IC_OK) return s;
    s = check_paged(pc, d->Lk);
    if (s != IC_OK) return s;
    if (!Q || !KV_pool || !idx || !O) return fail(IC_ERR_NULL, "Q, KV_pool, idx and O must not be NULL");
    s = check_ws(workspace, workspace_bytes, attn_ws_bytes(d));
    if (s != IC_OK) return s;
    return run_attn(d, Q, KV_pool, idx, O, lse, workspace, (hipStream_t)stream, pc);
}

ic_status ic_pattern_from_string(const char *fs, uint8_t *full_mask, int32_t n)
{
    if (!fs || !full_mask) return fail(IC_ERR_NULL, "pattern string and mask must not be NULL");
    if (n <= 0) return fail(IC_ERR_SHAPE, "n must be positive");
    if ((int64_t)strlen(fs) != n) return fail(IC_ERR_SHAPE, "pattern has %zu characters, expected %d", strlen(fs), n);
    for (int l = 0; l < n; ++l) {
        if (fs[l] == 'F')
            full_mask[l] = 1;
        else if (fs[l] == 'S')
            full_mask[l] = 0;
        else
            return fail(IC_ERR_PATTERN, "pattern character %d is '%c', expected F or S", l, fs[l]);
    }
    if (!full_mask[0]) return fail(IC_ERR_PATTERN, "the first layer must be Full");
    return IC_OK;
}

ic_status ic_pattern_uniform(int32_t n, int32_t r, uint8_t *full_mask)
{
    if (!full_mask) return fail(IC_ERR_NULL, "mask must not be NULL");
    if (n <= 0 || r <= 0) return fail(IC_ERR_SHAPE, "n and r must be positive");
    for (int l = 0; l < n; ++l) full_mask[l] = (l % r) == 0;
    return IC_OK;
}

size_t ic_cosine_rows_workspace(void) { return kAlign; }

ic_status ic_cosine_rows(const void *A, const void *B, int64_t n_rows, int64_t row_len, double *mean, float *per_row,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (!A || !B || !mean) return fail(IC_ERR_NULL, "A, B and mean must not be NULL");
    if (n_rows <= 0 || row_len <= 0 || n_rows > INT32_MAX) return fail(IC_ERR_SHAPE, "n_rows and row_len must be positive");
    ic_status s = check_ws(workspace, workspace_bytes, ic_cosine_rows_workspace());
    if (s != IC_OK) return s;
    hipError_t e = ic::launch_cosine(A, B, n_rows, row_len, mean, per_row, (double *)workspace, (hipStream_t)stream);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "cosine launch failed: %s", hipGetErrorString(e));
    return IC_OK;
}

namespace {

// layers of the similarity matrix share one attention shape (any layer's index tensor fits any layer)
ic_status check_sim_layers(const ic_layer *layers, int32_t n_layers)
{
    if (!layers) return fail(IC_ERR_NULL, "layers is NULL");
    if (n_layers <= 0 || n_layers > IC_MAX_OVERLAP_LAYERS)
        return fail(IC_ERR_SHAPE, "n_layers must be in [1, %d]", IC_MAX_OVERLAP_LAYERS);
    for (int l = 0; l < n_layers; ++l) {
        ic_status s = check_attn(&layers[l].at);
        if (s != IC_OK) return s;
        if (!layers[l].Q || !layers[l].KV || !layers[l].O) return fail(IC_ERR_NULL, "layer %d: Q, KV and O must not be NULL", l);
        const ic_attn_desc &a = layers[l].at, &b = layers[0].at;
        if (a.B != b.B || a.Tq != b.Tq || a.k_sel != b.k_sel || a.H_q != b.H_q || a.d_v != b.d_v)
            return fail(IC_ERR_SHAPE, "layer %d: attention shape differs from layer 0", l);
    }
    return IC_OK;
}

size_t sim_o_bytes(const ic_attn_desc *a) { return align_up((size_t)a->B * a->Tq * a->H_q * a->d_v * 2); }

} // namespace

size_t ic_similarity_matrix_workspace(const ic_layer *layers, int32_t n_layers)
{
    if (!layers || n_layers <= 0 || n_layers > IC_MAX_OVERLAP_LAYERS) return 0;
    size_t at = 0;
    for (int l = 0; l < n_layers; ++l) {
        const size_t a = attn_ws_bytes(&layers[l].at);
        if (a > at) at = a;
    }
    return sim_o_bytes(&layers[0].at) + align_up(at) + kAlign;
}

ic_status ic_similarity_matrix(const ic_layer *layers, int32_t n_layers, const int32_t *const *idx_layers, double *S,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    ic_status s = check_sim_layers(layers, n_layers);
    if (s != IC_OK) return s;
    if (!idx_layers || !S) return fail(IC_ERR_NULL, "idx_layers and S must not be NULL");
    for (int l = 0; l < n_layers; ++l)
        if (!idx_layers[l]) return fail(IC_ERR_NULL, "idx_layers[%d] is NULL", l);
    s = check_ws(workspace, workspace_bytes, ic_similarity_matrix_workspace(layers, n_layers));
    if (s != IC_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    void *o_reuse = ws;
    void *attn_ws = ws + sim_o_bytes(&layers[0].at);
    double *acc = (double *)(ws + ic_similarity_matrix_workspace(layers, n_layers) - kAlign);
    hipError_t e = ic::launch_sim_init(S, n_layers, st);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "similarity init failed: %s", hipGetErrorString(e));
    const ic_attn_desc *a0 = &layers[0].at;
    const int64_t n_rows = (int64_t)a0->B * a0->Tq, row_len = (int64_t)a0->H_q * a0->d_v;
    for (int i = 0; i < n_layers; ++i) {
        const ic_layer *L = &layers[i];
        s = run_attn(&L->at, L->Q, L->KV, idx_layers[i], L->O, nullptr, attn_ws, st);       // own indices
        if (s != IC_OK) return s;
        for (int j = 0; j < i; ++j) {
            s = run_attn(&L->at, L->Q, L->KV, idx_layers[j], o_reuse, nullptr, attn_ws, st); // as a Shared layer reading j
            if (s != IC_OK) return s;
            e = ic::launch_cosine(L->O, o_reuse, n_rows, row_len, S + (size_t)i * n_layers + j, nullptr, acc, st);
            if (e != hipSuccess) return fail(IC_ERR_HIP, "cosine launch failed: %s", hipGetErrorString(e));
        }
    }
    return IC_OK;
}

ic_status ic_pattern_search_dp(const double *S, int32_t n_layers, int32_t n_full, uint8_t *full_mask, double *total)
{
    if (!S || !full_mask) return fail(IC_ERR_NULL, "S and full_mask must not be NULL");
    if (n_layers <= 0 || n_full <= 0 || n_full > n_layers)
        return fail(IC_ERR_SHAPE, "need 1 <= n_full <= n_layers (n_full=%d n_layers=%d)", n_full, n_layers);
    const int N = n_layers, M = n_full;
    // run[j][i] = sum of S[m][j] over j < m < i: what the Shared layers between Full layers j and i collect
    std::vector<double> run((size_t)N * (N + 1), 0.0);
    for (int j = 0; j < N; ++j)
        for (int i = j + 1; i <= N; ++i)
            run[(size_t)j * (N + 1) + i] = (i == j + 1) ? 0.0 : run[(size_t)j * (N + 1) + i - 1] + S[(size_t)(i - 1) * N + j];
    const double NEG = -1e300;
    std::vector<double> dp((size_t)N * (M + 1), NEG);       // dp[i][c]: layer i Full, c Full layers in 0..i
    std::vector<int> from((size_t)N * (M + 1), -1);
    dp[(size_t)0 * (M + 1) + 1] = 0.0;                         // the first layer is always Full
    for (int i = 1; i < N; ++i)
        for (int c = 2; c <= M && c <= i + 1; ++c)
            for (int j = c - 2; j < i; ++j) {
                const double prev = dp[(size_t)j * (M + 1) + c - 1];
                if (prev <= NEG) continue;
                const double v = prev + run[(size_t)j * (N + 1) + i];
                if (v > dp[(size_t)i * (M + 1) + c]) {
                    dp[(size_t)i * (M + 1) + c] = v;
                    from[(size_t)i * (M + 1) + c] = j;
                }
            }
    double best = NEG;
    int last = -1;
    for (int i = M - 1; i < N; ++i) {                          // the last Full layer; everything after it reads it
        const double prev = dp[(size_t)i * (M + 1) + M];
        if (prev <= NEG) continue;
        const double v = prev + run[(size_t)i * (N + 1) + N];
        if (v > best) {
            best = v;
            last = i;
        }
    }
    if (last < 0) return fail(IC_ERR_SHAPE, "no pattern with %d Full layers", M);
    for (int l = 0; l < N; ++l) full_mask[l] = 0;
    for (int i = last, c = M; i >= 0 && c >= 1; --c) {
        full_mask[i] = 1;
        i = from[(size_t)i * (M + 1) + c];
    }
    if (total) *total = best;
    return IC_OK;
}

// ---- greedy layer selection (paper Alg. 1) over a surrogate loss ---------------------------------

extern "C++" {
namespace {

// Alg. 1 with the blocked variant of Sec. 3.2: `eval` fills losses[i] with the loss of the current
// pattern with layer cands[i] flipped to Shared as well.  Ties go to the lowest layer.
template <typename Eval>
ic_status greedy_core(int N, int K, int P, uint8_t *mask, int32_t *order, double *curve, Eval eval)
{
    if (N <= 0 || K < 0 || K > N - 1 || P < 1 || P > N)
        return fail(IC_ERR_SHAPE, "need 0 <= n_shared <= n_layers-1 and 1 <= n_blocks <= n_layers (n_layers=%d n_shared=%d n_blocks=%d)", N, K, P);
    const int size = (N + P - 1) / P;
    int n_cand = 0;
    for (int b0 = 0; b0 < N; b0 += size) n_cand += (b0 + size < N ? size : N - b0) - 1;   // a block's first layer stays Full
    if (K > n_cand) return fail(IC_ERR_SHAPE, "n_shared=%d but only %d layers may become Shared with %d blocks", K, n_cand, P);
    for (int l = 0; l < N; ++l) mask[l] = 1;
    std::vector<int32_t> cands;
    std::vector<double> losses;
    int done = 0;
    while (done < K) {
        for (int b0 = 0; b0 < N && done < K; b0 += size) {
            const int b1 = b0 + size < N ? b0 + size : N;
            cands.clear();
            for (int l = b0 + 1; l < b1; ++l)
                if (mask[l]) cands.push_back(l);
            if (cands.empty()) continue;
            losses.assign(cands.size(), 0.0);
            ic_status s = eval(mask, cands, losses);
            if (s != IC_OK) return s;
            size_t arg = 0;
            for (size_t i = 1; i < cands.size(); ++i)
                if (losses[i] < losses[arg]) arg = i;
            mask[cands[arg]] = 0;
            if (order) order[done] = cands[arg];
            if (curve) curve[done] = losses[arg];
            ++done;
        }
    }
    return IC_OK;
}

size_t pattern_loss_ws(const ic_layer *layers, int32_t n_layers)
{
    size_t fw = ic_forward_stack_workspace(layers, n_layers);
    return align_up(fw) + align_up((size_t)n_layers * sizeof(double)) + kAlign;
}

ic_status run_pattern_loss(const ic_layer *layers, int32_t n_layers, const uint8_t *full_mask, const void *const *O_ref,
                           int32_t *idx_cache, double *loss, void *workspace, hipStream_t st)
{
    char *ws = (char *)workspace;
    const size_t fw = align_up(ic_forward_stack_workspace(layers, n_layers));
    double *sims = (double *)(ws + fw);
    double *acc = (double *)(ws + fw + align_up((size_t)n_layers * sizeof(double)));
    ic_status s = ic_forward_stack(layers, n_layers, full_mask, idx_cache, workspace, fw, (void *)st);
    if (s != IC_OK) return s;
    const ic_attn_desc *a0 = &layers[0].at;
    const int64_t n_rows = (int64_t)a0->B * a0->Tq, row_len = (int64_t)a0->H_q * a0->d_v;
    for (int l = 0; l < n_layers; ++l) {
        hipError_t e = ic::launch_cosine(layers[l].O, O_ref[l], n_rows, row_len, sims + l, nullptr, acc, st);
        if (e != hipSuccess) return fail(IC_ERR_HIP, "cosine launch failed: %s", hipGetErrorString(e));
    }
    hipError_t e = ic::launch_loss_finish(sims, n_layers, loss, st);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "loss reduction launch failed: %s", hipGetErrorString(e));
    return IC_OK;
}

ic_status check_loss_args(const ic_layer *layers, int32_t n_layers, const void *const *O_ref, const int32_t *idx_cache)
{
    ic_status s = check_sim_layers(layers, n_layers);
    if (s != IC_OK) return s;
    if (!O_ref || !idx_cache) return fail(IC_ERR_NULL, "O_ref and idx_cache must not be NULL");
    for (int l = 0; l < n_layers; ++l) {
        if (!O_ref[l]) return fail(IC_ERR_NULL, "O_ref[%d] is NULL", l);
        if (O_ref[l] == layers[l].O) return fail(IC_ERR_SHAPE, "O_ref[%d] is the layer's own output buffer", l);
    }
    return IC_OK;
}

} // namespace
} // extern "C++"

ic_status ic_pattern_search_greedy(const double *S, int32_t n_layers, int32_t n_shared, int32_t n_blocks,
                                   uint8_t *full_mask, int32_t *order, double *loss_curve)
{
    if (!S || !full_mask) return fail(IC_ERR_NULL, "S and full_mask must not be NULL");
    const int N = n_layers;
    auto loss_of = [&](const uint8_t *m) {
        double t = 0.0;
        int src = 0;
        for (int l = 0; l < N; ++l) {
            if (m[l]) src = l;
            else t += 1.0 - S[(size_t)l * N + src];
        }
        return t / N;
    };
    return greedy_core(N, n_shared, n_blocks, full_mask, order, loss_curve,
                       [&](uint8_t *m, const std::vector<int32_t> &cands, std::vector<double> &out) {
                           for (size_t i = 0; i < cands.size(); ++i) {
                               m[cands[i]] = 0;
                               out[i] = loss_of(m);
                               m[cands[i]] = 1;
                           }
                           return IC_OK;
                       });
}

size_t ic_pattern_loss_workspace(const ic_layer *layers, int32_t n_layers)
{
    if (!layers || n_layers <= 0 || n_layers > IC_MAX_OVERLAP_LAYERS) return 0;
    return pattern_loss_ws(layers, n_layers);
}

ic_status ic_pattern_loss(const ic_layer *layers, int32_t n_layers, const uint8_t *full_mask, const void *const *O_ref,
                          int32_t *idx_cache, double *loss, void *workspace, size_t workspace_bytes, void *stream)
{
    ic_status s = check_loss_args(layers, n_layers, O_ref, idx_cache);
    if (s != IC_OK) return s;
    if (!full_mask || !loss) return fail(IC_ERR_NULL, "full_mask and loss must not be NULL");
    s = check_ws(workspace, workspace_bytes, pattern_loss_ws(layers, n_layers));
    if (s != IC_OK) return s;
    return run_pattern_loss(layers, n_layers, full_mask, O_ref, idx_cache, loss, workspace, (hipStream_t)stream);
}

size_t ic_greedy_search_forward_workspace(const ic_layer *layers, int32_t n_layers)
{
    if (!layers || n_layers <= 0 || n_layers > IC_MAX_OVERLAP_LAYERS) return 0;
    return pattern_loss_ws(layers, n_layers) + align_up((size_t)n_layers * sizeof(double));
}

ic_status ic_greedy_search_forward(const ic_layer *layers, int32_t n_layers, int32_t n_shared, int32_t n_blocks,
                                   const void *const *O_ref, int32_t *idx_cache, uint8_t *full_mask, int32_t *order,
                                   double *loss_curve, void *workspace, size_t workspace_bytes, void *stream)
{
    ic_status s = check_loss_args(layers, n_layers, O_ref, idx_cache);
    if (s != IC_OK) return s;
    if (!full_mask) return fail(IC_ERR_NULL, "full_mask must not be NULL");
    s = check_ws(workspace, workspace_bytes, ic_greedy_search_forward_workspace(layers, n_layers));
    if (s != IC_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    double *dev_losses = (double *)((char *)workspace + pattern_loss_ws(layers, n_layers));
    return greedy_core(n_layers, n_shared, n_blocks, full_mask, order, loss_curve,
                       [&](uint8_t *m, const std::vector<int32_t> &cands, std::vector<double> &out) {
                           // one forward pass of the whole stack per candidate, all on the stream;
                           // then the host needs the losses to choose: one synchronisation per search step
                           for (size_t i = 0; i < cands.size(); ++i) {
                               m[cands[i]] = 0;
                               ic_status r = run_pattern_loss(layers, n_layers, m, O_ref, idx_cache, dev_losses + i, workspace, st);
                               m[cands[i]] = 1;
                               if (r != IC_OK) return r;
                           }
                           hipError_t e = hipStreamSynchronize(st);
                           if (e == hipSuccess) e = hipMemcpy(out.data(), dev_losses, cands.size() * sizeof(double), hipMemcpyDeviceToHost);
                           if (e != hipSuccess) return fail(IC_ERR_HIP, "reading the candidate losses failed: %s", hipGetErrorString(e));
                           return IC_OK;
                       });
}

// ---- distillation loss forward (paper Sec. 3.3) ---------------------------------------------------

ic_status ic_attn_probs(const ic_attn_desc *d, const void *Q, const void *KV, const int32_t *idx, const float *lse,
                        float *probs, void *stream)
{
    ic_status s = check_attn(d);
    if (s != IC_OK) return s;
    if (!Q || !KV || !idx || !lse || !probs) return fail(IC_ERR_NULL, "Q, KV, idx, lse and probs must not be NULL");
    ic::ProbsArgs a;
    memset(&a, 0, sizeof a);
    a.Q = Q;
    a.KV = KV;
    a.idx = idx;
    a.lse = lse;
    a.probs = probs;
    a.B = d->B;
    a.Tq = d->Tq;
    a.Lk = d->Lk;
    a.H_q = d->H_q;
    a.row_elems = d->row_elems;
    a.k_sel = d->k_sel;
    a.scale_log2e = d->sm_scale * 1.4426950408889634f;
    hipError_t e = ic::launch_attn_probs(a, d->d_qk, (hipStream_t)stream);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "attention-probability launch failed: %s", hipGetErrorString(e));
    return IC_OK;
}

size_t ic_distill_loss_workspace(int64_t nq)
{
    if (nq <= 0) return kAlign;
    return 2 * align_up((size_t)nq * sizeof(double));
}

ic_status ic_distill_loss(const float *const *probs, int32_t n_targets, const float *sel_scores, int64_t nq, int32_t k_sel,
                          double *loss_multi, double *loss_avg, float *grad, void *workspace, size_t workspace_bytes,
                          void *stream)
{
    if (!probs || !sel_scores) return fail(IC_ERR_NULL, "probs and sel_scores must not be NULL");
    if (n_targets < 1 || n_targets > IC_MAX_DISTILL_TARGETS)
        return fail(IC_ERR_SHAPE, "n_targets=%d must be in [1, %d]", n_targets, IC_MAX_DISTILL_TARGETS);
    if (nq < 0 || nq > INT32_MAX || k_sel <= 0) return fail(IC_ERR_SHAPE, "need 0 <= nq <= 2^31-1 and k_sel > 0");
    for (int j = 0; j < n_targets; ++j)
        if (!probs[j]) return fail(IC_ERR_NULL, "probs[%d] is NULL", j);
    if (!loss_multi && !loss_avg && !grad) return fail(IC_ERR_NULL, "at least one output must be given");
    ic_status s = check_ws(workspace, workspace_bytes, ic_distill_loss_workspace(nq));
    if (s != IC_OK) return s;
    ic::DistillArgs a;
    memset(&a, 0, sizeof a);
    for (int j = 0; j < n_targets; ++j) a.probs[j] = probs[j];
    a.n_targets = n_targets;
    a.k_sel = k_sel;
    a.scores = sel_scores;
    a.row_multi = (double *)workspace;
    a.row_avg = (double *)((char *)workspace + align_up((size_t)(nq > 0 ? nq : 1) * sizeof(double)));
    a.grad = grad;
    hipError_t e = ic::launch_distill(a, nq, loss_multi, loss_avg, (hipStream_t)stream);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "distillation loss launch failed: %s", hipGetErrorString(e));
    return IC_OK;
}

size_t ic_topk_overlap_workspace(int32_t n_layers)
{
    if (n_layers <= 0 || n_layers > IC_MAX_OVERLAP_LAYERS) return 0;
    return align_up(ic::overlap_ws_bytes(n_layers));
}

ic_status ic_topk_overlap(const int32_t *const *idx_layers, int32_t n_layers, int64_t nq, int32_t k_sel, int32_t Lk,
                          double *overlap, uint64_t *inter, uint64_t *sizes, void *workspace, size_t workspace_bytes,
                          void *stream)
{
    if (!idx_layers) return fail(IC_ERR_NULL, "idx_layers must not be NULL");
    if (n_layers <= 0 || nq < 0 || k_sel <= 0 || Lk <= 0) return fail(IC_ERR_SHAPE, "overlap sizes must be positive");
    if (n_layers > IC_MAX_OVERLAP_LAYERS)
        return fail(IC_ERR_UNSUPPORTED, "n_layers=%d exceeds IC_MAX_OVERLAP_LAYERS=%d", n_layers, IC_MAX_OVERLAP_LAYERS);
    if (Lk > IC_MAX_OVERLAP_LK) return fail(IC_ERR_UNSUPPORTED, "Lk=%d exceeds IC_MAX_OVERLAP_LK=%d", Lk, IC_MAX_OVERLAP_LK);
    if ((nq + 15) / 16 * n_layers > (int64_t)INT32_MAX) return fail(IC_ERR_SHAPE, "nq * n_layers too large");
    for (int l = 0; l < n_layers; ++l)
        if (!idx_layers[l]) return fail(IC_ERR_NULL, "idx_layers[%d] is NULL", l);
    if (!overlap && !inter && !sizes) return fail(IC_ERR_NULL, "at least one output must be given");
    ic_status s = check_ws(workspace, workspace_bytes, ic_topk_overlap_workspace(n_layers));
    if (s != IC_OK) return s;
    hipError_t e = ic::launch_overlap(idx_layers, n_layers, nq, k_sel, Lk, overlap, (unsigned long long *)inter,
                                      (unsigned long long *)sizes, workspace, (hipStream_t)stream);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "overlap launch failed: %s", hipGetErrorString(e));
    return IC_OK;
}

ic_status ic_debug_indexer_scores(const ic_indexer_desc *d, const void *q, const void *k, const float *w,
                                  int32_t row0, int32_t n_rows, float *out, void *stream)
{
    ic_status s = check_indexer(d);
    if (s != IC_OK) return s;
    if (!q || !k || !w || !out) return fail(IC_ERR_NULL, "q, k, w and out must not be NULL");
    if (row0 < 0 || n_rows <= 0 || (int64_t)row0 + n_rows > d->Tq)
        return fail(IC_ERR_SHAPE, "rows [%d, %d) outside [0, Tq=%d)", row0, row0 + n_rows, d->Tq);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = ic::launch_fill(out, (int64_t)d->B * n_rows * d->Lk, -INFINITY, st);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "fill launch failed: %s", hipGetErrorString(e));
    ic::ScoreArgs sa;
    memset(&sa, 0, sizeof sa);
    sa.q = q;
    sa.k = k;
    sa.w = w;
    sa.q_scale = d->q_scale;
    sa.k_scale = d->k_scale;
    sa.strip = out;
    sa.ld = d->Lk;
    sa.q_pos0 = d->q_pos0;
    sa.Tq = d->Tq;
    sa.Lk = d->Lk;
    sa.H_I = d->H_I;
    sa.b0 = 0;
    sa.i0 = row0;
    sa.Ri = n_rows;
    ProfScope ps(0, st);
    e = ic::launch_score(sa, d->dtype, d->d_I, d->B, st);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "indexer score launch failed: %s", hipGetErrorString(e));
    return IC_OK;
}

uint64_t ic_debug_indexer_launch_count(void) { return g_indexer_launches.load(); }

ic_status ic_calibrate(int32_t kind, const void *src, void *dst, const int32_t *idx, int64_t n, int64_t table_rows,
                       int32_t row_bytes, int32_t wgs, void *stream)
{
    if (kind < IC_CALIB_READ || kind > IC_CALIB_LDS_TR8_ROWS1) return fail(IC_ERR_SHAPE, "unknown calibration kind %d", kind);
    if (!dst) return fail(IC_ERR_NULL, "dst must not be NULL");
    if (wgs < 1 || wgs > (1 << 20)) return fail(IC_ERR_SHAPE, "wgs=%d outside [1, 2^20]", wgs);
    if (n < 0) return fail(IC_ERR_SHAPE, "n must not be negative");
    if (kind == IC_CALIB_READ || kind == IC_CALIB_COPY) {
        if (!src) return fail(IC_ERR_NULL, "src must not be NULL");
        if (n % 16 != 0) return fail(IC_ERR_SHAPE, "n=%lld bytes is not a multiple of 16", (long long)n);
    } else if (kind == IC_CALIB_GATHER) {
        if (!src || !idx) return fail(IC_ERR_NULL, "src and idx must not be NULL");
        if (table_rows < 1) return fail(IC_ERR_SHAPE, "table_rows must be positive");
        if (row_bytes != 1152 && row_bytes != 256) return fail(IC_ERR_UNSUPPORTED, "row_bytes=%d (1152 or 256)", row_bytes);
    } else if (kind >= IC_CALIB_LDS_READ16_PADDED) {
        if (n > INT32_MAX) return fail(IC_ERR_SHAPE, "too many rounds");
    } else if (kind >= IC_CALIB_TILE_GATHER) {
        if (!src || !idx) return fail(IC_ERR_NULL, "src and idx must not be NULL");
        if (table_rows < 1) return fail(IC_ERR_SHAPE, "table_rows must be positive");
        if (row_bytes != 1152) return fail(IC_ERR_UNSUPPORTED, "row_bytes=%d (1152)", row_bytes);
        if (n % 64 != 0) return fail(IC_ERR_SHAPE, "n=%lld rows is not a multiple of 64", (long long)n);
    } else if (n > INT32_MAX) {
        return fail(IC_ERR_SHAPE, "too many rounds");
    }
    hipError_t e = ic::launch_calib(kind, src, dst, idx, n, table_rows, row_bytes, wgs, (hipStream_t)stream);
    if (e != hipSuccess) return fail(IC_ERR_HIP, "calibration launch failed: %s", hipGetErrorString(e));
    return IC_OK;
}

void ic_prof_enable(int32_t on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = on != 0;
}

ic_status ic_prof_collect(void)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    ic_status rc = IC_OK;
    for (ProfRec &r : g_prof_recs) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r.e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.e0, r.e1);
        if (e == hipSuccess) {
            g_prof_n[r.which] += 1;
            g_prof_ms[r.which] += ms;
        } else {
            rc = fail(IC_ERR_HIP, "event timing failed: %s", hipGetErrorString(e));
        }
        (void)hipEventDestroy(r.e0);
        (void)hipEventDestroy(r.e1);
    }
    g_prof_recs.clear();
    return rc;
}

ic_status ic_prof_get(int32_t which, int64_t *launches, double *total_ms)
{
    if (which < 0 || which >= kProfClasses) return fail(IC_ERR_SHAPE, "kernel class %d outside [0,%d)", which, kProfClasses);
    if (!launches || !total_ms) return fail(IC_ERR_NULL, "output pointers must not be NULL");
    std::lock_guard<std::mutex> lk(g_prof_mu);
    *launches = g_prof_n[which];
    *total_ms = g_prof_ms[which];
    return IC_OK;
}

void ic_prof_reset(void)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (int i = 0; i < kProfClasses; ++i) {
        g_prof_n[i] = 0;
        g_prof_ms[i] = 0;
    }
}

} // extern "C"
