/*
 * indexcache.h -- C ABI of the MI355X (gfx950) IndexCache / DSA hot-path library.
 *
 * The library computes, on one GPU, the attention-side hot path of DeepSeek Sparse
 * Attention with IndexCache's cross-layer index reuse:
 *   (1) the causal lightning-indexer score  I[t,s] = sum_j w[t,j] * ReLU(q[t,j,:] . k[s,:])
 *       (the ReLU-gated, head-weighted dot-product indexer over the earlier tokens, paper Sec. 2.1;
 *       score vector I_t of Sec. 3 Notation),
 *   (2) the per-query index set T_t = Top-k(I_t) (Sec. 3 Notation),
 *   (3) sparse core attention over exactly the selected rows (Sec. 2.1, MLA/MQA form),
 *   (4) the inference loop of Fig. 2(b): Full layers run (1)+(2) and overwrite the cached
 *       index tensor, Shared layers reuse it (Sec. 3 Overview).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer unless the comment says "host".
 *     Descriptors, masks and pattern strings are host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued asynchronously on it; no call synchronises the device.
 *   - The caller owns every buffer, including the workspace; the library never allocates,
 *     frees or keeps device memory.  Inputs are read-only, outputs are fully overwritten.
 *   - Arguments are validated on the host before anything is launched; on error nothing has
 *     been enqueued, a status is returned and ic_last_error() describes it.  Nothing aborts.
 *   - Causality: key s of a sequence is visible to query row i iff s <= q_pos0 + i and
 *     s < Lk (inclusive causal mask).  Prefill: Tq = Lk, q_pos0 = 0.  Decode: Tq = 1,
 *     q_pos0 = Lk - 1 (the new token's key is already in the cache).
 */
#ifndef INDEXCACHE_H
#define INDEXCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ic_status {
    IC_OK = 0,
    IC_ERR_NULL = 1,        /* a required pointer is NULL */
    IC_ERR_SHAPE = 2,       /* a size is non-positive, inconsistent or overflows int32 indexing */
    IC_ERR_UNSUPPORTED = 3, /* dtype / head count / head dim / k_sel outside what the kernels cover */
    IC_ERR_WORKSPACE = 4,   /* workspace NULL, misaligned (256 B) or smaller than *_workspace() */
    IC_ERR_PATTERN = 5,     /* layer pattern invalid: the first layer must be Full (Sec. 3 Overview) */
    IC_ERR_HIP = 6          /* a HIP runtime call or kernel launch failed */
} ic_status;

typedef enum ic_dtype {
    IC_BF16 = 0,     /* bfloat16 q and k */
    IC_FP8_E4M3 = 1  /* OCP e4m3 q and k with one fp32 scale per token */
} ic_dtype;

#define IC_MAX_K 2048       /* largest supported k_sel */
#define IC_MAX_HEADS_I 64   /* largest supported number of indexer heads */
#define IC_MAX_HEADS_Q 32   /* largest supported number of attention query heads */

/* One indexer + top-k problem over B independent sequences. */
typedef struct ic_indexer_desc {
    int32_t B;        /* sequences */
    int32_t Tq;       /* query rows per sequence */
    int32_t Lk;       /* keys per sequence */
    int32_t H_I;      /* indexer heads, 1..IC_MAX_HEADS_I */
    int32_t d_I;      /* indexer head dim: 64 or 128 */
    int32_t k_sel;    /* k of Top-k, 1..IC_MAX_K */
    int64_t q_pos0;   /* absolute position of query row 0 */
    int32_t dtype;    /* ic_dtype of q and k */
    uint32_t flags;   /* reserved, must be 0 */
    const float *q_scale; /* [B,Tq] device, fp8 only (else NULL): q = q8 * q_scale */
    const float *k_scale; /* [B,Lk] device, fp8 only (else NULL): k = k8 * k_scale */
} ic_indexer_desc;

/* Bytes of workspace ic_indexer_topk needs for this problem (0 on an invalid descriptor).
 * The workspace holds a strip of score rows for the query rows in flight (never Tq x Lk for
 * long sequences); a larger workspace is accepted and lets more rows fly per launch. */
size_t ic_indexer_topk_workspace(const ic_indexer_desc *desc);

/*
 * Indexer score + per-query top-k (Sec. 2.1; Sec. 3 Notation: T_t = Top-k(I_t)).
 *   q   [B,Tq,H_I,d_I]  bf16 (or e4m3 bytes)     k [B,Lk,d_I] same type     w [B,Tq,H_I] fp32
 *   idx [B,Tq,k_sel] int32 out: the n = min(visible keys, k_sel) best positions of each query
 *       row in ASCENDING position order, the tail filled with -1.  Equal scores are
 *       resolved towards the lower position.
 *   sel_scores [B,Tq,k_sel] fp32 out, nullable: I[t, idx] aligned with idx (tail: -inf).
 */
ic_status ic_indexer_topk(const ic_indexer_desc *desc, const void *q, const void *k, const float *w,
                          int32_t *idx, float *sel_scores,
                          void *workspace, size_t workspace_bytes, void *stream);

/* One sparse-attention problem (MQA: all H_q heads share the single KV row of a position). */
typedef struct ic_attn_desc {
    int32_t B;          /* sequences */
    int32_t Tq;         /* query rows per sequence */
    int32_t Lk;         /* KV rows per sequence */
    int32_t H_q;        /* query heads, 1..IC_MAX_HEADS_Q */
    int32_t d_qk;       /* logits use KV[row, 0:d_qk]          (supported: 576 or 64) */
    int32_t d_v;        /* values are KV[row, v_off:v_off+d_v] (supported: 512 or 64) */
    int32_t v_off;      /* multiple of 8 */
    int32_t row_elems;  /* elements per KV row, >= max(d_qk, v_off + d_v), multiple of 8 */
    int32_t k_sel;      /* entries per query row in idx */
    float sm_scale;     /* logit scale (the paper leaves it to the model; 1/sqrt(d_qk) is usual) */
} ic_attn_desc;

size_t ic_sparse_attn_workspace(const ic_attn_desc *desc);

/*
 * Sparse core attention over the selected rows only (Sec. 2.1).
 *   Q  [B,Tq,H_q,d_qk] bf16     KV [B,Lk,row_elems] bf16     idx [B,Tq,k_sel] int32
 *   For each (b,t,h): z_m = sm_scale * <Q[b,t,h,:], KV[b,idx_m,0:d_qk]> over the entries with
 *   0 <= idx_m < Lk (others are skipped), p = softmax(z), O[b,t,h,:] = sum_m p_m KV[b,idx_m,v_off:+d_v].
 *   O   [B,Tq,H_q,d_v] bf16 out (a row with no valid entry gives zeros)
 *   lse [B,Tq,H_q] fp32 out, nullable: log sum_m exp(z_m) (-inf for an empty row)
 */
ic_status ic_sparse_attn(const ic_attn_desc *desc, const void *Q, const void *KV, const int32_t *idx,
                         void *O, float *lse, void *workspace, size_t workspace_bytes, void *stream);

/*
 * ic_sparse_attn for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same computation and the same kernels, with the
 * split-attention partials in a scratch array that is part of the library's code object instead of a
 * caller workspace.  Nothing is allocated or freed, by the library or any routine it calls.
 *   - The scratch holds IC_STATIC_SCRATCH_BYTES per GPU for the life of the process.  A descriptor
 *     whose ic_sparse_attn_workspace() exceeds it is rejected with IC_ERR_WORKSPACE before any launch.
 *   - The device the stream belongs to must be the current device of the calling thread.
 *   - Every call on one GPU shares that GPU's scratch: calls that overlap in time on one GPU (other
 *     streams, other threads) race.  Calls on one stream are ordered and safe.  The kernels overwrite
 *     every partial they later read, so nothing needs clearing between calls.
 * Arguments, results and error behaviour are otherwise those of ic_sparse_attn.
 */
#define IC_STATIC_SCRATCH_BYTES (16u << 20)
ic_status ic_sparse_attn_static(const ic_attn_desc *desc, const void *Q, const void *KV, const int32_t *idx,
                                void *O, float *lse, void *stream);

/* One attention layer of the stack: its indexer problem and its attention problem. */
typedef struct ic_layer {
    ic_indexer_desc ix;
    const void *q;      /* indexer inputs; may be NULL on Shared layers */
    const void *k;
    const float *w;
    ic_attn_desc at;
    const void *Q;      /* the layer's own attention inputs, used on Full and Shared layers alike */
    const void *KV;
    void *O;            /* [B,Tq,H_q,d_v] bf16 out */
} ic_layer;

/* Workspace for ic_forward_stack = the largest per-layer need (layers is host memory). */
size_t ic_forward_stack_workspace(const ic_layer *layers, int32_t n_layers);

/*
 * IndexCache inference loop (Fig. 2b; all-ones full_mask gives standard DSA, Fig. 2a).
 *   layers    host array of n_layers descriptors; every layer must agree on B, Tq and k_sel
 *   full_mask host array, 1 = Full (run the indexer, overwrite idx_cache), 0 = Shared (reuse
 *             idx_cache as the nearest preceding Full layer left it); full_mask[0] must be 1
 *   idx_cache [B,Tq,k_sel] int32 device, caller-owned: the paper's T_cache, the only index
 *             buffer of the pass; on return it holds the last Full layer's indices
 * Every layer then runs sparse attention on its own Q/KV with idx_cache.  At most two kernel
 * groups per layer are enqueued on `stream`, with no host synchronisation in between.
 */
ic_status ic_forward_stack(const ic_layer *layers, int32_t n_layers, const uint8_t *full_mask,
                           int32_t *idx_cache, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Decode against a full, paged KV cache with sequences of different lengths (the paper's third
 * serving measurement, Sec. 4.3: decode throughput with the KV cache filled).
 *
 * ic_paged_cache describes how every cache of the call (index keys and KV rows) is laid out:
 *   seq_lens    device [B] int32, nullable: the visible length Lk_b <= Lk of sequence b.  The Tq
 *               query rows of a sequence are then its LAST Tq positions (Tq = 1 in decode: the new
 *               token, whose own row is already in the cache), and q_pos0 of the descriptor is
 *               ignored.  NULL: every sequence has Lk positions and q_pos0 applies.
 *   page_table  device [B, max_pages] int32, nullable: physical page of logical page p of sequence
 *               b; logical position s lives in row page_table[b][s / page_size] * page_size +
 *               s % page_size of the POOL passed in place of k / KV ([n_pages * page_size, d_I] or
 *               [.., row_elems]).  NULL: dense [B, Lk, ..] layout.  Entries beyond a sequence's
 *               length are never read.
 *   page_size   positions per page, a power of two >= 64;  max_pages * page_size >= Lk
 * Lk in the descriptors is the bound on the lengths (it sizes launches and the workspace, which is
 * what the un-paged workspace queries return).  Index tensors hold LOGICAL positions.  A paged
 * index-key cache must be bf16.  One ic_paged_cache serves all layers of ic_forward_stack_paged
 * (each layer brings its own pools in layers[l].k and layers[l].KV).
 */
typedef struct {
    int32_t page_size;
    int32_t max_pages;
    const int32_t *page_table;
    const int32_t *seq_lens;
} ic_paged_cache;

ic_status ic_indexer_topk_paged(const ic_indexer_desc *d, const ic_paged_cache *pc, const void *q, const void *k_pool,
                                const float *w, int32_t *idx, float *sel_scores, void *workspace, size_t workspace_bytes,
                                void *stream);
ic_status ic_sparse_attn_paged(const ic_attn_desc *d, const ic_paged_cache *pc, const void *Q, const void *KV_pool,
                               const int32_t *idx, void *O, float *lse, void *workspace, size_t workspace_bytes, void *stream);
ic_status ic_forward_stack_paged(const ic_layer *layers, int32_t n_layers, const uint8_t *full_mask, const ic_paged_cache *pc,
                                 int32_t *idx_cache, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Forward of the indexer's distillation loss (paper Sec. 3.3), in the form of the sparse training
 * phase: both distributions live on the k selected positions of a query.
 *
 * ic_attn_probs: the attention distribution of a layer aggregated over its heads (the indexer's
 * training target, Sec. 2.1) on the rows named by idx,
 *     probs[b,t,m] = 1/H_q sum_h softmax_m(sm_scale * Q[b,t,h] . K[idx[b,t,m]])     (0 on empty slots)
 * K = the first d_qk features of a KV row.  lse [B,Tq,H_q] fp32: the log-sum-exps ic_sparse_attn
 * returns for the same Q, KV, idx (the per-head normalisers); probs [B,Tq,k_sel] fp32, out.
 * Dense caches only.  Asynchronous.
 *
 * ic_distill_loss: for one Full layer's indexer and the n_targets = m+1 layers it serves (itself and
 * its m Shared followers, all attending to the SAME index tensor):
 *     q_t = Softmax(sel_scores[t, :]) over the finite entries        (the indexer's distribution on T_t)
 *     loss_multi = sum_j 1/(m+1) sum_t KL(probs_j[t] || q_t)                               (Eq. 1)
 *     loss_avg   = sum_t KL(mean_j probs_j[t] || q_t)                                      (Eq. 2)
 *     grad[t,m]  = q_t[m] * |mean_j probs_j[t]| - mean_j probs_j[t][m]
 * grad is the derivative of EITHER loss with respect to the indexer's logits (Prop. 1: the two
 * losses differ by a term without q).  Reading of the sparse-phase restriction: both distributions
 * are renormalised over the selected set.
 *   probs       HOST array of n_targets DEVICE tensors [nq, k_sel] fp32 (ic_attn_probs of each layer)
 *   sel_scores  device [nq, k_sel] fp32 as ic_indexer_topk returns them (-inf on empty slots)
 *   loss_multi, loss_avg  device doubles, out, each nullable;  grad device [nq, k_sel] fp32, nullable
 *   workspace   ic_distill_loss_workspace(nq) bytes
 * 1 <= n_targets <= IC_MAX_DISTILL_TARGETS.  Asynchronous; the sums are taken in a fixed order.
 */
#define IC_MAX_DISTILL_TARGETS 16
ic_status ic_attn_probs(const ic_attn_desc *d, const void *Q, const void *KV, const int32_t *idx, const float *lse,
                        float *probs, void *stream);
size_t ic_distill_loss_workspace(int64_t nq);
ic_status ic_distill_loss(const float *const *probs, int32_t n_targets, const float *sel_scores, int64_t nq, int32_t k_sel,
                          double *loss_multi, double *loss_avg, float *grad, void *workspace, size_t workspace_bytes,
                          void *stream);

/* Host-only helpers for the pattern string c = c_1..c_N in {F,S}^N (Sec. 3 Overview). */
ic_status ic_pattern_from_string(const char *fs, uint8_t *full_mask, int32_t n);
/* Uniform interleave: F at layers l with l % r == 0, "FSSSFSSS.." for r = 4 (Sec. 3.1). */
ic_status ic_pattern_uniform(int32_t n, int32_t r, uint8_t *full_mask);

/*
 * Pairwise cross-layer overlap of the top-k index sets (paper App. A: |T(i) ^ T(j)| / k for every
 * pair of layers, averaged over the queries; the diagnostic behind the sharing idea).
 *   idx_layers  HOST array of n_layers DEVICE pointers, each an index tensor [nq, k_sel] int32 as
 *               ic_indexer_topk writes it (entries < 0 or >= Lk are not members; the members of one
 *               row are distinct; any order).  1 <= n_layers <= IC_MAX_OVERLAP_LAYERS.
 *   nq          rows per tensor (B*Tq); Lk: positions are in [0, Lk), Lk <= IC_MAX_OVERLAP_LK
 *   overlap     device [n_layers, n_layers] double, out (nullable):
 *                 overlap[i][j] = sum_t |T_t(i) ^ T_t(j)| / sum_t |T_t(i)|
 *               which is the appendix's ratio when every row holds k entries, and stays in [0,1]
 *               with 1 on the diagonal when early rows hold fewer; 0 for a layer with no members
 *   inter       device [n_layers, n_layers] uint64, out (nullable): the summed intersection sizes
 *   sizes       device [n_layers] uint64, out (nullable): the summed set sizes
 *   workspace   device, ic_topk_overlap_workspace(n_layers) bytes, 256-byte aligned; the library
 *               zeroes it itself
 * Errors (host, before any launch): IC_ERR_NULL, IC_ERR_SHAPE, IC_ERR_UNSUPPORTED (limits),
 * IC_ERR_WORKSPACE.  Asynchronous on `stream`.
 */
/*
 * Similarity-based pattern search (paper App. C).
 *
 * ic_cosine_rows: mean over the rows of the cosine similarity of corresponding rows of two bf16
 * device tensors [n_rows, row_len] (a row = one query token's attention output over all heads).
 * Reading where the paper is silent: the cosine is taken per token and averaged; two all-zero rows
 * count as 1, a zero row against a non-zero one as 0.  mean: device double, out; per_row: device
 * [n_rows] float, out, nullable; workspace: ic_cosine_rows_workspace() bytes, 256-byte aligned.
 *
 * ic_similarity_matrix: S[i][j], j < i = that similarity between layer i's sparse attention under
 * its OWN index tensor (written to layers[i].O) and under layer j's index tensor (as if layer i
 * were a Shared layer reading layer j); S[i][i] = 1, S[i][j] = 0 for j > i.  layers: the
 * attention part (at, Q, KV, O) of n_layers layers of one shape; idx_layers: HOST array of
 * n_layers DEVICE index tensors [B,Tq,k_sel]; S: device [n_layers, n_layers] double, out;
 * workspace: ic_similarity_matrix_workspace(layers, n_layers) bytes.  n_layers (n_layers-1) / 2 + n_layers
 * attention launches on `stream`.
 *
 * ic_pattern_search_dp (host only): the pattern with exactly n_full Full layers (the first layer
 * Full) that maximises the sum over the Shared layers l of S[l][src(l)], src(l) the nearest
 * preceding Full layer -- exact dynamic program over (last Full layer, number of Full layers so
 * far).  S: HOST [n_layers, n_layers] double, only j < i is read; full_mask: out; total: out,
 * nullable.  Among equal optima the pattern found is unspecified.
 */
size_t ic_cosine_rows_workspace(void);
ic_status ic_cosine_rows(const void *A, const void *B, int64_t n_rows, int64_t row_len, double *mean, float *per_row,
                         void *workspace, size_t workspace_bytes, void *stream);
size_t ic_similarity_matrix_workspace(const ic_layer *layers, int32_t n_layers);
ic_status ic_similarity_matrix(const ic_layer *layers, int32_t n_layers, const int32_t *const *idx_layers, double *S,
                               void *workspace, size_t workspace_bytes, void *stream);
ic_status ic_pattern_search_dp(const double *S, int32_t n_layers, int32_t n_full, uint8_t *full_mask, double *total);

/*
 * Greedy layer selection (paper Alg. 1, Sec. 3.2) with a surrogate loss.
 *
 * The algorithm starts from all-Full and, n_shared times, flips to Shared the candidate layer whose
 * flip gives the lowest EvalLoss (ties: the lowest layer); layer 0 is never a candidate.  n_blocks
 * > 1 is the pipeline-parallel variant of the same section: contiguous blocks of
 * ceil(n_layers / n_blocks) layers, a block's first layer stays Full, and within one step the
 * blocks are searched in order, each committing its own best flip before the next is searched.
 *
 * EvalLoss in the paper is the language-model loss on calibration batches, which needs the model.
 * Its stand-in here is the attention-output error of a pattern against the all-Full stack:
 *     loss(c) = 1/N sum_l (1 - sim_l(c)),
 *     sim_l(c) = mean per-token cosine (as ic_cosine_rows) of layer l's output under c and under F^N
 *
 * ic_pattern_loss: that loss for one pattern, measured the way Alg. 1 measures it: the whole stack
 * is run under full_mask (ic_forward_stack: outputs land in layers[l].O, idx_cache is overwritten)
 * and every layer's output is compared with O_ref[l], the output of the all-Full run.  O_ref: HOST
 * array of n_layers DEVICE tensors [B,Tq,H_q,d_v] bf16, none of them a layer's own O; loss: device
 * double, out.  Layers of one attention shape, n_layers <= IC_MAX_OVERLAP_LAYERS.  Asynchronous.
 *
 * ic_greedy_search_forward: Alg. 1 driven by ic_pattern_loss, one forward pass of the stack per
 * candidate (n_layers (n_layers - 1) / 2 passes for a full search with one block).  The host has to
 * read the candidates' losses to choose, so this call SYNCHRONISES `stream` once per search step.
 *
 * ic_pattern_search_greedy (host only): the same search on a similarity matrix S as
 * ic_similarity_matrix produces it (HOST [n_layers, n_layers] double, j < i read), with
 * sim_l(c) = S[l][src(l)], which is what the forward passes measure when a layer's inputs do not
 * depend on earlier layers' outputs (the attention-only stack).
 *
 * Outputs (host): full_mask [n_layers]; order [n_shared], nullable: the flipped layers in commit
 * order; loss_curve [n_shared], nullable: the loss after each commit.
 * Errors: IC_ERR_NULL, IC_ERR_SHAPE (n_shared > candidates, bad block count, layer shapes),
 * IC_ERR_PATTERN never (the search keeps layer 0 Full), IC_ERR_WORKSPACE, IC_ERR_HIP.
 */
ic_status ic_pattern_search_greedy(const double *S, int32_t n_layers, int32_t n_shared, int32_t n_blocks,
                                   uint8_t *full_mask, int32_t *order, double *loss_curve);
size_t ic_pattern_loss_workspace(const ic_layer *layers, int32_t n_layers);
ic_status ic_pattern_loss(const ic_layer *layers, int32_t n_layers, const uint8_t *full_mask, const void *const *O_ref,
                          int32_t *idx_cache, double *loss, void *workspace, size_t workspace_bytes, void *stream);
size_t ic_greedy_search_forward_workspace(const ic_layer *layers, int32_t n_layers);
ic_status ic_greedy_search_forward(const ic_layer *layers, int32_t n_layers, int32_t n_shared, int32_t n_blocks,
                                   const void *const *O_ref, int32_t *idx_cache, uint8_t *full_mask, int32_t *order,
                                   double *loss_curve, void *workspace, size_t workspace_bytes, void *stream);

#define IC_MAX_OVERLAP_LAYERS 128
#define IC_MAX_OVERLAP_LK (1 << 20)
size_t ic_topk_overlap_workspace(int32_t n_layers);
ic_status ic_topk_overlap(const int32_t *const *idx_layers, int32_t n_layers, int64_t nq, int32_t k_sel, int32_t Lk,
                          double *overlap, uint64_t *inter, uint64_t *sizes, void *workspace, size_t workspace_bytes,
                          void *stream);

/* Message for the last error on the calling thread ("" if none). Host string, do not free. */
const char *ic_last_error(void);

/*
 * Parity aid: the raw indexer scores of query rows [row0, row0+n_rows) of every sequence,
 * computed by the same scoring kernel the top-k path uses.
 *   out [B,n_rows,Lk] fp32 device; keys hidden by the causal mask are -inf.
 */
ic_status ic_debug_indexer_scores(const ic_indexer_desc *desc, const void *q, const void *k,
                                  const float *w, int32_t row0, int32_t n_rows, float *out,
                                  void *stream);

/* Number of ic_indexer_topk problems launched by this process so far (for the
 * "indexer runs exactly on the Full layers" invariant). */
uint64_t ic_debug_indexer_launch_count(void);

/*
 * Calibration (a measurement aid for the roofline figures of Sec. 4.3-style throughput reports, not part of
 * the method): what the chip sustains on the patterns the hot path is made of, launched on `stream` through
 * this library so that a benchmark can time them beside the real kernels.
 *   IC_CALIB_READ       read n bytes from src (n a multiple of 16); dst: >= 4 * wgs bytes, rarely written
 *   IC_CALIB_COPY       copy n bytes from src to dst
 *   IC_CALIB_GATHER     read n rows of row_bytes (1152 or 256) from the table src [table_rows, row_bytes],
 *                       row numbers in idx [n] int32 (device; values outside the table are clamped), eight
 *                       lanes per 128-byte line as the attention kernels do; dst as for READ
 *   IC_CALIB_MFMA_BF16  n back-to-back rounds of four v_mfma_f32_32x32x16_bf16 per wave (4 waves per
 *   IC_CALIB_MFMA_FP8   workgroup), or of four 32x32x64 e4m3 instructions; dst: >= 1024 * wgs bytes
 *   IC_CALIB_TILE_*     the data movement of the prefill sparse-attention tile loop without its arithmetic, over
 *                       n rows (a multiple of 64; tiles of 64 rows) of 1152 bytes named by idx as for GATHER, one
 *                       workgroup per CU, row numbers fetched a tile ahead of the rows: _GATHER rows into
 *                       registers, one tile ahead; _STORE also stores each tile to LDS; _READ also reads it back
 *                       once in 16-byte pieces; _READ2 also reads the first 1024 bytes of every row a second time
 *                       through the transposing LDS read (the reads of a phase are all in flight together);
 *                       _8WAVES moves exactly the bytes of _READ2 with eight waves per workgroup instead of four
 *                       (wgs then counts workgroups of 512 threads); _INTERLEAVED moves them with four waves and
 *                       the stores and gathers spread between the reads instead of in a phase of their own
 *   IC_CALIB_LDS_*      n rounds of 16 LDS reads per wave in one access pattern of the attention tile, no global memory
 *                       (src, idx unused; wgs counts workgroups of 1024 threads; dst as for READ): _READ16_PADDED the
 *                       16-byte score-operand read of 16 rows 1184 bytes apart, _READ16_SWIZZLED the same with rows 1152
 *                       bytes apart and XOR-swizzled slots, _TR8_ROWS2 / _TR8_ROWS1 the 8-byte transposing read over
 *                       four rows two apart / four consecutive rows (rows 1184 apart)
 * wgs = workgroups of 256 threads to launch (1 .. 2^20).  All pointers are device pointers owned by the
 * caller; nothing is allocated.  Errors: IC_ERR_NULL, IC_ERR_SHAPE, IC_ERR_UNSUPPORTED (row_bytes), IC_ERR_HIP.
 */
enum { IC_CALIB_READ = 0, IC_CALIB_COPY = 1, IC_CALIB_GATHER = 2, IC_CALIB_MFMA_BF16 = 3, IC_CALIB_MFMA_FP8 = 4,
       IC_CALIB_TILE_GATHER = 5, IC_CALIB_TILE_STORE = 6, IC_CALIB_TILE_READ = 7, IC_CALIB_TILE_READ2 = 8,
       IC_CALIB_TILE_8WAVES = 9, IC_CALIB_TILE_INTERLEAVED = 10,
       IC_CALIB_LDS_READ16_PADDED = 11, IC_CALIB_LDS_READ16_SWIZZLED = 12, IC_CALIB_LDS_TR8_ROWS2 = 13, IC_CALIB_LDS_TR8_ROWS1 = 14 };
ic_status ic_calibrate(int32_t kind, const void *src, void *dst, const int32_t *idx, int64_t n, int64_t table_rows,
                       int32_t row_bytes, int32_t wgs, void *stream);

/*
 * Per-kernel timing with HIP events recorded on the launch stream (a measuring aid; off by
 * default).  ic_prof_enable(1) starts recording an event pair around every kernel launch
 * (bounded pool of 8192 pairs; launches beyond it are not recorded), ic_prof_enable(0) stops.
 * ic_prof_collect waits for the recorded events (host-blocking) and adds their durations to
 * per-class totals; ic_prof_get reads the totals of kernel class `which`
 * (0 = indexer score, 1 = top-k select, 2 = sparse attention, 3 = attention split merge):
 * number of launches and summed duration in milliseconds; ic_prof_reset zeroes the totals.
 */
void ic_prof_enable(int32_t on);
ic_status ic_prof_collect(void);
ic_status ic_prof_get(int32_t which, int64_t *launches, double *total_ms);
void ic_prof_reset(void);

#ifdef __cplusplus
}
#endif
#endif /* INDEXCACHE_H */
