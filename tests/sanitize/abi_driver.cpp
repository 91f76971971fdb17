// Walks the C ABI's host-side paths (argument validation, workspace planning, pattern helpers, the dynamic
// program and the greedy search over a similarity matrix) in a build whose HOST code carries
// -fsanitize=address,undefined.  No GPU is needed: every device entry point is called with arguments that
// are rejected before any launch.  Test infrastructure (tests/test_sanitizers.py builds and runs it);
// prints "abi sanitizer run ok".
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "indexcache.h"

#define CHECK(x) do { if (!(x)) { std::fprintf(stderr, "check failed line %d: %s (%s)\n", __LINE__, #x, ic_last_error()); return 1; } } while (0)

int main()
{
    void *one = (void *)4096;
    ic_indexer_desc ix;
    std::memset(&ix, 0, sizeof ix);
    ix.B = 1; ix.Tq = 128; ix.Lk = 128; ix.H_I = 32; ix.d_I = 128; ix.k_sel = 256; ix.dtype = IC_BF16;
    ic_attn_desc at;
    std::memset(&at, 0, sizeof at);
    at.B = 1; at.Tq = 128; at.Lk = 128; at.H_q = 32; at.d_qk = 576; at.d_v = 512; at.row_elems = 576; at.k_sel = 256; at.sm_scale = 0.04f;

    CHECK(ic_indexer_topk_workspace(&ix) > 0 && ic_indexer_topk_workspace(nullptr) == 0);
    CHECK(ic_indexer_topk(&ix, nullptr, one, (const float *)one, (int32_t *)one, nullptr, one, 1u << 30, nullptr) == IC_ERR_NULL);
    CHECK(ic_indexer_topk(&ix, one, one, (const float *)one, (int32_t *)one, nullptr, nullptr, 0, nullptr) == IC_ERR_WORKSPACE);
    CHECK(ic_indexer_topk(&ix, one, one, (const float *)one, (int32_t *)one, nullptr, (void *)4097, 1u << 30, nullptr) == IC_ERR_WORKSPACE);
    ic_indexer_desc bad = ix;
    bad.k_sel = IC_MAX_K + 1;
    CHECK(ic_indexer_topk(&bad, one, one, (const float *)one, (int32_t *)one, nullptr, one, 1u << 30, nullptr) == IC_ERR_UNSUPPORTED);
    bad = ix; bad.d_I = 96;
    CHECK(ic_indexer_topk(&bad, one, one, (const float *)one, (int32_t *)one, nullptr, one, 1u << 30, nullptr) == IC_ERR_UNSUPPORTED);
    bad = ix; bad.dtype = IC_FP8_E4M3;
    CHECK(ic_indexer_topk(&bad, one, one, (const float *)one, (int32_t *)one, nullptr, one, 1u << 30, nullptr) == IC_ERR_NULL);
    CHECK(ic_debug_indexer_scores(&ix, one, one, (const float *)one, 100, 100, (float *)one, nullptr) == IC_ERR_SHAPE);

    CHECK(ic_sparse_attn_workspace(&at) > 0);
    CHECK(ic_sparse_attn(&at, one, one, (const int32_t *)one, one, nullptr, nullptr, 0, nullptr) == IC_ERR_WORKSPACE);
    CHECK(ic_sparse_attn(&at, one, nullptr, (const int32_t *)one, one, nullptr, one, 1u << 30, nullptr) == IC_ERR_NULL);
    ic_attn_desc bat = at;
    bat.H_q = 33;
    CHECK(ic_sparse_attn(&bat, one, one, (const int32_t *)one, one, nullptr, one, 1u << 30, nullptr) == IC_ERR_UNSUPPORTED);
    bat = at; bat.B = 255; bat.Tq = 1; bat.Lk = 65536; bat.k_sel = 2048;
    CHECK(ic_sparse_attn_static(&bat, one, one, (const int32_t *)one, one, nullptr, nullptr) == IC_ERR_WORKSPACE);

    ic_paged_cache pc;
    std::memset(&pc, 0, sizeof pc);
    CHECK(ic_sparse_attn_paged(&at, &pc, one, one, (const int32_t *)one, one, nullptr, one, 1u << 30, nullptr) == IC_ERR_NULL);
    pc.page_table = (const int32_t *)one; pc.page_size = 48; pc.max_pages = 4;
    CHECK(ic_indexer_topk_paged(&ix, &pc, one, one, (const float *)one, (int32_t *)one, nullptr, one, 1u << 30, nullptr) == IC_ERR_SHAPE);
    pc.page_size = 64; pc.max_pages = 1;
    CHECK(ic_sparse_attn_paged(&at, &pc, one, one, (const int32_t *)one, one, nullptr, one, 1u << 30, nullptr) == IC_ERR_SHAPE);

    std::vector<ic_layer> layers(3);
    for (auto &L : layers) {
        std::memset(&L, 0, sizeof L);
        L.ix = ix; L.at = at;
        L.q = L.k = L.Q = L.KV = one; L.w = (const float *)one; L.O = one;
    }
    const size_t ws = ic_forward_stack_workspace(layers.data(), 3);
    CHECK(ws > 0);
    uint8_t mask[3] = {0, 1, 0};
    CHECK(ic_forward_stack(layers.data(), 3, mask, (int32_t *)one, one, ws, nullptr) == IC_ERR_PATTERN);
    mask[0] = 1;
    CHECK(ic_forward_stack(layers.data(), 3, mask, (int32_t *)one, one, 16, nullptr) == IC_ERR_WORKSPACE);
    layers[2].at.Lk = 64;
    CHECK(ic_forward_stack(layers.data(), 3, mask, (int32_t *)one, one, ws, nullptr) == IC_ERR_SHAPE);
    layers[2].at.Lk = 128;
    layers[1].ix.Lk = 256;
    CHECK(ic_forward_stack(layers.data(), 3, mask, (int32_t *)one, one, ws, nullptr) == IC_ERR_SHAPE);
    CHECK(ic_forward_stack_paged(layers.data(), 3, mask, nullptr, (int32_t *)one, one, ws, nullptr) == IC_ERR_NULL);

    uint8_t m47[47];
    CHECK(ic_pattern_uniform(47, 4, m47) == IC_OK && m47[0] == 1 && m47[1] == 0 && m47[44] == 1);
    CHECK(ic_pattern_from_string("FSSF", m47, 4) == IC_OK && m47[3] == 1);
    CHECK(ic_pattern_from_string("SFSF", m47, 4) == IC_ERR_PATTERN);
    CHECK(ic_pattern_from_string("FSxF", m47, 4) == IC_ERR_PATTERN);
    CHECK(ic_pattern_from_string("FS", m47, 4) == IC_ERR_SHAPE);

    const int N = 9;
    std::vector<double> S(N * N, 0.0);
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < i; ++j) S[i * N + j] = 1.0 / (1 + i - j);
    uint8_t fm[N];
    double total = 0;
    for (int m = 1; m <= N; ++m) CHECK(ic_pattern_search_dp(S.data(), N, m, fm, &total) == IC_OK && fm[0] == 1);
    CHECK(ic_pattern_search_dp(S.data(), N, N + 1, fm, &total) == IC_ERR_SHAPE);
    int32_t order[N];
    double curve[N];
    CHECK(ic_pattern_search_greedy(S.data(), N, 5, 1, fm, order, curve) == IC_OK);
    CHECK(ic_pattern_search_greedy(S.data(), N, 4, 3, fm, order, curve) == IC_OK);
    CHECK(ic_pattern_search_greedy(S.data(), N, N, 1, fm, order, curve) == IC_ERR_SHAPE);

    const void *ptrs[3] = {one, nullptr, one};
    CHECK(ic_topk_overlap((const int32_t *const *)ptrs, 3, 10, 8, 100, (double *)one, nullptr, nullptr, one, ic_topk_overlap_workspace(3), nullptr) == IC_ERR_NULL);
    CHECK(ic_cosine_rows(one, one, 0, 8, (double *)one, nullptr, one, 256, nullptr) == IC_ERR_SHAPE);
    CHECK(ic_calibrate(IC_CALIB_GATHER, one, one, (const int32_t *)one, 8, 8, 100, 1, nullptr) == IC_ERR_UNSUPPORTED);
    CHECK(ic_calibrate(99, one, one, nullptr, 8, 8, 100, 1, nullptr) == IC_ERR_SHAPE);
    int64_t n = 0;
    double ms = 0;
    CHECK(ic_prof_get(9, &n, &ms) == IC_ERR_SHAPE);
    ic_prof_reset();
    CHECK(ic_prof_get(0, &n, &ms) == IC_OK && n == 0);
    std::puts("abi sanitizer run ok");
    return 0;
}
