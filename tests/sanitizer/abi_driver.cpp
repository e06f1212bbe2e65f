// Host side of the C ABI under AddressSanitizer / UndefinedBehaviorSanitizer: every call below is refused by
// the argument validation (or is host-only arithmetic), so no kernel is launched and no GPU is needed.
// Built by tests/test_sanitizers_cpu.py with the sanitizers applied to the host pass only.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "criticalkv.h"

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

static ckv_layer_desc good()
{
    ckv_layer_desc d;
    memset(&d, 0, sizeof d);
    d.batch = 1; d.n_q_heads = 8; d.n_kv_heads = 2; d.head_dim = 128; d.d_model = 256; d.n_ctx = 1000; d.window = 16;
    d.pool_kernel = 7; d.dtype = CKV_BF16; d.norm = CKV_NORM_L1; d.window_reduce = CKV_MEAN; d.eps = 1e-4f;
    return d;
}

int main()
{
    alignas(256) static char buf[1024];
    void *p = buf;
    ckv_layer_desc d = good();
    const size_t need = criticalkv_workspace_bytes(&d, 100);
    CHECK(need > 0 && need % 256 == 0);
    CHECK(criticalkv_workspace_bytes(nullptr, 1) == 0);
    CHECK(criticalkv_workspace_bytes(&d, -1) == 0);
    CHECK(criticalkv_workspace_bytes(&d, 1000) > need);
    // descriptors that must be refused
    struct { int field; int value; int code; } bad[] = {
        {0, 0, CKV_E_INVALID_ARG}, {1, 7, CKV_E_INVALID_ARG}, {2, 0, CKV_E_INVALID_ARG}, {3, 2000, CKV_E_INVALID_ARG},
        {4, 4, CKV_E_INVALID_ARG}, {5, 5, CKV_E_INVALID_ARG}, {6, 96, CKV_E_UNSUPPORTED}, {7, 100, CKV_E_UNSUPPORTED},
        {8, 3, CKV_E_INVALID_ARG}, {9, 64, CKV_E_INVALID_ARG}, {10, 65, CKV_E_UNSUPPORTED}};
    for (auto &c : bad) {
        ckv_layer_desc x = good();
        switch (c.field) {
        case 0: x.batch = c.value; break;
        case 1: x.n_q_heads = c.value; break;
        case 2: x.window = c.value; break;
        case 3: x.window = c.value; break;
        case 4: x.pool_kernel = c.value; break;
        case 5: x.dtype = c.value; break;
        case 6: x.head_dim = c.value; break;
        case 7: x.d_model = c.value; break;
        case 8: x.norm = c.value; break;
        case 9: x.flags = (uint32_t)c.value; break;
        case 10: x.pool_kernel = c.value; break;
        }
        CHECK(criticalkv_score(&x, p, p, p, p, (float *)p, (float *)p, nullptr, p, (size_t)1 << 40, nullptr) == c.code);
        CHECK(criticalkv_compact(&x, p, p, (const int32_t *)p, (const int32_t *)p, 10, p, p, nullptr) == c.code);
        CHECK(criticalkv_workspace_bytes(&x, 10) == 0);
        CHECK(criticalkv_gram_bytes(&x) == 0);
        CHECK(criticalkv_prepared_wo_bytes(&x) == 0);
    }
    ckv_layer_desc s = good();
    s.softmax_scale = -1.0f;
    CHECK(criticalkv_score(&s, p, p, p, p, (float *)p, (float *)p, nullptr, p, need, nullptr) == CKV_E_INVALID_ARG);
    s = good();
    s.eps = NAN;
    CHECK(criticalkv_score(&s, p, p, p, p, (float *)p, (float *)p, nullptr, p, need, nullptr) == CKV_E_INVALID_ARG);
    s = good();
    s.k_stride[0] = 128000; s.k_stride[1] = 64000; s.k_stride[2] = 100;       // token stride below head_dim
    CHECK(criticalkv_score(&s, p, p, p, p, (float *)p, (float *)p, nullptr, p, need, nullptr) == CKV_E_INVALID_ARG);
    // pointers, alignment, workspace
    CHECK(criticalkv_score(&d, nullptr, p, p, p, (float *)p, (float *)p, nullptr, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_score(&d, p, buf + 8, p, p, (float *)p, (float *)p, nullptr, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_score(&d, p, p, p, p, (float *)p, (float *)p, nullptr, nullptr, need, nullptr) == CKV_E_WORKSPACE);
    CHECK(criticalkv_score(&d, p, p, p, p, (float *)p, (float *)p, nullptr, buf + 8, need, nullptr) == CKV_E_WORKSPACE);
    CHECK(criticalkv_score(&d, p, p, p, p, (float *)p, (float *)p, nullptr, p, 4096, nullptr) == CKV_E_WORKSPACE);
    const float *f = (const float *)p;
    const int32_t *i = (const int32_t *)p;
    int32_t *o = (int32_t *)p;
    CHECK(criticalkv_select(&d, f, f, i, 1.5f, 100, o, o, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_select(&d, f, f, i, NAN, 100, o, o, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_select(&d, f, f, i, 0.5f, 0, o, o, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_select(&d, f, f, i, 0.5f, 1001, o, o, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_select(&d, f, f, nullptr, 0.5f, 100, o, o, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_select(&d, f, f, i, 0.5f, 100, o, o, p, 16, nullptr) == CKV_E_WORKSPACE);
    CHECK(criticalkv_select_noalloc(&d, f, f, i, 1.5f, 100, o, o, nullptr) == CKV_E_INVALID_ARG);
    ckv_layer_desc big = good();
    big.n_q_heads = big.n_kv_heads = 8; big.n_ctx = 1 << 20;
    CHECK(criticalkv_select_noalloc(&big, f, f, i, 0.5f, 100, o, o, nullptr) == CKV_E_STATIC_LIMIT);
    CHECK(criticalkv_allocate(&d, f, -1, 0.5f, o, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_allocate(&d, f, 100, 1.5f, o, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_allocate(&d, f, d.n_kv_heads * d.n_ctx + 1, 0.5f, o, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_allocate(&d, f, d.n_kv_heads * 1000, 0.0f, o, p, 4096, nullptr) == CKV_E_WORKSPACE);
    CHECK(criticalkv_diagnostics(&d, p, nullptr, nullptr, i, i, 100, (float *)p, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_diagnostics(&d, p, p, nullptr, i, i, 1001, (float *)p, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_diagnostics(&d, p, p, nullptr, i, i, 100, (float *)p, p, 4096, nullptr) == CKV_E_WORKSPACE);
    CHECK(criticalkv_compact(&d, p, p, i, nullptr, 10, p, p, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_compact(&d, p, p, i, i, 0, p, p, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_prepare_wo(&d, p, p, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_probe_mfma_bf16(nullptr, 10, nullptr, (float *)p, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_probe_mfma_bf16(buf + 8, 10, nullptr, (float *)p, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_probe_mfma_bf16(p, 0, nullptr, (float *)p, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_probe_hbm_read(p, 8, (uint32_t *)p, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_probe_hbm_read(nullptr, 4096, (uint32_t *)p, nullptr) == CKV_E_INVALID_ARG);
    ckv_layer_desc g = good();
    g.d_model = 512; g.norm = CKV_NORM_L2;
    CHECK(criticalkv_gram_bytes(&g) == (size_t)8 * 2 * 128 * 128 * 2);
    CHECK(criticalkv_prepare_gram(&g, nullptr, p, p, need, nullptr) == CKV_E_INVALID_ARG);
    CHECK(criticalkv_prepare_gram(&g, p, buf + 256, p, 64, nullptr) == CKV_E_WORKSPACE);
    for (int code = -7; code <= 0; ++code) CHECK(strlen(criticalkv_strerror(code)) > 3);
    puts("C ABI sanitizer run: OK");
    return 0;
}
