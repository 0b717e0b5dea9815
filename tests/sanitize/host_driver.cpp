// Drives the host side of libvsprefill (argument validation, workspace layouts, error strings) with the library's own
// sources compiled under AddressSanitizer and UndefinedBehaviorSanitizer for the host pass.  Every call below is refused
// before anything is launched, so no GPU is needed: what runs is exactly the code that sits between the C ABI and the
// first kernel launch.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "vsprefill.h"

#define EXPECT(call, want) do { const long long got_ = static_cast<long long>(call); if (got_ != static_cast<long long>(want)) { \
    std::fprintf(stderr, "line %d: %s returned %lld, expected %lld\n", __LINE__, #call, got_, static_cast<long long>(want)); return 1; } } while (0)

int main() {
    alignas(16) static unsigned char buf[4096];
    void* p = buf;                      // a 16-byte aligned non-null pointer; never dereferenced by a refused call
    void* odd = buf + 2;                // misaligned
    int32_t* ip = reinterpret_cast<int32_t*>(buf);
    float* fp = reinterpret_cast<float*>(buf);

    // sizes and layouts
    EXPECT(vs_sparse_prefill_workspace(32, 8, 8, 0), 0);
    EXPECT(vs_sparse_prefill_workspace(32, 8, 5, 1024), 0);
    EXPECT(vs_sparse_prefill_workspace(32, 8, 8, (1ll << 20) + 1), 0);
    if (vs_sparse_prefill_workspace(32, 8, 8, 131072) == 0 || vs_sparse_prefill_workspace(1, 1, 1, 1) == 0) return 2;
    if (vs_sparse_prefill_workspace(32, 8, 8, 1 << 20) <= vs_sparse_prefill_workspace(32, 8, 8, 131072)) return 3;
    EXPECT(vs_index_score_workspace(8, 1024, 100), 0);
    if (vs_index_score_workspace(8, 131072, 256) == 0 || vs_aggregate_workspace(32, 8, 8, 4096) == 0) return 4;
    EXPECT(vs_aggregate_workspace(32, 8, 8, 0), 0);
    (void)vs_select_budget_workspace(8, 131072);
    if (vs_index_train_workspace(8, 4096, 256) == 0) return 7;
    EXPECT(vs_index_train_workspace(8, 4096, 100), 0);

    // attention calls
    EXPECT(vs_sparse_prefill(nullptr, p, p, 4, 1, 64, 0.1f, ip, ip, 4, ip, ip, 4, 1, p, nullptr, p, 4096, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_sparse_prefill(odd, p, p, 4, 1, 64, 0.1f, ip, ip, 4, ip, ip, 4, 1, p, nullptr, p, 4096, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_sparse_prefill(p, p, p, 3, 2, 64, 0.1f, ip, ip, 4, ip, ip, 4, 2, p, nullptr, p, 4096, nullptr), VS_ERR_UNSUPPORTED);
    EXPECT(vs_sparse_prefill(p, p, p, 4, 1, 64, -1.f, ip, ip, 4, ip, ip, 4, 1, p, nullptr, p, 4096, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_sparse_prefill(p, p, p, 4, 1, 64, 0.1f, ip, ip, 0, ip, ip, 4, 1, p, nullptr, p, 4096, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_sparse_prefill(p, p, p, 4, 1, 64, 0.1f, ip, ip, 4, ip, ip, 4, 3, p, nullptr, p, 4096, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_sparse_prefill(p, p, p, 4, 1, 64, 0.1f, ip, ip, 4, ip, ip, 4, 1, p, nullptr, p, 16, nullptr), VS_ERR_WORKSPACE);
    EXPECT(vs_sparse_prefill(p, p, p, 4, 1, 64, 0.1f, ip, ip, 4, ip, ip, 4, 1, p, nullptr, nullptr, 0, nullptr), VS_ERR_WORKSPACE);
    EXPECT(vs_sparse_prefill_tiled(p, p, p, 4, 1, 64, 0.1f, ip, ip, 4, ip, ip, 4, 1, 16, p, nullptr, p, 4096, nullptr), VS_ERR_UNSUPPORTED);
    EXPECT(vs_sparse_prefill_static(p, p, p, 32, 32, 1 << 20, 0.1f, ip, ip, 4, ip, ip, 4, 32, p, nullptr, nullptr), VS_ERR_STATIC_LIMIT);
    EXPECT(vs_sparse_prefill_chunk(p, p, p, 4, 1, 32, 64, 40, 0.1f, ip, ip, 4, ip, ip, 4, 1, 1, p, nullptr, p, 4096, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_sparse_prefill_chunk(p, p, p, 4, 1, 32, 64, 5, 0.1f, ip, ip, 4, ip, ip, 4, 1, 32, p, nullptr, p, 4096, nullptr), VS_ERR_UNSUPPORTED);
    EXPECT(vs_dense_prefill(p, p, nullptr, 4, 1, 64, 0.1f, p, nullptr, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_dense_prefill(p, p, p, 4, 1, (1ll << 20) + 1, 0.1f, p, nullptr, nullptr), VS_ERR_UNSUPPORTED);
    EXPECT(vs_dense_prefill_chunk(p, p, p, 4, 1, 32, 64, 33, 0.1f, p, nullptr, nullptr), VS_ERR_INVALID_ARG);
    int64_t tiles = 0;
    EXPECT(vs_sparse_prefill_tiles(nullptr, 0, nullptr, &tiles), VS_ERR_INVALID_ARG);
    EXPECT(vs_validate_lists(nullptr, ip, 4, 1, 64, ip, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_validate_lists(ip, ip, 0, 1, 64, ip, nullptr), VS_ERR_INVALID_ARG);

    // indexer, selection, aggregation, rope
    vs_indexer_t w;
    std::memset(&w, 0, sizeof w);
    EXPECT(vs_index_score(p, p, 2, 64, &w, fp, fp, p, 4096, nullptr), VS_ERR_INVALID_ARG);
    w.W_U = w.b_U = w.W_V = w.W_S = fp;
    w.d_h = 100;
    w.act = 1;
    EXPECT(vs_index_score(p, p, 2, 64, &w, fp, fp, p, 4096, nullptr), VS_ERR_UNSUPPORTED);
    w.d_h = 256;
    w.act = 7;
    EXPECT(vs_index_score(p, p, 2, 64, &w, fp, fp, p, 4096, nullptr), VS_ERR_INVALID_ARG);
    w.act = 0;
    EXPECT(vs_index_score(p, p, 2, 64, &w, fp, fp, p, 16, nullptr), VS_ERR_WORKSPACE);
    vs_budget_t b;
    std::memset(&b, 0, sizeof b);
    b.tau_v = b.tau_s = 0.9;
    b.cap_v = b.cap_s = 8;
    EXPECT(vs_select_budget(nullptr, fp, 1, 64, &b, ip, ip, ip, ip, ip, nullptr, 0, nullptr), VS_ERR_INVALID_ARG);
    b.tau_v = 1.5;
    EXPECT(vs_select_budget(fp, fp, 1, 64, &b, ip, ip, ip, ip, ip, nullptr, 0, nullptr), VS_ERR_INVALID_ARG);
    b.tau_v = 0.9;
    b.n_sink = 9;
    EXPECT(vs_select_budget(fp, fp, 1, 64, &b, ip, ip, ip, ip, ip, nullptr, 0, nullptr), VS_ERR_CAPACITY);
    b.n_sink = 0;
    b.cap_s = 0;
    EXPECT(vs_select_budget(fp, fp, 1, 64, &b, ip, ip, ip, ip, ip, nullptr, 0, nullptr), VS_ERR_CAPACITY);
    EXPECT(vs_aggregate(p, p, 4, 1, 64, 0.1f, nullptr, 3, fp, fp, nullptr, nullptr, 0, nullptr, nullptr, 0, 0, nullptr, p, 1 << 20, nullptr),
           VS_ERR_UNSUPPORTED);
    EXPECT(vs_aggregate(p, p, 4, 1, 64, 0.1f, nullptr, 4, fp, fp, nullptr, nullptr, 0, nullptr, nullptr, 0, 0, nullptr, p, 16, nullptr),
           VS_ERR_WORKSPACE);
    w.d_h = 256;
    w.act = 1;
    EXPECT(vs_index_train_step(p, p, 2, 64, &w, fp, fp, 0.f, fp, fp, fp, fp, fp, p, 1 << 30, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_index_train_step(p, p, 2, 64, &w, fp, fp, 1e-30f, fp, fp, fp, fp, fp, p, 16, nullptr), VS_ERR_WORKSPACE);
    EXPECT(vs_rope_apply(nullptr, 4, 64, 0, 1e6, 0, nullptr), VS_ERR_INVALID_ARG);
    EXPECT(vs_rope_apply(p, 4, 64, 0, 1e6, 5, nullptr), VS_ERR_INVALID_ARG);
    for (int code = 1; code >= -8; --code)
        if (!vs_strerror(code) || !vs_strerror(code)[0]) return 5;
    if (!vs_version()[0]) return 6;
    std::puts("host sanitizer run ok");
    return 0;
}
