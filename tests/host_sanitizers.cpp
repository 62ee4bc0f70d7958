// Host-side sanitizer harness (AddressSanitizer + UndefinedBehaviorSanitizer on the host pass
// only): builds partitions with every assignment mode on small random graphs, including a long
// row, k = 1 and k = n, and walks the metadata queries.  No GPU call is made.  Built and run by
// test_host_sanitizers.py.
#include "gnnmi.h"
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <algorithm>
#include <cstdint>
static uint64_t rs = 88172645463325252ull;
static uint64_t rnd() { rs ^= rs << 13; rs ^= rs >> 7; rs ^= rs << 17; return rs; }
#define CHECK(x) do { gnn_status st = (x); if (st != GNN_OK) { printf("line %d: status %d: %s\n", __LINE__, (int)st, gnn_last_error(ctx)); return 1; } } while (0)
int run(int64_t n, int64_t m_draw, int32_t k, int32_t mode, int model, bool sym, bool hub)
{
    std::vector<std::pair<int32_t, int32_t>> e;
    for (int64_t i = 0; i < m_draw; ++i) {
        int32_t a = (int32_t)(rnd() % n), b = (int32_t)(rnd() % n);
        if (hub && (i % 3 == 0)) b = 0;                 // one long row
        if (a == b) continue;
        e.push_back({a, b});
        if (sym) e.push_back({b, a});
    }
    if (model == GNN_GCN) for (int32_t v = 0; v < n; ++v) e.push_back({v, v});
    std::sort(e.begin(), e.end());
    e.erase(std::unique(e.begin(), e.end()), e.end());
    std::vector<int64_t> rp(n + 1, 0);
    std::vector<int32_t> col(e.size());
    for (auto& p : e) rp[p.first + 1]++;
    for (int64_t v = 0; v < n; ++v) rp[v + 1] += rp[v];
    for (size_t i = 0; i < e.size(); ++i) col[i] = e[i].second;
    int32_t dims[4] = {20, 36, 24, 7};
    gnn_config cfg{};
    cfg.model = model; cfg.dtype = GNN_F32; cfg.n_layers = 3; cfg.dims = dims; cfg.has_bias = 1;
    gnn_ctx* ctx = nullptr;
    CHECK(gnn_create(&cfg, &ctx));
    std::vector<int32_t> user(n);
    for (int64_t v = 0; v < n; ++v) user[v] = (int32_t)(rnd() % k);
    CHECK(gnn_build_partitions(ctx, n, rp.data(), col.data(), k, mode, 12345, mode == GNN_PART_USER ? user.data() : nullptr));
    const int32_t* part; int32_t kk;
    CHECK(gnn_get_partition(ctx, &part, &kk));
    int64_t total = 0;
    for (int32_t p = 0; p < kk; ++p) {
        const int32_t* idx; int64_t cnt;
        CHECK(gnn_get_boundary(ctx, p, &idx, &cnt));
        for (int64_t i = 0; i < cnt; ++i) if (idx[i] < 0 || idx[i] >= n || part[idx[i]] == p) { printf("bad boundary\n"); return 1; }
        total += cnt;
    }
    gnn_stats stats;
    CHECK(gnn_get_stats(ctx, &stats));
    if (stats.sum_boundary != total) { printf("sum_boundary mismatch\n"); return 1; }
    const int32_t* order;
    CHECK(gnn_get_schedule(ctx, &order));
    CHECK(gnn_set_layer_order(ctx, GNN_ORDER_AUTO));
    int64_t a, b;
    CHECK(gnn_workspace_bytes(ctx, &a, &b));
    int32_t it[64]; double obj[64];
    (void)gnn_get_partitioner_history(ctx, it, obj, 64);
    gnn_destroy(ctx);
    return 0;
}
int main()
{
    int bad = 0;
    for (int mode : {GNN_PART_USER, GNN_PART_RANDOM, GNN_PART_LP, GNN_PART_SWITCHING})
        for (int model : {GNN_GCN, GNN_SAGE_MEAN, GNN_GAT})
            for (int k : {1, 2, 5, 16}) {
                bad += run(3000, 20000, k, mode, model, true, false);
                bad += run(2000, 9000, k, mode, model, false, true);
            }
    bad += run(50, 100, 50, GNN_PART_RANDOM, GNN_GCN, true, false);   // k = n
    bad += run(7, 3, 3, GNN_PART_SWITCHING, GNN_SAGE_MEAN, true, false);
    printf("failures: %d\n", bad);
    return bad != 0;
}
