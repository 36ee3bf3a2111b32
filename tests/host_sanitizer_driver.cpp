// Exercises the host entry points of the library on random graphs under AddressSanitizer and
// UndefinedBehaviorSanitizer (built and run by test_host_sanitizers.py; host code only, no GPU).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "gnn.h"

#define CHECK(cond)                                                  \
    do {                                                             \
        if (!(cond)) {                                               \
            std::fprintf(stderr, "check failed: %s (line %d)\n", #cond, __LINE__); \
            std::exit(1);                                            \
        }                                                            \
    } while (0)

static void random_symmetric(int n, int m, unsigned seed, bool loops, std::vector<int32_t> &rp, std::vector<int32_t> &ci)
{
    std::mt19937 rng(seed);
    std::vector<std::vector<int32_t>> adj(n);
    for (int e = 0; e < m && n > 0; ++e) {
        const int a = (int)(rng() % n), b = (int)(rng() % n);
        adj[a].push_back(b);  // duplicates and self loops on purpose: the library must cope
        adj[b].push_back(a);
    }
    if (loops)
        for (int i = 0; i < n; ++i) adj[i].push_back(i);
    rp.assign(n + 1, 0);
    ci.clear();
    for (int i = 0; i < n; ++i) {
        for (int32_t j : adj[i]) ci.push_back(j);
        rp[i + 1] = (int32_t)ci.size();
    }
}

int main()
{
    const int shapes[][2] = {{0, 0}, {1, 0}, {1, 3}, {2, 1}, {17, 40}, {300, 900}, {2000, 30000}, {5000, 6000},
                             {40000, 450000} /* large enough for the worker threads of the row-parallel passes */};
    unsigned seed = 1;
    for (const auto &sh : shapes) {
        for (int loops = 0; loops < 2; ++loops) {
            const int n = sh[0];
            std::vector<int32_t> rp, ci;
            random_symmetric(n, sh[1], seed++, loops != 0, rp, ci);
            const int64_t nnz = rp[n];
            std::vector<int32_t> perm(n + 1), iperm(n + 1);
            double aes = -1;
            int did = -1;
            CHECK(gnn_reorder(n, rp.data(), ci.data(), perm.data(), iperm.data(), &aes, &did, 1) == GNN_OK);
            for (int i = 0; i < n; ++i) CHECK(perm[i] >= 0 && perm[i] < n && iperm[perm[i]] == i);
            CHECK(gnn_reorder(n, rp.data(), ci.data(), perm.data(), iperm.data(), nullptr, nullptr, 0) == GNN_OK);
            int64_t s = -1;
            CHECK(gnn_aes(n, rp.data(), ci.data(), &s, &aes) == GNN_OK && s >= 0);
            std::vector<float> ew(nnz + 1), ew2(nnz + 1), ewt(nnz + 1);
            CHECK(gnn_gcn_norm(n, rp.data(), ci.data(), ew.data()) == GNN_OK);
            std::vector<int32_t> rp2(n + 1), ci2(nnz + 1), rpt(n + 1), cit(nnz + 1);
            CHECK(gnn_apply_perm_csr(n, rp.data(), ci.data(), ew.data(), perm.data(), rp2.data(), ci2.data(), ew2.data()) == GNN_OK);
            CHECK(rp2[n] == nnz);
            CHECK(gnn_apply_perm_csr(n, rp.data(), ci.data(), nullptr, perm.data(), rp2.data(), ci2.data(), nullptr) == GNN_OK);
            CHECK(gnn_csr_transpose(n, rp.data(), ci.data(), ew.data(), rpt.data(), cit.data(), ewt.data()) == GNN_OK);
            CHECK(rpt[n] == nnz);
            for (int dim : {1, 3, 16, 22, 64, 96, 1323}) {
                int32_t ngs = 0, dw = 0, wpb = 0;
                CHECK(gnn_decide(n, nnz, 0, dim, &ngs, &dw, &wpb) == GNN_OK);
                CHECK(ngs >= 1 && dw >= 1 && dw <= 64 && (dw & (dw - 1)) == 0 && wpb >= 1 && wpb <= 16);
            }
        }
    }
    // malformed input is refused, not read out of bounds
    {
        std::vector<int32_t> rp = {0, 2, 1}, ci = {0, 1}, perm(2), iperm(2);
        CHECK(gnn_reorder(2, rp.data(), ci.data(), perm.data(), iperm.data(), nullptr, nullptr, 1) == GNN_ECSR);
        std::vector<int32_t> rp3 = {0, 1, 2}, ci3 = {0, 7};
        CHECK(gnn_reorder(2, rp3.data(), ci3.data(), perm.data(), iperm.data(), nullptr, nullptr, 1) == GNN_ECSR);
        CHECK(gnn_reorder(2, nullptr, ci3.data(), perm.data(), iperm.data(), nullptr, nullptr, 1) == GNN_EINVAL);
    }
    int dwp = 0;
    double wpt = 0;
    int64_t smem = 0;
    CHECK(gnn_paper_model(64, 32, 128, 8, &dwp, &wpt, &smem) == GNN_OK);
    std::puts("host sanitizer driver: ok");
    return 0;
}
