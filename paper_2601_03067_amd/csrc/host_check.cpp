// Exercises the host-only entry points of libkvfuse (tree construction and workspace layout, the request ordering,
// the threshold closed forms, argument checks) without a GPU.  tests/test_sanitizers.py links it against a build of
// the library whose host code is compiled with the address and undefined-behaviour sanitizers; any report ends the
// run with a non-zero status.  Prints one line per section so that the test can see how far it got.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../../include/kvfuse.h"

static int fails = 0;
#define EXPECT(cond)                                              \
    do {                                                          \
        if (!(cond)) {                                            \
            std::printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #cond); \
            ++fails;                                              \
        }                                                         \
    } while (0)

static kvfuse_tree_spec spec_of(const std::vector<int32_t> &ls, const std::vector<int32_t> &lc, const std::vector<int32_t> &up,
                                int gs)
{
    kvfuse_tree_spec s;
    s.n_leaves = (int32_t)ls.size();
    s.leaf_start = ls.data();
    s.leaf_count = lc.data();
    s.n_units = (int32_t)up.size() - 1;
    s.unit_leaf_ptr = up.data();
    s.group_size = gs;
    return s;
}

int main()
{
    // ---- trees of many shapes through the workspace query (builds the tree, the heights, the tile tables, the layout)
    uint32_t st = 12345u;
    auto rnd = [&](uint32_t m) { st = st * 1664525u + 1013904223u; return (st >> 8) % m; };
    for (int trial = 0; trial < 200; ++trial) {
        const int n_units = 1 + (int)rnd(9);
        std::vector<int32_t> ls, lc, up{0};
        int pos = 0;
        for (int u = 0; u < n_units; ++u) {
            const int leaves = (int)rnd(4);                       // 0 .. 3 leaves: empty units happen
            for (int l = 0; l < leaves; ++l) {
                const int cnt = (int)rnd(300);                    // 0 .. 299 blocks: empty leaves happen
                pos += (int)rnd(3);                               // gaps: blocks in no leaf
                ls.push_back(pos);
                lc.push_back(cnt);
                pos += cnt;
            }
            up.push_back((int32_t)ls.size());
        }
        const int n = pos + (int)rnd(5);
        const kvfuse_tree_spec s = spec_of(ls, lc, up, (int)rnd(4));
        size_t bytes = 0;
        const int rc = kvfuse_workspace_bytes(1 + (int)rnd(4), n, &s, 1 + (int)rnd(64), &bytes);
        EXPECT(rc == KVFUSE_OK && bytes >= 256);
        std::vector<int32_t> ols(ls.size()), olc(lc.size()), oup(up.size()), order(n_units > 1 ? n_units : ls.size());
        EXPECT(kvfuse_tree_spec_shortest_first(&s, ols.data(), olc.data(), oup.data(), order.data()) == KVFUSE_OK);
        int64_t a = 0, b = 0;
        for (int32_t x : lc) a += x;
        for (int32_t x : olc) b += x;
        EXPECT(a == b && oup.back() == (int32_t)ls.size());
    }
    std::printf("trees ok\n");
    // ---- bad specs are errors
    {
        std::vector<int32_t> ls{0, 4}, lc{8, 8}, up{0, 1, 2};
        kvfuse_tree_spec s = spec_of(ls, lc, up, 0);
        size_t bytes = 0;
        EXPECT(kvfuse_workspace_bytes(1, 16, &s, 16, &bytes) == KVFUSE_EINVAL);   // overlapping leaves
        EXPECT(kvfuse_workspace_bytes(1, 10, &s, 16, &bytes) == KVFUSE_EINVAL);   // leaf beyond the table
        EXPECT(kvfuse_workspace_bytes(0, 16, &s, 16, &bytes) == KVFUSE_EINVAL);
        EXPECT(kvfuse_workspace_bytes(1, 16, nullptr, 16, &bytes) == KVFUSE_EINVAL);
        EXPECT(kvfuse_workspace_bytes(1, 16, &s, 65, &bytes) == KVFUSE_EINVAL);
    }
    std::printf("bad specs ok\n");
    // ---- a deep, large tree: 512 ragged requests of 1 - 4 chunks (the largest configuration's shape)
    {
        std::vector<int32_t> ls, lc, up{0};
        int pos = 0;
        for (int u = 0; u < 512; ++u) {
            const int blocks = 32 + (int)rnd(481);
            for (int done = 0; done < blocks; done += 128) {
                ls.push_back(pos + done);
                lc.push_back(blocks - done < 128 ? blocks - done : 128);
            }
            pos += blocks + 1;
            up.push_back((int32_t)ls.size());
        }
        kvfuse_tree_spec s = spec_of(ls, lc, up, 0);
        size_t bytes = 0;
        EXPECT(kvfuse_workspace_bytes(8, pos, &s, 64, &bytes) == KVFUSE_OK && bytes > (size_t)pos * 8);
    }
    std::printf("large tree ok\n");
    // ---- closed forms and the decode workspace query
    {
        EXPECT(std::fabs(kvfuse_exceedance_rate(1000.0, 0.0, 1.0, 0.0) - 500.0) < 1e-9);
        const double u = kvfuse_threshold_for_rate(1e6, 0.01, 0.02, 3.0);
        EXPECT(std::fabs(kvfuse_exceedance_rate(1e6, 0.01, 0.02, u) - 3.0) < 1e-6);
        EXPECT(std::isnan(kvfuse_threshold_for_rate(10.0, 0.0, 0.0, 1.0)));
        double rates[3] = {1.0, 0.0, 2.5}, cr = 0.0, p0[3];
        EXPECT(kvfuse_predict_compression(rates, 3, 100.0, &cr, p0) == KVFUSE_OK && cr > 1.0 && p0[1] == 1.0);
        EXPECT(kvfuse_predict_compression(nullptr, 0, 1.0, nullptr, nullptr) != KVFUSE_OK);
        EXPECT(kvfuse_threshold_feedback(0.9, 2.0, 1.5, 0.1, 0.5, 0.99) > 0.9);
        size_t bytes = 0;
        EXPECT(kvfuse_decode_workspace_bytes(2, 3, 8, 2, 128, 40, &bytes) == KVFUSE_OK && bytes >= 256);
        EXPECT(kvfuse_decode_workspace_bytes(-1, 3, 8, 2, 128, 40, &bytes) == KVFUSE_EINVAL);
    }
    std::printf("closed forms ok\n");
    // ---- null arguments
    EXPECT(kvfuse_create(nullptr, 0, nullptr) != KVFUSE_OK);
    EXPECT(kvfuse_block_norms(nullptr, nullptr, nullptr) != KVFUSE_OK);
    EXPECT(kvfuse_fuse_tree(nullptr, nullptr, 0.9, 1e-3, nullptr, nullptr, nullptr, nullptr, 0) != KVFUSE_OK);
    EXPECT(kvfuse_plan_destroy(nullptr) == KVFUSE_OK);
    std::printf("null arguments ok\n");
    std::printf(fails ? "host check FAILED\n" : "host check passed\n");
    return fails ? 1 : 0;
}
