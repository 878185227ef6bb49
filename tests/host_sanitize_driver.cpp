// Host-side exerciser of the C ABI for a build with AddressSanitizer and UndefinedBehaviorSanitizer on the host
// code (tests/test_host_sanitizers.py compiles the library's sources host-only together with this file and runs
// the result).  Everything here stays on the host: contexts are created, queried and destroyed, and every
// compute entry point is called in ways its argument validation must refuse before anything is launched.
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#include "koala.h"

static int failures = 0;
#define EXPECT(cond)                                                         \
    do {                                                                     \
        if (!(cond)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
    } while (0)

struct Tree {
    std::vector<int32_t> parent, rank, topk;
    int depth;
    koala_tree c() const { return koala_tree{(int)parent.size(), depth, parent.data(), rank.data(), topk.data()}; }
};

// level d keeps `widths[d]` nodes, children handed out in order to the previous level's nodes, ranks by arrival
static Tree make_tree(const std::vector<int> &topk, const std::vector<int> &widths) {
    Tree t;
    t.depth = (int)topk.size();
    t.topk.assign(topk.begin(), topk.end());
    t.parent.push_back(-1);
    t.rank.push_back(0);
    int first = 0, count = 1;
    for (size_t d = 0; d < topk.size(); ++d) {
        int made = 0;
        for (int r = 0; r < topk[d] && made < widths[d + 1]; ++r)
            for (int p = first; p < first + count && made < widths[d + 1]; ++p) {
                t.parent.push_back(p);
                t.rank.push_back(r);
                ++made;
            }
        // nodes must be ordered by depth only; siblings' ranks are distinct by construction
        first += count;
        count = made;
    }
    return t;
}

int main() {
    const koala_shape shape{256, 4, 64, 688, 1000, 4, 1e-6f, 1e4f, KOALA_FP32};
    const koala_shape shape_bf{512, 4, 128, 1408, 4000, 3, 1e-6f, 1e4f, KOALA_BF16};
    const koala_draft_shape eagle{KOALA_DRAFT_EAGLE, 2, 0, 8};
    const koala_draft_shape medusa{KOALA_DRAFT_MEDUSA, 2, 4, 1};
    const Tree trees[] = {make_tree({2, 2}, {1, 2, 4}), make_tree({4, 2, 2, 1, 1}, {1, 4, 8, 6, 4, 3}),
                          make_tree({10, 5, 3, 2}, {1, 10, 20, 18, 15}), make_tree({}, {1}),
                          make_tree(std::vector<int>(63, 1), std::vector<int>(64, 1))};
    for (const Tree &t : trees)
        for (const koala_shape *s : {&shape, &shape_bf})
            for (const koala_draft_shape *d : {&eagle, &medusa}) {
                for (int mb : {1, 3, 8}) {
                    koala_ctx *c = nullptr;
                    const koala_tree ct = t.c();
                    const koala_status st = koala_create(s, d, &ct, mb, &c);
                    if (d->kind == KOALA_DRAFT_MEDUSA && d->medusa_heads < t.depth) {
                        EXPECT(st == KOALA_E_SHAPE && c == nullptr);
                        continue;
                    }
                    EXPECT(st == KOALA_OK && c != nullptr);
                    if (!c) continue;
                    size_t bytes = 0;
                    EXPECT(koala_workspace_bytes(c, &bytes) == KOALA_OK && bytes > 0);
                    EXPECT(koala_workspace_bytes(c, nullptr) == KOALA_E_NULL);
                    // unbound: every compute call is refused on the host
                    int32_t dummy[8] = {0};
                    float fdummy[8] = {0};
                    koala_gen_stats stats;
                    EXPECT(koala_tree_verify(c, nullptr, 1, dummy, fdummy, nullptr, dummy) == KOALA_E_WORKSPACE);
                    EXPECT(koala_draft_expand(c, nullptr, 1, fdummy, dummy, 1, dummy, nullptr) == KOALA_E_WORKSPACE);
                    EXPECT(koala_accept_prefix(c, nullptr, 1, dummy, dummy, dummy, dummy, dummy, 0) == KOALA_E_WORKSPACE);
                    EXPECT(koala_accept_sample_static(c, nullptr, 1, dummy, fdummy, fdummy, fdummy, fdummy, 1.f, dummy,
                                                      dummy, dummy, 0) == KOALA_E_WORKSPACE);
                    EXPECT(koala_generate(c, nullptr, fdummy, dummy, 1, 1, 1, 1, dummy, &stats) == KOALA_E_WORKSPACE);
                    EXPECT(koala_tree_verify(c, nullptr, 0, dummy, fdummy, nullptr, dummy) != KOALA_OK);
                    EXPECT(koala_last_error(c) != nullptr && koala_last_error(c)[0] != 0);
                    EXPECT(koala_bind(c, nullptr, nullptr, nullptr, 0) == KOALA_E_NULL);
                    EXPECT(koala_profile_begin(c, 0) == KOALA_E_SHAPE);
                    koala_destroy(c);
                }
            }
    // malformed trees and shapes
    {
        koala_ctx *c = nullptr;
        const int32_t p1[] = {0, 0}, r1[] = {0, 0}, k1[] = {1};
        koala_tree bad{2, 1, p1, r1, k1};
        EXPECT(koala_create(&shape, &eagle, &bad, 1, &c) == KOALA_E_SHAPE && !c);
        const int32_t p2[] = {-1, 0, 0}, r2[] = {0, 0, 0}, k2[] = {2};
        koala_tree dup{3, 1, p2, r2, k2};
        EXPECT(koala_create(&shape, &eagle, &dup, 1, &c) == KOALA_E_SHAPE && !c);
        const int32_t p3[] = {-1, 0, 1, 0}, r3[] = {0, 0, 0, 1}, k3[] = {2, 1};
        koala_tree unordered{4, 2, p3, r3, k3};
        EXPECT(koala_create(&shape, &eagle, &unordered, 1, &c) == KOALA_E_SHAPE && !c);
        koala_shape s2 = shape;
        s2.hidden = 250;
        const koala_tree ok = trees[0].c();
        EXPECT(koala_create(&s2, &eagle, &ok, 1, &c) == KOALA_E_SHAPE && !c);
        s2 = shape;
        s2.dtype = 9;
        EXPECT(koala_create(&s2, &eagle, &ok, 1, &c) == KOALA_E_UNSUPPORTED && !c);
        EXPECT(koala_create(&shape, &eagle, &ok, 0, &c) == KOALA_E_SHAPE && !c);
        EXPECT(koala_create(nullptr, &eagle, &ok, 1, &c) == KOALA_E_NULL);
        EXPECT(koala_last_error(nullptr) != nullptr);
        koala_destroy(nullptr);
    }
    // training entry points: argument validation only
    {
        koala_disc_shape ds{64, 100, 32, 2};
        size_t bytes = 0;
        EXPECT(koala_train_workspace_bytes(&ds, 8, &bytes) == KOALA_OK && bytes > 0);
        EXPECT(koala_train_workspace_bytes(&ds, 0, &bytes) == KOALA_E_SHAPE);
        ds.n_fc = 4;
        EXPECT(koala_train_workspace_bytes(&ds, 8, &bytes) == KOALA_E_SHAPE);
        ds.n_fc = 2;
        koala_disc_params dp{};
        float x[4] = {0};
        EXPECT(koala_train_disc_step(&ds, &dp, nullptr, 8, x, x, x, 0.1f, x, 1u << 30, x) == KOALA_E_NULL);
        EXPECT(koala_train_disc_step(&ds, nullptr, nullptr, 8, x, x, x, 0.1f, x, 1u << 30, x) == KOALA_E_NULL);
        EXPECT(koala_train_gen_grad(&ds, &dp, nullptr, 8, x, x, x, -1.f, x, 1u << 30, x, x) == KOALA_E_SHAPE);
        EXPECT(koala_train_medusa_workspace_bytes(8, 64, 9, &bytes) == KOALA_E_SHAPE);
        EXPECT(koala_train_medusa_workspace_bytes(8, 64, 2, &bytes) == KOALA_OK && bytes > 0);
        float *blocks[2] = {nullptr, nullptr};
        EXPECT(koala_train_medusa_head_step(nullptr, 8, 64, 100, 2, blocks, x, x, x, 0.1f, x, 1u << 30) == KOALA_E_NULL);
        EXPECT(koala_train_medusa_head_step(nullptr, 8, 64, 100, 2, blocks, x, x, x, 0.1f, x, 16) == KOALA_E_WORKSPACE);
        double gbs = 0;
        EXPECT(koala_measure_stream_read(nullptr, nullptr, 64, x, 1, &gbs) == KOALA_E_NULL);
    }
    printf(failures ? "host sanitize driver: %d failures\n" : "host sanitize driver: ok\n", failures);
    return failures ? 1 : 0;
}
