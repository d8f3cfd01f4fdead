// Calls the library's host-only entry points (tree plan, tree construction, hardware-aware
// choice) so that the test suite can run them under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Built and run by tests/test_host_sanitizers.py; no GPU is touched.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "seqtree.h"

#define CHECK(x) do { if (!(x)) { std::printf("failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main() {
    const double p[31] = {0.7732, 0.1039, 0.0402, 0.0206, 0.0128, 0.0081, 0.0064, 0.0043, 0.0035, 0.0026, 0.0025,
                          0.0021, 0.0016, 0.0014, 0.0010, 0.0010, 0.0010, 0.0007, 0.0007, 0.0006, 0.0007, 0.0006,
                          0.0004, 0.0004, 0.0005, 0.0006, 0.0004, 0.0003, 0.0002, 0.0004, 0.0001};
    for (int n : {1, 2, 17, 64, 300}) {
        for (int depth : {0, 1, 5, 400}) {
            std::vector<int32_t> parent(n), d(n), cs(n + 1), cl(n > 1 ? n - 1 : 1);
            std::vector<uint32_t> anc((size_t)n * 2 * ((n + 63) / 64));
            double f = 0, g = 0;
            const int rc = seq_build_tree(p, 31, n, depth, parent.data(), &f);
            if (rc == SEQ_ERR_SHAPE) continue;      // no tree of that size within the bounds
            CHECK(rc == SEQ_OK);
            CHECK(seq_tree_plan_host(parent.data(), n, d.data(), cs.data(), cl.data(), anc.data()) == SEQ_OK);
            CHECK(seq_tree_expected_tokens(parent.data(), n, p, 31, &g) == SEQ_OK);
            CHECK(g > f - 1e-9 && g < f + 1e-9);
        }
    }
    const int32_t sizes[4] = {1, 8, 32, 128};
    const double t[4] = {10.0, 10.5, 12.0, 20.0};
    int32_t bn = 0, bd = 0;
    double bs = 0;
    CHECK(seq_pick_tree_shape(p, 31, sizes, t, 4, 10, 10.0, 0.5, &bn, &bd, &bs) == SEQ_OK && bs >= 1.0);
    // argument checks that must not read or write anything
    const int32_t bad_parent[3] = {-1, 1, 0};
    CHECK(seq_tree_plan_host(bad_parent, 3, nullptr, nullptr, nullptr, nullptr) == SEQ_ERR_TREE);
    CHECK(seq_build_tree(p, 31, SEQ_MAX_TREE + 1, 3, nullptr, nullptr) != SEQ_OK);
    CHECK(seq_strerror(SEQ_ERR_ALGORITHM) != nullptr && seq_version() > 0);
    std::printf("ok\n");
    return 0;
}
