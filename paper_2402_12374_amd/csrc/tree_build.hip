// Sequoia tree construction and the hardware-aware choice of tree size and depth: host code,
// run once per deployment (the tree is fixed ahead of time, Sec. 4.1), no GPU involved.
//
// Sec. 3.1.2: with acceptance rates p[k] per child position, the expected number of tokens a
// verification of tree T generates is F(T) = sum over nodes of the product of the rates along
// the node's path.  The dynamic program of Algorithm 1, with the depth bound of its appendix:
//
//     T[1, d, 0]   = 1
//     T[n, d, b]   = max over 1 <= m < n of  T[n - m, d, b - 1] + p[b] * Tmax[m, d - 1]
//     Tmax[n, d]   = max over b of T[n, d, b]
//
// (the root keeps its first b-1 children; a subtree of m nodes and one level less hangs below
// its b-th child).  The arg-max m of every cell and the arg-max b of every (n, d) are kept, which
// is all it takes to rebuild an optimal tree: peel the root's children off from the last one.
//
// Layout: levels are the slow index so that the inner loop over m reads two contiguous rows,
// T[*, d, b-1] backwards and Tmax[*, d-1] forwards.  n = 1024, 32 levels, 64 branches is about
// a second on one core.
#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

#include "seq_internal.h"

namespace seqtree {
namespace {

constexpr double kNone = -std::numeric_limits<double>::infinity();

struct Program {
    int N = 0, L = 0, B = 0;                  // nodes, levels (depth limit + 1), branches
    std::vector<double> t;                    // [L + 1][B + 1][N + 1]
    std::vector<double> tmax;                 // [L + 1][N + 1]
    std::vector<int16_t> arg_m;               // [L + 1][B + 1][N + 1]
    std::vector<int16_t> arg_b;               // [L + 1][N + 1]
    double& T(int d, int b, int n) { return t[((size_t)d * (B + 1) + b) * (N + 1) + n]; }
    int16_t& M(int d, int b, int n) { return arg_m[((size_t)d * (B + 1) + b) * (N + 1) + n]; }
    double& Tmax(int d, int n) { return tmax[(size_t)d * (N + 1) + n]; }
    int16_t& Bbest(int d, int n) { return arg_b[(size_t)d * (N + 1) + n]; }
};

void run_program(Program& pr, const double* p, int p_len, int N, int levels, int B) {
    pr.N = N; pr.L = levels; pr.B = B;
    pr.t.assign((size_t)(levels + 1) * (B + 1) * (N + 1), kNone);
    pr.arg_m.assign(pr.t.size(), 0);
    pr.tmax.assign((size_t)(levels + 1) * (N + 1), kNone);
    pr.arg_b.assign(pr.tmax.size(), 0);
    for (int d = 1; d <= levels; ++d) {
        pr.T(d, 0, 1) = 1.0;
        pr.Tmax(d, 1) = 1.0;
    }
    for (int d = 2; d <= levels; ++d) {
        // all sizes of one level count before the next level: Tmax[*, d - 1] is complete
        for (int n = 2; n <= N; ++n) {
            double best_of_n = kNone;
            int best_b = 0;
            for (int b = 1; b <= B && b < n; ++b) {
                const double rate = b <= p_len ? p[b - 1] : 0.0;
                const double* tree1 = &pr.T(d, b - 1, 0);      // indexed by n - m
                const double* tree2 = &pr.Tmax(d - 1, 0);      // indexed by m
                double best = kNone;
                int best_m = 0;
                for (int m = 1; m < n; ++m) {
                    const double v = tree1[n - m] + rate * tree2[m];   // -inf stays -inf (rates are finite, >= 0)
                    if (v > best) { best = v; best_m = m; }
                }
                pr.T(d, b, n) = best;
                pr.M(d, b, n) = (int16_t)best_m;
                if (best > best_of_n) { best_of_n = best; best_b = b; }
            }
            pr.Tmax(d, n) = best_of_n;
            pr.Bbest(d, n) = (int16_t)best_b;
        }
    }
}

// Children subtree sizes of the best tree with n nodes and d levels, first child first.
void children_sizes(Program& pr, int n, int d, std::vector<int>* sizes) {
    sizes->clear();
    int left = n;
    for (int b = pr.Bbest(d, n); b >= 1; --b) {
        const int m = pr.M(d, b, left);
        sizes->push_back(m);
        left -= m;
    }
    std::reverse(sizes->begin(), sizes->end());
}

int check_rates(const double* acceptance, int32_t max_branch) {
    if (!acceptance) return SEQ_ERR_NULL;
    if (max_branch < 1 || max_branch > SEQ_MAX_CHILDREN) return SEQ_ERR_SHAPE;
    for (int b = 0; b < max_branch; ++b)
        if (!(acceptance[b] >= 0.0) || !(acceptance[b] <= 1.0)) return SEQ_ERR_SHAPE;
    return SEQ_OK;
}

}  // namespace
}  // namespace seqtree

using namespace seqtree;

extern "C" int seq_build_tree(const double* acceptance, int32_t max_branch, int32_t n_tree, int32_t max_depth,
                              int32_t* parent, double* expected_tokens) {
    int rc = check_rates(acceptance, max_branch);
    if (rc != SEQ_OK) return rc;
    if (!parent) return SEQ_ERR_NULL;
    if (n_tree < 1 || n_tree > SEQ_MAX_TREE || max_depth < 0) return SEQ_ERR_SHAPE;
    const int levels = std::min(max_depth, n_tree - 1) + 1;
    const int B = std::min(max_branch, std::max(n_tree - 1, 1));
    Program pr;
    run_program(pr, acceptance, max_branch, n_tree, levels, B);
    if (pr.Tmax(levels, n_tree) == kNone) return SEQ_ERR_SHAPE;   // no tree of this size within the bounds
    if (expected_tokens) *expected_tokens = pr.Tmax(levels, n_tree);

    // breadth-first numbering: parent[i] < i, and the children of a node get ascending ids in
    // the order of their child positions (the order they are drafted and verified in)
    struct Pending { int node, size, levels; };
    std::vector<Pending> queue;
    queue.push_back({0, n_tree, levels});
    parent[0] = -1;
    int next_id = 1;
    std::vector<int> sizes;
    for (size_t head = 0; head < queue.size(); ++head) {
        const Pending cur = queue[head];
        if (cur.size == 1) continue;
        children_sizes(pr, cur.size, cur.levels, &sizes);
        for (int m : sizes) {
            parent[next_id] = cur.node;
            queue.push_back({next_id, m, cur.levels - 1});
            ++next_id;
        }
    }
    return next_id == n_tree ? SEQ_OK : SEQ_ERR_TREE;
}

extern "C" int seq_tree_expected_tokens(const int32_t* parent, int32_t n_tree, const double* acceptance,
                                        int32_t max_branch, double* expected_tokens) {
    int rc = check_rates(acceptance, max_branch);
    if (rc != SEQ_OK) return rc;
    if (!parent || !expected_tokens) return SEQ_ERR_NULL;
    if (n_tree < 1 || n_tree > SEQ_MAX_TREE) return SEQ_ERR_SHAPE;
    rc = validate_parent(parent, n_tree);
    if (rc != SEQ_OK) return rc;
    std::vector<double> score(n_tree, 0.0);
    std::vector<int> seen(n_tree, 0);
    score[0] = 1.0;
    double total = 1.0;
    for (int i = 1; i < n_tree; ++i) {
        const int position = ++seen[parent[i]];      // ascending id among siblings = child position
        score[i] = score[parent[i]] * (position <= max_branch ? acceptance[position - 1] : 0.0);
        total += score[i];
    }
    *expected_tokens = total;
    return SEQ_OK;
}

extern "C" int seq_pick_tree_shape(const double* acceptance, int32_t max_branch, const int32_t* sizes,
                                   const double* verify_time, int32_t n_sizes, int32_t max_depth,
                                   double decode_time, double draft_time, int32_t* best_size,
                                   int32_t* best_depth, double* best_speedup) {
    int rc = check_rates(acceptance, max_branch);
    if (rc != SEQ_OK) return rc;
    if (!sizes || !verify_time || !best_size || !best_depth) return SEQ_ERR_NULL;
    if (n_sizes < 1 || max_depth < 0 || !(decode_time > 0.0) || !(draft_time >= 0.0)) return SEQ_ERR_SHAPE;
    int largest = 0;
    for (int i = 0; i < n_sizes; ++i) {
        if (sizes[i] < 1 || sizes[i] > SEQ_MAX_TREE || !(verify_time[i] > 0.0)) return SEQ_ERR_SHAPE;
        largest = std::max(largest, sizes[i]);
    }
    const int levels = std::min(max_depth, largest - 1) + 1;
    const int B = std::min(max_branch, std::max(largest - 1, 1));
    Program pr;
    run_program(pr, acceptance, max_branch, largest, levels, B);
    double best = -1.0;
    for (int i = 0; i < n_sizes; ++i) {
        for (int d = 0; d < levels; ++d) {        // d = edges below the root = draft steps
            const double g = pr.Tmax(d + 1, sizes[i]);
            if (g == kNone) continue;
            const double s = g / (verify_time[i] / decode_time + d * (draft_time / decode_time));
            if (s > best) { best = s; *best_size = sizes[i]; *best_depth = d; }
        }
    }
    if (best < 0.0) return SEQ_ERR_SHAPE;
    if (best_speedup) *best_speedup = best;
    return SEQ_OK;
}
