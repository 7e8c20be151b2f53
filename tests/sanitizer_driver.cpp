// Host-only driver for the sanitizer test (tests/test_sanitizers.py): built with
// -fsanitize=address,undefined together with the model compiler (forest_pack.cpp,
// forest_api_host.cpp) and the CPU oracle (forest_oracle.c), it walks the compiler through valid
// models of every shape, through every error path and the documented limits, reads everything the
// packed views expose, and runs the oracle on the worked depth-2 example.  Any out-of-bounds access,
// use after free, leak, signed overflow or misaligned access ends it with a non-zero status.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include <random>
#include <vector>

#include "../include/forest.h"
#include "../include/forest_testing.h"

extern "C" int oracle_predict(int32_t n_trees, int32_t n_features, int32_t n_outputs, int32_t leaf_width,
                              const int64_t *tree_offset, const int32_t *feature, const float *threshold,
                              const int32_t *left, const int32_t *right, const float *leaf_value,
                              const int32_t *tree_output, int32_t aggregate, const float *base_score,
                              int32_t transform, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                              int32_t *leaf_node_id, double *raw_out, int32_t n_threads);

namespace {

int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

struct Model {
    std::vector<int64_t> off{0};
    std::vector<int32_t> feature, left, right, tree_output;
    std::vector<float> threshold, leaf_value, base;
    int F = 4, K = 1, W = 1;
    int aggregate = FOREST_AGG_SUM, transform = FOREST_TRANSFORM_NONE, output = FOREST_OUT_BOTH;

    forest_desc desc() const
    {
        forest_desc d{};
        d.n_trees = static_cast<int32_t>(off.size()) - 1;
        d.n_features = F;
        d.n_outputs = K;
        d.leaf_width = W;
        d.tree_offset = off.data();
        d.feature = feature.data();
        d.threshold = threshold.data();
        d.left = left.data();
        d.right = right.data();
        d.leaf_value = leaf_value.data();
        d.tree_output = tree_output.empty() ? nullptr : tree_output.data();
        d.aggregate = aggregate;
        d.base_score = base.empty() ? nullptr : base.data();
        d.transform = transform;
        d.output = output;
        return d;
    }
    int32_t add_node(int32_t f, float t)
    {
        feature.push_back(f);
        threshold.push_back(t);
        left.push_back(-1);
        right.push_back(-1);
        for (int k = 0; k < W; ++k) leaf_value.push_back(0.25f * static_cast<float>(feature.size() % 7));
        return static_cast<int32_t>(feature.size() - off.back() - 1);
    }
    void end_tree(int column = 0)
    {
        off.push_back(static_cast<int64_t>(feature.size()));
        tree_output.push_back(column);
    }
};

// a random tree in pre-order: every node below max_depth is a leaf with probability `stop`
void random_tree(Model &m, std::mt19937 &rng, int max_depth, double stop, bool full)
{
    struct Item {
        int32_t node;
        int depth;
    };
    std::uniform_real_distribution<double> u(0, 1);
    std::normal_distribution<float> n(0, 1);
    const int64_t base = m.off.back();
    std::vector<Item> stack{{m.add_node(-1, 0.0f), 0}};
    while (!stack.empty()) {
        const Item it = stack.back();
        stack.pop_back();
        const bool leaf = it.depth >= max_depth || (!full && u(rng) < stop);
        if (leaf) continue;
        const int pick = static_cast<int>(rng() % 10);
        m.feature[base + it.node] = static_cast<int32_t>(rng() % m.F);
        m.threshold[base + it.node] = pick == 0 ? 1.0f : pick == 1 ? INFINITY : pick == 2 ? -0.0f : pick == 3 ? -INFINITY : n(rng);
        const int32_t a = m.add_node(-1, 0.0f), b = m.add_node(-1, 0.0f);
        m.left[base + it.node] = a;
        m.right[base + it.node] = b;
        stack.push_back({a, it.depth + 1});
        stack.push_back({b, it.depth + 1});
    }
}

// packs the model, reads every array the view exposes, frees it; returns the pack status
int pack_and_read(const Model &m, forest_packed_view *keep = nullptr)
{
    const forest_desc d = m.desc();
    forest_packed *p = nullptr;
    const int rc = forest_pack(&d, &p);
    if (rc != FOREST_OK) {
        EXPECT(p == nullptr);
        return rc;
    }
    forest_packed_view v{};
    EXPECT(forest_pack_view(p, &v) == FOREST_OK);
    EXPECT(v.n_trees == d.n_trees);
    int64_t sum = 0;
    for (int32_t t = 0; t < v.n_trees; ++t) {
        sum += v.tree_n_internal[t] + v.tree_depth[t] + v.tree_is_full[t];
        for (int64_t i = v.node_base[t]; i < v.node_base[t + 1]; ++i) {
            EXPECT(v.split_feature[i] >= 0 && v.split_feature[i] < d.n_features);
            EXPECT(!std::isnan(v.split_threshold[i]));
            sum += v.child_left[i] + v.child_right[i];
        }
        for (int64_t j = v.leaf_base[t]; j < v.leaf_base[t + 1]; ++j) {
            sum += v.leaf_node[j];
            for (int k = 0; k < d.leaf_width; ++k) sum += static_cast<int64_t>(v.leaf_value[j * d.leaf_width + k]);
        }
        if (v.program_groups) sum += v.program_groups[t];
    }
    if (v.rank_threshold) {
        for (int32_t f = 0; f < d.n_features; ++f) {
            for (int32_t i = v.rank_threshold_base[f]; i + 1 < v.rank_threshold_base[f + 1]; ++i)
                EXPECT(v.rank_threshold[i] < v.rank_threshold[i + 1]);
            const forest_rank_bucket &b = v.rank_bucket[f];
            for (int32_t k = 0; k < b.n_buckets; ++k)
                EXPECT(v.rank_bucket_start[b.start_base + k] <= v.rank_bucket_start[b.start_base + k + 1]);
        }
    }
    if (v.wave_tree)
        for (int w = 0; w < v.workgroup_waves; ++w) EXPECT(v.wave_tree[w] <= v.wave_tree[w + 1]);
    if (keep) *keep = v;
    volatile int64_t sink = sum;
    (void)sink;
    forest_pack_free(p);
    return rc;
}

void valid_models()
{
    std::mt19937 rng(13441);
    // full trees of every depth the register kernels take, and one beyond
    for (int depth = 1; depth <= 9; ++depth) {
        Model m;
        m.F = 7;
        for (int t = 0; t < 5; ++t) {
            random_tree(m, rng, depth, 0.0, true);
            m.end_tree();
        }
        forest_packed_view v{};
        EXPECT(pack_and_read(m, &v) == FOREST_OK);
        EXPECT(v.kernel_kind == (depth <= 8 ? depth : 0));
    }
    // irregular trees: scalar and vector leaves, several columns, roots that are leaves
    for (int variant = 0; variant < 12; ++variant) {
        Model m;
        m.F = 1 + static_cast<int>(rng() % 300);
        m.K = 1 + variant % 4;
        m.W = (variant & 4) ? m.K : 1;
        m.aggregate = variant & 1;
        m.transform = m.K > 1 ? FOREST_TRANSFORM_SOFTMAX : FOREST_TRANSFORM_SIGMOID;
        m.base.assign(static_cast<size_t>(m.K), 0.5f);
        const int T = 1 + static_cast<int>(rng() % 40);
        for (int t = 0; t < T; ++t) {
            random_tree(m, rng, static_cast<int>(rng() % 12), 0.2, false);
            m.end_tree(static_cast<int>(rng() % m.K));
        }
        EXPECT(pack_and_read(m) == FOREST_OK);
    }
    // an empty forest and a forest of single leaves are legal
    Model none;
    EXPECT(pack_and_read(none) == FOREST_OK);
    Model leaves;
    for (int t = 0; t < 3; ++t) {
        leaves.add_node(-1, 0.0f);
        leaves.end_tree();
    }
    EXPECT(pack_and_read(leaves) == FOREST_OK);
}

Model stump()
{
    Model m;
    const int32_t r = m.add_node(0, 0.5f);
    m.left[r] = m.add_node(-1, 0.0f);
    m.right[r] = m.add_node(-1, 0.0f);
    m.end_tree();
    return m;
}

void error_paths()
{
    forest_packed *p = nullptr;
    forest_desc d = stump().desc();
    EXPECT(forest_pack(nullptr, &p) == FOREST_EINVAL);
    EXPECT(forest_pack(&d, nullptr) == FOREST_EINVAL);
    EXPECT(forest_pack_view(nullptr, nullptr) == FOREST_EINVAL);
    forest_pack_free(nullptr);

    auto expect = [](Model m, int want) { EXPECT(pack_and_read(m) == want); };
    Model m = stump();
    m.right[0] = 3;  // child out of range
    expect(m, FOREST_ETREE);
    m = stump();
    m.right[0] = -1;
    expect(m, FOREST_ETREE);
    m = stump();
    m.right[0] = 1;  // node reached twice
    expect(m, FOREST_ETREE);
    m = stump();
    m.left[0] = 0;  // cycle
    expect(m, FOREST_ETREE);
    m = stump();
    m.add_node(-1, 0.0f);  // unreachable node
    m.off.back() = 4;
    expect(m, FOREST_ETREE);
    m = stump();
    m.off.push_back(m.off.back());  // empty tree
    m.tree_output.push_back(0);
    expect(m, FOREST_ETREE);
    m = stump();
    m.feature[0] = m.F;
    expect(m, FOREST_EFEATURE);
    m = stump();
    m.threshold[0] = NAN;
    expect(m, FOREST_ENONFINITE);
    m = stump();
    m.base.assign(1, NAN);
    expect(m, FOREST_ENONFINITE);
    m = stump();
    m.aggregate = 2;
    expect(m, FOREST_EINVAL);
    m = stump();
    m.transform = FOREST_TRANSFORM_SOFTMAX;  // needs two outputs
    expect(m, FOREST_EINVAL);
    m = stump();
    m.output = 3;
    expect(m, FOREST_EINVAL);
    m = stump();
    m.tree_output[0] = 1;
    expect(m, FOREST_EINVAL);
    m = stump();
    m.W = 2;  // neither 1 nor K
    m.leaf_value.resize(6);
    expect(m, FOREST_EINVAL);
    m = stump();
    m.off[0] = 1;
    expect(m, FOREST_EINVAL);
}

void limits()
{
    Model m = stump();
    m.F = FOREST_MAX_FEATURES;
    m.feature[0] = FOREST_MAX_FEATURES - 1;
    EXPECT(pack_and_read(m) == FOREST_OK);
    m.F = FOREST_MAX_FEATURES + 1;
    EXPECT(pack_and_read(m) == FOREST_ELIMIT);
    m = stump();
    m.K = FOREST_MAX_OUTPUTS + 1;
    EXPECT(pack_and_read(m) == FOREST_ELIMIT);
    // a left chain of FOREST_MAX_DEPTH tests loads, one more does not
    for (int extra = 0; extra < 2; ++extra) {
        Model c;
        const int depth = FOREST_MAX_DEPTH + extra;
        int32_t cur = c.add_node(0, 0.0f);
        for (int l = 0; l < depth; ++l) {
            const int32_t a = c.add_node(l + 1 < depth ? l % c.F : -1, static_cast<float>(l));
            const int32_t b = c.add_node(-1, 0.0f);
            c.left[cur] = a;
            c.right[cur] = b;
            cur = a;
        }
        c.end_tree();
        EXPECT(pack_and_read(c) == (extra ? FOREST_ELIMIT : FOREST_OK));
    }
    uint16_t code = 0, entry = 0;
    const int n = forest_rank_code(0, &code, &entry);
    EXPECT(n > 1);
    EXPECT(forest_rank_code(n - 1, &code, &entry) == n);
    EXPECT(forest_rank_code(n, &code, &entry) == FOREST_EINVAL);
    EXPECT(forest_rank_code(-1, &code, &entry) == FOREST_EINVAL);
    EXPECT(forest_rank_code(0, nullptr, &entry) == FOREST_EINVAL);
    EXPECT(forest_strerror(FOREST_ETREE)[0] == 'm' && forest_strerror(12345)[0] == 'u');
}

// The hand-derived depth-2 example (tests/golden/depth2_worked_example.json): I0: x2 <= 0.5,
// I1 (left): x0 <= -1, I2 (right): x1 <= 2; leaves in-order hold 0.1 .. 0.4.
void oracle_worked_example()
{
    const int64_t off[2] = {0, 7};
    const int32_t feature[7] = {2, 0, 1, -1, -1, -1, -1};
    const float threshold[7] = {0.5f, -1.0f, 2.0f, 0, 0, 0, 0};
    const int32_t left[7] = {1, 3, 5, -1, -1, -1, -1}, right[7] = {2, 4, 6, -1, -1, -1, -1};
    const float value[7] = {0, 0, 0, 0.1f, 0.2f, 0.3f, 0.4f};
    const float X[4][3] = {{0, 3, 0.7f}, {-2, 0, 0.5f}, {5, 9, 0.1f}, {5, 1, 0.9f}};
    float scores[4];
    int32_t labels[4], leaf[4];
    double raw[4];
    for (int threads = 1; threads <= 3; threads += 2) {
        EXPECT(oracle_predict(1, 3, 1, 1, off, feature, threshold, left, right, value, nullptr, 0, nullptr, 0,
                              &X[0][0], 4, scores, labels, leaf, raw, threads) == 0);
        const int32_t want_leaf[4] = {6, 3, 4, 5};
        const float want[4] = {0.4f, 0.1f, 0.2f, 0.3f};
        for (int r = 0; r < 4; ++r) EXPECT(leaf[r] == want_leaf[r] && scores[r] == want[r] && labels[r] == 0);
    }
    EXPECT(oracle_predict(1, 3, 1, 2, off, feature, threshold, left, right, value, nullptr, 0, nullptr, 0,
                          &X[0][0], 4, scores, labels, leaf, raw, 1) == -1);
    EXPECT(oracle_predict(1, 3, 1, 1, off, feature, threshold, left, right, value, nullptr, 0, nullptr, 0,
                          &X[0][0], 0, nullptr, nullptr, nullptr, nullptr, 4) == 0);
}

}  // namespace

int main()
{
    valid_models();
    error_paths();
    limits();
    oracle_worked_example();
    if (failures) {
        std::fprintf(stderr, "%d expectation(s) failed\n", failures);
        return 1;
    }
    std::puts("sanitizer driver: ok");
    return 0;
}
