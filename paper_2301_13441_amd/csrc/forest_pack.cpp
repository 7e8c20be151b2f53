// Host-side model compiler: caller's per-node arrays -> packed operator representation.
//
// Follows Section 3.1.2 / Table 2: internal nodes are numbered in level order (I_0, I_1, ..),
// leaves in in-order (L_0, L_1, ..).  The weights W1 (feature selection) and W2 (thresholds)
// become the split program; W3 (equivalently the path matrix C and path lengths D) becomes
// child references; the leaf payloads become the table E.  All weights are converted at
// compile time so that nothing is re-typed at run time (Section 3.2, "weights can be handled
// both during compilation and runtime").
//
// Split-program order.  The kernels shift one outcome bit per entry into a 32-bit word
// (word = 2 * word + outcome), so the first entry of a 32-entry block lands in bit 31.  To
// make bit j of word w the outcome of position 32 * w + j, each block is stored in
// descending position.  "Position" is the level-order ordinal i for the generic kernel and
// the heap index h = i + 1 for full trees (root 1, children 2h and 2h + 1, position 0 is
// padding), which keeps every level of a full tree inside whole words from depth 5 on.
// Padding entries test feature 0 against +Inf; the walk never visits them.
//
// Rank family (dtype rewriting of the INPUT, Section 4.3.1 taken one step further: a
// comparison only needs to know where x falls among the thresholds it is compared with).
// For feature f let tau_0 < tau_1 < ... < tau_{m-1} be the distinct thresholds of all nodes
// that test f, and rank(x) = #{i : tau_i < x} (m for NaN).  A node with threshold tau_j sends
// x right iff !(x <= tau_j) iff rank(x) > j: an integer comparison with exactly the float
// comparison's result for every x, including NaN, infinities and signed zeros.  One rank
// register covers a segment of RANK_SEG = 12287 consecutive thresholds; local ranks and node
// indices,
//     rv = clamp(rank - RANK_SEG s, 0, L_s),   j' = j - RANK_SEG s,
// are stored as f16 codes (forest_model.hpp) such that one packed fused multiply-add with clamp
// gives the outcome bit rv > j' exactly.  Two rows share a register (low / high half), so one
// packed instruction compares two rows.  The kernels turn the 8 outcomes of a block of 8
// entries into one outcome byte per row, first entry in bit 7 (on the matrix core, or with a
// tree of packed fused multiply-adds: forest_kernels_rank.hip).  Entries are therefore stored
// in blocks of 8, descending position inside a block.
//
// Rank lookup tables: per feature a uniform bucket grid over the finite threshold range with,
// per bucket, the number of thresholds in lower buckets (build_rank_tables below); the kernels
// get a bracket of rank(x) from it and finish with a short search (forest_rank_common.hpp).
#include <algorithm>
#include <array>
#include <cassert>
#include <cmath>
#include <cstring>
#include <limits>
#include <numeric>

#include "forest_model.hpp"

namespace forest_impl {
namespace {

struct TreeShape {
    std::vector<int32_t> internal;      // caller node index of I_0, I_1, ... (level order)
    std::vector<int32_t> leaves;        // caller node index of L_0, L_1, ... (in-order)
    std::vector<int32_t> ordinal;       // per caller node: internal ordinal or ~leaf ordinal
    std::vector<int32_t> level_begin;   // internal[level_begin[l] .. level_begin[l+1]) sit at depth l
    int32_t depth = 0;                  // longest root-to-leaf path, counted in tests
    bool full = true;                   // every leaf at `depth`
};

// Level-order walk from the root.  Rejects out-of-range children, nodes reached twice
// (shared subtrees and cycles) and nodes never reached.
int analyse_tree(const forest_desc &d, int64_t base, int64_t n, TreeShape &s)
{
    if (n < 1 || n > std::numeric_limits<int32_t>::max()) return FOREST_ETREE;
    std::vector<uint8_t> seen(static_cast<size_t>(n), 0);
    std::vector<int32_t> level{0}, next;
    std::vector<int32_t> node_depth(static_cast<size_t>(n), 0);
    seen[0] = 1;
    s.ordinal.assign(static_cast<size_t>(n), 0);
    int32_t depth = 0, leaf_min = std::numeric_limits<int32_t>::max(), leaf_max = 0;
    int64_t reached = 0;
    while (!level.empty()) {
        next.clear();
        s.level_begin.push_back(static_cast<int32_t>(s.internal.size()));
        for (int32_t v : level) {
            ++reached;
            const int32_t f = d.feature[base + v];
            if (f < 0) {
                leaf_min = std::min(leaf_min, depth);
                leaf_max = std::max(leaf_max, depth);
                continue;
            }
            if (f >= d.n_features) return FOREST_EFEATURE;
            if (std::isnan(d.threshold[base + v])) return FOREST_ENONFINITE;
            s.ordinal[v] = static_cast<int32_t>(s.internal.size());
            s.internal.push_back(v);
            const int32_t kids[2] = {d.left[base + v], d.right[base + v]};
            for (int32_t c : kids) {
                if (c < 0 || c >= n) return FOREST_ETREE;
                if (seen[c]) return FOREST_ETREE;
                seen[c] = 1;
                next.push_back(c);
            }
        }
        level.swap(next);
        if (!level.empty()) ++depth;
        if (depth > FOREST_MAX_DEPTH) return FOREST_ELIMIT;
    }
    if (reached != n) return FOREST_ETREE;  // unreachable nodes
    while (s.level_begin.size() > 1 && s.level_begin.back() == static_cast<int32_t>(s.internal.size()))
        s.level_begin.pop_back();  // levels that hold only leaves
    if (s.internal.empty()) s.level_begin.clear();
    s.level_begin.push_back(static_cast<int32_t>(s.internal.size()));
    s.depth = leaf_max;
    s.full = (leaf_min == leaf_max);

    // In-order leaf numbering: left subtree, node, right subtree; only leaves get a number.
    std::vector<int32_t> stack;
    int32_t v = 0;
    for (;;) {
        while (d.feature[base + v] >= 0) {
            stack.push_back(v);
            v = d.left[base + v];
        }
        s.ordinal[v] = ~static_cast<int32_t>(s.leaves.size());
        s.leaves.push_back(v);
        if (stack.empty()) break;
        v = d.right[base + stack.back()];
        stack.pop_back();
    }
    return FOREST_OK;
}


int check_desc(const forest_desc &d)
{
    if (d.n_trees < 0 || d.n_features < 1 || d.n_outputs < 1) return FOREST_EINVAL;
    if (d.n_features > FOREST_MAX_FEATURES || d.n_outputs > FOREST_MAX_OUTPUTS) return FOREST_ELIMIT;
    if (d.leaf_width != 1 && d.leaf_width != d.n_outputs) return FOREST_EINVAL;
    if (d.aggregate != FOREST_AGG_SUM && d.aggregate != FOREST_AGG_MEAN) return FOREST_EINVAL;
    if (d.transform < FOREST_TRANSFORM_NONE || d.transform > FOREST_TRANSFORM_SOFTMAX) return FOREST_EINVAL;
    if (d.transform == FOREST_TRANSFORM_SOFTMAX && d.n_outputs < 2) return FOREST_EINVAL;
    if (d.output < FOREST_OUT_SCORES || d.output > FOREST_OUT_BOTH) return FOREST_EINVAL;
    if (!d.tree_offset) return FOREST_EINVAL;
    if (d.tree_offset[0] != 0) return FOREST_EINVAL;
    for (int32_t t = 0; t < d.n_trees; ++t)
        if (d.tree_offset[t + 1] <= d.tree_offset[t]) return FOREST_ETREE;  // empty tree
    if (d.n_trees > 0 && (!d.feature || !d.threshold || !d.left || !d.right || !d.leaf_value))
        return FOREST_EINVAL;
    if (d.tree_output && d.leaf_width == 1)
        for (int32_t t = 0; t < d.n_trees; ++t)
            if (d.tree_output[t] < 0 || d.tree_output[t] >= d.n_outputs) return FOREST_EINVAL;
    if (d.base_score)
        for (int32_t k = 0; k < d.n_outputs; ++k)
            if (std::isnan(d.base_score[k])) return FOREST_ENONFINITE;
    return FOREST_OK;
}

}  // namespace

// Trees of irregular shape differ in program length, and a workgroup ends with its slowest
// wave: cut the trees (processing order) into lds_waves contiguous runs so that the wave that
// finishes last finishes as early as possible.  Cost of a tree: its groups plus two for the work
// at its end.  The waves of a workgroup do not run equally fast: wave w sits on SIMD w mod 4, and
// of the waves a workgroup has on one SIMD the one launched first is served first.  Measured on
// 12-wave workgroups (two per CU, 128 trees of ~124 groups): 540, 610 and 700 clock ticks per
// group for waves 0-3, 4-7 and 8-11.  A run's length is therefore weighed by its wave's pace.
static int wave_pace_permille(int waves, int w)
{
    if (waves != 12) return 1000;  // one or two waves per SIMD: not measured, taken as equal
    return w < 4 ? 876 : (w < 8 ? 989 : 1135);  // ticks per group relative to their mean of 617
}

static void balance_waves(PackedModel &m)
{
    const int waves = m.lds_waves;
    const int32_t T = m.n_trees;
    auto cost = [&](int32_t t) { return static_cast<int64_t>(m.tree[t].n_words) + 2; };
    int64_t lo = 0, hi = 0;  // time of the last wave, in cost x permille: between 0 and all trees on the slowest
    for (int32_t t = 0; t < T; ++t) hi += cost(t) * 1135;
    // greedy cut under a time cap; returns the number of runs and fills `cut` when asked
    auto runs = [&](int64_t cap, int32_t *cut) {
        int n = 0;
        int64_t sum = 0;
        for (int32_t t = 0; t < T; ++t) {
            const int pace = wave_pace_permille(waves, n > 0 ? std::min(n - 1, waves - 1) : 0);
            if (t == 0 || (sum + cost(t)) * pace > cap) {
                if (cut && n <= waves) cut[n] = t;
                ++n;
                sum = 0;
            }
            sum += cost(t);
        }
        return n;
    };
    // a cap below a single tree's time on its wave makes that wave's run empty and the count
    // exceed `waves`, so the search settles on a feasible cap
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (runs(mid, nullptr) <= waves) hi = mid;
        else lo = mid + 1;
    }
    int32_t cut[RANKLDS_WAVES_WIDE + 2] = {};
    const int n = T > 0 ? runs(lo, cut) : 0;
    for (int w = 0; w <= waves; ++w) m.wave_tree[w] = w < n ? cut[w] : T;  // spare waves get no trees
}

int compile_forest(const forest_desc &d, PackedModel &m)
{
    if (int rc = check_desc(d)) return rc;
    const int32_t T = d.n_trees, K = d.n_outputs, W = d.leaf_width;
    m = PackedModel{};
    m.n_trees = T;
    m.n_features = d.n_features;
    m.n_outputs = K;
    m.leaf_width = W;
    m.aggregate = d.aggregate;
    m.transform = d.transform;
    m.output = d.output;
    m.col_trees.assign(K, 0.0);
    m.base.assign(K, 0.0f);
    if (d.base_score) std::copy(d.base_score, d.base_score + K, m.base.begin());

    std::vector<TreeShape> shape(static_cast<size_t>(T));
    bool all_full = T > 0;
    int32_t common_depth = -1;
    for (int32_t t = 0; t < T; ++t) {
        const int64_t base = d.tree_offset[t], n = d.tree_offset[t + 1] - base;
        if (int rc = analyse_tree(d, base, n, shape[t])) return rc;
        const TreeShape &s = shape[t];
        m.max_depth = std::max(m.max_depth, s.depth);
        m.n_internal += static_cast<int64_t>(s.internal.size());
        m.n_leaves += static_cast<int64_t>(s.leaves.size());
        if (!s.full) all_full = false;
        if (common_depth < 0) common_depth = s.depth;
        else if (common_depth != s.depth) all_full = false;
        if (W == 1) m.col_trees[d.tree_output ? d.tree_output[t] : 0] += 1.0;
        else for (int32_t k = 0; k < K; ++k) m.col_trees[k] += 1.0;
    }
    if (m.n_internal > FOREST_MAX_NODES || m.n_leaves > FOREST_MAX_NODES) return FOREST_ELIMIT;
    m.kind = (all_full && common_depth >= 1 && common_depth <= FULL_MAX_DEPTH) ? common_depth
                                                                              : KIND_GENERIC;

    // Choice of kernel family.  The rank families need the per-feature sorted distinct thresholds.
    std::vector<std::vector<float>> per_feature(static_cast<size_t>(d.n_features));
    for (int32_t t = 0; t < T; ++t)
        for (int32_t v : shape[t].internal)
            per_feature[d.feature[d.tree_offset[t] + v]].push_back(d.threshold[d.tree_offset[t] + v]);
    int64_t regs = 0;
    for (auto &v : per_feature) {
        std::sort(v.begin(), v.end());
        v.erase(std::unique(v.begin(), v.end()), v.end());  // -0 == +0: one threshold
        regs += static_cast<int64_t>((v.size() + RANK_SEG - 1) / RANK_SEG);
    }
    auto build_rank_tables = [&]() {
        m.rank_regs = static_cast<int32_t>(regs);
        m.feat_thr_base.assign(1, 0);
        int32_t next_reg = 0;
        for (auto &v : per_feature) {
            m.feat_vfirst.push_back(next_reg);
            next_reg += static_cast<int32_t>((v.size() + RANK_SEG - 1) / RANK_SEG);
            m.thr_sorted.insert(m.thr_sorted.end(), v.begin(), v.end());
            m.feat_thr_base.push_back(static_cast<int32_t>(m.thr_sorted.size()));
        }
        // one spare element: the kernels read a feature's threshold 0 even if it has none
        m.thr_sorted.push_back(std::numeric_limits<float>::infinity());
        // Bucket tables: a uniform grid over the feature's finite threshold range, one bucket
        // per threshold (the kernels resolve brackets of up to 8 thresholds in one step, and a
        // finer grid would only take L2 from the other tables), and for every bucket the number
        // of thresholds in lower buckets.
        // bucket_index is monotone, so thresholds in lower buckets are below x and thresholds in
        // higher buckets are not: start[b] <= rank(x) <= start[b + 1] for b = bucket(x).  The
        // kernels check the bracket against the thresholds themselves before they trust it.
        for (auto &v : per_feature) {
            FeatBucket fb{0.0f, 0.0f, 1, static_cast<int32_t>(m.bucket_start.size())};
            size_t a = 0, b = v.size();
            while (a < b && !std::isfinite(v[a])) ++a;
            while (b > a && !std::isfinite(v[b - 1])) --b;
            if (b > a) {
                fb.lo = v[a];
                const float range = v[b - 1] - v[a];
                const int64_t want = static_cast<int64_t>(v.size()) * RANK_BUCKETS_PER_THRESHOLD;
                const int32_t nb = static_cast<int32_t>(std::min<int64_t>(want, RANK_MAX_BUCKETS));
                const float scale = static_cast<float>(nb) / range;
                if (range > 0.0f && std::isfinite(scale)) {
                    fb.scale = scale;
                    fb.n_buckets = nb;
                }
            }
            size_t i = 0;
            for (int32_t bk = 0; bk <= fb.n_buckets; ++bk) {
                while (i < v.size() && bucket_index(v[i], fb.lo, fb.scale, fb.n_buckets) < bk) ++i;
                m.bucket_start.push_back(static_cast<int32_t>(i));
            }
            m.feat_bucket.push_back(fb);
        }
        // Fast lookup tables.  A uniform grid over the feature's finite thresholds, refined until
        // no bucket holds more than FAST_BUCKET_FILL of them (or the table is as large as it may
        // get); the entry of a bucket is where the window of thresholds the lookup reads begins.
        // The kernel checks every window against x, so nothing rests on its arithmetic placing x
        // in the bucket the arithmetic here does; what a window does not decide takes the general
        // lookup.
        m.fast_feat.assign(static_cast<size_t>(d.n_features), FastLookup{});
        for (int32_t f = 0; f < d.n_features; ++f) {
            const float *v = m.thr_sorted.data() + m.feat_thr_base[f];
            const int32_t n = m.feat_thr_base[f + 1] - m.feat_thr_base[f];
            FastLookup &bf = m.fast_feat[f];
            bf.n = n;
            bf.thr_off = static_cast<uint32_t>(m.feat_thr_base[f]) * sizeof(float);
            bf.tab_off = static_cast<uint32_t>(m.fast_tab.size() * sizeof(uint16_t));
            int32_t a = 0, b = n;
            while (a < b && !std::isfinite(v[a])) ++a;
            while (b > a && !std::isfinite(v[b - 1])) --b;
            bool fast = n >= FAST_WINDOW && n <= FAST_MAX_THRESHOLDS && b > a && v[b - 1] - v[a] > 0.0f;
            std::vector<int32_t> start;
            if (fast) {
                const float lo = v[a], range = v[b - 1] - v[a];
                for (int64_t nb = 2 * static_cast<int64_t>(n);; nb *= 2) {
                    nb = std::min<int64_t>(nb, FAST_MAX_BUCKETS);
                    const float scale = static_cast<float>(nb) / range;
                    if (!std::isfinite(scale)) {
                        fast = false;
                        break;
                    }
                    start.assign(static_cast<size_t>(nb) + 1, 0);
                    int32_t i = 0, fill = 0;
                    for (int32_t bk = 0; bk <= nb; ++bk) {
                        while (i < n && bucket_index(v[i], lo, scale, static_cast<int32_t>(nb)) < bk) ++i;
                        start[bk] = i;
                        if (bk > 0) fill = std::max(fill, start[bk] - start[bk - 1]);
                    }
                    bf.lo = lo;
                    bf.scale = scale;
                    bf.last_bucket = static_cast<float>(nb - 1);
                    if (fill <= FAST_BUCKET_FILL || nb == FAST_MAX_BUCKETS) break;
                }
            }
            bf.fast = fast ? 1 : 0;
            if (fast)
                for (size_t bk = 0; bk + 1 < start.size(); ++bk)
                    m.fast_tab.push_back(static_cast<uint16_t>(std::clamp(start[bk] - 1, 0, n - FAST_WINDOW)));
        }
        m.fast_tab.push_back(0);  // never empty
    };
    if (m.kind != KIND_GENERIC) {
        const size_t rank_lds = std::max(sizeof(double) * 4 * K * 128,
                                         sizeof(uint32_t) * 64 * static_cast<size_t>(regs > 64 ? 128 : 64));
        if (regs <= RANK_MAX_REGS && rank_lds <= 64 * 1024) {
            m.path = PATH_RANK;
            m.x_in_registers = 1;
            m.reg_r = 2;
            build_rank_tables();
        } else if (d.n_features <= 128) {
            // float32 features in vector registers
            m.reg_nv = d.n_features <= 32 ? 1 : d.n_features <= 64 ? 2 : 4;
            m.reg_r = m.reg_nv == 4 ? 1 : 2;
            const size_t rows = 64 * static_cast<size_t>(m.reg_r);
            const size_t lds = sizeof(double) * 4 * K * rows + sizeof(float) * 32 * m.reg_nv * rows;
            if (lds <= 64 * 1024) {
                m.path = PATH_REG;
                m.x_in_registers = 1;
            } else {
                m.reg_nv = m.reg_r = 0;  // many outputs: LDS family
            }
        }
    }
    if (m.path == PATH_LDS && T > 0) {
        // Rank family with the ranks held in LDS: any tree shape.  The workgroup size that puts
        // the most wavefronts on a CU wins (two workgroups of 12 waves when their LDS allows; the
        // small sizes are for many output columns, whose partial sums take 1 KB per wave and
        // column: two waves fit whatever the model).  Models that need more than 256 rank rows
        // stay in the plain family, whose kernels take any model.
        // The small workgroups (4 and 2 waves) are for irregular trees only: measured faster than
        // the plain family's irregular-tree kernel on models with 12- to 32-wide leaves, while
        // shallow full trees with such leaves run faster in the plain full-tree kernels.
        const bool small_workgroups = m.kind == KIND_GENERIC;
        int best_waves = 0;
        size_t best_per_cu = 0;
        for (int waves : RANKLDS_WAVE_CHOICES) {
            if (!small_workgroups && waves < 8) continue;
            const size_t lds = ranklds_lds_bytes(static_cast<int>(std::min<int64_t>(regs, RANKLDS_MAX_REGS)), K, W, waves);
            if (lds > RANKLDS_MAX_LDS) continue;
            // 80 vector registers per lane: at most 6 waves per SIMD, 24 per CU
            const size_t per_cu = std::min<size_t>((CU_LDS_BYTES / lds) * static_cast<size_t>(waves), 24);
            if (per_cu > best_per_cu) {
                best_per_cu = per_cu;
                best_waves = waves;
            }
        }
        if (regs <= RANKLDS_MAX_REGS && best_waves > 0) {
            m.path = PATH_RANK_LDS;
            m.lds_waves = best_waves;
            build_rank_tables();
        }
    }
    const int32_t feature_scale = m.path == PATH_REG ? 1 : 64;
    // split-program entry of internal node `v` of tree `t`
    auto entry_of = [&](int32_t t, int32_t v) -> SplitEntry {
        const int64_t n = d.tree_offset[t] + v;
        const int32_t f = d.feature[n];
        if (m.path != PATH_RANK && m.path != PATH_RANK_LDS) return SplitEntry{f * feature_scale, d.threshold[n]};
        const float *lo = m.thr_sorted.data() + m.feat_thr_base[f];
        const float *hi = m.thr_sorted.data() + m.feat_thr_base[f + 1];
        const int32_t j = static_cast<int32_t>(std::lower_bound(lo, hi, d.threshold[n]) - lo);
        assert(lo + j < hi && lo[j] == d.threshold[n]);
        const int32_t seg = j / RANK_SEG;
        const uint32_t h = rank_entry_bits(j - seg * RANK_SEG);
        const uint32_t pair = h | (h << 16);
        SplitEntry e;
        e.feature_slot = m.feat_vfirst[f] + seg;
        std::memcpy(&e.threshold, &pair, sizeof(pair));
        return e;
    };

    // caller-order views (tests of the compiler read these)
    m.v_node_base.assign(1, 0);
    m.v_leaf_base.assign(1, 0);
    for (int32_t t = 0; t < T; ++t) {
        const TreeShape &s = shape[t];
        const int64_t base = d.tree_offset[t];
        m.v_n_internal.push_back(static_cast<int32_t>(s.internal.size()));
        m.v_depth.push_back(s.depth);
        m.v_is_full.push_back(s.full ? 1 : 0);
        for (int32_t v : s.internal) {
            m.v_feature.push_back(d.feature[base + v]);
            m.v_threshold.push_back(d.threshold[base + v]);
            m.v_left.push_back(s.ordinal[d.left[base + v]]);
            m.v_right.push_back(s.ordinal[d.right[base + v]]);
        }
        for (int32_t v : s.leaves) {
            m.v_leaf_node.push_back(v);
            for (int32_t k = 0; k < W; ++k) m.v_leaf_value.push_back(d.leaf_value[(base + v) * W + k]);
        }
        m.v_node_base.push_back(static_cast<int64_t>(m.v_feature.size()));
        m.v_leaf_base.push_back(static_cast<int64_t>(m.v_leaf_node.size()));
    }

    // processing order: by output column, ties in caller order (keeps each column's sum in
    // ascending tree index)
    std::vector<int32_t> order(static_cast<size_t>(T));
    std::iota(order.begin(), order.end(), 0);
    auto column_of = [&](int32_t t) { return (W == 1 && d.tree_output) ? d.tree_output[t] : 0; };
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return column_of(a) < column_of(b); });

    const float inf = std::numeric_limits<float>::infinity();
    SplitEntry pad{0, inf};
    if (m.path == PATH_RANK || m.path == PATH_RANK_LDS) {
        // register 0 against the largest code: no local rank exceeds it, the outcome bit is 0
        const uint32_t h = rank_entry_bits(RANK_SEG);
        const uint32_t pair = h | (h << 16);
        std::memcpy(&pad.threshold, &pair, sizeof(pair));
    }
    for (int32_t t : order) {
        const TreeShape &s = shape[t];
        const int64_t base = d.tree_offset[t];
        const int32_t n_int = static_cast<int32_t>(s.internal.size());
        TreeMeta tm{};
        tm.prog_base = static_cast<int32_t>(m.prog.size());
        tm.child_base = static_cast<int32_t>(m.child.size());
        tm.leaf_base = static_cast<int32_t>(m.leaf_node.size());
        tm.root_ref = n_int > 0 ? 0 : ~0;
        tm.column = column_of(t);
        tm.caller_tree = t;
        tm.n_internal = n_int;

        if (m.path == PATH_RANK_LDS) {
            // Stream of 8-entry groups, level by level (each level padded to whole groups).  The
            // first entry of a group carries three flags in its low byte: bit 0 = last group of
            // its level, bit 1 = last group of the tree, bit 2 = last group of a chunk (every
            // eighth group of a level, and its last: the walk looks at its nodes chunk by
            // chunk).  The child-reference table is indexed like the stream; a reference >= 0 is
            // the node's ordinal inside the next level.
            const size_t n_levels = s.level_begin.size() - 1;
            if (n_levels == 0) {  // the root is a leaf: one group of padding closes the tree
                for (int j = 0; j < 8; ++j) {
                    m.prog.push_back(pad);
                    m.child.push_back(ChildRef{~0, ~0});
                }
                m.prog[m.prog.size() - 8].feature_slot |= 7 << 16;
            }
            for (size_t l = 0; l < n_levels; ++l) {
                const int32_t lb = s.level_begin[l], le = s.level_begin[l + 1];
                const int32_t next_begin = le;  // ordinals of the next level start here
                // entries: groups of 8 in descending ordinal (the first entry of a group becomes
                // bit 7 of the outcome byte); child references: ascending ordinal
                for (int32_t g0 = lb; g0 < le; g0 += 8) {
                    for (int32_t k = 7; k >= 0; --k)
                        m.prog.push_back(g0 + k < le ? entry_of(t, s.internal[g0 + k]) : pad);
                    if ((g0 - lb) / 8 % RANKLDS_CHUNK_GROUPS == RANKLDS_CHUNK_GROUPS - 1)
                        m.prog[m.prog.size() - 8].feature_slot |= 4 << 16;
                }
                for (int32_t i = lb; i < le; ++i) {
                    const int32_t v = s.internal[i];
                    auto ref_of = [&](int32_t c) {
                        const int32_t o = s.ordinal[c];
                        return o >= 0 ? o - next_begin : o;
                    };
                    m.child.push_back(ChildRef{ref_of(d.left[base + v]), ref_of(d.right[base + v])});
                }
                while (m.child.size() < m.prog.size()) m.child.push_back(ChildRef{~0, ~0});
                const size_t last_group = m.prog.size() - 8;
                m.prog[last_group].feature_slot |= (l + 1 == n_levels ? 7 : 5) << 16;
            }
            tm.n_words = static_cast<int32_t>((m.prog.size() - tm.prog_base) / 8);
            for (int32_t v : s.leaves) {
                m.leaf_node.push_back(v);
                for (int32_t k = 0; k < W; ++k) m.leaf_value.push_back(d.leaf_value[(base + v) * W + k]);
            }
            m.tree.push_back(tm);
            continue;
        }
        // positions: heap index for the full-tree kernels, level-order ordinal otherwise
        const int32_t shift = (m.kind != KIND_GENERIC) ? 1 : 0;
        const int32_t n_pos = n_int + shift;
        const int32_t block = m.path == PATH_RANK ? 8
                              : (m.kind != KIND_GENERIC && m.kind < 5) ? (1 << m.kind) : 32;
        const int32_t n_blocks = std::max(1, (n_pos + block - 1) / block);
        tm.n_words = n_blocks;
        for (int32_t w = 0; w < n_blocks; ++w)
            for (int32_t j = 0; j < block; ++j) {
                const int32_t pos = w * block + (block - 1 - j);
                // where a node sits in the tree's bit string: by heap index, or in the fields
                // the table walk of the rank kernels reads (forest_model.hpp)
                const bool staged = m.path == PATH_RANK && m.kind >= STAGED_MIN_DEPTH && m.kind <= STAGED_TOP_MAX_DEPTH;
                const int32_t i = staged ? staged_position_node(m.kind, pos) : pos - shift;
                if (i < 0 || i >= n_int) {
                    m.prog.push_back(pad);
                } else {
                    m.prog.push_back(entry_of(t, s.internal[i]));
                }
            }
        m.max_words = std::max(m.max_words, n_blocks);
        for (int32_t v : s.internal)
            m.child.push_back(ChildRef{s.ordinal[d.left[base + v]], s.ordinal[d.right[base + v]]});
        for (int32_t v : s.leaves) {
            m.leaf_node.push_back(v);
            for (int32_t k = 0; k < W; ++k) m.leaf_value.push_back(d.leaf_value[(base + v) * W + k]);
        }
        m.tree.push_back(tm);
    }
    if (m.path == PATH_RANK_LDS) balance_waves(m);
    if (m.path == PATH_RANK_LDS && m.kind == KIND_GENERIC && m.rank_regs >= 1 &&
        m.rank_regs <= BANK_WAVES * BANK_REGS && ((K == 1 && W == 1) || (W == K && K <= 2))) {
        // Register-bank program.  A rank register's feature and segment.
        std::vector<int32_t> reg_feature(static_cast<size_t>(m.rank_regs)), reg_segment(static_cast<size_t>(m.rank_regs));
        for (int32_t f = 0; f < d.n_features; ++f) {
            const int32_t r_end = f + 1 < d.n_features ? m.feat_vfirst[f + 1] : m.rank_regs;
            for (int32_t r = m.feat_vfirst[f]; r < r_end; ++r) {
                reg_feature[r] = f;
                reg_segment[r] = r - m.feat_vfirst[f];
            }
        }
        // Rank registers to waves, one block of BANK_PASS_FEATURES columns of X (a prologue pass)
        // after the other: heaviest first, each to the wave with the fewest nodes so far that
        // still has a free register and not yet its share of the block (the waves of a workgroup
        // look the block's registers up side by side, so each should have about as many).
        std::vector<int64_t> reg_nodes(static_cast<size_t>(m.rank_regs), 0);
        for (int32_t t = 0; t < T; ++t)
            for (int32_t v : shape[t].internal) ++reg_nodes[entry_of(t, v).feature_slot];
        std::vector<int32_t> reg_wave(static_cast<size_t>(m.rank_regs)), reg_index(static_cast<size_t>(m.rank_regs));
        struct Block { int32_t f0, f1, r0, r1; };
        std::vector<Block> blocks;
        {
            int64_t load[BANK_WAVES] = {};
            int32_t held[BANK_WAVES] = {};
            for (int32_t f0 = 0; f0 < d.n_features; f0 += BANK_PASS_FEATURES) {
                const int32_t f1 = std::min<int32_t>(f0 + BANK_PASS_FEATURES, d.n_features);
                const int32_t r0 = m.feat_vfirst[f0], r1 = f1 < d.n_features ? m.feat_vfirst[f1] : m.rank_regs;
                if (r0 == r1) continue;  // no thresholds on these columns: the block is never read
                blocks.push_back(Block{f0, f1, r0, r1});
                std::vector<int32_t> by_weight(static_cast<size_t>(r1 - r0));
                std::iota(by_weight.begin(), by_weight.end(), r0);
                std::stable_sort(by_weight.begin(), by_weight.end(),
                                 [&](int32_t a, int32_t b) { return reg_nodes[a] > reg_nodes[b]; });
                const int32_t share = (r1 - r0 + BANK_WAVES - 1) / BANK_WAVES;
                int32_t here[BANK_WAVES] = {};
                for (int32_t r : by_weight) {
                    int best = -1;
                    for (int pass = 0; pass < 2 && best < 0; ++pass)  // second try: the share no longer binds
                        for (int w = 0; w < BANK_WAVES; ++w)
                            if (held[w] < BANK_REGS && (pass == 1 || here[w] < share) && (best < 0 || load[w] < load[best])) best = w;
                    reg_wave[r] = best;
                    ++held[best];
                    ++here[best];
                    load[best] += reg_nodes[r];
                }
            }
        }
        // nodes of every tree (processing order) by rank register
        std::vector<std::vector<std::pair<int32_t, int32_t>>> tree_regs(static_cast<size_t>(T));  // (register, nodes)
        for (int32_t ti = 0; ti < T; ++ti) {
            std::vector<int32_t> count(static_cast<size_t>(m.rank_regs), 0);
            for (int32_t v : shape[order[ti]].internal) ++count[entry_of(order[ti], v).feature_slot];
            for (int32_t r = 0; r < m.rank_regs; ++r)
                if (count[r]) tree_regs[ti].emplace_back(r, count[r]);
        }
        // nodes of every tree by wave, under the current dealing
        std::vector<std::array<int32_t, BANK_WAVES>> per_wave(static_cast<size_t>(T));
        auto count_per_wave = [&] {
            for (int32_t ti = 0; ti < T; ++ti) {
                per_wave[ti].fill(0);
                for (const auto &rc : tree_regs[ti]) per_wave[ti][reg_wave[rc.first]] += rc.second;
            }
        };
        // units of a batch of trees a and b (b < 0: a alone), and the units of its busiest wave
        auto batch_units = [&](int32_t a, int32_t b, int64_t *busiest) {
            int64_t units = 0, most = 0;
            for (int w = 0; w < BANK_WAVES; ++w) {
                const int64_t u = (per_wave[a][w] + (b >= 0 ? per_wave[b][w] : 0) + BANK_UNIT - 1) / BANK_UNIT;
                units += u;
                most = std::max(most, u);
            }
            if (busiest) *busiest = most;
            return units;
        };
        // a unit takes BANK_UNIT / 8 bytes per row and 4 bytes of child references per slot; the
        // kernel keeps one row of bytes in front of the buffer
        const int64_t budget_units =
            static_cast<int64_t>((BANK_MAX_LDS - BANK_ROWS) / (BANK_ROWS * (BANK_UNIT / 8) + 4 * BANK_UNIT));
        bool fits = true;
        // Which trees share a batch.  Every batch costs the workgroup two barriers and a walk, and
        // its waves wait for the busiest of them, so: as few batches as the buffer allows (largest
        // tree first, paired with one of the largest trees that still fit beside it), and among
        // those candidates the partner that leaves the busiest wave the least to do.  The trees of
        // a model that takes this path all feed the same output columns, so their order only
        // decides the order of the float64 additions.
        static_assert(BANK_TREES == 2, "batches are pairs");
        std::vector<int32_t> by_size(static_cast<size_t>(T));
        std::iota(by_size.begin(), by_size.end(), 0);
        std::stable_sort(by_size.begin(), by_size.end(), [&](int32_t a, int32_t b) {
            return shape[order[a]].internal.size() > shape[order[b]].internal.size();
        });
        std::vector<std::array<int32_t, BANK_TREES>> batches;
        auto pair_trees = [&] {
            count_per_wave();
            batches.clear();
            std::vector<char> taken(static_cast<size_t>(T), 0);
            for (int32_t a : by_size) {
                if (taken[a]) continue;
                taken[a] = 1;
                if (batch_units(a, -1, nullptr) > budget_units) {
                    fits = false;  // a single tree too large for the buffer
                    return;
                }
                int32_t partner = -1, seen = 0;
                int64_t partner_busiest = 0;
                for (int32_t b : by_size) {
                    if (taken[b]) continue;
                    int64_t busiest;
                    if (batch_units(a, b, &busiest) > budget_units) continue;
                    if (partner < 0 || busiest < partner_busiest) {
                        partner = b;
                        partner_busiest = busiest;
                    }
                    if (++seen == 8) break;
                }
                if (partner >= 0) taken[partner] = 1;
                batches.push_back({std::min(a, partner < 0 ? a : partner), partner < 0 ? -1 : std::max(a, partner)});
            }
            std::sort(batches.begin(), batches.end());
        };
        pair_trees();
        // the registers' places inside the banks, the passes and the waves' to-do lists (fast lookups first)
        m.bank_reg.assign(BANK_WAVES * BANK_REGS, 0);
        {
            int32_t held[BANK_WAVES] = {};
            for (const Block &blk : blocks) {
                std::vector<BankTodo> mine[BANK_WAVES][2];
                for (int32_t r = blk.r0; r < blk.r1; ++r) {
                    const int w = reg_wave[r];
                    reg_index[r] = held[w];
                    m.bank_reg[w * BANK_REGS + held[w]] = r;
                    ++held[w];
                    const int32_t f = reg_feature[r];
                    const int32_t n = m.feat_thr_base[f + 1] - m.feat_thr_base[f];
                    const int32_t first = reg_segment[r] * RANK_SEG;
                    const bool fast = n >= FAST_WINDOW && n <= FAST_MAX_THRESHOLDS;  // refined below
                    mine[w][fast ? 0 : 1].push_back(BankTodo{reg_index[r], f, first, std::min<int32_t>(n - first, RANK_SEG)});
                }
                m.bank_pass.push_back(BankPass{blk.f0, blk.f1});
                for (int w = 0; w < BANK_WAVES; ++w) {
                    m.bank_pass_wave.push_back(BankPassWave{static_cast<int32_t>(m.bank_todo.size()),
                                                            static_cast<int32_t>(mine[w][0].size()),
                                                            static_cast<int32_t>(mine[w][1].size()), 0});
                    for (int k = 0; k < 2; ++k) m.bank_todo.insert(m.bank_todo.end(), mine[w][k].begin(), mine[w][k].end());
                }
            }
        }
        // a to-do item is fast only if its feature's table was built
        for (size_t pw = 0; pw < m.bank_pass_wave.size(); ++pw) {
            BankPassWave &q = m.bank_pass_wave[pw];
            std::stable_partition(m.bank_todo.begin() + q.begin, m.bank_todo.begin() + q.begin + q.n_fast + q.n_slow,
                                  [&](const BankTodo &td) { return m.fast_feat[td.feature].fast != 0; });
            const int32_t total = q.n_fast + q.n_slow;
            q.n_fast = static_cast<int32_t>(std::count_if(m.bank_todo.begin() + q.begin, m.bank_todo.begin() + q.begin + total,
                                                          [&](const BankTodo &td) { return m.fast_feat[td.feature].fast != 0; }));
            q.n_slow = total - q.n_fast;
        }
        // Batches of up to BANK_TREES trees whose bit buffer fits the LDS budget.  Inside a batch every
        // wave gets the nodes that test its registers, padded to whole units of BANK_UNIT entries;
        // a node's slot is BANK_UNIT * (index of its unit in the batch's bit buffer) + its bit.
        // The kernel collects the entries of a unit in groups of 8, first entry of a group in bit 7
        // of the group's byte.
        std::vector<std::vector<uint32_t>> stream(BANK_WAVES);
        uint32_t pad32;
        std::memcpy(&pad32, &pad.threshold, sizeof(pad32));
        pad32 &= 0xffff0000u;  // bank register 0 against the largest code: outcome 0
        int64_t max_units = 0;
        struct Node { int32_t tree, ordinal; };
        int32_t n_batches = 0;
        for (size_t bi = 0; bi < batches.size() && fits; ++bi, ++n_batches) {
            const std::array<int32_t, BANK_TREES> &members = batches[bi];
            const int32_t count = members[1] < 0 ? 1 : 2;
            std::vector<Node> mine[BANK_WAVES];
            for (int32_t j = 0; j < count; ++j) {
                const int32_t t = order[members[j]];
                const TreeShape &sh = shape[t];
                for (int32_t i = 0; i < static_cast<int32_t>(sh.internal.size()); ++i)
                    mine[reg_wave[entry_of(t, sh.internal[i]).feature_slot]].push_back(Node{j, i});
            }
            // slots
            std::vector<std::vector<int32_t>> slot_of(BANK_TREES);
            for (int32_t j = 0; j < count; ++j) slot_of[j].assign(shape[order[members[j]]].internal.size(), -1);
            int32_t unit_base = 0;
            for (int w = 0; w < BANK_WAVES; ++w) {
                const int32_t n_units = static_cast<int32_t>((mine[w].size() + BANK_UNIT - 1) / BANK_UNIT);
                m.bank_span.push_back(BankSpan{n_units, unit_base});
                for (int32_t k = 0; k < n_units * BANK_UNIT; ++k) {
                    // entry k of the wave's batch stream fills bit 8 * (group inside the unit) + 7 - k % 8
                    // of unit k / BANK_UNIT
                    const int32_t bit = 8 * ((k >> 3) % (BANK_UNIT / 8)) + 7 - (k & 7);
                    const int32_t local = (k / BANK_UNIT) * BANK_UNIT + bit;  // which of the wave's nodes sits at this entry
                    if (local < static_cast<int32_t>(mine[w].size())) {
                        const Node nd = mine[w][local];
                        const int32_t t = order[members[nd.tree]];
                        const SplitEntry e = entry_of(t, shape[t].internal[nd.ordinal]);
                        uint32_t pair;
                        std::memcpy(&pair, &e.threshold, sizeof(pair));
                        stream[w].push_back((pair & 0xffff0000u) | static_cast<uint32_t>(reg_index[e.feature_slot]));
                        slot_of[nd.tree][nd.ordinal] = (unit_base + k / BANK_UNIT) * BANK_UNIT + bit;
                    } else {
                        stream[w].push_back(pad32);
                    }
                }
                unit_base += n_units;
            }
            max_units = std::max<int64_t>(max_units, unit_base);
            // child references by slot, and the trees' records
            // The walk takes a fixed number of steps: as many as the deepest tree of the batch has
            // internal nodes on a path, less one.  A step moves to the child the outcome bit picks;
            // where that child is a leaf the reference is the slot's own, so the lane stays there,
            // and after the last step the outcome bit of where it stands picks its leaf.
            int32_t steps = 0;
            for (int32_t j = 0; j < count; ++j) steps = std::max(steps, shape[order[members[j]]].depth - 1);
            m.bank_batch.push_back(BankBatch{static_cast<int32_t>(m.bank_child.size()), unit_base * BANK_UNIT, steps, 0});
            const size_t child_at = m.bank_child.size();
            // slots without a node: a word that leads to slot 0 (lanes with nothing to walk start
            // there and must stay inside the buffer)
            m.bank_child.resize(child_at + static_cast<size_t>(unit_base) * BANK_UNIT, 0u);
            m.bank_leaf.resize(child_at + static_cast<size_t>(unit_base) * BANK_UNIT, 0x80008000u);
            for (int32_t j = 0; j < BANK_TREES; ++j) {
                if (j >= count) {
                    m.bank_tree.push_back(BankTree{static_cast<int32_t>(BANK_LEAF_FLAG), 0, 0, 0});
                    continue;
                }
                const int32_t ti = members[j];
                const int32_t t = order[ti];
                const TreeShape &sh = shape[t];
                const TreeMeta &tm = m.tree[ti];
                const int64_t base = d.tree_offset[t];
                if (static_cast<int64_t>(sh.leaves.size()) > static_cast<int64_t>(BANK_LEAF_FLAG)) fits = false;
                // where a step from slot `self` goes for child `caller_node`: the child's slot, or
                // `self` again if the child is a leaf; as the byte offset of the slot's word
                auto next_of = [&](int32_t caller_node, int32_t self) -> uint32_t {
                    const int32_t o = sh.ordinal[caller_node];
                    return 4u * static_cast<uint32_t>(o >= 0 ? slot_of[j][o] : self);
                };
                // the leaf a child is (in-order ordinal inside the tree), 0xffff for an internal child
                auto leaf_of = [&](int32_t caller_node) -> uint32_t {
                    const int32_t o = sh.ordinal[caller_node];
                    return o >= 0 ? 0xffffu : static_cast<uint32_t>(~o) & 0x7fffu;
                };
                for (int32_t i = 0; i < static_cast<int32_t>(sh.internal.size()); ++i) {
                    const int32_t v = sh.internal[i], self = slot_of[j][i];
                    m.bank_child[child_at + self] = next_of(d.left[base + v], self) | (next_of(d.right[base + v], self) << 16);
                    m.bank_leaf[child_at + self] = leaf_of(d.left[base + v]) | (leaf_of(d.right[base + v]) << 16);
                }
                // the root: its slot's byte offset, or, if the tree is one leaf, that leaf
                const int32_t root_ref = sh.internal.empty() ? static_cast<int32_t>(BANK_LEAF_FLAG) : 4 * slot_of[j][0];
                m.bank_tree.push_back(BankTree{root_ref, tm.leaf_base, tm.caller_tree, 1});
            }
        }
        if (fits) {
            m.bank_enabled = 1;
            m.bank_batches = n_batches;
            m.bank_max_units = static_cast<int32_t>(max_units);
            for (int w = 0; w < BANK_WAVES; ++w) {
                m.bank_stream_base[w] = static_cast<int32_t>(m.bank_prog.size());
                m.bank_prog.insert(m.bank_prog.end(), stream[w].begin(), stream[w].end());
                m.bank_prog.insert(m.bank_prog.end(), BANK_PAD_ENTRIES, pad32);
            }
        } else {
            m.bank_child.clear();
            m.bank_leaf.clear();
            m.bank_batch.clear();
            m.bank_tree.clear();
            m.bank_span.clear();
            m.bank_reg.clear();
            m.bank_pass.clear();
            m.bank_pass_wave.clear();
            m.bank_todo.clear();
        }
    }
    for (const TreeMeta &tm : m.tree) m.v_program_groups.push_back(tm.n_words);
    for (size_t ti = 0; ti < m.tree.size(); ++ti) {
        const size_t end = ti + 1 < m.tree.size() ? static_cast<size_t>(m.tree[ti + 1].leaf_base) : m.leaf_node.size();
        m.v_order_leaf_tree.insert(m.v_order_leaf_tree.end(), end - static_cast<size_t>(m.tree[ti].leaf_base),
                                   m.tree[ti].caller_tree);
    }
    m.tree.push_back(TreeMeta{});  // spare record: the stream kernels read the root of "the next tree"
    // Padding: the kernels prefetch (and may evaluate, without using the result) up to eleven
    // groups past the entries of their trees.
    for (int j = 0; j < PROGRAM_PAD_ENTRIES; ++j) m.prog.push_back(pad);
    if (m.path == PATH_RANK || m.path == PATH_RANK_LDS) {
        // compact form: one dword per entry, f16(-j') in the high half.  RANK: rank register in
        // the low byte.  RANK_LDS: rank register in bits 8..15 (its LDS row offset is reg * 256),
        // group flags in the low byte.
        m.prog32.reserve(m.prog.size());
        for (const SplitEntry &e : m.prog) {
            uint32_t pair;
            std::memcpy(&pair, &e.threshold, sizeof(pair));
            const uint32_t reg = static_cast<uint32_t>(e.feature_slot) & 0xffffu;
            const uint32_t flags = static_cast<uint32_t>(e.feature_slot) >> 16;
            m.prog32.push_back((pair & 0xffff0000u) | (m.path == PATH_RANK ? reg : (reg << 8) | flags));
        }
        m.prog.clear();
        m.prog.shrink_to_fit();
    }
    return FOREST_OK;
}

}  // namespace forest_impl
