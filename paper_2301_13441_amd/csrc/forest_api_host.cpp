// The entry points of the C ABI that need no device: the host-only views into the model compiler
// (include/forest_testing.h) and forest_strerror.  Kept free of HIP so that it builds with a plain
// host compiler (the sanitizer test compiles it with forest_pack.cpp under ASan and UBSan).
#include <new>

#include "forest_model.hpp"

using namespace forest_impl;

struct forest_packed {
    PackedModel m;
};

extern "C" {

int forest_pack(const forest_desc *desc, forest_packed **out)
{
    if (!desc || !out) return FOREST_EINVAL;
    forest_packed *p = new (std::nothrow) forest_packed;
    if (!p) return FOREST_ENOMEM;
    int rc;
    try {
        rc = compile_forest(*desc, p->m);
    } catch (const std::bad_alloc &) {
        rc = FOREST_ENOMEM;
    }
    if (rc != FOREST_OK) {
        delete p;
        return rc;
    }
    *out = p;
    return FOREST_OK;
}

int forest_rank_code(int32_t q, uint16_t *code, uint16_t *entry)
{
    if (!code || !entry || q < 0 || q >= RANK_CODES) return FOREST_EINVAL;
    *code = rank_code_bits(q);
    *entry = rank_entry_bits(q);
    return RANK_CODES;
}

int forest_staged_position(int32_t depth, int32_t pos, int32_t *node)
{
    if (!node || depth < STAGED_MIN_DEPTH || depth > STAGED_TOP_MAX_DEPTH || pos < 0 || pos >= (1 << depth))
        return FOREST_EINVAL;
    *node = staged_position_node(depth, pos);
    return FOREST_OK;
}

int forest_pack_view(const forest_packed *p, forest_packed_view *v)
{
    if (!p || !v) return FOREST_EINVAL;
    const PackedModel &m = p->m;
    v->n_trees = m.n_trees;
    v->kernel_kind = m.kind;
    v->kernel_path = m.path;
    v->rank_registers = m.rank_regs;
    v->tree_n_internal = m.v_n_internal.data();
    v->tree_depth = m.v_depth.data();
    v->tree_is_full = m.v_is_full.data();
    v->node_base = m.v_node_base.data();
    v->leaf_base = m.v_leaf_base.data();
    v->split_feature = m.v_feature.data();
    v->split_threshold = m.v_threshold.data();
    v->child_left = m.v_left.data();
    v->child_right = m.v_right.data();
    v->leaf_node = m.v_leaf_node.data();
    v->leaf_value = m.v_leaf_value.data();
    const bool ranks = m.path == PATH_RANK || m.path == PATH_RANK_LDS;
    static_assert(sizeof(forest_rank_bucket) == sizeof(FeatBucket), "same four fields");
    v->rank_threshold = ranks ? m.thr_sorted.data() : nullptr;
    v->rank_threshold_base = ranks ? m.feat_thr_base.data() : nullptr;
    v->rank_bucket = ranks ? reinterpret_cast<const forest_rank_bucket *>(m.feat_bucket.data()) : nullptr;
    v->rank_bucket_start = ranks ? m.bucket_start.data() : nullptr;
    v->workgroup_waves = m.path == PATH_RANK_LDS ? m.lds_waves : 0;
    v->wave_tree = m.path == PATH_RANK_LDS ? m.wave_tree : nullptr;
    v->program_groups = m.path == PATH_RANK_LDS ? m.v_program_groups.data() : nullptr;
    const bool bank = m.bank_enabled != 0;
    static_assert(sizeof(BankSpan) == 2 * sizeof(int32_t) && sizeof(BankTree) == 4 * sizeof(int32_t) &&
                      sizeof(BankBatch) == 4 * sizeof(int32_t), "viewed as plain int32 arrays");
    v->bank_batches = bank ? m.bank_batches : 0;
    v->bank_waves = BANK_WAVES;
    v->bank_regs = BANK_REGS;
    v->bank_trees = BANK_TREES;
    v->bank_max_units = bank ? m.bank_max_units : 0;
    v->bank_unit = BANK_UNIT;
    v->bank_prog_entries = bank ? static_cast<int64_t>(m.bank_prog.size()) : 0;
    v->bank_prog = bank ? m.bank_prog.data() : nullptr;
    v->bank_stream_base = bank ? m.bank_stream_base : nullptr;
    v->bank_span = bank ? reinterpret_cast<const int32_t *>(m.bank_span.data()) : nullptr;
    v->bank_child = bank ? m.bank_child.data() : nullptr;
    v->bank_leaf = bank ? m.bank_leaf.data() : nullptr;
    v->bank_batch = bank ? reinterpret_cast<const int32_t *>(m.bank_batch.data()) : nullptr;
    v->bank_tree = bank ? reinterpret_cast<const int32_t *>(m.bank_tree.data()) : nullptr;
    v->bank_reg = bank ? m.bank_reg.data() : nullptr;
    static_assert(sizeof(BankPass) == 2 * sizeof(int32_t) && sizeof(BankPassWave) == 4 * sizeof(int32_t) &&
                      sizeof(BankTodo) == 4 * sizeof(int32_t) && sizeof(FastLookup) == 8 * sizeof(uint32_t),
                  "viewed as plain 32-bit arrays");
    v->bank_passes = bank ? static_cast<int32_t>(m.bank_pass.size()) : 0;
    v->fast_window = FAST_WINDOW;
    v->bank_todo_items = bank ? static_cast<int64_t>(m.bank_todo.size()) : 0;
    v->fast_tab_entries = ranks ? static_cast<int64_t>(m.fast_tab.size()) : 0;
    v->bank_pass = bank ? reinterpret_cast<const int32_t *>(m.bank_pass.data()) : nullptr;
    v->bank_pass_wave = bank ? reinterpret_cast<const int32_t *>(m.bank_pass_wave.data()) : nullptr;
    v->bank_todo = bank ? reinterpret_cast<const int32_t *>(m.bank_todo.data()) : nullptr;
    v->fast_feat = ranks ? reinterpret_cast<const uint32_t *>(m.fast_feat.data()) : nullptr;
    v->fast_tab = ranks ? m.fast_tab.data() : nullptr;
    v->order_leaf_node = m.leaf_node.data();
    v->order_leaf_tree = m.v_order_leaf_tree.data();
    return FOREST_OK;
}

void forest_pack_free(forest_packed *p) { delete p; }

const char *forest_strerror(int code)
{
    switch (code) {
        case FOREST_OK: return "ok";
        case FOREST_EINVAL: return "invalid argument";
        case FOREST_ETREE: return "malformed tree";
        case FOREST_EFEATURE: return "split feature out of range";
        case FOREST_ENONFINITE: return "NaN threshold or base score";
        case FOREST_ENOMEM: return "out of memory";
        case FOREST_EHIP: return "HIP runtime error";
        case FOREST_ELIMIT: return "model exceeds a kernel limit";
        default: return "unknown error";
    }
}

}  // extern "C"
