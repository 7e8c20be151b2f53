// C ABI of the library (see include/forest.h): validation, packing, upload, launch.  The entry
// points that need no device are in forest_api_host.cpp.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <new>

#include "forest_device.hpp"

using namespace forest_impl;

// Small batches cut the trees into shares whose partial sums meet in a workspace.  A handle owns
// WS_SLOTS workspaces.  Work on one stream is ordered, so a stream keeps the slot it was given;
// a stream under graph capture gets a slot for that capture (the graph may be replayed on any
// stream later).  Slots are never handed back before forest_free; a caller that finds none free
// runs its small batch unsplit, which needs no workspace.  So calls on one handle never share
// memory unless they are ordered by their stream, whatever the batch size.
constexpr int WS_SLOTS = 4;

struct SlotOwner {
    bool used = false;
    bool capture = false;            // key is a capture sequence id, else a stream handle
    unsigned long long key = 0;
};

struct forest {
    PackedModel host;  // tables kept for forest_info; large arrays are released after upload
    DevModel dev{};
    void *blob = nullptr;  // one device allocation holding every table and the workspaces
    int64_t blob_bytes = 0;       // packed model
    int64_t workspace_bytes = 0;  // all slots, same allocation
    int device = 0;
    Workspace slot[WS_SLOTS];
    mutable std::mutex slot_mutex;
    mutable SlotOwner owner[WS_SLOTS];
};

namespace {

// Kernel attributes (dynamic LDS sizes) are per device: set once for every device a model is
// loaded on.
constexpr int MAX_DEVICES = 64;
std::mutex g_init_mutex;
bool g_init_done[MAX_DEVICES] = {};
hipError_t g_init_status[MAX_DEVICES] = {};

hipError_t init_device(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_init_mutex);
    if (!g_init_done[device]) {
        g_init_status[device] = init_kernels();
        g_init_done[device] = true;
    }
    return g_init_status[device];
}

template <class T>
size_t place(size_t &cursor, size_t count)
{
    cursor = (cursor + 255) & ~size_t{255};
    const size_t at = cursor;
    cursor += sizeof(T) * (count ? count : 1);
    return at;
}

int check_out_args(const forest *f, int64_t n_rows)
{
    if (!f || n_rows < 0) return FOREST_EINVAL;
    if (n_rows > FOREST_MAX_ROWS) return FOREST_ELIMIT;
    return FOREST_OK;
}

// The workspace slot of the caller's stream (or of the graph capture the stream is in), claiming
// a free one the first time; null when every slot belongs to someone else.
const Workspace *claim_slot(const forest *f, hipStream_t stream)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    unsigned long long id = 0;
    if (hipStreamGetCaptureInfo(stream, &status, &id) != hipSuccess) {
        (void)hipGetLastError();
        status = hipStreamCaptureStatusNone;
    }
    const bool capture = status == hipStreamCaptureStatusActive;
    const unsigned long long key = capture ? id : static_cast<unsigned long long>(reinterpret_cast<uintptr_t>(stream));
    std::lock_guard<std::mutex> lock(f->slot_mutex);
    for (int i = 0; i < WS_SLOTS; ++i)
        if (f->owner[i].used && f->owner[i].capture == capture && f->owner[i].key == key) return &f->slot[i];
    for (int i = 0; i < WS_SLOTS; ++i)
        if (!f->owner[i].used) {
            f->owner[i] = SlotOwner{true, capture, key};
            return &f->slot[i];
        }
    return nullptr;
}

bool small_batch(const forest *f, int64_t n_rows)
{
    return n_rows < SPLIT_BELOW_BLOCKS * static_cast<int64_t>(family_rows_per_block(f->dev));
}

// The handle's tables live on the device it was loaded on.
int check_device(const forest *f)
{
    int current = -1;
    if (hipGetDevice(&current) != hipSuccess) {
        (void)hipGetLastError();
        return FOREST_EHIP;
    }
    return current == f->device ? FOREST_OK : FOREST_EINVAL;
}

}  // namespace

extern "C" {

int forest_load(const forest_desc *desc, forest **out)
{
    if (!desc || !out) return FOREST_EINVAL;
    forest *f = new (std::nothrow) forest;
    if (!f) return FOREST_ENOMEM;
    int rc;
    try {
        rc = compile_forest(*desc, f->host);
    } catch (const std::bad_alloc &) {
        rc = FOREST_ENOMEM;
    }
    if (rc != FOREST_OK) {
        delete f;
        return rc;
    }
    if (!model_fits(f->host)) {
        delete f;
        return FOREST_ELIMIT;
    }
    // Everything below needs a device.
    if (hipGetDevice(&f->device) != hipSuccess || init_device(f->device) != hipSuccess) {
        (void)hipGetLastError();
        delete f;
        return FOREST_EHIP;
    }
    PackedModel &m = f->host;
    size_t cur = 0;
    const size_t o_prog = place<SplitEntry>(cur, m.prog.size());
    const size_t o_prog32 = place<uint32_t>(cur, m.prog32.size());
    const size_t o_child = place<ChildRef>(cur, m.child.size());
    const size_t o_leafv = place<float>(cur, m.leaf_value.size());
    const size_t o_leafn = place<int32_t>(cur, m.leaf_node.size());
    const size_t o_tree = place<TreeMeta>(cur, m.tree.size());
    const size_t o_colt = place<double>(cur, m.col_trees.size());
    const size_t o_base = place<float>(cur, m.base.size());
    const size_t o_thrs = place<float>(cur, m.thr_sorted.size());
    const size_t o_ftb = place<int32_t>(cur, m.feat_thr_base.size());
    const size_t o_fvf = place<int32_t>(cur, m.feat_vfirst.size());
    const size_t o_fbk = place<FeatBucket>(cur, m.feat_bucket.size());
    const size_t o_bst = place<int32_t>(cur, m.bucket_start.size());
    const size_t o_bprog = place<uint32_t>(cur, m.bank_prog.size());
    const size_t o_bchild = place<uint32_t>(cur, m.bank_child.size());
    const size_t o_bleaf = place<uint32_t>(cur, m.bank_leaf.size());
    const size_t o_btree = place<BankTree>(cur, m.bank_tree.size());
    const size_t o_bspan = place<BankSpan>(cur, m.bank_span.size());
    const size_t o_bslot = place<BankBatch>(cur, m.bank_batch.size());
    const size_t o_bpass = place<BankPass>(cur, m.bank_pass.size());
    const size_t o_bpw = place<BankPassWave>(cur, m.bank_pass_wave.size());
    const size_t o_btodo = place<BankTodo>(cur, m.bank_todo.size());
    const size_t o_bfeat = place<FastLookup>(cur, m.fast_feat.size());
    const size_t o_btab = place<uint16_t>(cur, m.fast_tab.size());
    const size_t model_bytes = (cur + 255) & ~size_t{255};
    // workspaces of split launches, not uploaded
    const bool ranks = m.path == PATH_RANK || m.path == PATH_RANK_LDS;
    const size_t slot_bytes = full_workspace_bytes(ranks ? m.rank_regs : 0, m.n_outputs);
    size_t o_slot[WS_SLOTS];
    for (int i = 0; i < WS_SLOTS; ++i) {
        o_slot[i] = place<char>(cur, slot_bytes);
    }
    cur = (cur + 255) & ~size_t{255};
    if (hipMalloc(&f->blob, cur) != hipSuccess) {
        (void)hipGetLastError();
        delete f;
        return FOREST_ENOMEM;
    }
    f->blob_bytes = static_cast<int64_t>(model_bytes);
    f->workspace_bytes = static_cast<int64_t>(cur - model_bytes);
    char *b = static_cast<char *>(f->blob);
    auto up = [&](size_t off, const void *src, size_t bytes) {
        return bytes == 0 || hipMemcpy(b + off, src, bytes, hipMemcpyHostToDevice) == hipSuccess;
    };
    const bool ok = up(o_prog, m.prog.data(), m.prog.size() * sizeof(SplitEntry)) &&
                    up(o_prog32, m.prog32.data(), m.prog32.size() * sizeof(uint32_t)) &&
                    up(o_child, m.child.data(), m.child.size() * sizeof(ChildRef)) &&
                    up(o_leafv, m.leaf_value.data(), m.leaf_value.size() * sizeof(float)) &&
                    up(o_leafn, m.leaf_node.data(), m.leaf_node.size() * sizeof(int32_t)) &&
                    up(o_tree, m.tree.data(), m.tree.size() * sizeof(TreeMeta)) &&
                    up(o_colt, m.col_trees.data(), m.col_trees.size() * sizeof(double)) &&
                    up(o_base, m.base.data(), m.base.size() * sizeof(float)) &&
                    up(o_thrs, m.thr_sorted.data(), m.thr_sorted.size() * sizeof(float)) &&
                    up(o_ftb, m.feat_thr_base.data(), m.feat_thr_base.size() * sizeof(int32_t)) &&
                    up(o_fvf, m.feat_vfirst.data(), m.feat_vfirst.size() * sizeof(int32_t)) &&
                    up(o_fbk, m.feat_bucket.data(), m.feat_bucket.size() * sizeof(FeatBucket)) &&
                    up(o_bst, m.bucket_start.data(), m.bucket_start.size() * sizeof(int32_t)) &&
                    up(o_bprog, m.bank_prog.data(), m.bank_prog.size() * sizeof(uint32_t)) &&
                    up(o_bchild, m.bank_child.data(), m.bank_child.size() * sizeof(uint32_t)) &&
                    up(o_bleaf, m.bank_leaf.data(), m.bank_leaf.size() * sizeof(uint32_t)) &&
                    up(o_btree, m.bank_tree.data(), m.bank_tree.size() * sizeof(BankTree)) &&
                    up(o_bspan, m.bank_span.data(), m.bank_span.size() * sizeof(BankSpan)) &&
                    up(o_bslot, m.bank_batch.data(), m.bank_batch.size() * sizeof(BankBatch)) &&
                    up(o_bpass, m.bank_pass.data(), m.bank_pass.size() * sizeof(BankPass)) &&
                    up(o_bpw, m.bank_pass_wave.data(), m.bank_pass_wave.size() * sizeof(BankPassWave)) &&
                    up(o_btodo, m.bank_todo.data(), m.bank_todo.size() * sizeof(BankTodo)) &&
                    up(o_bfeat, m.fast_feat.data(), m.fast_feat.size() * sizeof(FastLookup)) &&
                    up(o_btab, m.fast_tab.data(), m.fast_tab.size() * sizeof(uint16_t));
    if (!ok) {
        (void)hipGetLastError();
        (void)hipFree(f->blob);
        delete f;
        return FOREST_EHIP;
    }
    DevModel &d = f->dev;
    d.prog = reinterpret_cast<const SplitEntry *>(b + o_prog);
    d.prog32 = reinterpret_cast<const uint32_t *>(b + o_prog32);
    d.child = reinterpret_cast<const ChildRef *>(b + o_child);
    d.leaf_value = reinterpret_cast<const float *>(b + o_leafv);
    d.leaf_node = reinterpret_cast<const int32_t *>(b + o_leafn);
    d.tree = reinterpret_cast<const TreeMeta *>(b + o_tree);
    d.col_trees = reinterpret_cast<const double *>(b + o_colt);
    d.base = reinterpret_cast<const float *>(b + o_base);
    d.n_trees = m.n_trees;
    d.n_features = m.n_features;
    d.n_outputs = m.n_outputs;
    d.leaf_width = m.leaf_width;
    d.aggregate = m.aggregate;
    d.transform = m.transform;
    d.output = m.output;
    d.kind = m.kind;
    d.max_words = m.max_words;
    d.path = m.path;
    d.reg_nv = m.reg_nv;
    d.reg_r = m.reg_r;
    d.rank_regs = m.rank_regs;
    d.lds_waves = m.lds_waves;
    for (int w = 0; w <= RANKLDS_WAVES_WIDE; ++w) d.wave_tree[w] = m.wave_tree[w];
    d.feat_bucket = reinterpret_cast<const FeatBucket *>(b + o_fbk);
    d.bucket_start = reinterpret_cast<const int32_t *>(b + o_bst);
    d.thr_sorted = reinterpret_cast<const float *>(b + o_thrs);
    d.feat_thr_base = reinterpret_cast<const int32_t *>(b + o_ftb);
    d.feat_vfirst = reinterpret_cast<const int32_t *>(b + o_fvf);
    d.bank.prog = reinterpret_cast<const uint32_t *>(b + o_bprog);
    d.bank.child = reinterpret_cast<const uint32_t *>(b + o_bchild);
    d.bank.leaf = reinterpret_cast<const uint32_t *>(b + o_bleaf);
    d.bank.tree = reinterpret_cast<const BankTree *>(b + o_btree);
    d.bank.span = reinterpret_cast<const BankSpan *>(b + o_bspan);
    d.bank.batch = reinterpret_cast<const BankBatch *>(b + o_bslot);
    d.bank.pass = reinterpret_cast<const BankPass *>(b + o_bpass);
    d.bank.pass_wave = reinterpret_cast<const BankPassWave *>(b + o_bpw);
    d.bank.todo = reinterpret_cast<const BankTodo *>(b + o_btodo);
    d.fast_feat = reinterpret_cast<const FastLookup *>(b + o_bfeat);
    d.fast_tab = reinterpret_cast<const uint16_t *>(b + o_btab);
    for (int w = 0; w < BANK_WAVES; ++w) d.bank.stream_base[w] = m.bank_stream_base[w];
    d.bank.batches = m.bank_batches;
    d.bank.max_units = m.bank_max_units;
    d.bank.enabled = m.bank_enabled;
    d.bank.passes = static_cast<int32_t>(m.bank_pass.size());
    d.n_splits = 1;
    d.n_entries = static_cast<int64_t>(m.prog32.size() > m.prog.size() ? m.prog32.size() : m.prog.size());
    d.split_rows = 0;
    d.partial = nullptr;  // set per launch from the workspace in use
    d.partial_capacity = 0;
    d.rank_tiles = nullptr;
    for (int i = 0; i < WS_SLOTS; ++i) f->slot[i] = carve_workspace(d, b + o_slot[i], slot_bytes, SPLIT_BELOW_BLOCKS);
    // the caller-order views are only for forest_pack_view; drop the bulk on the load path
    m.prog = {};
    m.prog32 = {};
    m.bank_prog = {};
    m.bank_child = {};
    m.bank_leaf = {};
    m.child = {};
    m.thr_sorted = {};
    m.v_feature = {};
    m.v_threshold = {};
    m.v_left = {};
    m.v_right = {};
    m.v_leaf_node = {};
    m.v_leaf_value = {};
    *out = f;
    return FOREST_OK;
}

void forest_free(forest *f)
{
    if (!f) return;
    if (f->blob) (void)hipFree(f->blob);
    delete f;
}

int forest_info(const forest *f, forest_info_t *info)
{
    if (!f || !info) return FOREST_EINVAL;
    const PackedModel &m = f->host;
    info->n_trees = m.n_trees;
    info->n_features = m.n_features;
    info->n_outputs = m.n_outputs;
    info->leaf_width = m.leaf_width;
    info->n_internal = m.n_internal;
    info->n_leaves = m.n_leaves;
    info->max_depth = m.max_depth;
    info->kernel_kind = m.kind;
    info->packed_bytes = f->blob_bytes;
    info->x_in_registers = m.x_in_registers;
    info->kernel_path = m.path;
    info->rows_per_workgroup = family_rows_per_block(f->dev);
    info->workspace_bytes = f->workspace_bytes;
    info->small_batch_rows = SPLIT_BELOW_BLOCKS * info->rows_per_workgroup;
    info->workgroup_waves = family_waves_per_block(f->dev);
    info->rank_banks = m.bank_enabled;
    return FOREST_OK;
}

int forest_out_layout(const forest *f, int64_t n_rows, int64_t *scores_offset, int64_t *labels_offset)
{
    if (int rc = check_out_args(f, n_rows)) return rc;
    const int64_t score_bytes = n_rows * f->host.n_outputs * static_cast<int64_t>(sizeof(float));
    int64_t so = -1, lo = -1;
    switch (f->host.output) {
        case FOREST_OUT_SCORES: so = 0; break;
        case FOREST_OUT_LABELS: lo = 0; break;
        default: so = 0; lo = score_bytes; break;
    }
    if (scores_offset) *scores_offset = so;
    if (labels_offset) *labels_offset = lo;
    return FOREST_OK;
}

int64_t forest_out_bytes(const forest *f, int64_t n_rows)
{
    if (int rc = check_out_args(f, n_rows)) return rc;
    const int64_t score_bytes = n_rows * f->host.n_outputs * static_cast<int64_t>(sizeof(float));
    const int64_t label_bytes = n_rows * static_cast<int64_t>(sizeof(int32_t));
    switch (f->host.output) {
        case FOREST_OUT_SCORES: return score_bytes;
        case FOREST_OUT_LABELS: return label_bytes;
        default: return score_bytes + label_bytes;
    }
}

namespace {

// forest_predict and forest_predict_static: argument checks, output layout, launch.
int predict_with(const forest *f, const float *X, int64_t n_rows, void *out, hipStream_t stream, bool use_static)
{
    if (int rc = check_out_args(f, n_rows)) return rc;
    if (n_rows == 0) return FOREST_OK;
    if (!X || !out) return FOREST_EINVAL;
    if (int rc = check_device(f)) return rc;
    int64_t so, lo;
    forest_out_layout(f, n_rows, &so, &lo);
    char *o = static_cast<char *>(out);
    float *scores = so >= 0 ? reinterpret_cast<float *>(o + so) : nullptr;
    int32_t *labels = lo >= 0 ? reinterpret_cast<int32_t *>(o + lo) : nullptr;
    hipError_t e;
    if (use_static) {
        // the whole array is this call's workspace, sized for the batch at hand
        const int64_t rb = family_rows_per_block(f->dev);
        const Workspace ws = carve_workspace(f->dev, static_scratch(f->device), static_scratch_bytes(),
                                             (n_rows + rb - 1) / rb);
        e = launch_predict(f->dev, &ws, true, X, n_rows, scores, labels, nullptr, stream);
        if (e == hipErrorMemoryAllocation) return FOREST_ELIMIT;
    } else {
        const Workspace *ws = small_batch(f, n_rows) ? claim_slot(f, stream) : nullptr;
        e = launch_predict(f->dev, ws, false, X, n_rows, scores, labels, nullptr, stream);
    }
    return e == hipSuccess ? FOREST_OK : FOREST_EHIP;
}

}  // namespace

int forest_predict(const forest *f, const float *X, int64_t n_rows, void *out, void *stream)
{
    return predict_with(f, X, n_rows, out, static_cast<hipStream_t>(stream), false);
}

int forest_predict_static(const forest *f, const float *X, int64_t n_rows, void *out, void *stream)
{
    return predict_with(f, X, n_rows, out, static_cast<hipStream_t>(stream), true);
}

int forest_predict_leaves(const forest *f, const float *X, int64_t n_rows, int32_t *leaf_node_id,
                          void *stream)
{
    if (int rc = check_out_args(f, n_rows)) return rc;
    if (n_rows == 0 || f->host.n_trees == 0) return FOREST_OK;
    if (!X || !leaf_node_id) return FOREST_EINVAL;
    if (int rc = check_device(f)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Workspace *ws = small_batch(f, n_rows) ? claim_slot(f, st) : nullptr;
    const hipError_t e = launch_predict(f->dev, ws, false, X, n_rows, nullptr, nullptr, leaf_node_id, st);
    return e == hipSuccess ? FOREST_OK : FOREST_EHIP;
}

}  // extern "C"
