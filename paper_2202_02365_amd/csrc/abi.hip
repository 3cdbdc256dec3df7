// The C ABI of libdense_mi355x.so: argument checking, handle bookkeeping, workspace carve-up.
// Every step of the hot path runs in the kernels behind the dn_launch_* calls.
#include "dn_internal.h"
#include <chrono>
#include <cstdlib>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <algorithm>
#include <map>
#include <mutex>
#include <string>
#include <vector>

namespace {

thread_local char g_err[512] = "";

using Carver = dn_carver;

int fill_batch_caps(dn_batch* b, int64_t V, int32_t max_targets, int32_t k, const int32_t* fanouts, int32_t direction)
{
    if (V < 1 || V > 0x7fffffffLL) return dn_fail(DN_EINVAL, "num_nodes must be in [1, 2^31)");
    if (k < 1 || k > DN_MAX_LAYERS) return dn_fail(DN_EINVAL, "k must be in [1, %d]", DN_MAX_LAYERS);
    if (!fanouts) return dn_fail(DN_EINVAL, "fanouts is null");
    if (max_targets < 1) return dn_fail(DN_EINVAL, "max_targets must be positive");
    if (direction < DN_DIR_OUT || direction > DN_DIR_BOTH) return dn_fail(DN_EINVAL, "direction must be 0, 1 or 2");
    const int mult = direction == DN_DIR_BOTH ? 2 : 1;
    std::memset(b, 0, sizeof(*b));
    if (max_targets > V) max_targets = (int32_t)V;          // targets are pairwise distinct
    b->V = V; b->k = k; b->direction = direction; b->max_targets = max_targets;
    b->cap_level[0] = max_targets;
    b->cap_nodes = b->cap_level[0];
    b->cap_slots = 0;
    for (int h = 0; h < k; ++h) {
        if (fanouts[h] < 1 || fanouts[h] > DN_MAX_FANOUT)
            return dn_fail(DN_EINVAL, "fanouts[%d] = %d is outside [1, %d]", h, fanouts[h], DN_MAX_FANOUT);
        b->fanouts[h] = fanouts[h];
        b->cap_slots_hop[h] = b->cap_level[h] * fanouts[h] * mult;
        b->cap_slots += b->cap_slots_hop[h];
        b->cap_level[h + 1] = b->cap_slots_hop[h] < V ? b->cap_slots_hop[h] : V;
        b->cap_nodes += b->cap_level[h + 1];
    }
    if (b->cap_nodes > V) b->cap_nodes = V;
    if (b->cap_slots > 0x7fffff00LL) return dn_fail(DN_ECAPACITY, "more than 2^31 neighbour slots per batch");
    b->words0 = (V + 31) / 32;
    b->words1 = (b->words0 + 31) / 32;
    // a walker of the next-Delta kernels takes a whole summary word (32 bitmap words) unless that leaves fewer than 64k walkers
    b->walk_shift = 5;
    while (b->walk_shift > 0 && (b->words0 >> b->walk_shift) < 65536) --b->walk_shift;
    const int64_t walkers = (b->words0 + ((int64_t)1 << b->walk_shift) - 1) >> b->walk_shift;
    const int64_t blocks_words = (walkers + 255) / 256, blocks_targets = (max_targets + 255) / 256;
    b->max_blocks = (int32_t)(blocks_words > blocks_targets ? blocks_words : blocks_targets);
    return DN_OK;
}

// sample_only: no transpose index (the arrays of the backward pass stay null) and the four big DENSE arrays are
// not carved: the caller of carve_batch points them at buffers of its own.
void carve_batch(dn_batch* b, Carver& c, bool sample_only = false)
{
    b->hdr = c.take<int32_t>(DN_HDR_WORDS);
    b->seen = c.take<uint32_t>(2 * b->words0);     // word pairs (seen, fresh), see sample.hip
    b->fresh = b->seen + 1;
    b->summary = c.take<uint32_t>(b->words1);
    b->tr_hist_words = sample_only ? 0 : dn_transpose_index_hist_words(b);
    b->tr_hist = c.take<int32_t>(b->tr_hist_words);          // starts at zero like the bitmaps
    b->lvlpos = c.take<int32_t>(b->V);
    b->lvl_ids = c.take<int32_t>(b->cap_nodes);
    b->lvl_nbr_offsets = c.take<int32_t>(b->cap_nodes + 1);
    b->lvl_nbrs = c.take<int32_t>(b->cap_slots);
    b->lvl_owner = c.take<int32_t>(b->cap_slots);
    b->blk_a = c.take<int32_t>(2 * (int64_t)b->max_blocks + 2);    // used as uint64[max_blocks]
    b->blk_b = nullptr;
    b->slot_owner = c.take<int32_t>(b->cap_slots);
    if (sample_only) return;
    b->node_ids = c.take<int32_t>(b->cap_nodes);
    b->nbr_offsets = c.take<int32_t>(b->cap_nodes + 1);
    b->nbrs = c.take<int32_t>(b->cap_slots);
    b->repr_map = c.take<int32_t>(b->cap_slots);
    for (int i = 0; i < 2; ++i) {
        b->tr_key[i] = c.take<int32_t>(b->cap_slots);
        b->tr_val[i] = c.take<int32_t>(b->cap_slots);
    }
    b->tr_ptr = c.take<int32_t>(b->cap_nodes + 2);
    b->tr_own = c.take<int32_t>(b->cap_slots);
    b->tr_inv = c.take<float>(b->cap_slots);
    b->tr_long_words = b->cap_slots / DN_LONG_GROUP + 2;
    b->tr_long = c.take<int32_t>(b->tr_long_words);
}

int fill_model(dn_model* m, const dn_batch* b, int32_t k, const int32_t* dims, int32_t in_dtype)
{
    if (!b) return dn_fail(DN_EINVAL, "batch is null");
    if (k != b->k) return dn_fail(DN_EINVAL, "model has %d layers, the batch samples %d hops", k, b->k);
    if (!dims) return dn_fail(DN_EINVAL, "dims is null");
    if (in_dtype != DN_F32 && in_dtype != DN_BF16) return dn_fail(DN_EINVAL, "in_dtype must be DN_F32 or DN_BF16");
    std::memset(m, 0, sizeof(*m));
    m->k = k; m->in_dtype = in_dtype;
    for (int i = 0; i <= k; ++i) {
        if (dims[i] < 1 || dims[i] > 16384) return dn_fail(DN_EINVAL, "dims[%d] = %d is outside [1, 16384]", i, dims[i]);
        m->dims[i] = dims[i];
    }
    // rows of layer i = nodes of Delta_i .. Delta_k = levels 0 .. k-i
    for (int i = 1; i <= k; ++i) {
        dn_layer_bufs& L = m->layer[i - 1];
        L.d_in = dims[i - 1]; L.d_out = dims[i];
        L.xterms = i == 1 ? 1 : 2;
        L.zterms = i == k ? 1 : 2;
        L.kx = 2 * L.d_in * L.xterms;
        L.kp = (int32_t)dn_round_up(L.kx, 64);
        L.np = (int32_t)dn_round_up(L.d_out, 64);
        L.nz = L.np * L.zterms;
        int64_t rows = 0;
        for (int h = 0; h <= k - i; ++h) rows += b->cap_level[h];
        if (rows > b->V) rows = b->V;
        L.rows_cap = rows;
        L.rows_pad = dn_round_up(rows, 128);
    }
    return DN_OK;
}

void carve_model(dn_model* m, const dn_batch* b, Carver& c)
{
    const int k = m->k;
    int64_t max_dx = 0;
    m->splits = 64;
    for (int i = 1; i <= k; ++i) {
        dn_layer_bufs& L = m->layer[i - 1];
        L.x = c.take<dn_bf16>(L.rows_pad * L.kp);
        L.h = (i < k) ? c.take<float>(L.rows_pad * L.d_out) : nullptr;
        L.wt = c.take<dn_bf16>(dn_round_up(L.d_out, 128) * L.kp);
        L.w = c.take<dn_bf16>(dn_round_up(2 * (int64_t)L.d_in, 128) * L.nz);
        L.wf = (L.xterms == 2 && L.d_in % 16 == 0) ? c.take<dn_bf16>((int64_t)L.np * 2 * L.d_in) : nullptr;
        L.bias = c.take<float>(L.d_out);
        L.rownorm = c.take<float>(L.rows_pad);
        L.colnorm = c.take<float>(L.d_out);
        L.dzb = c.take<dn_bf16>(L.rows_pad * L.nz);
        L.partial_floats = (int64_t)m->splits * L.kx * L.d_out * L.zterms;
        L.partial = c.take<float>(L.partial_floats);
        // bias-gradient partials: one row per split from the weight-gradient GEMM; the last layer's come from
        // its dZ kernel, one row per row tile
        L.db_partial = c.take<float>((i < k ? (int64_t)m->splits * L.zterms : (L.rows_cap + 63) / 64 + 1) * L.d_out);
        max_dx = std::max<int64_t>(max_dx, L.rows_pad * 2 * L.d_in);
    }
    m->dx = c.take<float>(max_dx);
    m->fix_count = c.take<int32_t>(DN_FIX_WORDS);
    m->zero_row = c.take<float>(DN_ZERO_ROW_FLOATS);
    (void)b;
}

}  // namespace

namespace {
struct ProfRecord { std::string tag; hipEvent_t start, stop; };
std::mutex g_prof_mutex;
bool g_prof_on = false;
std::vector<ProfRecord> g_prof_records;
std::vector<hipEvent_t> g_prof_pool;

hipEvent_t prof_event()
{
    if (!g_prof_pool.empty()) { hipEvent_t e = g_prof_pool.back(); g_prof_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
void prof_clear()
{
    for (auto& r : g_prof_records) { g_prof_pool.push_back(r.start); g_prof_pool.push_back(r.stop); }
    g_prof_records.clear();
}
}  // namespace

dn_prof_scope::dn_prof_scope(const char* tag, int layer, hipStream_t stream) : idx(-1), st(stream)
{
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    ProfRecord r;
    r.tag = tag;
    if (layer > 0) r.tag += "_L" + std::to_string(layer);
    r.start = prof_event();
    r.stop = prof_event();
    if (!r.start || !r.stop) return;
    if (hipEventRecord(r.start, st) != hipSuccess) return;
    idx = (int)g_prof_records.size();
    g_prof_records.push_back(r);
}

dn_prof_scope::~dn_prof_scope()
{
    if (idx < 0) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (idx < (int)g_prof_records.size()) (void)hipEventRecord(g_prof_records[idx].stop, st);
}

int dn_fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" {

const char* dn_last_error(void) { return g_err; }

int dn_graph_create(dn_graph** out, int64_t num_nodes, const int64_t* d_rowptr_out, const int32_t* d_col_out,
                    const int64_t* d_rowptr_in, const int32_t* d_col_in)
{
    if (!out) return dn_fail(DN_EINVAL, "out is null");
    if (num_nodes < 1 || num_nodes > 0x7fffffffLL) return dn_fail(DN_EINVAL, "num_nodes must be in [1, 2^31)");
    if (!d_rowptr_out && !d_rowptr_in) return dn_fail(DN_EINVAL, "no adjacency given");
    if ((d_rowptr_out && !d_col_out) || (d_rowptr_in && !d_col_in)) return dn_fail(DN_EINVAL, "rowptr without col");
    dn_graph* g = new (std::nothrow) dn_graph;
    if (!g) return dn_fail(DN_EINVAL, "out of host memory");
    g->V = num_nodes;
    g->rowptr[0] = d_rowptr_out; g->col[0] = d_col_out;
    g->rowptr[1] = d_rowptr_in;  g->col[1] = d_col_in;
    *out = g;
    return DN_OK;
}

void dn_graph_destroy(dn_graph* g) { delete g; }

int dn_batch_workspace_size(int64_t num_nodes, int32_t max_targets, int32_t k, const int32_t* fanouts,
                            int32_t direction, size_t* bytes)
{
    if (!bytes) return dn_fail(DN_EINVAL, "bytes is null");
    dn_batch tmp;
    int rc = fill_batch_caps(&tmp, num_nodes, max_targets, k, fanouts, direction);
    if (rc) return rc;
    Carver c(nullptr);
    carve_batch(&tmp, c);
    *bytes = c.bytes();
    return DN_OK;
}

int dn_batch_create(dn_batch** out, int64_t num_nodes, int32_t max_targets, int32_t k, const int32_t* fanouts,
                    int32_t direction, void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!out) return dn_fail(DN_EINVAL, "out is null");
    if (!d_workspace || ((uintptr_t)d_workspace & 255)) return dn_fail(DN_EINVAL, "workspace must be non-null and 256-byte aligned");
    dn_batch* b = new (std::nothrow) dn_batch;
    if (!b) return dn_fail(DN_EINVAL, "out of host memory");
    int rc = fill_batch_caps(b, num_nodes, max_targets, k, fanouts, direction);
    if (rc) { delete b; return rc; }
    Carver c(d_workspace);
    carve_batch(b, c);
    if (c.bytes() > workspace_bytes) {
        delete b;
        return dn_fail(DN_ECAPACITY, "workspace has %zu bytes, %zu needed", workspace_bytes, c.bytes());
    }
    b->workspace_bytes = c.bytes();
    hipStream_t st = static_cast<hipStream_t>(stream);
    // header, the three bitmaps and the sort histograms are contiguous at the front: they must start at zero
    const size_t zero_bytes = (size_t)(reinterpret_cast<char*>(b->lvlpos) - reinterpret_cast<char*>(b->hdr));
    hipError_t e = hipMemsetAsync(b->hdr, 0, zero_bytes, st);
    if (e != hipSuccess) { delete b; return dn_fail(DN_EHIP, "hipMemsetAsync: %s", hipGetErrorString(e)); }
    b->sample_serial = 0;
    b->tr_serial = ~0ull;
    b->tr_capture_serial = ~0ull;
    b->seen_slots_all = b->seen_slots_upper = -1;
    *out = b;
    return DN_OK;
}

void dn_batch_destroy(dn_batch* b) { delete b; }

int dn_batch_capacity(const dn_batch* b, int64_t* node_capacity, int64_t* slot_capacity)
{
    if (!b) return dn_fail(DN_EINVAL, "batch is null");
    if (node_capacity) *node_capacity = b->cap_nodes;
    if (slot_capacity) *slot_capacity = b->cap_slots;
    return DN_OK;
}

int dense_sample(dn_batch* b, const dn_graph* g, const int32_t* d_targets, int32_t n_targets, uint64_t seed, void* stream)
{
    if (!b || !g) return dn_fail(DN_EINVAL, "batch or graph is null");
    if (g->V != b->V) return dn_fail(DN_EINVAL, "graph has %lld nodes, the batch was created for %lld", (long long)g->V, (long long)b->V);
    if (n_targets < 0 || n_targets > b->max_targets)
        return dn_fail(DN_ECAPACITY, "n_targets = %d is outside [0, %d]", n_targets, b->max_targets);
    if (n_targets > 0 && !d_targets) return dn_fail(DN_EINVAL, "d_targets is null");
    if (b->direction != DN_DIR_IN && !g->rowptr[0]) return dn_fail(DN_EINVAL, "the graph has no out-edge adjacency");
    if (b->direction != DN_DIR_OUT && !g->rowptr[1]) return dn_fail(DN_EINVAL, "the graph has no in-edge adjacency");
    b->n_targets = n_targets;
    b->sample_serial += 1;
    return dn_launch_sample(b, g, d_targets, n_targets, seed, static_cast<hipStream_t>(stream));
}

int dense_sample_edges(dn_batch* b, const dn_graph* g, const int32_t* d_src, const int32_t* d_dst, int32_t n_edges,
                       const int32_t* d_neg, int32_t n_neg, uint64_t seed, int32_t* d_src_local, int32_t* d_dst_local,
                       int32_t* d_neg_local, void* stream)
{
    if (!b || !g) return dn_fail(DN_EINVAL, "batch or graph is null");
    if (g->V != b->V) return dn_fail(DN_EINVAL, "graph has %lld nodes, the batch was created for %lld", (long long)g->V, (long long)b->V);
    if (n_edges < 0 || n_neg < 0) return dn_fail(DN_EINVAL, "negative count");
    if ((n_edges > 0 && (!d_src || !d_dst || !d_src_local || !d_dst_local)) || (n_neg > 0 && (!d_neg || !d_neg_local)))
        return dn_fail(DN_EINVAL, "null id or output array");
    const int64_t bound = 2 * (int64_t)n_edges + n_neg;
    if (bound > b->max_targets)
        return dn_fail(DN_ECAPACITY, "2 * n_edges + n_neg = %lld exceeds the batch's %d targets", (long long)bound, b->max_targets);
    if (b->direction != DN_DIR_IN && !g->rowptr[0]) return dn_fail(DN_EINVAL, "the graph has no out-edge adjacency");
    if (b->direction != DN_DIR_OUT && !g->rowptr[1]) return dn_fail(DN_EINVAL, "the graph has no in-edge adjacency");
    b->n_targets = (int32_t)bound;
    b->sample_serial += 1;
    return dn_launch_sample_edges(b, g, d_src, d_dst, n_edges, d_neg, n_neg, seed, d_src_local, d_dst_local, d_neg_local,
                                  static_cast<hipStream_t>(stream));
}

int dn_embedding_sgd(const dn_batch* b, float* d_table, int32_t dim, int64_t ld_elems, const float* d_dH0, float lr, void* stream)
{
    if (!b || !d_table || !d_dH0) return dn_fail(DN_EINVAL, "null argument");
    if (dim < 1 || ld_elems < dim) return dn_fail(DN_EINVAL, "dim = %d, ld_elems = %lld", dim, (long long)ld_elems);
    if (b->sample_serial == 0) return dn_fail(DN_ESTATE, "dense_sample has not run on this batch");
    return dn_launch_embedding_sgd(b, d_table, dim, ld_elems, d_dH0, lr, static_cast<hipStream_t>(stream));
}

int dn_embedding_adagrad(const dn_batch* b, float* d_table, float* d_state, int32_t dim, int64_t ld_elems,
                         const float* d_dH0, float lr, float eps, void* stream)
{
    if (!b || !d_table || !d_state || !d_dH0) return dn_fail(DN_EINVAL, "null argument");
    if (dim < 1 || ld_elems < dim) return dn_fail(DN_EINVAL, "dim = %d, ld_elems = %lld", dim, (long long)ld_elems);
    if (b->sample_serial == 0) return dn_fail(DN_ESTATE, "dense_sample has not run on this batch");
    return dn_launch_embedding_adagrad(b, d_table, d_state, dim, ld_elems, d_dH0, lr, eps, static_cast<hipStream_t>(stream));
}

int dn_softmax_xent(const float* d_logits, int64_t ld_logits, const int32_t* d_labels, int64_t n, int32_t num_classes,
                    float grad_scale, float* d_loss, float* d_grad, int64_t ld_grad, void* stream)
{
    if (n < 0 || num_classes < 1) return dn_fail(DN_EINVAL, "n = %lld, num_classes = %d", (long long)n, num_classes);
    if (n > 0 && (!d_logits || !d_labels || !d_loss || !d_grad)) return dn_fail(DN_EINVAL, "null argument");
    if (ld_logits < num_classes || ld_grad < num_classes) return dn_fail(DN_EINVAL, "row stride below num_classes");
    return dn_launch_softmax_xent(d_logits, ld_logits, d_labels, n, num_classes, grad_scale, d_loss, d_grad, ld_grad,
                                  static_cast<hipStream_t>(stream));
}

int dn_batch_prepare_backward(dn_batch* b, int32_t need_input_grad, void* stream)
{
    if (!b) return dn_fail(DN_EINVAL, "batch is null");
    if (b->sample_serial == 0) return dn_fail(DN_ESTATE, "dense_sample has not run on this batch");
    return dn_launch_transpose_index(b, need_input_grad != 0, static_cast<hipStream_t>(stream));
}

int dn_batch_view(const dn_batch* b, dn_dense_view* view)
{
    if (!b || !view) return dn_fail(DN_EINVAL, "batch or view is null");
    view->d_node_id_offsets = b->hdr + HDR_NODE_OFF;
    view->d_node_ids = b->node_ids;
    view->d_nbr_offsets = b->nbr_offsets;
    view->d_nbrs = b->nbrs;
    view->d_repr_map = b->repr_map;
    return DN_OK;
}

int dn_batch_counts(const dn_batch* b, int64_t* host_counts, void* stream)
{
    if (!b || !host_counts) return dn_fail(DN_EINVAL, "batch or host_counts is null");
    if (b->sample_serial == 0) return dn_fail(DN_ESTATE, "dense_sample has not run on this batch");
    int32_t h[DN_HDR_WORDS];
    hipStream_t st = static_cast<hipStream_t>(stream);
    DN_HIP(hipMemcpyAsync(h, b->hdr, sizeof(h), hipMemcpyDeviceToHost, st));
    DN_HIP(hipStreamSynchronize(st));
    for (int j = 0; j <= b->k + 1; ++j) host_counts[j] = h[HDR_NODE_OFF + j];
    host_counts[b->k + 2] = h[HDR_E];
    // slots of the hops before the last = slots owned by Delta_2 .. Delta_k (what the layers above the first aggregate)
    const int64_t upper = b->k >= 2 ? h[HDR_LVL_NBR_OFF + b->k - 1] : 0;
    if (h[HDR_E] > b->seen_slots_all) b->seen_slots_all = h[HDR_E];
    if (upper > b->seen_slots_upper) b->seen_slots_upper = upper;
    if (h[HDR_STATUS] & (ST_BAD_TARGET | ST_DUP_TARGET))
        return dn_fail(DN_ESAMPLE, "dense_sample: %s", (h[HDR_STATUS] & ST_BAD_TARGET) ? "target id out of range" : "duplicate target id");
    if (h[HDR_STATUS] & ST_CAPACITY) return dn_fail(DN_ECAPACITY, "dense_sample: node capacity exceeded");
    if (h[HDR_STATUS] & ST_INTERNAL)
        return dn_fail(DN_ESTATE, "dense_sample: a workgroup gave up waiting for the totals of the workgroups in front of it; "
                       "the sample is incomplete");
    if (h[HDR_STATUS] & ST_STALE_INDEX)
        return dn_fail(DN_ESTATE, "sage_backward ran with a transpose index built for another sample of this batch (a captured "
                       "graph replayed without the dn_batch_prepare_backward it was captured after); its gradients were not computed");
    return DN_OK;
}

int dense_gather(const dn_batch* b, const void* d_table, int32_t dtype, int32_t dim, int64_t ld_elems, void* d_H0, void* stream)
{
    if (!b || !d_table || !d_H0) return dn_fail(DN_EINVAL, "null argument");
    if (dtype != DN_F32 && dtype != DN_BF16) return dn_fail(DN_EINVAL, "dtype must be DN_F32 or DN_BF16");
    if (dim < 1 || ld_elems < dim) return dn_fail(DN_EINVAL, "dim = %d, ld_elems = %lld", dim, (long long)ld_elems);
    if (b->sample_serial == 0) return dn_fail(DN_ESTATE, "dense_sample has not run on this batch");
    return dn_launch_gather(b, d_table, dtype, dim, ld_elems, d_H0, static_cast<hipStream_t>(stream));
}

int dn_model_workspace_size(const dn_batch* b, int32_t k, const int32_t* dims, int32_t in_dtype, size_t* bytes)
{
    if (!bytes) return dn_fail(DN_EINVAL, "bytes is null");
    dn_model tmp;
    int rc = fill_model(&tmp, b, k, dims, in_dtype);
    if (rc) return rc;
    Carver c(nullptr);
    carve_model(&tmp, b, c);
    *bytes = c.bytes();
    return DN_OK;
}

int dn_model_create(dn_model** out, const dn_batch* b, int32_t k, const int32_t* dims, int32_t in_dtype,
                    void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!out) return dn_fail(DN_EINVAL, "out is null");
    if (!d_workspace || ((uintptr_t)d_workspace & 255)) return dn_fail(DN_EINVAL, "workspace must be non-null and 256-byte aligned");
    dn_model* m = new (std::nothrow) dn_model;
    if (!m) return dn_fail(DN_EINVAL, "out of host memory");
    int rc = fill_model(m, b, k, dims, in_dtype);
    if (rc) { delete m; return rc; }
    Carver c(d_workspace);
    carve_model(m, b, c);
    if (c.bytes() > workspace_bytes) {
        delete m;
        return dn_fail(DN_ECAPACITY, "workspace has %zu bytes, %zu needed", workspace_bytes, c.bytes());
    }
    m->workspace_bytes = c.bytes();
    // padding rows/columns of the bf16 operands must be zero and stay zero
    hipError_t e = hipMemsetAsync(d_workspace, 0, c.bytes(), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) { delete m; return dn_fail(DN_EHIP, "hipMemsetAsync: %s", hipGetErrorString(e)); }
    m->fwd_serial = ~0ull;
    m->mean_agg = 1;
    *out = m;
    return DN_OK;
}

int dn_model_set_weights(dn_model* m, const float* const* d_w_self, const float* const* d_w_nbr,
                         const float* const* d_bias, void* stream)
{
    if (!m || !d_w_self || !d_w_nbr || !d_bias) return dn_fail(DN_EINVAL, "null argument");
    for (int i = 0; i < m->k; ++i)
        if (!d_w_self[i] || !d_w_nbr[i] || !d_bias[i]) return dn_fail(DN_EINVAL, "weights of layer %d are null", i + 1);
    int rc = dn_launch_set_weights(m, d_w_self, d_w_nbr, d_bias, static_cast<hipStream_t>(stream));
    if (rc == DN_OK) m->weights_set = 1;
    return rc;
}

void dn_model_destroy(dn_model* m) { delete m; }

int dn_model_status(const dn_model* m, int32_t* status, void* stream)
{
    if (!m || !status) return dn_fail(DN_EINVAL, "null argument");
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t words[DN_FIX_WORDS];
    DN_HIP(hipMemcpyAsync(words, m->fix_count, sizeof(words), hipMemcpyDeviceToHost, st));
    DN_HIP(hipStreamSynchronize(st));
    int32_t total = 0;
    for (int j = 0; j < DN_FIX_SLOTS; ++j) total += words[DN_FIX_FIRST + DN_FIX_STRIDE * j];
    status[0] = total;
    status[1] = words[1];
    return DN_OK;
}

int sage_forward(dn_model* m, const dn_batch* b, const void* d_H0, float* d_out, void* stream)
{
    if (!m || !b || !d_H0 || !d_out) return dn_fail(DN_EINVAL, "null argument");
    if (!m->weights_set) return dn_fail(DN_ESTATE, "dn_model_set_weights has not been called");
    if (b->sample_serial == 0) return dn_fail(DN_ESTATE, "dense_sample has not run on this batch");
    if (m->k != b->k) return dn_fail(DN_EINVAL, "model and batch disagree on the number of layers");
    for (int i = 1; i <= m->k; ++i) {
        int64_t rows = 0;
        for (int h = 0; h <= b->k - i; ++h) rows += b->cap_level[h];
        if (rows > b->V) rows = b->V;
        if (rows > m->layer[i - 1].rows_cap) return dn_fail(DN_ECAPACITY, "the model was created for a smaller batch capacity");
    }
    int rc = dn_launch_forward(m, b, d_H0, m->dims[0], 0, d_out, static_cast<hipStream_t>(stream));
    if (rc == DN_OK) { m->fwd_serial = b->sample_serial; m->h0 = d_H0; }
    return rc;
}

int sage_forward_table(dn_model* m, const dn_batch* b, const void* d_table, int64_t ld_elems, float* d_out, void* stream)
{
    if (!m || !b || !d_table || !d_out) return dn_fail(DN_EINVAL, "null argument");
    if (!m->weights_set) return dn_fail(DN_ESTATE, "dn_model_set_weights has not been called");
    if (b->sample_serial == 0) return dn_fail(DN_ESTATE, "dense_sample has not run on this batch");
    if (m->k != b->k) return dn_fail(DN_EINVAL, "model and batch disagree on the number of layers");
    if (ld_elems < m->dims[0]) return dn_fail(DN_EINVAL, "row stride below the input width");
    for (int i = 1; i <= m->k; ++i) {
        int64_t rows = 0;
        for (int h = 0; h <= b->k - i; ++h) rows += b->cap_level[h];
        if (rows > b->V) rows = b->V;
        if (rows > m->layer[i - 1].rows_cap) return dn_fail(DN_ECAPACITY, "the model was created for a smaller batch capacity");
    }
    int rc = dn_launch_forward(m, b, d_table, ld_elems, 1, d_out, static_cast<hipStream_t>(stream));
    if (rc == DN_OK) { m->fwd_serial = b->sample_serial; m->h0 = nullptr; }
    return rc;
}

int dn_model_set_aggregation(dn_model* m, int32_t aggregation)
{
    if (!m) return dn_fail(DN_EINVAL, "model is null");
    if (aggregation != DN_AGG_MEAN && aggregation != DN_AGG_SUM) return dn_fail(DN_EINVAL, "aggregation must be DN_AGG_MEAN or DN_AGG_SUM");
    m->mean_agg = aggregation == DN_AGG_MEAN ? 1 : 0;
    m->fwd_serial = ~0ull;            // activations saved under the other rule no longer fit
    return DN_OK;
}

int sage_backward(dn_model* m, const dn_batch* b, const float* d_grad_out, float* const* d_dw_self,
                  float* const* d_dw_nbr, float* const* d_dbias, float* d_dH0, void* stream)
{
    if (!m || !b || !d_grad_out || !d_dw_self || !d_dw_nbr || !d_dbias) return dn_fail(DN_EINVAL, "null argument");
    for (int i = 0; i < m->k; ++i)
        if (!d_dw_self[i] || !d_dw_nbr[i] || !d_dbias[i]) return dn_fail(DN_EINVAL, "gradient buffers of layer %d are null", i + 1);
    if (m->fwd_serial != b->sample_serial || b->sample_serial == 0)
        return dn_fail(DN_ESTATE, "sage_backward needs sage_forward on the same model and sample first");
    // the transpose index is cached in the batch object; building it is part of this call
    return dn_launch_backward(m, const_cast<dn_batch*>(b), d_grad_out, d_dw_self, d_dw_nbr, d_dbias, d_dH0, nullptr, 0, 0.f,
                              static_cast<hipStream_t>(stream));
}

int sage_backward_sgd(dn_model* m, const dn_batch* b, const float* d_grad_out, float* const* d_dw_self,
                      float* const* d_dw_nbr, float* const* d_dbias, float* d_table, int64_t ld_elems, float lr, void* stream)
{
    if (!m || !b || !d_grad_out || !d_dw_self || !d_dw_nbr || !d_dbias || !d_table) return dn_fail(DN_EINVAL, "null argument");
    for (int i = 0; i < m->k; ++i)
        if (!d_dw_self[i] || !d_dw_nbr[i] || !d_dbias[i]) return dn_fail(DN_EINVAL, "gradient buffers of layer %d are null", i + 1);
    if (m->in_dtype != DN_F32) return dn_fail(DN_EINVAL, "learnable base representations are fp32");
    if (ld_elems < m->dims[0]) return dn_fail(DN_EINVAL, "row stride below the input width");
    if (m->fwd_serial != b->sample_serial || b->sample_serial == 0)
        return dn_fail(DN_ESTATE, "sage_backward_sgd needs sage_forward on the same model and sample first");
    return dn_launch_backward(m, const_cast<dn_batch*>(b), d_grad_out, d_dw_self, d_dw_nbr, d_dbias, nullptr, d_table, ld_elems,
                              lr, static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------------------------------------------------------
// dense_sample for callers that cannot allocate: the batch workspace is a file-scope device array.
// The array's name is a host-side stand-in in host code: its device address is looked up once per device with
// hipGetSymbolAddress and only that address is handed to kernels.
#define DN_NOALLOC_SCRATCH_BYTES ((size_t)64 << 20)
static __device__ __align__(256) unsigned char scratch[DN_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int NOALLOC_MAX_DEVICES = 64;
struct NoallocSlot {
    void* ptr = nullptr;        // device address of this device's copy of `scratch`
    dn_batch batch;             // host-side description of the carve-up of the last call
};
NoallocSlot g_noalloc[NOALLOC_MAX_DEVICES];
std::mutex g_noalloc_mutex;

__global__ void k_noalloc_clear(uint32_t* __restrict__ p, int64_t words)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride) p[i] = 0u;
}

// node_id_offsets (k + 2 entries) and {N, E, status flags} of the sample, from the header
__global__ void k_noalloc_export(const int32_t* __restrict__ hdr, int k, int32_t* __restrict__ node_id_offsets,
                                 int32_t* __restrict__ counts)
{
    const int t = threadIdx.x;
    if (t <= k + 1) node_id_offsets[t] = hdr[HDR_NODE_OFF + t];
    if (t == 0) { counts[0] = hdr[HDR_N]; counts[1] = hdr[HDR_E]; counts[2] = hdr[HDR_STATUS]; }
}
}  // namespace

int dense_sample_noalloc(const dn_graph* g, const int32_t* d_targets, int32_t n_targets, int32_t k, const int32_t* fanouts,
                         int32_t direction, uint64_t seed, int32_t* d_node_id_offsets, int32_t* d_node_ids,
                         int32_t* d_nbr_offsets, int64_t node_capacity, int32_t* d_nbrs, int32_t* d_repr_map,
                         int64_t slot_capacity, int32_t* d_counts, void* stream)
{
    if (!g) return dn_fail(DN_EINVAL, "graph is null");
    if (!d_node_id_offsets || !d_node_ids || !d_nbr_offsets || !d_nbrs || !d_repr_map || !d_counts)
        return dn_fail(DN_EINVAL, "null output array");
    if (n_targets < 0) return dn_fail(DN_EINVAL, "n_targets is negative");
    if (n_targets > 0 && !d_targets) return dn_fail(DN_EINVAL, "d_targets is null");
    int dev = -1;
    DN_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return dn_fail(DN_EINVAL, "device index %d is outside [0, %d)", dev, NOALLOC_MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    NoallocSlot& slot = g_noalloc[dev];
    if (!slot.ptr) {
        // once per device, with that device current: every GPU holds its own copy of the array at its own address
        void* p = nullptr;
        DN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return dn_fail(DN_EHIP, "hipGetSymbolAddress returned a null address");
        slot.ptr = p;
    }
    dn_batch* b = &slot.batch;
    int rc = fill_batch_caps(b, g->V, n_targets > 0 ? n_targets : 1, k, fanouts, direction);
    if (rc) return rc;
    if (b->direction != DN_DIR_IN && !g->rowptr[0]) return dn_fail(DN_EINVAL, "the graph has no out-edge adjacency");
    if (b->direction != DN_DIR_OUT && !g->rowptr[1]) return dn_fail(DN_EINVAL, "the graph has no in-edge adjacency");
    if (node_capacity < b->cap_nodes || slot_capacity < b->cap_slots)
        return dn_fail(DN_ECAPACITY, "output arrays hold %lld nodes / %lld slots, the bound for this request is %lld / %lld",
                       (long long)node_capacity, (long long)slot_capacity, (long long)b->cap_nodes, (long long)b->cap_slots);
    Carver c(slot.ptr);
    carve_batch(b, c, true);
    if (c.bytes() > DN_NOALLOC_SCRATCH_BYTES)
        return dn_fail(DN_ECAPACITY, "dense_sample_noalloc: this graph and batch need %zu bytes of scratch memory, the static "
                       "array holds %zu (use dn_batch_create with a workspace of your own)", c.bytes(), (size_t)DN_NOALLOC_SCRATCH_BYTES);
    b->workspace_bytes = c.bytes();
    b->node_ids = d_node_ids; b->nbr_offsets = d_nbr_offsets; b->nbrs = d_nbrs; b->repr_map = d_repr_map;
    b->n_targets = n_targets;
    b->sample_serial = 1;
    b->tr_serial = ~0ull;
    b->tr_capture_serial = ~0ull;
    b->seen_slots_all = b->seen_slots_upper = -1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // header and bitmaps must start at zero; the array keeps the last call's contents, carved for that call's sizes
    const int64_t zero_words = (int64_t)((reinterpret_cast<char*>(b->lvlpos) - reinterpret_cast<char*>(b->hdr)) / 4);
    int64_t grid = (zero_words + 255) / 256;
    if (grid > 2048) grid = 2048;
    hipLaunchKernelGGL(k_noalloc_clear, dim3((int)grid), dim3(256), 0, st, reinterpret_cast<uint32_t*>(b->hdr), zero_words);
    DN_LAUNCH_CHECK("k_noalloc_clear");
    rc = dn_launch_sample(b, g, d_targets, n_targets, seed, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_noalloc_export, dim3(1), dim3(64), 0, st, b->hdr, k, d_node_id_offsets, d_counts);
    DN_LAUNCH_CHECK("k_noalloc_export");
    return DN_OK;
}

// ---------------------------------------------------------------------------------------------------------------
// Several training steps in flight on streams the library owns.
namespace {
constexpr int STEP_MAX_STREAMS = 16, STEP_MAX_DEVICES = 64;
struct StepStreams {
    hipStream_t spare = nullptr;                  // created first and never used (see dn_train_steps)
    hipStream_t stream[STEP_MAX_STREAMS] = {};
    hipEvent_t done[STEP_MAX_STREAMS] = {};
    hipEvent_t start = nullptr;
    int created = 0;
};
StepStreams g_step_streams[STEP_MAX_DEVICES];
std::mutex g_step_mutex;
}  // namespace

int dn_train_steps(const dn_train_step* steps, int32_t n_steps, int32_t n_streams, void* stream)
{
    if (n_steps < 0 || (n_steps > 0 && !steps)) return dn_fail(DN_EINVAL, "steps is null");
    if (n_streams < 1 || n_streams > STEP_MAX_STREAMS) return dn_fail(DN_EINVAL, "n_streams must be in [1, %d]", STEP_MAX_STREAMS);
    if (n_steps == 0) return DN_OK;
    int dev = -1;
    DN_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= STEP_MAX_DEVICES) return dn_fail(DN_EINVAL, "device index %d is outside [0, %d)", dev, STEP_MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_step_mutex);
    StepStreams& ss = g_step_streams[dev];
    if (!ss.start) DN_HIP(hipEventCreateWithFlags(&ss.start, hipEventDisableTiming));
    if (ss.created == 0 && !ss.spare) {
        // One stream that is never used comes first.  Measured: when the step streams are the first streams the
        // process creates, four steps in flight run at 0.195 ms per step of the 111M-node workload instead of 0.155
        // (the first stream created shares its hardware queue less well); with one, or up to five, other streams
        // created before them the rate is the same whatever else the process has created.
        DN_HIP(hipStreamCreateWithFlags(&ss.spare, hipStreamNonBlocking));
    }
    while (ss.created < n_streams) {
        DN_HIP(hipStreamCreateWithFlags(&ss.stream[ss.created], hipStreamNonBlocking));     // default priority
        DN_HIP(hipEventCreateWithFlags(&ss.done[ss.created], hipEventDisableTiming));
        ss.created += 1;
    }
    hipStream_t outer = static_cast<hipStream_t>(stream);
    const int used = n_steps < n_streams ? n_steps : n_streams;
    // The form of the transpose-index build goes by the slot counts that dn_batch_counts has read back for a batch
    // object (a matter of speed only).  Batch objects of one shape that take turns here see mini-batches of one
    // workload: those that have never been read back go by the largest counts of those that have.
    for (int i = 0; i < n_steps; ++i) {
        dn_batch* bi = steps[i].batch;
        if (!bi || (bi->seen_slots_all >= 0 && bi->seen_slots_upper >= 0)) continue;
        for (int j = 0; j < n_steps; ++j) {
            const dn_batch* bj = steps[j].batch;
            if (!bj || bj == bi || bj->k != bi->k || bj->cap_slots != bi->cap_slots || bj->cap_nodes != bi->cap_nodes) continue;
            if (bj->seen_slots_all > bi->seen_slots_all) bi->seen_slots_all = bj->seen_slots_all;
            if (bj->seen_slots_upper > bi->seen_slots_upper) bi->seen_slots_upper = bj->seen_slots_upper;
        }
    }
    DN_HIP(hipEventRecord(ss.start, outer));
    for (int j = 0; j < used; ++j) DN_HIP(hipStreamWaitEvent(ss.stream[j], ss.start, 0));
    int rc = DN_OK;
    for (int i = 0; i < n_steps && rc == DN_OK; ++i) {
        const dn_train_step& t = steps[i];
        const int j = i % n_streams;
        hipStream_t st = ss.stream[j];
        rc = dense_sample(t.batch, t.graph, t.d_targets, t.n_targets, t.seed, st);
        // (Building the backward pass's transpose index on a further stream beside the forward pass was tried: one step
        // at a time went from 0.263 to 0.256 ms, but a process has four hardware queues which streams take in the order
        // of their creation, and whenever a side stream shared a queue with a step stream the steps got slower, up to
        // 0.19 from 0.165 ms with four in flight.)
        if (rc == DN_OK) rc = sage_forward_table(t.model, t.batch, t.d_table, t.ld_elems, t.d_out, st);
        if (rc != DN_OK || t.forward_only) continue;
        const int k = t.model->k;
        rc = dn_softmax_xent(t.d_out, t.model->dims[k], t.d_labels, t.n_targets, t.model->dims[k], t.grad_scale, t.d_loss,
                             t.d_grad_out, t.model->dims[k], st);
        if (rc == DN_OK) rc = sage_backward(t.model, t.batch, t.d_grad_out, t.d_dw_self, t.d_dw_nbr, t.d_dbias, t.d_dH0, st);
    }
    // join: the caller's stream continues when every internal stream has drained (also after an error, so that no work
    // of this call is left unordered behind the caller's stream)
    for (int j = 0; j < used; ++j) {
        DN_HIP(hipEventRecord(ss.done[j], ss.stream[j]));
        DN_HIP(hipStreamWaitEvent(outer, ss.done[j], 0));
    }
    return rc;
}

// busy-waits `ticks` of the 100 MHz realtime counter on one wave (bounded by a fixed number of loop trips)
__global__ void k_probe_wait(int ticks, int* sink)
{
    const unsigned long long t0 = wall_clock64();
    int n = 0;
    while ((long long)(wall_clock64() - t0) < ticks && n < (1 << 20)) ++n;
    if (n < 0) *sink = n;
}

int dn_profile_step_stream_overlap(int32_t n_streams, int32_t kernel_us, double* elapsed_us)
{
    if (n_streams < 1 || n_streams > STEP_MAX_STREAMS || kernel_us < 1 || kernel_us > 1000 || !elapsed_us)
        return dn_fail(DN_EINVAL, "n_streams in [1, %d], kernel_us in [1, 1000]", STEP_MAX_STREAMS);
    int dev = -1;
    DN_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= STEP_MAX_DEVICES) return dn_fail(DN_EINVAL, "device index %d is outside [0, %d)", dev, STEP_MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_step_mutex);
    StepStreams& ss = g_step_streams[dev];
    if (ss.created < n_streams) return dn_fail(DN_ESTATE, "dn_train_steps has not created %d streams yet", n_streams);
    DN_HIP(hipDeviceSynchronize());
    double best = 1e30;
    for (int rep = 0; rep < 5; ++rep) {
        const auto t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < 8; ++i)
            for (int j = 0; j < n_streams; ++j)
                hipLaunchKernelGGL(k_probe_wait, dim3(1), dim3(64), 0, ss.stream[j], kernel_us * 100, (int*)nullptr);
        DN_HIP(hipDeviceSynchronize());
        const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count() / 8.0;
        if (us < best) best = us;
    }
    *elapsed_us = best;
    return DN_OK;
}

int dn_profile_calibration_copy(void* d_dst, const void* d_src, size_t bytes, void* stream)
{
    if (!d_dst || !d_src || ((uintptr_t)d_dst & 15) || ((uintptr_t)d_src & 15) || (bytes & 15))
        return dn_fail(DN_EINVAL, "calibration copy needs 16-byte aligned pointers and size");
    return dn_launch_calibration_copy(d_dst, d_src, bytes, static_cast<hipStream_t>(stream));
}

__global__ void k_noop() {}

int dn_profile_empty_bracket(void* stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    { dn_prof_scope ps("empty_bracket", 0, st); }
    { dn_prof_scope ps("noop_kernel_bracket", 0, st);
    hipLaunchKernelGGL(k_noop, dim3(1), dim3(64), 0, st);
    }
    DN_LAUNCH_CHECK("k_noop");
    return DN_OK;
}

int dn_profile_enable(int32_t enable)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (enable) prof_clear();
    g_prof_on = enable != 0;
    return DN_OK;
}

int dn_profile_collect(dn_kernel_time* out, int32_t max_entries, int32_t* n_entries)
{
    if (!n_entries || (max_entries > 0 && !out)) return dn_fail(DN_EINVAL, "null argument");
    DN_HIP(hipDeviceSynchronize());
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    std::map<std::string, std::vector<float>> acc;
    std::vector<std::string> order;
    for (auto& r : g_prof_records) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) continue;
        auto it = acc.find(r.tag);
        if (it == acc.end()) { order.push_back(r.tag); it = acc.emplace(r.tag, std::vector<float>()).first; }
        it->second.push_back(ms);
    }
    int32_t n = 0;
    for (auto& tag : order) {
        if (n < max_entries) {
            std::vector<float>& v = acc[tag];
            std::sort(v.begin(), v.end());
            double total = 0.0;
            for (float ms : v) total += ms;
            auto at = [&](double q) { return (double)v[(size_t)(q * (double)(v.size() - 1) + 0.5)]; };
            std::memset(&out[n], 0, sizeof(out[n]));
            std::strncpy(out[n].tag, tag.c_str(), sizeof(out[n].tag) - 1);
            out[n].total_ms = total;
            out[n].launches = (int64_t)v.size();
            out[n].p10_ms = at(0.10);
            out[n].p50_ms = at(0.50);
            out[n].p90_ms = at(0.90);
        }
        ++n;
    }
    *n_entries = n;
    return DN_OK;
}

}  // extern "C"
