// Internal declarations shared by the HIP translation units of libdense_mi355x.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "dense.h"

typedef uint16_t dn_bf16;   // bfloat16 bit pattern

// ---------------------------------------------------------------- device-resident header
// One int32[DN_HDR_WORDS] block per batch keeps every size that depends on the sample, so that
// no kernel launch needs a host read-back.  "Level" h = hop distance from the targets
// (level 0 = targets = Delta_k, level h = Delta_{k-h}); staging arrays are in level order,
// the final DENSE arrays in the paper's order (Delta_0 first).
enum {
    HDR_LVL_OFF = 0,       // [k+2] start of level h in the staging node array, then N
    HDR_LVL_NBR_OFF = 8,   // [k+1] start of hop h's slots in the staging neighbour array, then E
    HDR_NODE_OFF = 16,     // [k+2] final node_id_offsets
    HDR_N = 24,
    HDR_E = 25,
    HDR_STATUS_ACC = 26,   // flags raised while sampling; moved to HDR_STATUS by the last kernel
    HDR_STATUS = 27,
    HDR_NTARGETS = 28,
    HDR_TR_FIRST = 32,     // first slot covered by the transpose index
    HDR_TR_COUNT = 33,     // number of slots covered by it
    HDR_SAMPLE_SEQ = 34,   // counts the samples built in this workspace (bumped on the device by the last sampling kernel)
    HDR_TR_SEQ = 35,       // HDR_SAMPLE_SEQ of the sample the transpose index was built for
    HDR_TR_ALL = 36,       // 1 if that index covers every slot (input gradient of layer 1), 0 if only layers 2..k
    DN_HDR_WORDS = 64
};
enum { ST_BAD_TARGET = 1, ST_DUP_TARGET = 2, ST_CAPACITY = 4, ST_STALE_INDEX = 8,
       ST_INTERNAL = 16 };   // a bounded wait between workgroups of one kernel ran out (never seen; see k_next_delta)

struct dn_graph {
    int64_t V;
    const int64_t* rowptr[2];   // [0] by source (out-edges), [1] by destination (in-edges)
    const int32_t* col[2];
};

struct dn_batch {
    int64_t V;
    int32_t k, direction, max_targets;
    int32_t fanouts[DN_MAX_LAYERS];
    int64_t cap_level[DN_MAX_LAYERS + 1];   // node capacity per level
    int64_t cap_slots_hop[DN_MAX_LAYERS];   // slot capacity per hop
    int64_t cap_nodes, cap_slots;
    int64_t words0, words1;                 // bitmap words: one bit per node / per bitmap word
    int32_t walk_shift;                     // log2 of the bitmap words one thread of the next-Delta kernels walks
    int32_t max_blocks;
    // workspace carve-up (device pointers)
    int32_t* hdr;
    uint32_t *seen, *fresh, *summary;
    int32_t* lvlpos;                        // [V] node id -> staging position (valid for sampled nodes only)
    int32_t *lvl_ids, *lvl_nbr_offsets, *lvl_nbrs, *lvl_owner;
    int32_t *blk_a, *blk_b;
    int32_t *node_ids, *nbr_offsets, *nbrs, *repr_map, *slot_owner;
    // transpose index for the backward pass (slots grouped by the input row they read)
    int32_t *tr_key[2], *tr_val[2], *tr_ptr, *tr_hist;
    int32_t* tr_own;                        // owner (output row) of slot tr_val[0][t]
    float* tr_inv;                          // 1 / (number of slots of that owner)
    int32_t* tr_long;                       // [cap_slots / DN_LONG_GROUP + 2] rows read by more than DN_LONG_GROUP slots
    int64_t tr_long_words;
    int64_t tr_hist_words;
    int32_t n_targets;
    // largest slot counts that dn_batch_counts has read back so far (-1: none yet): all slots, and the slots of the
    // layers above the first; they choose the form of the transpose-index build (a matter of speed only)
    mutable int64_t seen_slots_all, seen_slots_upper;
    uint64_t sample_serial;                 // bumped by every dense_sample
    uint64_t tr_serial;                     // sample the transpose index was built for
    int32_t tr_covers_all;
    uint64_t tr_capture_serial;             // the same pair for builds recorded into a HIP graph (not executed yet)
    int32_t tr_capture_covers_all;
    size_t workspace_bytes;
};

struct dn_layer_bufs {
    int32_t d_in, d_out;
    int32_t xterms;      // bf16 terms per activation operand: 1 for layer 1 (derived from inputs), 2 above
    int32_t zterms;      // bf16 terms of dZ in the backward GEMMs: 1 for the last layer (caller's gradient), 2 below
    int32_t kx;          // valid columns of X: 2*d_in*xterms  = [self | mean] per term
    int32_t kp;          // kx rounded up to 64: reduction length of the forward GEMM
    int32_t np;          // d_out rounded up to 64
    int32_t nz;          // np*zterms: row length of bf16(dZ) = reduction length of the dX GEMM
    int64_t rows_cap;    // capacity of output rows of this layer
    int64_t rows_pad;    // rows_cap rounded up to 128
    dn_bf16* x;          // [rows_pad x kp]
    float* h;            // [rows_pad x d_out] layer output (not for the last layer)
    dn_bf16* wt;         // [round128(d_out) x kp]   Wcat^T repeated per X term, zero padded
    dn_bf16* w;          // [round128(2*d_in) x nz]  Wcat repeated per dZ term, zero padded
    // layers above the first with d_in a multiple of 16: Wcat^T once more in the order v_mfma_f32_16x16x32_bf16 takes
    // its B operand, [np/16 column tiles][2*d_in/32 reduction steps][64 lanes][8]: lane l of the fragment of tile T,
    // step s holds Wcat^T[16 T + l % 16][32 s + 8 (l / 16) .. + 8]; rows >= d_out are zero.  Null otherwise.
    dn_bf16* wf;
    float* bias;         // [d_out]
    float* rownorm;      // [rows_pad] L2 norm of each X row (bounds the accumulation error of Z)
    float* colnorm;      // [d_out]    L2 norm of each Wcat^T row
    // bf16 terms of dZ, row-major [rows_pad x nz] (term t in columns [t*np, (t+1)*np)): A operand of the dX GEMM and,
    // with X, operand of the weight-gradient GEMM (both are read with the node index as the reduction index);
    // per layer, because the weight gradients of all layers are computed in one launch after the chain
    dn_bf16* dzb;
    float* partial;      // split-K partials of dWcat
    int64_t partial_floats;
    float* db_partial;   // per row-tile column sums of dZ
};

struct dn_model {
    int32_t k, in_dtype;
    int32_t dims[DN_MAX_LAYERS + 1];
    dn_layer_bufs layer[DN_MAX_LAYERS];
    // backward temporaries, sized for the largest layer
    float* dx;
    int32_t splits;

    // pre-activations too close to zero for the fp32 accumulation to settle their sign
    // exact recomputations in the last ReLU layer: DN_FIX_SLOTS counters on cache lines of their own (a workgroup adds to
    // slot (workgroup number % DN_FIX_SLOTS): one counter for all would queue a thousand atomics on one line), at
    // fix_count[DN_FIX_FIRST + DN_FIX_STRIDE * j]; [1] sticky overflow flag
    int32_t* fix_count;
    float* zero_row;               // DN_ZERO_ROW_FLOATS zeros that nothing writes (a place to read for a slot that does not exist)
    const void* h0;                // H^0 of the last forward
    uint64_t fwd_serial;           // sample the saved activations belong to
    int32_t weights_set;
    int32_t mean_agg;              // 1: neighbour mean (default), 0: neighbour sum (Algorithm 3 as printed)
    size_t workspace_bytes;
};

constexpr int DN_ZERO_ROW_FLOATS = 1024;
constexpr int DN_FIX_SLOTS = 32, DN_FIX_STRIDE = 16, DN_FIX_FIRST = 64;
constexpr int DN_FIX_WORDS = DN_FIX_FIRST + DN_FIX_SLOTS * DN_FIX_STRIDE;

// error plumbing (abi.cpp)
int dn_fail(int code, const char* fmt, ...);
#define DN_HIP(call)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess) return dn_fail(DN_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)
#define DN_LAUNCH_CHECK(name)                                                            \
    do {                                                                                 \
        hipError_t e_ = hipGetLastError();                                               \
        if (e_ != hipSuccess) return dn_fail(DN_EHIP, "launch %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

// Optional per-launch event pair (see dn_profile_enable); a no-op unless profiling is on.
struct dn_prof_scope {
    int idx;
    hipStream_t st;
    dn_prof_scope(const char* tag, int layer, hipStream_t stream);
    ~dn_prof_scope();
};

static inline int64_t dn_round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// fp32 <-> bfloat16 bit patterns, round to nearest even (a NaN stays a quiet NaN)
__device__ __forceinline__ uint16_t f32_to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

struct dn_carver {       // hands out 256-byte aligned pieces of one workspace; counts when base == nullptr
    char* base;
    size_t off = 0;
    explicit dn_carver(void* b) : base(static_cast<char*>(b)) {}
    template <typename T>
    T* take(int64_t count)
    {
        off = (off + 255) & ~size_t(255);
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += sizeof(T) * (size_t)(count > 0 ? count : 0);
        return p;
    }
    size_t bytes() const { return (off + 255) & ~size_t(255); }
};

// launchers (one per step of the hot path)
int dn_launch_sample(dn_batch* b, const dn_graph* g, const int32_t* d_targets, int32_t n_targets,
                     uint64_t seed, hipStream_t st);
int dn_launch_sample_edges(dn_batch* b, const dn_graph* g, const int32_t* d_src, const int32_t* d_dst, int32_t n_edges,
                           const int32_t* d_neg, int32_t n_neg, uint64_t seed, int32_t* d_src_local,
                           int32_t* d_dst_local, int32_t* d_neg_local, hipStream_t st);
int dn_launch_embedding_sgd(const dn_batch* b, float* table, int32_t dim, int64_t ld, const float* dh0, float lr,
                            hipStream_t st);
int dn_launch_embedding_adagrad(const dn_batch* b, float* table, float* state, int32_t dim, int64_t ld, const float* dh0,
                                float lr, float eps, hipStream_t st);
int dn_launch_softmax_xent(const float* logits, int64_t ld, const int32_t* labels, int64_t n, int32_t num_classes, float scale,
                           float* loss, float* grad, int64_t ldg, hipStream_t st);
int dn_launch_gather(const dn_batch* b, const void* table, int32_t dtype, int32_t dim, int64_t ld,
                     void* h0, hipStream_t st);
int dn_launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
int dn_launch_transpose_index(dn_batch* b, int need_all, hipStream_t st);
int64_t dn_transpose_index_hist_words(const dn_batch* b);

// Stable radix sort of (key, value) pairs whose count lives in device memory (transpose_index.hip).
// The caller's own kernel writes the pairs into key[passes & 1] / val[passes & 1] and counts, per
// tile of DN_SORT_TILE consecutive pairs, the first digit:
//   hist[(key & ((1 << bits) - 1)) * dn_sort_tiles(count) + i / DN_SORT_TILE]++.
// The histograms' rows are as long as the tiles in use, not as the capacity: scans and clears touch what a
// mini-batch fills.
constexpr int DN_SORT_TILE = 1024;
__host__ __device__ inline int dn_sort_tiles(int count) { return count > 0 ? (count + DN_SORT_TILE - 1) / DN_SORT_TILE : 1; }
struct dn_sort_plan { int passes, bits, nblocks, total, sblocks; };
dn_sort_plan dn_sort_make_plan(int64_t key_range, int64_t cap_items);
int64_t dn_sort_hist_words(const dn_sort_plan& p);
bool dn_sort_counts_separately(const dn_sort_plan& p);   // true: the caller's first kernel must NOT count the first digit
// Optional by-products of the last kernel, for values that are slot numbers of a DENSE sample (null otherwise):
// own_out[t] = slot_owner[val[t]], inv_out[t] = 1 / (number of slots of that owner), and
// long_out[first / DN_LONG_GROUP] = key + 1 for every key whose group of more than DN_LONG_GROUP sorted pairs
// starts at index `first` (no two such groups start in one block of DN_LONG_GROUP indices; the caller clears
// long_out beforehand).
constexpr int DN_LONG_GROUP = 64;
constexpr int64_t DN_TR_SMALL_MAX_PAIRS = 40960;          // up to here the index is built by one kernel
struct dn_sort_slot_info { const int32_t* slot_owner; const int32_t* nbr_offsets; int32_t* own_out; float* inv_out;
                           int32_t* long_out;
                           int32_t* hdr; int covers_all; };   // batch header: the last kernel stamps the index with the sample's sequence number
int dn_sort_pairs_run(const dn_sort_plan& pl, const int32_t* count_ptr, int32_t* const key[2], int32_t* const val[2],
                      int32_t* hist_space, const int32_t* nkeys_ptr, int64_t nkeys_cap, int32_t* ptr_out, hipStream_t st,
                      const dn_sort_slot_info* info = nullptr);
int dn_launch_set_weights(dn_model* m, const float* const* ws, const float* const* wn,
                          const float* const* bias, hipStream_t st);
int dn_launch_forward(dn_model* m, const dn_batch* b, const void* h0, int64_t ldh, int from_table, float* out,
                      hipStream_t st);
int dn_launch_backward(dn_model* m, dn_batch* b, const float* grad_out, float* const* dws,
                       float* const* dwn, float* const* dbias, float* dh0, float* sgd_table, int64_t sgd_ld, float sgd_lr,
                       hipStream_t st);

// row-tile workgroups of the dZ kernel = partial column sums the bias-gradient reduction adds up
constexpr unsigned DN_DZ_MAX_ROW_BLOCKS = 512;

// GEMM entry points (gemm.hip), layer index i is 1-based
int dn_gemm_forward(const dn_model* m, const dn_batch* b, int i, float* out, int64_t ldc, hipStream_t st);
// a layer above the first as one launch (layer_fused.hip): aggregation + linear map + bias + ReLU
bool dn_layer_is_fused(const dn_model* m, int i);
int dn_launch_layer_fused(const dn_model* m, const dn_batch* b, int i, float* out, int64_t ldc, hipStream_t st);
int dn_gemm_dx(const dn_model* m, const dn_batch* b, int i, hipStream_t st);
int dn_gemm_dw_all(const dn_model* m, const dn_batch* b, float* const* dws, float* const* dwn, float* const* dbias,
                   hipStream_t st);
