/*
 * dense.h -- C ABI of libdense_mi355x.so: DENSE mini-batch construction and the GraphSage-mean
 * encoder that consumes it, on one MI355X (gfx950), graph and features resident in HBM.
 *
 * Citations are to the MariusGNN paper (arXiv 2202.02365): Section 4.1 / Algorithm 1
 * (multi-hop sampling into DENSE), Section 4.2 (repr_map, H^0, Step 1 / Step 2,
 * Algorithm 2 = DENSE update per layer, Algorithm 3 = layer aggregation), Section 2
 * (the generic GNN layer and the backward pass), Section 7.1 (fanout order, directions).
 *
 * Conventions
 *   - Every pointer whose name starts with d_ is a DEVICE pointer; everything else is host memory.
 *   - The caller owns the graph, the feature table, weights, outputs and the workspaces it
 *     hands over; the library allocates no device memory.  Handles (dn_graph, dn_batch,
 *     dn_model) are small host objects; destroy them with the matching *_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued asynchronously; the only entry point that waits for the device is
 *     dn_batch_counts.  Sizes that depend on the sample stay in device memory.
 *   - Return value: DN_OK (0) or a negative DN_E* code; dn_last_error() then returns a
 *     thread-local description.  No entry point aborts or throws.
 *   - k = number of layers = number of hops, 1 <= k <= DN_MAX_LAYERS.  fanouts[h] is the
 *     fanout of hop h, ordered AWAY from the targets (Section 7.1), 1 <= fanouts[h] <= 64.
 *   - Delta_k = targets (caller order).  Delta_{k-1-h} = nodes first reached at hop h, in
 *     ascending node id.  node_ids = Delta_0 | Delta_1 | ... | Delta_k (Algorithm 1 stacks
 *     each new Delta in front).  Both offset arrays carry an end sentinel.
 *   - Determinism: the same (graph, targets, fanouts, direction, seed) gives byte-identical
 *     arrays, and the same inputs give bit-identical embeddings and gradients, run to run.
 */
#ifndef DENSE_MI355X_H
#define DENSE_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported symbol */
#define DN_API __attribute__((visibility("default")))

#define DN_MAX_LAYERS 6
#define DN_MAX_FANOUT 64

enum {
    DN_OK = 0,
    DN_EINVAL = -1,     /* bad argument (null pointer, size or fanout out of range, unsupported dtype) */
    DN_ECAPACITY = -2,  /* a workspace is too small for the request */
    DN_EHIP = -3,       /* a HIP runtime call failed; dn_last_error() carries hipGetErrorString */
    DN_ESTATE = -4,     /* call order violated (e.g. sage_backward before sage_forward) */
    DN_ESAMPLE = -5     /* reported by dn_batch_counts: duplicate or out-of-range target id */
};

enum { DN_F32 = 0, DN_BF16 = 1 };
enum { DN_DIR_OUT = 0, DN_DIR_IN = 1, DN_DIR_BOTH = 2 };

typedef struct dn_graph dn_graph;
typedef struct dn_batch dn_batch;
typedef struct dn_model dn_model;

/* Device pointers to the five arrays of one sampled mini-batch (valid until the next
 * dense_sample on the same dn_batch).  Element counts are those of dn_batch_counts. */
typedef struct dn_dense_view {
    const int32_t* d_node_id_offsets; /* [k+2] start of Delta_0..Delta_k in node_ids, then N      */
    const int32_t* d_node_ids;        /* [N]                                                      */
    const int32_t* d_nbr_offsets;     /* [N - n_0 + 1] entry q: start in nbrs of the node at
                                         position node_id_offsets[1]+q; last entry = E            */
    const int32_t* d_nbrs;            /* [E] sampled neighbours, sequential per node              */
    const int32_t* d_repr_map;        /* [E] position in node_ids (= row of H^0) of nbrs[j]       */
} dn_dense_view;

DN_API const char* dn_last_error(void);

/* ---- graph store (Section 4.1: edges sorted by source and by destination with per-node offsets,
 *      held here as CSR / CSC in HBM).  Borrows the caller's device buffers.
 *      d_rowptr_* : int64[V+1]; d_col_* : int32[rowptr[V]].  The in-edge pair may be NULL when only
 *      DN_DIR_OUT is sampled (and vice versa). */
DN_API int  dn_graph_create(dn_graph** out, int64_t num_nodes,
                     const int64_t* d_rowptr_out, const int32_t* d_col_out,
                     const int64_t* d_rowptr_in, const int32_t* d_col_in);
DN_API void dn_graph_destroy(dn_graph* g);

/* ---- mini-batch object: capacities and workspace.
 *      dn_batch_workspace_size: bytes of device workspace needed for batches of at most
 *      max_targets targets on a graph of num_nodes nodes (upper bound max_targets * prod(fanouts),
 *      capped by num_nodes; twice the fanout per hop for DN_DIR_BOTH).
 *      dn_batch_create: binds the workspace (256-byte aligned, owned by the caller, must outlive
 *      the batch) and zeroes the part that must start at zero on `stream`. */
DN_API int  dn_batch_workspace_size(int64_t num_nodes, int32_t max_targets, int32_t k, const int32_t* fanouts,
                             int32_t direction, size_t* bytes);
DN_API int  dn_batch_create(dn_batch** out, int64_t num_nodes, int32_t max_targets, int32_t k,
                     const int32_t* fanouts, int32_t direction,
                     void* d_workspace, size_t workspace_bytes, void* stream);
DN_API void dn_batch_destroy(dn_batch* b);
/* Capacities the workspace was sized for: rows of node_ids / H^0, and neighbour slots. */
DN_API int  dn_batch_capacity(const dn_batch* b, int64_t* node_capacity, int64_t* slot_capacity);

/* ---- dense_sample: Algorithm 1.  One-hop sampling (Section 4.1: a node with more than f neighbours
 *      gets f of them, otherwise all) is uniform without replacement over adjacency positions by
 *      Floyd's subset algorithm; step s of node v at hop h draws word (s & 3) of
 *      Philox4x32-10(counter = (s >> 2, v, h, direction bit), key = (seed lo, seed hi)) and maps
 *      it to [0, deg - f + s] by a 32-bit multiply-high.  Neighbours are stored in Floyd
 *      insertion order (adjacency order when deg <= f); for DN_DIR_BOTH a node's segment is its
 *      out-sample followed by its in-sample.  Also builds repr_map (Section 4.2).
 *      d_targets: int32[n_targets], pairwise distinct ids in [0, V); a violation is reported by
 *      the next dn_batch_counts as DN_ESAMPLE (the arrays are then unspecified but in bounds). */
DN_API int  dense_sample(dn_batch* b, const dn_graph* g, const int32_t* d_targets, int32_t n_targets,
                  uint64_t seed, void* stream);

/* ---- dense_sample_noalloc: dense_sample for callers that cannot allocate device memory or hold a workspace: code
 *      under HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same sampling, same arrays,
 *      bit for bit; the batch workspace is a static device array inside the library (64 MiB per GPU, held until
 *      the process ends) and the five DENSE arrays are written straight into the caller's buffers.  The call
 *      allocates nothing on the device (no hipMalloc / hipFree, no library that would), creates no handle, and
 *      enqueues kernels only (no hipMemsetAsync).
 *      k, fanouts (host array), direction: as in dn_batch_create.  Outputs (device, caller-owned):
 *        d_node_id_offsets int32[k+2]; d_node_ids int32[node_capacity]; d_nbr_offsets int32[node_capacity + 1];
 *        d_nbrs, d_repr_map int32[slot_capacity]; d_counts int32[3] = {N, E, status} with status != 0 for an invalid
 *        target set (1 = id out of range, 2 = duplicate id, 4 = capacity), the arrays then unspecified but in bounds.
 *      The capacities must cover the request's upper bound (DN_ECAPACITY otherwise, the message names the bound):
 *        level_0 = max(n_targets, 1), level_{h+1} = min(V, level_h * fanouts[h] * m), m = 2 for DN_DIR_BOTH else 1;
 *        slot_capacity >= sum_h level_h * fanouts[h] * m;  node_capacity >= min(V, sum of all levels).
 *      Limit: graph and batch must fit the static array, about 4.3 bytes per node of the graph plus 8 bytes per
 *      node and 12 bytes per slot of the bound (a 2^20-node graph with 1000 targets and fanouts 15/10/5 needs 23 MiB);
 *      larger requests return DN_ECAPACITY and belong to dn_batch_create with a caller-supplied workspace.
 *      Every call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU (different streams
 *      or threads) race and must be serialised by the caller; calls on different GPUs are independent. */
DN_API int  dense_sample_noalloc(const dn_graph* g, const int32_t* d_targets, int32_t n_targets, int32_t k,
                                 const int32_t* fanouts, int32_t direction, uint64_t seed,
                                 int32_t* d_node_id_offsets, int32_t* d_node_ids, int32_t* d_nbr_offsets, int64_t node_capacity,
                                 int32_t* d_nbrs, int32_t* d_repr_map, int64_t slot_capacity, int32_t* d_counts, void* stream);

/* ---- dense_sample_edges: the link-prediction front end (Section 2: a training example is a pair of target
 *      nodes; Section 7.1: neighbours over incoming and outgoing edges).  The targets are the distinct ids
 *      among d_src[0..n_edges), d_dst[0..n_edges) and d_neg[0..n_neg), in ASCENDING id (they form Delta_k);
 *      sampling then proceeds exactly as dense_sample.  d_*_local (int32, same lengths as the inputs) receive,
 *      for every endpoint and negative, its index in that target list = the row of sage_forward's output.
 *      Requires 2 * n_edges + n_neg <= max_targets of the batch.  Out-of-range ids are reported by
 *      dn_batch_counts as DN_ESAMPLE. */
DN_API int  dense_sample_edges(dn_batch* b, const dn_graph* g, const int32_t* d_src, const int32_t* d_dst, int32_t n_edges,
                               const int32_t* d_neg, int32_t n_neg, uint64_t seed,
                               int32_t* d_src_local, int32_t* d_dst_local, int32_t* d_neg_local, void* stream);

/* ---- dn_embedding_sgd: update of learnable base representations (Section 2: "updates for learned base
 *      representations" applied to the lookup table): d_table[node_ids[r], :] -= lr * d_dH0[r, :] for r < N, fp32,
 *      multiply and subtract rounded separately.  node_ids holds every node once, so no two rows collide.
 *      The paper does not name the optimiser; plain SGD is the reading taken here. */
DN_API int  dn_embedding_sgd(const dn_batch* b, float* d_table, int32_t dim, int64_t ld_elems, const float* d_dH0,
                             float lr, void* stream);

/* ---- dn_embedding_adagrad: the same update with Adagrad per element (another reading of the unnamed optimiser):
 *      d_state[v, :] += g * g;  d_table[v, :] -= (lr * g) / (sqrt(d_state[v, :]) + eps)   for v = node_ids[r], g = d_dH0[r, :],
 *      fp32, every operation rounded on its own.  d_state: fp32 accumulators laid out like d_table (same ld_elems). */
DN_API int  dn_embedding_adagrad(const dn_batch* b, float* d_table, float* d_state, int32_t dim, int64_t ld_elems,
                                 const float* d_dH0, float lr, float eps, void* stream);

/* ---- dn_softmax_xent: node-classification loss head (Section 2: the forward pass ends in a loss whose gradients
 *      flow back; the paper does not name the loss, softmax cross-entropy is the reading taken).  For row i < n:
 *      d_loss[i] = logsumexp(d_logits[i, :]) - d_logits[i, d_labels[i]],
 *      d_grad[i, :] = grad_scale * (softmax(d_logits[i, :]) - onehot(d_labels[i]))   (what sage_backward takes as dL/dH^k).
 *      Row strides ld_logits, ld_grad in floats.  A label outside [0, num_classes) gives d_loss[i] = NaN and no
 *      onehot term; no access leaves the arrays. */
DN_API int  dn_softmax_xent(const float* d_logits, int64_t ld_logits, const int32_t* d_labels, int64_t n, int32_t num_classes,
                            float grad_scale, float* d_loss, float* d_grad, int64_t ld_grad, void* stream);

/* Optional: builds, on `stream`, the index sage_backward needs for the transpose of the neighbour mean
 * (neighbour slots grouped by the row of H they read; with need_input_grad = 0 only the slots of layers
 * 2..k).  sage_backward builds it itself when this was not called for the current sample; calling it
 * right after dense_sample moves that work off the forward/backward chain, e.g. onto the stream
 * that constructs mini-batches.
 * HIP-graph capture: whether sage_backward enqueues the build is decided on the HOST when the call is made: it is
 * skipped if a build for the batch's current sample was already issued, eager builds counting for eager calls and
 * builds recorded into a graph for calls under capture.  So graphs captured from [dense_sample,
 * dn_batch_prepare_backward] and then [sage_backward] hold one build between them, in the first graph, and the second
 * graph is valid only behind a replay of the first; a sage_backward captured without a recorded
 * dn_batch_prepare_backward for its sample holds its own build and can be replayed after any sample.  The device
 * checks it: every sample carries a sequence number in the workspace, the build stamps the index with it, and a
 * backward aggregation that finds another number computes nothing and raises a flag that dn_batch_counts returns as
 * DN_ESTATE. */
DN_API int  dn_batch_prepare_backward(dn_batch* b, int32_t need_input_grad, void* stream);

/* Device pointers of the current sample. */
DN_API int  dn_batch_view(const dn_batch* b, dn_dense_view* view);

/* Copies node_id_offsets[0..k+1] followed by E (k+3 values) to host_counts and WAITS for `stream`.
 * Returns DN_ESAMPLE if the last dense_sample saw an invalid target set.
 * DN_ESTATE is also returned if a workgroup of the next-Delta kernel ever gave up its (bounded) wait for the totals of the
 * workgroups in front of it: the sample is then incomplete, and the batch object must not be sampled into again (its
 * bitmaps are no longer clean).  The library launches that kernel only where every workgroup of every such kernel the
 * process can have in flight is resident at once (hardware queues of the process, GPU_MAX_HW_QUEUES or 4, times the
 * workgroups per XCD within the chip's slots), where no wait can starve, and uses two kernels without waits
 * otherwise; the bound exists so that the kernel ends whatever happens.
 * The batch object remembers the largest slot counts read back so far: the transpose-index build of sage_backward /
 * dn_batch_prepare_backward takes its one-kernel form for a batch object whose mini-batches have stayed below a few
 * ten thousand slots and the multi-pass sort otherwise or when no size was ever read back (both forms are correct for
 * any size; a training loop that reads the sizes once per batch object, e.g. to log them, gets the faster one).
 * dn_train_steps hands the counts on between batch objects of one shape that take turns in its step list. */
DN_API int  dn_batch_counts(const dn_batch* b, int64_t* host_counts, void* stream);

/* ---- dense_gather: H^0[r, :] = table[node_ids[r], :] for r < N (Section 4.2).
 *      d_table: [V x dim] row-major with row stride ld_elems elements, dtype DN_F32 or DN_BF16.
 *      d_H0:    [N x dim] dense row-major, same dtype, capacity >= the batch's node capacity rows. */
DN_API int  dense_gather(const dn_batch* b, const void* d_table, int32_t dtype, int32_t dim, int64_t ld_elems,
                  void* d_H0, void* stream);

/* ---- GraphSage-mean encoder.  dims[0..k]: dims[0] = width of H^0, dims[i] = width of layer i.
 *      Layer i (Step 1 + Algorithm 3 with mean, Algorithm 2 applied as offset arithmetic):
 *        M[p]   = mean over p's neighbour slots j of H^{i-1}[repr_map[j]]   (0 when p has none),
 *                 fp32 sum in ascending slot order, fp32 division
 *        Z[p]   = bf16(H^{i-1}[p]) W_self^i + bf16(M[p]) W_nbr^i + b^i     bf16 MFMA operands, fp32 accumulate
 *        H^i[p] = ReLU(Z[p]) for i < k, Z[p] for i = k                      stored fp32
 *      for every node p of node_ids after Delta_{i-1}.
 *      dn_model_workspace_size / dn_model_create: workspace for activations saved for the backward
 *      pass and for backward temporaries, sized from the batch's capacities; in_dtype = dtype of H^0.
 *      dn_model_set_weights: d_w_self[i-1], d_w_nbr[i-1]: fp32 [dims[i-1] x dims[i]] row-major,
 *      d_bias[i-1]: fp32 [dims[i]]; converted once to the bf16 layouts the kernels use (call it
 *      again after every optimiser step). */
DN_API int  dn_model_workspace_size(const dn_batch* b, int32_t k, const int32_t* dims, int32_t in_dtype, size_t* bytes);
DN_API int  dn_model_create(dn_model** out, const dn_batch* b, int32_t k, const int32_t* dims, int32_t in_dtype,
                     void* d_workspace, size_t workspace_bytes, void* stream);
DN_API int  dn_model_set_weights(dn_model* m, const float* const* d_w_self, const float* const* d_w_nbr,
                          const float* const* d_bias, void* stream);
DN_API void dn_model_destroy(dn_model* m);
/* Diagnostics of the last sage_forward; WAITS for `stream`.  status[0] = pre-activations, over all
 * ReLU layers, whose sign the fp32 accumulation could not settle and that were recomputed in fp64;
 * status[1] = 1 if that queue ever overflowed since dn_model_create (the surplus kept its fp32 sign). */
DN_API int  dn_model_status(const dn_model* m, int32_t* status, void* stream);

/* sage_forward: d_H0 = output of dense_gather (dtype in_dtype); d_out: fp32 [n_targets x dims[k]],
 * row t = embedding of target t (caller order). */
DN_API int  sage_forward(dn_model* m, const dn_batch* b, const void* d_H0, float* d_out, void* stream);

/* sage_forward_table: sage_forward without the H^0 round trip: layer 1 reads the rows of the lookup table
 * (Section 4.2: base representations are looked up by node_ids) directly, d_table[node_ids[p], :] for a node's own
 * row and d_table[nbrs[j], :] for neighbour slot j, so dense_gather and its buffer are not needed.  d_table:
 * [V x dims[0]] of the model's in_dtype with row stride ld_elems elements.  Same values, same arithmetic, same
 * results as dense_gather followed by sage_forward; sage_backward follows it in the same way. */
DN_API int  sage_forward_table(dn_model* m, const dn_batch* b, const void* d_table, int64_t ld_elems, float* d_out,
                               void* stream);

/* dn_model_set_aggregation: DN_AGG_MEAN (default; the GraphSage-mean layer above) or DN_AGG_SUM, the additive
 * aggregation of Algorithm 3 as printed (segment sum of the neighbours' rows, no division); applies to
 * sage_forward / sage_forward_table / sage_backward calls that follow. */
enum { DN_AGG_MEAN = 0, DN_AGG_SUM = 1 };
DN_API int  dn_model_set_aggregation(dn_model* m, int32_t aggregation);

/* sage_backward (Section 2: "loss and gradients"): given d_grad_out = dL/dH^k, fp32
 * [n_targets x dims[k]], writes dL/dW_self^i, dL/dW_nbr^i (fp32 [dims[i-1] x dims[i]]) and dL/db^i
 * (fp32 [dims[i]]) for every layer, and, when d_dH0 is not NULL, dL/dH^0 (fp32 [N x dims[0]],
 * capacity >= node capacity rows; needed for learnable base representations).  Uses the
 * activations saved by the last sage_forward on the same model and batch.  Neighbour-mean
 * gradients are summed per input row in ascending slot order (no floating-point atomics).
 * dL/db^k sums the fp32 rows of d_grad_out; below the last layer dL/db^i sums dZ^i as the two bf16 terms
 * (16 mantissa bits per element) that the weight-gradient contraction multiplies, accumulated in fp32. */
DN_API int  sage_backward(dn_model* m, const dn_batch* b, const float* d_grad_out,
                   float* const* d_dw_self, float* const* d_dw_nbr, float* const* d_dbias,
                   float* d_dH0, void* stream);

/* sage_backward_sgd: sage_backward for learnable base representations without the dL/dH^0 round trip: the layer-1
 * input gradient of node_ids[r] is applied to the lookup table as it is formed,
 *   d_table[node_ids[r], :] -= lr * dL/dH^0[r, :]      (fp32, product and difference rounded separately),
 * which leaves the table exactly as sage_backward with d_dH0 followed by dn_embedding_sgd does.  The forward pass of
 * the same sample must have read the table before (sage_forward_table, or dense_gather + sage_forward). */
DN_API int  sage_backward_sgd(dn_model* m, const dn_batch* b, const float* d_grad_out,
                              float* const* d_dw_self, float* const* d_dw_nbr, float* const* d_dbias,
                              float* d_table, int64_t ld_elems, float lr, void* stream);

/* ---- DistMult decoder with shared negatives (link prediction).  The paper names the DistMult score function
 *      (Section 7.1, link prediction: datasets, models and metrics) and the number of negatives (Section 7.3) only;
 *      score, loss and negative scheme are the textbook ones:
 *        f(s, r, d) = sum_j h_s[j] r[j] h_d[j];
 *        edges are cut into chunks of `chunk` consecutive edges, chunk q shares the negatives d_neg[q, 0..num_neg);
 *        side 0 corrupts the destination, f(s, r, neg), side 1 the source, f(neg, r, d);
 *        loss[e] = sum over both sides of logsumexp([pos, that side's negatives]) - pos.
 *      The negatives' scores are a bf16 MFMA contraction (operands bf16(h * r), formed in fp32, and bf16(h_neg),
 *      fp32 accumulation); the positive's score uses the fp32 inputs.
 *
 *      dn_decoder_create carves the caller's 256-byte aligned device workspace (size from
 *      dn_decoder_workspace_size) for at most max_edges edges per call, rows of H below max_rows and num_rel
 *      relations, and clears it on `stream`.  The library allocates no device memory.
 *
 *      distmult_forward: d_H [n_rows x dim] fp32 with row stride ldh (the encoder's output for the batch's targets),
 *      d_R [num_rel x dim] fp32 with row stride ldr, d_src / d_rel / d_dst int32[n_edges] (rows of H, relation ids),
 *      d_neg int32[ceil(n_edges / chunk) x num_neg] rows of H.  Outputs d_pos, d_loss: fp32[n_edges].
 *      An index outside its range makes that edge (negative) count as a zero row and raises a flag that
 *      dn_decoder_status returns (1 = node index, 2 = relation); no access leaves its array.
 *      The decoder keeps the input pointers: they must stay valid and unchanged until distmult_backward ran.
 *
 *      distmult_backward: gradients of sum_e loss[e] of the last distmult_forward: d_dH [n_rows x dim] (row stride
 *      ld_dh) and d_dR [num_rel x dim] (row stride ld_dr), every row written (zero where nothing contributes),
 *      summed in a fixed order (bit-identical from run to run).  Rounding to bf16 is differentiated as the identity.
 *
 *      dn_decoder_scores: device pointer and strides (in floats) of the negatives' scores of the last forward,
 *      score of edge e against negative n = d_scores[(e / chunk) * chunk_stride + (e % chunk) * row_stride + n].
 *      The forward pass does not keep the scores (only each row's log-sum-exp): this call computes them, for both
 *      sides, asynchronously on `stream` from the operands of the last forward, into the decoder's workspace.
 *      dn_decoder_status WAITS for `stream`.  All other calls are asynchronous on `stream`. */
typedef struct dn_decoder dn_decoder;
DN_API int  dn_decoder_workspace_size(int64_t max_edges, int32_t chunk, int32_t num_neg, int32_t dim, int64_t max_rows,
                                      int64_t num_rel, size_t* bytes);
DN_API int  dn_decoder_create(dn_decoder** out, int64_t max_edges, int32_t chunk, int32_t num_neg, int32_t dim,
                              int64_t max_rows, int64_t num_rel, void* d_workspace, size_t workspace_bytes, void* stream);
DN_API void dn_decoder_destroy(dn_decoder* d);
DN_API int  distmult_forward(dn_decoder* d, const float* d_H, int64_t ldh, int64_t n_rows, const float* d_R, int64_t ldr,
                             const int32_t* d_src, const int32_t* d_rel, const int32_t* d_dst, int64_t n_edges,
                             const int32_t* d_neg, float* d_pos, float* d_loss, void* stream);
DN_API int  distmult_backward(dn_decoder* d, float* d_dH, int64_t ld_dh, float* d_dR, int64_t ld_dr, void* stream);
DN_API int  dn_decoder_scores(const dn_decoder* d, int32_t side, const float** d_scores, int64_t* chunk_stride,
                              int64_t* row_stride, void* stream);
DN_API int  dn_decoder_status(const dn_decoder* d, int32_t* flags, void* stream);

/* ---- dn_train_steps: several mini-batches in flight, scheduled by the library (Section 3: the mini-batch pipeline keeps
 *      construction and compute of different mini-batches busy at once; here on one device).
 *      A node-classification training step is the chain dense_sample -> sage_forward_table -> dn_softmax_xent ->
 *      sage_backward on one (batch, model) pair; a mini-batch of a thousand targets is a chain of some thirty short
 *      kernels, most of them too small to fill the device, so independent chains are run side by side.  steps[i] runs
 *      on internal stream i % n_streams (1 <= n_streams <= 16; the library creates them once per device, default
 *      priority): steps that share a dn_batch / dn_model must therefore be n_streams apart (they then follow each other
 *      on one stream); steps on different streams must use different batch and model objects and output buffers.  The
 *      internal streams first wait for everything enqueued on `stream`, and `stream` afterwards waits for all of them,
 *      so the call behaves like one asynchronous operation on `stream` (it can also be captured into a HIP graph).
 *      Fields as in the calls named above; d_dH0 may be NULL.  d_grad_out: fp32 [n_targets x dims[k]] scratch for
 *      dL/dH^k.  Results are those of the same calls made one after the other (bit for bit). */
typedef struct dn_train_step {
    dn_batch* batch;
    dn_model* model;
    const dn_graph* graph;
    const int32_t* d_targets;
    int32_t n_targets;
    uint64_t seed;
    const void* d_table;          /* lookup table of the model's in_dtype, row stride ld_elems */
    int64_t ld_elems;
    float* d_out;                 /* [n_targets x dims[k]] logits */
    const int32_t* d_labels;      /* [n_targets] */
    float grad_scale;
    float* d_loss;                /* [n_targets] */
    float* d_grad_out;            /* [n_targets x dims[k]] */
    float* const* d_dw_self;      /* host arrays of k device pointers, as for sage_backward */
    float* const* d_dw_nbr;
    float* const* d_dbias;
    float* d_dH0;
    int32_t forward_only;         /* 1: stop after sage_forward_table (sample + gather + forward) */
} dn_train_step;
DN_API int  dn_train_steps(const dn_train_step* steps, int32_t n_steps, int32_t n_streams, void* stream);

/* ---- per-kernel timing for benchmarks (off by default; not a step of the path).
 *      dn_profile_enable(1): from now on every kernel launch of this library is bracketed by a pair of
 *      HIP events on the stream it is launched on; dn_profile_enable(0) stops that.  Enabling also
 *      discards earlier records.  dn_profile_collect WAITS for the device, adds up the elapsed time per
 *      kernel tag (with three percentiles of the single brackets) and writes up to `max_entries` entries;
 *      *n_entries = number of distinct tags. */
typedef struct dn_kernel_time {
    char    tag[48];     /* e.g. "gather", "aggregate_L1", "gemm_fwd_L1" */
    double  total_ms;
    int64_t launches;
    double  p10_ms, p50_ms, p90_ms;   /* 10th, 50th and 90th percentile of the launches' brackets */
} dn_kernel_time;
DN_API int  dn_profile_enable(int32_t enable);
/* A plain device-to-device streaming copy (kernel k_calibration_copy) of `bytes` bytes (multiple of 16,
 * 16-byte aligned pointers): the known-size reference that hardware byte counters are scaled by. */
DN_API int  dn_profile_calibration_copy(void* d_dst, const void* d_src, size_t bytes, void* stream);
/* Records an event pair with nothing in between under the tag "empty_bracket": what a bracket costs by
 * itself, to be subtracted from the per-kernel averages; then a pair around a one-wave kernel that does
 * nothing under the tag "noop_kernel_bracket": the difference is the latency of a launch as such, which every
 * bracketed kernel's figure still contains. */
DN_API int  dn_profile_empty_bracket(void* stream);
/* Diagnostic for dn_train_steps' streams (HIP does not tell which hardware queue a stream runs on, and two streams on
 * one queue take turns): eight rounds of one single-wave kernel that busy-waits kernel_us microseconds on each of the
 * first n_streams step streams; *elapsed_us = best time per round of five tries.  About kernel_us if the streams run
 * side by side, a multiple of it if some share a queue.  WAITS for the device.  DN_ESTATE before dn_train_steps has
 * created that many streams. */
DN_API int  dn_profile_step_stream_overlap(int32_t n_streams, int32_t kernel_us, double* elapsed_us);
DN_API int  dn_profile_collect(dn_kernel_time* out, int32_t max_entries, int32_t* n_entries);

#ifdef __cplusplus
}
#endif
#endif /* DENSE_MI355X_H */
