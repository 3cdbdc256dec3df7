// GraphSage-mean encoder over DENSE: the memory-bound half (Algorithm 3 of the paper with mean
// aggregation, its transpose for the backward pass, and the small reshaping kernels around the
// MFMA GEMMs), and the per-layer orchestration of forward and backward.
//
// Algorithm 2 (drop the first Delta and rebase after every layer) moves no data here: layer i
// reads input rows at (position - node_id_offsets[i-1]) and writes rows at
// (position - node_id_offsets[i]); repr_map is kept relative to the full node_ids.
#include "dn_internal.h"
#include <algorithm>

namespace {

constexpr int TPB = 256;

__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ float load_elem(const uint16_t* p) { return bf16_to_f32(*p); }

// ---------------------------------------------------------------- forward aggregation
// One group of LANES lanes per output row; lane handles columns lane*V .. lane*V+V-1, then
// +LANES*V, ...  The neighbour sum runs over the row's slots in ascending order in fp32 and is
// divided by the count in fp32 (this fixes the value that gets rounded to bf16).
// Writes the A operand of the layer's GEMM, X[row] = [ self | mean ] as bf16, followed for
// TERMS == 2 by the bf16 of what the first rounding left over, [ self_lo | mean_lo ]; and the
// L2 norm of the row (bound of the accumulation error of its dot products).
// TABLE: H is the feature table itself (row stride ldh) and rows are addressed by node id, node_ids[p] for
// the row's own representation and nbrs[j] for slot j, instead of by position in a gathered H^0; the values
// read, and so every result, are the same.  mean = 0 gives the additive aggregation of Algorithm 3 as printed.
template <typename TIN, int V, int LANES, int TERMS, bool TABLE>
__global__ __launch_bounds__(TPB) void k_aggregate(const int32_t* __restrict__ hdr, int layer,
                                                   const int32_t* __restrict__ nbr_offsets,
                                                   const int32_t* __restrict__ repr_map, const TIN* __restrict__ H,
                                                   int64_t ldh, const int32_t* __restrict__ node_ids,
                                                   const int32_t* __restrict__ nbrs, int mean_agg,
                                                   int d, uint16_t* __restrict__ X, int kp, float* __restrict__ rownorm,
                                                   int32_t* __restrict__ fix_count)
{
    const int N = hdr[HDR_N];
    const int off_in = hdr[HDR_NODE_OFF + layer - 1];     // H row 0 = node_ids position off_in
    const int off_out = hdr[HDR_NODE_OFF + layer];
    const int off1 = hdr[HDR_NODE_OFF + 1];
    const int rows = N - off_out;
    const int lane = threadIdx.x % LANES;
    constexpr int GROUPS = TPB / LANES;
    // the first kernel of a forward pass clears the counters of exact recomputations that its ReLU layers add to
    if (layer == 1 && blockIdx.x == 0 && threadIdx.x < DN_FIX_SLOTS) fix_count[DN_FIX_FIRST + DN_FIX_STRIDE * threadIdx.x] = 0;
    for (int ro = blockIdx.x * GROUPS + threadIdx.x / LANES; ro < rows; ro += gridDim.x * GROUPS) {
        const int p = off_out + ro;
        const int q = p - off1;
        const int beg = nbr_offsets[q], end = nbr_offsets[q + 1];
        const float cnt_f = (float)(end - beg);
        const TIN* self = TABLE ? H + (int64_t)node_ids[p] * ldh : H + (int64_t)(p - off_in) * ldh;
        uint16_t* xrow = X + (int64_t)ro * kp;
        float sq = 0.f;
        const int iters = (d + LANES * V - 1) / (LANES * V);      // the same for every lane: the shuffles below need the whole group
        for (int it = 0; it < iters; ++it) {
            const int c0 = (it * LANES + lane) * V;
            const bool col_ok = c0 < d;
            const int cc = col_ok ? c0 : 0;                        // lanes beyond the row read its first columns and drop them
            float acc[V], sv[V];
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] = 0.f;
            // the row's own values are fetched now, so that their latency overlaps the walk over the slots
#pragma unroll
            for (int e = 0; e < V; ++e) sv[e] = load_elem(self + cc + e);
            // The group's lanes fetch the slots' row numbers side by side and hand them round by shuffles, so that the
            // row loads of up to eight slots are in flight at once; the additions keep the ascending slot order.
            for (int base = beg; base < end; base += LANES) {
                const int t = base + lane;
                int row = 0;
                if (t < end) row = TABLE ? nbrs[t] : repr_map[t] - off_in;
                const int cnt = min(LANES, end - base);
                for (int l = 0; l < cnt; l += 8) {
                    float v[8][V];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int ru = __shfl(row, min(l + u, cnt - 1), LANES);
                        const TIN* nb = H + (int64_t)ru * ldh + cc;
#pragma unroll
                        for (int e = 0; e < V; ++e) v[u][e] = load_elem(nb + e);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (l + u < cnt) {
#pragma unroll
                            for (int e = 0; e < V; ++e) acc[e] += v[u][e];
                        }
                }
            }
            if (!col_ok) continue;
            // the lane's V values of each block of the row leave in one store (V = 4 only with d a multiple of 4, and
            // rows of X start on 128-byte boundaries: 8-byte aligned); as 2-byte stores they were 8 to 16 store
            // instructions per lane
            uint16_t o_sh[V], o_mh[V], o_sl[V], o_ml[V];
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float mean = end > beg ? (mean_agg ? acc[e] / cnt_f : acc[e]) : 0.f;
                const uint16_t s_hi = f32_to_bf16(sv[e]), m_hi = f32_to_bf16(mean);
                o_sh[e] = s_hi;
                o_mh[e] = m_hi;
                const float s_hf = bf16_to_f32(s_hi), m_hf = bf16_to_f32(m_hi);
                sq += s_hf * s_hf + m_hf * m_hf;
                o_sl[e] = 0; o_ml[e] = 0;
                if (TERMS == 2) {
                    const uint16_t s_lo = f32_to_bf16(sv[e] - s_hf), m_lo = f32_to_bf16(mean - m_hf);
                    o_sl[e] = s_lo;
                    o_ml[e] = m_lo;
                    const float s_lf = bf16_to_f32(s_lo), m_lf = bf16_to_f32(m_lo);
                    sq += s_lf * s_lf + m_lf * m_lf;
                }
            }
            auto put = [&](uint16_t* dst, const uint16_t (&o)[V]) {
                if constexpr (V == 4) {
                    *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
                } else {
#pragma unroll
                    for (int e = 0; e < V; ++e) dst[e] = o[e];
                }
            };
            put(xrow + c0, o_sh);
            put(xrow + d + c0, o_mh);
            if (TERMS == 2) {
                put(xrow + 2 * d + c0, o_sl);
                put(xrow + 3 * d + c0, o_ml);
            }
        }
#pragma unroll
        for (int o = LANES / 2; o > 0; o >>= 1) sq += __shfl_xor(sq, o, LANES);
        if (lane == 0) rownorm[ro] = sqrtf(sq) * 1.0001f;
    }
}

// ---------------------------------------------------------------- backward: dZ and db of the last layer
// Tile of 64 rows x 64 columns per workgroup (striding over the row tiles beyond the grid).
// dZ = G (.) [H > 0] (ReLU layers) or G.  Writes the bf16 terms of dZ row-major [rows x TERMS*np] (hi block, then
// lo block; zero in the padding columns) and the workgroup's column sums of the unrounded dZ for the bias gradient.
// Only the layer that receives the caller's gradient runs this (its dZ is one bf16 term, so its bias gradient
// cannot come from the terms); for the others the backward aggregation of the layer above writes dZ itself
// (GradSink::dzb) and the weight-gradient GEMM sums the two terms' columns.
template <int TERMS>
__global__ __launch_bounds__(TPB) void k_dz(const int32_t* __restrict__ hdr, int layer, const float* __restrict__ G, int ldg,
                                            const float* __restrict__ Hout, int d_out, int np, int relu,
                                            uint16_t* __restrict__ dzb, float* __restrict__ db_partial)
{
    __shared__ float colsum[4][64];
    const int rows = hdr[HDR_N] - hdr[HDR_NODE_OFF + layer];
    const int c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;    // ty: 0..3
    const int nz = TERMS * np;
    const int n = c0 + tx;
    float csum = 0.f;                    // this thread's column sum over all row tiles of this workgroup, in order
    for (int rt = blockIdx.y; rt * 64 < rows; rt += gridDim.y) {
        const int r0 = rt * 64;
        // the thread's 16 rows are requested together (one after the other, each load waited for, they took most of
        // the kernel's 5 us); the sums keep the order of the rows
        float g[16], h[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int r = r0 + ty + 4 * u;
            const bool ok = r < rows && n < d_out;
            g[u] = ok ? G[(int64_t)r * ldg + n] : 0.f;
            h[u] = (ok && relu) ? Hout[(int64_t)r * d_out + n] : 1.f;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int r = r0 + ty + 4 * u;
            if (r >= rows) break;
            const float v = (h[u] > 0.f) ? g[u] : 0.f;
            csum += v;
            const uint16_t hi = f32_to_bf16(v);
            dzb[(int64_t)r * nz + n] = hi;
            if (TERMS == 2) dzb[(int64_t)r * nz + np + n] = f32_to_bf16(v - bf16_to_f32(hi));
        }
    }
    // one partial column sum per workgroup that had row tiles (the reduction reads min(gridDim.y, tiles) of them)
    if ((int)blockIdx.y * 64 < rows) {
        colsum[ty][tx] = csum;
        __syncthreads();
        if (ty == 0 && n < d_out)
            db_partial[(int64_t)blockIdx.y * d_out + n] = (colsum[0][tx] + colsum[1][tx]) + (colsum[2][tx] + colsum[3][tx]);
    }
}

// ---------------------------------------------------------------- backward aggregation (transpose of the mean)
// One group of lanes per INPUT row r of the layer: G_in[r] = dX_self[r] (if r is also an output
// row) + sum over the slots that read r, in ascending slot order, of dX_mean[owner] / count[owner].
// tr_ptr / tr_val: slots grouped by the node_ids position they read, ascending within a group;
// a layer's slots are those >= its first slot, i.e. a suffix of every group.
// where the input gradient of a row goes: into G_in, or straight into the lookup table as a plain SGD step
// (learnable base representations; product and difference rounded separately, as dn_embedding_sgd does)
struct GradSink {
    float* gin;                  // [rows_in x d], or null
    float* table; int64_t ld;    // update mode: table[node_ids[p], :] -= lr * gradient
    const int32_t* node_ids;
    float lr;
    // dZ mode (the layer below has a ReLU): the row is the gradient with respect to H of the layer below; masked
    // by [H > 0] it IS that layer's dZ, which goes out as two bf16 terms [rows x 2*np] (hi block, lo block)
    // without a pass of its own.  hmask = that layer's output H [rows x d].
    uint16_t* dzb; int nz, np; const float* hmask;
};
__device__ __forceinline__ void sink_store(const GradSink& k, int r, int p, int d, int c, float v)
{
#pragma clang fp contract(off)
    if (k.dzb) {
        if (!(k.hmask[(int64_t)r * d + c] > 0.f)) v = 0.f;
        const uint16_t hi = f32_to_bf16(v);
        k.dzb[(int64_t)r * k.nz + c] = hi;
        k.dzb[(int64_t)r * k.nz + k.np + c] = f32_to_bf16(v - bf16_to_f32(hi));
    } else if (k.table) {
        float* w = k.table + (int64_t)k.node_ids[p] * k.ld + c;
        const float step = k.lr * v;
        *w = *w - step;
    } else {
        k.gin[(int64_t)r * d + c] = v;
    }
}
// V consecutive columns starting at c0 (V = 4: one 16-byte access when the table's rows allow it)
// `w` / `old`: the table row's four values at c0, fetched by the caller before it walked the slots (null: not fetched)
// dZ mode: with `mask_fetched`, `old` holds the four values of the mask row at c0 instead
template <int V>
__device__ __forceinline__ void sink_store_vec(const GradSink& k, int r, int p, int d, int c0, const float (&v)[V],
                                               float4* w, float4 old, bool mask_fetched = false)
{
#pragma clang fp contract(off)
    if (w) {
        const float s0 = k.lr * v[0], s1 = k.lr * v[1], s2 = k.lr * v[2], s3 = k.lr * v[3];
        old.x = old.x - s0; old.y = old.y - s1; old.z = old.z - s2; old.w = old.w - s3;
        *w = old;
        return;
    }
    if constexpr (V == 4) if (k.dzb) {
        // four columns at once: one 16-byte read of the mask row, two 8-byte stores (d and np are multiples of 4 here)
        const float4 h = mask_fetched ? old : *reinterpret_cast<const float4*>(k.hmask + (int64_t)r * d + c0);
        const float hv[4] = {h.x, h.y, h.z, h.w};
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float z = hv[e] > 0.f ? v[e] : 0.f;
            hi[e] = f32_to_bf16(z);
            lo[e] = f32_to_bf16(z - bf16_to_f32(hi[e]));
        }
        uint16_t* row = k.dzb + (int64_t)r * k.nz + c0;
        *reinterpret_cast<uint2*>(row) = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
        *reinterpret_cast<uint2*>(row + k.np) = make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
        return;
    }
#pragma unroll
    for (int e = 0; e < V; ++e) sink_store(k, r, p, d, c0 + e, v[e]);
}

constexpr int HUB_ENTRIES_PER_BLOCK = 4;
template <int V, int LANES, int ITERS>
__global__ __launch_bounds__(TPB) void k_aggregate_bwd(int32_t* __restrict__ hdr, int layer,
                                                       const int32_t* __restrict__ nbr_offsets,
                                                       const int32_t* __restrict__ tr_ptr, const int32_t* __restrict__ tr_val,
                                                       const int32_t* __restrict__ tr_own, const float* __restrict__ tr_inv,
                                                       const int32_t* __restrict__ tr_long, int n_long, int row_blocks,
                                                       int mean_agg,
                                                       const float* __restrict__ dX, int ldx, int d,
                                                       GradSink sink)
{
    // The transpose index must be the one built for the sample in the workspace (and cover layer 1's slots if this
    // is layer 1).  The host checks that when it launches eagerly; a captured graph replayed after another sample has
    // been drawn into the batch (without the build in the graph) is caught here: flag it and touch nothing.
    if (hdr[HDR_TR_SEQ] != hdr[HDR_SAMPLE_SEQ] || (layer == 1 && hdr[HDR_TR_ALL] == 0)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&hdr[HDR_STATUS], ST_STALE_INDEX);
        return;
    }
    const int N = hdr[HDR_N];
    const int off_in = hdr[HDR_NODE_OFF + layer - 1];
    const int off_out = hdr[HDR_NODE_OFF + layer];
    const int off1 = hdr[HDR_NODE_OFF + 1];
    const int rows_in = N - off_in;
    const int first_slot = nbr_offsets[off_out - off1];      // first slot owned by this layer's output rows
    const int lane = threadIdx.x % LANES;
    constexpr int GROUPS = TPB / LANES;
    const float* dXm = dX + (int64_t)(off1 - off_out) * ldx + d;     // row q of this: dX_mean of owner q

    if ((int)blockIdx.x >= row_blocks) {
        // Rows read by more than DN_LONG_GROUP slots (hubs): each workgroup after the row blocks looks at a few
        // entries of the register of such rows and sums the rows it finds there with all of its lanes.
        // Lane group g takes the slots g, g + GROUPS, ... in ascending order, four in flight; the groups' sums are
        // added in order of g.
        __shared__ float part[GROUPS][LANES * V * ITERS];
        const int g = threadIdx.x / LANES;
        {
            const int c0 = ((int)blockIdx.x - row_blocks) * HUB_ENTRIES_PER_BLOCK;
            for (int f = 0; f < HUB_ENTRIES_PER_BLOCK; ++f) {
                const int entry = c0 + f < n_long ? tr_long[c0 + f] : 0;
                if (entry <= off_in || entry > N) continue;    // none, or a row that is no input of this layer
                const int p = entry - 1;
                const int r = p - off_in;
                const int beg = tr_ptr[p], end = tr_ptr[p + 1];
                // the register is not cleared between batches by every form of the index build: an entry counts only if
                // row p is such a row in THIS index and its group starts in this entry's block of slots
                if (end - beg <= DN_LONG_GROUP || beg / DN_LONG_GROUP != c0 + f) continue;
                float acc[ITERS][V];
#pragma unroll
                for (int it = 0; it < ITERS; ++it)
#pragma unroll
                    for (int e = 0; e < V; ++e) acc[it][e] = 0.f;
                for (int t0 = beg + g; t0 < end; t0 += 4 * GROUPS) {
                    int q[4];
                    float inv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int t = t0 + u * GROUPS;
                        const bool valid = t < end && tr_val[t] >= first_slot;
                        q[u] = valid ? tr_own[t] : -1;
                        inv[u] = valid ? (mean_agg ? tr_inv[t] : 1.f) : 0.f;
                    }
                    float v[4][ITERS][V];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int it = 0; it < ITERS; ++it) {
                            const int c0v = (it * LANES + lane) * V;
#pragma unroll
                            for (int e = 0; e < V; ++e) v[u][it][e] = (q[u] >= 0 && c0v < d) ? dXm[(int64_t)q[u] * ldx + c0v + e] : 0.f;
                        }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int it = 0; it < ITERS; ++it)
#pragma unroll
                            for (int e = 0; e < V; ++e) acc[it][e] += v[u][it][e] * inv[u];
                }
#pragma unroll
                for (int it = 0; it < ITERS; ++it)
#pragma unroll
                    for (int e = 0; e < V; ++e) part[g][(it * LANES + lane) * V + e] = acc[it][e];
                __syncthreads();
                for (int c = threadIdx.x; c < d; c += TPB) {
                    float tot = (p >= off_out) ? dX[(int64_t)(p - off_out) * ldx + c] : 0.f;
                    for (int w = 0; w < GROUPS; ++w) tot += part[w][c];
                    sink_store(sink, r, p, d, c, tot);
                }
                if (sink.dzb)                                  // the padding columns of both terms stay zero
                    for (int c = d + threadIdx.x; c < sink.np; c += TPB) {
                        sink.dzb[(int64_t)r * sink.nz + c] = 0;
                        sink.dzb[(int64_t)r * sink.nz + sink.np + c] = 0;
                    }
                __syncthreads();
            }
        }
        return;
    }

    // A small lane group per row (each lane carries up to ITERS pieces of V columns) keeps many rows in flight per
    // wave: the row's chain of dependent loads (tr_ptr -> slot info -> dX rows) is what bounds this kernel.
    for (int r = blockIdx.x * GROUPS + threadIdx.x / LANES; r < rows_in; r += row_blocks * GROUPS) {
        const int p = off_in + r;
        const int beg = tr_ptr[p], end = tr_ptr[p + 1];
        if (end - beg > DN_LONG_GROUP) continue;             // left to a workgroup of its own (above)
        // update mode: the table row is fetched now, so that its latency overlaps the walk over the slots
        float4* wrow = nullptr;
        float4 wold = {0.f, 0.f, 0.f, 0.f};
        if (V == 4 && ITERS == 1 && sink.table && (sink.ld & 3) == 0 && lane * V < d) {
            wrow = reinterpret_cast<float4*>(sink.table + (int64_t)sink.node_ids[p] * sink.ld + lane * V);
            wold = *wrow;
        }
        // dZ mode: likewise the row of the ReLU mask
        const bool mask_fetched = V == 4 && ITERS == 1 && sink.dzb != nullptr && lane * V < d;
        if (mask_fetched) wold = *reinterpret_cast<const float4*>(sink.hmask + (int64_t)r * d + lane * V);
        float acc[ITERS][V];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int c0 = (it * LANES + lane) * V;
#pragma unroll
            for (int e = 0; e < V; ++e) acc[it][e] = (c0 < d && p >= off_out) ? dX[(int64_t)(p - off_out) * ldx + c0 + e] : 0.f;
        }
        // the lanes fetch the slots' owner and 1/count side by side and hand them around by shuffles; the sums run
        // in ascending slot order
        for (int base = beg; base < end; base += LANES) {
            const int t = base + lane;
            const bool valid = t < end && tr_val[t] >= first_slot;
            const int q = valid ? tr_own[t] : -1;
            const float inv = valid ? (mean_agg ? tr_inv[t] : 1.f) : 0.f;
            const int cnt = min(LANES, end - base);
            if (ITERS == 1) {
                // rows with many slots: four gradient rows in flight at a time (a slot that does not count reads the
                // first row with weight 0); the rest one by one
                const int c0 = lane * V;
                const int cc = c0 < d ? c0 : 0;
                int l = 0;
                for (; l + 4 <= cnt; l += 4) {
                    float v[4][V], w[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int ql = __shfl(q, l + u, LANES);
                        w[u] = ql >= 0 ? __shfl(inv, l + u, LANES) : 0.f;
                        const float* src = (ql >= 0 ? dXm + (int64_t)ql * ldx : dX + d) + cc;
#pragma unroll
                        for (int e = 0; e < V; ++e) v[u][e] = src[e];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (w[u] != 0.f) {
#pragma unroll
                            for (int e = 0; e < V; ++e) acc[0][e] += v[u][e] * w[u];
                        }
                }
                for (; l < cnt; ++l) {
                    const int ql = __shfl(q, l, LANES);
                    const float il = __shfl(inv, l, LANES);
                    if (ql < 0 || c0 >= d) continue;
                    const float* src = dXm + (int64_t)ql * ldx + c0;
#pragma unroll
                    for (int e = 0; e < V; ++e) acc[0][e] += src[e] * il;
                }
            } else {
                for (int l = 0; l < cnt; ++l) {
                    const int ql = __shfl(q, l, LANES);
                    const float il = __shfl(inv, l, LANES);
                    if (ql < 0) continue;
                    const float* src = dXm + (int64_t)ql * ldx;
#pragma unroll
                    for (int it = 0; it < ITERS; ++it) {
                        const int c0 = (it * LANES + lane) * V;
                        if (c0 < d) {
#pragma unroll
                            for (int e = 0; e < V; ++e) acc[it][e] += src[c0 + e] * il;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int c0 = (it * LANES + lane) * V;
            if (c0 < d) {
                sink_store_vec<V>(sink, r, p, d, c0, acc[it], wrow, wold, mask_fetched);
            }
        }
        if (sink.dzb)                                          // the padding columns of both terms stay zero
            for (int c = d + lane; c < sink.np; c += LANES) {
                sink.dzb[(int64_t)r * sink.nz + c] = 0;
                sink.dzb[(int64_t)r * sink.nz + sink.np + c] = 0;
            }
    }
}

template <typename TIN, int TERMS, bool TABLE>
int launch_aggregate_t(const dn_model* m, const dn_batch* b, int i, const TIN* H, int64_t ldh, hipStream_t st)
{
    const dn_layer_bufs& L = m->layer[i - 1];
    const int d = L.d_in;
    uint16_t* X = reinterpret_cast<uint16_t*>(L.x);
    const bool vec4 = (d % 4 == 0);
    int lanes = 4;
    const int per = vec4 ? 4 : 1;
    while (lanes * per < d && lanes < 64) lanes <<= 1;
    const int groups = TPB / lanes;
    int64_t grid = (L.rows_cap + groups - 1) / groups;
    if (grid > 8192) grid = 8192;
    if (grid < 1) grid = 1;
    dn_prof_scope ps(TABLE ? "aggregate_table" : "aggregate", i, st);
#define DN_AGG(VV, LL)                                                                                                 \
    hipLaunchKernelGGL((k_aggregate<TIN, VV, LL, TERMS, TABLE>), dim3((int)grid), dim3(TPB), 0, st, b->hdr, i,         \
                       b->nbr_offsets, b->repr_map, H, ldh, b->node_ids, b->nbrs, m->mean_agg, d, X, L.kp, L.rownorm, \
                       m->fix_count)
    if (vec4) {
        switch (lanes) {
            case 4: DN_AGG(4, 4); break;
            case 8: DN_AGG(4, 8); break;
            case 16: DN_AGG(4, 16); break;
            case 32: DN_AGG(4, 32); break;
            default: DN_AGG(4, 64); break;
        }
    } else {
        switch (lanes) {
            case 4: DN_AGG(1, 4); break;
            case 8: DN_AGG(1, 8); break;
            case 16: DN_AGG(1, 16); break;
            case 32: DN_AGG(1, 32); break;
            default: DN_AGG(1, 64); break;
        }
    }
#undef DN_AGG
    DN_LAUNCH_CHECK("k_aggregate");
    return DN_OK;
}

int launch_aggregate_bwd(const dn_model* m, const dn_batch* b, int i, const GradSink& sink, hipStream_t st)
{
    const dn_layer_bufs& L = m->layer[i - 1];
    const int d = L.d_in;
    const bool vec4 = (d % 4 == 0);
    if (d > 1024) return dn_fail(DN_EINVAL, "aggregate_bwd: input width %d above 1024", d);
    // vec4: lanes x 4 columns cover the row (4 pieces per lane above 256 columns); otherwise 64 lanes x 1 column x 4 or 16 pieces
    int lanes = vec4 ? 4 : 64;
    if (vec4) while (lanes * 4 < d && lanes < 64) lanes <<= 1;
    const int groups = TPB / lanes;
    const int64_t rows_in_cap = i >= 2 ? m->layer[i - 2].rows_cap : b->cap_nodes;
    int64_t row_blocks = (rows_in_cap + groups - 1) / groups;
    // capacity is an upper bound that real batches stay far below: a block per eight capacity row groups, within [8192, 65536]
    int64_t want = row_blocks / 8;
    if (want < 8192) want = 8192;
    if (want > 65536) want = 65536;
    if (row_blocks > want) row_blocks = want;
    if (row_blocks < 1) row_blocks = 1;
    // a few more workgroups scan the register of hub rows (one entry per DN_LONG_GROUP transposed slots) and sum those
    const int n_long = (int)(b->cap_slots / DN_LONG_GROUP + 1);
    const int hub_blocks = (n_long + HUB_ENTRIES_PER_BLOCK - 1) / HUB_ENTRIES_PER_BLOCK;
    const int64_t grid = row_blocks + hub_blocks;
    dn_prof_scope ps("aggregate_bwd", i, st);
#define DN_AGGB(VV, LL, II)                                                                                           \
    hipLaunchKernelGGL((k_aggregate_bwd<VV, LL, II>), dim3((int)grid), dim3(TPB), 0, st, b->hdr, i, b->nbr_offsets,   \
                       b->tr_ptr, b->tr_val[0], b->tr_own, b->tr_inv, b->tr_long, n_long, (int)row_blocks, m->mean_agg, m->dx,  \
                       2 * d, d, sink)
    if (vec4 && d <= 256) {
        switch (lanes) {
            case 4: DN_AGGB(4, 4, 1); break;
            case 8: DN_AGGB(4, 8, 1); break;
            case 16: DN_AGGB(4, 16, 1); break;
            case 32: DN_AGGB(4, 32, 1); break;
            default: DN_AGGB(4, 64, 1); break;
        }
    } else if (vec4) {
        DN_AGGB(4, 64, 4);
    } else if (d <= 256) {
        DN_AGGB(1, 64, 4);
    } else {
        DN_AGGB(1, 64, 16);
    }
#undef DN_AGGB
    DN_LAUNCH_CHECK("k_aggregate_bwd");
    return DN_OK;
}

}  // namespace

int dn_launch_forward(dn_model* m, const dn_batch* b, const void* h0, int64_t ldh, int from_table, float* out, hipStream_t st)
{
    const int k = m->k;
    for (int i = 1; i <= k; ++i) {
        int rc;
        if (i == 1 && m->in_dtype == DN_BF16)
            rc = from_table ? launch_aggregate_t<uint16_t, 1, true>(m, b, 1, static_cast<const uint16_t*>(h0), ldh, st)
                            : launch_aggregate_t<uint16_t, 1, false>(m, b, 1, static_cast<const uint16_t*>(h0), ldh, st);
        else if (i == 1)
            rc = from_table ? launch_aggregate_t<float, 1, true>(m, b, 1, static_cast<const float*>(h0), ldh, st)
                            : launch_aggregate_t<float, 1, false>(m, b, 1, static_cast<const float*>(h0), ldh, st);
        else if (dn_layer_is_fused(m, i) && b->cap_slots > 0) {
            // aggregation, linear map, bias and ReLU of the layer in one launch
            const dn_layer_bufs& Lf = m->layer[i - 1];
            rc = dn_launch_layer_fused(m, b, i, i == k ? out : Lf.h, Lf.d_out, st);
            if (rc) return rc;
            continue;
        } else
            rc = launch_aggregate_t<float, 2, false>(m, b, i, m->layer[i - 2].h, m->layer[i - 1].d_in, st);
        if (rc) return rc;
        const dn_layer_bufs& L = m->layer[i - 1];
        rc = dn_gemm_forward(m, b, i, i == k ? out : L.h, L.d_out, st);
        if (rc) return rc;
    }
    return DN_OK;
}

int dn_launch_backward(dn_model* m, dn_batch* b, const float* grad_out, float* const* dws,
                       float* const* dwn, float* const* dbias, float* dh0, float* sgd_table, int64_t sgd_ld, float sgd_lr,
                       hipStream_t st)
{
    const int k = m->k;
    const bool need_input_grad = dh0 != nullptr || sgd_table != nullptr;
    int rc = dn_launch_transpose_index(b, need_input_grad, st);     // no-op when prepared for this sample
    if (rc) return rc;
    // The chain that carries the gradient down the layers comes first: dZ^i -> dX^i -> transpose of
    // the mean -> dZ^{i-1}.  What nothing downstream waits for (the dW GEMMs, the reductions of dW and db)
    // follows in two launches that cover all layers; every layer has its own operands.
    {
        // dZ of the last layer from the caller's gradient (no activation there)
        const dn_layer_bufs& L = m->layer[k - 1];
        unsigned row_tiles = (unsigned)((L.rows_cap + 63) / 64);
        if (row_tiles > DN_DZ_MAX_ROW_BLOCKS) row_tiles = DN_DZ_MAX_ROW_BLOCKS;   // the kernel strides over the row tiles beyond the grid
        dn_prof_scope ps("dz", k, st);
        if (L.zterms == 2)
            hipLaunchKernelGGL((k_dz<2>), dim3((unsigned)(L.np / 64), row_tiles ? row_tiles : 1), dim3(TPB), 0, st, b->hdr,
                               k, grad_out, L.d_out, nullptr, L.d_out, L.np, 0, reinterpret_cast<uint16_t*>(L.dzb), L.db_partial);
        else
            hipLaunchKernelGGL((k_dz<1>), dim3((unsigned)(L.np / 64), row_tiles ? row_tiles : 1), dim3(TPB), 0, st, b->hdr,
                               k, grad_out, L.d_out, nullptr, L.d_out, L.np, 0, reinterpret_cast<uint16_t*>(L.dzb), L.db_partial);
    }
    DN_LAUNCH_CHECK("k_dz");
    for (int i = k; i >= 1; --i) {
        if (i == 1 && !need_input_grad) break;          // nothing consumes the input gradient of layer 1
        rc = dn_gemm_dx(m, b, i, st);
        if (rc) return rc;
        GradSink sink = { dh0, nullptr, 0, b->node_ids, 0.f, nullptr, 0, 0, nullptr };
        if (i == 1) {
            if (sgd_table) { sink.gin = nullptr; sink.table = sgd_table; sink.ld = sgd_ld; sink.lr = sgd_lr; }
        } else {
            // the gradient with respect to H^{i-1}, masked by its ReLU, is dZ^{i-1}: written as that layer's bf16 terms
            const dn_layer_bufs& Lb = m->layer[i - 2];
            sink.gin = nullptr;
            sink.dzb = reinterpret_cast<uint16_t*>(Lb.dzb); sink.nz = Lb.nz; sink.np = Lb.np; sink.hmask = Lb.h;
        }
        rc = launch_aggregate_bwd(m, b, i, sink, st);
        if (rc) return rc;
    }
    return dn_gemm_dw_all(m, b, dws, dwn, dbias, st);
}
