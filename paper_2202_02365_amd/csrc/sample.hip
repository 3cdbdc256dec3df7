// DENSE construction on the device: Algorithm 1 of the paper (multi-hop sampling with one-hop
// sample reuse) plus repr_map of Section 4.2, as a fixed sequence of kernels with every
// sample-dependent size kept in device memory.
//
// Per hop h (targets are level 0):
//   k_sample        one lane group per frontier node: Floyd subset over adjacency positions with
//                   Philox4x32-10 words, neighbours written sequentially at the node's offset,
//                   and every neighbour id "claimed" in two bitmaps: `seen` (all of node_ids so
//                   far) and `fresh` (first seen in this hop), with a summary bitmap over the
//                   words of `fresh` so that later passes touch only words that are in use.
//   k_fresh_count / k_fresh_emit
//                   computeNextDelta: walk the summary in ascending order, so the new Delta comes
//                   out in ascending node id without a sort; the same pass hands every new node
//                   its staging position and the offset of its future neighbour segment
//                   (exclusive sums of min(deg, fanout)), and clears the bits it consumed.
// k_assemble lays the staging arrays (level order) out in the paper's order (Delta_0 first, last
// hop's neighbours first) and translates every neighbour id to its position in node_ids.
#include "dn_internal.h"
#include <cstdlib>

namespace {
// `seen` and `fresh` are interleaved: word w of `seen` and word w of `fresh` are the two halves of one aligned
// 8-byte pair (fresh = seen + 1), so that the sampling kernel marks a node in both with one atomic.
#define BM(w) (2 * (int64_t)(w))

constexpr int TPB = 256;

struct GraphDev {
    const int64_t* rp[2];
    const int32_t* col[2];
};

// ---------------------------------------------------------------- Philox4x32-10 (Salmon et al., SC'11)
__device__ __forceinline__ uint32_t philox4x32_10_word(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                       uint32_t k0, uint32_t k1, int word)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return word == 0 ? c0 : word == 1 ? c1 : word == 2 ? c2 : c3;
}

// ---------------------------------------------------------------- block-wide helpers (256 threads)
__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive scan of one value per thread over the block; `total` gets the block sum.
__device__ __forceinline__ uint64_t block_exclusive_scan(uint64_t v, uint64_t& total, uint64_t* sm /* [TPB/64] */)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t incl = wave_inclusive_scan(v);
    if (lane == 63) sm[wave] = incl;
    __syncthreads();
    uint64_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < TPB / 64; ++w) {
        const uint64_t s = sm[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    total = tot;
    return base + incl - v;
}

// Sum of part[0 .. n) computed cooperatively by the block (the "look-behind" over the per-block
// partial sums of the previous kernel; n is at most a few thousand).
__device__ __forceinline__ uint64_t block_sum_prefix(const uint64_t* part, int n, uint64_t* sm)
{
    uint64_t acc = 0;
    for (int i = threadIdx.x; i < n; i += TPB) acc += part[i];
    uint64_t total;
    block_exclusive_scan(acc, total, sm);
    return total;
}

__device__ __forceinline__ int node_sample_count(const GraphDev& g, int u, int f, int direction)
{
    int c = 0;
    if (direction != DN_DIR_IN) {
        const int64_t d = g.rp[0][u + 1] - g.rp[0][u];
        c += d < f ? (int)d : f;
    }
    if (direction != DN_DIR_OUT) {
        const int64_t d = g.rp[1][u + 1] - g.rp[1][u];
        c += d < f ? (int)d : f;
    }
    return c;
}

__device__ __forceinline__ uint64_t pack(int nodes, int slots) { return (uint64_t)(uint32_t)nodes | ((uint64_t)(uint32_t)slots << 32); }

// ---------------------------------------------------------------- level 0: the targets
// One thread per target: copy it to the staging array, mark it seen, count its neighbour slots.
__global__ __launch_bounds__(TPB) void k_init_targets(GraphDev g, int64_t V, const int32_t* __restrict__ targets,
                                                      int n, int f0, int direction, int32_t* __restrict__ hdr,
                                                      uint32_t* __restrict__ seen, int32_t* __restrict__ lvlpos,
                                                      int32_t* __restrict__ lvl_ids, int32_t* __restrict__ lvl_nbr_offsets,
                                                      uint64_t* __restrict__ blk)
{
    __shared__ uint64_t sm[TPB / 64];
    const int i = blockIdx.x * TPB + threadIdx.x;
    int c = 0;
    if (i < n) {
        int t = targets[i];
        if (t < 0 || (int64_t)t >= V) {
            atomicOr(&hdr[HDR_STATUS_ACC], ST_BAD_TARGET);
            t = 0;                                       // keep every later access in bounds
            lvl_ids[i] = 0;
        } else {
            const uint32_t bit = 1u << (t & 31);
            const uint32_t old = atomicOr(&seen[BM(t >> 5)], bit);
            if (old & bit) atomicOr(&hdr[HDR_STATUS_ACC], ST_DUP_TARGET);
            lvl_ids[i] = t;
            lvlpos[t] = i;
            c = node_sample_count(g, t, f0, direction);
        }
        lvl_nbr_offsets[i] = c;                          // count for now; k_init_offsets turns it into an offset
    }
    uint64_t total;
    block_exclusive_scan((uint64_t)c, total, sm);
    if (threadIdx.x == 0) blk[blockIdx.x] = total;
}

__global__ __launch_bounds__(TPB) void k_init_offsets(int n, int32_t* __restrict__ hdr,
                                                      int32_t* __restrict__ lvl_nbr_offsets,
                                                      const uint64_t* __restrict__ blk)
{
    __shared__ uint64_t sm[TPB / 64];
    const uint64_t base = block_sum_prefix(blk, blockIdx.x, sm);
    const int i = blockIdx.x * TPB + threadIdx.x;
    const int c = i < n ? lvl_nbr_offsets[i] : 0;
    uint64_t total;
    const uint64_t ex = block_exclusive_scan((uint64_t)c, total, sm);
    if (i < n) lvl_nbr_offsets[i] = (int)(base + ex);
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        hdr[HDR_LVL_OFF + 0] = 0;
        hdr[HDR_LVL_OFF + 1] = n;
        hdr[HDR_LVL_NBR_OFF + 0] = 0;
        hdr[HDR_LVL_NBR_OFF + 1] = (int)(base + total);
        hdr[HDR_NTARGETS] = n;
    }
}

// Both steps in one launch for target lists of a few thousand ids: a workgroup adds up the counts of the targets in
// front of its own by itself (reading their row offsets once more: at most INIT_FUSED_MAX / TPB rounds per thread),
// so no workgroup waits for another and the second launch is gone.  Results are those of the two kernels above.
constexpr int INIT_FUSED_MAX = 4096;
__global__ __launch_bounds__(TPB) void k_init_level0(GraphDev g, int64_t V, const int32_t* __restrict__ targets,
                                                     int n, int f0, int direction, int32_t* __restrict__ hdr,
                                                     uint32_t* __restrict__ seen, int32_t* __restrict__ lvlpos,
                                                     int32_t* __restrict__ lvl_ids, int32_t* __restrict__ lvl_nbr_offsets)
{
    __shared__ uint64_t sm[TPB / 64];
    const int first = blockIdx.x * TPB;
    const int i = first + threadIdx.x;
    // the ids are requested first, the thread's own and those in front of the workgroup four at a time, then everything
    // that depends on them: two chains of dependent loads side by side instead of one after the other
    int t = i < n ? targets[i] : -1;
    const bool valid = t >= 0 && (int64_t)t < V;
    uint64_t before = 0;
    for (int j0 = threadIdx.x; j0 < first; j0 += 4 * TPB) {
        int tb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) tb[u] = j0 + u * TPB < first ? targets[j0 + u * TPB] : -1;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (tb[u] >= 0 && (int64_t)tb[u] < V) before += (uint64_t)node_sample_count(g, tb[u], f0, direction);
    }
    int c = 0;
    if (i < n) {
        if (!valid) {
            atomicOr(&hdr[HDR_STATUS_ACC], ST_BAD_TARGET);
            lvl_ids[i] = 0;                              // keeps every later access in bounds
        } else {
            const uint32_t bit = 1u << (t & 31);
            const uint32_t old = atomicOr(&seen[BM(t >> 5)], bit);
            lvl_ids[i] = t;
            lvlpos[t] = i;
            c = node_sample_count(g, t, f0, direction);
            if (old & bit) atomicOr(&hdr[HDR_STATUS_ACC], ST_DUP_TARGET);
        }
    }
    uint64_t base;
    block_exclusive_scan(before, base, sm);              // base = slots of all targets in front of this workgroup
    uint64_t total;
    const uint64_t ex = block_exclusive_scan((uint64_t)c, total, sm);
    if (i < n) lvl_nbr_offsets[i] = (int)(base + ex);
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        hdr[HDR_LVL_OFF + 0] = 0;
        hdr[HDR_LVL_OFF + 1] = n;
        hdr[HDR_LVL_NBR_OFF + 0] = 0;
        hdr[HDR_LVL_NBR_OFF + 1] = (int)(base + total);
        hdr[HDR_NTARGETS] = n;
    }
}

// ---------------------------------------------------------------- level 0 from training edges
// Link prediction (Section 2: a training example is a pair of target nodes): the targets are the
// distinct endpoints of the batch's edges plus the negative nodes.  Their ids are marked in the
// `fresh` bitmap; the ordered walk that builds every other level then yields them in ascending id.
__global__ __launch_bounds__(TPB) void k_mark_ids(int64_t V, const int32_t* __restrict__ a, int na,
                                                  const int32_t* __restrict__ b, int nb, const int32_t* __restrict__ c, int nc,
                                                  int32_t* __restrict__ hdr, uint32_t* __restrict__ fresh,
                                                  uint32_t* __restrict__ summary, unsigned long long* __restrict__ blk, int n_blk)
{
    const int total = na + nb + nc;
    const int stride = gridDim.x * TPB;
    for (int i = blockIdx.x * TPB + threadIdx.x; i < n_blk; i += stride) blk[i] = 0ull;     // as in k_sample
    for (int i = blockIdx.x * TPB + threadIdx.x; i < total; i += stride) {
        const int u = i < na ? a[i] : (i < na + nb ? b[i - na] : c[i - na - nb]);
        if (u < 0 || (int64_t)u >= V) { atomicOr(&hdr[HDR_STATUS_ACC], ST_BAD_TARGET); continue; }
        const uint32_t w = (uint32_t)u >> 5, bit = 1u << (u & 31);
        if (!(__hip_atomic_load(&fresh[BM(w)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit)) {
            const uint32_t old_word = atomicOr(&fresh[BM(w)], bit);
            if (old_word == 0) atomicOr(&summary[w >> 5], 1u << (w & 31));
        }
    }
}

// position of every endpoint / negative in the target list (= row of the encoder's output)
__global__ __launch_bounds__(TPB) void k_local_ids(int64_t V, const int32_t* __restrict__ a, int na,
                                                   const int32_t* __restrict__ b, int nb, const int32_t* __restrict__ c, int nc,
                                                   const int32_t* __restrict__ lvlpos, int32_t* __restrict__ la,
                                                   int32_t* __restrict__ lb, int32_t* __restrict__ lc)
{
    const int total = na + nb + nc;
    const int stride = gridDim.x * TPB;
    for (int i = blockIdx.x * TPB + threadIdx.x; i < total; i += stride) {
        const int u = i < na ? a[i] : (i < na + nb ? b[i - na] : c[i - na - nb]);
        const int pos = (u < 0 || (int64_t)u >= V) ? 0 : lvlpos[u];
        if (i < na) la[i] = pos;
        else if (i < na + nb) lb[i - na] = pos;
        else lc[i - na - nb] = pos;
    }
}

// ---------------------------------------------------------------- one-hop sample of a level
// G lanes cooperate on one node (G = power of two >= fanout).  Lane s owns Floyd step s: it draws
// t_s in [0, deg-f+s]; the picks are then settled in step order with a G-wide ballot, which is the
// sequential part of Floyd's algorithm ("take j if t is already in the set").
template <int G>
__global__ __launch_bounds__(TPB) void k_sample(GraphDev g, int hop, int f, int direction, uint32_t key0, uint32_t key1,
                                                const int32_t* __restrict__ hdr, const int32_t* __restrict__ lvl_ids,
                                                const int32_t* __restrict__ lvl_nbr_offsets,
                                                int32_t* __restrict__ lvl_nbrs, int32_t* __restrict__ lvl_owner,
                                                int64_t cap_slots, uint32_t* __restrict__ seen,
                                                uint32_t* __restrict__ fresh, uint32_t* __restrict__ summary,
                                                unsigned long long* __restrict__ blk, int n_blk)
{
    constexpr int GROUPS = TPB / G;
    // the totals that the workgroups of the next-Delta kernel publish to each other start at zero ("not yet there")
    for (int i = blockIdx.x * TPB + threadIdx.x; i < n_blk; i += gridDim.x * TPB) blk[i] = 0ull;
    const int lane = threadIdx.x & 63;
    const int s = threadIdx.x % G;
    const uint64_t gmask = (G == 64) ? ~0ull : (((1ull << G) - 1ull) << ((lane / G) * G));
    const int lvl_begin = hdr[HDR_LVL_OFF + hop];
    const int n = hdr[HDR_LVL_OFF + hop + 1] - lvl_begin;

    for (int gid = blockIdx.x * GROUPS + threadIdx.x / G; gid < n; gid += gridDim.x * GROUPS) {
        const int p = lvl_begin + gid;
        const int v = lvl_ids[p];
        int o = lvl_nbr_offsets[p];
#pragma unroll 1
        for (int dir = 0; dir < 2; ++dir) {
            if ((dir == 0 && direction == DN_DIR_IN) || (dir == 1 && direction == DN_DIR_OUT)) continue;
            const int64_t base = g.rp[dir][v];
            const int64_t deg = g.rp[dir][v + 1] - base;
            const int c = deg < f ? (int)deg : f;
            const bool floyd = deg > f;
            uint32_t t = 0xffffffffu, j = 0;
            if (floyd && s < f) {
                j = (uint32_t)(deg - f + s);
                const uint32_t r = philox4x32_10_word((uint32_t)(s >> 2), (uint32_t)v, (uint32_t)hop, (uint32_t)dir,
                                                      key0, key1, s & 3);
                t = __umulhi(r, j + 1u);                 // uniform in [0, j]
            }
            uint32_t pick = t;
            for (int sp = 1; sp < f; ++sp) {
                const uint32_t ts = __shfl(t, sp, G);
                const bool hit = floyd && s < sp && pick == ts;
                const uint64_t any = __ballot(hit) & gmask;
                if (s == sp && any) pick = j;
            }
            const int64_t pos = floyd ? (int64_t)pick : (int64_t)s;
            if (s < c && (int64_t)(o + s) < cap_slots) {
                const int u = g.col[dir][base + pos];
                lvl_nbrs[o + s] = u;
                lvl_owner[o + s] = p;
                const uint32_t w = (uint32_t)u >> 5, bit = 1u << (u & 31);
                // relaxed device-scope load first: hubs are claimed once and then only read.  A clear bit means the
                // node is in no earlier level (those kernels are complete), so it is new at this hop whichever lane
                // marks it first: every lane that sees it clear marks it in `seen` and in `fresh` with one 64-bit
                // atomic on the pair of words (the bitmaps end the same whoever comes first).
                if (!(__hip_atomic_load(&seen[BM(w)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit)) {
                    const unsigned long long both = (unsigned long long)bit | ((unsigned long long)bit << 32);
                    const unsigned long long old_pair = atomicOr(reinterpret_cast<unsigned long long*>(&seen[BM(w)]), both);
                    const uint32_t old_word = (uint32_t)(old_pair >> 32);
                    if (old_word == 0) atomicOr(&summary[w >> 5], 1u << (w & 31));
                }
            }
            o += c;
        }
    }
}

// ---------------------------------------------------------------- computeNextDelta
// One thread per `span` = 2^walk_shift consecutive bitmap words: a whole summary word (32 bitmap words = 1024 node
// ids) on graphs of tens of millions of nodes, fewer on small graphs, where a thread per 1024 ids would leave a level
// of ten thousand nodes to a thousand threads, each working its nodes off one dependent load after the other (measured
// 43 + 39 us for the middle hop of the 2^20-node workload).  Pass 1 counts the new nodes and the neighbour slots they
// will need at the next hop; pass 2 (k_fresh_emit) turns the counts into positions.  Both walk bits in ascending order,
// so positions follow ascending node id.
// A walker's bits of the summary: those of its own bitmap words, moved to bit 0; `full` = the whole summary word.
__device__ __forceinline__ uint32_t walker_bits(const uint32_t* __restrict__ summary, int64_t w0, int walk_shift, uint32_t& full)
{
    full = summary[w0 >> 5];
    const uint32_t mask = walk_shift >= 5 ? 0xffffffffu : ((1u << (1 << walk_shift)) - 1u);
    return (full >> (w0 & 31)) & mask;
}

__global__ __launch_bounds__(TPB) void k_fresh_count(GraphDev g, int64_t words0, int walk_shift, int f_next, int direction,
                                                     const uint32_t* __restrict__ fresh,
                                                     const uint32_t* __restrict__ summary, uint64_t* __restrict__ blk)
{
    __shared__ uint64_t sm[TPB / 64];
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    int nodes = 0, slots = 0;
    const int64_t w0 = i << walk_shift;
    if (w0 < words0) {
        uint32_t full;
        uint32_t sw = walker_bits(summary, w0, walk_shift, full);
        while (sw) {
            const int b = __ffs(sw) - 1;
            sw &= sw - 1;
            const int64_t w = w0 + b;
            uint32_t fw = fresh[BM(w)];
            nodes += __popc(fw);
            if (f_next > 0) {
                while (fw) {
                    const int bit = __ffs(fw) - 1;
                    fw &= fw - 1;
                    slots += node_sample_count(g, (int)(w * 32 + bit), f_next, direction);
                }
            }
        }
    }
    uint64_t total;
    block_exclusive_scan(pack(nodes, slots), total, sm);
    if (threadIdx.x == 0) blk[blockIdx.x] = total;
}

__global__ __launch_bounds__(TPB) void k_fresh_emit(GraphDev g, int64_t words0, int walk_shift, int next_level, int f_next, int direction,
                                                    int32_t* __restrict__ hdr, uint32_t* __restrict__ fresh,
                                                    uint32_t* __restrict__ summary, const uint64_t* __restrict__ blk,
                                                    int32_t* __restrict__ lvlpos, int32_t* __restrict__ lvl_ids,
                                                    int32_t* __restrict__ lvl_nbr_offsets, int64_t cap_nodes,
                                                    uint32_t* __restrict__ seen_or_null)
{
    __shared__ uint64_t sm[TPB / 64];
    const uint64_t before = block_sum_prefix(blk, blockIdx.x, sm);
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    // recount (the words are in cache from pass 1)
    int nodes = 0, slots = 0;
    uint32_t sw0 = 0, full = 0;
    const int64_t w0 = i << walk_shift;
    if (w0 < words0) {
        sw0 = walker_bits(summary, w0, walk_shift, full);
        uint32_t sw = sw0;
        while (sw) {
            const int b = __ffs(sw) - 1;
            sw &= sw - 1;
            const int64_t w = w0 + b;
            uint32_t fw = fresh[BM(w)];
            nodes += __popc(fw);
            if (f_next > 0) {
                while (fw) {
                    const int bit = __ffs(fw) - 1;
                    fw &= fw - 1;
                    slots += node_sample_count(g, (int)(w * 32 + bit), f_next, direction);
                }
            }
        }
    }
    uint64_t total;
    const uint64_t ex = block_exclusive_scan(pack(nodes, slots), total, sm) + before;
    const int node_base = hdr[HDR_LVL_OFF + next_level];
    const int slot_base = f_next > 0 ? hdr[HDR_LVL_NBR_OFF + next_level] : 0;
    int p = node_base + (int)(uint32_t)(ex & 0xffffffffu);
    int so = slot_base + (int)(uint32_t)(ex >> 32);
    uint32_t sw = sw0;
    while (sw) {
        const int b = __ffs(sw) - 1;
        sw &= sw - 1;
        const int64_t w = w0 + b;
        uint32_t fw = fresh[BM(w)];
        // after the last hop nothing reads `seen` any more: the pair of words is cleared together, and the final pass
        // need not come back to this level's nodes (most of a mini-batch) to clear their bits one random store each
        if (f_next == 0 && !seen_or_null) *reinterpret_cast<uint2*>(&fresh[BM(w) - 1]) = make_uint2(0u, 0u);
        else fresh[BM(w)] = 0;
        if (seen_or_null) seen_or_null[BM(w)] = fw;          // level 0 from an id set: these nodes are the targets
        while (fw) {
            const int bit = __ffs(fw) - 1;
            fw &= fw - 1;
            const int u = (int)(w * 32 + bit);
            if (p < cap_nodes) {
                lvl_ids[p] = u;
                lvlpos[u] = p;
                if (f_next > 0) {
                    lvl_nbr_offsets[p] = so;
                    so += node_sample_count(g, u, f_next, direction);
                }
            }
            ++p;
        }
    }
    // the walkers that share a summary word are neighbours in one wave and have all read it (first instruction above):
    // the one at its first bitmap word clears it
    if (full && (w0 & 31) == 0) summary[w0 >> 5] = 0;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const uint64_t all = before + total;
        int n_new = (int)(uint32_t)(all & 0xffffffffu);
        if ((int64_t)node_base + n_new > cap_nodes) {
            atomicOr(&hdr[HDR_STATUS_ACC], ST_CAPACITY);
            n_new = (int)(cap_nodes - node_base);
        }
        hdr[HDR_LVL_OFF + next_level + 1] = node_base + n_new;
        if (f_next > 0) hdr[HDR_LVL_NBR_OFF + next_level + 1] = slot_base + (int)(uint32_t)(all >> 32);
        if (seen_or_null) hdr[HDR_NTARGETS] = n_new;
    }
}

// computeNextDelta in ONE launch: count, hand the workgroup's totals to the workgroups behind it, emit.
// Workgroup b publishes pack(nodes, slots) of its id range with bit 63 set in blk[b] (one 64-bit atomic exchange at
// device scope: value and "it is there" in one word, so no fence is needed), then adds up blk[0 .. b), waiting for
// the words that are still zero (the sampling kernel in front of this one cleared them).  Every workgroup publishes
// BEFORE it waits and waits only for workgroups with a smaller number; the host launches this kernel only where all
// of them are running by then (next_delta_fused below): workgroup 0 waits for nobody, and by induction every wait
// ends.  As a second line of defence a wait gives up after ND_SPIN_MAX
// looks (far beyond the few microseconds the kernel runs): the workgroup then raises ST_INTERNAL, which
// dn_batch_counts reports, emits nothing and leaves, so the kernel ends whatever the hardware does.
constexpr unsigned long long ND_VALID = 1ull << 63;
constexpr int ND_SPIN_MAX = 1 << 20;
__global__ __launch_bounds__(TPB) void k_next_delta(GraphDev g, int64_t words0, int walk_shift, int next_level, int f_next, int direction,
                                                    int32_t* __restrict__ hdr, uint32_t* __restrict__ fresh,
                                                    uint32_t* __restrict__ summary, unsigned long long* __restrict__ blk,
                                                    int32_t* __restrict__ lvlpos, int32_t* __restrict__ lvl_ids,
                                                    int32_t* __restrict__ lvl_nbr_offsets, int64_t cap_nodes,
                                                    uint32_t* __restrict__ seen_or_null)
{
    __shared__ uint64_t sm[TPB / 64];
    __shared__ int s_gave_up;
    if (threadIdx.x == 0) s_gave_up = 0;
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    // ---- count
    int nodes = 0, slots = 0;
    uint32_t sw0 = 0, full = 0;
    const int64_t w0 = i << walk_shift;
    if (w0 < words0) {
        sw0 = walker_bits(summary, w0, walk_shift, full);
        uint32_t sw = sw0;
        while (sw) {
            const int b = __ffs(sw) - 1;
            sw &= sw - 1;
            const int64_t w = w0 + b;
            uint32_t fw = fresh[BM(w)];
            nodes += __popc(fw);
            if (f_next > 0) {
                while (fw) {
                    const int bit = __ffs(fw) - 1;
                    fw &= fw - 1;
                    slots += node_sample_count(g, (int)(w * 32 + bit), f_next, direction);
                }
            }
        }
    }
    uint64_t total;
    const uint64_t ex_local = block_exclusive_scan(pack(nodes, slots), total, sm);     // (its barriers also publish s_gave_up = 0)
    // ---- publish, then collect what lies in front
    if (threadIdx.x == 0)
        __hip_atomic_exchange(&blk[blockIdx.x], (unsigned long long)total | ND_VALID, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint64_t acc = 0;
    for (int j = threadIdx.x; j < (int)blockIdx.x; j += TPB) {
        unsigned long long v = 0;
        int spins = 0;
        while (!((v = __hip_atomic_load(&blk[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) & ND_VALID)) {
            if (++spins >= ND_SPIN_MAX) { s_gave_up = 1; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        acc += (uint64_t)(v & ~ND_VALID);
    }
    uint64_t before;
    block_exclusive_scan(acc, before, sm);
    if (s_gave_up) {                                         // read after the scan's barriers: the same for all threads
        if (threadIdx.x == 0) atomicOr(&hdr[HDR_STATUS_ACC], ST_INTERNAL);
        return;
    }
    // ---- emit (the words are in cache from the count)
    const uint64_t ex = ex_local + before;
    const int node_base = hdr[HDR_LVL_OFF + next_level];
    const int slot_base = f_next > 0 ? hdr[HDR_LVL_NBR_OFF + next_level] : 0;
    int p = node_base + (int)(uint32_t)(ex & 0xffffffffu);
    int so = slot_base + (int)(uint32_t)(ex >> 32);
    uint32_t sw = sw0;
    while (sw) {
        const int b = __ffs(sw) - 1;
        sw &= sw - 1;
        const int64_t w = w0 + b;
        uint32_t fw = fresh[BM(w)];
        // after the last hop nothing reads `seen` any more: the pair of words is cleared together, and the final pass
        // need not come back to this level's nodes (most of a mini-batch) to clear their bits one random store each
        if (f_next == 0 && !seen_or_null) *reinterpret_cast<uint2*>(&fresh[BM(w) - 1]) = make_uint2(0u, 0u);
        else fresh[BM(w)] = 0;
        if (seen_or_null) seen_or_null[BM(w)] = fw;          // level 0 from an id set: these nodes are the targets
        while (fw) {
            const int bit = __ffs(fw) - 1;
            fw &= fw - 1;
            const int u = (int)(w * 32 + bit);
            if (p < cap_nodes) {
                lvl_ids[p] = u;
                lvlpos[u] = p;
                if (f_next > 0) {
                    lvl_nbr_offsets[p] = so;
                    so += node_sample_count(g, u, f_next, direction);
                }
            }
            ++p;
        }
    }
    // the walkers that share a summary word are neighbours in one wave and have all read it (first thing above):
    // the one at its first bitmap word clears it
    if (full && (w0 & 31) == 0) summary[w0 >> 5] = 0;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const uint64_t all = before + total;
        int n_new = (int)(uint32_t)(all & 0xffffffffu);
        if ((int64_t)node_base + n_new > cap_nodes) {
            atomicOr(&hdr[HDR_STATUS_ACC], ST_CAPACITY);
            n_new = (int)(cap_nodes - node_base);
        }
        hdr[HDR_LVL_OFF + next_level + 1] = node_base + n_new;
        if (f_next > 0) hdr[HDR_LVL_NBR_OFF + next_level + 1] = slot_base + (int)(uint32_t)(all >> 32);
        if (seen_or_null) hdr[HDR_NTARGETS] = n_new;
    }
}

// Which form computeNextDelta takes.  In the one-launch form a workgroup waits for the workgroups with smaller
// numbers.  The eight XCDs work through their shares of a grid (every eighth workgroup) independently of each other,
// so a workgroup can be running while one with a smaller number, in another XCD's share, still waits for a free slot;
// if every slot it could get were held by waiting workgroups of several such kernels, none of them would ever leave
// (the bounded wait would then end the kernel with ST_INTERNAL and an unfinished level).  That cannot happen while all
// workgroups of all such kernels in flight fit the chip at once, XCD by XCD: each then holds a slot of its own and
// waits only for workgroups that run.  A compute unit holds 8 workgroups of 256 threads (the kernel needs 35 vector
// registers and 40 bytes of LDS: eight waves per SIMD); a process has as many
// kernels in flight as it has hardware queues (GPU_MAX_HW_QUEUES in the environment, 4 if it is not set: the
// runtime's default).  The one-launch form is therefore used only where
//     queues x ceil(workgroups / 8)  <=  8 x compute units / 8,
// which holds for graphs up to 134M nodes on 256 compute units with the default 4 queues (424 and 466 workgroups at
// the 111M- and 122M-node workloads); otherwise, or with DN_NEXT_DELTA_TWO_PASS=1 in the environment, two kernels
// (count, then emit), in which no workgroup waits for another.  All of it is read once per process.
static bool next_delta_fused(int grid_words)
{
    static const bool forced_two_pass = [] { const char* e = getenv("DN_NEXT_DELTA_TWO_PASS"); return e && e[0] == '1'; }();
    static const int queues = [] { const char* e = getenv("GPU_MAX_HW_QUEUES"); const int v = e ? atoi(e) : 0; return v > 0 ? v : 4; }();
    static const int slots_per_xcd = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        return cus;                                              // 8 workgroups per compute unit, 8 XCDs
    }();
    if (forced_two_pass) return false;
    return (int64_t)queues * ((grid_words + 7) / 8) <= (int64_t)slots_per_xcd;
}

// ---------------------------------------------------------------- final layout + repr_map
// staging position -> position in node_ids: level h occupies [N - LVL_OFF[h+1], N - LVL_OFF[h]).
__device__ __forceinline__ int final_node_pos(int p, const int* lvl_off, int k, int N)
{
    int h = 0;
    while (h < k && p >= lvl_off[h + 1]) ++h;
    return N - lvl_off[h + 1] + (p - lvl_off[h]);
}

__global__ __launch_bounds__(TPB) void k_assemble(int k, int32_t* __restrict__ hdr, const int32_t* __restrict__ lvl_ids,
                                                  const int32_t* __restrict__ lvl_nbr_offsets,
                                                  const int32_t* __restrict__ lvl_nbrs, const int32_t* __restrict__ lvl_owner,
                                                  const int32_t* __restrict__ lvlpos, uint32_t* __restrict__ seen,
                                                  int32_t* __restrict__ node_ids, int32_t* __restrict__ nbr_offsets,
                                                  int32_t* __restrict__ nbrs, int32_t* __restrict__ repr_map,
                                                  int32_t* __restrict__ slot_owner)
{
    int lvl_off[DN_MAX_LAYERS + 2], nbr_off[DN_MAX_LAYERS + 1];
    for (int h = 0; h <= k + 1; ++h) lvl_off[h] = hdr[HDR_LVL_OFF + h];
    for (int h = 0; h <= k; ++h) nbr_off[h] = hdr[HDR_LVL_NBR_OFF + h];
    const int N = lvl_off[k + 1], E = nbr_off[k];
    const int off1 = N - lvl_off[k];                         // |Delta_0|: nodes without a neighbour segment
    const int stride = gridDim.x * TPB;
    const int tid = blockIdx.x * TPB + threadIdx.x;

    for (int p = tid; p < N; p += stride) {
        int h = 0;
        while (h < k && p >= lvl_off[h + 1]) ++h;
        const int fp = N - lvl_off[h + 1] + (p - lvl_off[h]);
        const int u = lvl_ids[p];
        node_ids[fp] = u;
        // leave the bitmap clean for the next batch (the words of the last level's nodes were cleared when it was formed)
        if (h < k) seen[BM((uint32_t)u >> 5)] = 0;
        if (h < k)
            nbr_offsets[fp - off1] = E - nbr_off[h + 1] + (lvl_nbr_offsets[p] - nbr_off[h]);
    }
    for (int e = tid; e < E; e += stride) {
        int h = 0;
        while (h < k - 1 && e >= nbr_off[h + 1]) ++h;
        const int fe = E - nbr_off[h + 1] + (e - nbr_off[h]);
        const int u = lvl_nbrs[e];
        nbrs[fe] = u;
        repr_map[fe] = final_node_pos(lvlpos[u], lvl_off, k, N);
        slot_owner[fe] = final_node_pos(lvl_owner[e], lvl_off, k, N) - off1;
    }
    if (tid == 0) {
        nbr_offsets[N - off1] = E;
        for (int j = 0; j <= k; ++j) hdr[HDR_NODE_OFF + j] = N - lvl_off[k - j + 1];
        hdr[HDR_NODE_OFF + k + 1] = N;
        hdr[HDR_N] = N;
        hdr[HDR_E] = E;
        hdr[HDR_STATUS] = hdr[HDR_STATUS_ACC];
        hdr[HDR_STATUS_ACC] = 0;
        hdr[HDR_SAMPLE_SEQ] = hdr[HDR_SAMPLE_SEQ] + 1;           // a transpose index stamped with the old number is stale now
    }
}

template <int G>
void launch_sample_g(int grid, hipStream_t st, GraphDev gd, int hop, int f, int direction, uint32_t k0, uint32_t k1,
                     dn_batch* b, int n_blk)
{
    hipLaunchKernelGGL((k_sample<G>), dim3(grid), dim3(TPB), 0, st, gd, hop, f, direction, k0, k1, b->hdr, b->lvl_ids,
                       b->lvl_nbr_offsets, b->lvl_nbrs, b->lvl_owner, b->cap_slots, b->seen, b->fresh, b->summary,
                       reinterpret_cast<unsigned long long*>(b->blk_a), n_blk);
}

}  // namespace

static int launch_hops_and_assemble(dn_batch* b, const GraphDev& gd, int64_t level0_bound, uint64_t seed, hipStream_t st);

int dn_launch_sample_edges(dn_batch* b, const dn_graph* g, const int32_t* d_src, const int32_t* d_dst, int32_t n_edges,
                           const int32_t* d_neg, int32_t n_neg, uint64_t seed, int32_t* d_src_local,
                           int32_t* d_dst_local, int32_t* d_neg_local, hipStream_t st)
{
    GraphDev gd;
    gd.rp[0] = g->rowptr[0]; gd.rp[1] = g->rowptr[1];
    gd.col[0] = g->col[0];   gd.col[1] = g->col[1];
    const int dir = b->direction;
    uint64_t* blk = reinterpret_cast<uint64_t*>(b->blk_a);
    const int total = 2 * n_edges + n_neg;
    int grid = (total + TPB - 1) / TPB;
    if (grid > 2048) grid = 2048;
    if (grid < 1) grid = 1;
    const int grid_words = (int)((((b->words0 + ((int64_t)1 << b->walk_shift) - 1) >> b->walk_shift) + TPB - 1) / TPB);
    const bool fused_nd = next_delta_fused(grid_words);
    unsigned long long* blk_u = reinterpret_cast<unsigned long long*>(b->blk_a);
    { dn_prof_scope ps("mark_ids", 0, st);
    hipLaunchKernelGGL(k_mark_ids, dim3(grid), dim3(TPB), 0, st, b->V, d_src, n_edges, d_dst, n_edges, d_neg, n_neg, b->hdr,
                       b->fresh, b->summary, blk_u, fused_nd ? grid_words : 0);
    }
    DN_LAUNCH_CHECK("k_mark_ids");
    if (fused_nd) {
        { dn_prof_scope ps("next_delta_hop", 0, st);
        hipLaunchKernelGGL(k_next_delta, dim3(grid_words), dim3(TPB), 0, st, gd, b->words0, b->walk_shift, 0, b->fanouts[0], dir, b->hdr,
                           b->fresh, b->summary, blk_u, b->lvlpos, b->lvl_ids, b->lvl_nbr_offsets, b->cap_nodes, b->seen);
        }
        DN_LAUNCH_CHECK("k_next_delta");
    } else {
        { dn_prof_scope ps("fresh_count_hop", 0, st);
        hipLaunchKernelGGL(k_fresh_count, dim3(grid_words), dim3(TPB), 0, st, gd, b->words0, b->walk_shift, b->fanouts[0], dir, b->fresh,
                           b->summary, blk);
        }
        DN_LAUNCH_CHECK("k_fresh_count");
        { dn_prof_scope ps("fresh_emit_hop", 0, st);
        hipLaunchKernelGGL(k_fresh_emit, dim3(grid_words), dim3(TPB), 0, st, gd, b->words0, b->walk_shift, 0, b->fanouts[0], dir, b->hdr,
                           b->fresh, b->summary, blk, b->lvlpos, b->lvl_ids, b->lvl_nbr_offsets, b->cap_nodes, b->seen);
        }
        DN_LAUNCH_CHECK("k_fresh_emit");
    }
    { dn_prof_scope ps("local_ids", 0, st);
    hipLaunchKernelGGL(k_local_ids, dim3(grid), dim3(TPB), 0, st, b->V, d_src, n_edges, d_dst, n_edges, d_neg, n_neg,
                       b->lvlpos, d_src_local, d_dst_local, d_neg_local);
    }
    DN_LAUNCH_CHECK("k_local_ids");
    return launch_hops_and_assemble(b, gd, total, seed, st);
}

int dn_launch_sample(dn_batch* b, const dn_graph* g, const int32_t* d_targets, int32_t n_targets,
                     uint64_t seed, hipStream_t st)
{
    GraphDev gd;
    gd.rp[0] = g->rowptr[0]; gd.rp[1] = g->rowptr[1];
    gd.col[0] = g->col[0];   gd.col[1] = g->col[1];
    const int dir = b->direction;
    uint64_t* blk = reinterpret_cast<uint64_t*>(b->blk_a);

    const int grid0 = n_targets > 0 ? (n_targets + TPB - 1) / TPB : 1;
    if (grid0 > b->max_blocks) return dn_fail(DN_ECAPACITY, "dense_sample: %d targets exceed the batch capacity", n_targets);
    if (n_targets <= INIT_FUSED_MAX) {
        { dn_prof_scope ps("init_level0", 0, st);
        hipLaunchKernelGGL(k_init_level0, dim3(grid0), dim3(TPB), 0, st, gd, b->V, d_targets, n_targets, b->fanouts[0], dir,
                           b->hdr, b->seen, b->lvlpos, b->lvl_ids, b->lvl_nbr_offsets);
        }
        DN_LAUNCH_CHECK("k_init_level0");
        return launch_hops_and_assemble(b, gd, n_targets, seed, st);
    }
    { dn_prof_scope ps("init_targets", 0, st);
    hipLaunchKernelGGL(k_init_targets, dim3(grid0), dim3(TPB), 0, st, gd, b->V, d_targets, n_targets, b->fanouts[0], dir,
                       b->hdr, b->seen, b->lvlpos, b->lvl_ids, b->lvl_nbr_offsets, blk);
    }
    DN_LAUNCH_CHECK("k_init_targets");
    { dn_prof_scope ps("init_offsets", 0, st);
    hipLaunchKernelGGL(k_init_offsets, dim3(grid0), dim3(TPB), 0, st, n_targets, b->hdr, b->lvl_nbr_offsets, blk);
    }
    DN_LAUNCH_CHECK("k_init_offsets");
    return launch_hops_and_assemble(b, gd, n_targets, seed, st);
}

// the k hops (sample, next Delta) and the final layout, common to both front ends
static int launch_hops_and_assemble(dn_batch* b, const GraphDev& gd, int64_t level0_bound, uint64_t seed, hipStream_t st)
{
    const int k = b->k, dir = b->direction;
    uint64_t* blk = reinterpret_cast<uint64_t*>(b->blk_a);
    const uint32_t key0 = (uint32_t)(seed & 0xffffffffu), key1 = (uint32_t)(seed >> 32);
    const int grid_words = (int)((((b->words0 + ((int64_t)1 << b->walk_shift) - 1) >> b->walk_shift) + TPB - 1) / TPB);
    const bool fused_nd = next_delta_fused(grid_words);
    int64_t level_bound = level0_bound;                     // upper bound of the level size, known on the host
    for (int h = 0; h < k; ++h) {
        const int f = b->fanouts[h];
        int G = 4;
        while (G < f) G <<= 1;
        const int64_t groups = level_bound > 0 ? level_bound : 1;
        int64_t grid = (groups * G + TPB - 1) / TPB;
        if (grid > 8192) grid = 8192;                       // grid-stride beyond this
        { dn_prof_scope ps("sample_hop", h + 1, st);
        switch (G) {
            case 4:  launch_sample_g<4>((int)grid, st, gd, h, f, dir, key0, key1, b, fused_nd ? grid_words : 0); break;
            case 8:  launch_sample_g<8>((int)grid, st, gd, h, f, dir, key0, key1, b, fused_nd ? grid_words : 0); break;
            case 16: launch_sample_g<16>((int)grid, st, gd, h, f, dir, key0, key1, b, fused_nd ? grid_words : 0); break;
            case 32: launch_sample_g<32>((int)grid, st, gd, h, f, dir, key0, key1, b, fused_nd ? grid_words : 0); break;
            default: launch_sample_g<64>((int)grid, st, gd, h, f, dir, key0, key1, b, fused_nd ? grid_words : 0); break;
        }
        }
        DN_LAUNCH_CHECK("k_sample");
        const int f_next = (h + 1 < k) ? b->fanouts[h + 1] : 0;
        if (fused_nd) {
            { dn_prof_scope ps("next_delta_hop", h + 1, st);
            hipLaunchKernelGGL(k_next_delta, dim3(grid_words), dim3(TPB), 0, st, gd, b->words0, b->walk_shift, h + 1, f_next, dir, b->hdr,
                               b->fresh, b->summary, reinterpret_cast<unsigned long long*>(b->blk_a), b->lvlpos, b->lvl_ids,
                               b->lvl_nbr_offsets, b->cap_nodes, (uint32_t*)nullptr);
            }
            DN_LAUNCH_CHECK("k_next_delta");
        } else {
            { dn_prof_scope ps("fresh_count_hop", h + 1, st);
            hipLaunchKernelGGL(k_fresh_count, dim3(grid_words), dim3(TPB), 0, st, gd, b->words0, b->walk_shift, f_next, dir, b->fresh,
                               b->summary, blk);
            }
            DN_LAUNCH_CHECK("k_fresh_count");
            { dn_prof_scope ps("fresh_emit_hop", h + 1, st);
            hipLaunchKernelGGL(k_fresh_emit, dim3(grid_words), dim3(TPB), 0, st, gd, b->words0, b->walk_shift, h + 1, f_next, dir, b->hdr,
                               b->fresh, b->summary, blk, b->lvlpos, b->lvl_ids, b->lvl_nbr_offsets, b->cap_nodes,
                               (uint32_t*)nullptr);
            }
            DN_LAUNCH_CHECK("k_fresh_emit");
        }
        const int mult = dir == DN_DIR_BOTH ? 2 : 1;
        level_bound = level_bound * f * mult;
        if (level_bound > b->cap_level[h + 1]) level_bound = b->cap_level[h + 1];
    }
    int64_t work = b->cap_nodes > b->cap_slots ? b->cap_nodes : b->cap_slots;
    int64_t grid_asm = (work + TPB - 1) / TPB;
    if (grid_asm > 2048) grid_asm = 2048;
    if (grid_asm < 1) grid_asm = 1;
    { dn_prof_scope ps("assemble", 0, st);
    hipLaunchKernelGGL(k_assemble, dim3((int)grid_asm), dim3(TPB), 0, st, k, b->hdr, b->lvl_ids, b->lvl_nbr_offsets,
                       b->lvl_nbrs, b->lvl_owner, b->lvlpos, b->seen, b->node_ids, b->nbr_offsets, b->nbrs, b->repr_map,
                       b->slot_owner);
    }
    DN_LAUNCH_CHECK("k_assemble");
    return DN_OK;
}
