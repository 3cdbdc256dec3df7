// DENSE construction on the device: Algorithm 1 of the paper (multi-hop sampling with one-hop
// sample reuse) plus repr_map of Section 4.2, as a fixed sequence of k + 3 kernels with every
// sample-dependent size kept in device memory.
//
// The node ids are cut into ranges of 2^s consecutive ids, one per workgroup of the hop kernel (s is chosen
// so that a graph gives one to two thousand ranges).  One kernel per level L (targets are level 0):
//
//   k_hop, level L   first the next-Delta step of Algorithm 1 for its own id range: the nodes first reached
//                    at hop L - 1 were marked in a bitmap (`fresh`) by the kernel before; the workgroup walks
//                    its range of that bitmap in ascending order, so the new Delta comes out in ascending node
//                    id without a sort, gives every node its staging position and the offset of its neighbour
//                    segment (exclusive sums of min(deg, fanout)), and clears the bits it consumed.  What lies
//                    before the range (nodes, slots) is the sum of the per-range totals that the marking kernel
//                    accumulated, so no separate counting pass exists.
//                    Then the one-hop sample of those same nodes (they are in this workgroup's hands): one lane
//                    group per node, Floyd's subset algorithm over adjacency positions with Philox4x32-10 words,
//                    neighbours written sequentially at the node's offset, every neighbour id "claimed" in the
//                    bitmaps `seen` (all of node_ids so far) and `fresh` (first reached at this hop) with one
//                    64-bit atomic; the lane that claims a node first adds it (and the slots it will need at the
//                    next hop) to its range's total for level L + 1.
//                    The kernel of level k has no hop left: it only forms the last Delta.
//   k_assemble       lays the staging arrays (level order) out in the paper's order (Delta_0 first, last hop's
//                    neighbours first) and translates every neighbour id to its position in node_ids.
//
// Level 0 is the caller's target array (k_targets: mark, count, offsets in one kernel) or, for the link-prediction
// front end, the distinct ids among edge endpoints and negatives (k_mark_ids marks them like a hop would).
//
// Two levels are in flight inside one hop kernel (a workgroup may still be forming level L from `fresh` while
// another already marks level L + 1), so `fresh`, its summary and `seen` exist twice, by parity of the level;
// a node is in node_ids if either `seen` word has its bit.  The per-range totals rotate through three buffers:
// the kernel of level L reads buffer L % 3, adds into (L + 1) % 3 and clears (L + 2) % 3.
#include "dn_internal.h"

namespace {
// Bitmap layout: word index w (32 node ids) owns four consecutive words [seen0, fresh0, seen1, fresh1];
// (seen_p, fresh_p) of parity p form one aligned 8-byte pair, marked with a single atomic.
#define BITS_SEEN(w, p) (4 * (int64_t)(w) + 2 * (p))
#define BITS_FRESH(w, p) (4 * (int64_t)(w) + 2 * (p) + 1)

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

// Sum of part[0 .. n) computed cooperatively by the block (n is at most a few thousand).
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

// Marks node u as first reached now, in `seen` and `fresh` of parity p at once, unless it already is in node_ids.
// A relaxed device-scope load comes first: hubs are claimed once and then only read.  A clear bit means the node is in no
// earlier level (those kernels are complete), so it is new whichever lane marks it first: every lane that sees it
// clear marks it with one 64-bit atomic on the pair of words (the bitmaps end the same whoever comes first), and
// the one lane that finds the bit clear in the atomic's return value is the node's claimant: it adds the node, and
// the slots it will need at the next hop, to the totals of its id range.
__device__ __forceinline__ void claim(const GraphDev& g, int u, int p, uint32_t* __restrict__ bits,
                                      uint32_t* __restrict__ summary_p, uint64_t* __restrict__ totals_next, int shift,
                                      int f_next, int direction)
{
    const uint32_t w = (uint32_t)u >> 5, bit = 1u << (u & 31);
    unsigned long long* pairs = reinterpret_cast<unsigned long long*>(bits + 4 * (int64_t)w);
    const unsigned long long pair0 = __hip_atomic_load(pairs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long pair1 = __hip_atomic_load(pairs + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (((uint32_t)pair0 | (uint32_t)pair1) & bit) return;              // low halves: the two `seen` words
    const unsigned long long both = (unsigned long long)bit | ((unsigned long long)bit << 32);
    const unsigned long long old_pair = atomicOr(pairs + p, both);
    if ((uint32_t)old_pair & bit) return;                               // another lane was first
    if ((uint32_t)(old_pair >> 32) == 0) atomicOr(&summary_p[w >> 5], 1u << (w & 31));
    const int slots = f_next > 0 ? node_sample_count(g, u, f_next, direction) : 0;
    atomicAdd(reinterpret_cast<unsigned long long*>(&totals_next[(uint32_t)u >> shift]), (unsigned long long)pack(1, slots));
}

// ---------------------------------------------------------------- level 0: the targets
// Up to a few thousand targets: one kernel.  A thread per target copies it to the staging array, marks it seen
// (parity 0) and counts its neighbour slots; what lies before a workgroup's targets it adds up itself from the
// targets' degrees (no second kernel for the offsets).
__global__ __launch_bounds__(TPB) void k_targets(GraphDev g, int64_t V, const int32_t* __restrict__ targets,
                                                 int n, int f0, int direction, int32_t* __restrict__ hdr,
                                                 uint32_t* __restrict__ bits, int32_t* __restrict__ lvlpos,
                                                 int32_t* __restrict__ lvl_ids, int32_t* __restrict__ lvl_nbr_offsets)
{
    __shared__ uint64_t sm[TPB / 64];
    uint64_t before = 0;
    {
        uint64_t acc = 0;
        for (int j = threadIdx.x; j < (int)blockIdx.x * TPB; j += TPB) {
            const int t = targets[j];
            if (t >= 0 && (int64_t)t < V) acc += (uint64_t)node_sample_count(g, t, f0, direction);
        }
        uint64_t total;
        block_exclusive_scan(acc, total, sm);
        before = total;
    }
    const int i = blockIdx.x * TPB + threadIdx.x;
    int c = 0;
    if (i < n) {
        const int t = targets[i];
        if (t < 0 || (int64_t)t >= V) {
            atomicOr(&hdr[HDR_STATUS_ACC], ST_BAD_TARGET);
            lvl_ids[i] = 0;                                  // keeps every later access in bounds
        } else {
            const uint32_t bit = 1u << (t & 31);
            const uint32_t old = atomicOr(&bits[BITS_SEEN(t >> 5, 0)], bit);
            if (old & bit) atomicOr(&hdr[HDR_STATUS_ACC], ST_DUP_TARGET);
            lvl_ids[i] = t;
            lvlpos[t] = i;
            c = node_sample_count(g, t, f0, direction);
        }
    }
    uint64_t total;
    const uint64_t ex = block_exclusive_scan((uint64_t)c, total, sm);
    if (i < n) lvl_nbr_offsets[i] = (int)(before + ex);
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        hdr[HDR_LVL_OFF + 0] = 0;
        hdr[HDR_LVL_OFF + 1] = n;
        hdr[HDR_LVL_NBR_OFF + 0] = 0;
        hdr[HDR_LVL_NBR_OFF + 1] = (int)(before + total);
        hdr[HDR_NTARGETS] = n;
    }
}

// The same in two kernels for larger target arrays: per-block sums, then offsets.
__global__ __launch_bounds__(TPB) void k_init_targets(GraphDev g, int64_t V, const int32_t* __restrict__ targets,
                                                      int n, int f0, int direction, int32_t* __restrict__ hdr,
                                                      uint32_t* __restrict__ bits, int32_t* __restrict__ lvlpos,
                                                      int32_t* __restrict__ lvl_ids, int32_t* __restrict__ lvl_nbr_offsets,
                                                      uint64_t* __restrict__ blk)
{
    __shared__ uint64_t sm[TPB / 64];
    const int i = blockIdx.x * TPB + threadIdx.x;
    int c = 0;
    if (i < n) {
        const int t = targets[i];
        if (t < 0 || (int64_t)t >= V) {
            atomicOr(&hdr[HDR_STATUS_ACC], ST_BAD_TARGET);
            lvl_ids[i] = 0;
        } else {
            const uint32_t bit = 1u << (t & 31);
            const uint32_t old = atomicOr(&bits[BITS_SEEN(t >> 5, 0)], bit);
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

// ---------------------------------------------------------------- level 0 from training edges
// Link prediction (Section 2: a training example is a pair of target nodes): the targets are the
// distinct endpoints of the batch's edges plus the negative nodes.  Their ids are marked as a hop
// would mark newly reached nodes; the level-0 hop kernel then yields them in ascending id.
__global__ __launch_bounds__(TPB) void k_mark_ids(GraphDev g, int64_t V, const int32_t* __restrict__ a, int na,
                                                  const int32_t* __restrict__ b, int nb, const int32_t* __restrict__ c, int nc,
                                                  int32_t* __restrict__ hdr, uint32_t* __restrict__ bits,
                                                  uint32_t* __restrict__ summary0, uint64_t* __restrict__ totals0, int shift,
                                                  int f0, int direction)
{
    const int total = na + nb + nc;
    const int stride = gridDim.x * TPB;
    for (int i = blockIdx.x * TPB + threadIdx.x; i < total; i += stride) {
        const int u = i < na ? a[i] : (i < na + nb ? b[i - na] : c[i - na - nb]);
        if (u < 0 || (int64_t)u >= V) { atomicOr(&hdr[HDR_STATUS_ACC], ST_BAD_TARGET); continue; }
        claim(g, u, 0, bits, summary0, totals0, shift, f0, direction);
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

// ---------------------------------------------------------------- one level: next Delta, then its one-hop sample
struct HopArgs {
    int level;            // the level this kernel forms and samples
    int f;                // fanout of hop `level` (0: the last level, nothing to sample)
    int f_next;           // fanout of the hop after it (0 if none): slots a newly claimed node will need
    int direction;
    uint32_t key0, key1;
    int from_targets;     // level 0 given as an array: its nodes are staged already, taken by position
    int set_ntargets;     // level 0 from marked ids: its size is the number of targets
    int shift;            // log2 of the ids per range
    int n_ranges;
    int32_t* hdr;
    uint32_t* bits;
    uint32_t* summary[2];
    uint64_t* totals[3];
    int32_t *lvlpos, *lvl_ids, *lvl_nbr_offsets, *lvl_nbrs, *lvl_owner;
    int64_t cap_nodes, cap_slots;
};

// the bitmap walk of one thread: its fresh words of parity p in ascending order (words whose summary bit is clear are
// skipped unread)
template <typename F>
__device__ __forceinline__ void walk_fresh(const uint32_t* bits, const uint32_t* summary_p, int p,
                                           int64_t w_begin, int n_words, F&& per_word)
{
    uint32_t sw = 0;
    for (int j = 0; j < n_words; ++j) {
        const int64_t w = w_begin + j;
        if (j == 0 || (w & 31) == 0) sw = summary_p[w >> 5];
        if (!((sw >> (w & 31)) & 1u)) continue;
        per_word(w, bits[BITS_FRESH(w, p)]);
    }
}

// G lanes cooperate on one node (G = power of two >= fanout).  Lane s owns Floyd step s: it draws
// t_s in [0, deg-f+s]; the picks are then settled in step order with a G-wide ballot, which is the
// sequential part of Floyd's algorithm ("take j if t is already in the set").
template <int G>
__global__ __launch_bounds__(TPB) void k_hop(GraphDev g, HopArgs a)
{
    __shared__ uint64_t sm[TPB / 64];
    constexpr int GROUPS = TPB / G;
    const int L = a.level, p = L & 1, f = a.f;
    const int wg = blockIdx.x;

    // the totals two levels on are nobody's at the moment: clear them for the kernel after this one
    {
        uint64_t* z = a.totals[(L + 2) % 3];
        for (int i = blockIdx.x * TPB + threadIdx.x; i < a.n_ranges; i += gridDim.x * TPB) z[i] = 0;
    }

    int node_begin = 0, node_count = 0;       // staging positions of this workgroup's nodes
    if (!a.from_targets) {
        if (wg >= a.n_ranges) return;
        // ---- next Delta of this id range
        const uint64_t* totals = a.totals[L % 3];
        const uint64_t before = block_sum_prefix(totals, wg, sm);
        const int words_per_range = 1 << (a.shift - 5);
        const int per_thread = words_per_range >= TPB ? words_per_range / TPB : 1;
        const bool walker = (int)threadIdx.x * per_thread < words_per_range;
        const int64_t w_begin = (int64_t)wg * words_per_range + (int64_t)threadIdx.x * per_thread;
        int nodes = 0, slots = 0;
        if (walker)
            walk_fresh(a.bits, a.summary[p], p, w_begin, per_thread, [&](int64_t w, uint32_t fw) {
                nodes += __popc(fw);
                if (f > 0)
                    while (fw) {
                        const int bit = __ffs(fw) - 1;
                        fw &= fw - 1;
                        slots += node_sample_count(g, (int)(w * 32 + bit), f, a.direction);
                    }
            });
        uint64_t total;
        const uint64_t ex = block_exclusive_scan(pack(nodes, slots), total, sm) + before;
        const int node_base = a.hdr[HDR_LVL_OFF + L];
        const int slot_base = f > 0 ? a.hdr[HDR_LVL_NBR_OFF + L] : 0;
        int pos = node_base + (int)(uint32_t)(ex & 0xffffffffu);
        int so = slot_base + (int)(uint32_t)(ex >> 32);
        if (walker)
            walk_fresh(a.bits, a.summary[p], p, w_begin, per_thread, [&](int64_t w, uint32_t fw) {
                a.bits[BITS_FRESH(w, p)] = 0;
                while (fw) {
                    const int bit = __ffs(fw) - 1;
                    fw &= fw - 1;
                    const int u = (int)(w * 32 + bit);
                    if (pos < a.cap_nodes) {
                        a.lvl_ids[pos] = u;
                        a.lvlpos[u] = pos;
                        if (f > 0) {
                            a.lvl_nbr_offsets[pos] = so;
                            so += node_sample_count(g, u, f, a.direction);
                        }
                    }
                    ++pos;
                }
            });
        __syncthreads();                                   // every walker has read its summary bits
        {
            const int summary_words = words_per_range >> 5;    // whole summary words: a range holds at least 1024 ids
            for (int j = threadIdx.x; j < summary_words; j += TPB) a.summary[p][(int64_t)wg * summary_words + j] = 0;
        }
        node_begin = node_base + (int)(uint32_t)(before & 0xffffffffu);
        node_count = (int)(uint32_t)(total & 0xffffffffu);
        if (node_begin > a.cap_nodes) node_begin = (int)a.cap_nodes;
        if ((int64_t)node_begin + node_count > a.cap_nodes) node_count = (int)(a.cap_nodes - node_begin);
        if (wg == a.n_ranges - 1 && threadIdx.x == 0) {
            const uint64_t all = before + total;
            int n_new = (int)(uint32_t)(all & 0xffffffffu);
            if ((int64_t)node_base + n_new > a.cap_nodes) {
                atomicOr(&a.hdr[HDR_STATUS_ACC], ST_CAPACITY);
                n_new = (int)(a.cap_nodes - node_base);
            }
            a.hdr[HDR_LVL_OFF + L + 1] = node_base + n_new;
            if (f > 0) a.hdr[HDR_LVL_NBR_OFF + L + 1] = slot_base + (int)(uint32_t)(all >> 32);
            if (a.set_ntargets) a.hdr[HDR_NTARGETS] = n_new;
        }
        if (f == 0) return;
        __syncthreads();                                   // the staging entries written above are read below
    } else {
        node_begin = a.hdr[HDR_LVL_OFF + L];
        node_count = a.hdr[HDR_LVL_OFF + L + 1] - node_begin;
    }

    // ---- one-hop sample of the nodes [node_begin, node_begin + node_count)
    const int lane = threadIdx.x & 63;
    const int s = threadIdx.x % G;
    const uint64_t gmask = (G == 64) ? ~0ull : (((1ull << G) - 1ull) << ((lane / G) * G));
    uint64_t* totals_next = a.totals[(L + 1) % 3];
    uint32_t* summary_next = a.summary[p ^ 1];
    const int first = a.from_targets ? (int)blockIdx.x * GROUPS : 0;
    const int step = a.from_targets ? (int)gridDim.x * GROUPS : GROUPS;
    for (int gid = first + threadIdx.x / G; gid < node_count; gid += step) {
        const int pn = node_begin + gid;
        const int v = a.lvl_ids[pn];
        int o = a.lvl_nbr_offsets[pn];
#pragma unroll 1
        for (int dir = 0; dir < 2; ++dir) {
            if ((dir == 0 && a.direction == DN_DIR_IN) || (dir == 1 && a.direction == DN_DIR_OUT)) continue;
            const int64_t base = g.rp[dir][v];
            const int64_t deg = g.rp[dir][v + 1] - base;
            const int c = deg < f ? (int)deg : f;
            const bool floyd = deg > f;
            uint32_t t = 0xffffffffu, j = 0;
            if (floyd && s < f) {
                j = (uint32_t)(deg - f + s);
                const uint32_t r = philox4x32_10_word((uint32_t)(s >> 2), (uint32_t)v, (uint32_t)L, (uint32_t)dir,
                                                      a.key0, a.key1, s & 3);
                t = __umulhi(r, j + 1u);                 // uniform in [0, j]
            }
            uint32_t pick = t;
            for (int sp = 1; sp < f; ++sp) {
                const uint32_t ts = __shfl(t, sp, G);
                const bool hit = floyd && s < sp && pick == ts;
                const uint64_t any = __ballot(hit) & gmask;
                if (s == sp && any) pick = j;
            }
            const int64_t posn = floyd ? (int64_t)pick : (int64_t)s;
            if (s < c && (int64_t)(o + s) < a.cap_slots) {
                const int u = g.col[dir][base + posn];
                a.lvl_nbrs[o + s] = u;
                a.lvl_owner[o + s] = pn;
                claim(g, u, p ^ 1, a.bits, summary_next, totals_next, a.shift, a.f_next, a.direction);
            }
            o += c;
        }
    }
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
                                                  const int32_t* __restrict__ lvlpos, uint32_t* __restrict__ bits,
                                                  uint64_t* __restrict__ totals_last, int n_ranges,
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

    for (int i = tid; i < n_ranges; i += stride) totals_last[i] = 0;     // the last level's totals: all three buffers are clear again
    for (int p = tid; p < N; p += stride) {
        int h = 0;
        while (h < k && p >= lvl_off[h + 1]) ++h;
        const int fp = N - lvl_off[h + 1] + (p - lvl_off[h]);
        const int u = lvl_ids[p];
        node_ids[fp] = u;
        // leave the bitmaps clean for the next batch (the `fresh` words are clear already: every level was formed)
        *reinterpret_cast<uint4*>(&bits[4 * (int64_t)((uint32_t)u >> 5)]) = make_uint4(0u, 0u, 0u, 0u);
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

GraphDev graph_dev(const dn_graph* g)
{
    GraphDev gd;
    gd.rp[0] = g->rowptr[0]; gd.rp[1] = g->rowptr[1];
    gd.col[0] = g->col[0];   gd.col[1] = g->col[1];
    return gd;
}

template <int G>
void launch_hop_g(int grid, hipStream_t st, const GraphDev& gd, const HopArgs& a)
{
    hipLaunchKernelGGL((k_hop<G>), dim3(grid), dim3(TPB), 0, st, gd, a);
}

// targets handled by the one-kernel form of level 0 (every workgroup re-reads the degrees of the targets before its own)
constexpr int ONE_KERNEL_TARGETS = 8192;

}  // namespace

// The kernels of levels 0 .. k and the final layout, common to both front ends.
static int launch_levels_and_assemble(dn_batch* b, const GraphDev& gd, bool level0_from_targets, int64_t level0_bound,
                                      uint64_t seed, hipStream_t st)
{
    const int k = b->k, dir = b->direction;
    for (int L = 0; L <= k; ++L) {
        HopArgs a;
        a.level = L;
        a.f = L < k ? b->fanouts[L] : 0;
        a.f_next = L + 1 < k ? b->fanouts[L + 1] : 0;
        a.direction = dir;
        a.key0 = (uint32_t)(seed & 0xffffffffu);
        a.key1 = (uint32_t)(seed >> 32);
        a.from_targets = (L == 0 && level0_from_targets) ? 1 : 0;
        a.set_ntargets = (L == 0 && !level0_from_targets) ? 1 : 0;
        a.shift = b->range_shift;
        a.n_ranges = b->n_ranges;
        a.hdr = b->hdr;
        a.bits = b->bits;
        a.summary[0] = b->summary2[0]; a.summary[1] = b->summary2[1];
        for (int i = 0; i < 3; ++i) a.totals[i] = b->totals[i];
        a.lvlpos = b->lvlpos; a.lvl_ids = b->lvl_ids; a.lvl_nbr_offsets = b->lvl_nbr_offsets;
        a.lvl_nbrs = b->lvl_nbrs; a.lvl_owner = b->lvl_owner;
        a.cap_nodes = b->cap_nodes; a.cap_slots = b->cap_slots;
        int G = 4;
        while (G < a.f) G <<= 1;
        int grid = b->n_ranges;
        if (a.from_targets) {
            // nodes by position: one lane group per target
            const int64_t groups = level0_bound > 0 ? level0_bound : 1;
            int64_t want = (groups * G + TPB - 1) / TPB;
            if (want > 8192) want = 8192;
            grid = (int)want;
        }
        { dn_prof_scope ps(L < k ? "hop" : "last_delta", L < k ? L + 1 : 0, st);
        switch (G) {
            case 4:  launch_hop_g<4>(grid, st, gd, a); break;
            case 8:  launch_hop_g<8>(grid, st, gd, a); break;
            case 16: launch_hop_g<16>(grid, st, gd, a); break;
            case 32: launch_hop_g<32>(grid, st, gd, a); break;
            default: launch_hop_g<64>(grid, st, gd, a); break;
        }
        }
        DN_LAUNCH_CHECK("k_hop");
    }
    int64_t work = b->cap_nodes > b->cap_slots ? b->cap_nodes : b->cap_slots;
    int64_t grid_asm = (work + TPB - 1) / TPB;
    if (grid_asm > 2048) grid_asm = 2048;
    if (grid_asm < 1) grid_asm = 1;
    { dn_prof_scope ps("assemble", 0, st);
    hipLaunchKernelGGL(k_assemble, dim3((int)grid_asm), dim3(TPB), 0, st, k, b->hdr, b->lvl_ids, b->lvl_nbr_offsets,
                       b->lvl_nbrs, b->lvl_owner, b->lvlpos, b->bits, b->totals[k % 3], b->n_ranges, b->node_ids,
                       b->nbr_offsets, b->nbrs, b->repr_map, b->slot_owner);
    }
    DN_LAUNCH_CHECK("k_assemble");
    return DN_OK;
}

int dn_launch_sample_edges(dn_batch* b, const dn_graph* g, const int32_t* d_src, const int32_t* d_dst, int32_t n_edges,
                           const int32_t* d_neg, int32_t n_neg, uint64_t seed, int32_t* d_src_local,
                           int32_t* d_dst_local, int32_t* d_neg_local, hipStream_t st)
{
    const GraphDev gd = graph_dev(g);
    const int total = 2 * n_edges + n_neg;
    int grid = (total + TPB - 1) / TPB;
    if (grid > 2048) grid = 2048;
    if (grid < 1) grid = 1;
    { dn_prof_scope ps("mark_ids", 0, st);
    hipLaunchKernelGGL(k_mark_ids, dim3(grid), dim3(TPB), 0, st, gd, b->V, d_src, n_edges, d_dst, n_edges, d_neg, n_neg, b->hdr,
                       b->bits, b->summary2[0], b->totals[0], b->range_shift, b->fanouts[0], b->direction);
    }
    DN_LAUNCH_CHECK("k_mark_ids");
    // The level-0 kernel gives every target its position; the endpoints' local ids are looked up after the whole
    // chain (nothing in it reads them).
    const int rc = launch_levels_and_assemble(b, gd, false, total, seed, st);
    if (rc) return rc;
    { dn_prof_scope ps("local_ids", 0, st);
    hipLaunchKernelGGL(k_local_ids, dim3(grid), dim3(TPB), 0, st, b->V, d_src, n_edges, d_dst, n_edges, d_neg, n_neg,
                       b->lvlpos, d_src_local, d_dst_local, d_neg_local);
    }
    DN_LAUNCH_CHECK("k_local_ids");
    return DN_OK;
}

int dn_launch_sample(dn_batch* b, const dn_graph* g, const int32_t* d_targets, int32_t n_targets,
                     uint64_t seed, hipStream_t st)
{
    const GraphDev gd = graph_dev(g);
    const int dir = b->direction;
    const int grid0 = n_targets > 0 ? (n_targets + TPB - 1) / TPB : 1;
    if (grid0 > b->max_blocks) return dn_fail(DN_ECAPACITY, "dense_sample: %d targets exceed the batch capacity", n_targets);
    if (n_targets <= ONE_KERNEL_TARGETS) {
        dn_prof_scope ps("targets", 0, st);
        hipLaunchKernelGGL(k_targets, dim3(grid0), dim3(TPB), 0, st, gd, b->V, d_targets, n_targets, b->fanouts[0], dir,
                           b->hdr, b->bits, b->lvlpos, b->lvl_ids, b->lvl_nbr_offsets);
        DN_LAUNCH_CHECK("k_targets");
    } else {
        uint64_t* blk = reinterpret_cast<uint64_t*>(b->blk_a);
        { dn_prof_scope ps("init_targets", 0, st);
        hipLaunchKernelGGL(k_init_targets, dim3(grid0), dim3(TPB), 0, st, gd, b->V, d_targets, n_targets, b->fanouts[0], dir,
                           b->hdr, b->bits, b->lvlpos, b->lvl_ids, b->lvl_nbr_offsets, blk);
        }
        DN_LAUNCH_CHECK("k_init_targets");
        { dn_prof_scope ps("init_offsets", 0, st);
        hipLaunchKernelGGL(k_init_offsets, dim3(grid0), dim3(TPB), 0, st, n_targets, b->hdr, b->lvl_nbr_offsets, blk);
        }
        DN_LAUNCH_CHECK("k_init_offsets");
    }
    return launch_levels_and_assemble(b, gd, true, n_targets, seed, st);
}
