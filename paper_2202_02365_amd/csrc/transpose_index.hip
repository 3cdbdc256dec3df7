// Transpose index of repr_map for the backward pass: neighbour slots grouped by the node_ids
// position they read, ascending slot number inside a group, so that the gradient of the
// neighbour mean is a gather with a fixed summation order (no floating-point atomics).
// Built by a stable least-significant-digit radix sort of (repr_map[j], j) pairs with up to
// 11 bits per pass (two passes for up to 4M positions); group boundaries by binary search.
// The number of pairs lives in device memory; grids are sized by capacity.
//
// Launches: k_tr_init (copy + histogram of the first digit), then per pass a scan of the histogram (one kernel
// while the histogram is small, block sums + look-behind otherwise) and one scatter that also histograms the next
// digit at the element's new position, then k_tr_ptr.  Histograms are integer atomics (order-independent); their
// rows are as long as the tiles in use.  Two buffers of counts alternate: pass p scans buffer p % 2 into a
// buffer of offsets, and its scatter counts the next digit into the other one and clears the one just scanned.
// Both are zero on entry and zero again on exit, so a build depends on no host-side state and can be replayed
// from a HIP graph in any order.
#include "dn_internal.h"

namespace {

constexpr int TPB = 256;
constexpr int ITEMS = 4;                   // elements per thread: 1024-pair tiles (with 2048 the two scatters of a 40k-pair
                                           // index took 15 us each, four rounds fewer per workgroup brought 47 -> 40 us in all;
                                           // 512 gains nothing more there and costs 20 % at three million pairs)
constexpr int TILE = TPB * ITEMS;          // elements per workgroup
static_assert(TILE == DN_SORT_TILE, "the kernels that count the first digit use DN_SORT_TILE");
constexpr int MAX_BITS = 11;
constexpr int MAX_RADIX = 1 << MAX_BITS;

__global__ void k_tr_init(int32_t* __restrict__ hdr, int need_all, int k, const int32_t* __restrict__ nbr_offsets,
                          const int32_t* __restrict__ repr_map, int32_t* __restrict__ key, int32_t* __restrict__ val,
                          int radix_mask, int32_t* __restrict__ hist, int32_t* __restrict__ tr_long, int long_words)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < long_words; i += gridDim.x * blockDim.x) tr_long[i] = 0;
    const int E = hdr[HDR_E];
    int first = 0;
    if (!need_all) {
        // gradients reach the inputs of layers 2..k only: slots owned by Delta_2 .. Delta_k
        first = k >= 2 ? nbr_offsets[hdr[HDR_NODE_OFF + 2] - hdr[HDR_NODE_OFF + 1]] : E;
    }
    const int cnt = E - first;
    const int nblocks = dn_sort_tiles(cnt);
    const int stride = gridDim.x * blockDim.x;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < cnt; i += stride) {
        const int kv = repr_map[first + i];
        key[i] = kv;
        val[i] = first + i;
        if (hist) atomicAdd(&hist[(kv & radix_mask) * nblocks + i / TILE], 1);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        hdr[HDR_TR_FIRST] = first;
        hdr[HDR_TR_COUNT] = cnt;
    }
}

// Digit histogram per tile without global atomics, for sorts of millions of pairs (there the atomics of the
// fused counting, one per pair at scattered addresses, cost more than a pass over the keys): a workgroup counts a
// tile's digits in LDS and stores the tile's column of the histogram.
__global__ __launch_bounds__(TPB) void k_radix_hist(const int32_t* __restrict__ count_ptr, const int32_t* __restrict__ key,
                                                    int shift, int bits, int32_t* __restrict__ hist)
{
    __shared__ int cnt[MAX_RADIX];
    const int radix = 1 << bits;
    const int n = *count_ptr;
    const int nblocks = dn_sort_tiles(n);
    for (int tile = blockIdx.x; tile * TILE < n; tile += gridDim.x) {
        for (int d = threadIdx.x; d < radix; d += TPB) cnt[d] = 0;
        __syncthreads();
        const int base = tile * TILE;
        for (int e = threadIdx.x; e < TILE; e += TPB)
            if (base + e < n) atomicAdd(&cnt[(key[base + e] >> shift) & (radix - 1)], 1);
        __syncthreads();
        for (int d = threadIdx.x; d < radix; d += TPB) hist[d * nblocks + tile] = cnt[d];
        __syncthreads();
    }
}

// two-kernel exclusive scan in place (block partial sums, then look-behind) of the histogram rows in use:
// radix x dn_sort_tiles(count) ints; workgroups past them have nothing to do
__global__ __launch_bounds__(TPB) void k_scan_partial(const int32_t* __restrict__ data, const int32_t* __restrict__ count_ptr,
                                                      int radix, int32_t* __restrict__ part)
{
    __shared__ int sm[TPB / 64];
    const int total = radix * dn_sort_tiles(*count_ptr);
    if ((int)blockIdx.x * TILE >= total) return;
    const int base = blockIdx.x * TILE + threadIdx.x * ITEMS;
    int s = 0;
    for (int e = 0; e < ITEMS; ++e) if (base + e < total) s += data[base + e];
    for (int d = 32; d > 0; d >>= 1) s += __shfl_down(s, d, 64);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = sm[0] + sm[1] + sm[2] + sm[3];
}

// The exclusive scan of block `blockIdx.x`'s TILE ints, given the sum of everything before them; the offsets
// go to `out` (the counts stay, for the scatter to clear).
__device__ __forceinline__ void scan_tile(const int32_t* __restrict__ data, int total, int before, int32_t* __restrict__ out,
                                          int* sm)
{
    const int base = blockIdx.x * TILE + threadIdx.x * ITEMS;
    int v[ITEMS], s = 0;
    for (int e = 0; e < ITEMS; ++e) { v[e] = (base + e < total) ? data[base + e] : 0; s += v[e]; }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = s;
    for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_up(incl, d, 64); if (lane >= d) incl += t; }
    __syncthreads();
    if (lane == 63) sm[wave] = incl;
    __syncthreads();
    int wbase = 0;
    for (int w = 0; w < wave; ++w) wbase += sm[w];
    int run = before + wbase + incl - s;
    for (int e = 0; e < ITEMS; ++e) {
        if (base + e < total) out[base + e] = run;
        run += v[e];
    }
}

// second half of the two-kernel scan
__global__ __launch_bounds__(TPB) void k_scan_apply(const int32_t* __restrict__ data, const int32_t* __restrict__ count_ptr,
                                                    int radix, const int32_t* __restrict__ part, int32_t* __restrict__ out)
{
    __shared__ int sm[TPB / 64];
    __shared__ int s_before;
    const int total = radix * dn_sort_tiles(*count_ptr);
    if ((int)blockIdx.x * TILE >= total) return;
    // sum of the partials of all earlier blocks
    int acc = 0;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += TPB) acc += part[i];
    for (int d = 32; d > 0; d >>= 1) acc += __shfl_down(acc, d, 64);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) s_before = sm[0] + sm[1] + sm[2] + sm[3];
    __syncthreads();
    scan_tile(data, total, s_before, out, sm);
}

// The scan in one kernel, for histograms of a few hundred tiles at most: every workgroup adds up all the counts
// before its own tile itself (sixteen-byte loads, eight in flight) instead of waiting for a kernel of partial sums.
__global__ __launch_bounds__(TPB) void k_scan_single(const int32_t* __restrict__ data, const int32_t* __restrict__ count_ptr,
                                                     int radix, int32_t* __restrict__ out)
{
    __shared__ int sm[TPB / 64];
    __shared__ int s_before;
    const int total = radix * dn_sort_tiles(*count_ptr);
    if ((int)blockIdx.x * TILE >= total) return;
    const int4* d4 = reinterpret_cast<const int4*>(data);
    const int quads = (int)blockIdx.x * (TILE / 4);
    int part8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = threadIdx.x; i < quads; i += 8 * TPB) {
        int4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = d4[min(i + u * TPB, quads - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (i + u * TPB < quads) part8[u] += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
    int acc = ((part8[0] + part8[1]) + (part8[2] + part8[3])) + ((part8[4] + part8[5]) + (part8[6] + part8[7]));
    for (int d = 32; d > 0; d >>= 1) acc += __shfl_down(acc, d, 64);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) s_before = sm[0] + sm[1] + sm[2] + sm[3];
    __syncthreads();
    scan_tile(data, total, s_before, out, sm);
}

// stable scatter: element order inside a tile is (wave, round, lane); a lane's rank among equal
// digits of its round comes from one ballot per digit bit, rounds and waves are chained through
// counters in LDS.  Also counts the next pass's digit at the element's new position, and clears the counts
// that this pass's offsets `hist` were scanned from.
__global__ __launch_bounds__(TPB) void k_radix_scatter(const int32_t* __restrict__ count_ptr, const int32_t* __restrict__ key_in,
                                                       const int32_t* __restrict__ val_in, int shift, int bits,
                                                       const int32_t* __restrict__ hist, int32_t* __restrict__ key_out,
                                                       int32_t* __restrict__ val_out, int next_bits,
                                                       int32_t* __restrict__ next_hist, int32_t* __restrict__ counts)
{
    __shared__ int cnt[TPB / 64][MAX_RADIX];
    const int radix = 1 << bits;
    const int n = *count_ptr;
    const int nblocks = dn_sort_tiles(n);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (blockIdx.x * TILE >= n) return;
    for (int i = blockIdx.x * TPB + threadIdx.x; i < radix * nblocks; i += nblocks * TPB) counts[i] = 0;   // nblocks workgroups get here
    for (int w = 0; w < TPB / 64; ++w)
        for (int d = threadIdx.x; d < radix; d += TPB) cnt[w][d] = 0;
    __syncthreads();
    const int wbase = blockIdx.x * TILE + wave * (TILE / (TPB / 64));
    int keys[ITEMS], vals[ITEMS];
    uint64_t peers[ITEMS];
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {              // all loads first: one memory latency, not one per round
        const int idx = wbase + r * 64 + lane;
        keys[r] = idx < n ? key_in[idx] : 0;
        vals[r] = idx < n ? val_in[idx] : 0;
    }
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const int idx = wbase + r * 64 + lane;
        const bool ok = idx < n;
        const int d = (keys[r] >> shift) & (radix - 1);
        uint64_t mask = __ballot(ok);
        for (int bit = 0; bit < bits; ++bit) {
            const uint64_t bal = __ballot((d >> bit) & 1);
            mask &= ((d >> bit) & 1) ? bal : ~bal;
        }
        peers[r] = ok ? mask : 0ull;
        if (ok && (mask & ((1ull << lane) - 1ull)) == 0) cnt[wave][d] += __popcll(mask);   // lowest lane of each digit
        __builtin_amdgcn_wave_barrier();       // the next round's leader may be another lane of this wave (the counters are the wave's own)
    }
    __syncthreads();
    // thread t owns digits t, t+TPB, ...: turn per-wave counts into per-wave start positions
    for (int d = threadIdx.x; d < radix; d += TPB) {
        int g = hist[d * nblocks + blockIdx.x];
        for (int w = 0; w < TPB / 64; ++w) {
            const int c = cnt[w][d];
            cnt[w][d] = g;
            g += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const uint64_t mask = peers[r];
        if (mask) {
            const int d = (keys[r] >> shift) & (radix - 1);
            const int start = cnt[wave][d];
            __builtin_amdgcn_wave_barrier();   // all lanes have read the counter before its owner advances it
            const int rank = __popcll(mask & ((1ull << lane) - 1ull));
            const int pos = start + rank;
            key_out[pos] = keys[r];
            val_out[pos] = vals[r];
            if (next_bits > 0)
                atomicAdd(&next_hist[((keys[r] >> (shift + bits)) & ((1 << next_bits) - 1)) * nblocks + pos / TILE], 1);
            if (rank == 0) cnt[wave][d] = start + __popcll(mask);
        }
        __builtin_amdgcn_wave_barrier();       // counters are read by every lane of the wave's next round
    }
}

// tr_ptr[p] = first index of sorted keys >= p, for p = 0..N: a binary search inside the range of p's most
// significant digit, whose bounds the last pass's offsets give (offs[d * tiles] = first sorted index of digit d)
__global__ __launch_bounds__(TPB) void k_tr_ptr(const int32_t* __restrict__ count_ptr, const int32_t* __restrict__ nkeys_ptr,
                                                int nkeys_const, const int32_t* __restrict__ key,
                                                int32_t* __restrict__ tr_ptr, const int32_t* __restrict__ val,
                                                const int32_t* __restrict__ offs, int top_shift, int top_radix,
                                                dn_sort_slot_info info)
{
    const int N = nkeys_ptr ? *nkeys_ptr : nkeys_const, n = *count_ptr;
    const int tiles = dn_sort_tiles(n);
    const int stride = gridDim.x * TPB;
    if (info.hdr && blockIdx.x == 0 && threadIdx.x == 0) {
        // the index now belongs to the sample in the workspace: the backward aggregation checks this stamp on the device
        info.hdr[HDR_TR_SEQ] = info.hdr[HDR_SAMPLE_SEQ];
        info.hdr[HDR_TR_ALL] = info.covers_all;
    }
    if (info.own_out) {
        for (int t = blockIdx.x * TPB + threadIdx.x; t < n; t += stride) {
            const int q = info.slot_owner[val[t]];
            info.own_out[t] = q;
            info.inv_out[t] = 1.0f / (float)(info.nbr_offsets[q + 1] - info.nbr_offsets[q]);
        }
    }
    for (int p = blockIdx.x * TPB + threadIdx.x; p <= N; p += stride) {
        const int d = p >> top_shift;
        int lo = n, hi = n;
        if (d < top_radix) {
            lo = offs[(int64_t)d * tiles];
            if (d + 1 < top_radix) hi = offs[(int64_t)(d + 1) * tiles];
        }
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (key[mid] < p) lo = mid + 1; else hi = mid;
        }
        tr_ptr[p] = lo;
        if (info.long_out && lo + DN_LONG_GROUP < n && key[lo + DN_LONG_GROUP] == p) info.long_out[lo / DN_LONG_GROUP] = p + 1;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// The whole index in ONE kernel, for the few ten thousand pairs of a node-classification mini-batch (the general
// path above is six launches, which cost more than the work).  Workgroup b owns SMALL_KEYS consecutive keys
// and reads ALL pairs itself, twice, each of its waves a contiguous part of them, in order:
//   pass 1  counts, per wave, the pairs of each of its keys (LDS atomics: counts do not depend on the order) and the
//           pairs with smaller keys (they precede the workgroup's output);
//   scan    turns the counts into tr_ptr of its keys and into one output cursor per (wave, key), waves in order;
//   pass 2  hands every pair its place: cursor of (wave, key) plus its rank among the equal keys of its 64-pair step
//           (ballots), steps in order.  Equal keys therefore keep their input order: the sort is stable.
// No workgroup waits for another and nothing is sized by the number of pairs, so any count is handled (time grows with
// count x workgroups in use: the caller chooses this path only for small counts).
// Keys per workgroup, as a power of two.  Measured at the 111M-node workload (about 40k pairs on 17k keys), index build /
// step with four mini-batches in flight: 512 keys 27.8 us / 0.155 ms, 256 keys 23.3 / 0.155, 128 keys 20.7 / 0.159,
// 64 keys 22.8 / 0.170, 32 keys 42 / 0.192: fewer keys shorten a workgroup's second pass, but every workgroup reads
// all pairs, and hundreds of 1024-thread workgroups take the compute units from the kernels of the other mini-batches.
#ifndef DN_TR_SMALL_KEY_BITS
#define DN_TR_SMALL_KEY_BITS 8
#endif
constexpr int SMALL_TPB = 1024, SMALL_WAVES = SMALL_TPB / 64, SMALL_KEY_BITS = DN_TR_SMALL_KEY_BITS, SMALL_KEYS = 1 << SMALL_KEY_BITS;
#ifndef DN_TR_SMALL_LIST_CAP
#define DN_TR_SMALL_LIST_CAP 512
#endif
constexpr int SMALL_LIST_CAP = DN_TR_SMALL_LIST_CAP;     // entries per wave (a small value, for a test build, sends most waves the other way)
static_assert(SMALL_KEYS <= 0x10000, "a key's offset in the workgroup's range must fit 16 bits");
constexpr int SMALL_BATCH = 8;     // 64-pair steps whose key loads a wave has in flight together (the loops stay short:
                                   // a kernel this brief cannot afford long straight-line code, its instruction fetch is cold)

// rank of a lane's pair among the pairs with the same key in its 64-pair step, and the number of those (one ballot
// per key bit; taking the distinct keys of a step one after the other instead measured slower, 44 against 31 us)
__device__ __forceinline__ void step_peers(int kl, bool mine, int lane, int& rank, int& count)
{
    uint64_t peers = __ballot(mine);
#pragma unroll
    for (int bit = 0; bit < SMALL_KEY_BITS; ++bit) {
        const uint64_t bal = __ballot((kl >> bit) & 1);
        peers &= ((kl >> bit) & 1) ? bal : ~bal;
    }
    rank = __popcll(peers & ((1ull << lane) - 1ull));
    count = __popcll(peers);
}

__global__ __launch_bounds__(SMALL_TPB) void k_tr_small(int32_t* __restrict__ hdr, int need_all, int k,
                                                        const int32_t* __restrict__ nbr_offsets,
                                                        const int32_t* __restrict__ repr_map, const int32_t* __restrict__ slot_owner,
                                                        int32_t* __restrict__ tr_ptr, int32_t* __restrict__ tr_val,
                                                        int32_t* __restrict__ tr_own, float* __restrict__ tr_inv,
                                                        int32_t* __restrict__ tr_long)
{
    __shared__ int cnt[SMALL_WAVES][SMALL_KEYS];
    __shared__ int s_part[SMALL_WAVES];
    // the pairs of this workgroup's keys that a wave met in pass 1, in their order: (key offset << 16) | (pair index
    // relative to the wave's first pair).  Pass 2 then ranks and places a list of a few dozen entries instead of walking
    // all of the wave's 64-pair steps again (a ballot per key bit and two LDS round trips per step: 11 of the kernel's
    // 23 us).  A wave whose list would overflow (or whose part is too long for 16 bits) walks its steps as before.
    __shared__ uint32_t s_list[SMALL_WAVES][SMALL_LIST_CAP];
    const int N = hdr[HDR_N], E = hdr[HDR_E];
    // Without layer 1's slots every pair's key is a node of Delta_1 .. Delta_k (the slots of Delta_2 .. Delta_k select
    // nodes at most one level further from the targets): the workgroups share out the positions from node_id_offsets[1]
    // on, and tr_ptr below that position, which no layer above the first reads, is left alone.  (Workgroups for the
    // positions of Delta_0, 85 % of a mini-batch's nodes, would each read every pair only to find none of theirs.)
    const int key_lo = need_all ? 0 : hdr[HDR_NODE_OFF + 1];
    const int range_start = key_lo + (int)blockIdx.x * SMALL_KEYS;
    if (range_start > N) return;
    int first = 0;
    if (!need_all) first = k >= 2 ? nbr_offsets[hdr[HDR_NODE_OFF + 2] - hdr[HDR_NODE_OFF + 1]] : E;
    const int n = E - first;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        hdr[HDR_TR_FIRST] = first;
        hdr[HDR_TR_COUNT] = n;
        hdr[HDR_TR_SEQ] = hdr[HDR_SAMPLE_SEQ];
        hdr[HDR_TR_ALL] = need_all;
    }
    for (int i = threadIdx.x; i < SMALL_WAVES * SMALL_KEYS; i += SMALL_TPB) (&cnt[0][0])[i] = 0;
    // this wave's part of the pairs: whole steps of 64
    const int steps = (n + 63) / 64;
    const int steps_per_wave = (steps + SMALL_WAVES - 1) / SMALL_WAVES;
    const int s_begin = wave * steps_per_wave, s_end = min(steps, s_begin + steps_per_wave);
    const int32_t* keys = repr_map + first;
    constexpr int NONE = 0x7fffffff;

    __syncthreads();                                           // the counts are zero

    // ---- pass 1
    int below = 0;
    int list_n = 0;                                            // entries of this wave's list (wave-uniform); above the capacity: not usable
    for (int st = s_begin; st < s_end; st += SMALL_BATCH) {
        int kv[SMALL_BATCH];
#pragma unroll
        for (int u = 0; u < SMALL_BATCH; ++u) {
            const int i = (st + u) * 64 + lane;
            kv[u] = (st + u < s_end && i < n) ? keys[i] - range_start : NONE;
        }
#pragma unroll
        for (int u = 0; u < SMALL_BATCH; ++u) {
            below += kv[u] < 0;
            const bool mine = kv[u] >= 0 && kv[u] < SMALL_KEYS;
            if (mine) atomicAdd(&cnt[wave][kv[u]], 1);
            const uint64_t m = __ballot(mine);
            if (m) {                                           // the same for the whole wave
                const int rel = (st + u - s_begin) * 64 + lane;
                const int pos = list_n + __popcll(m & ((1ull << lane) - 1ull));
                if (mine && pos < SMALL_LIST_CAP && rel < 0x10000) s_list[wave][pos] = ((uint32_t)kv[u] << 16) | (uint32_t)rel;
                list_n += __popcll(m);
                if ((st + u - s_begin) * 64 + 63 >= 0x10000) list_n = SMALL_LIST_CAP + 1;      // index beyond 16 bits: this wave walks its steps
            }
        }
    }
    for (int d = 32; d > 0; d >>= 1) below += __shfl_down(below, d, 64);
    if (lane == 0) s_part[wave] = below;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < SMALL_WAVES; ++w) before += s_part[w];
    __syncthreads();

    // ---- scan: the first SMALL_KEYS threads take a key each
    int tot = 0;
    if (threadIdx.x < SMALL_KEYS) {
#pragma unroll
        for (int w = 0; w < SMALL_WAVES; ++w) tot += cnt[w][threadIdx.x];
    }
    int incl = tot;
    for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_up(incl, d, 64); if (lane >= d) incl += t; }
    if (lane == 63) s_part[wave] = incl;
    __syncthreads();
    int run = before + incl - tot;
#pragma unroll
    for (int w = 0; w < SMALL_WAVES; ++w) if (w < wave) run += s_part[w];
    int mine_total = 0;                                        // pairs of this workgroup's keys
#pragma unroll
    for (int w = 0; w < SMALL_WAVES; ++w) mine_total += s_part[w];  // threads without a key added nothing
    if (threadIdx.x < SMALL_KEYS) {
        const int kl = threadIdx.x;
        const int p = range_start + kl;
        if (p <= N) {
            tr_ptr[p] = run;
            // a row read by more than DN_LONG_GROUP slots is registered for the workgroups that sum such rows
            if (tot > DN_LONG_GROUP) tr_long[run / DN_LONG_GROUP] = p + 1;
        }
        int c = run;
#pragma unroll
        for (int w = 0; w < SMALL_WAVES; ++w) {
            const int x = cnt[w][kl];
            cnt[w][kl] = c;                                    // the cursor of (wave, key)
            c += x;
        }
    }
    __syncthreads();

    // ---- pass 2: places.  From the wave's list, 64 entries at a time in list order (= pair order)...
    if (list_n <= SMALL_LIST_CAP) {
        for (int base = 0; base < list_n; base += 64) {
            const bool mine = base + lane < list_n;
            const uint32_t ent = mine ? s_list[wave][base + lane] : 0u;
            const int kl = (int)(ent >> 16);
            int rank, count;
            step_peers(kl, mine, lane, rank, count);
            if (mine) tr_val[cnt[wave][kl] + rank] = first + s_begin * 64 + (int)(ent & 0xffffu);
            __builtin_amdgcn_wave_barrier();                   // every lane has read the cursor before its leader moves it
            if (mine && rank == 0) cnt[wave][kl] += count;
            __builtin_amdgcn_wave_barrier();
        }
    } else
    // ... or, for a wave whose list did not fit, from the keys again (a batch of loads at a time; the stores are not waited for)
    for (int st = s_begin; st < s_end; st += SMALL_BATCH) {
        int kv[SMALL_BATCH];
#pragma unroll
        for (int u = 0; u < SMALL_BATCH; ++u) {
            const int i = (st + u) * 64 + lane;
            kv[u] = (st + u < s_end && i < n) ? keys[i] - range_start : NONE;
        }
#pragma unroll
        for (int u = 0; u < SMALL_BATCH; ++u) {
            const int kl = kv[u];
            const bool mine = kl >= 0 && kl < SMALL_KEYS;
            // a workgroup owns 512 of ~100k keys: three of four steps hold none of its pairs, and the kernel is bound
            // by the instructions its 16 waves issue on one compute unit, so those steps end here
            if (__ballot(mine) == 0) continue;
            int rank, count;
            step_peers(kl, mine, lane, rank, count);
            if (mine) tr_val[cnt[wave][kl] + rank] = first + (st + u) * 64 + lane;
            __builtin_amdgcn_wave_barrier();                   // every lane has read the cursor before its leader moves it
            if (mine && rank == 0) cnt[wave][kl] += count;
            __builtin_amdgcn_wave_barrier();
        }
    }
    __syncthreads();                                           // this workgroup's part of tr_val is written

    // ---- owner and 1 / count of every slot placed by this workgroup (a thread per place: the loads run side by side)
    for (int t = threadIdx.x; t < mine_total; t += SMALL_TPB) {
        const int j = tr_val[before + t];
        const int q = slot_owner[j];
        tr_own[before + t] = q;
        tr_inv[before + t] = 1.0f / (float)(nbr_offsets[q + 1] - nbr_offsets[q]);
    }
}

}  // namespace

dn_sort_plan dn_sort_make_plan(int64_t key_range, int64_t cap_items)
{
    dn_sort_plan p;
    int key_bits = 1;
    while (((int64_t)1 << key_bits) < key_range) ++key_bits;
    p.passes = (key_bits + MAX_BITS - 1) / MAX_BITS;
    p.bits = (key_bits + p.passes - 1) / p.passes;           // bits per pass, <= MAX_BITS
    const int64_t nb = (cap_items + TILE - 1) / TILE;        // always planned for the capacity, so the extent is fixed
    p.nblocks = (int)(nb > 0 ? nb : 1);
    p.total = (1 << p.bits) * p.nblocks;
    p.sblocks = (p.total + TILE - 1) / TILE;
    return p;
}

// Sorts planned for more than two million pairs count digits in a pass of their own (k_radix_hist); the caller's
// first kernel then leaves the histogram alone.
bool dn_sort_counts_separately(const dn_sort_plan& p) { return p.nblocks > 2048; }

// ints of histogram space (two alternating histograms of counts, the scanned offsets, scan partials); they must
// start at zero
static int64_t hist_stride(const dn_sort_plan& p) { return ((int64_t)p.total + 3) & ~(int64_t)3; }   // 16-byte loads
int64_t dn_sort_hist_words(const dn_sort_plan& p) { return 3 * hist_stride(p) + p.sblocks + 64; }

// histograms up to this many ints (by capacity) are scanned by one kernel (k_scan_single)
constexpr int64_t SINGLE_SCAN_MAX = 1 << 20;

// Sorts the pairs that the caller's first kernel left in key[plan.passes & 1] / val[plan.passes & 1]
// (with the first digit's per-tile counts in hist[0 .. total)) by key, stably; the result is in
// key[0] / val[0], and ptr_out[p] = first sorted index with key >= p for p = 0 .. number of keys.
int dn_sort_pairs_run(const dn_sort_plan& pl, const int32_t* count_ptr, int32_t* const key[2], int32_t* const val[2],
                      int32_t* hist_space, const int32_t* nkeys_ptr, int64_t nkeys_cap, int32_t* ptr_out, hipStream_t st,
                      const dn_sort_slot_info* info)
{
    int32_t* hist[2] = { hist_space, hist_space + hist_stride(pl) };
    int32_t* offs = hist_space + 2 * hist_stride(pl);
    int32_t* part = hist_space + 3 * hist_stride(pl);
    const bool single = pl.total <= SINGLE_SCAN_MAX;
    int src = pl.passes & 1;                                // so that the last pass lands in buffer 0
    int h = 0;                                              // histogram buffer 0 is zero on entry
    const bool big = dn_sort_counts_separately(pl);
    int hist_grid = pl.nblocks < 4096 ? pl.nblocks : 4096;
    if (big) {
        // the caller's kernel left the first digit uncounted
        hipLaunchKernelGGL(k_radix_hist, dim3(hist_grid), dim3(TPB), 0, st, count_ptr, key[src], 0, pl.bits, hist[0]);
        DN_LAUNCH_CHECK("k_radix_hist");
    }
    for (int p = 0; p < pl.passes; ++p) {
        const int shift = pl.bits * p;
        const int hn = h ^ 1;
        if (single) {
            hipLaunchKernelGGL(k_scan_single, dim3(pl.sblocks), dim3(TPB), 0, st, hist[h], count_ptr, 1 << pl.bits, offs);
            DN_LAUNCH_CHECK("k_scan_single");
        } else {
            hipLaunchKernelGGL(k_scan_partial, dim3(pl.sblocks), dim3(TPB), 0, st, hist[h], count_ptr, 1 << pl.bits, part);
            DN_LAUNCH_CHECK("k_scan_partial");
            hipLaunchKernelGGL(k_scan_apply, dim3(pl.sblocks), dim3(TPB), 0, st, hist[h], count_ptr, 1 << pl.bits, part, offs);
            DN_LAUNCH_CHECK("k_scan_apply");
        }
        const int next_bits = (p + 1 < pl.passes) ? pl.bits : 0;
        hipLaunchKernelGGL(k_radix_scatter, dim3(pl.nblocks), dim3(TPB), 0, st, count_ptr, key[src], val[src],
                           shift, pl.bits, offs, key[src ^ 1], val[src ^ 1], big ? 0 : next_bits, hist[hn], hist[h]);
        DN_LAUNCH_CHECK("k_radix_scatter");
        if (big && next_bits > 0) {
            hipLaunchKernelGGL(k_radix_hist, dim3(hist_grid), dim3(TPB), 0, st, count_ptr, key[src ^ 1], shift + pl.bits, pl.bits,
                               hist[hn]);
            DN_LAUNCH_CHECK("k_radix_hist");
        }
        src ^= 1;
        h = hn;
    }
    int64_t gp = (nkeys_cap + 1 + TPB - 1) / TPB;
    if (gp > 2048) gp = 2048;
    dn_sort_slot_info si = { nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0 };
    if (info) si = *info;
    hipLaunchKernelGGL(k_tr_ptr, dim3((int)gp), dim3(TPB), 0, st, count_ptr, nkeys_ptr, (int)nkeys_cap, key[0], ptr_out,
                       val[0], offs, pl.bits * (pl.passes - 1), 1 << pl.bits, si);
    DN_LAUNCH_CHECK("k_tr_ptr");
    return DN_OK;
}

int64_t dn_transpose_index_hist_words(const dn_batch* b)
{
    return dn_sort_hist_words(dn_sort_make_plan(b->cap_nodes, b->cap_slots));
}

int dn_launch_transpose_index(dn_batch* b, int need_all, hipStream_t st)
{
    // Built already for this sample?  Work recorded into a HIP graph has not run: captured builds are tracked apart
    // from executed ones, so that an eager call after a capture still builds, and a capture after an eager build too.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) { (void)hipGetLastError(); cap = hipStreamCaptureStatusNone; }
    const bool capturing = cap == hipStreamCaptureStatusActive;
    uint64_t& serial = capturing ? b->tr_capture_serial : b->tr_serial;
    int32_t& covers = capturing ? b->tr_capture_covers_all : b->tr_covers_all;
    if (serial == b->sample_serial && (covers || !need_all)) return DN_OK;
    dn_prof_scope ps("transpose_index", 0, st);             // the whole build counts as one step
    // A few ten thousand pairs: the one-kernel form.  The host does not know the count (it lives on the device); it
    // goes by the largest counts that dn_batch_counts has read back for this batch object so far.  Both forms are
    // correct for any count; the choice only decides the time.
    const int64_t seen_pairs = need_all ? b->seen_slots_all : b->seen_slots_upper;
    if (seen_pairs >= 0 && seen_pairs <= DN_TR_SMALL_MAX_PAIRS) {
        const unsigned grid = (unsigned)((b->cap_nodes + 1 + SMALL_KEYS - 1) / SMALL_KEYS);
        hipLaunchKernelGGL(k_tr_small, dim3(grid), dim3(SMALL_TPB), 0, st, b->hdr, need_all, b->k, b->nbr_offsets, b->repr_map,
                           b->slot_owner, b->tr_ptr, b->tr_val[0], b->tr_own, b->tr_inv, b->tr_long);
        DN_LAUNCH_CHECK("k_tr_small");
        serial = b->sample_serial;
        covers = need_all ? 1 : 0;
        return DN_OK;
    }
    const dn_sort_plan pl = dn_sort_make_plan(b->cap_nodes, b->cap_slots);
    if (dn_sort_hist_words(pl) > b->tr_hist_words) return dn_fail(DN_ECAPACITY, "transpose index: histogram space");
    int64_t g = (b->cap_slots + TPB - 1) / TPB;
    if (g > 2048) g = 2048;
    if (g < 1) g = 1;
    const int src = pl.passes & 1;
    hipLaunchKernelGGL(k_tr_init, dim3((int)g), dim3(TPB), 0, st, b->hdr, need_all, b->k, b->nbr_offsets, b->repr_map,
                       b->tr_key[src], b->tr_val[src], (1 << pl.bits) - 1,
                       dn_sort_counts_separately(pl) ? nullptr : b->tr_hist, b->tr_long,
                       (int)b->tr_long_words);
    DN_LAUNCH_CHECK("k_tr_init");
    const dn_sort_slot_info info = { b->slot_owner, b->nbr_offsets, b->tr_own, b->tr_inv, b->tr_long, b->hdr, need_all ? 1 : 0 };
    const int rc = dn_sort_pairs_run(pl, b->hdr + HDR_TR_COUNT, b->tr_key, b->tr_val, b->tr_hist, b->hdr + HDR_N,
                                     b->cap_nodes, b->tr_ptr, st, &info);
    if (rc != DN_OK) return rc;
    serial = b->sample_serial;
    covers = need_all ? 1 : 0;
    return DN_OK;
}
