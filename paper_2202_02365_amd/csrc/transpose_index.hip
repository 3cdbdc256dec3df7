// Transpose index of repr_map for the backward pass: neighbour slots grouped by the node_ids
// position they read, ascending slot number inside a group, so that the gradient of the
// neighbour mean is a gather with a fixed summation order (no floating-point atomics).
// Built by a stable least-significant-digit radix sort of (repr_map[j], j) pairs, 8 bits per
// pass; group boundaries by binary search.  The number of pairs lives in device memory; grids
// are sized by capacity.
#include "dn_internal.h"

namespace {

constexpr int TPB = 256;
constexpr int ITEMS = 8;                   // elements per thread
constexpr int TILE = TPB * ITEMS;          // elements per workgroup
constexpr int RADIX = 256;

__global__ void k_tr_init(int32_t* __restrict__ hdr, int need_all, int k, const int32_t* __restrict__ nbr_offsets,
                          const int32_t* __restrict__ repr_map, int32_t* __restrict__ key, int32_t* __restrict__ val)
{
    const int E = hdr[HDR_E];
    int first = 0;
    if (!need_all) {
        // gradients reach the inputs of layers 2..k only: slots owned by Delta_2 .. Delta_k
        first = k >= 2 ? nbr_offsets[hdr[HDR_NODE_OFF + 2] - hdr[HDR_NODE_OFF + 1]] : E;
    }
    const int cnt = E - first;
    const int stride = gridDim.x * blockDim.x;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < cnt; i += stride) {
        key[i] = repr_map[first + i];
        val[i] = first + i;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        hdr[HDR_TR_FIRST] = first;
        hdr[HDR_TR_COUNT] = cnt;
    }
}

// digit histogram of each tile, stored digit-major: hist[d * nblocks + block]
__global__ __launch_bounds__(TPB) void k_radix_hist(const int32_t* __restrict__ hdr, const int32_t* __restrict__ key,
                                                    int shift, int nblocks, int32_t* __restrict__ hist)
{
    __shared__ int lh[RADIX];
    const int n = hdr[HDR_TR_COUNT];
    lh[threadIdx.x] = 0;
    __syncthreads();
    const int base = blockIdx.x * TILE;
    for (int it = 0; it < ITEMS; ++it) {
        const int idx = base + it * TPB + threadIdx.x;
        if (idx < n) atomicAdd(&lh[(key[idx] >> shift) & (RADIX - 1)], 1);
    }
    __syncthreads();
    hist[threadIdx.x * nblocks + blockIdx.x] = lh[threadIdx.x];
}

// two-kernel exclusive scan of `total` ints in place (block partial sums, then look-behind)
__global__ __launch_bounds__(TPB) void k_scan_partial(const int32_t* __restrict__ data, int total, int32_t* __restrict__ part)
{
    __shared__ int sm[TPB / 64];
    const int base = blockIdx.x * TILE + threadIdx.x * ITEMS;
    int s = 0;
    for (int e = 0; e < ITEMS; ++e) if (base + e < total) s += data[base + e];
    for (int d = 32; d > 0; d >>= 1) s += __shfl_down(s, d, 64);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = sm[0] + sm[1] + sm[2] + sm[3];
}

__global__ __launch_bounds__(TPB) void k_scan_apply(int32_t* __restrict__ data, int total, const int32_t* __restrict__ part)
{
    __shared__ int sm[TPB / 64];
    __shared__ int s_before;
    // sum of the partials of all earlier blocks
    int acc = 0;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += TPB) acc += part[i];
    for (int d = 32; d > 0; d >>= 1) acc += __shfl_down(acc, d, 64);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) s_before = sm[0] + sm[1] + sm[2] + sm[3];
    __syncthreads();
    const int before = s_before;
    // exclusive scan inside the block: per-thread serial over ITEMS, then across threads
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
        if (base + e < total) data[base + e] = run;
        run += v[e];
    }
}

// stable scatter: element order inside a tile is (wave, round, lane); a lane's rank among equal
// digits of its round comes from 8 ballots, rounds and waves are chained through counters in LDS.
__global__ __launch_bounds__(TPB) void k_radix_scatter(const int32_t* __restrict__ hdr, const int32_t* __restrict__ key_in,
                                                       const int32_t* __restrict__ val_in, int shift, int nblocks,
                                                       const int32_t* __restrict__ hist, int32_t* __restrict__ key_out,
                                                       int32_t* __restrict__ val_out)
{
    __shared__ int cnt[TPB / 64][RADIX];
    const int n = hdr[HDR_TR_COUNT];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (blockIdx.x * TILE >= n) return;
    for (int w = 0; w < TPB / 64; ++w) cnt[w][threadIdx.x] = 0;
    __syncthreads();
    const int wbase = blockIdx.x * TILE + wave * (TILE / (TPB / 64));
    int keys[ITEMS], vals[ITEMS];
    uint64_t peers[ITEMS];
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const int idx = wbase + r * 64 + lane;
        const bool ok = idx < n;
        keys[r] = ok ? key_in[idx] : 0;
        vals[r] = ok ? val_in[idx] : 0;
        const int d = (keys[r] >> shift) & (RADIX - 1);
        uint64_t mask = __ballot(ok);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const uint64_t bal = __ballot((d >> bit) & 1);
            mask &= ((d >> bit) & 1) ? bal : ~bal;
        }
        peers[r] = ok ? mask : 0ull;
        if (ok && (mask & ((1ull << lane) - 1ull)) == 0) cnt[wave][d] += __popcll(mask);   // lowest lane of each digit
        __syncthreads();                       // the next round's leader may be another lane
    }
    {   // thread t owns digit t: turn per-wave counts into per-wave start positions
        int g = hist[threadIdx.x * nblocks + blockIdx.x];
        for (int w = 0; w < TPB / 64; ++w) {
            const int c = cnt[w][threadIdx.x];
            cnt[w][threadIdx.x] = g;
            g += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const uint64_t mask = peers[r];
        if (mask) {
            const int d = (keys[r] >> shift) & (RADIX - 1);
            const int start = cnt[wave][d];
            __builtin_amdgcn_wave_barrier();   // all lanes have read the counter before its owner advances it
            const int rank = __popcll(mask & ((1ull << lane) - 1ull));
            key_out[start + rank] = keys[r];
            val_out[start + rank] = vals[r];
            if (rank == 0) cnt[wave][d] = start + __popcll(mask);
        }
        __syncthreads();                       // counters are read by every lane of the next round
    }
}

// tr_ptr[p] = first index of sorted keys >= p, for p = 0..N
__global__ __launch_bounds__(TPB) void k_tr_ptr(const int32_t* __restrict__ hdr, const int32_t* __restrict__ key,
                                                int32_t* __restrict__ tr_ptr)
{
    const int N = hdr[HDR_N], n = hdr[HDR_TR_COUNT];
    const int stride = gridDim.x * TPB;
    for (int p = blockIdx.x * TPB + threadIdx.x; p <= N; p += stride) {
        int lo = 0, hi = n;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (key[mid] < p) lo = mid + 1; else hi = mid;
        }
        tr_ptr[p] = lo;
    }
}

}  // namespace

int dn_launch_transpose_index(dn_batch* b, int need_all, hipStream_t st)
{
    if (b->tr_serial == b->sample_serial && (b->tr_covers_all || !need_all)) return DN_OK;
    int64_t cap = b->cap_slots;
    if (!need_all) cap -= b->cap_slots_hop[b->k - 1];      // the last hop's slots belong to layer 1 only
    int bits = 1;
    while (((int64_t)1 << bits) < b->cap_nodes) ++bits;
    const int passes = (bits + 7) / 8;
    int src = passes & 1;                                   // so that the last pass lands in buffer 0
    int64_t g = (cap + TPB - 1) / TPB;
    if (g > 2048) g = 2048;
    if (g < 1) g = 1;
    dn_prof_scope ps("transpose_index", 0, st);       // the whole sort counts as one step
    hipLaunchKernelGGL(k_tr_init, dim3((int)g), dim3(TPB), 0, st, b->hdr, need_all, b->k, b->nbr_offsets, b->repr_map,
                       b->tr_key[src], b->tr_val[src]);
    DN_LAUNCH_CHECK("k_tr_init");
    if (cap > 0) {
        const int nblocks = (int)((cap + TILE - 1) / TILE);
        const int total = RADIX * nblocks;
        const int sblocks = (total + TILE - 1) / TILE;
        if ((int64_t)total + sblocks > b->tr_hist_words) return dn_fail(DN_ECAPACITY, "transpose index: histogram space");
        int32_t* part = b->tr_hist + total;
        for (int p = 0; p < passes; ++p) {
            const int shift = 8 * p;
            hipLaunchKernelGGL(k_radix_hist, dim3(nblocks), dim3(TPB), 0, st, b->hdr, b->tr_key[src], shift, nblocks,
                               b->tr_hist);
            DN_LAUNCH_CHECK("k_radix_hist");
            hipLaunchKernelGGL(k_scan_partial, dim3(sblocks), dim3(TPB), 0, st, b->tr_hist, total, part);
            DN_LAUNCH_CHECK("k_scan_partial");
            hipLaunchKernelGGL(k_scan_apply, dim3(sblocks), dim3(TPB), 0, st, b->tr_hist, total, part);
            DN_LAUNCH_CHECK("k_scan_apply");
            hipLaunchKernelGGL(k_radix_scatter, dim3(nblocks), dim3(TPB), 0, st, b->hdr, b->tr_key[src], b->tr_val[src],
                               shift, nblocks, b->tr_hist, b->tr_key[src ^ 1], b->tr_val[src ^ 1]);
            DN_LAUNCH_CHECK("k_radix_scatter");
            src ^= 1;
        }
    }
    int64_t gp = (b->cap_nodes + 1 + TPB - 1) / TPB;
    if (gp > 2048) gp = 2048;
    hipLaunchKernelGGL(k_tr_ptr, dim3((int)gp), dim3(TPB), 0, st, b->hdr, b->tr_key[0], b->tr_ptr);
    DN_LAUNCH_CHECK("k_tr_ptr");
    b->tr_serial = b->sample_serial;
    b->tr_covers_all = need_all ? 1 : 0;
    return DN_OK;
}
