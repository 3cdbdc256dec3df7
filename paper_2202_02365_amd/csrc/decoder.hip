// DistMult decoder with shared negatives (link prediction; the paper names the score function in
// Section 7.1 and uses 500 negatives per edge in Section 7.3, without formulas: textbook DistMult,
// softmax cross-entropy of the positive against each corrupted side's negatives).
//
//   score f(s, r, d) = sum_j h_s[j] r[j] h_d[j];  edges are cut into chunks of `chunk` consecutive
//   edges, chunk q shares the negative nodes neg[q, 0..Nn).  Corrupted destination: f(s, r, neg),
//   corrupted source: f(neg, r, d).  Per edge: loss = sum over the two sides of
//   logsumexp([pos, negs]) - pos.
//
// The negatives' scores are the dense contraction: per (side, chunk) one
//   S[chunk x Nn] = Q[chunk x d] * E[Nn x d]^T,   Q = bf16(h_a * r), E = bf16(h_neg)
// on bf16 MFMA (reduction length padded to a multiple of 64), batched over sides and chunks in one
// launch.  The forward pass keeps only each row's log-sum-exp of them.  Backward computes the scores again and
// turns them into P = softmax probabilities of the negatives in the same kernel, then has two more
// contractions per (side, chunk): dQ = P * E and dE = P^T * Q.  P is computed on the device (its last bits differ from
// any other implementation's), so it enters as two bf16 terms hi + lo, two column blocks of one row-major
// matrix.  dQ contracts over the negatives (P's columns): the terms lie side by side along the reduction
// index and E^T's tile loads wrap round.  dE contracts over the chunk's edges (the rows of P and of Q): both
// are read as they lie in memory through the LDS transpose read, and the two terms come out as two row
// blocks of the result.  Row-wise sums that collect
// the per-edge / per-negative gradients into dH and dR run over an index sorted by node (relation)
// in a fixed order: no floating-point atomics, bit-identical from run to run.
//
// All padding rows and columns of the bf16 operands are written as zeros by the kernels that
// produce them, so no tile load needs a bounds check and no padding value reaches a sum.
#include "dn_internal.h"
#include "mfma_tile.h"
#include <new>
#include <cstring>

using namespace dn_mma;

enum { DM_HDR_STATUS = 0, DM_HDR_NODE_COUNT = 1, DM_HDR_REL_COUNT = 2, DM_HDR_STATUS_ACC = 3, DM_HDR_WORDS = 16 };
enum { DM_BAD_NODE = 1, DM_BAD_REL = 2 };

struct dn_decoder {
    int64_t max_edges, max_rows, num_rel;
    int32_t chunk, num_neg, dim;
    int32_t kp;        // dim rounded up to 64: reduction length of the score contraction
    int32_t np;        // dim rounded up to 128: row count of the transposed operands / width of dQ, dE
    int32_t cpad;      // chunk rounded up to 128
    int32_t npad;      // num_neg rounded up to 128
    int64_t max_chunks;
    int64_t max_entries;              // 2 * max_edges + max_chunks * num_neg index entries
    // workspace
    int32_t* hdr;
    dn_bf16 *Q, *En, *Ent, *P;
    float *S, *lse, *dpos, *dQ, *dEn, *rows, *long_partial, *pmax, *psum;
    int32_t *nkey[2], *nval[2], *nptr, *nhist;
    int32_t *rkey[2], *rval[2], *rptr, *rhist;
    int32_t* long_seg;                // per 64-row block of a sorted index: long segment starting there + 1, or 0
    dn_sort_plan nplan, rplan;
    // inputs of the last forward (borrowed)
    const float *H, *R;
    int64_t ldh, ldr, n_rows, n_edges, n_chunks;
    const int32_t *src, *rel, *dst, *neg;
    int32_t have_forward;
    size_t workspace_bytes;
};

namespace {

constexpr int TPB_ = 256;

// ------------------------------------------------------------------ operands of the score contraction
// One group of 16 lanes per operand row.  Rows [0, 2*C*cpad): Q[side][q][i] = bf16(h_a * r) for edge
// e = q*chunk + i (a = source for side 0, destination for side 1), zero rows where there is no edge.
// Rows after that: En[q][n] = bf16(h_neg[q][n]), zero rows for n >= Nn.  Side-0 groups also compute
// the positive's score in fp32.
__global__ __launch_bounds__(TPB_) void k_dm_prepare(const float* __restrict__ H, int64_t ldh, int n_rows,
                                                     const float* __restrict__ R, int64_t ldr, int num_rel,
                                                     const int32_t* __restrict__ src, const int32_t* __restrict__ rel,
                                                     const int32_t* __restrict__ dst, const int32_t* __restrict__ neg,
                                                     int B, int C, int chunk, int Nn, int d, int kp, int cpad, int npad,
                                                     uint16_t* __restrict__ Q, uint16_t* __restrict__ En,
                                                     float* __restrict__ pos, int32_t* __restrict__ hdr)
{
    const int64_t row = ((int64_t)blockIdx.x * TPB_ + threadIdx.x) >> 4;
    const int sl = threadIdx.x & 15;
    const int64_t q_rows = 2ll * C * cpad;
    if (row >= q_rows + (int64_t)C * npad) return;
    if (row < q_rows) {
        const int side = (int)(row / ((int64_t)C * cpad));
        const int64_t rem = row - (int64_t)side * C * cpad;
        const int q = (int)(rem / cpad), i = (int)(rem % cpad);
        const int64_t e = (int64_t)q * chunk + i;
        uint16_t* out = Q + row * kp;
        bool ok = i < chunk && e < B;
        int a = 0, o = 0, rr = 0;
        if (ok) {
            a = side == 0 ? src[e] : dst[e];
            o = side == 0 ? dst[e] : src[e];
            rr = rel[e];
            if ((unsigned)a >= (unsigned)n_rows || (unsigned)o >= (unsigned)n_rows) { ok = false; if (sl == 0) atomicOr(&hdr[DM_HDR_STATUS_ACC], DM_BAD_NODE); }
            if ((unsigned)rr >= (unsigned)num_rel) { ok = false; if (sl == 0) atomicOr(&hdr[DM_HDR_STATUS_ACC], DM_BAD_REL); }
        }
        const float* ha = H + (int64_t)a * ldh;
        const float* ho = H + (int64_t)o * ldh;
        const float* rv = R + (int64_t)rr * ldr;
        float acc = 0.f;
        for (int j = sl; j < kp; j += 16) {
            float qv = 0.f;
            if (ok && j < d) {
                qv = ha[j] * rv[j];
                acc += qv * ho[j];
            }
            out[j] = f32_to_bf16(qv);
        }
        if (side == 0 && i < chunk && e < B) {
            for (int s = 8; s > 0; s >>= 1) acc += __shfl_down(acc, s, 16);
            if (sl == 0) pos[e] = acc;
        }
    } else {
        const int64_t rem = row - q_rows;
        const int q = (int)(rem / npad), n = (int)(rem % npad);
        uint16_t* out = En + rem * kp;
        bool ok = n < Nn;
        int v = 0;
        if (ok) {
            v = neg[(int64_t)q * Nn + n];
            if ((unsigned)v >= (unsigned)n_rows) { ok = false; if (sl == 0) atomicOr(&hdr[DM_HDR_STATUS_ACC], DM_BAD_NODE); }
        }
        const float* hv = H + (int64_t)v * ldh;
        for (int j = sl; j < kp; j += 16) out[j] = f32_to_bf16(ok && j < d ? hv[j] : 0.f);
    }
}

// out[b][c][r] = in[b][r][c] for r < rows, c < cols (bf16, 64 x 64 tiles through LDS); rows and cols are multiples of 64
__global__ __launch_bounds__(TPB_) void k_dm_transpose(const uint16_t* __restrict__ in, int rows, int cols,
                                                       uint16_t* __restrict__ out, int64_t out_batch_stride)
{
    __shared__ uint16_t tile[64][66];
    const int64_t b = blockIdx.z;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const uint16_t* src = in + b * (int64_t)rows * cols;
    uint16_t* dst = out + b * out_batch_stride;
    for (int rr = ty; rr < 64; rr += 4) tile[rr][tx] = src[(int64_t)(r0 + rr) * cols + c0 + tx];
    __syncthreads();
    for (int cc = ty; cc < 64; cc += 4) dst[(int64_t)(c0 + cc) * rows + r0 + tx] = tile[tx][cc];
}

// ------------------------------------------------------------------ batched contraction C[z] = A[z] * B[z % b_mod]^T
struct DmGemm {
    const uint16_t* A; int64_t lda, stride_a;
    const uint16_t* B; int64_t ldb, stride_b; int b_mod;
    int kchunks;            // reduction length of A in units of 64
    int b_wrap_chunks;      // B repeats after this many units (WRAP only)
    float* C; int64_t ldc, stride_c;
    int ncols;              // columns stored (rows: every row of the tile; C is padded to whole tiles)
    // LSE epilogue: per row and column tile, max and sum of exp(x - max) over the tile's columns below lse_cols
    float* pmax; float* psum; int lse_cols;
    // probability epilogue: P = exp(x - lse) for valid (edge, negative) pairs, 0 elsewhere, as two bf16 terms
    const float* lse; int n_edges, n_chunks, chunk, n_neg, npad; uint16_t* P;
};

// What becomes of the tile: stored as it is; reduced to the (max, sum of exp) pairs of its rows (the scores
// themselves are not kept: whoever needs them again computes them again, which costs less than 0.4 GB of
// writes and as much of reads); or turned into probabilities with the rows' finished log-sum-exp.
enum { DM_EPI_STORE = 0, DM_EPI_LSE = 1, DM_EPI_PROBS = 2 };

template <bool WRAP, int EPI>
__global__ __launch_bounds__(TPB, 2) void k_dm_gemm(DmGemm g)
{
    const int z = blockIdx.z;
    const int row0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    const uint16_t* A = g.A + (int64_t)z * g.stride_a + (int64_t)row0 * g.lda;
    const uint16_t* B = g.B + (int64_t)(z % g.b_mod) * g.stride_b + (int64_t)col0 * g.ldb;
    f32x16 acc[2][2];
    mainloop<BM, BN, WRAP>(A, g.lda, B, g.ldb, 0, g.kchunks, g.b_wrap_chunks, acc);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    if (EPI == DM_EPI_STORE) {
        float* C = g.C + (int64_t)z * g.stride_c;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = col0 + wn * 64 + j * 32 + (lane & 31);
                if (n >= g.ncols) continue;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = row0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    C[(int64_t)m * g.ldc + n] = acc[i][j][e];
                }
            }
    }
    if (EPI == DM_EPI_PROBS) {
        // P[z][m][term * npad + n] (z = side * n_chunks + q), every element of the padded tile written
        const int side = z / g.n_chunks, q = z % g.n_chunks;
        uint16_t* Pz = g.P + (int64_t)z * ((int64_t)gridDim.y * BM) * 2 * g.npad;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = row0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const int64_t edge = (int64_t)q * g.chunk + m;
                const bool row_ok = m < g.chunk && edge < g.n_edges;
                const float l = row_ok ? g.lse[(int64_t)side * g.n_edges + edge] : 0.f;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int n = col0 + wn * 64 + j * 32 + (lane & 31);
                    const float pr = (row_ok && n < g.n_neg) ? expf(acc[i][j][e] - l) : 0.f;
                    const uint16_t hi = f32_to_bf16(pr);
                    const uint16_t lo = f32_to_bf16(pr - bf16_to_f32(hi));
                    Pz[(int64_t)m * 2 * g.npad + n] = hi;
                    Pz[(int64_t)m * 2 * g.npad + g.npad + n] = lo;
                }
            }
    }
    if (EPI == DM_EPI_LSE) {
        // per row: max and sum of exp(x - max) over this tile's valid columns.  A row's 128 columns sit in the 32
        // lanes of one half-wave (two registers each) of the two waves wn = 0, 1.  The 16 rows a lane holds
        // (for one i) are reduced over the half-wave by a butterfly that halves the number of rows a lane
        // carries at every step, so that 32 lane exchanges serve 16 rows; a (max, sum) pair merges as
        // max = larger max, sum = sum_of_larger + sum_of_smaller * exp(smaller max - larger max).
        __shared__ float s_max[2][BM], s_sum[2][BM];
        const int n0 = col0 + wn * 64 + (lane & 31), n1 = n0 + 32;
        const bool ok0 = n0 < g.lse_cols, ok1 = n1 < g.lse_cols;
        auto merge = [](float& m, float& sm, const float m2, const float s2) {
            const float big = fmaxf(m, m2), small = fminf(m, m2);
            const float s_big = m >= m2 ? sm : s2, s_small = m >= m2 ? s2 : sm;
            sm = s_big + (small > -INFINITY ? s_small * __expf(small - big) : 0.f);   // hardware exp2: error ~1e-7 |x|, far below the sums' own
            m = big;
        };
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float pm[16], ps[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float v0 = ok0 ? acc[i][0][e] : -INFINITY, v1 = ok1 ? acc[i][1][e] : -INFINITY;
                pm[e] = v0;
                ps[e] = ok0 ? 1.f : 0.f;
                merge(pm[e], ps[e], v1, ok1 ? 1.f : 0.f);
            }
#pragma unroll
            for (int half = 8; half >= 1; half >>= 1) {
                const int sft = half * 2;                       // lane bit that decides which half this lane keeps
                const bool upper = (lane & sft) != 0;
#pragma unroll
                for (int k = 0; k < half; ++k) {
                    const float send_m = upper ? pm[k] : pm[k + half], send_s = upper ? ps[k] : ps[k + half];
                    float keep_m = upper ? pm[k + half] : pm[k], keep_s = upper ? ps[k + half] : ps[k];
                    const float rm = __shfl_xor(send_m, sft, 64), rs = __shfl_xor(send_s, sft, 64);
                    merge(keep_m, keep_s, rm, rs);
                    pm[k] = keep_m;
                    ps[k] = keep_s;
                }
            }
            {   // last lane bit: both partners end with the full result
                const float rm = __shfl_xor(pm[0], 1, 64), rs = __shfl_xor(ps[0], 1, 64);
                merge(pm[0], ps[0], rm, rs);
            }
            if ((lane & 1) == 0) {
                const int e = (lane & 31) >> 1;                 // the register index whose row this lane ended up with
                const int ml = wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                s_max[wn][ml] = pm[0];
                s_sum[wn][ml] = ps[0];
            }
        }
        __syncthreads();
        if (t < BM) {
            const float m0 = s_max[0][t], m1 = s_max[1][t];
            const float mx = fmaxf(m0, m1);
            float sm = 0.f;
            if (mx > -INFINITY) sm = (m0 > -INFINITY ? s_sum[0][t] * expf(m0 - mx) : 0.f) + (m1 > -INFINITY ? s_sum[1][t] * expf(m1 - mx) : 0.f);
            const int64_t idx = ((int64_t)z * (gridDim.y * BM) + row0 + t) * gridDim.x + blockIdx.x;
            g.pmax[idx] = mx;
            g.psum[idx] = sm;
        }
    }
}

// ------------------------------------------------------------------ softmax over [pos, negatives]
// One thread per edge, both sides: combines the score contraction's per-tile (max, sum) pairs with the
// positive: lse[side][e], loss[e] = (lse0 - pos) + (lse1 - pos), dpos[e] = (exp(pos - lse0) - 1) + (exp(pos - lse1) - 1).
__global__ __launch_bounds__(TPB_) void k_dm_lse(const float* __restrict__ pmax, const float* __restrict__ psum,
                                                 const float* __restrict__ pos, int B, int C, int chunk, int cpad, int ntn,
                                                 float* __restrict__ lse, float* __restrict__ loss, float* __restrict__ dpos,
                                                 int32_t* __restrict__ hdr)
{
    const int e = blockIdx.x * TPB_ + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x == 0) {      // flags raised by the operand kernel of this call become the status
        hdr[DM_HDR_STATUS] = hdr[DM_HDR_STATUS_ACC];
        hdr[DM_HDR_STATUS_ACC] = 0;
    }
    if (e >= B) return;
    const int q = e / chunk, i = e % chunk;
    const float p = pos[e];
    float l[2];
    for (int side = 0; side < 2; ++side) {
        const int64_t base = (((int64_t)side * C + q) * cpad + i) * ntn;
        float m = p;
        for (int tn = 0; tn < ntn; ++tn) m = fmaxf(m, pmax[base + tn]);
        float sum = expf(p - m);
        for (int tn = 0; tn < ntn; ++tn) {
            const float pm = pmax[base + tn];
            if (pm > -INFINITY) sum += psum[base + tn] * expf(pm - m);
        }
        l[side] = m + logf(sum);
        lse[(int64_t)side * B + e] = l[side];
    }
    loss[e] = (l[0] - p) + (l[1] - p);
    dpos[e] = (expf(p - l[0]) - 1.f) + (expf(p - l[1]) - 1.f);
}

// dE[z] = P[z]^T * Q[z]: the contraction runs over the chunk's edges, the row index of both P and Q, so both are
// read as they lie in memory through the LDS transpose read (mainloop_tn).  The two terms of P are two column
// blocks of it, i.e. two row blocks of the result: C[z] is [2*npad x np], rows [0, npad) from the hi term and
// [npad, 2*npad) from the lo term; whoever consumes dE adds the two.
struct DmGemmTn {
    const uint16_t* A; int64_t lda, stride_a; int a_cols;
    const uint16_t* B; int64_t ldb, stride_b; int b_cols;
    int k_rows;
    float* C; int64_t ldc, stride_c; int ncols;
};
__global__ __launch_bounds__(TPB, 2) void k_dm_gemm_tn(DmGemmTn g)
{
    const int z = blockIdx.z;
    const int row0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    f32x16 acc[2][2];
    mainloop_tn<BM, BN>(g.A + (int64_t)z * g.stride_a, g.lda, g.a_cols, g.B + (int64_t)z * g.stride_b, g.ldb, g.b_cols, 1, 0, row0, col0,
                        0, (g.k_rows + BK - 1) / BK, g.k_rows, acc);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    float* C = g.C + (int64_t)z * g.stride_c;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = col0 + wn * 64 + j * 32 + (lane & 31);
            if (n >= g.ncols) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = row0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                C[(int64_t)m * g.ldc + n] = acc[i][j][e];
            }
        }
}

// One atomic per distinct digit among a wave's active lanes (all of a wave's elements lie in one tile):
// frequent keys (a popular relation, a hub node) would otherwise serialise on a few counters.
__device__ __forceinline__ void hist_add_wave(int32_t* __restrict__ hist, int digit, int bits, int nblocks, int tile)
{
    const int lane = threadIdx.x & 63;
    uint64_t mask = __ballot(1);
    for (int bit = 0; bit < bits; ++bit) {
        const uint64_t bal = __ballot((digit >> bit) & 1);
        mask &= ((digit >> bit) & 1) ? bal : ~bal;
    }
    if ((mask & ((1ull << lane) - 1ull)) == 0) atomicAdd(&hist[digit * nblocks + tile], __popcll(mask));
}

// ------------------------------------------------------------------ gradient collection
// Index entries: [0, B) edge e as a source, [B, 2B) edge e as a destination, [2B, 2B + C*Nn) negative
// slot (q, n); key = the row of H the entry's gradient goes to (out-of-range ids go to the extra key n_rows).
__global__ __launch_bounds__(TPB_) void k_dm_node_index_init(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                                             const int32_t* __restrict__ neg, int B, int n_neg, int n_rows,
                                                             int32_t* __restrict__ key, int32_t* __restrict__ val,
                                                             int radix_bits, int32_t* __restrict__ hist,
                                                             int32_t* __restrict__ hdr)
{
    const int radix_mask = (1 << radix_bits) - 1;
    const int total = 2 * B + n_neg;
    const int stride = gridDim.x * blockDim.x;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        int kv = i < B ? src[i] : (i < 2 * B ? dst[i - B] : neg[i - 2 * B]);
        if ((unsigned)kv >= (unsigned)n_rows) kv = n_rows;
        key[i] = kv;
        val[i] = i;
        if (hist) hist_add_wave(hist, kv & radix_mask, radix_bits, dn_sort_tiles(total), i / DN_SORT_TILE);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) hdr[DM_HDR_NODE_COUNT] = total;
}

__global__ __launch_bounds__(TPB_) void k_dm_rel_index_init(const int32_t* __restrict__ rel, int B, int num_rel,
                                                            int32_t* __restrict__ key, int32_t* __restrict__ val,
                                                            int radix_bits, int32_t* __restrict__ hist,
                                                            int32_t* __restrict__ hdr)
{
    const int radix_mask = (1 << radix_bits) - 1;
    const int stride = gridDim.x * blockDim.x;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < B; i += stride) {
        int kv = rel[i];
        if ((unsigned)kv >= (unsigned)num_rel) kv = num_rel;
        key[i] = kv;
        val[i] = i;
        if (hist) hist_add_wave(hist, kv & radix_mask, radix_bits, dn_sort_tiles(B), i / DN_SORT_TILE);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) hdr[DM_HDR_REL_COUNT] = B;
}

struct DmGrad {
    const float *H, *R; int64_t ldh, ldr; int n_rows, num_rel;
    const int32_t *src, *rel, *dst;
    const float *dpos, *dQ, *dEn;
    int B, C, chunk, Nn, d, np, cpad, npad;
};

__device__ __forceinline__ bool dm_edge_ok(const DmGrad& g, int e, int& s, int& o, int& r)
{
    s = g.src[e]; o = g.dst[e]; r = g.rel[e];
    return (unsigned)s < (unsigned)g.n_rows && (unsigned)o < (unsigned)g.n_rows && (unsigned)r < (unsigned)g.num_rel;
}

// rows[i][:] = gradient row of the i-th entry of the node index (sorted order), 32 lanes per entry:
//   edge e as a source:       dpos[e] * (r * h_dst) + dQ[0][e] * r
//   edge e as a destination:  dpos[e] * (r * h_src) + dQ[1][e] * r
//   negative slot (q, n):     dE[0][q][n] + dE[1][q][n]   (each the sum of its hi-term and lo-term rows)
__global__ __launch_bounds__(TPB_) void k_dm_node_rows(DmGrad g, const int32_t* __restrict__ val, int total,
                                                       float* __restrict__ rows)
{
    const int i = (blockIdx.x * TPB_ + threadIdx.x) >> 5, sl = threadIdx.x & 31;
    if (i >= total) return;
    const int v = val[i];
    float* out = rows + (int64_t)i * g.d;
    if (v < 2 * g.B) {
        const int side = v < g.B ? 0 : 1;
        const int e = v - side * g.B;
        int s, o, r;
        const bool ok = dm_edge_ok(g, e, s, o, r);
        const int q = e / g.chunk, ii = e % g.chunk;
        const float* other = g.H + (int64_t)(side == 0 ? o : s) * g.ldh;
        const float* rv = g.R + (int64_t)r * g.ldr;
        const float* dq = g.dQ + (((int64_t)side * g.C + q) * g.cpad + ii) * g.np;
        const float dp = ok ? g.dpos[e] : 0.f;
        for (int j = sl; j < g.d; j += 32) out[j] = ok ? dp * (rv[j] * other[j]) + dq[j] * rv[j] : 0.f;
    } else {
        const int m = v - 2 * g.B;
        const int q = m / g.Nn, n = m % g.Nn;
        // per side z: rows [0, npad) hold the hi-term part, rows [npad, 2 npad) the lo-term part
        const float* e0 = g.dEn + ((int64_t)q * 2 * g.npad + n) * g.np;
        const float* e1 = g.dEn + (((int64_t)g.C + q) * 2 * g.npad + n) * g.np;
        const int64_t lo = (int64_t)g.npad * g.np;
        for (int j = sl; j < g.d; j += 32) out[j] = (e0[j] + e0[lo + j]) + (e1[j] + e1[lo + j]);
    }
}

// rows[i][:] = dR contribution of the i-th edge of the relation index:
//   dpos[e] * (h_src * h_dst) + dQ[0][e] * h_src + dQ[1][e] * h_dst
__global__ __launch_bounds__(TPB_) void k_dm_rel_rows(DmGrad g, const int32_t* __restrict__ val, float* __restrict__ rows)
{
    const int i = (blockIdx.x * TPB_ + threadIdx.x) >> 5, sl = threadIdx.x & 31;
    if (i >= g.B) return;
    const int e = val[i];
    int s, o, r;
    const bool ok = dm_edge_ok(g, e, s, o, r);
    const int q = e / g.chunk, ii = e % g.chunk;
    const float* hs = g.H + (int64_t)s * g.ldh;
    const float* hd = g.H + (int64_t)o * g.ldh;
    const float* dq0 = g.dQ + (((int64_t)q) * g.cpad + ii) * g.np;
    const float* dq1 = g.dQ + (((int64_t)g.C + q) * g.cpad + ii) * g.np;
    const float dp = ok ? g.dpos[e] : 0.f;
    float* out = rows + (int64_t)i * g.d;
    for (int j = sl; j < g.d; j += 32) out[j] = ok ? dp * (hs[j] * hd[j]) + dq0[j] * hs[j] + dq1[j] * hd[j] : 0.f;
}

// out[s][:] = sum of rows[ptr[s] .. ptr[s+1]) in a fixed order.  Segments of at most LONG_SEG rows: 32 lanes
// per segment, ascending order.  Longer segments (a hub node, a frequent relation) are cut into LONG_PARTS
// slices, one workgroup each: the workgroup's 8 lane groups take the slice's rows g, g+8, ... in order and
// their sums are added in order of g; a second kernel adds the slices' sums in order.  A long segment is
// registered under the 64-row block its first row lies in (no two long segments start in one block):
// long_seg[block] = segment + 1, written by the short-segment kernel, reset to 0 by the last one, and the
// slices' partial sums are kept under the same block number.
constexpr int LONG_SEG = 64;
constexpr int LONG_PARTS = 64;
__global__ __launch_bounds__(TPB_) void k_dm_segment_sum(const float* __restrict__ rows, const int32_t* __restrict__ ptr,
                                                         int nseg, int d, float* __restrict__ out, int64_t ldo,
                                                         int32_t* __restrict__ long_seg)
{
    const int s = (blockIdx.x * TPB_ + threadIdx.x) >> 5, sl = threadIdx.x & 31;
    if (s >= nseg) return;
    const int lo = ptr[s], hi = ptr[s + 1];
    if (hi - lo > LONG_SEG) {
        if (sl == 0) long_seg[lo / LONG_SEG] = s + 1;
        return;
    }
    for (int j = sl; j < d; j += 32) {
        float acc = 0.f;
        for (int i = lo; i < hi; ++i) acc += rows[(int64_t)i * d + j];
        out[(int64_t)s * ldo + j] = acc;
    }
}

__global__ __launch_bounds__(TPB_) void k_dm_long_partial(const float* __restrict__ rows, const int32_t* __restrict__ ptr,
                                                          const int32_t* __restrict__ long_seg, int d,
                                                          float* __restrict__ partial)
{
    __shared__ float part[TPB_ / 32][32];
    constexpr int G = TPB_ / 32;
    const int c = blockIdx.x, p = blockIdx.y;
    const int s = long_seg[c] - 1;
    if (s < 0) return;
    const int lo = ptr[s], hi = ptr[s + 1];
    const int per = (hi - lo + LONG_PARTS - 1) / LONG_PARTS;
    const int begin = lo + p * per, end = min(hi, begin + per);
    const int grp = threadIdx.x >> 5, sl = threadIdx.x & 31;
    float* dst = partial + ((int64_t)c * LONG_PARTS + p) * d;
    for (int j0 = 0; j0 < d; j0 += 32) {
        const int j = j0 + sl;
        float acc = 0.f;
        if (j < d) {
            int i = begin + grp;
            for (; i + 3 * G < end; i += 4 * G) {          // four rows in flight, added in order
                const float a0 = rows[(int64_t)i * d + j], a1 = rows[(int64_t)(i + G) * d + j];
                const float a2 = rows[(int64_t)(i + 2 * G) * d + j], a3 = rows[(int64_t)(i + 3 * G) * d + j];
                acc += a0; acc += a1; acc += a2; acc += a3;
            }
            for (; i < end; i += G) acc += rows[(int64_t)i * d + j];
        }
        part[grp][sl] = acc;
        __syncthreads();
        if (grp == 0 && j < d) {
            float tot = part[0][sl];
            for (int w = 1; w < G; ++w) tot += part[w][sl];
            dst[j] = tot;
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(64) void k_dm_long_final(int32_t* __restrict__ long_seg, int d, const float* __restrict__ partial,
                                                      float* __restrict__ out, int64_t ldo)
{
    const int c = blockIdx.x;
    const int s = long_seg[c] - 1;
    if (s < 0) return;
    const float* src = partial + (int64_t)c * LONG_PARTS * d;
    for (int j = threadIdx.x; j < d; j += 64) {
        float tot = src[j];
        for (int p = 1; p < LONG_PARTS; ++p) tot += src[(int64_t)p * d + j];
        out[(int64_t)s * ldo + j] = tot;
    }
    __syncthreads();                              // every lane has read the entry before it is reset for the next call
    if (threadIdx.x == 0) long_seg[c] = 0;
}

int launch_segment_sums(const float* rows, const int32_t* ptr, int nseg, int total_rows, int d, float* partial,
                        int32_t* long_seg, float* out, int64_t ldo, hipStream_t st)
{
    hipLaunchKernelGGL(k_dm_segment_sum, dim3((int)(((int64_t)nseg * 32 + TPB_ - 1) / TPB_)), dim3(TPB_), 0, st, rows, ptr, nseg, d,
                       out, ldo, long_seg);
    DN_LAUNCH_CHECK("k_dm_segment_sum");
    const int cand = (total_rows + LONG_SEG - 1) / LONG_SEG;
    if (cand > 0) {
        hipLaunchKernelGGL(k_dm_long_partial, dim3(cand, LONG_PARTS), dim3(TPB_), 0, st, rows, ptr, long_seg, d, partial);
        DN_LAUNCH_CHECK("k_dm_long_partial");
        hipLaunchKernelGGL(k_dm_long_final, dim3(cand), dim3(64), 0, st, long_seg, d, partial, out, ldo);
        DN_LAUNCH_CHECK("k_dm_long_final");
    }
    return DN_OK;
}

int fill_decoder(dn_decoder* d, int64_t max_edges, int32_t chunk, int32_t num_neg, int32_t dim, int64_t max_rows,
                 int64_t num_rel)
{
    if (max_edges < 1 || max_edges > (1 << 24)) return dn_fail(DN_EINVAL, "max_edges must be in [1, 2^24]");
    if (chunk < 1 || chunk > (1 << 16)) return dn_fail(DN_EINVAL, "chunk must be in [1, 65536]");
    if (num_neg < 1 || num_neg > (1 << 16)) return dn_fail(DN_EINVAL, "num_neg must be in [1, 65536]");
    if (dim < 1 || dim > 1024) return dn_fail(DN_EINVAL, "dim must be in [1, 1024]");
    if (max_rows < 1 || max_rows > (1 << 28)) return dn_fail(DN_EINVAL, "max_rows must be in [1, 2^28]");
    if (num_rel < 1 || num_rel > (1 << 28)) return dn_fail(DN_EINVAL, "num_rel must be in [1, 2^28]");
    std::memset(d, 0, sizeof(*d));
    d->max_edges = max_edges; d->chunk = chunk; d->num_neg = num_neg; d->dim = dim;
    d->max_rows = max_rows; d->num_rel = num_rel;
    d->kp = (int32_t)dn_round_up(dim, 64);
    d->np = (int32_t)dn_round_up(dim, 128);
    d->cpad = (int32_t)dn_round_up(chunk, 128);
    d->npad = (int32_t)dn_round_up(num_neg, 128);
    d->max_chunks = (max_edges + chunk - 1) / chunk;
    d->max_entries = 2 * max_edges + d->max_chunks * num_neg;
    if (d->max_entries > (1ll << 30)) return dn_fail(DN_EINVAL, "more than 2^30 gradient entries (2 * max_edges + chunks * num_neg)");
    if (2 * d->max_chunks > 65535) return dn_fail(DN_EINVAL, "more than 32767 chunks");
    d->nplan = dn_sort_make_plan(max_rows + 1, d->max_entries);
    d->rplan = dn_sort_make_plan(num_rel + 1, max_edges);
    return DN_OK;
}

void carve_decoder(dn_decoder* d, dn_carver& c)
{
    const int64_t C = d->max_chunks;
    d->hdr = c.take<int32_t>(DM_HDR_WORDS);
    d->nhist = c.take<int32_t>(dn_sort_hist_words(d->nplan));
    d->rhist = c.take<int32_t>(dn_sort_hist_words(d->rplan));
    d->long_seg = c.take<int32_t>(d->max_entries / LONG_SEG + 2);
    d->Q = c.take<dn_bf16>(2 * C * d->cpad * d->kp);
    d->En = c.take<dn_bf16>(C * d->npad * d->kp);
    d->Ent = c.take<dn_bf16>(C * (int64_t)d->np * d->npad);
    d->S = c.take<float>(2 * C * (int64_t)d->cpad * d->npad);
    d->pmax = c.take<float>(2 * C * (int64_t)d->cpad * (d->npad / BN));
    d->psum = c.take<float>(2 * C * (int64_t)d->cpad * (d->npad / BN));
    d->lse = c.take<float>(2 * d->max_edges);
    d->dpos = c.take<float>(d->max_edges);
    d->P = c.take<dn_bf16>(2 * C * (int64_t)d->cpad * 2 * d->npad);
    d->dQ = c.take<float>(2 * C * (int64_t)d->cpad * d->np);
    d->dEn = c.take<float>(2 * C * (int64_t)2 * d->npad * d->np);
    d->rows = c.take<float>(d->max_entries * d->dim);
    d->long_partial = c.take<float>((d->max_entries / LONG_SEG + 2) * LONG_PARTS * d->dim);
    for (int i = 0; i < 2; ++i) {
        d->nkey[i] = c.take<int32_t>(d->max_entries);
        d->nval[i] = c.take<int32_t>(d->max_entries);
        d->rkey[i] = c.take<int32_t>(d->max_edges);
        d->rval[i] = c.take<int32_t>(d->max_edges);
    }
    d->nptr = c.take<int32_t>(d->max_rows + 2);
    d->rptr = c.take<int32_t>(d->num_rel + 2);
}

int launch_gemm(const DmGemm& g, bool wrap, int epi, int mtiles, int ntiles, int batch, hipStream_t st, const char* tag)
{
    dn_prof_scope ps(tag, 0, st);
    const dim3 grid(ntiles, mtiles, batch);
    if (wrap) hipLaunchKernelGGL((k_dm_gemm<true, DM_EPI_STORE>), grid, dim3(TPB), 0, st, g);
    else if (epi == DM_EPI_LSE) hipLaunchKernelGGL((k_dm_gemm<false, DM_EPI_LSE>), grid, dim3(TPB), 0, st, g);
    else if (epi == DM_EPI_PROBS) hipLaunchKernelGGL((k_dm_gemm<false, DM_EPI_PROBS>), grid, dim3(TPB), 0, st, g);
    else hipLaunchKernelGGL((k_dm_gemm<false, DM_EPI_STORE>), grid, dim3(TPB), 0, st, g);
    DN_LAUNCH_CHECK(tag);
    return DN_OK;
}

// the score contraction S[z] = Q[z] * E[q]^T of the last forward's operands (they stay until the next forward)
DmGemm score_gemm(const dn_decoder* d)
{
    DmGemm g{};
    const int C = (int)d->n_chunks;
    g.A = d->Q; g.lda = d->kp; g.stride_a = (int64_t)d->cpad * d->kp;
    g.B = d->En; g.ldb = d->kp; g.stride_b = (int64_t)d->npad * d->kp; g.b_mod = C;
    g.kchunks = d->kp / BK; g.b_wrap_chunks = 1;
    g.C = d->S; g.ldc = d->npad; g.stride_c = (int64_t)d->cpad * d->npad; g.ncols = d->npad;
    g.pmax = d->pmax; g.psum = d->psum; g.lse_cols = d->num_neg;
    g.lse = d->lse; g.n_edges = (int)d->n_edges; g.n_chunks = C; g.chunk = d->chunk; g.n_neg = d->num_neg; g.npad = d->npad;
    g.P = d->P;
    return g;
}

int blocks_for(int64_t items, int per_block) { return (int)((items + per_block - 1) / per_block); }

}  // namespace

extern "C" {

int dn_decoder_workspace_size(int64_t max_edges, int32_t chunk, int32_t num_neg, int32_t dim, int64_t max_rows,
                              int64_t num_rel, size_t* bytes)
{
    if (!bytes) return dn_fail(DN_EINVAL, "bytes is null");
    dn_decoder tmp;
    const int rc = fill_decoder(&tmp, max_edges, chunk, num_neg, dim, max_rows, num_rel);
    if (rc) return rc;
    dn_carver c(nullptr);
    carve_decoder(&tmp, c);
    *bytes = c.bytes();
    return DN_OK;
}

int dn_decoder_create(dn_decoder** out, int64_t max_edges, int32_t chunk, int32_t num_neg, int32_t dim, int64_t max_rows,
                      int64_t num_rel, void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!out) return dn_fail(DN_EINVAL, "out is null");
    if (!d_workspace || ((uintptr_t)d_workspace & 255)) return dn_fail(DN_EINVAL, "workspace must be non-null and 256-byte aligned");
    dn_decoder* d = new (std::nothrow) dn_decoder;
    if (!d) return dn_fail(DN_EINVAL, "out of host memory");
    const int rc = fill_decoder(d, max_edges, chunk, num_neg, dim, max_rows, num_rel);
    if (rc) { delete d; return rc; }
    dn_carver c(d_workspace);
    carve_decoder(d, c);
    if (c.bytes() > workspace_bytes) {
        delete d;
        return dn_fail(DN_ECAPACITY, "workspace has %zu bytes, %zu needed", workspace_bytes, c.bytes());
    }
    d->workspace_bytes = c.bytes();
    // header and sort histograms must start at zero (the sort leaves its histograms zero again); the operand
    // buffers are cleared too so that tile rows no kernel writes hold finite values
    hipError_t e = hipMemsetAsync(d_workspace, 0, c.bytes(), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) { delete d; return dn_fail(DN_EHIP, "hipMemsetAsync: %s", hipGetErrorString(e)); }
    *out = d;
    return DN_OK;
}

void dn_decoder_destroy(dn_decoder* d) { delete d; }

int distmult_forward(dn_decoder* d, const float* d_H, int64_t ldh, int64_t n_rows, const float* d_R, int64_t ldr,
                     const int32_t* d_src, const int32_t* d_rel, const int32_t* d_dst, int64_t n_edges,
                     const int32_t* d_neg, float* d_pos, float* d_loss, void* stream)
{
    if (!d || !d_H || !d_R) return dn_fail(DN_EINVAL, "null argument");
    if (n_edges > 0 && (!d_src || !d_rel || !d_dst || !d_neg || !d_pos || !d_loss))
        return dn_fail(DN_EINVAL, "null argument");
    if (n_edges < 0 || n_edges > d->max_edges) return dn_fail(DN_ECAPACITY, "n_edges %lld exceeds the decoder's %lld",
                                                             (long long)n_edges, (long long)d->max_edges);
    if (n_rows < 1 || n_rows > d->max_rows) return dn_fail(DN_ECAPACITY, "n_rows %lld outside [1, %lld]",
                                                           (long long)n_rows, (long long)d->max_rows);
    if (ldh < d->dim || ldr < d->dim) return dn_fail(DN_EINVAL, "row stride below dim");
    hipStream_t st = static_cast<hipStream_t>(stream);
    d->H = d_H; d->R = d_R; d->ldh = ldh; d->ldr = ldr; d->n_rows = n_rows; d->n_edges = n_edges;
    d->src = d_src; d->rel = d_rel; d->dst = d_dst; d->neg = d_neg;
    d->n_chunks = (n_edges + d->chunk - 1) / d->chunk;
    d->have_forward = 1;
    if (n_edges == 0) return DN_OK;
    const int B = (int)n_edges, C = (int)d->n_chunks;
    {
        dn_prof_scope ps("dm_prepare", 0, st);
        const int64_t rows = 2ll * C * d->cpad + (int64_t)C * d->npad;
        hipLaunchKernelGGL(k_dm_prepare, dim3(blocks_for(rows * 16, TPB_)), dim3(TPB_), 0, st, d_H, ldh, (int)n_rows, d_R, ldr,
                           (int)d->num_rel, d_src, d_rel, d_dst, d_neg, B, C, d->chunk, d->num_neg, d->dim, d->kp, d->cpad,
                           d->npad, d->Q, d->En, d_pos, d->hdr);
        DN_LAUNCH_CHECK("k_dm_prepare");
    }
    int rc = launch_gemm(score_gemm(d), false, DM_EPI_LSE, d->cpad / BM, d->npad / BN, 2 * C, st, "dm_gemm_scores");
    if (rc) return rc;
    {
        dn_prof_scope ps("dm_lse", 0, st);
        hipLaunchKernelGGL(k_dm_lse, dim3(blocks_for(B, TPB_)), dim3(TPB_), 0, st, d->pmax, d->psum, d_pos, B, C, d->chunk,
                           d->cpad, d->npad / BN, d->lse, d_loss, d->dpos, d->hdr);
        DN_LAUNCH_CHECK("k_dm_lse");
    }
    return DN_OK;
}

int distmult_backward(dn_decoder* d, float* d_dH, int64_t ld_dh, float* d_dR, int64_t ld_dr, void* stream)
{
    if (!d || !d_dH || !d_dR) return dn_fail(DN_EINVAL, "null argument");
    if (!d->have_forward) return dn_fail(DN_ESTATE, "distmult_backward needs a distmult_forward first");
    if (ld_dh < d->dim || ld_dr < d->dim) return dn_fail(DN_EINVAL, "row stride below dim");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = (int)d->n_edges, C = (int)d->n_chunks, n_rows = (int)d->n_rows;
    const int n_neg = C * d->num_neg, total = 2 * B + n_neg;
    if (B > 0) {
        // the scores again, this time turned into probabilities with the rows' log-sum-exp
        int rc = launch_gemm(score_gemm(d), false, DM_EPI_PROBS, d->cpad / BM, d->npad / BN, 2 * C, st, "dm_probs");
        if (rc) return rc;
        {
            dn_prof_scope ps("dm_transpose", 0, st);
            hipLaunchKernelGGL(k_dm_transpose, dim3(d->kp / 64, d->npad / 64, C), dim3(TPB_), 0, st, d->En, d->npad, d->kp,
                               d->Ent, (int64_t)d->np * d->npad);
            DN_LAUNCH_CHECK("k_dm_transpose(E)");
        }
        DmGemm g{};
        g.pmax = nullptr; g.psum = nullptr; g.lse_cols = 0;
        // dQ[z] = P[z] (two terms along the reduction) * E[q] : B operand = E^T [np x npad], repeated per term
        g.A = d->P; g.lda = 2 * d->npad; g.stride_a = (int64_t)d->cpad * 2 * d->npad;
        g.B = d->Ent; g.ldb = d->npad; g.stride_b = (int64_t)d->np * d->npad; g.b_mod = C;
        g.kchunks = 2 * d->npad / BK; g.b_wrap_chunks = d->npad / BK;
        g.C = d->dQ; g.ldc = d->np; g.stride_c = (int64_t)d->cpad * d->np; g.ncols = d->dim;
        rc = launch_gemm(g, true, DM_EPI_STORE, d->cpad / BM, d->np / BN, 2 * C, st, "dm_gemm_dq");
        if (rc) return rc;
        // dE[z] = P[z]^T * Q[z], both operands read with the edge index as the reduction index
        {
            DmGemmTn t;
            t.A = d->P; t.lda = 2 * d->npad; t.stride_a = (int64_t)d->cpad * 2 * d->npad; t.a_cols = 2 * d->npad;
            t.B = d->Q; t.ldb = d->kp; t.stride_b = (int64_t)d->cpad * d->kp; t.b_cols = d->kp;
            t.k_rows = d->cpad;
            t.C = d->dEn; t.ldc = d->np; t.stride_c = (int64_t)2 * d->npad * d->np; t.ncols = d->dim;
            dn_prof_scope ps("dm_gemm_de", 0, st);
            hipLaunchKernelGGL(k_dm_gemm_tn, dim3(d->np / BN, 2 * d->npad / BM, 2 * C), dim3(TPB), 0, st, t);
            DN_LAUNCH_CHECK("k_dm_gemm_tn");
        }
    }
    DmGrad a;
    a.H = d->H; a.R = d->R; a.ldh = d->ldh; a.ldr = d->ldr; a.n_rows = n_rows; a.num_rel = (int)d->num_rel;
    a.src = d->src; a.rel = d->rel; a.dst = d->dst; a.dpos = d->dpos; a.dQ = d->dQ; a.dEn = d->dEn;
    a.B = B; a.C = C; a.chunk = d->chunk; a.Nn = d->num_neg; a.d = d->dim; a.np = d->np; a.cpad = d->cpad; a.npad = d->npad;
    // ---- dH: entries sorted by node, gradient rows in that order, segment sums
    {
        dn_prof_scope ps("dm_node_index", 0, st);
        int gb = blocks_for(total, TPB_);
        if (gb > 2048) gb = 2048;
        if (gb < 1) gb = 1;
        const int srcbuf = d->nplan.passes & 1;
        hipLaunchKernelGGL(k_dm_node_index_init, dim3(gb), dim3(TPB_), 0, st, d->src, d->dst, d->neg, B, n_neg, n_rows,
                           d->nkey[srcbuf], d->nval[srcbuf], d->nplan.bits,
                           dn_sort_counts_separately(d->nplan) ? nullptr : d->nhist, d->hdr);
        DN_LAUNCH_CHECK("k_dm_node_index_init");
        const int rc = dn_sort_pairs_run(d->nplan, d->hdr + DM_HDR_NODE_COUNT, d->nkey, d->nval, d->nhist, nullptr, n_rows,
                                         d->nptr, st);
        if (rc) return rc;
    }
    {
        dn_prof_scope ps("dm_dh", 0, st);
        if (total > 0) {
            hipLaunchKernelGGL(k_dm_node_rows, dim3(blocks_for((int64_t)total * 32, TPB_)), dim3(TPB_), 0, st, a, d->nval[0], total,
                               d->rows);
            DN_LAUNCH_CHECK("k_dm_node_rows");
        }
        const int rc = launch_segment_sums(d->rows, d->nptr, n_rows, total, d->dim, d->long_partial, d->long_seg, d_dH, ld_dh, st);
        if (rc) return rc;
    }
    // ---- dR: edges sorted by relation
    {
        dn_prof_scope ps("dm_rel_index", 0, st);
        int gb = blocks_for(B, TPB_);
        if (gb > 2048) gb = 2048;
        if (gb < 1) gb = 1;
        const int srcbuf = d->rplan.passes & 1;
        hipLaunchKernelGGL(k_dm_rel_index_init, dim3(gb), dim3(TPB_), 0, st, d->rel, B, (int)d->num_rel, d->rkey[srcbuf],
                           d->rval[srcbuf], d->rplan.bits, dn_sort_counts_separately(d->rplan) ? nullptr : d->rhist,
                           d->hdr);
        DN_LAUNCH_CHECK("k_dm_rel_index_init");
        const int rc = dn_sort_pairs_run(d->rplan, d->hdr + DM_HDR_REL_COUNT, d->rkey, d->rval, d->rhist, nullptr, d->num_rel,
                                         d->rptr, st);
        if (rc) return rc;
    }
    {
        dn_prof_scope ps("dm_dr", 0, st);
        const int nr = (int)d->num_rel;
        if (B > 0) {
            hipLaunchKernelGGL(k_dm_rel_rows, dim3(blocks_for((int64_t)B * 32, TPB_)), dim3(TPB_), 0, st, a, d->rval[0], d->rows);
            DN_LAUNCH_CHECK("k_dm_rel_rows");
        }
        const int rc = launch_segment_sums(d->rows, d->rptr, nr, B, d->dim, d->long_partial, d->long_seg, d_dR, ld_dr, st);
        if (rc) return rc;
    }
    return DN_OK;
}

int dn_decoder_scores(const dn_decoder* d, int32_t side, const float** d_scores, int64_t* chunk_stride, int64_t* row_stride,
                      void* stream)
{
    if (!d || !d_scores || !chunk_stride || !row_stride) return dn_fail(DN_EINVAL, "null argument");
    if (side < 0 || side > 1) return dn_fail(DN_EINVAL, "side must be 0 or 1");
    if (!d->have_forward) return dn_fail(DN_ESTATE, "no distmult_forward yet");
    if (d->n_edges > 0) {
        // the forward pass keeps only the rows' log-sum-exp: the scores of both sides are computed here, on request
        const int rc = launch_gemm(score_gemm(d), false, DM_EPI_STORE, d->cpad / BM, d->npad / BN, 2 * (int)d->n_chunks,
                                   static_cast<hipStream_t>(stream), "dm_scores_on_request");
        if (rc) return rc;
    }
    *d_scores = d->S + (int64_t)side * d->n_chunks * d->cpad * d->npad;
    *chunk_stride = (int64_t)d->cpad * d->npad;
    *row_stride = d->npad;
    return DN_OK;
}

int dn_decoder_status(const dn_decoder* d, int32_t* flags, void* stream)
{
    if (!d || !flags) return dn_fail(DN_EINVAL, "null argument");
    hipStream_t st = static_cast<hipStream_t>(stream);
    DN_HIP(hipMemcpyAsync(flags, d->hdr + DM_HDR_STATUS, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    DN_HIP(hipStreamSynchronize(st));
    return DN_OK;
}

}  // extern "C"
