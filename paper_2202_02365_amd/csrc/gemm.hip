// bf16 MFMA GEMMs of the GraphSage linear layers (the one dense contraction of the path).
//
//   forward : C = A * B^T   A = X^i = [bf16(H_self) | bf16(mean)]   B = Wcat^T     epilogue + bias, ReLU
//   dX      : C = A * B^T   A = bf16 terms of dZ                     B = Wcat       plain store
//     both operands row-major with the reduction index contiguous (mainloop of mfma_tile.h), 64 x 64 tiles:
//     a layer has few output rows per mini-batch and a short reduction, so many small workgroups, several per
//     compute unit, hide the memory latency of the few k-steps better than 128 x 128 tiles do;
//   dW      : C = A^T * B   A = X^i, B = bf16 terms of dZ: the reduction runs over the nodes, the ROW index of both
//     operands as they lie in memory, which mainloop_tn reads in place through the LDS transpose read; 128 x 128
//     tiles, split over the reduction, partial tiles reduced afterwards in a fixed order (deterministic).  The
//     128 x 128 tile loads its operand tiles from global memory straight into LDS (mainloop_tn_direct).
// Four waves (2 x 2) per workgroup, v_mfma_f32_32x32x16_bf16, two register stages of global prefetch and two LDS
// buffers (dW: two LDS buffers filled directly).  M and the dW reduction length live in device memory (they depend
// on the sample); grids are sized by capacity and surplus workgroups leave at once.
//
// Operand terms: an operand the device computed through an MFMA accumulation is carried as two
// bf16 terms (hi + lo), laid side by side along the reduction index, with the other operand
// repeated; an operand that derives from the caller's inputs is one term.
//
// ReLU sign: where |Z| is below a probabilistic bound on the fp32 accumulation error (8 sqrt(K) 2^-24 |x| |w|), the
// epilogue queues the element in LDS and the workgroup then recomputes that dot product in fp64,
// so that the stored activation and the mask [Z > 0] used by the backward pass are those of the
// exact sum.
#include "dn_internal.h"
#include "mfma_tile.h"
#include <algorithm>
#include <cstdlib>

namespace {

using namespace dn_mma;

// sign fix-ups one workgroup can queue: one sixteenth of its outputs
enum { EPI_BIAS_ACT = 0, EPI_PLAIN = 1, EPI_SPLIT = 2 };
// Weight gradient with two bf16 terms of dZ: 0 = each term is a reduction split of its own (twice the workgroups, X is
// read once per term), 1 = one workgroup reduces both terms (X read once, half the partial tiles, but LDS for two
// terms leaves room for one workgroup per compute unit).  Measured at the 111M-node workload: 25 us and 131 MB through
// HBM against 36 us and 66 MB; with four mini-batches in flight both give the same step rate.  0 is built.
#ifndef DN_DW_FUSE_TERMS
#define DN_DW_FUSE_TERMS 0
#endif
constexpr bool DW_FUSE = DN_DW_FUSE_TERMS != 0;
// The 128 x 128 weight-gradient tile takes its operand tiles from global memory straight into LDS
// (mainloop_tn_direct) with this many LDS buffers of DN_TN_DIRECT_ROWS reduction rows; 0: through registers
// (mainloop_tn).  Measured per launch at the 111M- / 122M-node workloads, through registers 24.7 / 75.0 us:
// 2 x 64 rows 21.8 / 63.0 (two workgroups per compute unit), 3 x 64 29.4 / 73.4 and 4 x 64 30.7 / 75.6 (one
// workgroup per compute unit), 4 x 32 rows 23.8 / 67.6, 3 x 32 rows 26.1 / 64.7.
#ifndef DN_TN_DIRECT_BUFFERS
#define DN_TN_DIRECT_BUFFERS 2
#endif
#ifndef DN_TN_DIRECT_ROWS
#define DN_TN_DIRECT_ROWS 64
#endif
// The forward GEMM of a layer with a long reduction (NT_DIRECT_MIN_K columns of X or more) runs on 128 x 128 tiles
// whose operand tiles go from global memory straight into LDS (mainloop_direct), NT_DIRECT_BUFFERS LDS buffers.
#ifndef DN_NT_DIRECT_BUFFERS
#define DN_NT_DIRECT_BUFFERS 2
#endif
constexpr int NT_DIRECT_BUFFERS = DN_NT_DIRECT_BUFFERS;
constexpr int NT_DIRECT_MIN_K = 1024;
#ifndef DN_NT_STAGES
#define DN_NT_STAGES 2
#endif
#ifndef DN_TN_STAGES
#define DN_TN_STAGES 2
#endif
// register stages of global prefetch (see mainloop).  More than two were measured slower: four stages on the 64 x 64
// forward tiles (two workgroups per compute unit instead of four) 22.5 against 16.5 us at the 111M-node workload and
// 59.5 against 46.9 at the 122M-node one; three stages on the weight gradient 26.3 against 24.8 and 79.7 against 77.6.
constexpr int NT_STAGES = DN_NT_STAGES, TN_STAGES = DN_TN_STAGES;


struct GemmArgs {
    const uint16_t* A; int64_t lda;
    const uint16_t* B; int64_t ldb;
    float* C; int64_t ldc;
    const int32_t* hdr;
    int layer;          // rows of this layer's output = hdr[N] - hdr[NODE_OFF + layer]
    int m_const;        // >= 0: M is this constant; < 0: M = rows of `layer`
    int ncols;          // valid output columns
    int red_const;      // >= 0: reduction length (multiple of 64); < 0: rows of `layer`, rounded up to 64
    const float* bias;
    int relu;
    int64_t split_stride;   // floats between consecutive split partials
    int terms;              // dW: bf16 terms (hi, lo) of B, both reduced by every workgroup
    int64_t b_term_stride;  // dW: elements between B's terms
    int a_cols, b_cols;     // dW: allocated columns of A, of one term of B (loads beyond them read zero)
    int min_chunks;         // dW: see effective_splits
    float* db_partial;      // dW: [splits x ncols] column sums of this split's rows of B, all terms (the bias gradient's partials)
    // ReLU sign fix-up (EPI_BIAS_ACT with relu)
    const float* rownorm; const float* colnorm; float gamma;
    int* fix_count;         // counters of exact recomputations (see dn_model), [1] sticky overflow flag
};

// fewest k-steps (of 64 rows) a split of the weight-gradient reduction is given
__device__ __forceinline__ int effective_splits(int groups, int chunks, int min_chunks)
{
    const int want = chunks / min_chunks;
    return want < 1 ? 1 : (want < groups ? want : groups);
}

// One BM_ x BN_ output tile (one reduction split for EPI_SPLIT): block coordinates (bx, by, bz of nz).
template <int EPI, int BM_, int BN_, bool DIRECT = false>
__device__ __forceinline__ void gemm_tile(const GemmArgs& a, const int bx, const int by, const int bz, const int nz)
{
    constexpr int MI = BM_ / 64, NJ = BN_ / 64;
    constexpr int LOCAL_FIX_CAP = BM_ * BN_ / 16;
    const int rows_layer = a.hdr[HDR_N] - a.hdr[HDR_NODE_OFF + a.layer];
    const int M = a.m_const >= 0 ? a.m_const : rows_layer;
    const int red = a.red_const >= 0 ? a.red_const : ((rows_layer + BK - 1) / BK) * BK;
    const int row0 = by * BM_, col0 = bx * BN_;
    if (row0 >= M || col0 >= a.ncols) return;

    // reduction range of this split (dW: the splits of every term cover the whole range)
    const int chunks = red / BK;
    const int groups = (EPI == EPI_SPLIT) ? (DW_FUSE ? nz : nz / a.terms) : 1;
    const int term = (EPI == EPI_SPLIT && !DW_FUSE) ? bz / groups : 0;
    const int grp = (EPI == EPI_SPLIT) ? bz % groups : 0;
    // dW: the grid has `groups` splits by capacity; only as many are used as leave at least min_chunks k-steps
    // per split for the rows that exist (the others leave at once and the reduction skips them)
    const int eff_groups = (EPI == EPI_SPLIT) ? effective_splits(groups, chunks, a.min_chunks) : 1;
    if (grp >= eff_groups) return;
    const int per = (chunks + eff_groups - 1) / eff_groups;
    const int kc_begin = grp * per;
    const int kc_end = min(chunks, kc_begin + per);
    const uint16_t* Bbase = a.B + (int64_t)term * a.b_term_stride;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // what the epilogue needs from memory (bias, column norms, row norms) is requested before the main loop, so that
    // its latency passes under the k-steps instead of after them
    float pre_bias[NJ], pre_cn[NJ], pre_rn = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) { pre_bias[j] = 0.f; pre_cn[j] = 0.f; }
    if constexpr (EPI == EPI_BIAS_ACT) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int n = min(col0 + wn * (BN_ / 2) + j * 32 + (lane & 31), a.ncols - 1);
            pre_bias[j] = a.bias[n];
            if (a.relu) pre_cn[j] = a.colnorm[n];
        }
        if (a.relu && t < BM_) pre_rn = a.rownorm[min(row0 + t, M - 1)];
    }

    f32x16 acc[MI][NJ];
    if constexpr (EPI == EPI_SPLIT) {
        // weight gradient: both operands have the reduction index (the node) as their row index.  The first row
        // tile's upper waves also multiply a row of ones with their fragments of dZ: the column sums of this
        // split's rows of dZ, which are its share of the bias gradient.
        f32x16 ones_acc[NJ];
        const bool do_ones = by == 0 && wm == 0 && a.db_partial != nullptr;
        if constexpr (BM_ == 128 && BN_ == 128 && !DW_FUSE && DN_TN_DIRECT_BUFFERS > 0)
            mainloop_tn_direct<true, DN_TN_DIRECT_BUFFERS, DN_TN_DIRECT_ROWS>(a.A, a.lda, a.a_cols, Bbase, a.ldb, a.b_cols, row0, col0, kc_begin, kc_end,
                                                           rows_layer, acc, ones_acc, do_ones);
        else
        mainloop_tn<BM_, BN_, true, DW_FUSE, TN_STAGES>(a.A, a.lda, a.a_cols, Bbase, a.ldb, a.b_cols, DW_FUSE ? a.terms : 1, a.b_term_stride,
                                             row0, col0, kc_begin, kc_end, rows_layer, acc, ones_acc, do_ones);
        if (do_ones && lane < 32) {                           // register 0 of lanes 0..31: row 0 of the 32 x 32 tile
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int n = col0 + wn * (BN_ / 2) + j * 32 + lane;
                if (n < a.ncols) a.db_partial[(int64_t)bz * a.ncols + n] = ones_acc[j][0];
            }
        }
    } else if constexpr (DIRECT)
        mainloop_direct<BM_, BN_, NT_DIRECT_BUFFERS>(a.A + (int64_t)row0 * a.lda, a.lda, Bbase + (int64_t)col0 * a.ldb, a.ldb, kc_begin, kc_end, acc);
    else
        mainloop<BM_, BN_, false, NT_STAGES>(a.A + (int64_t)row0 * a.lda, a.lda, Bbase + (int64_t)col0 * a.ldb, a.ldb, kc_begin, kc_end, 0, acc);

    // epilogue: lane holds column (lane & 31); register e holds row 8*(e/4) + 4*(lane/32) + e%4
    float* C = a.C;
    if (EPI == EPI_SPLIT) C += (int64_t)bz * a.split_stride;
    __shared__ int s_fix_n;
    __shared__ long long local_fix[LOCAL_FIX_CAP];
    __shared__ float s_rownorm[BM_];
    if (EPI == EPI_BIAS_ACT && a.relu) {
        if (t == 0) s_fix_n = 0;
        if (t < BM_) s_rownorm[t] = row0 + t < M ? pre_rn : 0.f;
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int n = col0 + wn * (BN_ / 2) + j * 32 + (lane & 31);
            if (n >= a.ncols) continue;
            const float bv = pre_bias[j];
            const float cn = a.gamma * pre_cn[j];                  // both zero unless EPI_BIAS_ACT (with ReLU)
            const float bt = fabsf(bv) * 4.76837158e-7f;          // 2^-21 |b|: rounding of the bias add
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = row0 + wm * (BM_ / 2) + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (m < M) {
                    float v = acc[i][j][e];
                    if (EPI == EPI_BIAS_ACT) {
                        v += bv;
                        if (a.relu) {
                            if (fabsf(v) <= cn * s_rownorm[m - row0] + bt) {
                                // the fp32 sum cannot settle this sign: queue the element for the exact pass below
                                const int lp = atomicAdd(&s_fix_n, 1);
                                if (lp < LOCAL_FIX_CAP) local_fix[lp] = ((long long)m << 16) | (long long)n;
                            }
                            v = fmaxf(v, 0.f);
                        }
                    }
                    C[(int64_t)m * a.ldc + n] = v;
                }
            }
        }
    if (EPI == EPI_BIAS_ACT && a.relu) {
        // Exact pass: 16 lanes per queued element recompute Z = sum_k A[m][k] B[n][k] + b[n] in fp64
        // (bf16 products are exact in fp64, the sum is good to 2^-53 of the magnitudes) and stores
        // fp32(max(Z, 0)), so that the activation and the mask [Z > 0] of the backward pass are
        // those of the exact sum.
        __syncthreads();
        const int queued = s_fix_n;
        const int n_local = min(queued, LOCAL_FIX_CAP);
        if (t == 0 && queued > 0) {
            atomicAdd(&a.fix_count[DN_FIX_FIRST + DN_FIX_STRIDE * ((bx + 7 * by) % DN_FIX_SLOTS)], n_local);
            if (queued > LOCAL_FIX_CAP) a.fix_count[1] = 1;       // surplus keeps its fp32 sign
        }
        // 16 lanes per queued element, 16 elements in flight per workgroup
        const int sub = t >> 4, sl = t & 15;
        for (int q = sub; q < n_local; q += TPB / 16) {
            const long long ent = local_fix[q];
            const int m = (int)(ent >> 16), n = (int)(ent & 0xffff);
            const uint16_t* xr = a.A + (int64_t)m * a.lda;
            const uint16_t* wr = Bbase + (int64_t)n * a.ldb;
            double sum = 0.0;
            for (int c = sl; c < red / 8; c += 16) {
                const u32x4 xv = *reinterpret_cast<const u32x4*>(xr + c * 8);
                const u32x4 wv = *reinterpret_cast<const u32x4*>(wr + c * 8);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sum += (double)__uint_as_float(xv[e] << 16) * (double)__uint_as_float(wv[e] << 16);
                    sum += (double)__uint_as_float(xv[e] & 0xffff0000u) * (double)__uint_as_float(wv[e] & 0xffff0000u);
                }
            }
            for (int d = 8; d > 0; d >>= 1) sum += __shfl_down(sum, d, 16);
            if (sl == 0) {
                const double z = sum + (double)a.bias[n];
                C[(int64_t)m * a.ldc + n] = (float)(z > 0.0 ? z : 0.0);
            }
        }
    }
}

// LAYER_TAG only gives every layer's launch its own kernel symbol, so that a profiler's per-kernel
// statistics do not mix the layers (tag 4 stands for "layer 4 and above").
// Workgroups are handed to the 8 XCDs (each with an L2 of its own) round-robin in launch order.  The column
// tiles of one row tile read the same rows of A: the launch order is therefore re-read as chunks of 8 x (column
// tiles), in which the workgroups j, j + 8, j + 16, ... (same XCD) are the column tiles of one row tile.
// gridDim.y is a multiple of 8 and at most GEMM_MAX_ROW_BLOCKS: a workgroup takes the row tiles by, by + gridDim.y, ...
// (the capacity of rows is several times what a mini-batch fills, and a grid sized by it consists mostly of workgroups
// that find no rows and leave: at 1 us each they delayed the end of a 15 us kernel by a third).
constexpr int GEMM_MAX_ROW_BLOCKS = 512;
template <int EPI, int LAYER_TAG, int BM_, int BN_, bool DIRECT = false>
__global__ __launch_bounds__(TPB, (BM_ == 64 && BN_ == 64) ? 4 : 2) void k_gemm_nt(GemmArgs a)
{
    const int nx = gridDim.x;
    const int id = blockIdx.x + nx * blockIdx.y;
    const int chunk = id / (8 * nx), j = id - chunk * 8 * nx;
    const int M = a.m_const >= 0 ? a.m_const : a.hdr[HDR_N] - a.hdr[HDR_NODE_OFF + a.layer];
    for (int by = chunk * 8 + (j & 7); by * BM_ < M; by += gridDim.y) {
        gemm_tile<EPI, BM_, BN_, DIRECT>(a, j >> 3, by, blockIdx.z, gridDim.z);
        __syncthreads();                  // the tile's LDS buffers are free for the next one
    }
}

// The dW GEMMs of all layers in one launch: a 1-D grid, each layer owns the workgroups
// [begin[i], begin[i+1]) = column tiles x row tiles x reduction splits of its own problem.
struct GemmGroup {
    GemmArgs g[DN_MAX_LAYERS];
    int begin[DN_MAX_LAYERS + 1];
    int gx[DN_MAX_LAYERS], gy[DN_MAX_LAYERS], gz[DN_MAX_LAYERS];
    int n, place;
};
template <int BM_, int BN_>
__global__ __launch_bounds__(TPB, 2) void k_gemm_dw_group(GemmGroup G)
{
    int gi = 0;
    while (gi + 1 < G.n && (int)blockIdx.x >= G.begin[gi + 1]) ++gi;
    // Workgroups go to the 8 XCDs round-robin in launch order.  place 0: the column tiles of one (row tile, split)
    // read the same rows of X: launch order is re-read as chunks of 8 x (column tiles), in which the workgroups
    // j, j + 8, ... (same XCD, shared L2) are those column tiles.  place 1: all tiles of one split share an XCD.
    const int local = (int)blockIdx.x - G.begin[gi];
    const int nx = G.gx[gi];
    int bx, by, bz;
    if (G.place == 0) {
        const int chunk = local / (8 * nx), j = local - chunk * 8 * nx;
        const int r = chunk * 8 + (j & 7);                       // r = bz * gy + by
        bx = j >> 3; by = r % G.gy[gi]; bz = r / G.gy[gi];
    } else {
        const int tiles = nx * G.gy[gi];
        const int chunk = local / (8 * tiles), j = local - chunk * 8 * tiles;
        const int tile = j >> 3;
        bz = chunk * 8 + (j & 7); bx = tile % nx; by = tile / nx;
    }
    if (bz >= G.gz[gi]) return;
    gemm_tile<EPI_SPLIT, BM_, BN_>(G.g[gi], bx, by, bz, G.gz[gi]);
}

// dW[kk][n] = sum over the X terms (rows kk + t*2d) and over the splits, in a fixed order;
// rows kk < d go to dW_self, d <= kk < 2d to dW_nbr.
// W = outputs per thread: 4 (16-byte loads) where d_in * d_out is a multiple of 4, which keeps every partial tile
// and the boundary between dW_self and dW_nbr 16-byte aligned; 1 otherwise.
template <int W>
__device__ __forceinline__ void dw_reduce_block(const int block, const float* __restrict__ partial, int64_t split_stride,
                                                int groups, int zterms, int rows, int xterms, int d_in, int d_out,
                                                int min_chunks, float* __restrict__ dws, float* __restrict__ dwn)
{
    // 64 W consecutive outputs per workgroup; each of its 4 waves sums a quarter of the list of partials
    __shared__ float quarter[4][64 * W];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int idx = (block * 64 + tx) * W;
    const bool live = idx < 2 * d_in * d_out;
    const int eff = effective_splits(groups, (rows + BK - 1) / BK, min_chunks);   // the splits the GEMM actually wrote
    // Wave ty takes the splits ty, ty + 4, ... of every (X term, dZ term) combination, eight loads in flight into
    // eight running sums (a load past the last split re-reads the last one and counts as zero).  The order is fixed.
    typedef float vecw __attribute__((ext_vector_type(W)));
    const float* base = partial + (live ? idx : 0);
    vecw acc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = vecw(0.f);
    if (live) {
        for (int t = 0; t < xterms; ++t)
            for (int zt = 0; zt < zterms; ++zt) {
                const float* src = base + (int64_t)zt * groups * split_stride + (int64_t)t * 2 * d_in * d_out;
                for (int z = ty; z < eff; z += 32) {
                    vecw v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const vecw*>(src + (int64_t)min(z + 4 * u, eff - 1) * split_stride);
#pragma unroll
                    for (int u = 0; u < 8; ++u) acc[u] += (z + 4 * u < eff) ? v[u] : vecw(0.f);
                }
            }
    }
    const vecw mine = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
#pragma unroll
    for (int e = 0; e < W; ++e) quarter[ty][tx * W + e] = mine[e];
    __syncthreads();
    if (ty == 0 && live) {
#pragma unroll
        for (int e = 0; e < W; ++e) {
            const float s = (quarter[0][tx * W + e] + quarter[1][tx * W + e]) + (quarter[2][tx * W + e] + quarter[3][tx * W + e]);
            const int o = idx + e;                               // = kk * d_out + n over [self ; nbr]
            if (o < d_in * d_out) dws[o] = s;
            else dwn[o - d_in * d_out] = s;
        }
    }
}

// db[n] = sum over the bias-gradient partials that the dW workgroups of the first row tile wrote, one per (dZ
// term, split), in a fixed order.  One thread per column.
constexpr int DB_COLS = TPB;
__device__ __forceinline__ void db_reduce_block(const int block, int rows, const float* __restrict__ db_partial, int groups,
                                                int zterms, int d_out, int min_chunks, float* __restrict__ db)
{
    const int n = block * DB_COLS + threadIdx.x;
    if (n >= d_out) return;
    const int eff = effective_splits(groups, (rows + BK - 1) / BK, min_chunks);   // the splits the GEMM actually wrote
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int zt = 0; zt < zterms; ++zt)
        for (int z = 0; z < eff; z += 4) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = db_partial[(int64_t)(zt * groups + min(z + u, eff - 1)) * d_out + n];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] += (z + u < eff) ? v[u] : 0.f;
        }
    db[n] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

// Last layer: db[n] = sum over the partial column sums of the dZ kernel's row-tile workgroups.  16 columns per workgroup; thread
// group g of 16 takes the tiles g, g + 16, ..., eight loads in flight; the sixteen partial sums are combined in a
// fixed order.
constexpr int DB_TILE_COLS = 16;
__device__ __forceinline__ void db_reduce_tiles(const int block, int rows, const float* __restrict__ db_partial, int d_out,
                                                float* __restrict__ db)
{
    __shared__ float part[TPB / DB_TILE_COLS][DB_TILE_COLS];
    constexpr int G = TPB / DB_TILE_COLS;
    const int tx = threadIdx.x % DB_TILE_COLS, g = threadIdx.x / DB_TILE_COLS;
    const int n = block * DB_TILE_COLS + tx;
    const int all_tiles = (rows + 63) / 64;
    const int tiles = all_tiles < (int)DN_DZ_MAX_ROW_BLOCKS ? all_tiles : (int)DN_DZ_MAX_ROW_BLOCKS;   // partial sums the dZ kernel wrote
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (n < d_out && tiles > 0) {
        for (int t = g; t < tiles; t += 8 * G) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = db_partial[(int64_t)min(t + G * u, tiles - 1) * d_out + n];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc[u] += (t + G * u < tiles) ? v[u] : 0.f;
        }
    }
    part[g][tx] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
    __syncthreads();
    if (g == 0 && n < d_out) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < G; ++j) s += part[j][tx];
        db[n] = s;
    }
}

// All reductions of the backward pass in one launch: each layer owns workgroups [begin[y], begin[y+1]); the
// first dw_blocks of them reduce the split-K partials of dW, the rest reduce the column sums for db.
struct ReduceGroup {
    const float* partial[DN_MAX_LAYERS]; int64_t split_stride[DN_MAX_LAYERS]; int groups[DN_MAX_LAYERS], zterms[DN_MAX_LAYERS];
    int xterms[DN_MAX_LAYERS], d_in[DN_MAX_LAYERS], d_out[DN_MAX_LAYERS], layer[DN_MAX_LAYERS];
    float *dws[DN_MAX_LAYERS], *dwn[DN_MAX_LAYERS], *db[DN_MAX_LAYERS];
    const float* db_partial[DN_MAX_LAYERS];
    int dw_blocks[DN_MAX_LAYERS], db_blocks[DN_MAX_LAYERS], vec4[DN_MAX_LAYERS];
    int db_from_tiles[DN_MAX_LAYERS];    // last layer: the partials are the dZ kernel's, one per row tile
    int begin[DN_MAX_LAYERS + 1];
    int n, min_chunks;
};
__global__ __launch_bounds__(TPB) void k_bwd_reduce_group(ReduceGroup R, const int32_t* __restrict__ hdr)
{
    int y = 0;
    while (y + 1 < R.n && (int)blockIdx.x >= R.begin[y + 1]) ++y;
    const int x = (int)blockIdx.x - R.begin[y];
    const int rows = hdr[HDR_N] - hdr[HDR_NODE_OFF + R.layer[y]];
    if (x < R.dw_blocks[y]) {
        if (R.vec4[y])
            dw_reduce_block<4>(x, R.partial[y], R.split_stride[y], R.groups[y], R.zterms[y], rows, R.xterms[y], R.d_in[y],
                               R.d_out[y], R.min_chunks, R.dws[y], R.dwn[y]);
        else
            dw_reduce_block<1>(x, R.partial[y], R.split_stride[y], R.groups[y], R.zterms[y], rows, R.xterms[y], R.d_in[y],
                               R.d_out[y], R.min_chunks, R.dws[y], R.dwn[y]);
    } else if (x < R.dw_blocks[y] + R.db_blocks[y]) {
        if (R.db_from_tiles[y]) db_reduce_tiles(x - R.dw_blocks[y], rows, R.db_partial[y], R.d_out[y], R.db[y]);
        else db_reduce_block(x - R.dw_blocks[y], rows, R.db_partial[y], R.groups[y], R.zterms[y], R.d_out[y], R.min_chunks, R.db[y]);
    }
}

// fp32 weights -> the two zero-padded bf16 layouts (round to nearest even).
__global__ __launch_bounds__(TPB) void k_pack_weights(const float* __restrict__ ws, const float* __restrict__ wn,
                                                      const float* __restrict__ bias, int d_in, int d_out, int kp, int np,
                                                      int nz, int xterms, int zterms, uint16_t* __restrict__ wt,
                                                      uint16_t* __restrict__ w, uint16_t* __restrict__ wf,
                                                      float* __restrict__ bias_out)
{
    const int idx = blockIdx.x * TPB + threadIdx.x;
    if (idx < d_out) bias_out[idx] = bias[idx];
    if (idx >= 2 * d_in * d_out) return;
    const int kk = idx / d_out, n = idx - kk * d_out;
    const float v = kk < d_in ? ws[(int64_t)kk * d_out + n] : wn[(int64_t)(kk - d_in) * d_out + n];
    const uint16_t h = f32_to_bf16(v);
    for (int t = 0; t < xterms; ++t) wt[(int64_t)n * kp + t * 2 * d_in + kk] = h;
    for (int t = 0; t < zterms; ++t) w[(int64_t)kk * nz + t * np + n] = h;
    // fragment order (dn_layer_bufs::wf): tile n / 16, step kk / 32, lane 16 ((kk % 32) / 8) + n % 16, element kk % 8
    if (wf) wf[((((int64_t)(n >> 4) * (2 * d_in / 32) + (kk >> 5)) * 64) + 16 * ((kk & 31) >> 3) + (n & 15)) * 8 + (kk & 7)] = h;
}

// colnorm[n] = L2 norm of row n of Wcat^T (all terms), one thread per row
__global__ __launch_bounds__(TPB) void k_col_norms(const uint16_t* __restrict__ wt, int d_out, int kp, float* __restrict__ colnorm)
{
    const int n = blockIdx.x * TPB + threadIdx.x;
    if (n >= d_out) return;
    float s = 0.f;
    for (int kk = 0; kk < kp; ++kk) {
        const float v = __uint_as_float((uint32_t)wt[(int64_t)n * kp + kk] << 16);
        s += v * v;
    }
    colnorm[n] = sqrtf(s) * 1.0001f;
}

// Tile edge of the GraphSage GEMMs.  Forward and dX have few rows per mini-batch (the output rows of a layer) and a
// short reduction: 64 x 64 tiles give four times the workgroups, several per compute unit, which hides the
// memory latency of the few k-steps (measured 9.6 vs 20.8 us on the last layer, 15.3 vs 24.7 on the middle
// one of the 111M-node workload).  The weight gradients reduce over the rows and are split along them anyway:
// 128 x 128 tiles re-read less.  DN_GEMM_TILE / DN_GEMM_TILE_DW (64 or 128) in the environment override, read once.
int tile_from_env(const char* name, int fallback)
{
    const char* e = getenv(name);
    const int v = e ? atoi(e) : 0;
    return (v == 64 || v == 128) ? v : fallback;
}
int gemm_tile_edge()
{
    static const int edge = tile_from_env("DN_GEMM_TILE", 64);
    return edge;
}
// Workgroups the weight-gradient GEMM of one layer aims for when it splits the reduction.  A layer of few output
// tiles (8 at 256 x 256 weights) gets one workgroup per compute unit: every further split is another 64 KB partial
// tile per output tile to write and to read back, more than the shorter loops save (111M-node workload: 21.8 us at
// 256, 29.8 at 384).  A layer of many output tiles (48 at 1536 x 256) has long reductions per split and gains from
// a second workgroup on half of the compute units (122M-node workload: 63.0 us at 288 workgroups, 57.1 at 336,
// 52.2 at 384, 58.9 at 432, 54.1 at 480).  DN_DW_BLOCKS in the environment overrides both, read once.
int dw_target_blocks(int tiles)
{
    static const int n = [] { const char* e = getenv("DN_DW_BLOCKS"); const int v = e ? atoi(e) : 0; return v > 0 ? v : 0; }();
    return n > 0 ? n : (tiles >= 32 ? 384 : 256);
}
// DN_DW_MIN_CHUNKS in the environment overrides the fewest k-steps per split (default 8), read once
int dw_min_chunks()
{
    static const int n = [] { const char* e = getenv("DN_DW_MIN_CHUNKS"); const int v = e ? atoi(e) : 0; return v > 0 ? v : 8; }();
    return n;
}
int dw_place()
{
    static const int n = [] { const char* e = getenv("DN_DW_PLACE"); return e ? atoi(e) : 0; }();
    return n;
}
int gemm_tile_edge_dw()
{
    static const int edge = tile_from_env("DN_GEMM_TILE_DW", 128);
    return edge;
}

template <int EPI, int T>
int launch_t(const GemmArgs& a, int64_t m_cap, int splits, hipStream_t st)
{
    dim3 grid((unsigned)((a.ncols + T - 1) / T), (unsigned)dn_round_up((m_cap + T - 1) / T, 8), (unsigned)splits);
    if (grid.y == 0) grid.y = 8;
    if (grid.y > (unsigned)GEMM_MAX_ROW_BLOCKS) grid.y = GEMM_MAX_ROW_BLOCKS;
    switch (a.layer) {
        case 1: hipLaunchKernelGGL((k_gemm_nt<EPI, 1, T, T>), grid, dim3(TPB), 0, st, a); break;
        case 2: hipLaunchKernelGGL((k_gemm_nt<EPI, 2, T, T>), grid, dim3(TPB), 0, st, a); break;
        case 3: hipLaunchKernelGGL((k_gemm_nt<EPI, 3, T, T>), grid, dim3(TPB), 0, st, a); break;
        default: hipLaunchKernelGGL((k_gemm_nt<EPI, 4, T, T>), grid, dim3(TPB), 0, st, a); break;
    }
    DN_LAUNCH_CHECK("k_gemm_nt");
    return DN_OK;
}

// forward GEMM, 128 x 128 tiles loaded straight into LDS
int launch_direct(const GemmArgs& a, int64_t m_cap, hipStream_t st)
{
    constexpr int T = 128;
    constexpr unsigned lds = NT_DIRECT_BUFFERS * 2u * T * BK * 2u;
    dim3 grid((unsigned)((a.ncols + T - 1) / T), (unsigned)dn_round_up((m_cap + T - 1) / T, 8), 1u);
    if (grid.y == 0) grid.y = 8;
    if (grid.y > (unsigned)GEMM_MAX_ROW_BLOCKS) grid.y = GEMM_MAX_ROW_BLOCKS;
    if (lds > 65536u) {                                         // more dynamic LDS than a kernel gets without asking
        static const hipError_t attr = [] {
            hipError_t e = hipSuccess;
            const void* fns[4] = {reinterpret_cast<const void*>(&k_gemm_nt<EPI_BIAS_ACT, 1, T, T, true>),
                                  reinterpret_cast<const void*>(&k_gemm_nt<EPI_BIAS_ACT, 2, T, T, true>),
                                  reinterpret_cast<const void*>(&k_gemm_nt<EPI_BIAS_ACT, 3, T, T, true>),
                                  reinterpret_cast<const void*>(&k_gemm_nt<EPI_BIAS_ACT, 4, T, T, true>)};
            for (const void* f : fns) {
                const hipError_t r = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (r != hipSuccess) e = r;
            }
            return e;
        }();
        if (attr != hipSuccess) return dn_fail(DN_EHIP, "hipFuncSetAttribute(dynamic LDS of the forward GEMM)");
    }
    switch (a.layer) {
        case 1: hipLaunchKernelGGL((k_gemm_nt<EPI_BIAS_ACT, 1, T, T, true>), grid, dim3(TPB), lds, st, a); break;
        case 2: hipLaunchKernelGGL((k_gemm_nt<EPI_BIAS_ACT, 2, T, T, true>), grid, dim3(TPB), lds, st, a); break;
        case 3: hipLaunchKernelGGL((k_gemm_nt<EPI_BIAS_ACT, 3, T, T, true>), grid, dim3(TPB), lds, st, a); break;
        default: hipLaunchKernelGGL((k_gemm_nt<EPI_BIAS_ACT, 4, T, T, true>), grid, dim3(TPB), lds, st, a); break;
    }
    DN_LAUNCH_CHECK("k_gemm_nt (direct)");
    return DN_OK;
}
// DN_GEMM_DIRECT=0 in the environment keeps every forward GEMM on the register path, read once
bool nt_direct_enabled()
{
    static const bool on = [] { const char* e = getenv("DN_GEMM_DIRECT"); return !(e && atoi(e) == 0); }();
    return on;
}

template <int EPI>
int launch(const GemmArgs& a, int64_t m_cap, int splits, hipStream_t st, const char* tag)
{
    dn_prof_scope ps(tag, a.layer, st);
    if (EPI == EPI_BIAS_ACT && a.red_const >= NT_DIRECT_MIN_K && splits == 1 && nt_direct_enabled()) return launch_direct(a, m_cap, st);
    return gemm_tile_edge() == 64 ? launch_t<EPI, 64>(a, m_cap, splits, st) : launch_t<EPI, 128>(a, m_cap, splits, st);
}

}  // namespace

// Forward linear of layer i (1-based): out = act(X^i * Wcat + b).
int dn_gemm_forward(const dn_model* m, const dn_batch* b, int i, float* out, int64_t ldc, hipStream_t st)
{
    const dn_layer_bufs& L = m->layer[i - 1];
    GemmArgs a{};
    a.A = reinterpret_cast<const uint16_t*>(L.x); a.lda = L.kp;
    a.B = reinterpret_cast<const uint16_t*>(L.wt); a.ldb = L.kp;
    a.C = out; a.ldc = ldc;
    a.hdr = b->hdr; a.layer = i; a.m_const = -1; a.ncols = L.d_out; a.red_const = L.kp;
    a.bias = L.bias; a.relu = (i < m->k) ? 1 : 0; a.split_stride = 0; a.terms = 1; a.b_term_stride = 0;
    a.rownorm = L.rownorm; a.colnorm = L.colnorm;
    // bound on |fp32 sum - exact sum| / (|x| |w|): 8 sqrt(K) 2^-24.  K additions, each off by at most 2^-24 of a
    // partial sum that Cauchy-Schwarz bounds by |x| |w|; the errors add like a random walk, and 8 standard
    // deviations leave a failure probability below 1e-14 per element (the worst case, K 2^-24, needs aligned errors)
    a.gamma = 8.0f * sqrtf((float)L.kp) * 5.9604645e-8f;
    a.fix_count = m->fix_count;
    return launch<EPI_BIAS_ACT>(a, L.rows_cap, 1, st, "gemm_fwd");
}

// dX = bf16(dZ) * Wcat^T   -> m->dx [rows x kp], columns [0, 2*d_in) valid.
int dn_gemm_dx(const dn_model* m, const dn_batch* b, int i, hipStream_t st)
{
    const dn_layer_bufs& L = m->layer[i - 1];
    GemmArgs a{};
    a.A = reinterpret_cast<const uint16_t*>(L.dzb); a.lda = L.nz;
    a.B = reinterpret_cast<const uint16_t*>(L.w); a.ldb = L.nz;
    a.C = m->dx; a.ldc = 2 * L.d_in;
    a.hdr = b->hdr; a.layer = i; a.m_const = -1; a.ncols = 2 * L.d_in; a.red_const = L.nz;
    a.bias = nullptr; a.relu = 0; a.split_stride = 0; a.terms = 1; a.b_term_stride = 0;
    return launch<EPI_PLAIN>(a, L.rows_cap, 1, st, "gemm_dx");
}

// dWcat^i = X^i^T * bf16(dZ^i) for every layer in one launch (reduction over the layer's rows split several
// ways), then one launch that reduces the partials in a fixed order and finishes db.
int dn_gemm_dw_all(const dn_model* m, const dn_batch* b, float* const* dws, float* const* dwn, float* const* dbias,
                   hipStream_t st)
{
    GemmGroup G{};
    ReduceGroup R{};
    G.n = m->k;
    G.place = dw_place();
    R.n = m->k;
    R.min_chunks = dw_min_chunks();
    int blocks = 0, red_blocks = 0;
    const int T = gemm_tile_edge_dw();
    for (int i = 1; i <= m->k; ++i) {
        const dn_layer_bufs& L = m->layer[i - 1];
        int64_t chunks_cap = (L.rows_cap + BK - 1) / BK;
        // enough workgroups to fill the chip, no more: every split costs a partial tile to write and re-read
        const int tiles = ((L.kx + T - 1) / T) * ((L.d_out + T - 1) / T) * (DW_FUSE ? 1 : L.zterms);
        int splits = ((T == 64 ? 2048 : dw_target_blocks(tiles)) + tiles - 1) / tiles;
        if (splits > m->splits) splits = m->splits;
        if (splits > chunks_cap) splits = (int)(chunks_cap > 0 ? chunks_cap : 1);
        if (splits < 1) splits = 1;
        GemmArgs& a = G.g[i - 1];
        a.A = reinterpret_cast<const uint16_t*>(L.x); a.lda = L.kp; a.a_cols = L.kp;
        a.B = reinterpret_cast<const uint16_t*>(L.dzb); a.ldb = L.nz; a.b_cols = L.np;
        a.C = L.partial; a.ldc = L.d_out;
        a.hdr = b->hdr; a.layer = i; a.m_const = L.kx; a.ncols = L.d_out; a.red_const = -1;
        a.bias = nullptr; a.relu = 0; a.split_stride = (int64_t)L.kx * L.d_out;
        a.terms = L.zterms; a.b_term_stride = L.np; a.min_chunks = dw_min_chunks();
        a.db_partial = (i < m->k) ? L.db_partial : nullptr;          // the last layer's bias gradient comes from its dZ kernel
        const int zsplits = splits * (DW_FUSE ? 1 : L.zterms);
        if ((int64_t)zsplits * a.split_stride > L.partial_floats) return dn_fail(DN_ECAPACITY, "dW partial buffer too small");
        const int y = i - 1;
        G.gx[y] = (L.d_out + T - 1) / T;
        G.gy[y] = (L.kx + T - 1) / T;
        G.gz[y] = zsplits;
        G.begin[y] = blocks;
        blocks += G.place == 0 ? G.gx[y] * (int)dn_round_up((int64_t)G.gy[y] * G.gz[y], 8)   // a multiple of 8: every layer starts on XCD 0
                               : G.gx[y] * G.gy[y] * (int)dn_round_up(G.gz[y], 8);
        R.partial[y] = L.partial; R.split_stride[y] = a.split_stride; R.groups[y] = splits; R.zterms[y] = DW_FUSE ? 1 : L.zterms;   // fused: the GEMM reduced both dZ terms
        R.xterms[y] = L.xterms;
        R.d_in[y] = L.d_in; R.d_out[y] = L.d_out; R.layer[y] = i;
        R.dws[y] = dws[y]; R.dwn[y] = dwn[y]; R.db[y] = dbias[y]; R.db_partial[y] = L.db_partial;
        R.vec4[y] = ((int64_t)L.d_in * L.d_out) % 4 == 0 ? 1 : 0;
        R.dw_blocks[y] = R.vec4[y] ? (2 * L.d_in * L.d_out + 255) / 256 : (2 * L.d_in * L.d_out + 63) / 64;
        R.db_from_tiles[y] = (i == m->k) ? 1 : 0;
        R.db_blocks[y] = (i == m->k) ? (L.d_out + DB_TILE_COLS - 1) / DB_TILE_COLS : (L.d_out + DB_COLS - 1) / DB_COLS;
        R.begin[y] = red_blocks;
        red_blocks += R.dw_blocks[y] + R.db_blocks[y];
    }
    G.begin[m->k] = blocks;
    R.begin[m->k] = red_blocks;
    { dn_prof_scope ps("gemm_dw_all", 0, st);
    if (T == 64) hipLaunchKernelGGL((k_gemm_dw_group<64, 64>), dim3((unsigned)blocks), dim3(TPB), 0, st, G);
    else {
        constexpr unsigned direct_lds = (DN_TN_DIRECT_BUFFERS > 0 && !DW_FUSE) ? DN_TN_DIRECT_BUFFERS * 2u * DN_TN_DIRECT_ROWS * 128u * 2u : 0u;
        if (direct_lds > 65536u) {                              // more dynamic LDS than a kernel gets without asking
            static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_dw_group<128, 128>),
                                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)direct_lds);
            if (attr != hipSuccess) return dn_fail(DN_EHIP, "hipFuncSetAttribute(dynamic LDS of the weight-gradient GEMM)");
        }
        hipLaunchKernelGGL((k_gemm_dw_group<128, 128>), dim3((unsigned)blocks), dim3(TPB), direct_lds, st, G);
    }
    }
    DN_LAUNCH_CHECK("k_gemm_dw_group");
    { dn_prof_scope ps("bwd_reduce_all", 0, st);
    hipLaunchKernelGGL(k_bwd_reduce_group, dim3((unsigned)red_blocks), dim3(TPB), 0, st, R, b->hdr);
    }
    DN_LAUNCH_CHECK("k_bwd_reduce_group");
    return DN_OK;
}

int dn_launch_set_weights(dn_model* m, const float* const* ws, const float* const* wn,
                          const float* const* bias, hipStream_t st)
{
    for (int i = 0; i < m->k; ++i) {
        dn_layer_bufs& L = m->layer[i];
        const int total = 2 * L.d_in * L.d_out;
        const int n = total > L.d_out ? total : L.d_out;
        hipLaunchKernelGGL(k_pack_weights, dim3((n + TPB - 1) / TPB), dim3(TPB), 0, st, ws[i], wn[i], bias[i], L.d_in,
                           L.d_out, L.kp, L.np, L.nz, L.xterms, L.zterms, reinterpret_cast<uint16_t*>(L.wt),
                           reinterpret_cast<uint16_t*>(L.w), reinterpret_cast<uint16_t*>(L.wf), L.bias);
        DN_LAUNCH_CHECK("k_pack_weights");
        hipLaunchKernelGGL(k_col_norms, dim3((L.d_out + TPB - 1) / TPB), dim3(TPB), 0, st,
                           reinterpret_cast<const uint16_t*>(L.wt), L.d_out, L.kp, L.colnorm);
        DN_LAUNCH_CHECK("k_col_norms");
    }
    return DN_OK;
}
