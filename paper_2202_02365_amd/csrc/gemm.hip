// bf16 MFMA GEMM for the GraphSage linear layers (the one dense contraction of the path).
//
// One kernel form serves forward, dX and dW:   C[M x Nc] = A[M x R] * B[Nc x R]^T
// with A and B row-major bf16 and the reduction index R contiguous in both, which is the layout
// v_mfma_f32_32x32x16_bf16 wants (each lane supplies 8 consecutive reduction elements of one row).
//   forward : A = X^i  = [bf16(H_self) | bf16(mean)]   B = Wcat^T        epilogue + bias, ReLU
//   dX      : A = bf16(dZ)                              B = Wcat          plain store
//   dW      : A = X^T (reduction over batch rows)       B = bf16(dZ)^T    split over the reduction,
//             partial tiles reduced afterwards in a fixed order (deterministic).
// Tile: 128 x 128 x 64 per workgroup of 4 waves (2 x 2), each wave 64 x 64 = 2 x 2 MFMA tiles of
// 32 x 32.  Operand tiles go global -> registers -> LDS (16-byte slots, XOR-swizzled by row so the
// fragment reads of 32 consecutive rows spread over all banks); the next tile's global loads
// are in flight while the current one is multiplied.  M and the dW reduction length live in
// device memory (they depend on the sample); the grid is sized by capacity and surplus
// workgroups leave at once.
#include "dn_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 64, TPB = 256;
enum { EPI_BIAS_ACT = 0, EPI_PLAIN = 1, EPI_SPLIT = 2 };

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
};

__device__ __forceinline__ int slot(int row, int c) { return row * 8 + (c ^ (row & 7)); }

template <int EPI>
__global__ __launch_bounds__(TPB) void k_gemm_nt(GemmArgs a)
{
    __shared__ u32x4 As[BM * BK / 8];
    __shared__ u32x4 Bs[BN * BK / 8];

    const int rows_layer = a.hdr[HDR_N] - a.hdr[HDR_NODE_OFF + a.layer];
    const int M = a.m_const >= 0 ? a.m_const : rows_layer;
    const int red = a.red_const >= 0 ? a.red_const : ((rows_layer + BK - 1) / BK) * BK;
    const int row0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    if (row0 >= M) return;

    // reduction range of this split
    const int chunks = red / BK;
    const int per = (chunks + gridDim.z - 1) / gridDim.z;
    const int kc_begin = blockIdx.z * per;
    const int kc_end = min(chunks, kc_begin + per);

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    u32x4 ra[4], rb[4];
    auto load_tiles = [&](int kc) {
        const int64_t k0 = (int64_t)kc * BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = t + TPB * i, row = id >> 3, c = id & 7;
            ra[i] = *reinterpret_cast<const u32x4*>(a.A + (int64_t)(row0 + row) * a.lda + k0 + c * 8);
            rb[i] = *reinterpret_cast<const u32x4*>(a.B + (int64_t)(col0 + row) * a.ldb + k0 + c * 8);
        }
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = t + TPB * i, row = id >> 3, c = id & 7;
            As[slot(row, c)] = ra[i];
            Bs[slot(row, c)] = rb[i];
        }
    };

    if (kc_begin < kc_end) load_tiles(kc_begin);
    for (int kc = kc_begin; kc < kc_end; ++kc) {
        store_tiles();
        __syncthreads();
        if (kc + 1 < kc_end) load_tiles(kc + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int c = 2 * ks + (lane >> 5);
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = __builtin_bit_cast(bf16x8, As[slot(wm * 64 + i * 32 + (lane & 31), c)]);
                fb[i] = __builtin_bit_cast(bf16x8, Bs[slot(wn * 64 + i * 32 + (lane & 31), c)]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // epilogue: lane holds column (lane & 31); register e holds row 8*(e/4) + 4*(lane/32) + e%4
    float* C = a.C;
    if (EPI == EPI_SPLIT) C += (int64_t)blockIdx.z * a.split_stride;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = col0 + wn * 64 + j * 32 + (lane & 31);
            if (n >= a.ncols) continue;
            const float bv = (EPI == EPI_BIAS_ACT) ? a.bias[n] : 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = row0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (m < M) {
                    float v = acc[i][j][e];
                    if (EPI == EPI_BIAS_ACT) {
                        v += bv;
                        if (a.relu) v = fmaxf(v, 0.f);
                    }
                    C[(int64_t)m * a.ldc + n] = v;
                }
            }
        }
}

// dW[kk][n] = sum over splits, in split order; rows kk < d go to dW_self, d <= kk < 2d to dW_nbr.
__global__ __launch_bounds__(TPB) void k_dw_reduce(const float* __restrict__ partial, int64_t split_stride, int splits,
                                                   int d_in, int d_out, float* __restrict__ dws, float* __restrict__ dwn)
{
    const int idx = blockIdx.x * TPB + threadIdx.x;
    if (idx >= 2 * d_in * d_out) return;
    const int kk = idx / d_out, n = idx - kk * d_out;
    float s = 0.f;
    for (int z = 0; z < splits; ++z) s += partial[(int64_t)z * split_stride + (int64_t)kk * d_out + n];
    if (kk < d_in) dws[(int64_t)kk * d_out + n] = s;
    else dwn[(int64_t)(kk - d_in) * d_out + n] = s;
}

// fp32 weights -> the two zero-padded bf16 layouts (round to nearest even).
__device__ __forceinline__ uint16_t f32_to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__global__ __launch_bounds__(TPB) void k_pack_weights(const float* __restrict__ ws, const float* __restrict__ wn,
                                                      const float* __restrict__ bias, int d_in, int d_out, int kp, int np,
                                                      uint16_t* __restrict__ wt, uint16_t* __restrict__ w,
                                                      float* __restrict__ bias_out)
{
    const int idx = blockIdx.x * TPB + threadIdx.x;
    if (idx < d_out) bias_out[idx] = bias[idx];
    if (idx >= 2 * d_in * d_out) return;
    const int kk = idx / d_out, n = idx - kk * d_out;
    const float v = kk < d_in ? ws[(int64_t)kk * d_out + n] : wn[(int64_t)(kk - d_in) * d_out + n];
    const uint16_t h = f32_to_bf16(v);
    wt[(int64_t)n * kp + kk] = h;
    w[(int64_t)kk * np + n] = h;
}

template <int EPI>
int launch(const GemmArgs& a, int64_t m_cap, int splits, hipStream_t st)
{
    dim3 grid((unsigned)((a.ncols + BN - 1) / BN), (unsigned)((m_cap + BM - 1) / BM), (unsigned)splits);
    if (grid.y == 0) grid.y = 1;
    hipLaunchKernelGGL((k_gemm_nt<EPI>), grid, dim3(TPB), 0, st, a);
    DN_LAUNCH_CHECK("k_gemm_nt");
    return DN_OK;
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
    a.bias = L.bias; a.relu = (i < m->k) ? 1 : 0; a.split_stride = 0;
    return launch<EPI_BIAS_ACT>(a, L.rows_cap, 1, st);
}

// dX = bf16(dZ) * Wcat^T   -> m->dx [rows x kp], columns [0, 2*d_in) valid.
int dn_gemm_dx(const dn_model* m, const dn_batch* b, int i, hipStream_t st)
{
    const dn_layer_bufs& L = m->layer[i - 1];
    GemmArgs a{};
    a.A = reinterpret_cast<const uint16_t*>(m->dzb); a.lda = L.np;
    a.B = reinterpret_cast<const uint16_t*>(L.w); a.ldb = L.np;
    a.C = m->dx; a.ldc = L.kp;
    a.hdr = b->hdr; a.layer = i; a.m_const = -1; a.ncols = 2 * L.d_in; a.red_const = L.np;
    a.bias = nullptr; a.relu = 0; a.split_stride = 0;
    return launch<EPI_PLAIN>(a, L.rows_cap, 1, st);
}

// dWcat = X^T * bf16(dZ), reduction over the layer's rows split `splits` ways, then reduced in order.
int dn_gemm_dw(const dn_model* m, const dn_batch* b, int i, float* dws, float* dwn, hipStream_t st)
{
    const dn_layer_bufs& L = m->layer[i - 1];
    int64_t chunks_cap = (L.rows_cap + BK - 1) / BK;
    int splits = m->splits;
    if (splits > chunks_cap) splits = (int)(chunks_cap > 0 ? chunks_cap : 1);
    GemmArgs a{};
    a.A = reinterpret_cast<const uint16_t*>(m->xt); a.lda = L.rows_pad;
    a.B = reinterpret_cast<const uint16_t*>(m->dzbt); a.ldb = L.rows_pad;
    a.C = m->partial; a.ldc = L.d_out;
    a.hdr = b->hdr; a.layer = i; a.m_const = 2 * L.d_in; a.ncols = L.d_out; a.red_const = -1;
    a.bias = nullptr; a.relu = 0; a.split_stride = (int64_t)2 * L.d_in * L.d_out;
    if ((int64_t)splits * a.split_stride > m->partial_floats)
        return dn_fail(DN_ECAPACITY, "dW partial buffer too small");
    int rc = launch<EPI_SPLIT>(a, 2 * L.d_in, splits, st);
    if (rc) return rc;
    const int total = 2 * L.d_in * L.d_out;
    hipLaunchKernelGGL(k_dw_reduce, dim3((total + TPB - 1) / TPB), dim3(TPB), 0, st, m->partial, a.split_stride, splits,
                       L.d_in, L.d_out, dws, dwn);
    DN_LAUNCH_CHECK("k_dw_reduce");
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
                           L.d_out, L.kp, L.np, reinterpret_cast<uint16_t*>(L.wt), reinterpret_cast<uint16_t*>(L.w),
                           L.bias);
        DN_LAUNCH_CHECK("k_pack_weights");
    }
    return DN_OK;
}
