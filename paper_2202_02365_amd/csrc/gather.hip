// dense_gather: H^0[r, :] = table[node_ids[r], :]  (Section 4.2 of the paper: the array of base
// representations, one row per entry of node_ids).  Pure HBM traffic: N rows read at random row
// addresses, N rows written sequentially.  A group of lanes moves one row in 16-byte pieces so
// that every row is a run of full-width coalesced accesses; rows are dealt round-robin to a
// grid that stays resident (N lives in device memory, so the grid cannot be sized by it).
#include "dn_internal.h"

namespace {

constexpr int TPB = 256;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// LANES lanes per row, each moving 16-byte chunks lane, lane+LANES, ...
template <int LANES>
__global__ __launch_bounds__(TPB) void k_gather16(const int32_t* __restrict__ hdr, const int32_t* __restrict__ node_ids,
                                                  const u32x4* __restrict__ table, int64_t ld_chunks, int chunks,
                                                  u32x4* __restrict__ out)
{
    const int N = hdr[HDR_N];
    const int lane = threadIdx.x % LANES;
    constexpr int ROWS_PER_BLOCK = TPB / LANES;
    for (int r = blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / LANES; r < N; r += gridDim.x * ROWS_PER_BLOCK) {
        const int64_t src = (int64_t)node_ids[r] * ld_chunks;
        const int64_t dst = (int64_t)r * chunks;
        for (int c = lane; c < chunks; c += LANES)
            out[dst + c] = __builtin_nontemporal_load(&table[src + c]);
    }
}

// Fallback for rows that are not a multiple of 16 bytes or not 16-byte aligned: element by element.
template <typename T>
__global__ __launch_bounds__(TPB) void k_gather_elem(const int32_t* __restrict__ hdr, const int32_t* __restrict__ node_ids,
                                                     const T* __restrict__ table, int64_t ld, int dim, T* __restrict__ out)
{
    const int N = hdr[HDR_N];
    const int lane = threadIdx.x & 63;
    constexpr int ROWS_PER_BLOCK = TPB / 64;
    for (int r = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6); r < N; r += gridDim.x * ROWS_PER_BLOCK) {
        const int64_t src = (int64_t)node_ids[r] * ld;
        const int64_t dst = (int64_t)r * dim;
        for (int c = lane; c < dim; c += 64) out[dst + c] = table[src + c];
    }
}

// table[node_ids[r], :] -= lr * g[r, :] for r < N.  node_ids holds every node once, so rows never collide.
// Multiply and subtract are rounded separately (no fused multiply-add), as the plain formula is.
__global__ __launch_bounds__(TPB) void k_embedding_sgd(const int32_t* __restrict__ hdr, const int32_t* __restrict__ node_ids,
                                                       float* __restrict__ table, int64_t ld, int dim,
                                                       const float* __restrict__ g, float lr)
{
#pragma clang fp contract(off)             // lr * g is rounded before the subtraction: no fused multiply-add
    const int N = hdr[HDR_N];
    const int lane = threadIdx.x & 63;
    constexpr int ROWS_PER_BLOCK = TPB / 64;
    for (int r = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6); r < N; r += gridDim.x * ROWS_PER_BLOCK) {
        float* row = table + (int64_t)node_ids[r] * ld;
        const float* gr = g + (int64_t)r * dim;
        for (int c = lane; c < dim; c += 64) {
            const float step = lr * gr[c];
            row[c] = row[c] - step;
        }
    }
}

// Adagrad on the touched rows, per element and in fp32 with every operation rounded on its own:
//   state += g * g;  table -= (lr * g) / (sqrt(state) + eps).     (square root and division are correctly rounded)
__global__ __launch_bounds__(TPB) void k_embedding_adagrad(const int32_t* __restrict__ hdr, const int32_t* __restrict__ node_ids,
                                                           float* __restrict__ table, float* __restrict__ state, int64_t ld,
                                                           int dim, const float* __restrict__ g, float lr, float eps)
{
#pragma clang fp contract(off)
    const int N = hdr[HDR_N];
    const int lane = threadIdx.x & 63;
    constexpr int ROWS_PER_BLOCK = TPB / 64;
    for (int r = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6); r < N; r += gridDim.x * ROWS_PER_BLOCK) {
        const int64_t base = (int64_t)node_ids[r] * ld;
        const float* gr = g + (int64_t)r * dim;
        for (int c = lane; c < dim; c += 64) {
            const float gv = gr[c];
            const float sq = gv * gv;
            const float acc = state[base + c] + sq;
            state[base + c] = acc;
            const float num = lr * gv;
            const float den = sqrtf(acc) + eps;          // sqrtf and '/' are correctly rounded in device code by default
            const float step = num / den;
            table[base + c] = table[base + c] - step;
        }
    }
}

// Softmax cross-entropy head, one wave per row: loss = logsumexp(z) - z[label], grad = scale * (softmax(z) - onehot).
// A label outside [0, C) leaves loss = NaN and grad = scale * softmax(z).
__global__ __launch_bounds__(TPB) void k_softmax_xent(const float* __restrict__ logits, int64_t ld, const int32_t* __restrict__ labels,
                                                      int64_t n, int C, float scale, float* __restrict__ loss,
                                                      float* __restrict__ grad, int64_t ldg)
{
    const int64_t r = (int64_t)blockIdx.x * (TPB / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (r >= n) return;
    const float* z = logits + r * ld;
    float m = -INFINITY;
    for (int c = lane; c < C; c += 64) m = fmaxf(m, z[c]);
    for (int s = 32; s > 0; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, 64));
    float sum = 0.f;
    for (int c = lane; c < C; c += 64) sum += expf(z[c] - m);
    for (int s = 32; s > 0; s >>= 1) sum += __shfl_xor(sum, s, 64);
    const int lab = labels[r];
    const bool ok = (unsigned)lab < (unsigned)C;
    const float lse = m + logf(sum);
    if (lane == 0) loss[r] = ok ? lse - z[lab] : __int_as_float(0x7fc00000);
    const float inv = 1.f / sum;
    for (int c = lane; c < C; c += 64) {
        float p = expf(z[c] - m) * inv;
        if (ok && c == lab) p -= 1.f;
        grad[r * ldg + c] = scale * p;
    }
}

// Plain streaming copy of known size: the reference a profiler's byte counters are scaled by.
__global__ __launch_bounds__(TPB) void k_calibration_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * TPB;
    for (int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

int dn_launch_embedding_sgd(const dn_batch* b, float* table, int32_t dim, int64_t ld, const float* dh0, float lr,
                            hipStream_t st)
{
    int64_t grid = (b->cap_nodes + 3) / 4;
    if (grid > 4096) grid = 4096;
    if (grid < 1) grid = 1;
    dn_prof_scope ps("embedding_sgd", 0, st);
    hipLaunchKernelGGL(k_embedding_sgd, dim3((int)grid), dim3(TPB), 0, st, b->hdr, b->node_ids, table, ld, dim, dh0, lr);
    DN_LAUNCH_CHECK("k_embedding_sgd");
    return DN_OK;
}

int dn_launch_embedding_adagrad(const dn_batch* b, float* table, float* state, int32_t dim, int64_t ld, const float* dh0,
                                float lr, float eps, hipStream_t st)
{
    int64_t grid = (b->cap_nodes + 3) / 4;
    if (grid > 4096) grid = 4096;
    if (grid < 1) grid = 1;
    dn_prof_scope ps("embedding_adagrad", 0, st);
    hipLaunchKernelGGL(k_embedding_adagrad, dim3((int)grid), dim3(TPB), 0, st, b->hdr, b->node_ids, table, state, ld, dim, dh0,
                       lr, eps);
    DN_LAUNCH_CHECK("k_embedding_adagrad");
    return DN_OK;
}

int dn_launch_softmax_xent(const float* logits, int64_t ld, const int32_t* labels, int64_t n, int32_t num_classes, float scale,
                           float* loss, float* grad, int64_t ldg, hipStream_t st)
{
    if (n == 0) return DN_OK;
    dn_prof_scope ps("softmax_xent", 0, st);
    const int64_t grid = (n + TPB / 64 - 1) / (TPB / 64);
    hipLaunchKernelGGL(k_softmax_xent, dim3((int)grid), dim3(TPB), 0, st, logits, ld, labels, n, num_classes, scale, loss,
                       grad, ldg);
    DN_LAUNCH_CHECK("k_softmax_xent");
    return DN_OK;
}

int dn_launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t st)
{
    const int64_t n16 = (int64_t)(bytes / 16);
    int64_t grid = (n16 + TPB - 1) / TPB;
    if (grid > 16384) grid = 16384;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(k_calibration_copy, dim3((int)grid), dim3(TPB), 0, st, static_cast<const u32x4*>(src),
                       static_cast<u32x4*>(dst), n16);
    DN_LAUNCH_CHECK("k_calibration_copy");
    return DN_OK;
}

int dn_launch_gather(const dn_batch* b, const void* table, int32_t dtype, int32_t dim, int64_t ld,
                     void* h0, hipStream_t st)
{
    const int elt = dtype == DN_F32 ? 4 : 2;
    const int64_t row_bytes = (int64_t)dim * elt, ld_bytes = ld * elt;
    const bool vec = (row_bytes % 16 == 0) && (ld_bytes % 16 == 0) && ((uintptr_t)table % 16 == 0) && ((uintptr_t)h0 % 16 == 0);
    const int64_t cap = b->cap_nodes;
    dn_prof_scope ps("gather", 0, st);
    if (vec) {
        const int chunks = (int)(row_bytes / 16);
        int lanes = 4;
        while (lanes < chunks && lanes < 64) lanes <<= 1;
        const int rows_per_block = TPB / lanes;
        int64_t grid = (cap + rows_per_block - 1) / rows_per_block;
        if (grid > 4096) grid = 4096;
        if (grid < 1) grid = 1;
        const u32x4* t = static_cast<const u32x4*>(table);
        u32x4* o = static_cast<u32x4*>(h0);
        const int64_t ldc = ld_bytes / 16;
#define DN_GATHER_CASE(L)                                                                                         \
    case L: hipLaunchKernelGGL((k_gather16<L>), dim3((int)grid), dim3(TPB), 0, st, b->hdr, b->node_ids, t, ldc,   \
                               chunks, o); break;
        switch (lanes) {
            DN_GATHER_CASE(4) DN_GATHER_CASE(8) DN_GATHER_CASE(16) DN_GATHER_CASE(32)
            default: hipLaunchKernelGGL((k_gather16<64>), dim3((int)grid), dim3(TPB), 0, st, b->hdr, b->node_ids, t, ldc,
                                        chunks, o); break;
        }
#undef DN_GATHER_CASE
    } else {
        int64_t grid = (cap + 3) / 4;
        if (grid > 4096) grid = 4096;
        if (grid < 1) grid = 1;
        if (dtype == DN_F32)
            hipLaunchKernelGGL((k_gather_elem<float>), dim3((int)grid), dim3(TPB), 0, st, b->hdr, b->node_ids,
                               static_cast<const float*>(table), ld, dim, static_cast<float*>(h0));
        else
            hipLaunchKernelGGL((k_gather_elem<uint16_t>), dim3((int)grid), dim3(TPB), 0, st, b->hdr, b->node_ids,
                               static_cast<const uint16_t*>(table), ld, dim, static_cast<uint16_t*>(h0));
    }
    DN_LAUNCH_CHECK("k_gather");
    return DN_OK;
}
