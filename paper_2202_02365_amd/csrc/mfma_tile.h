// 128 x 128 x 64 (or 64 x 64 x 64) bf16 MFMA tile shared by the GEMM kernels of this library (gfx950).
//
//   acc += A_tile[128 x R] * B_tile[128 x R]^T     both row-major bf16, reduction index contiguous,
// which is the layout v_mfma_f32_32x32x16_bf16 wants (each lane supplies 8 consecutive reduction
// elements of one row).  One workgroup of 4 waves (2 x 2), each wave 64 x 64 = 2 x 2 MFMA tiles of
// 32 x 32.  Operand tiles go global -> registers -> LDS (16-byte slots, XOR-swizzled by row so the
// fragment reads of 32 consecutive rows spread over all banks); two register stages keep the next two
// tiles' global loads in flight while the current one is multiplied, two LDS buffers allow a single
// barrier per k-step.  Tile loads carry no bounds check: operands are padded to whole tiles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dn_mma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 64, TPB = 256;

// 16-byte slot of chunk c of tile row `row`: 16 consecutive rows of one chunk column land in 16 different
// 16-byte bank groups (row parity picks the half, (row >> 1) & 7 permutes the chunks within it)
__device__ __forceinline__ int slot(int row, int c) { return row * 8 + (c ^ ((row >> 1) & 7)); }

template <int LA, int LB>
struct TileRegs { u32x4 a[LA], b[LB]; };

// Accumulates the k-steps [kc_begin, kc_end) (units of BK) of the BM_ x BN_ tile whose first rows are A_tile /
// B_tile (BM_, BN_ in {64, 128}; the four waves form a 2 x 2 grid, each wave (BM_/2) x (BN_/2)).
// WRAP_B: B is shorter than A along the reduction index and repeats every b_wrap_chunks k-steps (an
// operand carried as several bf16 terms is multiplied with the other operand repeated).
// Register e of acc[i][j] holds row (BM_/2)*wm + 32*i + 8*(e/4) + 4*(lane/32) + e%4, column (BN_/2)*wn + 32*j + lane%32.
// The small tile is for problems with few rows: four times as many workgroups, several of them per compute
// unit, so that one workgroup's memory latency is covered by another's arithmetic.
template <int BM_, int BN_, bool WRAP_B>
__device__ __forceinline__ void mainloop(const uint16_t* __restrict__ A_tile, const int64_t lda,
                                         const uint16_t* __restrict__ B_tile, const int64_t ldb,
                                         const int kc_begin, const int kc_end, const int b_wrap_chunks,
                                         f32x16 (&acc)[BM_ / 64][BN_ / 64])
{
    constexpr int MI = BM_ / 64, NJ = BN_ / 64;      // 32 x 32 MFMA tiles per wave
    constexpr int LA = BM_ / 32, LB = BN_ / 32;      // 16-byte loads per thread and k-step
    __shared__ u32x4 As[2][BM_ * BK / 8];
    __shared__ u32x4 Bs[2][BN_ * BK / 8];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const uint16_t* a_ptr[LA];
    const uint16_t* b_ptr[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int id = t + TPB * i, row = id >> 3, c = id & 7;
        a_ptr[i] = A_tile + (int64_t)row * lda + c * 8;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int id = t + TPB * i, row = id >> 3, c = id & 7;
        b_ptr[i] = B_tile + (int64_t)row * ldb + c * 8;
    }
    auto load_tiles = [&](TileRegs<LA, LB>& r, int kc) {
        const int64_t k0 = (int64_t)kc * BK;
        const int64_t k0b = WRAP_B ? (int64_t)(kc % b_wrap_chunks) * BK : k0;
#pragma unroll
        for (int i = 0; i < LA; ++i) r.a[i] = *reinterpret_cast<const u32x4*>(a_ptr[i] + k0);
#pragma unroll
        for (int i = 0; i < LB; ++i) r.b[i] = *reinterpret_cast<const u32x4*>(b_ptr[i] + k0b);
    };
    auto store_tiles = [&](const TileRegs<LA, LB>& r, int buf) {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int id = t + TPB * i, row = id >> 3, c = id & 7;
            As[buf][slot(row, c)] = r.a[i];
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int id = t + TPB * i, row = id >> 3, c = id & 7;
            Bs[buf][slot(row, c)] = r.b[i];
        }
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int c = 2 * ks + (lane >> 5);
            bf16x8 fa[MI], fb[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                fa[i] = __builtin_bit_cast(bf16x8, As[buf][slot(wm * (BM_ / 2) + i * 32 + (lane & 31), c)]);
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                fb[j] = __builtin_bit_cast(bf16x8, Bs[buf][slot(wn * (BN_ / 2) + j * 32 + (lane & 31), c)]);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    };

    TileRegs<LA, LB> r0, r1;
    if (kc_begin + 0 < kc_end) load_tiles(r0, kc_begin + 0);
    if (kc_begin + 1 < kc_end) load_tiles(r1, kc_begin + 1);
    int kc = kc_begin, buf = 0;
#define DN_GEMM_STEP(R)                                       \
    if (kc >= kc_end) break;                                  \
    store_tiles(R, buf);                                      \
    __syncthreads();                                          \
    if (kc + 2 < kc_end) load_tiles(R, kc + 2);               \
    multiply(buf);                                            \
    buf ^= 1;                                                 \
    ++kc;
    for (;;) {
        DN_GEMM_STEP(r0)
        DN_GEMM_STEP(r1)
    }
#undef DN_GEMM_STEP
}

}  // namespace dn_mma
