// 128 x 128 x 64 bf16 MFMA tile shared by the GEMM kernels of this library (gfx950).
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

struct TileRegs { u32x4 a[4], b[4]; };

// Accumulates the k-steps [kc_begin, kc_end) (units of BK) of the tile whose first rows are A_tile / B_tile.
// WRAP_B: B is shorter than A along the reduction index and repeats every b_wrap_chunks k-steps (an
// operand carried as several bf16 terms is multiplied with the other operand repeated).
// Register e of acc[i][j] holds row 64*wm + 32*i + 8*(e/4) + 4*(lane/32) + e%4, column 64*wn + 32*j + lane%32.
template <bool WRAP_B>
__device__ __forceinline__ void mainloop(const uint16_t* __restrict__ A_tile, const int64_t lda,
                                         const uint16_t* __restrict__ B_tile, const int64_t ldb,
                                         const int kc_begin, const int kc_end, const int b_wrap_chunks,
                                         f32x16 (&acc)[2][2])
{
    __shared__ u32x4 As[2][BM * BK / 8];
    __shared__ u32x4 Bs[2][BN * BK / 8];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const uint16_t* a_ptr[4];
    const uint16_t* b_ptr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = t + TPB * i, row = id >> 3, c = id & 7;
        a_ptr[i] = A_tile + (int64_t)row * lda + c * 8;
        b_ptr[i] = B_tile + (int64_t)row * ldb + c * 8;
    }
    auto load_tiles = [&](TileRegs& r, int kc) {
        const int64_t k0 = (int64_t)kc * BK;
        const int64_t k0b = WRAP_B ? (int64_t)(kc % b_wrap_chunks) * BK : k0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r.a[i] = *reinterpret_cast<const u32x4*>(a_ptr[i] + k0);
            r.b[i] = *reinterpret_cast<const u32x4*>(b_ptr[i] + k0b);
        }
    };
    auto store_tiles = [&](const TileRegs& r, int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = t + TPB * i, row = id >> 3, c = id & 7;
            As[buf][slot(row, c)] = r.a[i];
            Bs[buf][slot(row, c)] = r.b[i];
        }
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int c = 2 * ks + (lane >> 5);
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = __builtin_bit_cast(bf16x8, As[buf][slot(wm * 64 + i * 32 + (lane & 31), c)]);
                fb[i] = __builtin_bit_cast(bf16x8, Bs[buf][slot(wn * 64 + i * 32 + (lane & 31), c)]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    };

    TileRegs r0, r1;
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
