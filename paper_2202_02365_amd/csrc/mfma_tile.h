// bf16 MFMA tile main loops shared by the GEMM kernels of this library (gfx950): T x T x 64 per k-step, T = 64 or 128.
//
//   mainloop     acc += A_tile[T x R] * B_tile[T x R]^T     both row-major bf16, reduction index contiguous,
// which is the layout v_mfma_f32_32x32x16_bf16 wants (each lane supplies 8 consecutive reduction
// elements of one row).  One workgroup of 4 waves (2 x 2), each wave (T/2) x (T/2) in MFMA tiles of
// 32 x 32.  Operand tiles go global -> registers -> LDS (16-byte slots, XOR-swizzled by row so the
// fragment reads of 32 consecutive rows spread over all banks); two register stages keep the next two
// tiles' global loads in flight while the current one is multiplied, two LDS buffers allow a single
// barrier per k-step.  Tile loads carry no bounds check: operands are padded to whole tiles.
//
//   mainloop_tn  the same contraction for operands whose ROW index is the reduction index (see there).
//   mainloop_tn_direct  mainloop_tn for 128 x 128 tiles with the tiles loaded from global memory straight into LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

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
// STAGES register stages of global prefetch: a k-step waits for a tile requested STAGES k-steps before.  More than
// two were measured slower (figures in gemm.hip): they cost the registers that let four workgroups share a compute unit.
template <int BM_, int BN_, bool WRAP_B, int STAGES = 2>
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
    // KG reduction sub-steps of 16 have their fragments requested together (all four on the small tile, two on the
    // large one, whose accumulators leave fewer registers): the LDS reads of a sub-step then overlap the matrix
    // instructions of the one before instead of being waited for one by one.
    constexpr int KG = (MI * NJ == 1) ? 4 : 2;
    auto multiply = [&](int buf) {
#pragma unroll
        for (int k0 = 0; k0 < BK / 16; k0 += KG) {
            bf16x8 fa[KG][MI], fb[KG][NJ];
#pragma unroll
            for (int kk = 0; kk < KG; ++kk) {
                const int c = 2 * (k0 + kk) + (lane >> 5);
#pragma unroll
                for (int i = 0; i < MI; ++i)
                    fa[kk][i] = __builtin_bit_cast(bf16x8, As[buf][slot(wm * (BM_ / 2) + i * 32 + (lane & 31), c)]);
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    fb[kk][j] = __builtin_bit_cast(bf16x8, Bs[buf][slot(wn * (BN_ / 2) + j * 32 + (lane & 31), c)]);
            }
#pragma unroll
            for (int kk = 0; kk < KG; ++kk)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk][i], fb[kk][j], acc[i][j], 0, 0, 0);
            // order within the scheduling region: the group's LDS reads, then its matrix instructions (left alone, the
            // scheduler puts each pair of reads right in front of its instruction and waits for both every time)
            __builtin_amdgcn_sched_group_barrier(0x100, KG * (MI + NJ), 0);
            __builtin_amdgcn_sched_group_barrier(0x008, KG * MI * NJ, 0);
        }
    };

    // The prefetch is issued without a condition (past the last k-step it fetches the last tile again and nobody
    // uses it): behind a branch the compiler no longer knows how many loads are outstanding, and then waits for ALL of
    // them before a tile goes to LDS, which leaves a single tile in flight.  For the same reason the loop body is
    // straight-line code of STAGES whole k-steps with the trip count fixed on entry, and the remaining k-steps follow
    // the loop: with an exit test between the stages the compiler's wait-count pass sees a path from the middle of the
    // body back to its top on which the loads are outstanding in another order, and drains them all at the top (found
    // in the generated code: vmcnt(0) in front of every other k-step).  The scheduling barriers keep the loads in
    // front of the multiplication.
    if (kc_begin >= kc_end) return;
    static_assert(STAGES == 2, "the LDS buffers alternate with the register stages");
    TileRegs<LA, LB> r[STAGES];
#pragma unroll
    for (int s = 0; s < STAGES; ++s) load_tiles(r[s], min(kc_begin + s, kc_end - 1));
    int kc = kc_begin;
    auto stage = [&](TileRegs<LA, LB>& rs, const int buf, const bool prefetch) {
        store_tiles(rs, buf);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        if (prefetch) load_tiles(rs, min(kc + STAGES, kc_end - 1));
        __builtin_amdgcn_sched_barrier(0);
        multiply(buf);
        __builtin_amdgcn_sched_barrier(0);
        ++kc;
    };
    const int trips = (kc_end - kc_begin) / STAGES;
    for (int it = 0; it < trips; ++it) {
        stage(r[0], 0, true);
        stage(r[1], 1, true);
    }
    if ((kc_end - kc_begin) & 1) stage(r[0], 0, false);
}

// ---------------------------------------------------------------------------------------------------------------
// The same contraction for operands stored the other way round: the reduction index is the ROW index of both,
//   acc += A[k][m0 .. m0 + BM_) ^T * B[k][n0 .. n0 + BN_)      A: [K x lda], B: [K x ldb] row-major bf16,
// which is what a weight gradient is (dW = X^T dZ: both X and dZ have one row per node).  Tiles of 64 reduction
// rows are copied to LDS as they are; the fragment v_mfma_f32_32x32x16_bf16 wants (8 values along the reduction
// index per lane) comes out of LDS through ds_read_b64_tr_b16, the LDS transpose read of this architecture: in
// every group of 16 lanes, lane r passes the address of 4 consecutive 16-bit values (row r of a 16 x 4 block) and
// lane l receives column l % 4 of rows l / 4, l / 4 + 4, l / 4 + 8, l / 4 + 12 (layout established by a probe that
// reads a known pattern).  With lane r = 4 e + q pointing at [reduction row k_e][4 q-th .. of 16 consecutive
// columns], lane l of the group gets column l of those 16 at the reduction rows k_0 .. k_3: two such reads give a
// lane its 8 reduction values.  LDS rows are padded by 32 bytes so that the 4 reduction rows a group touches start
// in different banks (the pieces of neighbouring rows still overlap: the hardware counter reads a third of the LDS
// cycles as bank conflicts; the chunk permutation of mainloop_tn_direct below has none).  Rows >= k_rows and
// columns >= a_cols / b_cols are read as zero (no padding assumed).
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// ONES: where `do_ones` holds (the same for a whole wave), ones_acc[j] also accumulates a row of ones times B's
// fragments: every row of that 32 x 32 tile is the sum of B over the reduction range, column by column.
// B may come as two terms (b_terms = 2: the second BN_ columns start b_term_stride elements after the first): both
// are multiplied with the same A fragments into the same accumulators, i.e. the reduction runs over both terms, and
// A is read once for the two.  TERMS2 = false leaves out the second term's LDS (b_terms must be 1 then).
template <int BM_, int BN_, bool ONES = false, bool TERMS2 = false, int STAGES = 2>
__device__ __forceinline__ void mainloop_tn(const uint16_t* __restrict__ A, const int64_t lda, const int a_cols,
                                            const uint16_t* __restrict__ B, const int64_t ldb, const int b_cols,
                                            const int b_terms, const int64_t b_term_stride,
                                            const int m0, const int n0, const int kc_begin, const int kc_end,
                                            const int k_rows, f32x16 (&acc)[BM_ / 64][BN_ / 64],
                                            f32x16* ones_acc = nullptr, const bool do_ones = false)
{
    constexpr int MI = BM_ / 64, NJ = BN_ / 64;
    constexpr int CA = BM_ / 8, CB = BN_ / 8;            // 16-byte chunks per reduction row
    constexpr int LA = BK * CA / TPB, LB = BK * CB / TPB;
    constexpr int RSA = BM_ + 16, RSB = BN_ + 16;        // LDS row stride in elements (32 bytes of padding)
    __shared__ __attribute__((aligned(16))) uint16_t As[2][BK * RSA];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][TERMS2 ? 2 : 1][BK * RSB];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const bool two = TERMS2 && b_terms == 2;
    const int64_t term2_off = b_term_stride * (int64_t)(b_terms - 1);     // 0 with one term: the read repeats the first
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    if (ONES) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) ones_acc[j][e] = 0.f;
    }
    const s16x8 one_bits = {0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80};     // bf16 1.0
    const bf16x8 one8 = __builtin_bit_cast(bf16x8, one_bits);

    // Every load is issued without a branch (a chunk outside the operand reads its last row or last 8 columns
    // instead; zeros replace it when the tile goes to LDS, one k-step later): only then does the compiler know how
    // many loads are outstanding and lets the wait for one k-step's tiles pass while the next k-step's are in flight.
    auto load_tiles = [&](TileRegs<LA, 2 * LB>& r, int kc) {
        const int k0 = kc * BK;
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int id = t + TPB * i, kr = id / CA, c = id % CA;
            r.a[i] = *reinterpret_cast<const u32x4*>(A + (int64_t)min(k0 + kr, k_rows - 1) * lda + min(m0 + c * 8, a_cols - 8));
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int id = t + TPB * i, kr = id / CB, c = id % CB;
            const uint16_t* src = B + (int64_t)min(k0 + kr, k_rows - 1) * ldb + min(n0 + c * 8, b_cols - 8);
            r.b[i] = *reinterpret_cast<const u32x4*>(src);
            // with one term the second read repeats the first and is not used
            if (TERMS2) r.b[LB + i] = *reinterpret_cast<const u32x4*>(src + term2_off);
        }
    };
    auto store_tiles = [&](const TileRegs<LA, 2 * LB>& r, int buf, int kc) {
        const int k0 = kc * BK;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int id = t + TPB * i, kr = id / CA, c = id % CA;
            const bool ok = k0 + kr < k_rows && m0 + c * 8 < a_cols;
            *reinterpret_cast<u32x4*>(&As[buf][kr * RSA + c * 8]) = ok ? r.a[i] : zero;
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int id = t + TPB * i, kr = id / CB, c = id % CB;
            const bool ok = k0 + kr < k_rows && n0 + c * 8 < b_cols;
            *reinterpret_cast<u32x4*>(&Bs[buf][0][kr * RSB + c * 8]) = ok ? r.b[i] : zero;
            if (two) *reinterpret_cast<u32x4*>(&Bs[buf][TERMS2 ? 1 : 0][kr * RSB + c * 8]) = ok ? r.b[LB + i] : zero;
        }
    };
    // this lane's part of the address pattern: reduction row offset and column offset inside a 32-column fragment
    const int g = lane >> 4, r16 = lane & 15;
    const int frag_k = 8 * (g >> 1) + (r16 >> 2);        // + 4 for the second read
    const int frag_c = 16 * (g & 1) + 4 * (r16 & 3);
    auto read_frag = [&](const uint16_t* tile, int rs, int kb, int col0) -> bf16x8 {
        typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
        const uint16_t* p0 = tile + (kb + frag_k) * rs + col0 + frag_c;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p0);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0 + 4 * rs));
        const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, v);
    };
    // One k-step as straight-line code: the fragments of sub-step ks + 1 are requested before the matrix instructions
    // of sub-step ks are issued (two sets of fragment registers), so that the LDS reads run under the arithmetic.
    // WITH_ONES is a parameter of the whole k-step: a test of do_ones per sub-step would cut the code into basic
    // blocks, and the scheduler moves nothing across their ends.
    auto multiply_steps = [&](int buf, auto with_ones) {
        constexpr bool WITH_ONES = decltype(with_ones)::value;
        constexpr int KS = BK / 16;
        constexpr int READS = 2 * (MI + NJ) + (TERMS2 ? 2 * NJ : 0);          // ds_read_b64_tr_b16 per sub-step (upper bound with one term)
        constexpr int MMAS = MI * NJ + (WITH_ONES ? NJ : 0);
        bf16x8 fa[2][MI], fb[2][NJ], fb2[2][NJ];
        auto fetch = [&](int set, int ks) {
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[set][i] = read_frag(As[buf], RSA, ks * 16, wm * (BM_ / 2) + i * 32);
#pragma unroll
            for (int j = 0; j < NJ; ++j) fb[set][j] = read_frag(Bs[buf][0], RSB, ks * 16, wn * (BN_ / 2) + j * 32);
            if (two) {
#pragma unroll
                for (int j = 0; j < NJ; ++j) fb2[set][j] = read_frag(Bs[buf][TERMS2 ? 1 : 0], RSB, ks * 16, wn * (BN_ / 2) + j * 32);
            }
        };
        fetch(0, 0);
        if (!TERMS2) __builtin_amdgcn_sched_group_barrier(0x100, READS, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int set = ks & 1;
            if (ks + 1 < KS) fetch(set ^ 1, ks + 1);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
            if (WITH_ONES) {
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    ones_acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(one8, fb[set][j], ones_acc[j], 0, 0, 0);
            }
            if (two) {
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb2[set][j], acc[i][j], 0, 0, 0);
                if (WITH_ONES) {
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        ones_acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(one8, fb2[set][j], ones_acc[j], 0, 0, 0);
                }
            }
            if (!TERMS2) {
                if (ks + 1 < KS) __builtin_amdgcn_sched_group_barrier(0x100, READS, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, MMAS, 0);
            }
        }
    };
    auto multiply = [&](int buf) {
        if (ONES && do_ones) multiply_steps(buf, std::true_type{});
        else multiply_steps(buf, std::false_type{});
    };

    // unconditional prefetch, two register stages, straight-line loop body and scheduling barriers as in mainloop
    if (kc_begin >= kc_end) return;
    static_assert(STAGES == 2, "the LDS buffers alternate with the register stages");
    TileRegs<LA, 2 * LB> r[STAGES];
#pragma unroll
    for (int s = 0; s < STAGES; ++s) load_tiles(r[s], min(kc_begin + s, kc_end - 1));
    int kc = kc_begin;
    auto stage = [&](TileRegs<LA, 2 * LB>& rs, const int buf, const bool prefetch) {
        store_tiles(rs, buf, kc);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        if (prefetch) load_tiles(rs, min(kc + STAGES, kc_end - 1));
        __builtin_amdgcn_sched_barrier(0);
        multiply(buf);
        __builtin_amdgcn_sched_barrier(0);
        ++kc;
    };
    const int trips = (kc_end - kc_begin) / STAGES;
    for (int it = 0; it < trips; ++it) {
        stage(r[0], 0, true);
        stage(r[1], 1, true);
    }
    if ((kc_end - kc_begin) & 1) stage(r[0], 0, false);
}

// ---------------------------------------------------------------------------------------------------------------
// mainloop_tn for 128 x 128 tiles with the operand tiles sent from global memory straight into LDS
// (global_load_lds_dwordx4: a wave's 64 lanes fill 1 KB of LDS in lane order, no registers and no LDS store
// instruction in between; in mainloop_tn the stores of a tile and the wait for its registers are a third of the
// k-step).  The loads are inline assembly on purpose: told about them, the compiler waits for ALL outstanding ones in
// front of every LDS read; here the loop counts them (8 per wave and pair of 64-row tiles) and waits for its own tiles only.
//
// LDS image of a tile: BKD (64 or 32) reduction rows of 256 bytes, no padding; the 16-byte chunk c of row r sits at chunk
// position c ^ 4 (r & 3), so that the four reduction rows a group of 16 lanes reads (64 bytes each) fall into four
// different quarters of the 64 banks.  The permutation is applied on the global side: the lane that fills chunk
// position p of row r fetches chunk p ^ 4 (r & 3) of that row.
// NB buffers: the next NB - 1 tile pairs are in flight while one is multiplied; one barrier per tile pair.
// The last tile of the reduction, if only part of its rows exist, goes through registers (rows past the end
// become zeros).  Columns past a_cols / b_cols repeat the last 8 columns: they only reach output rows / columns
// that the caller does not store.
// (M0, which carries the LDS address, is no register the compiler allocates; it sets M0 itself right in front of
// any instruction of its own that reads it.)
__device__ __forceinline__ void load_to_lds16(const void* gsrc, const uint32_t lds_wave_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gsrc), "s"(lds_wave_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_direct_loads()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

template <bool ONES, int NB, int BKD = BK>
__device__ __forceinline__ void mainloop_tn_direct(const uint16_t* __restrict__ A, const int64_t lda, const int a_cols,
                                                   const uint16_t* __restrict__ B, const int64_t ldb, const int b_cols,
                                                   const int m0, const int n0, const int kc_begin, const int kc_end,
                                                   const int k_rows, f32x16 (&acc)[2][2],
                                                   f32x16* ones_acc = nullptr, const bool do_ones = false)
{
    constexpr int T = 128, MI = 2, NJ = 2;
    constexpr int CH = T / 8;                            // 16-byte chunks per reduction row
    constexpr int TILE_BYTES = BKD * T * 2;              // 16 KB with 64 reduction rows per tile, 8 KB with 32
    constexpr int BUF_BYTES = 2 * TILE_BYTES;            // A tile, then B tile
    constexpr int D = NB - 1;                            // k-steps of prefetch
    constexpr int LJ = BKD / 16;                         // direct loads per wave, operand and tile (16 rows per round of the 4 waves)
    constexpr int LOADS = 2 * LJ;                        // per wave and tile pair
    constexpr int SUB = BK / BKD;                        // tiles per k-step of the caller's count
    static_assert(BKD == 32 || BKD == 64, "rows per tile");
    static_assert(NB >= 2 && NB <= 4 && D * LOADS < 64, "outstanding loads must fit the wait counter");
    // The buffers are the kernel's dynamic LDS (NB * 32 KB, set at launch): with a static array of that size the
    // compiler knows that one workgroup fills a compute unit, hands the wave all 512 registers and then moves the
    // accumulators between the two register files in every k-step (seen in the generated code).
    extern __shared__ __attribute__((aligned(1024))) uint8_t S[];
    typedef __attribute__((address_space(3))) uint8_t* lds_bytes;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    if (ONES) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) ones_acc[j][e] = 0.f;
    }
    const s16x8 one_bits = {0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80};     // bf16 1.0
    const bf16x8 one8 = __builtin_bit_cast(bf16x8, one_bits);
    if (kc_begin >= kc_end) return;

    const uint32_t s_base = (uint32_t)(uintptr_t)(lds_bytes)S;
    // direct loads: instruction j of wave w fills the rows 4 q .. 4 q + 3 of a tile, q = 4 j + w; lane L fills chunk
    // position L & 15 of row 4 q + (L >> 4) and therefore fetches chunk (L & 15) ^ 4 (L >> 4) of it
    const int rowl = lane >> 4, chunk = (lane & 15) ^ (4 * rowl);
    const uint16_t* a_src = A + (int64_t)(4 * wave + rowl) * lda + min(m0 + chunk * 8, a_cols - 8);
    const uint16_t* b_src = B + (int64_t)(4 * wave + rowl) * ldb + min(n0 + chunk * 8, b_cols - 8);
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(s_base + 1024u * (uint32_t)wave);
    const int h_begin = kc_begin * SUB, h_end = min(kc_end * SUB, (k_rows + BKD - 1) / BKD);   // tiles of BKD rows
    const int h_full_end = min(h_end, k_rows / BKD);     // tiles whose rows all exist
    auto issue = [&](int h, int buf) {                   // h: a tile with all rows (the caller clamps)
        const uint16_t* pa = a_src + (int64_t)h * BKD * lda;
        const uint16_t* pb = b_src + (int64_t)h * BKD * ldb;
#pragma unroll
        for (int j = 0; j < LJ; ++j) load_to_lds16(pa + (int64_t)(16 * j) * lda, wave_lds + buf * BUF_BYTES + 4096 * j);
#pragma unroll
        for (int j = 0; j < LJ; ++j) load_to_lds16(pb + (int64_t)(16 * j) * ldb, wave_lds + buf * BUF_BYTES + TILE_BYTES + 4096 * j);
    };

    // fragment reads (see mainloop_tn): this lane's reduction row and 8-byte piece inside a 32-column fragment
    const int g = lane >> 4, r16 = lane & 15;
    const int frag_k = 8 * (g >> 1) + (r16 >> 2);        // + 4 for the second read
    const int frag_c = 16 * (g & 1) + 4 * (r16 & 3);     // column inside the fragment, a multiple of 4
    const int x4 = 4 * (frag_k & 3);                     // this lane's rows all have the same r & 3
    uint32_t a_off[MI], b_off[NJ];                       // byte offsets inside a buffer for reduction row frag_k
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int col = wm * 64 + i * 32 + frag_c;
        a_off[i] = frag_k * (T * 2) + (((col >> 3) ^ x4) << 4) + ((col & 7) << 1);
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = wn * 64 + j * 32 + frag_c;
        b_off[j] = TILE_BYTES + frag_k * (T * 2) + (((col >> 3) ^ x4) << 4) + ((col & 7) << 1);
    }
    auto read_frag = [&](lds_bytes p, int ks) -> bf16x8 {
        typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + ks * 16 * (T * 2)));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + ks * 16 * (T * 2) + 4 * (T * 2)));
        const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, v);
    };
    auto multiply_steps = [&](int buf, auto with_ones) {
        constexpr bool WITH_ONES = decltype(with_ones)::value;
        constexpr int KS = BKD / 16;
        constexpr int READS = 2 * (MI + NJ);
        constexpr int MMAS = MI * NJ + (WITH_ONES ? NJ : 0);
        lds_bytes pa[MI], pb[NJ];
#pragma unroll
        for (int i = 0; i < MI; ++i) pa[i] = (lds_bytes)S + buf * BUF_BYTES + a_off[i];
#pragma unroll
        for (int j = 0; j < NJ; ++j) pb[j] = (lds_bytes)S + buf * BUF_BYTES + b_off[j];
        bf16x8 fa[2][MI], fb[2][NJ];
        auto fetch = [&](int set, int ks) {
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[set][i] = read_frag(pa[i], ks);
#pragma unroll
            for (int j = 0; j < NJ; ++j) fb[set][j] = read_frag(pb[j], ks);
        };
        fetch(0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, READS, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int set = ks & 1;
            if (ks + 1 < KS) fetch(set ^ 1, ks + 1);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
            if (WITH_ONES) {
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    ones_acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(one8, fb[set][j], ones_acc[j], 0, 0, 0);
            }
            if (ks + 1 < KS) __builtin_amdgcn_sched_group_barrier(0x100, READS, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, MMAS, 0);
        }
    };
    auto multiply = [&](int buf) {
        if (ONES && do_ones) multiply_steps(buf, std::true_type{});
        else multiply_steps(buf, std::false_type{});
    };

    const int n_full = h_full_end - h_begin;             // may be <= 0: the split is the partial tile alone
    if (n_full > 0) {
#pragma unroll
        for (int s = 0; s < D; ++s) issue(min(h_begin + s, h_full_end - 1), s);
        int buf = 0, pre = D;                            // buffer of this tile, buffer the prefetch goes to
        for (int k = 0; k < n_full; ++k) {
            wait_direct_loads<(D - 1) * LOADS>();        // this tile pair is in LDS (this wave's part)
            __syncthreads();                             // everybody's part; and buffer `pre` has been read by all
            __builtin_amdgcn_sched_barrier(0);
            issue(min(h_begin + k + D, h_full_end - 1), pre);
            __builtin_amdgcn_sched_barrier(0);
            multiply(buf);
            __builtin_amdgcn_sched_barrier(0);
            buf = buf + 1 == NB ? 0 : buf + 1;
            pre = pre + 1 == NB ? 0 : pre + 1;
        }
        wait_direct_loads<0>();                          // the surplus prefetches: nothing may land after this point
    }
    if (h_end > h_full_end) {
        // the partial tile: through registers into buffer 0, rows past the end as zeros
        const int k0 = h_full_end * BKD;
        u32x4 ra[LJ], rb[LJ];
#pragma unroll
        for (int j = 0; j < LJ; ++j) {
            const int row = 16 * j + 4 * wave + rowl;
            ra[j] = *reinterpret_cast<const u32x4*>(a_src + ((int64_t)min(k0 + row, k_rows - 1) - (4 * wave + rowl)) * lda);
            rb[j] = *reinterpret_cast<const u32x4*>(b_src + ((int64_t)min(k0 + row, k_rows - 1) - (4 * wave + rowl)) * ldb);
        }
        __syncthreads();                                 // all waves are done with buffer 0 and with their direct loads
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < LJ; ++j) {
            const int row = 16 * j + 4 * wave + rowl;
            const bool ok = k0 + row < k_rows;
            u32x4* dst_a = reinterpret_cast<u32x4*>(S + row * (T * 2) + (lane & 15) * 16);
            u32x4* dst_b = reinterpret_cast<u32x4*>(S + TILE_BYTES + row * (T * 2) + (lane & 15) * 16);
            *dst_a = ok ? ra[j] : zero;
            *dst_b = ok ? rb[j] : zero;
        }
        __syncthreads();
        multiply(0);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// mainloop with the operand tiles loaded from global memory straight into LDS (see mainloop_tn_direct for the
// instruction and why it is inline assembly).  The LDS image is mainloop's: 16-byte chunk c of tile row r at
// slot(r, c); a wave's load fills 8 consecutive rows, so the lane that fills chunk position p of row r fetches
// chunk p ^ ((r >> 1) & 7) of that row.  NB buffers in the kernel's dynamic LDS (NB * (BM_ + BN_) * 128 bytes),
// NB - 1 k-steps of tiles in flight, one barrier per k-step.  For long reductions: with few k-steps the two
// register stages of mainloop, which start two tiles at once, are ahead.
template <int BM_, int BN_, int NB>
__device__ __forceinline__ void mainloop_direct(const uint16_t* __restrict__ A_tile, const int64_t lda,
                                                const uint16_t* __restrict__ B_tile, const int64_t ldb,
                                                const int kc_begin, const int kc_end, f32x16 (&acc)[BM_ / 64][BN_ / 64])
{
    constexpr int MI = BM_ / 64, NJ = BN_ / 64;
    constexpr int A_BYTES = BM_ * BK * 2, B_BYTES = BN_ * BK * 2, BUF_BYTES = A_BYTES + B_BYTES;
    constexpr int JA = BM_ / 32, JB = BN_ / 32;          // direct loads per wave and k-step: 32 tile rows per round of the 4 waves
    constexpr int LOADS = JA + JB, D = NB - 1;
    static_assert(NB >= 2 && NB <= 4 && D * LOADS < 64, "outstanding loads must fit the wait counter");
    extern __shared__ __attribute__((aligned(1024))) uint8_t S[];
    typedef __attribute__((address_space(3))) uint8_t* lds_bytes;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    if (kc_begin >= kc_end) return;

    // this lane's row inside a round of 32 rows, and the chunk it fetches for chunk position lane & 7
    // ((row >> 1) & 7 of row 32 j + 8 wave + (lane >> 3) does not depend on j)
    const int r8 = lane >> 3;
    const int swz = (4 * (wave & 1) + (r8 >> 1)) & 7;
    const int chunk = (lane & 7) ^ swz;
    const uint16_t* a_src = A_tile + (int64_t)(8 * wave + r8) * lda + chunk * 8;
    const uint16_t* b_src = B_tile + (int64_t)(8 * wave + r8) * ldb + chunk * 8;
    const uint32_t s_base = (uint32_t)(uintptr_t)(lds_bytes)S;
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(s_base + 1024u * (uint32_t)wave);
    auto issue = [&](int kc, int buf) {
        const uint16_t* pa = a_src + (int64_t)kc * BK;
        const uint16_t* pb = b_src + (int64_t)kc * BK;
#pragma unroll
        for (int j = 0; j < JA; ++j) load_to_lds16(pa + (int64_t)(32 * j) * lda, wave_lds + buf * BUF_BYTES + 4096 * j);
#pragma unroll
        for (int j = 0; j < JB; ++j) load_to_lds16(pb + (int64_t)(32 * j) * ldb, wave_lds + buf * BUF_BYTES + A_BYTES + 4096 * j);
    };
    constexpr int KG = (MI * NJ == 1) ? 4 : 2;
    auto multiply = [&](int buf) {
        const u32x4* As = reinterpret_cast<const u32x4*>(S + buf * BUF_BYTES);
        const u32x4* Bs = reinterpret_cast<const u32x4*>(S + buf * BUF_BYTES + A_BYTES);
#pragma unroll
        for (int k0 = 0; k0 < BK / 16; k0 += KG) {
            bf16x8 fa[KG][MI], fb[KG][NJ];
#pragma unroll
            for (int kk = 0; kk < KG; ++kk) {
                const int c = 2 * (k0 + kk) + (lane >> 5);
#pragma unroll
                for (int i = 0; i < MI; ++i)
                    fa[kk][i] = __builtin_bit_cast(bf16x8, As[slot(wm * (BM_ / 2) + i * 32 + (lane & 31), c)]);
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    fb[kk][j] = __builtin_bit_cast(bf16x8, Bs[slot(wn * (BN_ / 2) + j * 32 + (lane & 31), c)]);
            }
#pragma unroll
            for (int kk = 0; kk < KG; ++kk)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk][i], fb[kk][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, KG * (MI + NJ), 0);
            __builtin_amdgcn_sched_group_barrier(0x008, KG * MI * NJ, 0);
        }
    };
    const int n_steps = kc_end - kc_begin;
#pragma unroll
    for (int s = 0; s < D; ++s) issue(min(kc_begin + s, kc_end - 1), s);
    int buf = 0, pre = D;
    for (int k = 0; k < n_steps; ++k) {
        wait_direct_loads<(D - 1) * LOADS>();            // this k-step's tiles are in LDS (this wave's part)
        __syncthreads();                                 // everybody's part; and buffer `pre` has been read by all
        __builtin_amdgcn_sched_barrier(0);
        issue(min(kc_begin + k + D, kc_end - 1), pre);
        __builtin_amdgcn_sched_barrier(0);
        multiply(buf);
        __builtin_amdgcn_sched_barrier(0);
        buf = buf + 1 == NB ? 0 : buf + 1;
        pre = pre + 1 == NB ? 0 : pre + 1;
    }
    wait_direct_loads<0>();                              // the surplus prefetches: nothing may land after this point
}

}  // namespace dn_mma
