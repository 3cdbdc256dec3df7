// One GraphSage layer above the first in one launch (Algorithm 3 of the paper, mean or sum variant, followed by
// the layer's linear map, bias and ReLU): a workgroup owns 16 output rows and ALL output columns.
//
//   phase 1  its 8 waves gather two rows each: the row's own representation and the mean (fp32 sum in ascending
//            slot order, fp32 division) of the rows its slots select through repr_map.  Both are split into two
//            bf16 terms and laid out as the row of the A operand  [ self_hi | mean_hi | self_lo | mean_lo ]  in
//            LDS, and written to X in memory for the weight gradient of the backward pass;
//   phase 2  wave w multiplies the 16 x 4d tile with columns [32 w, 32 w + 32) of the weights on
//            v_mfma_f32_16x16x32_bf16.  The B fragments go from memory straight into registers: the weights are kept
//            a second time in fragment order (dn_layer_bufs::wf: for every 16 columns and 32 reduction elements the
//            64 lanes' 16 bytes side by side), so that one load instruction of a wave reads 1 KB of consecutive
//            memory; read from the row-major copy the same instruction touches 16 to 64 cache lines, and the
//            compute unit's cache, which takes a line per clock, was what the kernel waited for (6 of its 13 us).
//            Every workgroup reads all of them and the L2 keeps them.  Both bf16 terms of A meet the same B fragment;
//   phase 3  bias, ReLU, store; pre-activations too close to zero for the fp32 accumulation to settle their sign are
//            queued and recomputed in fp64 from the tile in LDS (as the stand-alone GEMM does from memory).
//
// Layers above the first have few rows per mini-batch (a few thousand) and a reduction of 4 d_in: as two launches
// (aggregation, then a GEMM of 64 x 64 tiles with 16 dependent k-steps) they took 8 + 14 us and 4 + 10 us at the
// 111M-node workload, nearly all of it latency.  Here every memory access of the layer is issued by the workgroup
// that needs it, with as many in flight as registers allow, and 16-row tiles spread a layer over 2.5 to 10 times as
// many compute units.
#include "dn_internal.h"
#include <cstdlib>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int FT = 512;            // threads per workgroup (8 waves)
constexpr int FR = 16;             // output rows per workgroup
constexpr int FIX_CAP = 256;       // sign fix-ups one workgroup can queue (a sixteenth of a 16 x 256 tile)
constexpr int GB = 16;             // neighbour rows in flight per output row

struct FusedArgs {
    const int32_t* hdr; int layer;
    const int32_t* nbr_offsets; const int32_t* repr_map; int64_t slot_cap;   // slot_cap: allocated entries of repr_map (>= 1)
    const float* H; int64_t ldh;            // input rows H^{i-1}: row 0 = node_ids position node_id_offsets[i-1]
    const float* zero_row;                   // at least 256 zeros
    int mean_agg;
    uint16_t* X; int kp; float* rownorm;     // A operand and its row norms, kept for the backward pass
    const uint16_t* wt;                      // Wcat^T, bf16 [>= np x kp]; columns [0, 2d) are used (exact pass)
    const uint16_t* wf;                      // the same in fragment order (see dn_layer_bufs::wf)
    const float* bias; int d_out; int np;    // np = d_out rounded up to 64, <= 256
    float* C; int64_t ldc; int relu;
    const float* colnorm; float gamma; int32_t* fix_count;
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// two fp32 -> two bfloat16 (round to nearest even) in one v_cvt_pk_bf16_f32: x in the low half
__device__ __forceinline__ uint32_t cvt2(float x, float y)
{
    const f32x2 v = {x, y};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// four values as two bf16 terms: hi = bf16(v), lo = bf16(v - hi); adds the squares of the eight terms to sq
__device__ __forceinline__ void split4(const float (&v)[4], uint2& hi, uint2& lo, float& sq)
{
    hi = make_uint2(cvt2(v[0], v[1]), cvt2(v[2], v[3]));
    const float h[4] = {__uint_as_float(hi.x << 16), __uint_as_float(hi.x & 0xffff0000u),
                        __uint_as_float(hi.y << 16), __uint_as_float(hi.y & 0xffff0000u)};
    lo = make_uint2(cvt2(v[0] - h[0], v[1] - h[1]), cvt2(v[2] - h[2], v[3] - h[3]));
    const float l[4] = {__uint_as_float(lo.x << 16), __uint_as_float(lo.x & 0xffff0000u),
                        __uint_as_float(lo.y << 16), __uint_as_float(lo.y & 0xffff0000u)};
#pragma unroll
    for (int e = 0; e < 4; ++e) sq += h[e] * h[e] + l[e] * l[e];
}

// S = d_in / 64 (1..4): the reduction over [self | mean] has 2 d_in = 128 S elements per term.  LAYER_TAG only gives
// every layer's launch a kernel symbol of its own, so that a profiler's per-kernel statistics do not mix the layers
// (2, 3, and 4 for "layer 4 and above").
template <int S, int LAYER_TAG>
__global__ __launch_bounds__(FT) void k_sage_layer(FusedArgs a)
{
    constexpr int D = 64 * S;
    constexpr int ROW_BYTES = 8 * D + 16;          // 4 D bf16 + 16: rows r, r + 1 start 16 bytes apart modulo 256
    __shared__ __attribute__((aligned(16))) unsigned char A_lds[FR * ROW_BYTES];
    __shared__ float s_rownorm[FR];
    __shared__ int s_fix_n;
    __shared__ int s_fix[FIX_CAP];

    const int N = a.hdr[HDR_N];
    const int off_in = a.hdr[HDR_NODE_OFF + a.layer - 1];
    const int off_out = a.hdr[HDR_NODE_OFF + a.layer];
    const int off1 = a.hdr[HDR_NODE_OFF + 1];
    const int rows = N - off_out;
    const int row0 = blockIdx.x * FR;
    if (row0 >= rows) return;                      // grid sized by capacity: the surplus leaves at once
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    if (t == 0) s_fix_n = 0;

    const bool mm_wave = 32 * wave < a.np;
    const int lr = lane & 15, lg = lane >> 4;
    // fragment (column tile T, reduction step st) starts at element ((T * 4S + st) * 64) * 8; a wave without output
    // columns fetches wave 0's fragments and drops them (no branch, no register reuse to wait for)
    const uint16_t* brow[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) brow[j] = a.wf + ((int64_t)((mm_wave ? 2 * wave : 0) + j) * (4 * S) * 64 + lane) * 8;
    bf16x8 Bf[S][2][4];
    constexpr int S_EARLY = (S + 1) / 2;
    // what the epilogue needs of bias and column norms, requested before everything else
    float e_bias[2], e_cn[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = min(32 * wave + 16 * j + lr, a.d_out - 1);
        e_bias[j] = a.bias[n];
        e_cn[j] = a.colnorm[n];
    }

    // ---- phase 1: rows 2 wave, 2 wave + 1 of the tile; lane takes columns 4 lane .. 4 lane + 3.
    // Loads come back in the order they were issued, so the short dependent ones go first (segment bounds, slot
    // lists), then the rows, and the B fragments behind them.
    {
        const int c0 = 4 * lane;
        const bool col_ok = c0 < D;
        const int cc = col_ok ? c0 : 0;            // lanes beyond the row read its first columns and drop them
        const int ro0 = row0 + 2 * wave;
        const int last_q = N - off1;               // nbr_offsets has last_q + 1 entries
        const int q0 = off_out + ro0 - off1;
        int beg[2], end[2], cnt[2];
        bool live[2];
        {
            const int o0 = __builtin_amdgcn_readfirstlane(a.nbr_offsets[min(q0, last_q)]);
            const int o1 = __builtin_amdgcn_readfirstlane(a.nbr_offsets[min(q0 + 1, last_q)]);
            const int o2 = __builtin_amdgcn_readfirstlane(a.nbr_offsets[min(q0 + 2, last_q)]);
            beg[0] = o0; end[0] = o1; beg[1] = o1; end[1] = o2;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            live[j] = ro0 + j < rows;
            if (!live[j]) { beg[j] = 0; end[j] = 0; }
            cnt[j] = min(64, end[j] - beg[j]);
        }
        // both rows' slot lists are requested before either is waited for: every lane reads (an index past the row's
        // slots is clamped into the array and its value dropped)
        int fetched[2], idx[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) fetched[j] = a.repr_map[min((int64_t)beg[j] + lane, a.slot_cap - 1)];
        float4 sv[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t self_row = live[j] ? (int64_t)(off_out + ro0 + j - off_in) : 0;
            sv[j] = *reinterpret_cast<const float4*>(a.H + self_row * a.ldh + cc);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) idx[j] = lane < cnt[j] ? fetched[j] - off_in : 0;
        // the first GB slots of both rows are fetched together; a slot that does not exist reads zeros (all lanes the
        // same 16 bytes: one cache line for the wave), so that every fetched value is added without a branch.  The row
        // number of a slot is the same for the whole wave: a scalar
        float4 v[2][GB];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const int ru = __builtin_amdgcn_readlane(idx[j], max(min(u, cnt[j] - 1), 0));
                const bool real = u < cnt[j];
                const float* src = real ? a.H + (int64_t)ru * a.ldh : a.zero_row;
                v[j][u] = *reinterpret_cast<const float4*>(src + (real ? cc : 0));
            }
        // B fragments of the first half of the reduction: in flight while the rows are summed
#pragma unroll
        for (int ss = 0; ss < S_EARLY; ++ss)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int s = 0; s < 4; ++s) Bf[ss][j][s] = *reinterpret_cast<const bf16x8*>(brow[j] + (4 * ss + s) * 512);
        float acc[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][e] = 0.f;
#pragma unroll
            for (int u = 0; u < GB; ++u) { acc[j][0] += v[j][u].x; acc[j][1] += v[j][u].y; acc[j][2] += v[j][u].z; acc[j][3] += v[j][u].w; }
        }
        // rows with more slots than that: the rest of the first 64, then further chunks of 64, eight rows in flight
        auto more_slots = [&](const int rbeg, const int rend, const int first_rows, float (&sum)[4]) {
            for (int base = rbeg; base < rend; base += 64) {
                int row = first_rows;
                if (base != rbeg) { const int tt = base + lane; row = tt < rend ? a.repr_map[tt] - off_in : 0; }
                const int c = min(64, rend - base);
                for (int l = (base == rbeg) ? GB : 0; l < c; l += 8) {
                    float4 w[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int ru = __builtin_amdgcn_readlane(row, min(l + u, c - 1));
                        w[u] = *reinterpret_cast<const float4*>(a.H + (int64_t)ru * a.ldh + cc);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (l + u < c) { sum[0] += w[u].x; sum[1] += w[u].y; sum[2] += w[u].z; sum[3] += w[u].w; }
                }
            }
        };
        if (end[0] - beg[0] > GB) more_slots(beg[0], end[0], idx[0], acc[0]);
        if (end[1] - beg[1] > GB) more_slots(beg[1], end[1], idx[1], acc[1]);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int r = 2 * wave + j;
            const int n_slots = end[j] - beg[j];
            const float cnt_f = (float)n_slots;
            float sval[4] = {sv[j].x, sv[j].y, sv[j].z, sv[j].w}, mean[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (!live[j]) sval[e] = 0.f;
                mean[e] = n_slots > 0 ? (a.mean_agg ? acc[j][e] / cnt_f : acc[j][e]) : 0.f;
            }
            uint2 p_sh, p_sl, p_mh, p_ml;
            float sq = 0.f;
            split4(sval, p_sh, p_sl, sq);
            split4(mean, p_mh, p_ml, sq);
            if (!col_ok) sq = 0.f;
#pragma unroll
            for (int o2 = 32; o2 > 0; o2 >>= 1) sq += __shfl_xor(sq, o2);
            if (col_ok) {
                unsigned char* lrow = A_lds + r * ROW_BYTES + 2 * c0;
                *reinterpret_cast<uint2*>(lrow) = p_sh;
                *reinterpret_cast<uint2*>(lrow + 2 * D) = p_mh;
                *reinterpret_cast<uint2*>(lrow + 4 * D) = p_sl;
                *reinterpret_cast<uint2*>(lrow + 6 * D) = p_ml;
                if (live[j]) {
                    uint16_t* xrow = a.X + (int64_t)(ro0 + j) * a.kp + c0;
                    *reinterpret_cast<uint2*>(xrow) = p_sh;
                    *reinterpret_cast<uint2*>(xrow + D) = p_mh;
                    *reinterpret_cast<uint2*>(xrow + 2 * D) = p_sl;
                    *reinterpret_cast<uint2*>(xrow + 3 * D) = p_ml;
                }
            }
            if (lane == 0) {
                const float nrm = sqrtf(sq) * 1.0001f;
                s_rownorm[r] = nrm;
                if (live[j]) a.rownorm[ro0 + j] = nrm;
            }
        }
    }
    // ---- the other half of the B fragments, then the tile is complete
#pragma unroll
    for (int ss = S_EARLY; ss < S; ++ss)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int s = 0; s < 4; ++s) Bf[ss][j][s] = *reinterpret_cast<const bf16x8*>(brow[j] + (4 * ss + s) * 512);
    __syncthreads();

    // ---- phase 2: 16 x 32 outputs per wave; hi and lo terms accumulate apart (four independent MFMA chains)
    if (mm_wave) {
        f32x4 acc_hi[2], acc_lo[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) { acc_hi[j] = f32x4{0.f, 0.f, 0.f, 0.f}; acc_lo[j] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        const unsigned char* arow = A_lds + lr * ROW_BYTES + 16 * lg;      // lane group lg: elements 8 lg .. 8 lg + 7 of a step's 32
#pragma unroll
        for (int ss = 0; ss < S; ++ss)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 a_hi = *reinterpret_cast<const bf16x8*>(arow + 64 * (4 * ss + s));
                const bf16x8 a_lo = *reinterpret_cast<const bf16x8*>(arow + 4 * D + 64 * (4 * ss + s));
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc_hi[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, Bf[ss][j][s], acc_hi[j], 0, 0, 0);
                    acc_lo[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, Bf[ss][j][s], acc_lo[j], 0, 0, 0);
                }
            }
        // ---- phase 3: register e of lane holds row 4 (lane / 16) + e, column 32 wave + 16 j + lane % 16
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = 32 * wave + 16 * j + lr;
            if (n >= a.d_out) continue;
            const float bv = e_bias[j];
            const float cn = a.relu ? a.gamma * e_cn[j] : 0.f;
            const float bt = fabsf(bv) * 4.76837158e-7f;          // 2^-21 |b|: rounding of the bias add
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r = 4 * lg + e;
                if (row0 + r >= rows) continue;
                float z = (acc_hi[j][e] + acc_lo[j][e]) + bv;
                if (a.relu) {
                    if (fabsf(z) <= cn * s_rownorm[r] + bt) {
                        const int lp = atomicAdd(&s_fix_n, 1);
                        if (lp < FIX_CAP) s_fix[lp] = (r << 16) | n;
                    }
                    z = fmaxf(z, 0.f);
                }
                a.C[(int64_t)(row0 + r) * a.ldc + n] = z;
            }
        }
    }
    if (!a.relu) return;
    // ---- exact pass: 16 lanes per queued element recompute Z in fp64 (products of bf16 values are exact there)
    __syncthreads();
    const int queued = s_fix_n;
    const int n_fix = min(queued, FIX_CAP);
    if (t == 0 && queued > 0) {
        atomicAdd(&a.fix_count[DN_FIX_FIRST + DN_FIX_STRIDE * (blockIdx.x % DN_FIX_SLOTS)], n_fix);
        if (queued > FIX_CAP) a.fix_count[1] = 1;                // surplus keeps its fp32 sign
    }
    const int sub = t >> 4, sl = t & 15;
    for (int qi = sub; qi < n_fix; qi += FT / 16) {
        const int ent = s_fix[qi];
        const int r = ent >> 16, n = ent & 0xffff;
        const unsigned char* xr = A_lds + r * ROW_BYTES;
        const uint16_t* wr = a.wt + (int64_t)n * a.kp;
        double sum = 0.0;
        for (int c = sl; c < 2 * D / 8; c += 16) {
            const u32x4 xh = *reinterpret_cast<const u32x4*>(xr + 16 * c);
            const u32x4 xl = *reinterpret_cast<const u32x4*>(xr + 4 * D + 16 * c);
            const u32x4 wv = *reinterpret_cast<const u32x4*>(wr + 8 * c);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double w0 = (double)__uint_as_float(wv[e] << 16), w1 = (double)__uint_as_float(wv[e] & 0xffff0000u);
                sum += (double)__uint_as_float(xh[e] << 16) * w0;
                sum += (double)__uint_as_float(xh[e] & 0xffff0000u) * w1;
                sum += (double)__uint_as_float(xl[e] << 16) * w0;
                sum += (double)__uint_as_float(xl[e] & 0xffff0000u) * w1;
            }
        }
        for (int dd = 8; dd > 0; dd >>= 1) sum += __shfl_down(sum, dd, 16);
        if (sl == 0) {
            const double z = sum + (double)a.bias[n];
            a.C[(int64_t)(row0 + r) * a.ldc + n] = (float)(z > 0.0 ? z : 0.0);
        }
    }
}

bool fused_enabled()
{
    static const bool on = [] { const char* e = getenv("DN_FUSED_LAYERS"); return !(e && e[0] == '0'); }();
    return on;
}

}  // namespace

// True if layer i (1-based) of the model runs as the single launch above: two-term activations of 64, 128, 192 or
// 256 columns and at most 256 output columns.  DN_FUSED_LAYERS=0 in the environment (read once) turns it off.
bool dn_layer_is_fused(const dn_model* m, int i)
{
    if (i < 2 || !fused_enabled()) return false;
    const dn_layer_bufs& L = m->layer[i - 1];
    return L.xterms == 2 && L.d_in % 64 == 0 && L.d_in <= 256 && L.np <= 256 && L.kp == 4 * L.d_in;
}

int dn_launch_layer_fused(const dn_model* m, const dn_batch* b, int i, float* out, int64_t ldc, hipStream_t st)
{
    const dn_layer_bufs& L = m->layer[i - 1];
    FusedArgs a{};
    a.hdr = b->hdr; a.layer = i;
    a.nbr_offsets = b->nbr_offsets; a.repr_map = b->repr_map; a.slot_cap = b->cap_slots > 0 ? b->cap_slots : 1;
    a.H = m->layer[i - 2].h; a.ldh = L.d_in;
    a.zero_row = m->zero_row;
    a.mean_agg = m->mean_agg;
    a.X = reinterpret_cast<uint16_t*>(L.x); a.kp = L.kp; a.rownorm = L.rownorm;
    a.wt = reinterpret_cast<const uint16_t*>(L.wt);
    a.wf = reinterpret_cast<const uint16_t*>(L.wf);
    a.bias = L.bias; a.d_out = L.d_out; a.np = L.np;
    a.C = out; a.ldc = ldc; a.relu = (i < m->k) ? 1 : 0;
    a.colnorm = L.colnorm;
    a.gamma = 8.0f * sqrtf((float)L.kp) * 5.9604645e-8f;       // as dn_gemm_forward: 8 sqrt(K) 2^-24
    a.fix_count = m->fix_count;
    int64_t grid = (L.rows_cap + FR - 1) / FR;
    if (grid < 1) grid = 1;
    dn_prof_scope ps("sage_layer", i, st);
#define FUSED_LAUNCH(SS, TAG) hipLaunchKernelGGL((k_sage_layer<SS, TAG>), dim3((unsigned)grid), dim3(FT), 0, st, a)
#define FUSED_LAUNCH_S(SS) do { if (i == 2) FUSED_LAUNCH(SS, 2); else if (i == 3) FUSED_LAUNCH(SS, 3); else FUSED_LAUNCH(SS, 4); } while (0)
    switch (L.d_in / 64) {
        case 1: FUSED_LAUNCH_S(1); break;
        case 2: FUSED_LAUNCH_S(2); break;
        case 3: FUSED_LAUNCH_S(3); break;
        default: FUSED_LAUNCH_S(4); break;
    }
#undef FUSED_LAUNCH_S
#undef FUSED_LAUNCH
    DN_LAUNCH_CHECK("k_sage_layer");
    return DN_OK;
}
