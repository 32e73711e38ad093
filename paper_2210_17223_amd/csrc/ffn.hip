// Expert FFN (paper Sec. 2.1: every expert is a two-layer fully connected network)
// as two grouped GEMMs over the expert-major buffer:
//   H  = act(xe . W1[e] + b1[e])      rows of expert e only
//   ye = H . W2[e] + b2[e]
// Row ranges per expert are known only on the device; the kernels take them from a
// table of row tiles (plan_tiles) and the grid is sized for the worst case, surplus
// blocks exit at once.
//
// bf16 layers: MFMA 32x32x16 tiles.  Both operands are stored with the contraction
// index contiguous (activations by nature, weights after moe_pack_weights), staged
// through LDS in 64-deep stages, and the weight tile is fed as the MFMA "A" operand
// so that each lane ends up with four consecutive output columns of one row.
// grouped_gemm_w4_kernel runs the 256 x 256 output tiles of the large layers,
// grouped_gemm_mfma_kernel the smaller tile shapes.  H and ye are kept in fp16.
// fp32 layers: a plain LDS-tiled vector-ALU GEMM (correctness configuration).
#include "common.h"
#include <cstdio>

#include <hip/hip_ext.h>

#include <type_traits>

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// ---------------------------------------------------------------- activations
// GeLU(v) = v Phi(v) with Phi(v) ~ 1 / (1 + 2^(v Q(min(v^2, 49)))), Q a cubic fitted (minimax
// on |v| <= 7, both signs) to the logit of the normal CDF; the coefficients carry the factor
// -log2(e).  Absolute error of GeLU below 1.5e-5 everywhere, i.e. a few per cent of the fp16
// rounding of the hidden activation it feeds; two transcendental and eight plain
// instructions per element.
__device__ __forceinline__ float gelu_erf_fast(float v)
{
    const float s = fminf(v * v, 49.0f);
    float q = 2.1637799e-05f;
    q = __builtin_fmaf(q, s, 7.7587553e-04f);
    q = __builtin_fmaf(q, s, -1.0610976e-01f);
    q = __builtin_fmaf(q, s, -2.3015507e+00f);
    const float e = __builtin_amdgcn_exp2f(v * q);
    return v * __builtin_amdgcn_rcpf(1.0f + e);
}

template <int ACT, bool FAST>
__device__ __forceinline__ float activate(float v)
{
    if constexpr (ACT == MOE_ACT_GELU_ERF) {
        if constexpr (FAST) return gelu_erf_fast(v);
        return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));
    } else if constexpr (ACT == MOE_ACT_GELU_TANH) {
        return 0.5f * v * (1.0f + tanhf(0.7978845608028654f * (v + 0.044715f * v * v * v)));
    } else if constexpr (ACT == MOE_ACT_RELU) {
        return fmaxf(v, 0.0f);
    } else {
        return v;
    }
}

// ---------------------------------------------------------------- fp32 GEMM
// C[r, n] = act(sum_k A[r,k] B[e][k,n] + bias[e][n]); B canonical [E, K, N].
constexpr int kF32Tile = 64;
constexpr int kF32BK = 16;

template <int ACT>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(
    const float *__restrict__ A, const float *__restrict__ B, const float *__restrict__ bias,
    float *__restrict__ C, const WorkItem *__restrict__ items,
    const int32_t *__restrict__ nitems, int N, int K)
{
    if (static_cast<int>(blockIdx.x) >= *nitems) return;
    const WorkItem tile = items[blockIdx.x];
    const int n0 = tile.n0;

    __shared__ float As[kF32BK][kF32Tile + 4];
    __shared__ float Bs[kF32BK][kF32Tile + 4];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    float acc[4][4] = {};

    const int a_row = tid / 4, a_k = (tid % 4) * 4;
    const int a_row_g = min(tile.row0 + a_row, tile.row1 - 1);
    const int b_k = tid / 16, b_n = (tid % 16) * 4;
    const float *Bexp = B + static_cast<size_t>(tile.expert) * K * N;

    // the loads of stage k0 + 16 are in flight while stage k0 is multiplied
    float4 av, bv;
#define MOE_F32_LOAD(k0_)                                                                        \
    {                                                                                            \
        av = make_float4(0.f, 0.f, 0.f, 0.f);                                                    \
        bv = av;                                                                                 \
        if ((k0_) + a_k < K)                                                                     \
            av = *reinterpret_cast<const float4 *>(A + static_cast<size_t>(a_row_g) * K + (k0_) + a_k); \
        if ((k0_) + b_k < K && n0 + b_n < N)                                                     \
            bv = *reinterpret_cast<const float4 *>(Bexp + static_cast<size_t>((k0_) + b_k) * N + n0 + b_n); \
    }
    MOE_F32_LOAD(0)
    for (int k0 = 0; k0 < K; k0 += kF32BK) {
        __syncthreads();
        As[a_k + 0][a_row] = av.x;
        As[a_k + 1][a_row] = av.y;
        As[a_k + 2][a_row] = av.z;
        As[a_k + 3][a_row] = av.w;
        *reinterpret_cast<float4 *>(&Bs[b_k][b_n]) = bv;
        __syncthreads();
        if (k0 + kF32BK < K) MOE_F32_LOAD(k0 + kF32BK)
#pragma unroll
        for (int kk = 0; kk < kF32BK; ++kk) {
            const float4 a4 = *reinterpret_cast<const float4 *>(&As[kk][ty * 4]);
            const float4 b4 = *reinterpret_cast<const float4 *>(&Bs[kk][tx * 4]);
            const float a[4] = {a4.x, a4.y, a4.z, a4.w};
            const float b[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
        }
    }
#undef MOE_F32_LOAD
    const int n = n0 + tx * 4;
    if (n >= N) return;
    float4 bs = make_float4(0.f, 0.f, 0.f, 0.f);
    if (bias != nullptr)
        bs = *reinterpret_cast<const float4 *>(bias + static_cast<size_t>(tile.expert) * N + n);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = tile.row0 + ty * 4 + i;
        if (r >= tile.row1) continue;
        float4 o;
        o.x = activate<ACT, false>(acc[i][0] + bs.x);
        o.y = activate<ACT, false>(acc[i][1] + bs.y);
        o.z = activate<ACT, false>(acc[i][2] + bs.z);
        o.w = activate<ACT, false>(acc[i][3] + bs.w);
        *reinterpret_cast<float4 *>(C + static_cast<size_t>(r) * N + n) = o;
    }
}

// ---------------------------------------------------------------- MFMA GEMM
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

template <bool F16>
__device__ __forceinline__ f32x16 mfma_32x32x16(const u32x4 &a, const u32x4 &b, const f32x16 &c)
{
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ void store4(float *p, const float (&v)[4])
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4(_Float16 *p, const float (&v)[4])
{
    f16x4 h;
    h[0] = static_cast<_Float16>(v[0]);
    h[1] = static_cast<_Float16>(v[1]);
    h[2] = static_cast<_Float16>(v[2]);
    h[3] = static_cast<_Float16>(v[3]);
    *reinterpret_cast<f16x4 *>(p) = h;
}

// C[r, n] = act(sum_k A[r,k] W[e][n,k] + bias[e][n]);  A [rows, K], W [E, N, K],
// 16-bit elements (bf16, or fp16 when F16), C [rows, N] of TOut.
// WM x WN wavefronts, each owning (TM*32) rows x (TN*32) columns of the block's
// (WM*TM*32) x (WN*TN*32) output tile.  K is walked in stages of 64 through a
// double-buffered LDS tile; the global loads of stages kt+2 (and kt+3) are in flight while
// stage kt is multiplied, and the barrier of a stage sits before its last 16-deep step so
// that the MFMAs of that step cover the LDS latency of the next stage's first
// fragments.  The work list (one entry per output tile) is ordered so that each XCD
// walks a contiguous share of it: neighbouring blocks then reuse operand tiles in that
// XCD's L2.  32-row sub-tiles past the end of a ragged row tile are skipped.
// KEEP: the pre-activation values (accumulator + bias) also go to Pre [rows, N] as fp16, for
// the backward pass.
// row_src != NULL: A is not the expert-major buffer but the token matrix itself, and the row
// operand of slot i is token row_src[i] / row_div (the dispatch plan's src_of and k): the
// loader gathers the tokens where they lie, so the multiply does not wait for the pack.
template <bool F16, typename TOut, int ACT, int WM, int WN, int TM, int TN, bool KTAIL, bool KEEP>
// (two wavefronts per SIMD in every shape: two 4-wavefront blocks or one 8-wavefront block)
__global__ __launch_bounds__(64 * WM * WN, 2) void grouped_gemm_mfma_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W,
    const float *__restrict__ bias, TOut *__restrict__ C, _Float16 *__restrict__ Pre,
    const WorkItem *__restrict__ items, const int32_t *__restrict__ nitems, int N, int K,
    const int32_t *__restrict__ row_src, int row_div)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 64, LD = BK + 8;
    constexpr int NT = 64 * WM * WN;
    constexpr int AV = BM * 8 / NT, WV = BN * 8 / NT;   // 16-byte vectors per thread per stage
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile does not divide over the threads");

    const int total = *nitems;
    const int per_xcd = (total + 7) / 8;
    const int slot = blockIdx.x / 8;
    const int item_idx = (blockIdx.x % 8) * per_xcd + slot;
    if (slot >= per_xcd || item_idx >= total) return;
    const WorkItem item = items[item_idx];
    const int n0 = item.n0;
    const int rows = item.row1 - item.row0;

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    constexpr int A_BUF = BM * LD, W_BUF = BN * LD;
    uint16_t *As = smem;               // [2][BM][LD]
    uint16_t *Ws = smem + 2 * A_BUF;   // [2][BN][LD]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const uint16_t *Wexp = W + static_cast<size_t>(item.expert) * N * K;

    const uint16_t *a_src[AV];
    const uint16_t *w_src[WV];
    int a_off[AV], w_off[WV];
    const int ld_col = (tid & 7) * 8;
#pragma unroll
    for (int q = 0; q < AV; ++q) {
        const int r = (tid + NT * q) >> 3;
        a_off[q] = r * LD + ld_col;
        // row_src: the operand rows are gathered -- row i of the expert-major order is row
        // row_src[i] / row_div of A (the token that holds assignment row_src[i])
        int arow = min(item.row0 + r, item.row1 - 1);
        if (row_src != nullptr) arow = row_src[arow] / row_div;
        a_src[q] = A + static_cast<size_t>(arow) * K + ld_col;
    }
#pragma unroll
    for (int q = 0; q < WV; ++q) {
        const int r = (tid + NT * q) >> 3;
        w_off[q] = r * LD + ld_col;
        w_src[q] = Wexp + static_cast<size_t>(min(n0 + r, N - 1)) * K + ld_col;
    }
    // 32-row sub-tiles of this wavefront that hold real rows
    const int jact = min(TM, max(0, (rows - wm * TM * 32 + 31) / 32));

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // Register stages between the global loads and the LDS tile: two where the registers
    // allow it (the loads then have two stages of multiplies to arrive), one for the
    // 256 x 256 tile.
    constexpr int DEPTH = BM * BN < 256 * 256 ? 2 : 1;
    u32x4 a_reg[AV], w_reg[WV];
    u32x4 a_reg2[DEPTH == 2 ? AV : 1], w_reg2[DEPTH == 2 ? WV : 1];
    u32x4 wf[2][TN], af[2][TM];
    const int KT = (K + BK - 1) / BK;
    const int fr = lane & 31, fk = (lane >> 5) * 8;
    const int wfrag = (wn * TN * 32 + fr) * LD + fk;
    const int afrag = (wm * TM * 32 + fr) * LD + fk;

#define MOE_LOADG(kt_, AR, WR)                                                                  \
    {                                                                                           \
        const int k0_ = (kt_) * BK;                                                             \
        const bool in_ = !KTAIL || k0_ + ld_col < K;                                           \
        _Pragma("unroll") for (int q = 0; q < AV; ++q)                                          \
        {                                                                                       \
            if (in_) AR[q] = *reinterpret_cast<const u32x4 *>(a_src[q] + k0_);                  \
            else AR[q] = (u32x4){0u, 0u, 0u, 0u};                                               \
        }                                                                                       \
        _Pragma("unroll") for (int q = 0; q < WV; ++q)                                          \
        {                                                                                       \
            if (in_) WR[q] = *reinterpret_cast<const u32x4 *>(w_src[q] + k0_);                  \
            else WR[q] = (u32x4){0u, 0u, 0u, 0u};                                               \
        }                                                                                       \
    }
#define MOE_STOREL(buf, AR, WR)                                                                 \
    {                                                                                           \
        _Pragma("unroll") for (int q = 0; q < AV; ++q)                                          \
            *reinterpret_cast<u32x4 *>(As + (buf) * A_BUF + a_off[q]) = AR[q];                  \
        _Pragma("unroll") for (int q = 0; q < WV; ++q)                                          \
            *reinterpret_cast<u32x4 *>(Ws + (buf) * W_BUF + w_off[q]) = WR[q];                  \
    }
#define MOE_READF(slot_, buf, ks)                                                               \
    {                                                                                           \
        _Pragma("unroll") for (int i = 0; i < TN; ++i) wf[slot_][i] =                           \
            *reinterpret_cast<const u32x4 *>(Ws + (buf) * W_BUF + wfrag + i * 32 * LD + (ks) * 16); \
        _Pragma("unroll") for (int j = 0; j < TM; ++j) af[slot_][j] =                           \
            *reinterpret_cast<const u32x4 *>(As + (buf) * A_BUF + afrag + j * 32 * LD + (ks) * 16); \
    }
#define MOE_MMA(slot_)                                                                          \
    {                                                                                           \
        _Pragma("unroll") for (int j = 0; j < TM; ++j)                                          \
        {                                                                                       \
            if (FULL || j < jact) {                                                             \
                _Pragma("unroll") for (int i = 0; i < TN; ++i)                                  \
                    acc[i][j] = mfma_32x32x16<F16>(wf[slot_][i], af[slot_][j], acc[i][j]);      \
            }                                                                                   \
        }                                                                                       \
    }
// One stage kt held in LDS buffer `buf`: the registers AR/WR (stage kt+1) go to the other
// buffer and are refilled with stage kt+1+DEPTH.
#define MOE_STAGE(buf, AR, WR)                                                                  \
    {                                                                                           \
        const bool next1 = kt + 1 < KT, nextl = kt + 1 + DEPTH < KT;                            \
        if (next1) MOE_STOREL(buf ^ 1, AR, WR)                                                  \
        if (nextl) MOE_LOADG(kt + 1 + DEPTH, AR, WR)                                            \
        MOE_READF(1, buf, 1)                                                                    \
        MOE_MMA(0)                                                                              \
        MOE_READF(0, buf, 2)                                                                    \
        MOE_MMA(1)                                                                              \
        MOE_READF(1, buf, 3)                                                                    \
        MOE_MMA(0)                                                                              \
        __syncthreads();                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                      \
        if (next1) MOE_READF(0, buf ^ 1, 0)                                                     \
        MOE_MMA(1)                                                                              \
    }
#define MOE_MAIN_LOOP                                                                           \
    if constexpr (DEPTH == 2) {                                                                 \
        int kt = 0;                                                                             \
        for (; kt + 1 < KT; kt += 2) {                                                          \
            MOE_STAGE(0, a_reg, w_reg)                                                          \
            ++kt;                                                                               \
            MOE_STAGE(1, a_reg2, w_reg2)                                                        \
            --kt;                                                                               \
        }                                                                                       \
        if (kt < KT) MOE_STAGE(0, a_reg, w_reg)                                                 \
    } else {                                                                                    \
        for (int kt = 0; kt < KT; ++kt) {                                                       \
            const int buf = kt & 1;                                                             \
            MOE_STAGE(buf, a_reg, w_reg)                                                        \
        }                                                                                       \
    }

    // Prologue: stage 0 into LDS, stage 1 (and with two register stages also stage 2) in
    // flight.
    MOE_LOADG(0, a_reg, w_reg)
    MOE_STOREL(0, a_reg, w_reg)
    if (KT > 1) MOE_LOADG(1, a_reg, w_reg)
    if (DEPTH == 2 && KT > 2) MOE_LOADG(2, a_reg2, w_reg2)
    __syncthreads();
    MOE_READF(0, 0, 0)
    if (jact == TM) {          // every sub-tile of this wavefront holds rows: branch-free loop
        constexpr bool FULL = true;
        MOE_MAIN_LOOP
    } else {
        constexpr bool FULL = false;
        MOE_MAIN_LOOP
    }
#undef MOE_STAGE
#undef MOE_MAIN_LOOP
#undef MOE_LOADG
#undef MOE_STOREL
#undef MOE_READF
#undef MOE_MMA

    // acc[i][j][4*g + c]: column n0 + (wn*TN + i)*32 + 8*g + 4*(lane/32) + c,
    //                     row item.row0 + (wm*TM + j)*32 + lane%32
    const float *bexp = bias != nullptr ? bias + static_cast<size_t>(item.expert) * N : nullptr;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int r = item.row0 + (wm * TM + j) * 32 + fr;
        if (r >= item.row1) continue;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + (wn * TN + i) * 32 + 8 * g + 4 * (lane >> 5);
                if (n >= N) continue;
                float v[4], pre[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float s = acc[i][j][4 * g + c];
                    if (bexp != nullptr) s += bexp[n + c];
                    pre[c] = s;
                    v[c] = activate<ACT, true>(s);
                }
                if constexpr (KEEP) store4(Pre + static_cast<size_t>(r) * N + n, pre);
                store4(C + static_cast<size_t>(r) * N + n, v);
            }
        }
    }
}

#include "gemm_w4.h"

// ABL (measurement only, 0 in the layer): bit 0 leaves out the MFMAs, bit 1 the LDS fragment
// reads after the first step, bit 2 the global loads and LDS writes inside the loop, bit 3 the
// output stores.  Results are then wrong by construction; every access stays inside the buffers.
template <bool F16, int ACT, bool KEEP, int ABL = 0>
__global__ __launch_bounds__(256, 1) void grouped_gemm_w4_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W,
    const float *__restrict__ bias, _Float16 *__restrict__ C, _Float16 *__restrict__ Pre,
    const WorkItem *__restrict__ items, const int32_t *__restrict__ nitems, int N, int K,
    const int32_t *__restrict__ row_src, int row_div, int a_rows)
{
#include "gemm_w4_body.inc"

    // Epilogue.  acc[i][j][4*g + c]: column (wn*TN + i)*32 + 8*g + 4*(lane/32) + c, row
    // (wm*TM + j)*32 + lane%32 of the tile.  Every wavefront is past its last LDS read after
    // the barrier; the MFMA results have left the pipeline after the no-ops (the compiler does
    // not see through the inline assembly).  The wavefront's 128 x 128 sub-tile goes to its
    // own patch, row pitch 272 bytes.
    MOE_LGKM0();
    MOE_BAR();
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    constexpr int PITCH = 272;
    char *patch = reinterpret_cast<char *>(smem) + wave * (TM * 32) * PITCH;
    const float *bexp = bias != nullptr ? bias + static_cast<size_t>(item.expert) * N : nullptr;
    const int rbase = item.row0 + wm * TM * 32;
    const int ncol = n0 + wn * TN * 32 + (lane & 15) * 8;
#pragma unroll
    for (int pass = KEEP ? 0 : 1; pass < 2; ++pass) {      // pass 0: pre-activations, 1: outputs
        _Float16 *out = pass == 0 ? Pre : C;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = i * 32 + 8 * g + 4 * (lane >> 5);
                float b4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if (bexp != nullptr) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) b4[c] = bexp[min(n0 + wn * TN * 32 + col + c, N - 1)];
                }
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    float v[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float s = acc[i][j][4 * g + c] + b4[c];
                        v[c] = pass == 0 ? s : activate<ACT, true>(s);
                    }
                    store4(reinterpret_cast<_Float16 *>(patch + (j * 32 + fr) * PITCH) + col, v);
                }
                MOE_SB();      // a few accumulator registers at a time leave the AGPRs
            }
        MOE_LGKM0();
        __builtin_amdgcn_wave_barrier();
#pragma unroll 8
        for (int it = 0; it < TM * 8; ++it) {
            const int rr = it * 4 + (lane >> 4);
            const u32x4 q = *reinterpret_cast<const u32x4 *>(patch + rr * PITCH + (lane & 15) * 16);
            const int r = rbase + rr;
            if (r < item.row1 && ncol < N && (!(ABL & 8) || q[0] == 0x7fc07fc1u))
                *reinterpret_cast<u32x4 *>(out + static_cast<size_t>(r) * N + ncol) = q;
        }
        if (pass == 0) {
            MOE_LGKM0();
            __builtin_amdgcn_wave_barrier();
        }
    }
}
#undef MOE_LGKM0
#undef MOE_SB
#undef MOE_BAR

// ---------------------------------------------------------------- weight packing
// Out[e][n][k] = convert(In[e][k][n]); 64 x 64 tiles through LDS.
// MODE 0: bf16 -> bf16, MODE 1: bf16 -> fp16.
template <int MODE>
__global__ __launch_bounds__(256) void transpose_pack_kernel(
    const uint16_t *__restrict__ in, uint16_t *__restrict__ out, int K, int N)
{
    __shared__ uint16_t tile[64][66];
    const size_t eoff = static_cast<size_t>(blockIdx.z) * K * N;
    const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    for (int v = threadIdx.x; v < 64 * 64; v += 256) {
        const int kk = v / 64, nn = v % 64;
        uint16_t val = 0;
        if (k0 + kk < K && n0 + nn < N) val = in[eoff + static_cast<size_t>(k0 + kk) * N + n0 + nn];
        tile[kk][nn] = val;
    }
    __syncthreads();
    for (int v = threadIdx.x; v < 64 * 64; v += 256) {
        const int nn = v / 64, kk = v % 64;
        if (k0 + kk < K && n0 + nn < N) {
            uint16_t val = tile[kk][nn];
            if constexpr (MODE == 1) {
                const _Float16 h = static_cast<_Float16>(bf16_to_f32(val));
                val = __builtin_bit_cast(uint16_t, h);
            }
            out[eoff + static_cast<size_t>(n0 + nn) * K + k0 + kk] = val;
        }
    }
}

template <int ACT>
void launch_f32_pair(const moe_shape &s, const float *xe, const float *W1, const float *b1,
                     const float *W2, const float *b2, float *ye, const Workspace &w,
                     int chunk, hipStream_t st)
{
    float *H = static_cast<float *>(w.hidden);
    const WorkItem *it1 = w.items[0] + static_cast<size_t>(chunk) * w.gp[0].max_items;
    const WorkItem *it2 = w.items[1] + static_cast<size_t>(chunk) * w.gp[1].max_items;
    prof_begin(kStageGemm1, st);
    hipLaunchKernelGGL(grouped_gemm_f32_kernel<ACT>, dim3(w.gp[0].max_items), dim3(256), 0, st,
                       xe, W1, b1, H, it1, w.nitems[0] + chunk, s.d_ff, s.d_model);
    prof_end(kStageGemm1, st);
    prof_begin(kStageGemm2, st);
    hipLaunchKernelGGL(grouped_gemm_f32_kernel<MOE_ACT_IDENTITY>, dim3(w.gp[1].max_items),
                       dim3(256), 0, st, H, W2, b2, ye, it2, w.nitems[1] + chunk, s.d_model,
                       s.d_ff);
    prof_end(kStageGemm2, st);
}

template <bool F16, typename TOut, int ACT, int WM, int WN, int TM, int TN, bool KTAIL, bool KEEP>
void launch_mfma_cfg_k(const uint16_t *A, const uint16_t *W, const float *bias, TOut *C,
                     _Float16 *pre, const WorkItem *items, const int32_t *nitems, int max_items,
                     int N, int K, int stage, hipStream_t st, const int32_t *row_src, int row_div)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t lds = 2 * (BM + BN) * (64 + 8) * sizeof(uint16_t);
    auto kern = grouped_gemm_mfma_kernel<F16, TOut, ACT, WM, WN, TM, TN, KTAIL, KEEP>;
    static PerDeviceOnce once;   // raising the dynamic LDS limit: once per kernel and device
    once.raise_lds(reinterpret_cast<const void *>(kern), static_cast<int>(lds));
    const int grid = static_cast<int>(align_up(static_cast<size_t>(max_items), 8));
    hipEvent_t t0, t1;
    prof_kernel_events(stage, &t0, &t1);
    hipExtLaunchKernelGGL(kern, dim3(grid), dim3(64 * WM * WN), lds, st, t0, t1, 0, A, W, bias, C,
                          pre, items, nitems, N, K, row_src, row_div);
}

// The contraction depth is a multiple of the 64-deep stage in every benchmark shape;
// other depths take a variant that zero-fills the last stage.
template <bool F16, typename TOut, int ACT, bool KEEP, int WM, int WN, int TM, int TN>
void launch_mfma_cfg(const uint16_t *A, const uint16_t *W, const float *bias, TOut *C,
                     _Float16 *pre, const WorkItem *items, const int32_t *nitems, int max_items,
                     int N, int K, int stage, hipStream_t st, const int32_t *row_src, int row_div)
{
    if (K % 64 == 0)
        launch_mfma_cfg_k<F16, TOut, ACT, WM, WN, TM, TN, false, KEEP>(
            A, W, bias, C, pre, items, nitems, max_items, N, K, stage, st, row_src, row_div);
    else
        launch_mfma_cfg_k<F16, TOut, ACT, WM, WN, TM, TN, true, KEEP>(
            A, W, bias, C, pre, items, nitems, max_items, N, K, stage, st, row_src, row_div);
}

// The four-wavefront kernel addresses its operands with 32-bit byte offsets into buffer
// resources (the expert's weight matrix; the tile's rows, or the whole token matrix when the
// rows are gathered) and walks whole 64-deep stages.
inline bool w4_kernel_fits(int N, int K, bool gathered, uint64_t row_limit)
{
    return K % 64 == 0 && static_cast<uint64_t>(N) * K * 2 < (1ull << 31) &&
           (gathered ? row_limit * static_cast<uint64_t>(K) : 256ull * K) * 2 < (1ull << 31);
}

template <bool F16, typename TOut, int ACT, bool KEEP>
void launch_mfma(const GemmPlan &gp, const uint16_t *A, const uint16_t *W, const float *bias,
                 TOut *C, _Float16 *pre, const WorkItem *items, const int32_t *nitems, int N, int K,
                 int stage, hipStream_t st, const int32_t *row_src = nullptr, int row_div = 1,
                 uint64_t row_limit = 0)
{
#define MOE_MFMA_SHAPE(WM_, WN_, TM_, TN_)                                                        \
    launch_mfma_cfg<F16, TOut, ACT, KEEP, WM_, WN_, TM_, TN_>(A, W, bias, C, pre, items, nitems,    \
                                                              gp.max_items, N, K, stage, st,       \
                                                              row_src, row_div)
    if (gp.bm == 256) {
        if constexpr (std::is_same<TOut, _Float16>::value) {
            if (w4_kernel_fits(N, K, row_src != nullptr, row_limit)) {
                constexpr size_t lds = 2 * (256 + 256) * (64 + 8) * sizeof(uint16_t);
                auto kern = grouped_gemm_w4_kernel<F16, ACT, KEEP>;
                static PerDeviceOnce once;
                once.raise_lds(reinterpret_cast<const void *>(kern), static_cast<int>(lds));
                const int grid = static_cast<int>(align_up(static_cast<size_t>(gp.max_items), 8));
                hipEvent_t t0, t1;
                prof_kernel_events(stage, &t0, &t1);
                hipExtLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, t0, t1, 0, A, W, bias, C,
                                      pre, items, nitems, N, K, row_src, row_div,
                                      static_cast<int>(row_limit));
                return;
            }
        }
        MOE_MFMA_SHAPE(2, 4, 4, 2);
    }
    else if (gp.bm == 64)
        MOE_MFMA_SHAPE(1, 8, 2, 1);
    else if (gp.bn == 256)
        MOE_MFMA_SHAPE(2, 4, 2, 2);
    else
        MOE_MFMA_SHAPE(2, 2, 2, 2);
#undef MOE_MFMA_SHAPE
}

template <int ACT>
void launch_mfma_pair(const moe_shape &s, const uint16_t *xe, const uint16_t *W1p,
                      const float *b1, const uint16_t *W2p, const float *b2, _Float16 *ye,
                      _Float16 *pre, const Workspace &w, int chunk, hipStream_t st,
                      const int32_t *row_src, int row_div)
{
    _Float16 *H = static_cast<_Float16 *>(w.hidden);
    const WorkItem *it1 = w.items[0] + static_cast<size_t>(chunk) * w.gp[0].max_items;
    const WorkItem *it2 = w.items[1] + static_cast<size_t>(chunk) * w.gp[1].max_items;
    if (pre != nullptr)
        launch_mfma<false, _Float16, ACT, true>(w.gp[0], xe, W1p, b1, H, pre, it1,
                                                w.nitems[0] + chunk, s.d_ff, s.d_model,
                                                kStageGemm1, st, row_src, row_div, s.T);
    else
        launch_mfma<false, _Float16, ACT, false>(w.gp[0], xe, W1p, b1, H, nullptr, it1,
                                                 w.nitems[0] + chunk, s.d_ff, s.d_model,
                                                 kStageGemm1, st, row_src, row_div, s.T);
    launch_mfma<true, _Float16, MOE_ACT_IDENTITY, false>(w.gp[1], reinterpret_cast<const uint16_t *>(H),
                                                      W2p, b2, ye, nullptr, it2, w.nitems[1] + chunk,
                                                      s.d_model, s.d_ff, kStageGemm2, st);
}

}  // namespace

// Which kernel the layer launches for expert GEMM `which` (0: first, 1: second) of a bf16 layer,
// for labelling measurements: "<kernel> <tile rows>x<tile columns>".
void expert_gemm_kernel_name(const moe_shape &s, int which, int n_chunks, char *name, size_t len)
{
    const GemmPlan gp = choose_gemm_plan(s, which, n_chunks);
    const int N = which == 0 ? s.d_ff : s.d_model, K = which == 0 ? s.d_model : s.d_ff;
    const bool w4 = gp.bm == 256 && w4_kernel_fits(N, K, which == 0, static_cast<uint64_t>(s.T));
    std::snprintf(name, len, "%s %dx%d", w4 ? "grouped_gemm_w4_kernel" : "grouped_gemm_mfma_kernel",
                  gp.bm, gp.bn);
}

// Measurement aid: the 256 x 256 kernel alone on caller-made operands and work list, with
// parts of it left out (see ABL above).  gelu != 0 applies the activation.
moe_status launch_calib_gemm(const uint16_t *A, const uint16_t *W, _Float16 *C, const WorkItem *items,
                             const int32_t *nitems, int max_items, int N, int K, int abl, int gelu,
                             hipStream_t st)
{
    constexpr size_t lds = 2 * (256 + 256) * (64 + 8) * sizeof(uint16_t);
    const int grid = static_cast<int>(align_up(static_cast<size_t>(max_items), 8));
#define MOE_CALIB_CASE(ABL_)                                                                      \
    case ABL_: {                                                                                  \
        auto k1 = grouped_gemm_w4_kernel<false, MOE_ACT_GELU_ERF, false, ABL_>;                   \
        auto k0 = grouped_gemm_w4_kernel<false, MOE_ACT_IDENTITY, false, ABL_>;                   \
        static PerDeviceOnce once1, once0;                                                        \
        once1.raise_lds(reinterpret_cast<const void *>(k1), static_cast<int>(lds));               \
        once0.raise_lds(reinterpret_cast<const void *>(k0), static_cast<int>(lds));               \
        hipLaunchKernelGGL(gelu ? k1 : k0, dim3(grid), dim3(256), lds, st, A, W, nullptr, C,      \
                           nullptr, items, nitems, N, K, nullptr, 1, 0);                          \
        break;                                                                                    \
    }
    switch (abl) {
        MOE_CALIB_CASE(0)
        MOE_CALIB_CASE(1)
        MOE_CALIB_CASE(2)
        MOE_CALIB_CASE(4)
        MOE_CALIB_CASE(6)
        MOE_CALIB_CASE(7)
        MOE_CALIB_CASE(8)
    default:
        set_error("moe_calib_gemm: variant %d is not built (0, 1, 2, 4, 6, 7, 8)", abl);
        return MOE_EINVAL;
    }
#undef MOE_CALIB_CASE
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

// Tile shape of expert GEMM `which` (0: xe.W1, 1: H.W2) for this layer shape.  Large
// tiles cut the operand traffic per flop; they need enough output tiles to fill 256
// compute units, and a long contraction to amortise their prologue and epilogue.
GemmPlan choose_gemm_plan(const moe_shape &s, int which, int n_chunks)
{
    GemmPlan gp;
    const int N = which == 0 ? s.d_ff : s.d_model;
    const int K = which == 0 ? s.d_model : s.d_ff;
    const int64_t max_rows = moe_max_rows(&s);
    const int64_t chunk_tokens = (s.T + n_chunks - 1) / n_chunks;
    const int64_t chunk_rows = chunk_tokens * s.k < max_rows ? chunk_tokens * s.k : max_rows;
    if (s.dtype != MOE_BF16) {
        gp.bm = gp.bn = kF32Tile;
        gp.concurrent = 256;
    } else {
        const int64_t big_tiles = (chunk_rows / 256 + s.E / 2) * ((N + 255) / 256);
        if (big_tiles >= 768) {
            gp.bm = 256; gp.bn = 256; gp.concurrent = 32;
        } else if (K >= 2048 && N >= 256 && chunk_rows / s.E < 96 &&
                   (chunk_rows / 128 + s.E / 2) * ((N + 255) / 256) < 256) {
            // few rows per expert and fewer 128-row tiles than compute units: the GEMM
            // streams the weights once; shorter tiles put more units on the stream and
            // spend less of their loads on (mostly padded) rows
            gp.bm = 64; gp.bn = 256; gp.concurrent = 32;
        } else if (K >= 2048 && N >= 256) {
            gp.bm = 128; gp.bn = 256; gp.concurrent = 32;
        } else {
            gp.bm = 128; gp.bn = 128; gp.concurrent = 64;
        }
    }
    gp.tiles_n = (N + gp.bn - 1) / gp.bn;
    gp.max_row_tiles = static_cast<int32_t>((chunk_rows + gp.bm - 1) / gp.bm + s.E);
    gp.max_items = gp.max_row_tiles * gp.tiles_n;
    return gp;
}

moe_status launch_ffn(const moe_shape &s, const void *xe, const void *W1p, const float *b1,
                      const void *W2p, const float *b2, void *ye, const Workspace &w,
                      int chunk, hipStream_t st, void *pre, const int32_t *row_src)
{
    if (row_src != nullptr && s.dtype != MOE_BF16) {
        set_error("gathered token rows are for bf16 layers only");
        return MOE_EUNSUPPORTED;
    }
    if (pre != nullptr && s.dtype != MOE_BF16) {
        set_error("the pre-activations are kept for bf16 layers only");
        return MOE_EUNSUPPORTED;
    }
#define MOE_FFN_CASE(ACT)                                                                      \
    case ACT:                                                                                  \
        if (s.dtype == MOE_BF16)                                                               \
            launch_mfma_pair<ACT>(s, static_cast<const uint16_t *>(xe),                         \
                                  static_cast<const uint16_t *>(W1p), b1,                       \
                                  static_cast<const uint16_t *>(W2p), b2,                       \
                                  static_cast<_Float16 *>(ye), static_cast<_Float16 *>(pre), w, \
                                  chunk, st, row_src, s.k);                                     \
        else                                                                                   \
            launch_f32_pair<ACT>(s, static_cast<const float *>(xe),                             \
                                 static_cast<const float *>(W1p), b1,                           \
                                 static_cast<const float *>(W2p), b2, static_cast<float *>(ye), \
                                 w, chunk, st);                                                 \
        break;
    switch (s.act) {
        MOE_FFN_CASE(MOE_ACT_GELU_ERF)
        MOE_FFN_CASE(MOE_ACT_GELU_TANH)
        MOE_FFN_CASE(MOE_ACT_RELU)
        MOE_FFN_CASE(MOE_ACT_IDENTITY)
    default:
        set_error("unknown activation %d", s.act);
        return MOE_EINVAL;
    }
#undef MOE_FFN_CASE
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status launch_pack(const moe_shape &s, const void *W1, const void *W2, void *W1p,
                       void *W2p, hipStream_t st)
{
    const size_t elems = static_cast<size_t>(s.E) * s.d_model * s.d_ff;
    if (s.dtype == MOE_F32) {
        MOE_TRY_HIP(hipMemcpyAsync(W1p, W1, elems * 4, hipMemcpyDeviceToDevice, st));
        MOE_TRY_HIP(hipMemcpyAsync(W2p, W2, elems * 4, hipMemcpyDeviceToDevice, st));
        return MOE_OK;
    }
    // W1 [E, d, h] -> [E, h, d];  W2 [E, h, d] -> [E, d, h] as fp16
    hipLaunchKernelGGL(transpose_pack_kernel<0>,
                       dim3(ceil_div(s.d_ff, 64), ceil_div(s.d_model, 64), s.E), dim3(256), 0, st,
                       static_cast<const uint16_t *>(W1), static_cast<uint16_t *>(W1p), s.d_model,
                       s.d_ff);
    hipLaunchKernelGGL(transpose_pack_kernel<1>,
                       dim3(ceil_div(s.d_model, 64), ceil_div(s.d_ff, 64), s.E), dim3(256), 0, st,
                       static_cast<const uint16_t *>(W2), static_cast<uint16_t *>(W2p), s.d_ff,
                       s.d_model);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace moe
