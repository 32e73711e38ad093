// Backward pass of the MoE layer (chain rule of the forward of paper Sec. 2.1; the paper
// trains this layer and schedules its backward pass in Sec. 2.2 and Sec. 4).
//
//   combine_bwd      dye[slot] = g dy[t] (bf16), dgate = <ye[slot], dy[t]>
//   gemm (rows)      P = xe W1 (fp16) and Hb = act(P) (bf16) -- only when the forward did not
//                    keep P and its hidden activations
//   gemm (rows)      dP = (dye W2^T) * act'(P)                        (bf16)
//   gemm (rows)      dxe = dP W1^T                                    (fp32)
//   gemm (wgrad)     dW2[e] = act(P)^T dye, dW1[e] = xe^T dP          (fp32), operands row-major
//                    as they are: the fragments come out of LDS through transposing reads
//   gate_bwd         logits (from the packed gate matrix), softmax, dz,
//                    dx = sum of the token's dxe rows + dz Wg^T
//   dwg              dWg = x^T dz (partial sums over token ranges, then a fixed-order sum)
//
// The contractions use 128 x 128 (or 128 x 256) output tiles of 32x32x16 bf16 MFMAs fed
// through a double-buffered LDS tile, like the forward's expert GEMM; a row-grouped GEMM walks
// the forward's kind of work list, a weight-gradient GEMM contracts over one expert's rows.
#include "common.h"
#include "moe_train.h"

#include <algorithm>

#include <hip/hip_ext.h>

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

#include "gemm_w4.h"

constexpr int kBM = 128, kBK = 64, kLD = kBK + 8;
// output tile 128 x (64 WN): WN = 2 (four wavefronts) or 4 (eight)
constexpr size_t gemm_lds(int wn) { return 2 * (kBM + 64 * wn) * kLD * sizeof(uint16_t); }

// Phi(v), the normal CDF, as 1 / (1 + 2^(v Q(min(v^2, 49)))) with the cubic Q of the forward's
// GeLU (absolute error of v Phi(v) below 1.5e-5).
__device__ __forceinline__ float normal_cdf_fast(float v)
{
    const float s = fminf(v * v, 49.0f);
    float q = 2.1637799e-05f;
    q = __builtin_fmaf(q, s, 7.7587553e-04f);
    q = __builtin_fmaf(q, s, -1.0610976e-01f);
    q = __builtin_fmaf(q, s, -2.3015507e+00f);
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * q));
}

template <int ACT>
__device__ __forceinline__ float act_value(float v)
{
    if constexpr (ACT == MOE_ACT_GELU_ERF)
        return v * normal_cdf_fast(v);
    else if constexpr (ACT == MOE_ACT_GELU_TANH)
        return 0.5f * v * (1.0f + tanhf(0.7978845608028654f * (v + 0.044715f * v * v * v)));
    else if constexpr (ACT == MOE_ACT_RELU)
        return fmaxf(v, 0.0f);
    else
        return v;
}

template <int ACT>
__device__ __forceinline__ float act_derivative(float v)
{
    if constexpr (ACT == MOE_ACT_GELU_ERF) {
        // Phi(v) + v phi(v); phi(v) = exp(-v^2 / 2) / sqrt(2 pi) through exp2
        const float pdf = 0.3989422804014327f * __builtin_amdgcn_exp2f(-0.72134752044448171f * v * v);
        return normal_cdf_fast(v) + v * pdf;
    } else if constexpr (ACT == MOE_ACT_GELU_TANH) {
        const float c = 0.7978845608028654f, a = 0.044715f;
        const float th = tanhf(c * (v + a * v * v * v));
        return 0.5f * (1.0f + th) + 0.5f * v * (1.0f - th * th) * c * (1.0f + 3.0f * a * v * v);
    } else if constexpr (ACT == MOE_ACT_RELU) {
        return v > 0.0f ? 1.0f : 0.0f;
    } else {
        return 1.0f;
    }
}

__device__ __forceinline__ void store_bf16x4(uint16_t *p, const float (&v)[4])
{
    u32x2 o;
    o[0] = static_cast<uint32_t>(f32_to_bf16(v[0])) | (static_cast<uint32_t>(f32_to_bf16(v[1])) << 16);
    o[1] = static_cast<uint32_t>(f32_to_bf16(v[2])) | (static_cast<uint32_t>(f32_to_bf16(v[3])) << 16);
    *reinterpret_cast<u32x2 *>(p) = o;
}

// ---------------------------------------------------------------- combine backward
// One wavefront per token.
__global__ __launch_bounds__(256) void combine_bwd_kernel(
    const float *__restrict__ dy, const _Float16 *__restrict__ ye, const int32_t *__restrict__ slot_of,
    const float *__restrict__ gate, uint16_t *__restrict__ dye, float *__restrict__ dgate, int t0,
    int T, int d, int k, int max_rows)
{
    // tokens [t0, T)
    const int lane = lane_id();
    const int t = t0 + blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const float *dyrow = dy + static_cast<size_t>(t) * d;
    for (int j = 0; j < k; ++j) {
        const int slot = slot_of[static_cast<size_t>(t) * k + j];
        if (slot < 0 || slot >= max_rows) {
            if (lane == 0) dgate[static_cast<size_t>(t) * k + j] = 0.0f;
            continue;
        }
        const float g = gate[static_cast<size_t>(t) * k + j];
        const _Float16 *yerow = ye + static_cast<size_t>(slot) * d;
        uint16_t *out = dye + static_cast<size_t>(slot) * d;
        float dot = 0.0f;
        for (int c = lane * 4; c < d; c += kWave * 4) {
            const float4 a = *reinterpret_cast<const float4 *>(dyrow + c);
            typedef __attribute__((ext_vector_type(4))) _Float16 half4;
            const half4 b = *reinterpret_cast<const half4 *>(yerow + c);
            dot = __builtin_fmaf(a.x, static_cast<float>(b[0]), dot);
            dot = __builtin_fmaf(a.y, static_cast<float>(b[1]), dot);
            dot = __builtin_fmaf(a.z, static_cast<float>(b[2]), dot);
            dot = __builtin_fmaf(a.w, static_cast<float>(b[3]), dot);
            const float v[4] = {g * a.x, g * a.y, g * a.z, g * a.w};
            store_bf16x4(out + c, v);
        }
#pragma unroll
        for (int m = kWave / 2; m > 0; m >>= 1) dot += __shfl_xor(dot, m);
        if (lane == 0) dgate[static_cast<size_t>(t) * k + j] = dot;
    }
}

// ---------------------------------------------------------------- GEMM
// C[r, n] = sum_k A[r, k] W[e][n, k] for the rows of one work item.
// EPI 0: fp32 store.  EPI 1: P = acc as fp16 into Pbuf and act(acc) as bf16 into C.
// EPI 2: acc * act'(Pbuf) as bf16 into C.
template <int EPI, int ACT, bool KTAIL, int WN>
__global__ __launch_bounds__(128 * WN, 2) void bwd_gemm_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, void *__restrict__ Cout,
    _Float16 *__restrict__ Pbuf, const WorkItem *__restrict__ items,
    const int32_t *__restrict__ nitems, int N, int K)
{
    constexpr int WM = 2, TM = 2, TN = 2, NT = 128 * WN;   // 2 x WN wavefronts of 64 x 64
    constexpr int kBN = 64 * WN;
    constexpr int AV = kBM * 8 / NT, WV = kBN * 8 / NT;
    int expert, row0, row1, n0;
    {
        const int total = *nitems;
        const int per_xcd = (total + 7) / 8;
        const int slot = blockIdx.x / 8;
        const int idx = (blockIdx.x % 8) * per_xcd + slot;
        if (slot >= per_xcd || idx >= total) return;
        const WorkItem item = items[idx];
        expert = item.expert; row0 = item.row0; row1 = item.row1; n0 = item.n0;
    }
    const int KT = (K + kBK - 1) / kBK;
    const size_t w_base = static_cast<size_t>(expert) * N * K;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    constexpr int A_BUF = kBM * kLD, W_BUF = kBN * kLD;
    uint16_t *As = smem;
    uint16_t *Ws = smem + 2 * A_BUF;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int fr = lane & 31, fk = (lane >> 5) * 8;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    if (KT > 0) {
        const uint16_t *a_src[AV];
        const uint16_t *w_src[WV];
        int a_off[AV], w_off[WV];
        const int ld_col = (tid & 7) * 8;
#pragma unroll
        for (int q = 0; q < AV; ++q) {
            const int r = (tid + NT * q) >> 3;
            a_off[q] = r * kLD + ld_col;
            a_src[q] = A + static_cast<size_t>(min(row0 + r, row1 - 1)) * K + ld_col;
        }
#pragma unroll
        for (int q = 0; q < WV; ++q) {
            const int r = (tid + NT * q) >> 3;
            w_off[q] = r * kLD + ld_col;
            w_src[q] = W + w_base + static_cast<size_t>(min(n0 + r, N - 1)) * K + ld_col;
        }
        u32x4 a_reg[AV], w_reg[WV], a_reg2[AV], w_reg2[WV];   // two register stages of prefetch
        u32x4 wf[2][TN], af[2][TM];
        const int wfrag = (wn * TN * 32 + fr) * kLD + fk;
        const int afrag = (wm * TM * 32 + fr) * kLD + fk;
#define BWD_LOADG(kt_, AR, WR)                                                                  \
    {                                                                                           \
        const int k0_ = (kt_) * kBK;                                                            \
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
#define BWD_STOREL(buf, AR, WR)                                                                 \
    {                                                                                           \
        _Pragma("unroll") for (int q = 0; q < AV; ++q)                                          \
            *reinterpret_cast<u32x4 *>(As + (buf) * A_BUF + a_off[q]) = AR[q];                  \
        _Pragma("unroll") for (int q = 0; q < WV; ++q)                                          \
            *reinterpret_cast<u32x4 *>(Ws + (buf) * W_BUF + w_off[q]) = WR[q];                  \
    }
#define BWD_READF(slot_, buf, ks)                                                               \
    {                                                                                           \
        _Pragma("unroll") for (int i = 0; i < TN; ++i) wf[slot_][i] =                           \
            *reinterpret_cast<const u32x4 *>(Ws + (buf) * W_BUF + wfrag + i * 32 * kLD + (ks) * 16); \
        _Pragma("unroll") for (int j = 0; j < TM; ++j) af[slot_][j] =                           \
            *reinterpret_cast<const u32x4 *>(As + (buf) * A_BUF + afrag + j * 32 * kLD + (ks) * 16); \
    }
#define BWD_MMA(slot_)                                                                          \
    {                                                                                           \
        _Pragma("unroll") for (int j = 0; j < TM; ++j)                                          \
            _Pragma("unroll") for (int i = 0; i < TN; ++i)                                      \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                            \
                    __builtin_bit_cast(bf16x8, wf[slot_][i]),                                   \
                    __builtin_bit_cast(bf16x8, af[slot_][j]), acc[i][j], 0, 0, 0);              \
    }
// stage kt in LDS buffer `buf`: AR/WR (stage kt+1) go to the other buffer and are refilled
// with stage kt+3
#define BWD_STAGE(buf, AR, WR)                                                                  \
    {                                                                                           \
        const bool next1 = kt + 1 < KT, next3 = kt + 3 < KT;                                    \
        if (next1) BWD_STOREL(buf ^ 1, AR, WR)                                                  \
        if (next3) BWD_LOADG(kt + 3, AR, WR)                                                    \
        BWD_READF(1, buf, 1)                                                                    \
        BWD_MMA(0)                                                                              \
        BWD_READF(0, buf, 2)                                                                    \
        BWD_MMA(1)                                                                              \
        BWD_READF(1, buf, 3)                                                                    \
        BWD_MMA(0)                                                                              \
        __syncthreads();                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                      \
        if (next1) BWD_READF(0, buf ^ 1, 0)                                                     \
        BWD_MMA(1)                                                                              \
    }
        BWD_LOADG(0, a_reg, w_reg)
        BWD_STOREL(0, a_reg, w_reg)
        if (KT > 1) BWD_LOADG(1, a_reg, w_reg)
        if (KT > 2) BWD_LOADG(2, a_reg2, w_reg2)
        __syncthreads();
        BWD_READF(0, 0, 0)
        int kt = 0;
        for (; kt + 1 < KT; kt += 2) {
            BWD_STAGE(0, a_reg, w_reg)
            ++kt;
            BWD_STAGE(1, a_reg2, w_reg2)
            --kt;
        }
        if (kt < KT) BWD_STAGE(0, a_reg, w_reg)
#undef BWD_STAGE
#undef BWD_LOADG
#undef BWD_STOREL
#undef BWD_READF
#undef BWD_MMA
    }

    // acc[i][j][4*g + c]: column n0 + (wn*TN + i)*32 + 8*g + 4*(lane/32) + c,
    //                     row row0 + (wm*TM + j)*32 + lane%32
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int r = row0 + (wm * TM + j) * 32 + fr;
        if (r >= row1) continue;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + (wn * TN + i) * 32 + 8 * g + 4 * (lane >> 5);
                if (n >= N) continue;
                const size_t at = static_cast<size_t>(r) * N + n;
                float v[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) v[c] = acc[i][j][4 * g + c];
                if constexpr (EPI == 0) {
                    *reinterpret_cast<float4 *>(static_cast<float *>(Cout) + at) =
                        make_float4(v[0], v[1], v[2], v[3]);
                } else if constexpr (EPI == 1) {
                    f16x4 p;
                    float a[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        p[c] = static_cast<_Float16>(v[c]);
                        a[c] = act_value<ACT>(v[c]);
                    }
                    *reinterpret_cast<f16x4 *>(Pbuf + at) = p;
                    store_bf16x4(static_cast<uint16_t *>(Cout) + at, a);
                } else {
                    const f16x4 p = *reinterpret_cast<const f16x4 *>(Pbuf + at);
                    float a[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) a[c] = v[c] * act_derivative<ACT>(static_cast<float>(p[c]));
                    store_bf16x4(static_cast<uint16_t *>(Cout) + at, a);
                }
            }
        }
    }
}

// ---------------------------------------------------------------- GEMM, 256 x 256 tiles
// The same three products on the forward's four-wavefront layout (gemm_w4.h), for layers whose
// row GEMMs have enough 256 x 256 tiles to fill the chip.  The tile leaves through LDS as
// whole lines (16-bit outputs) or straight from the registers (fp32); for EPI 2 the tile of
// pre-activations comes in through the same LDS patch, as whole lines.
template <int EPI, int ACT>
__global__ __launch_bounds__(256, 1) void bwd_gemm_w4_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, void *__restrict__ Cout,
    _Float16 *__restrict__ Pbuf, const WorkItem *__restrict__ items,
    const int32_t *__restrict__ nitems, int N, int K)
{
    constexpr bool F16 = false;
    constexpr int ABL = 0;
    const int32_t *const row_src = nullptr;          // packed rows only
    constexpr int row_div = 1, a_rows = 0;
#include "gemm_w4_body.inc"

    // acc[i][j][4*g + c]: column (wn*TN + i)*32 + 8*g + 4*(lane/32) + c, row (wm*TM + j)*32 +
    // lane%32 of the tile.  Every wavefront is past its last LDS read after the barrier, the
    // MFMA results have left the pipeline after the no-ops.
    MOE_LGKM0();
    MOE_BAR();
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    const int rbase = item.row0 + wm * TM * 32;
    if constexpr (EPI == 0) {
        float *out = static_cast<float *>(Cout);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + (wn * TN + i) * 32 + 8 * g + 4 * (lane >> 5);
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    const int r = rbase + j * 32 + fr;
                    if (r < item.row1 && n < N)
                        *reinterpret_cast<float4 *>(out + static_cast<size_t>(r) * N + n) =
                            make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                                        acc[i][j][4 * g + 3]);
                }
                MOE_SB();      // a few accumulator registers at a time leave the AGPRs
            }
    } else {
        constexpr int PITCH = 272;                   // the wavefront's 128 x 128 patch of 16-bit values
        char *patch = reinterpret_cast<char *>(smem) + wave * (TM * 32) * PITCH;
        const int ncol = n0 + wn * TN * 32 + (lane & 15) * 8;
        // whole 256-byte row pieces between the patch and a [rows, N] matrix of 16-bit values
        auto lines_out = [&](uint16_t *dst) {
#pragma unroll 8
            for (int it = 0; it < TM * 8; ++it) {
                const int rr = it * 4 + (lane >> 4);
                const u32x4 q = *reinterpret_cast<const u32x4 *>(patch + rr * PITCH + (lane & 15) * 16);
                const int r = rbase + rr;
                if (r < item.row1 && ncol < N)
                    *reinterpret_cast<u32x4 *>(dst + static_cast<size_t>(r) * N + ncol) = q;
            }
        };
        if constexpr (EPI == 2) {
            const uint16_t *src = reinterpret_cast<const uint16_t *>(Pbuf);
#pragma unroll 8
            for (int it = 0; it < TM * 8; ++it) {
                const int rr = it * 4 + (lane >> 4);
                const int r = rbase + rr;
                u32x4 q = {0u, 0u, 0u, 0u};
                if (r < item.row1 && ncol < N)
                    q = *reinterpret_cast<const u32x4 *>(src + static_cast<size_t>(r) * N + ncol);
                *reinterpret_cast<u32x4 *>(patch + rr * PITCH + (lane & 15) * 16) = q;
            }
            MOE_LGKM0();
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
        for (int pass = EPI == 1 ? 0 : 1; pass < 2; ++pass) {     // EPI 1, pass 0: the pre-activations
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = i * 32 + 8 * g + 4 * (lane >> 5);
#pragma unroll
                    for (int j = 0; j < TM; ++j) {
                        char *at = patch + (j * 32 + fr) * PITCH + col * 2;
                        float v[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) v[c] = acc[i][j][4 * g + c];
                        if (EPI == 1 && pass == 0) {
                            f16x4 p;
#pragma unroll
                            for (int c = 0; c < 4; ++c) p[c] = static_cast<_Float16>(v[c]);
                            *reinterpret_cast<f16x4 *>(at) = p;
                        } else {
                            float a[4];
                            if constexpr (EPI == 1) {
#pragma unroll
                                for (int c = 0; c < 4; ++c) a[c] = act_value<ACT>(v[c]);
                            } else {
                                const f16x4 p = *reinterpret_cast<const f16x4 *>(at);
#pragma unroll
                                for (int c = 0; c < 4; ++c)
                                    a[c] = v[c] * act_derivative<ACT>(static_cast<float>(p[c]));
                            }
                            store_bf16x4(reinterpret_cast<uint16_t *>(at), a);
                        }
                    }
                    MOE_SB();
                }
            MOE_LGKM0();
            __builtin_amdgcn_wave_barrier();
            lines_out(EPI == 1 && pass == 0 ? reinterpret_cast<uint16_t *>(Pbuf)
                                            : static_cast<uint16_t *>(Cout));
            if (EPI == 1 && pass == 0) {
                MOE_LGKM0();
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
}

// ---------------------------------------------------------------- weight gradient, row-major operands
// C[e][m, n] = sum over the rows r of expert e of A[r, m] B[r, n]: both operands are stored
// with the contraction index (the row) as the SLOW one.  The tiles go to LDS as they are --
// 64 rows x 128 columns, 16-byte vectors -- and the MFMA fragments (eight consecutive rows for
// one column per lane) come out of LDS through gfx950's transposing 64-bit read, which hands
// each lane of a 16-lane group four consecutive ROWS of one column: lane i of the group points
// at row i / 4, columns 4 (i % 4) .. + 3, and receives rows 0 .. 3 of column i.  The 64-byte
// pieces of a row are XOR-swizzled with the row number so that the four rows a group reads
// fall into different banks.  128 x 128 output tile, four wavefronts, the row-grouped GEMM's
// software pipeline; rows beyond the expert's last one are zeroed in the last stage only.
typedef __attribute__((ext_vector_type(4))) short s16x4;

__device__ __forceinline__ u32x2 lds_read_tr16(const uint16_t *p)
{
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4 *)(p));
    return __builtin_bit_cast(u32x2, v);
}

// AF16: A holds fp16 values (the forward's hidden activations); they are rounded to bf16 on
// their way into LDS (two conversions to fp32 and one packed conversion per pair).
__device__ __forceinline__ uint32_t f16x2_to_bf16x2(uint32_t w)
{
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    const f16x2 hv = __builtin_bit_cast(f16x2, w);
    bf16x2 b;
    b[0] = static_cast<__bf16>(static_cast<float>(hv[0]));
    b[1] = static_cast<__bf16>(static_cast<float>(hv[1]));
    return __builtin_bit_cast(uint32_t, b);
}

template <bool AF16>
__global__ __launch_bounds__(256, 2) void wgrad_gemm_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, float *__restrict__ C,
    const int32_t *__restrict__ offsets, int E, int M, int N, int tiles_m, int tiles_n)
{
    constexpr int WM = 2, TM = 2, TN = 2, NT = 256;     // 2 x 2 wavefronts of 64 x 64
    constexpr int kTile = 128, kRowB = kTile * 2;        // tile columns, bytes per LDS row
    constexpr int kBuf = kBK * kTile;                    // elements per LDS buffer
    constexpr int V = kBK * (kTile / 8) / NT;            // 16-byte vectors per thread, stage, operand
    int expert, m0, n0;
    {
        const int total = E * tiles_m * tiles_n;
        const int per_xcd = (total + 7) / 8;
        const int slot = blockIdx.x / 8;
        const int idx = (blockIdx.x % 8) * per_xcd + slot;
        if (slot >= per_xcd || idx >= total) return;
        expert = idx / (tiles_m * tiles_n);
        const int rem = idx % (tiles_m * tiles_n);
        m0 = (rem / tiles_n) * kTile;
        n0 = (rem % tiles_n) * kTile;
    }
    const int r0 = offsets[expert], r1 = offsets[expert + 1];
    const int KT = (r1 - r0 + kBK - 1) / kBK;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *As = smem;                 // [2][kBK][kTile], swizzled
    uint16_t *Bs = smem + 2 * kBuf;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    if (KT > 0) {
        // staging: vector v = tid + 256 q is row v / 16, columns 8 (v % 16) .. + 7 of the tile
        int st_row[V], st_off[V];
        size_t a_col[V], b_col[V];
        const uint16_t *a_ptr[V], *b_ptr[V];
#pragma unroll
        for (int q = 0; q < V; ++q) {
            const int v = tid + NT * q;
            const int k = v >> 4, c16 = v & 15;
            st_row[q] = k;
            st_off[q] = (k * kRowB + (((c16 >> 2) ^ (k & 3)) << 6) + ((c16 & 3) << 4)) >> 1;   // elements
            a_col[q] = static_cast<size_t>(min(m0 + c16 * 8, M - 8));
            b_col[q] = static_cast<size_t>(min(n0 + c16 * 8, N - 8));
            a_ptr[q] = A + static_cast<size_t>(r0 + k) * M + a_col[q];
            b_ptr[q] = B + static_cast<size_t>(r0 + k) * N + b_col[q];
        }
        const size_t a_step = static_cast<size_t>(kBK) * M, b_step = static_cast<size_t>(kBK) * N;
        u32x4 a_reg[V], b_reg[V], a_reg2[V], b_reg2[V];
        u32x4 bf[2][TN], af[2][TM];
        // fragment addresses: lane = 16 g + i reads row 8 (g / 2) + i / 4 (+ 4 for the upper
        // half) of the 16-row step, columns 16 (g % 2) + 4 (i % 4) .. + 3 of the 32-column sub-tile
        const int fi = lane & 15, fg = lane >> 4;
        const int frow = 8 * (fg >> 1) + (fi >> 2);
        const int fcol = 16 * (fg & 1) + 4 * (fi & 3);
// Stages are loaded in ascending order: the pointers walk 64 rows per call; only a stage that
// reaches past the expert's last row (the last one) clamps its rows and zeroes the surplus.
#define WG_LOADG(kt_, AR, BR)                                                                   \
    {                                                                                           \
        const int rbase_ = r0 + (kt_) * kBK;                                                    \
        if (rbase_ + kBK <= r1) {                                                               \
            _Pragma("unroll") for (int q = 0; q < V; ++q)                                       \
            {                                                                                   \
                AR[q] = *reinterpret_cast<const u32x4 *>(a_ptr[q]);                             \
                BR[q] = *reinterpret_cast<const u32x4 *>(b_ptr[q]);                             \
                a_ptr[q] += a_step;                                                             \
                b_ptr[q] += b_step;                                                             \
            }                                                                                   \
        } else {                                                                                \
            _Pragma("unroll") for (int q = 0; q < V; ++q)                                       \
            {                                                                                   \
                const int row_ = rbase_ + st_row[q];                                            \
                const size_t at_ = static_cast<size_t>(min(row_, r1 - 1));                      \
                AR[q] = *reinterpret_cast<const u32x4 *>(A + at_ * M + a_col[q]);               \
                BR[q] = *reinterpret_cast<const u32x4 *>(B + at_ * N + b_col[q]);               \
                if (row_ >= r1) {                                                               \
                    AR[q] = (u32x4){0u, 0u, 0u, 0u};                                            \
                    BR[q] = (u32x4){0u, 0u, 0u, 0u};                                            \
                }                                                                               \
            }                                                                                   \
        }                                                                                       \
    }
#define WG_STOREL(buf, AR, BR)                                                                  \
    {                                                                                           \
        _Pragma("unroll") for (int q = 0; q < V; ++q)                                           \
        {                                                                                       \
            u32x4 av_ = AR[q];                                                                  \
            if constexpr (AF16)                                                                 \
                av_ = (u32x4){f16x2_to_bf16x2(av_[0]), f16x2_to_bf16x2(av_[1]),                 \
                              f16x2_to_bf16x2(av_[2]), f16x2_to_bf16x2(av_[3])};                \
            *reinterpret_cast<u32x4 *>(As + (buf) * kBuf + st_off[q]) = av_;                    \
            *reinterpret_cast<u32x4 *>(Bs + (buf) * kBuf + st_off[q]) = BR[q];                  \
        }                                                                                       \
    }
// eight consecutive rows of one column per lane: two transposing reads, four rows each
#define WG_FRAG(dst, base, cb, ks)                                                              \
    {                                                                                           \
        const int col_ = (cb) + fcol;                                                           \
        const int k_ = (ks) * 16 + frow;                                                        \
        const int lo_ = (k_ * kRowB + (((col_ >> 5) ^ (k_ & 3)) << 6) + ((col_ & 31) << 1)) >> 1; \
        const u32x2 l_ = lds_read_tr16((base) + lo_);                                           \
        const u32x2 h_ = lds_read_tr16((base) + lo_ + 4 * kTile);                               \
        dst = (u32x4){l_[0], l_[1], h_[0], h_[1]};                                              \
    }
#define WG_READF(slot_, buf, ks)                                                                \
    {                                                                                           \
        _Pragma("unroll") for (int i = 0; i < TN; ++i)                                          \
            WG_FRAG(bf[slot_][i], Bs + (buf) * kBuf, (wn * TN + i) * 32, ks)                    \
        _Pragma("unroll") for (int j = 0; j < TM; ++j)                                          \
            WG_FRAG(af[slot_][j], As + (buf) * kBuf, (wm * TM + j) * 32, ks)                    \
    }
#define WG_MMA(slot_)                                                                           \
    {                                                                                           \
        _Pragma("unroll") for (int j = 0; j < TM; ++j)                                          \
            _Pragma("unroll") for (int i = 0; i < TN; ++i)                                      \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                            \
                    __builtin_bit_cast(bf16x8, bf[slot_][i]),                                   \
                    __builtin_bit_cast(bf16x8, af[slot_][j]), acc[i][j], 0, 0, 0);              \
    }
#define WG_STAGE(buf, AR, BR)                                                                   \
    {                                                                                           \
        const bool next1 = kt + 1 < KT, next3 = kt + 3 < KT;                                    \
        if (next1) WG_STOREL(buf ^ 1, AR, BR)                                                   \
        if (next3) WG_LOADG(kt + 3, AR, BR)                                                     \
        WG_READF(1, buf, 1)                                                                     \
        WG_MMA(0)                                                                               \
        WG_READF(0, buf, 2)                                                                     \
        WG_MMA(1)                                                                               \
        WG_READF(1, buf, 3)                                                                     \
        WG_MMA(0)                                                                               \
        __syncthreads();                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                      \
        if (next1) WG_READF(0, buf ^ 1, 0)                                                      \
        WG_MMA(1)                                                                               \
    }
        WG_LOADG(0, a_reg, b_reg)
        WG_STOREL(0, a_reg, b_reg)
        if (KT > 1) WG_LOADG(1, a_reg, b_reg)
        if (KT > 2) WG_LOADG(2, a_reg2, b_reg2)
        __syncthreads();
        WG_READF(0, 0, 0)
        int kt = 0;
        for (; kt + 1 < KT; kt += 2) {
            WG_STAGE(0, a_reg, b_reg)
            ++kt;
            WG_STAGE(1, a_reg2, b_reg2)
            --kt;
        }
        if (kt < KT) WG_STAGE(0, a_reg, b_reg)
#undef WG_STAGE
#undef WG_LOADG
#undef WG_STOREL
#undef WG_FRAG
#undef WG_READF
#undef WG_MMA
    }

    // acc[i][j][4*g + c]: column n0 + (wn*TN + i)*32 + 8*g + 4*(lane/32) + c,
    //                     row m0 + (wm*TM + j)*32 + lane%32
    float *Ce = C + static_cast<size_t>(expert) * M * N;
    const int fr = lane & 31;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m0 + (wm * TM + j) * 32 + fr;
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + (wn * TN + i) * 32 + 8 * g + 4 * (lane >> 5);
                if (n >= N) continue;
                *reinterpret_cast<float4 *>(Ce + static_cast<size_t>(m) * N + n) =
                    make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                                acc[i][j][4 * g + 3]);
            }
        }
    }
}

// ---------------------------------------------------------------- weight gradient, 256 x 256 tiles
// The same product on the four-wavefront layout of gemm_w4.h, for layers whose weight
// gradients have enough 256 x 256 tiles: four wavefronts of 128 x 128 with their accumulators in
// AGPRs, two 64-row stages of buffer loads in flight in registers, double-buffered LDS stages
// [64 rows][256 columns] per operand (64-byte pieces XOR-swizzled with the row, as above), the
// MFMA fragments through the transposing LDS read, every memory instruction issued between
// MFMAs in a fixed order.  The operands' buffer resources end with the expert's last row, so
// rows past it -- and whole stages past the last one -- read as zeros: no clamping, no tail
// code.  M and N are multiples of 256 (the host checks).
template <bool AF16>
__global__ __launch_bounds__(256, 1) void wgrad_w4_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, float *__restrict__ C,
    const int32_t *__restrict__ offsets, int E, int M, int N, int tiles_m, int tiles_n)
{
    constexpr int TM = 4, TN = 4, NV = 8;
    constexpr int kRow = 512;                     // bytes of a 256-column LDS row
    constexpr int kOp = 64 * kRow;                // bytes of one operand's stage
    int expert, m0, n0;
    {
        const int total = E * tiles_m * tiles_n;
        const int per_xcd = (total + 7) / 8;
        const int slot = blockIdx.x / 8;
        const int idx = (blockIdx.x % 8) * per_xcd + slot;
        if (slot >= per_xcd || idx >= total) return;
        expert = idx / (tiles_m * tiles_n);
        const int rem = idx % (tiles_m * tiles_n);
        m0 = (rem / tiles_n) * 256;
        n0 = (rem % tiles_n) * 256;
    }
    const int r0 = offsets[expert], r1 = offsets[expert + 1];
    const int KT = (r1 - r0 + 63) / 64;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    char *lds = reinterpret_cast<char *>(smem);   // A stages at 0 and kOp, B stages at 2 kOp and 3 kOp
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    if (KT > 0) {
        // an operand's resource: from the tile's first column of the expert's first row to the end
        // of the expert's last row
        const unsigned rows = static_cast<unsigned>(r1 - r0);
        const __amdgpu_buffer_rsrc_t rsa = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(A + static_cast<size_t>(r0) * M + m0), 0,
            (rows * static_cast<unsigned>(M) - static_cast<unsigned>(m0)) * 2u, 0x00020000);
        const __amdgpu_buffer_rsrc_t rsb = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(B + static_cast<size_t>(r0) * N + n0), 0,
            (rows * static_cast<unsigned>(N) - static_cast<unsigned>(n0)) * 2u, 0x00020000);
        // staging: vector q of a stage is row tid / 32 + 8 q, 16-byte piece tid % 32 of the row
        const int srow = tid >> 5, piece = tid & 31;
        const int a_voff = (srow * M + piece * 8) * 2, b_voff = (srow * N + piece * 8) * 2;
        const int a_rowstep = 8 * M * 2, b_rowstep = 8 * N * 2;       // vector q -> q + 1
        const int a_stage = 64 * M * 2, b_stage = 64 * N * 2;         // stage kt -> kt + 1
        const int st_off = srow * kRow + (((piece >> 2) ^ (srow & 3)) << 6) + ((piece & 3) << 4);
        // fragments: lane = 16 g + i reads row 8 (g / 2) + i / 4 (+ 4 for the upper half) of the
        // 16-row step, columns 16 (g % 2) + 4 (i % 4) .. + 3 of the 32-column sub-tile t, whose
        // 64-byte piece sits at (t ^ swizzle) inside the wavefront's 256-byte half of the row
        const int fi = lane & 15, fg = lane >> 4;
        const int frow = 8 * (fg >> 1) + (fi >> 2), fcol = 16 * (fg & 1) + 4 * (fi & 3), fswz = fi >> 2;
        int a_fr[TM], b_fr[TN];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            a_fr[t] = frow * kRow + wm * 256 + ((t ^ fswz) << 6) + fcol * 2;
            b_fr[t] = 2 * kOp + frow * kRow + wn * 256 + ((t ^ fswz) << 6) + fcol * 2;
        }
        u32x4 ra[2][NV], rb[2][NV];
        u32x4 bf[2][TN], af[2][TM];
// (the whole offset goes into the per-lane operand: the range check that turns rows past the
// expert's end into zeros does not see the scalar offset)
#define WG4_LDA(set, q, kt_)                                                                      \
    ra[set][q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(                \
                                               rsa, a_voff + ((kt_) * a_stage + (q) * a_rowstep), 0, 0))
#define WG4_LDB(set, q, kt_)                                                                      \
    rb[set][q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(                \
                                               rsb, b_voff + ((kt_) * b_stage + (q) * b_rowstep), 0, 0))
#define WG4_STA(set, q, buf)                                                                      \
    {                                                                                            \
        u32x4 av_ = ra[set][q];                                                                  \
        if constexpr (AF16)                                                                      \
            av_ = (u32x4){f16x2_to_bf16x2(av_[0]), f16x2_to_bf16x2(av_[1]),                      \
                          f16x2_to_bf16x2(av_[2]), f16x2_to_bf16x2(av_[3])};                     \
        *reinterpret_cast<u32x4 *>(lds + (buf) * kOp + st_off + (q) * 8 * kRow) = av_;           \
    }
#define WG4_STB(set, q, buf)                                                                      \
    *reinterpret_cast<u32x4 *>(lds + (2 + (buf)) * kOp + st_off + (q) * 8 * kRow) = rb[set][q]
// half h (0: rows k .. k + 3, 1: rows k + 4 .. k + 7 of the lane's eight) of fragment t, step ks
#define WG4_RDA(slot_, t, h, buf, ks)                                                             \
    {                                                                                            \
        const u32x2 v_ = lds_read_tr16(reinterpret_cast<const uint16_t *>(                      \
            lds + a_fr[t] + (buf) * kOp + (ks) * 16 * kRow + (h) * 4 * kRow));                   \
        af[slot_][t][2 * (h)] = v_[0];                                                           \
        af[slot_][t][2 * (h) + 1] = v_[1];                                                       \
    }
#define WG4_RDB(slot_, t, h, buf, ks)                                                             \
    {                                                                                            \
        const u32x2 v_ = lds_read_tr16(reinterpret_cast<const uint16_t *>(                      \
            lds + b_fr[t] + (buf) * kOp + (ks) * 16 * kRow + (h) * 4 * kRow));                   \
        bf[slot_][t][2 * (h)] = v_[0];                                                           \
        bf[slot_][t][2 * (h) + 1] = v_[1];                                                       \
    }
// read v (0 .. 15) of a step: B fragments first (v < 8), halves interleaved
#define WG4_RD(slot_, v, buf, ks)                                                                 \
    do {                                                                                         \
        if constexpr ((v) < 8) WG4_RDB(slot_, (v) >> 1, (v) & 1, buf, ks)                        \
        else WG4_RDA(slot_, ((v) - 8) >> 1, (v) & 1, buf, ks)                                    \
    } while (0)
#define WG4_WR(set, v, buf)                                                                       \
    do {                                                                                         \
        if constexpr ((v) < 8) WG4_STA(set, (v), buf) else WG4_STB(set, (v) - 8, buf);           \
    } while (0)
#define WG4_LD(set, v, kt_)                                                                       \
    do {                                                                                         \
        if constexpr ((v) < 8) WG4_LDA(set, (v), kt_); else WG4_LDB(set, (v) - 8, kt_);          \
    } while (0)
#define WG4_MM(slot_, m)                                                                          \
    do {                                                                                         \
        constexpr int i_ = (m) & 3, j_ = (m) >> 2;                                               \
        mfma_32x32x16_agpr<false>(acc[i_][j_], bf[slot_][i_], af[slot_][j_]);                    \
    } while (0)
// MFMA m, the fragment read m of the next step, and after every second MFMA one of the eight
// write / load instructions of the step
#define WG4_PAIR(slot_, m, F)                                                                     \
    WG4_MM(slot_, m);                                                                            \
    F(std::integral_constant<int, (m)>{});                                                       \
    if constexpr (((m) & 1) != 0) F(std::integral_constant<int, 16 + ((m) >> 1)>{});             \
    MOE_SB();
#define WG4_KSTEP(slot_, F)                                                                       \
    {                                                                                            \
        WG4_PAIR(slot_, 0, F) WG4_PAIR(slot_, 1, F) WG4_PAIR(slot_, 2, F) WG4_PAIR(slot_, 3, F)   \
        WG4_PAIR(slot_, 4, F) WG4_PAIR(slot_, 5, F) WG4_PAIR(slot_, 6, F) WG4_PAIR(slot_, 7, F)   \
        WG4_PAIR(slot_, 8, F) WG4_PAIR(slot_, 9, F) WG4_PAIR(slot_, 10, F) WG4_PAIR(slot_, 11, F) \
        WG4_PAIR(slot_, 12, F) WG4_PAIR(slot_, 13, F) WG4_PAIR(slot_, 14, F) WG4_PAIR(slot_, 15, F) \
    }
// Stage kt from LDS buffer kt & 1; register set SET (stage kt + 1) goes to the other buffer
// (writes 6 / 5 / 5 over steps 0 .. 2) and is refilled with stage kt + 3 (loads 2 / 3 / 3 / 8).
#define WG4_STAGE(kt_, SET)                                                                       \
    {                                                                                            \
        const int kt = (kt_);                                                                    \
        const int buf = kt & 1;                                                                  \
        {                                                                                        \
            auto mem0 = [&](auto mc) {                                                           \
                constexpr int m = decltype(mc)::value;                                           \
                if constexpr (m < 16) WG4_RD(1, m, buf, 1);                                      \
                else if constexpr (m < 22) WG4_WR(SET, m - 16, buf ^ 1);                         \
                else WG4_LD(SET, m - 22, kt + 3);                                                \
            };                                                                                   \
            WG4_KSTEP(0, mem0)                                                                   \
        }                                                                                        \
        {                                                                                        \
            auto mem1 = [&](auto mc) {                                                           \
                constexpr int m = decltype(mc)::value;                                           \
                if constexpr (m < 16) WG4_RD(0, m, buf, 2);                                      \
                else if constexpr (m < 21) WG4_WR(SET, m - 16 + 6, buf ^ 1);                     \
                else WG4_LD(SET, m - 21 + 2, kt + 3);                                            \
            };                                                                                   \
            WG4_KSTEP(1, mem1)                                                                   \
        }                                                                                        \
        {                                                                                        \
            auto mem2 = [&](auto mc) {                                                           \
                constexpr int m = decltype(mc)::value;                                           \
                if constexpr (m < 16) WG4_RD(1, m, buf, 3);                                      \
                else if constexpr (m < 21) WG4_WR(SET, m - 16 + 11, buf ^ 1);                    \
                else WG4_LD(SET, m - 21 + 5, kt + 3);                                            \
            };                                                                                   \
            WG4_KSTEP(0, mem2)                                                                   \
        }                                                                                        \
        MOE_LGKM0();                                                                             \
        MOE_BAR();                                                                               \
        {                                                                                        \
            auto mem3 = [&](auto mc) {                                                           \
                constexpr int m = decltype(mc)::value;                                           \
                if constexpr (m < 16) WG4_RD(0, m, buf ^ 1, 0);                                  \
                else WG4_LD(SET, m - 16 + 8, kt + 3);                                            \
            };                                                                                   \
            WG4_KSTEP(1, mem3)                                                                   \
        }                                                                                        \
    }
        // prologue: stage 0 through set 0 into LDS buffer 0, stage 1 in set 1, stage 2 in set 0
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            WG4_LDA(0, q, 0);
            WG4_LDB(0, q, 0);
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            WG4_LDA(1, q, 1);
            WG4_LDB(1, q, 1);
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            WG4_STA(0, q, 0)
            WG4_STB(0, q, 0);
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            WG4_LDA(0, q, 2);
            WG4_LDB(0, q, 2);
        }
        MOE_LGKM0();
        MOE_BAR();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            WG4_RDB(0, t, 0, 0, 0)
            WG4_RDB(0, t, 1, 0, 0)
            WG4_RDA(0, t, 0, 0, 0)
            WG4_RDA(0, t, 1, 0, 0)
        }
        {
            int k2 = 0;
            for (; k2 + 1 < KT; k2 += 2) {
                WG4_STAGE(k2, 1)
                WG4_STAGE(k2 + 1, 0)
            }
            if (k2 < KT) WG4_STAGE(k2, 1)
        }
#undef WG4_STAGE
#undef WG4_KSTEP
#undef WG4_PAIR
#undef WG4_MM
#undef WG4_LD
#undef WG4_WR
#undef WG4_RD
#undef WG4_RDB
#undef WG4_RDA
#undef WG4_STB
#undef WG4_STA
#undef WG4_LDB
#undef WG4_LDA
        MOE_LGKM0();
        MOE_BAR();
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    }

    // acc[i][j][4*g + c]: column n0 + (wn*TN + i)*32 + 8*g + 4*(lane/32) + c,
    //                     row m0 + (wm*TM + j)*32 + lane%32.
    // The tile leaves through LDS, 32 columns of the wavefront's 128 x 128 at a time (a patch of
    // 128 rows, pitch 144 bytes, per wavefront), as whole 128-byte lines, 16 bytes per lane:
    // stores straight from the registers would put 32 bytes into each of 32 lines per instruction.
    float *Ce = C + static_cast<size_t>(expert) * M * N;
    const int fr = lane & 31;
    constexpr int PITCH = 144;
    char *patch = reinterpret_cast<char *>(smem) + wave * (TM * 32) * PITCH;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
#pragma unroll
            for (int j = 0; j < TM; ++j)
                *reinterpret_cast<float4 *>(patch + (j * 32 + fr) * PITCH + (8 * g + 4 * (lane >> 5)) * 4) =
                    make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                                acc[i][j][4 * g + 3]);
            MOE_SB();      // a few accumulator registers at a time leave the AGPRs
        }
        MOE_LGKM0();
        __builtin_amdgcn_wave_barrier();
        const int n = n0 + (wn * TN + i) * 32 + (lane & 7) * 4;
#pragma unroll 8
        for (int it = 0; it < TM * 4; ++it) {
            const int rr = it * 8 + (lane >> 3);
            const float4 q = *reinterpret_cast<const float4 *>(patch + rr * PITCH + (lane & 7) * 16);
            *reinterpret_cast<float4 *>(Ce + static_cast<size_t>(m0 + wm * TM * 32 + rr) * N + n) = q;
        }
        MOE_LGKM0();
        __builtin_amdgcn_wave_barrier();
    }
}

// ---------------------------------------------------------------- gate backward
// One wavefront per token.  Logits: lane = four consecutive columns of the model dimension,
// EP partial sums per lane (Wgp is the forward's packed gate matrix, fp32 [EP][dP],
// expert-major, zero padded), then a butterfly sum per expert; the order of the additions
// differs from the forward's chain, which only the top-k decision needed.  Softmax, dz with
// lane = expert, and finally, lane = column again,
// dx[t, i] = sum of the token's kept dxe rows + sum_e dz[e] Wg[i, e].
// MODE 1: the gate matrix (EP x d floats, at most 64 KiB) is copied to LDS once per block of
// 16 wavefronts (16 tokens) and read from there -- a wavefront that reads the matrix twice
// per token from the caches moves 8 EP d bytes per token through the L1, which is what
// bounded the kernel.  (Still one token per wavefront and four wavefronts per SIMD: the
// token's own chain of loads, butterflies and stores is covered by the other wavefronts.)
// MODE 2: a larger matrix goes through LDS in chunks of 64 KiB of its columns, once for the
// logits and once more for dx; every wavefront of the block walks all chunks (those without a
// token only stage and wait).
template <int EP, int MODE>
__global__ __launch_bounds__(MODE != 0 ? 1024 : 256) void gate_bwd_kernel(
    const uint16_t *__restrict__ x, const float *__restrict__ Wgp, const float *__restrict__ bias,
    int bias_stride, const int32_t *__restrict__ expert_idx, const int32_t *__restrict__ slot_of,
    const float *__restrict__ dgate, const float *__restrict__ dxe, float *__restrict__ dz,
    float *__restrict__ dx, int t0, int T, int d, int dP, int E, int k, int max_rows)
{   // tokens [t0, T).  MODE 0: the matrix from the caches; 1: staged whole in LDS; 2: staged in
    // chunks of DC columns, once for the logits and once for dx
    constexpr int NW = MODE != 0 ? 16 : 4;                           // wavefronts per block
    constexpr int DC = 16384 / EP >= 256 ? 16384 / EP : 256;         // columns per 64 KiB chunk (MODE 2)
    __shared__ float dzs[NW][kWave];
    extern __shared__ __attribute__((aligned(16))) float wlds[];     // MODE 1: [EP][d]; 2: [EP][DC]
    const int lane = lane_id();
    const int w = threadIdx.x / kWave;
    const float *Wsrc = Wgp;
    int wpitch = dP;
    if constexpr (MODE == 1) {
        const int rv = d / 4;                                        // 16-byte vectors per row
        for (int v = threadIdx.x; v < EP * rv; v += NW * kWave) {
            const int e = v / rv, i = (v % rv) * 4;
            *reinterpret_cast<float4 *>(wlds + e * d + i) =
                *reinterpret_cast<const float4 *>(Wgp + static_cast<size_t>(e) * dP + i);
        }
        __syncthreads();
        Wsrc = wlds;
        wpitch = d;
    }
    const int t = t0 + blockIdx.x * NW + w;
    const bool valid = t < T;
    if (MODE != 2 && !valid) return;
    // columns [c0, c0 + DC) of the packed matrix (zero padded up to dP) into LDS, all wavefronts
    auto stage_chunk = [&](int c0) {
        __syncthreads();
        constexpr int rv = DC / 4;
        for (int v = threadIdx.x; v < EP * rv; v += NW * kWave) {
            const int e = v / rv, i = (v % rv) * 4;
            float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c0 + i < dP) q = *reinterpret_cast<const float4 *>(Wgp + static_cast<size_t>(e) * dP + c0 + i);
            *reinterpret_cast<float4 *>(wlds + e * DC + i) = q;
        }
        __syncthreads();
    };
    const uint16_t *xrow = x + static_cast<size_t>(valid ? t : 0) * d;
    float acc[EP];
#pragma unroll
    for (int e = 0; e < EP; ++e) acc[e] = 0.0f;
    auto logits_part = [&](const float *wbase, int pitch, int i, int iw) {    // columns i .. i + 3 (iw: in wbase)
        const u32x2 xq = *reinterpret_cast<const u32x2 *>(xrow + i);
        const float x0 = __uint_as_float(xq[0] << 16), x1 = __uint_as_float(xq[0] & 0xFFFF0000u);
        const float x2 = __uint_as_float(xq[1] << 16), x3 = __uint_as_float(xq[1] & 0xFFFF0000u);
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            const float4 wv = *reinterpret_cast<const float4 *>(wbase + static_cast<size_t>(e) * pitch + iw);
            acc[e] = __builtin_fmaf(x0, wv.x, acc[e]);
            acc[e] = __builtin_fmaf(x1, wv.y, acc[e]);
            acc[e] = __builtin_fmaf(x2, wv.z, acc[e]);
            acc[e] = __builtin_fmaf(x3, wv.w, acc[e]);
        }
    };
    if constexpr (MODE == 2) {
        for (int c0 = 0; c0 < d; c0 += DC) {
            stage_chunk(c0);
            if (valid)
                for (int il = lane * 4; il < DC && c0 + il < d; il += kWave * 4)
                    logits_part(wlds, DC, c0 + il, il);
        }
    } else {
        for (int i = lane * 4; i < d; i += kWave * 4) logits_part(Wsrc, wpitch, i, i);
    }
    float z = 0.0f;
#pragma unroll
    for (int e = 0; e < EP; ++e) {
        float v = acc[e];
#pragma unroll
        for (int m = kWave / 2; m > 0; m >>= 1) v += __shfl_xor(v, m);
        if (lane == e) z = v;
    }
    const int e = lane;
    const bool live = e < E;
    const int tt = valid ? t : 0;
    if (bias != nullptr && live) z += bias[static_cast<size_t>(tt) * bias_stride + e];
    float zmax = live ? z : -3.0e38f;
#pragma unroll
    for (int m = kWave / 2; m > 0; m >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, m));
    float p = live ? expf(z - zmax) : 0.0f;
    float denom = p;
#pragma unroll
    for (int m = kWave / 2; m > 0; m >>= 1) denom += __shfl_xor(denom, m);
    p /= denom;
    float dg = 0.0f;
    if (live)
        for (int j = 0; j < k; ++j)
            if (expert_idx[static_cast<size_t>(tt) * k + j] == e) dg = dgate[static_cast<size_t>(tt) * k + j];
    float s = p * dg;
#pragma unroll
    for (int m = kWave / 2; m > 0; m >>= 1) s += __shfl_xor(s, m);
    const float dze = p * (dg - s);
    if (live && valid) dz[static_cast<size_t>(t) * E + e] = dze;
    dzs[w][lane] = live ? dze : 0.0f;
    __builtin_amdgcn_wave_barrier();
    float dzr[EP];
#pragma unroll
    for (int ee = 0; ee < EP; ++ee) dzr[ee] = dzs[w][ee];
    auto dx_part = [&](const float *wbase, int pitch, int i, int iw) {
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 0; j < k; ++j) {
            const int slot = slot_of[static_cast<size_t>(t) * k + j];
            if (slot >= 0 && slot < max_rows) {
                const float4 r = *reinterpret_cast<const float4 *>(dxe + static_cast<size_t>(slot) * d + i);
                o.x += r.x; o.y += r.y; o.z += r.z; o.w += r.w;
            }
        }
#pragma unroll
        for (int ee = 0; ee < EP; ++ee) {
            const float4 wv = *reinterpret_cast<const float4 *>(wbase + static_cast<size_t>(ee) * pitch + iw);
            o.x = __builtin_fmaf(dzr[ee], wv.x, o.x);
            o.y = __builtin_fmaf(dzr[ee], wv.y, o.y);
            o.z = __builtin_fmaf(dzr[ee], wv.z, o.z);
            o.w = __builtin_fmaf(dzr[ee], wv.w, o.w);
        }
        *reinterpret_cast<float4 *>(dx + static_cast<size_t>(t) * d + i) = o;
    };
    if constexpr (MODE == 2) {
        for (int c0 = 0; c0 < d; c0 += DC) {
            stage_chunk(c0);
            if (valid)
                for (int il = lane * 4; il < DC && c0 + il < d; il += kWave * 4)
                    dx_part(wlds, DC, c0 + il, il);
        }
    } else {
        for (int i = lane * 4; i < d; i += kWave * 4) dx_part(Wsrc, wpitch, i, i);
    }
}

// partial[s][i][e] = sum over the tokens of range s of x[t, i] dz[t, e].  Block = 64 columns
// i x 4 expert groups of EQ = EP / 4 experts (EP < 4: one expert per group, surplus groups
// idle); tokens go through LDS 64 at a time.
template <int EP>
__global__ __launch_bounds__(256) void dwg_partial_kernel(
    const uint16_t *__restrict__ x, const float *__restrict__ dz, float *__restrict__ partial, int T,
    int d, int E, int per_split)
{
    constexpr int EQ = EP >= 4 ? EP / 4 : 1;
    __shared__ float xs[64][65];
    __shared__ float zs[64][EP + 1];
    const int il = threadIdx.x % 64, eg = threadIdx.x / 64;
    const int i0 = blockIdx.x * 64;
    const int e0 = eg * EQ;
    const int t0 = blockIdx.y * per_split, t1 = min(T, t0 + per_split);
    float acc[EQ];
#pragma unroll
    for (int q = 0; q < EQ; ++q) acc[q] = 0.0f;
    for (int tb = t0; tb < t1; tb += 64) {
        __syncthreads();
        for (int v = threadIdx.x; v < 64 * 8; v += 256) {          // eight columns per load
            const int tt = v / 8, c8 = (v % 8) * 8;
            u32x4 q = {0u, 0u, 0u, 0u};
            if (tb + tt < t1 && i0 + c8 < d)
                q = *reinterpret_cast<const u32x4 *>(x + static_cast<size_t>(tb + tt) * d + i0 + c8);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                xs[tt][c8 + 2 * c] = __uint_as_float(q[c] << 16);
                xs[tt][c8 + 2 * c + 1] = __uint_as_float(q[c] & 0xFFFF0000u);
            }
        }
        for (int v = threadIdx.x; v < 64 * EP; v += 256) {
            const int tt = v / EP, ee = v % EP;
            zs[tt][ee] = (tb + tt < t1 && ee < E) ? dz[static_cast<size_t>(tb + tt) * E + ee] : 0.0f;
        }
        __syncthreads();
        if (e0 < EP) {
#pragma unroll 8
            for (int tt = 0; tt < 64; ++tt) {
                const float xv = xs[tt][il];
#pragma unroll
                for (int q = 0; q < EQ; ++q) acc[q] = __builtin_fmaf(xv, zs[tt][e0 + q], acc[q]);
            }
        }
    }
    if (i0 + il < d && e0 < EP) {
#pragma unroll
        for (int q = 0; q < EQ; ++q)
            if (e0 + q < E)
                partial[(static_cast<size_t>(blockIdx.y) * d + i0 + il) * E + e0 + q] = acc[q];
    }
}

__global__ void dwg_reduce_kernel(const float *__restrict__ partial, float *__restrict__ dWg, int n,
                                  int splits)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    float acc = 0.0f;
#pragma unroll 8
    for (int s = 0; s < splits; ++s) acc += partial[static_cast<size_t>(s) * n + idx];
    dWg[idx] = acc;
}

// ---------------------------------------------------------------- host side
struct BwdWorkspace {
    Workspace lists;          // work lists of the two row-grouped GEMM shapes
    _Float16 *P;              // [R][h]
    uint16_t *Hb, *dye, *dP;  // [R][h], [R][d], [R][h]
    float *dxe;               // [R][d]
    float *dz, *partial;      // [T][E], [splits][d][E]
    int splits, per_split;
    size_t bytes;
};

// 256 x 256 tiles (the four-wavefront kernel) when there are enough of them to fill the chip,
// as in the forward; else 128-row tiles, 256 columns wide when the contraction is long enough
// to pay for the larger tile's prologue, else 128
GemmPlan plan_rows(int N, int K, int64_t max_rows, int E)
{
    GemmPlan gp;
    const int64_t big_tiles = (max_rows / 256 + E / 2) * ((N + 255) / 256);
    const bool fits = K % 64 == 0 && static_cast<uint64_t>(N) * K * 2 < (1ull << 31) &&
                      256ull * K * 2 < (1ull << 31);
    if (big_tiles >= 768 && fits) {
        gp.bm = 256;
        gp.bn = 256;
        gp.concurrent = 32;
    } else {
        gp.bm = kBM;
        gp.bn = (K >= 2048 && N >= 256) ? 256 : 128;
        gp.concurrent = gp.bn == 256 ? 32 : 64;
    }
    gp.tiles_n = (N + gp.bn - 1) / gp.bn;
    gp.max_row_tiles = static_cast<int32_t>((max_rows + gp.bm - 1) / gp.bm + E);
    gp.max_items = gp.max_row_tiles * gp.tiles_n;
    return gp;
}

void layout_bwd(const moe_shape &s, void *base, BwdWorkspace *w)
{
    const int64_t R = moe_max_rows(&s);
    char *p = static_cast<char *>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *at = p + off;
        off += align_up(bytes, 256);
        return at;
    };
    w->lists = Workspace{};
    w->lists.gp[0] = plan_rows(s.d_ff, s.d_model, R, s.E);
    w->lists.gp[1] = plan_rows(s.d_model, s.d_ff, R, s.E);
    for (int g = 0; g < 2; ++g) {      // one list per FFN group of a chunked backward pass
        w->lists.items[g] = reinterpret_cast<WorkItem *>(
            take(sizeof(WorkItem) * w->lists.gp[g].max_items * kMaxChunks));
        w->lists.nitems[g] = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * kMaxChunks));
    }
    const size_t Rh = static_cast<size_t>(R) * s.d_ff, Rd = static_cast<size_t>(R) * s.d_model;
    w->P = reinterpret_cast<_Float16 *>(take(Rh * 2));
    w->Hb = reinterpret_cast<uint16_t *>(take(Rh * 2));
    w->dye = reinterpret_cast<uint16_t *>(take(Rd * 2));
    w->dP = reinterpret_cast<uint16_t *>(take(Rh * 2));
    w->dxe = reinterpret_cast<float *>(take(Rd * 4));
    w->dz = reinterpret_cast<float *>(take(static_cast<size_t>(s.T) * s.E * 4));
    w->splits = std::max(1, std::min(32, (s.T + 127) / 128));
    w->per_split = (s.T + w->splits - 1) / w->splits;
    w->partial = reinterpret_cast<float *>(take(static_cast<size_t>(w->splits) * s.d_model * s.E * 4));
    w->bytes = off;
}

bool supported(const moe_shape *s)
{
    if (s == nullptr || s->dtype != MOE_BF16 || s->renorm_topk != 0) return false;
    if (s->T < 1 || s->d_model < 8 || s->d_ff < 8 || s->E < 1 || s->E > kMaxExperts || s->k < 1 ||
        s->k > kMaxTopK || s->k > s->E || s->capacity < 1)
        return false;
    return s->d_model % 8 == 0 && s->d_ff % 8 == 0;
}

template <int EPI, int ACT, bool KTAIL, int WN>
void launch_gemm_k(const uint16_t *A, const uint16_t *W, void *C, _Float16 *P, const WorkItem *items,
                   const int32_t *nitems, int N, int K, int grid_items, int stage, hipStream_t st)
{
    auto kern = bwd_gemm_kernel<EPI, ACT, KTAIL, WN>;
    constexpr size_t kGemmLds = gemm_lds(WN);
    static PerDeviceOnce once;   // raising the dynamic LDS limit: once per kernel and device
    once.raise_lds(reinterpret_cast<const void *>(kern), static_cast<int>(kGemmLds));
    const int grid = static_cast<int>(align_up(static_cast<size_t>(grid_items), 8));
    hipEvent_t t0, t1;
    prof_kernel_events(stage, &t0, &t1);
    hipExtLaunchKernelGGL(kern, dim3(grid), dim3(128 * WN), kGemmLds, st, t0, t1, 0, A, W, C, P, items,
                          nitems, N, K);
}

template <int EPI, int ACT>
void launch_gemm(const uint16_t *A, const uint16_t *W, void *C, _Float16 *P, const WorkItem *items,
                 const int32_t *nitems, int N, int K, const GemmPlan &gp, int stage, hipStream_t st)
{
    const int grid_items = gp.max_items;
    if (gp.bm == 256) {
        constexpr size_t lds = 2 * (256 + 256) * (64 + 8) * sizeof(uint16_t);
        auto kern = bwd_gemm_w4_kernel<EPI, ACT>;
        static PerDeviceOnce once;
        once.raise_lds(reinterpret_cast<const void *>(kern), static_cast<int>(lds));
        const int grid = static_cast<int>(align_up(static_cast<size_t>(grid_items), 8));
        hipEvent_t t0, t1;
        prof_kernel_events(stage, &t0, &t1);
        hipExtLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, t0, t1, 0, A, W, C, P, items, nitems,
                              N, K);
        return;
    }
#define MOE_BWD_GEMM(KTAIL_, WN_)                                                                 \
    launch_gemm_k<EPI, ACT, KTAIL_, WN_>(A, W, C, P, items, nitems, N, K, grid_items, stage, st)
    const bool tail = K % kBK != 0;
    if (gp.bn == 256) {
        if (tail) MOE_BWD_GEMM(true, 4); else MOE_BWD_GEMM(false, 4);
    } else {
        if (tail) MOE_BWD_GEMM(true, 2); else MOE_BWD_GEMM(false, 2);
    }
#undef MOE_BWD_GEMM
}

// dW[e] [M][N] = A[rows of e]^T B[rows of e] from row-major operands
template <bool AF16>
void launch_wgrad(const uint16_t *A, const uint16_t *B, float *C, const int32_t *offsets, int E, int M,
                  int N, int64_t max_rows, int stage, hipStream_t st)
{
    hipEvent_t t0, t1;
    // 256 x 256 tiles on four wavefronts when they divide the matrix, fill the chip, and the
    // buffer offsets (an expert's rows times the row length, in bytes) stay below 2^31
    const uint64_t span = static_cast<uint64_t>(max_rows + 192) * static_cast<uint64_t>(std::max(M, N)) * 2;
    if (M % 256 == 0 && N % 256 == 0 && static_cast<int64_t>(E) * (M / 256) * (N / 256) >= 768 &&
        span < (1ull << 31)) {
        constexpr size_t kLds4 = 4 * 64 * 512;
        auto kern = wgrad_w4_kernel<AF16>;
        static PerDeviceOnce once;
        once.raise_lds(reinterpret_cast<const void *>(kern), static_cast<int>(kLds4));
        const int tiles_m = M / 256, tiles_n = N / 256;
        const int grid = static_cast<int>(align_up(static_cast<size_t>(E) * tiles_m * tiles_n, 8));
        prof_kernel_events(stage, &t0, &t1);
        hipExtLaunchKernelGGL(kern, dim3(grid), dim3(256), kLds4, st, t0, t1, 0, A, B, C, offsets, E, M,
                              N, tiles_m, tiles_n);
        return;
    }
    constexpr size_t kLds = 2 * 2 * kBK * 128 * sizeof(uint16_t);
    auto kern = wgrad_gemm_kernel<AF16>;
    static PerDeviceOnce once;
    once.raise_lds(reinterpret_cast<const void *>(kern), static_cast<int>(kLds));
    const int tiles_m = (M + 127) / 128, tiles_n = (N + 127) / 128;
    const int grid = static_cast<int>(align_up(static_cast<size_t>(E) * tiles_m * tiles_n, 8));
    prof_kernel_events(stage, &t0, &t1);
    hipExtLaunchKernelGGL(kern, dim3(grid), dim3(256), kLds, st, t0, t1, 0, A, B, C, offsets, E, M, N,
                          tiles_m, tiles_n);
}

// Side streams and events of a chunked backward pass, per device, kept for the process.
struct BwdResources {
    bool ready = false;
    std::mutex enqueue;                 // held while a call enqueues on the side streams
    hipStream_t grad_in = nullptr, grad_out = nullptr;
    hipEvent_t begun = nullptr, joined_in = nullptr, joined_out = nullptr;
    hipEvent_t dispatched[kMaxChunks] = {}, computed[kMaxChunks] = {};
};
std::mutex g_bwd_mutex;
BwdResources g_bwd[16];

moe_status bwd_resources(BwdResources **out)
{
    int dev = 0;
    MOE_TRY_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16) {
        set_error("device index %d out of range", dev);
        return MOE_EUNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_bwd_mutex);
    BwdResources &r = g_bwd[dev];
    if (!r.ready) {
        MOE_TRY_HIP(hipStreamCreateWithFlags(&r.grad_in, hipStreamNonBlocking));
        MOE_TRY_HIP(hipStreamCreateWithFlags(&r.grad_out, hipStreamNonBlocking));
        MOE_TRY_HIP(hipEventCreateWithFlags(&r.begun, hipEventDisableTiming));
        MOE_TRY_HIP(hipEventCreateWithFlags(&r.joined_in, hipEventDisableTiming));
        MOE_TRY_HIP(hipEventCreateWithFlags(&r.joined_out, hipEventDisableTiming));
        for (int c = 0; c < kMaxChunks; ++c) {
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.dispatched[c], hipEventDisableTiming));
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.computed[c], hipEventDisableTiming));
        }
        r.ready = true;
    }
    *out = &r;
    return MOE_OK;
}

// The backward pass, cut like the forward: tokens in n_chunks contiguous parts, the row-grouped
// GEMMs once per group of consecutive chunks (ffn_groups).  Gradient rows are dispatched to the
// expert-major order chunk by chunk on one side stream (the backward pass's first all-to-all
// carries them, Sec. 2.2), the two input-gradient GEMMs of a group start when its last chunk is
// there, and the rows that come back are folded into dx chunk by chunk on a second side stream
// (the second all-to-all) while the caller's stream goes on with the next group and then with
// the weight gradients.  Every result is the same bits for every n_chunks.
template <int ACT>
moe_status backward_t(const moe_shape &s, int n_chunks, const uint16_t *x, const float *Wgp,
                      const float *bias, int bias_stride, const uint16_t *W1, const uint16_t *W2,
                      const uint16_t *W1p, const int32_t *expert_idx, const float *gate,
                      const int32_t *offsets, const int32_t *slot_of, const int32_t *src_of,
                      const uint16_t *xe, const _Float16 *ye, const _Float16 *pre,
                      const _Float16 *hid, const float *dy, float *dx, float *dWg, float *dW1,
                      float *dW2, float *dgate, const BwdWorkspace &w, hipStream_t st)
{
    const int T = s.T, d = s.d_model, h = s.d_ff, E = s.E, k = s.k;
    const int R = static_cast<int>(moe_max_rows(&s));
    if (n_chunks > T) n_chunks = T;
    const int n_groups = ffn_groups(s, n_chunks);
    if (n_groups == 1) n_chunks = 1;
    moe_status rc = launch_items(s, n_chunks, n_groups, offsets, src_of, w.lists, st);
    if (rc != MOE_OK) return rc;
    const GemmPlan &g0 = w.lists.gp[0], &g1 = w.lists.gp[1];
    _Float16 *P = pre != nullptr ? const_cast<_Float16 *>(pre) : w.P;
    int EP = 1;
    while (EP < E) EP <<= 1;
    const int dPad = (d + 127) / 128 * 128;            // the packed gate matrix's row length
    auto bound = [&](int c) { return static_cast<int>(static_cast<int64_t>(c) * T / n_chunks); };

    // dye = g dy (bf16) and dgate = <ye, dy> for the tokens [t0, t1)
    auto grad_dispatch = [&](int t0, int t1, hipStream_t q) {
        if (t1 > t0)
            hipLaunchKernelGGL(combine_bwd_kernel, dim3(ceil_div(t1 - t0, 4)), dim3(256), 0, q, dy, ye,
                               slot_of, gate, w.dye, dgate, t0, t1, d, k, R);
    };
    // the row-grouped GEMMs of FFN group f
    auto group_gemms = [&](int f) {
        const WorkItem *it0 = w.lists.items[0] + static_cast<size_t>(f) * g0.max_items;
        const WorkItem *it1 = w.lists.items[1] + static_cast<size_t>(f) * g1.max_items;
        // P = xe W1 (fp16), Hb = act(P) (bf16) -- unless the forward kept P and its hidden activations
        if (pre == nullptr)
            launch_gemm<1, ACT>(xe, W1p, w.Hb, w.P, it0, w.lists.nitems[0] + f, h, d, g0,
                                kStageBwdRecompute, st);
        // dP = (dye W2^T) * act'(P): W2 [E][h][d] is already "rows n = h, contraction d contiguous"
        launch_gemm<2, ACT>(w.dye, W2, w.dP, P, it0, w.lists.nitems[0] + f, h, d, g0,
                            kStageBwdDP, st);
        // dxe = dP W1^T: W1 [E][d][h] is "rows n = d, contraction h contiguous"
        launch_gemm<0, ACT>(w.dP, W1, w.dxe, nullptr, it1, w.lists.nitems[1] + f, d, h, g1, kStageBwdDxe,
                            st);
    };
    // dW2[e] [h][d] = act(P)^T dye ; dW1[e] [d][h] = xe^T dP, operands as they are
    auto weight_grads = [&]() {
        if (pre != nullptr)      // the forward's own hidden activations, fp16
            launch_wgrad<true>(reinterpret_cast<const uint16_t *>(hid), w.dye, dW2, offsets, E, h, d, R,
                               kStageBwdWgrad2, st);
        else
            launch_wgrad<false>(w.Hb, w.dye, dW2, offsets, E, h, d, R, kStageBwdWgrad2, st);
        launch_wgrad<false>(xe, w.dP, dW1, offsets, E, d, h, R, kStageBwdWgrad1, st);
    };
    // gate: dz and dx for the tokens [t0, t1)
    auto grad_combine = [&](int t0, int t1, hipStream_t q) {
        if (t1 <= t0) return;
        const int n = t1 - t0;
#define MOE_GATE_BWD_CASE(EP_)                                                                    \
    if (EP == EP_) {                                                                              \
        const size_t wbytes = static_cast<size_t>(EP_) * d * sizeof(float);                       \
        if (wbytes <= 64 * 1024 && T >= 16 * 256) {                                               \
            auto kern = gate_bwd_kernel<EP_, 1>;                                                  \
            static PerDeviceOnce once;                                                            \
            once.raise_lds(reinterpret_cast<const void *>(kern), 64 * 1024);                      \
            hipLaunchKernelGGL(kern, dim3(ceil_div(n, 16)), dim3(1024), wbytes, q, x, Wgp, bias,  \
                               bias_stride, expert_idx, slot_of, dgate, w.dxe, w.dz, dx, t0, t1,  \
                               d, dPad, E, k, R);                                                 \
        } else if (wbytes > 64 * 1024 && T >= 16 * 256) {                                         \
            /* a matrix too large for LDS: 64 KiB chunks of its columns, staged per 16 tokens */  \
            auto kern = gate_bwd_kernel<EP_, 2>;                                                  \
            static PerDeviceOnce once;                                                            \
            once.raise_lds(reinterpret_cast<const void *>(kern), 64 * 1024);                      \
            hipLaunchKernelGGL(kern, dim3(ceil_div(n, 16)), dim3(1024), 64 * 1024, q, x, Wgp,     \
                               bias, bias_stride, expert_idx, slot_of, dgate, w.dxe, w.dz, dx,    \
                               t0, t1, d, dPad, E, k, R);                                         \
        } else {                                                                                  \
            hipLaunchKernelGGL((gate_bwd_kernel<EP_, 0>), dim3(ceil_div(n, 4)), dim3(256), 0,     \
                               q, x, Wgp, bias, bias_stride, expert_idx, slot_of, dgate, w.dxe,   \
                               w.dz, dx, t0, t1, d, dPad, E, k, R);                               \
        }                                                                                         \
    }
        MOE_GATE_BWD_CASE(1) MOE_GATE_BWD_CASE(2) MOE_GATE_BWD_CASE(4) MOE_GATE_BWD_CASE(8)
        MOE_GATE_BWD_CASE(16) MOE_GATE_BWD_CASE(32) MOE_GATE_BWD_CASE(64)
#undef MOE_GATE_BWD_CASE
    };
    // dWg = x^T dz: partial sums over fixed token ranges, then a fixed-order sum
    auto gate_weight_grad = [&]() {
#define MOE_DWG_CASE(EP_)                                                                         \
    if (EP == EP_)                                                                                \
        hipLaunchKernelGGL(dwg_partial_kernel<EP_>, dim3(ceil_div(d, 64), w.splits), dim3(256), 0, \
                           st, x, w.dz, w.partial, T, d, E, w.per_split);
        MOE_DWG_CASE(1) MOE_DWG_CASE(2) MOE_DWG_CASE(4) MOE_DWG_CASE(8)
        MOE_DWG_CASE(16) MOE_DWG_CASE(32) MOE_DWG_CASE(64)
#undef MOE_DWG_CASE
        hipLaunchKernelGGL(dwg_reduce_kernel, dim3(ceil_div(d * E, 256)), dim3(256), 0, st, w.partial,
                           dWg, d * E, w.splits);
    };

    if (n_chunks == 1) {
        grad_dispatch(0, T, st);
        group_gemms(0);
        weight_grads();
        grad_combine(0, T, st);
        gate_weight_grad();
        MOE_TRY_HIP(hipGetLastError());
        return MOE_OK;
    }

    BwdResources *r = nullptr;
    rc = bwd_resources(&r);
    if (rc != MOE_OK) return rc;
    std::lock_guard<std::mutex> enqueue(r->enqueue);
    MOE_TRY_HIP(hipEventRecord(r->begun, st));
    MOE_TRY_HIP(hipStreamWaitEvent(r->grad_in, r->begun, 0));
    MOE_TRY_HIP(hipStreamWaitEvent(r->grad_out, r->begun, 0));
    auto enqueue_chunks = [&]() -> moe_status {
        for (int c = 0; c < n_chunks; ++c) {
            grad_dispatch(bound(c), bound(c + 1), r->grad_in);
            MOE_TRY_HIP(hipEventRecord(r->dispatched[c], r->grad_in));
        }
        for (int f = 0; f < n_groups; ++f) {
            const int c0 = static_cast<int>(static_cast<int64_t>(f) * n_chunks / n_groups);
            const int c1 = static_cast<int>(static_cast<int64_t>(f + 1) * n_chunks / n_groups);
            MOE_TRY_HIP(hipStreamWaitEvent(st, r->dispatched[c1 - 1], 0));
            group_gemms(f);
            MOE_TRY_HIP(hipEventRecord(r->computed[f], st));
            MOE_TRY_HIP(hipStreamWaitEvent(r->grad_out, r->computed[f], 0));
            for (int c = c0; c < c1; ++c) grad_combine(bound(c), bound(c + 1), r->grad_out);
        }
        weight_grads();
        return MOE_OK;
    };
    rc = enqueue_chunks();
    // join both side streams (also after a failure part-way), then the gate matrix's gradient,
    // which needs every token's dz
    hipError_t je = hipEventRecord(r->joined_in, r->grad_in);
    if (je == hipSuccess) je = hipStreamWaitEvent(st, r->joined_in, 0);
    if (je == hipSuccess) je = hipEventRecord(r->joined_out, r->grad_out);
    if (je == hipSuccess) je = hipStreamWaitEvent(st, r->joined_out, 0);
    if (rc != MOE_OK) return rc;
    if (je != hipSuccess) return hip_fail(je, "joining the side streams");
    gate_weight_grad();
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

size_t moe_backward_workspace_bytes(const moe_shape *s)
{
    if (!supported(s)) return 0;
    BwdWorkspace w;
    layout_bwd(*s, reinterpret_cast<void *>(static_cast<uintptr_t>(256)), &w);   // sizes only
    return w.bytes;
}

moe_status moe_layer_backward(const moe_shape *s, const void *x, const void *Wgp,
                              const float *gate_bias, int32_t bias_token_stride,
                              const void *W1, const void *W2, const void *W1p,
                              const int32_t *expert_idx, const float *gate,
                              const int32_t *offsets, const int32_t *slot_of,
                              const int32_t *src_of, const void *xe, const void *ye,
                              const void *pre, const void *hid, const float *dy, float *dx,
                              float *dWg, float *dW1, float *dW2, float *dgate, void *workspace,
                              void *stream)
{
    return moe_layer_backward_chunked(s, 1, x, Wgp, gate_bias, bias_token_stride, W1, W2, W1p,
                                      expert_idx, gate, offsets, slot_of, src_of, xe, ye, pre, hid, dy,
                                      dx, dWg, dW1, dW2, dgate, workspace, stream);
}

moe_status moe_layer_backward_chunked(const moe_shape *s, int32_t n_chunks, const void *x,
                                      const void *Wgp, const float *gate_bias,
                                      int32_t bias_token_stride, const void *W1, const void *W2,
                                      const void *W1p, const int32_t *expert_idx, const float *gate,
                                      const int32_t *offsets, const int32_t *slot_of,
                                      const int32_t *src_of, const void *xe, const void *ye,
                                      const void *pre, const void *hid, const float *dy, float *dx,
                                      float *dWg, float *dW1, float *dW2, float *dgate,
                                      void *workspace, void *stream)
{
    if (!supported(s)) {
        set_error("moe_layer_backward: bf16 layers without top-k renormalisation only, E <= %d, "
                  "k <= %d, d_model and d_ff multiples of 8", kMaxExperts, kMaxTopK);
        return s == nullptr ? MOE_EINVAL : MOE_EUNSUPPORTED;
    }
    if (gate_bias != nullptr && bias_token_stride != 0 && bias_token_stride != s->E) {
        set_error("bias_token_stride must be 0 or E");
        return MOE_EINVAL;
    }
    if (n_chunks < 1 || n_chunks > kMaxChunks) {
        set_error("n_chunks must be in 1..%d, got %d", kMaxChunks, n_chunks);
        return MOE_EINVAL;
    }
    const void *need[] = {x, Wgp, W1, W2, W1p, expert_idx, gate, offsets, slot_of, src_of, xe, ye, dy,
                          dx, dWg, dW1, dW2, dgate, workspace};
    for (const void *p : need) {
        if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) != 0) {
            set_error("moe_layer_backward: a required pointer is NULL or not 16-byte aligned");
            return MOE_EINVAL;
        }
    }
    if (((reinterpret_cast<uintptr_t>(pre) | reinterpret_cast<uintptr_t>(hid)) & 15u) != 0 ||
        (pre == nullptr) != (hid == nullptr)) {
        set_error("moe_layer_backward: pre and hid come together (both or neither), 16-byte aligned");
        return MOE_EINVAL;
    }
    BwdWorkspace w;
    layout_bwd(*s, workspace, &w);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const _Float16 *preh = static_cast<const _Float16 *>(pre);
    const _Float16 *hidh = static_cast<const _Float16 *>(hid);
    const uint16_t *xb = static_cast<const uint16_t *>(x);
    const float *Wgf = static_cast<const float *>(Wgp);
    const uint16_t *W1b = static_cast<const uint16_t *>(W1), *W2b = static_cast<const uint16_t *>(W2);
    const uint16_t *W1pb = static_cast<const uint16_t *>(W1p), *xeb = static_cast<const uint16_t *>(xe);
#define MOE_BWD_CASE(ACT)                                                                         \
    case ACT:                                                                                     \
        return backward_t<ACT>(*s, n_chunks, xb, Wgf, gate_bias, bias_token_stride, W1b, W2b, W1pb, \
                               expert_idx, gate, offsets, slot_of, src_of, xeb,                   \
                               static_cast<const _Float16 *>(ye), preh, hidh,                     \
                               dy, dx, dWg, dW1, dW2, dgate, w, st);
    switch (s->act) {
        MOE_BWD_CASE(MOE_ACT_GELU_ERF)
        MOE_BWD_CASE(MOE_ACT_GELU_TANH)
        MOE_BWD_CASE(MOE_ACT_RELU)
        MOE_BWD_CASE(MOE_ACT_IDENTITY)
    }
#undef MOE_BWD_CASE
    set_error("unknown activation %d", static_cast<int>(s->act));
    return MOE_EINVAL;
}

}  // extern "C"
