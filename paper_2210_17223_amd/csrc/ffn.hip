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
// through LDS in 128 x 64 tiles, and the weight tile is fed as the MFMA "A" operand
// so that each lane ends up with four consecutive output columns of one row.
// H is kept in fp16, ye in fp32.
// fp32 layers: a plain LDS-tiled vector-ALU GEMM (correctness configuration).
#include "common.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// ---------------------------------------------------------------- activations
// Phi(v) = 0.5 erfc(-v / sqrt 2) from the rational-times-gaussian form of erfc
// (Abramowitz & Stegun 7.1.26, absolute error 1.5e-7), evaluated on |v| so that
// the negative tail has no cancellation.
__device__ __forceinline__ float gelu_erf_fast(float v)
{
    const float a = fabsf(v) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, a, 1.0f));
    float p = 1.061405429f;
    p = __builtin_fmaf(p, t, -1.453152027f);
    p = __builtin_fmaf(p, t, 1.421413741f);
    p = __builtin_fmaf(p, t, -0.284496736f);
    p = __builtin_fmaf(p, t, 0.254829592f);
    p *= t;
    const float q = 0.5f * p * __builtin_amdgcn_exp2f(-a * a * 1.4426950408889634f);
    return v * (v < 0.0f ? q : 1.0f - q);
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
    float *__restrict__ C, const RowTile *__restrict__ tiles,
    const int32_t *__restrict__ ntiles, int N, int K, int max_tiles)
{
    const int mt = blockIdx.x % max_tiles;
    const int nt = blockIdx.x / max_tiles;
    if (mt >= *ntiles) return;
    const RowTile tile = tiles[mt];
    const int n0 = nt * kF32Tile;

    __shared__ float As[kF32BK][kF32Tile + 4];
    __shared__ float Bs[kF32BK][kF32Tile + 4];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    float acc[4][4] = {};

    const int a_row = tid / 4, a_k = (tid % 4) * 4;
    const int a_row_g = min(tile.row0 + a_row, tile.row1 - 1);
    const int b_k = tid / 16, b_n = (tid % 16) * 4;
    const float *Bexp = B + static_cast<size_t>(tile.expert) * K * N;

    for (int k0 = 0; k0 < K; k0 += kF32BK) {
        float4 av = make_float4(0.f, 0.f, 0.f, 0.f), bv = av;
        if (k0 + a_k < K)
            av = *reinterpret_cast<const float4 *>(A + static_cast<size_t>(a_row_g) * K + k0 + a_k);
        if (k0 + b_k < K && n0 + b_n < N)
            bv = *reinterpret_cast<const float4 *>(Bexp + static_cast<size_t>(k0 + b_k) * N + n0 + b_n);
        __syncthreads();
        As[a_k + 0][a_row] = av.x;
        As[a_k + 1][a_row] = av.y;
        As[a_k + 2][a_row] = av.z;
        As[a_k + 3][a_row] = av.w;
        *reinterpret_cast<float4 *>(&Bs[b_k][b_n]) = bv;
        __syncthreads();
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
constexpr int kBM = 128;       // activation rows per block
constexpr int kBN = 128;       // output columns (weight rows) per block
constexpr int kBK = 64;        // contraction depth per LDS stage
constexpr int kLd = kBK + 8;   // LDS row pitch in elements (16 bytes of padding)

template <bool F16>
__device__ __forceinline__ f32x16 mfma_32x32x16(const uint4 &a, const uint4 &b, const f32x16 &c)
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
// 256 threads = 2 x 2 wavefronts, each owning a 64 x 64 patch = 2 x 2 MFMA tiles.
template <bool F16, typename TOut, int ACT>
__global__ __launch_bounds__(256) void grouped_gemm_mfma_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W,
    const float *__restrict__ bias, TOut *__restrict__ C, const RowTile *__restrict__ tiles,
    const int32_t *__restrict__ ntiles, int N, int K, int max_tiles)
{
    // Blocks are dealt round-robin to the 8 XCDs; renumber them so that each XCD
    // walks a contiguous range of tiles and neighbours share operands in its L2.
    const int nb = gridDim.x;
    const int lid = (blockIdx.x % 8) * (nb / 8) + blockIdx.x / 8;
    const int mt = lid % max_tiles;
    const int nt = lid / max_tiles;
    if (mt >= *ntiles || nt * kBN >= N) return;
    const RowTile tile = tiles[mt];
    const int n0 = nt * kBN;

    __shared__ __attribute__((aligned(16))) uint16_t As[2][kBM][kLd];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[2][kBN][kLd];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    // global -> LDS mapping: 1024 16-byte vectors per operand tile, 4 per thread
    const uint16_t *a_src[4];
    const uint16_t *w_src[4];
    int ld_row[4], ld_col[4];
    const uint16_t *Wexp = W + static_cast<size_t>(tile.expert) * N * K;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int v = tid + 256 * q;
        ld_row[q] = v >> 3;
        ld_col[q] = (v & 7) * 8;
        const int r = min(tile.row0 + ld_row[q], tile.row1 - 1);
        const int n = min(n0 + ld_row[q], N - 1);
        a_src[q] = A + static_cast<size_t>(r) * K + ld_col[q];
        w_src[q] = Wexp + static_cast<size_t>(n) * K + ld_col[q];
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    uint4 a_reg[4], w_reg[4];
#define MOE_LOAD_GLOBAL(k0)                                                              \
    _Pragma("unroll") for (int q = 0; q < 4; ++q)                                        \
    {                                                                                    \
        if ((k0) + ld_col[q] < K) {                                                      \
            a_reg[q] = *reinterpret_cast<const uint4 *>(a_src[q] + (k0));                \
            w_reg[q] = *reinterpret_cast<const uint4 *>(w_src[q] + (k0));                \
        } else {                                                                         \
            a_reg[q].x = a_reg[q].y = a_reg[q].z = a_reg[q].w = 0u;                      \
            w_reg[q].x = w_reg[q].y = w_reg[q].z = w_reg[q].w = 0u;                      \
        }                                                                                \
    }
#define MOE_STORE_LDS(buf)                                                               \
    _Pragma("unroll") for (int q = 0; q < 4; ++q)                                        \
    {                                                                                    \
        *reinterpret_cast<uint4 *>(&As[buf][ld_row[q]][ld_col[q]]) = a_reg[q];           \
        *reinterpret_cast<uint4 *>(&Ws[buf][ld_row[q]][ld_col[q]]) = w_reg[q];           \
    }

    const int KT = ceil_div(K, kBK);
    MOE_LOAD_GLOBAL(0)
    MOE_STORE_LDS(0)
    __syncthreads();
    const int fr = lane & 31;            // fragment row inside a 32-row MFMA tile
    const int fk = (lane >> 5) * 8;      // k offset of this lane's 8 elements
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) {
            MOE_LOAD_GLOBAL((kt + 1) * kBK)
        }
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            uint4 wf[2], af[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                wf[i] = *reinterpret_cast<const uint4 *>(&Ws[buf][wn * 64 + i * 32 + fr][ks * 16 + fk]);
                af[i] = *reinterpret_cast<const uint4 *>(&As[buf][wm * 64 + i * 32 + fr][ks * 16 + fk]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma_32x32x16<F16>(wf[i], af[j], acc[i][j]);
        }
        if (kt + 1 < KT) {
            MOE_STORE_LDS(buf ^ 1)
        }
        __syncthreads();
    }

#undef MOE_LOAD_GLOBAL
#undef MOE_STORE_LDS

    // acc[i][j][4*g + c]: output column n0 + wn*64 + i*32 + 8*g + 4*(lane/32) + c,
    //                     row tile.row0 + wm*64 + j*32 + lane%32
    const float *bexp = bias != nullptr ? bias + static_cast<size_t>(tile.expert) * N : nullptr;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = tile.row0 + wm * 64 + j * 32 + fr;
        if (r >= tile.row1) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * 64 + i * 32 + 8 * g + 4 * (lane >> 5);
                if (n >= N) continue;
                float v[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float s = acc[i][j][4 * g + c];
                    if (bexp != nullptr) s += bexp[n + c];
                    v[c] = activate<ACT, true>(s);
                }
                store4(C + static_cast<size_t>(r) * N + n, v);
            }
        }
    }
}

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
    const RowTile *tiles = w.tiles + static_cast<size_t>(chunk) * w.max_tiles;
    const int32_t *nt = w.ntiles + chunk;
    float *H = static_cast<float *>(w.hidden);
    prof_begin(kStageGemm1, st);
    hipLaunchKernelGGL(grouped_gemm_f32_kernel<ACT>,
                       dim3(w.max_tiles * ceil_div(s.d_ff, kF32Tile)), dim3(256), 0, st, xe, W1,
                       b1, H, tiles, nt, s.d_ff, s.d_model, w.max_tiles);
    prof_end(kStageGemm1, st);
    prof_begin(kStageGemm2, st);
    hipLaunchKernelGGL(grouped_gemm_f32_kernel<MOE_ACT_IDENTITY>,
                       dim3(w.max_tiles * ceil_div(s.d_model, kF32Tile)), dim3(256), 0, st, H, W2,
                       b2, ye, tiles, nt, s.d_model, s.d_ff, w.max_tiles);
    prof_end(kStageGemm2, st);
}

template <int ACT>
void launch_mfma_pair(const moe_shape &s, const uint16_t *xe, const uint16_t *W1p,
                      const float *b1, const uint16_t *W2p, const float *b2, float *ye,
                      const Workspace &w, int chunk, hipStream_t st)
{
    const RowTile *tiles = w.tiles + static_cast<size_t>(chunk) * w.max_tiles;
    const int32_t *nt = w.ntiles + chunk;
    _Float16 *H = static_cast<_Float16 *>(w.hidden);
    const int g1 = static_cast<int>(align_up(static_cast<size_t>(w.max_tiles) * ceil_div(s.d_ff, kBN), 8));
    const int g2 = static_cast<int>(align_up(static_cast<size_t>(w.max_tiles) * ceil_div(s.d_model, kBN), 8));
    prof_begin(kStageGemm1, st);
    hipLaunchKernelGGL((grouped_gemm_mfma_kernel<false, _Float16, ACT>), dim3(g1), dim3(256), 0, st,
                       xe, W1p, b1, H, tiles, nt, s.d_ff, s.d_model, w.max_tiles);
    prof_end(kStageGemm1, st);
    prof_begin(kStageGemm2, st);
    hipLaunchKernelGGL((grouped_gemm_mfma_kernel<true, float, MOE_ACT_IDENTITY>), dim3(g2),
                       dim3(256), 0, st, reinterpret_cast<const uint16_t *>(H), W2p, b2, ye, tiles,
                       nt, s.d_model, s.d_ff, w.max_tiles);
    prof_end(kStageGemm2, st);
}

}  // namespace

int ffn_tile_rows(const moe_shape &s) { return s.dtype == MOE_BF16 ? kBM : kF32Tile; }

moe_status launch_ffn(const moe_shape &s, const void *xe, const void *W1p, const float *b1,
                      const void *W2p, const float *b2, float *ye, const Workspace &w,
                      int chunk, hipStream_t st)
{
#define MOE_FFN_CASE(ACT)                                                                      \
    case ACT:                                                                                  \
        if (s.dtype == MOE_BF16)                                                               \
            launch_mfma_pair<ACT>(s, static_cast<const uint16_t *>(xe),                         \
                                  static_cast<const uint16_t *>(W1p), b1,                       \
                                  static_cast<const uint16_t *>(W2p), b2, ye, w, chunk, st);    \
        else                                                                                   \
            launch_f32_pair<ACT>(s, static_cast<const float *>(xe),                             \
                                 static_cast<const float *>(W1p), b1,                           \
                                 static_cast<const float *>(W2p), b2, ye, w, chunk, st);        \
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
