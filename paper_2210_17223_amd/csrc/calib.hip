// Calibration kernels of the measurement harness (not part of the layer): what this chip
// delivers on a plain device copy and on a register-resident MFMA loop, so that roofline
// fractions can be quoted against measured peaks beside the nominal ones.
#include "common.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// dst[i] = src[i], 16 bytes per lane and step, grid-stride.
__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4 *__restrict__ src,
                                                         uint4 *__restrict__ dst, size_t n)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
        dst[i] = src[i];
}

// Every wavefront issues `iters` rounds of eight independent 32x32x16 bf16 MFMAs on operands
// that stay in registers.  RANDOM: operand bits differ from lane to lane and register to
// register (values near +-1, so nothing overflows); otherwise all operands are 1.0 -- the
// matrix cores then toggle few bits, draw less power and hold a higher clock.
template <bool RANDOM>
__global__ __launch_bounds__(256) void calib_mfma_kernel(float *__restrict__ sink, int iters)
{
    const unsigned lane = threadIdx.x;
    u32x4 a[2], b[4];
#pragma unroll
    for (int q = 0; q < 6; ++q) {
        u32x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            unsigned s = (lane * 24u + q * 4u + c + 1u) * 2654435761u;
            s ^= s >> 13;
            s *= 0x9E3779B1u;
            // two bf16 values with exponent 0 (|v| in [1, 2)), random mantissa and sign
            const unsigned lo = 0x3f80u | ((s >> 4) & 0x7fu) | (((s >> 20) & 1u) << 15);
            const unsigned hi = 0x3f80u | ((s >> 12) & 0x7fu) | (((s >> 25) & 1u) << 15);
            v[c] = RANDOM ? (lo | (hi << 16)) : 0x3f803f80u;
        }
        if (q < 2) a[q] = v; else b[q - 2] = v;
    }
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i & 1]),
                                                             __builtin_bit_cast(bf16x8, b[i >> 1]),
                                                             acc[i], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink[static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x] = s;
}

}  // namespace

moe_status launch_calib_gemm(const uint16_t *A, const uint16_t *W, _Float16 *C, const WorkItem *items,
                             const int32_t *nitems, int max_items, int N, int K, int abl, int gelu,
                             hipStream_t st);
}  // namespace moe

using namespace moe;

extern "C" {

moe_status moe_calib_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (dst == nullptr || src == nullptr || bytes % 16 != 0 ||
        (reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u)) {
        set_error("moe_calib_copy: pointers and size must be multiples of 16 bytes");
        return MOE_EINVAL;
    }
    if (bytes == 0) return MOE_OK;
    hipLaunchKernelGGL(calib_copy_kernel, dim3(256 * 16), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint4 *>(src),
                       static_cast<uint4 *>(dst), bytes / 16);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

double moe_calib_mfma_flops(int32_t waves_per_simd, int32_t iters)
{
    return 256.0 * waves_per_simd * 4.0 * static_cast<double>(iters) * 8.0 * 2.0 * 32 * 32 * 16;
}

moe_status moe_calib_mfma(float *sink, int32_t waves_per_simd, int32_t iters, int32_t random_operands,
                          void *stream)
{
    if (sink == nullptr || waves_per_simd < 1 || waves_per_simd > 8 || iters < 1) {
        set_error("moe_calib_mfma: sink is NULL, or waves_per_simd outside 1..8, or iters < 1");
        return MOE_EINVAL;
    }
    // 256 compute units x waves_per_simd blocks of four wavefronts (one per SIMD)
    const dim3 grid(256 * waves_per_simd), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (random_operands)
        hipLaunchKernelGGL(calib_mfma_kernel<true>, grid, block, 0, st, sink, iters);
    else
        hipLaunchKernelGGL(calib_mfma_kernel<false>, grid, block, 0, st, sink, iters);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status moe_calib_gemm(const void *A, const void *W, void *C, const int32_t *items,
                          const int32_t *n_items, int32_t max_items, int32_t N, int32_t K,
                          int32_t variant, int32_t gelu, void *stream)
{
    if (A == nullptr || W == nullptr || C == nullptr || items == nullptr || n_items == nullptr ||
        max_items < 1 || N < 8 || K < 64 || K % 64 != 0 || N % 8 != 0 ||
        static_cast<uint64_t>(N) * K * 2 >= (1ull << 31) || 256ull * K * 2 >= (1ull << 31)) {
        set_error("moe_calib_gemm: NULL pointer, or N not a multiple of 8, or K not a multiple of 64");
        return MOE_EINVAL;
    }
    return launch_calib_gemm(static_cast<const uint16_t *>(A), static_cast<const uint16_t *>(W),
                             static_cast<_Float16 *>(C), reinterpret_cast<const WorkItem *>(items),
                             n_items, max_items, N, K, variant, gelu, static_cast<hipStream_t>(stream));
}

moe_status moe_expert_gemm_kernel(const moe_shape *s, int32_t which, char *name, size_t len)
{
    if (s == nullptr || name == nullptr || len == 0 || (which != 0 && which != 1) ||
        moe_max_rows(s) <= 0 || s->dtype != MOE_BF16) {
        set_error("moe_expert_gemm_kernel: which must be 0 or 1, name a buffer, the shape a supported bf16 layer");
        return MOE_EINVAL;
    }
    expert_gemm_kernel_name(*s, which, 1, name, len);
    return MOE_OK;
}

}  // extern "C"
