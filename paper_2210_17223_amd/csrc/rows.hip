// Row movers: pack tokens into the expert-major buffer (the payload of the first
// all-to-all, paper end of Sec. 2.1) and the gate-weighted unpack ("combine",
// Sec. 2.2 forward-pass timeline).  Both are bound by HBM bandwidth: one wavefront
// owns one token, every lane moves 16 bytes per step, a token's row is read once
// and written to each of its kept slots (pack) or its kept expert rows are read
// once and the weighted sum written once (unpack).  Expert outputs are stored in fp16 for
// bf16 layers (fp32 for fp32 layers); the weighted sum and y are fp32.
#include "common.h"

namespace moe {
namespace {

constexpr int kRowWaves = 4;
constexpr int kRowThreads = kRowWaves * kWave;

// xe[slot_of[t*k+j], :] = x[t, :] for kept j.  `vec` = 16-byte vectors per row.
__global__ __launch_bounds__(kRowThreads) void scatter_rows_kernel(
    const uint4 *__restrict__ x, const int32_t *__restrict__ slot_of,
    uint4 *__restrict__ xe, int t0, int t1, int k, int vec, int max_rows)
{
    const int lane = lane_id();
    const int t = t0 + blockIdx.x * kRowWaves + threadIdx.x / kWave;
    if (t >= t1) return;
    int my_slot = lane < k ? slot_of[static_cast<size_t>(t) * k + lane] : -1;
    if (my_slot >= max_rows) my_slot = -1;   // never follow a slot outside the buffer
    const uint64_t kept = __ballot(my_slot >= 0);
    if (kept == 0) return;
    int slots[kMaxTopK];
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) slots[j] = __shfl(my_slot, j);
    const uint4 *src = x + static_cast<size_t>(t) * vec;
    for (int c = lane; c < vec; c += kWave) {
        const uint4 v = src[c];
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j)
            if (j < k && slots[j] >= 0) xe[static_cast<size_t>(slots[j]) * vec + c] = v;
    }
}

// y[t,:] = sum_j gate[t,j] * ye[slot_of[t*k+j],:] over kept j, ascending j, in fp32.
// TIn: stored type of the expert outputs (fp16 for bf16 layers, fp32 for fp32 layers); a lane
// takes 16 bytes of every kept row per step (NV = 8 or 4 elements) and writes NV fp32 values.
// ACT_BYTES: element size of the optional copy in the activation dtype (0 = none).
template <typename TIn, int ACT_BYTES>
__global__ __launch_bounds__(kRowThreads) void combine_rows_kernel(
    const uint4 *__restrict__ ye, const int32_t *__restrict__ slot_of,
    const float *__restrict__ gate, float *__restrict__ y, void *__restrict__ y_act,
    int t0, int t1, int k, int vec, int max_rows)
{
    constexpr int NV = 16 / static_cast<int>(sizeof(TIn));
    const int lane = lane_id();
    const int t = t0 + blockIdx.x * kRowWaves + threadIdx.x / kWave;
    if (t >= t1) return;
    int my_slot = lane < k ? slot_of[static_cast<size_t>(t) * k + lane] : -1;
    if (my_slot >= max_rows) my_slot = -1;   // never follow a slot outside the buffer
    const float my_gate = lane < k ? gate[static_cast<size_t>(t) * k + lane] : 0.0f;
    int slots[kMaxTopK];
    float g[kMaxTopK];
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
        slots[j] = __shfl(my_slot, j);
        g[j] = __shfl(my_gate, j);
    }
    for (int c = lane; c < vec; c += kWave) {
        float acc[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = 0.0f;
        bool first = true;
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j) {
            if (j < k && slots[j] >= 0) {
                const uint4 raw = ye[static_cast<size_t>(slots[j]) * vec + c];
                float v[NV];
                if constexpr (NV == 8) {
                    typedef __attribute__((ext_vector_type(8))) _Float16 half8;
                    const half8 hv = __builtin_bit_cast(half8, raw);
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = static_cast<float>(hv[i]);
                } else {
                    v[0] = __uint_as_float(raw.x); v[1] = __uint_as_float(raw.y);
                    v[2] = __uint_as_float(raw.z); v[3] = __uint_as_float(raw.w);
                }
                if (first) {
#pragma unroll
                    for (int i = 0; i < NV; ++i) acc[i] = g[j] * v[i];
                    first = false;
                } else {
#pragma unroll
                    for (int i = 0; i < NV; ++i) acc[i] = __builtin_fmaf(g[j], v[i], acc[i]);
                }
            }
        }
        const size_t at = (static_cast<size_t>(t) * vec + c) * NV;       // element index in the row-major output
#pragma unroll
        for (int i = 0; i < NV; i += 4)
            *reinterpret_cast<float4 *>(y + at + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
        if constexpr (ACT_BYTES == 4) {
#pragma unroll
            for (int i = 0; i < NV; i += 4)
                *reinterpret_cast<float4 *>(static_cast<float *>(y_act) + at + i) =
                    make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
        } else if constexpr (ACT_BYTES == 2) {
            uint32_t p[NV / 2];
#pragma unroll
            for (int i = 0; i < NV; i += 2)
                p[i / 2] = f32_to_bf16(acc[i]) | (static_cast<uint32_t>(f32_to_bf16(acc[i + 1])) << 16);
            if constexpr (NV == 8)
                *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(y_act) + at) = make_uint4(p[0], p[1], p[2], p[3]);
            else
                *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(y_act) + at) = make_uint2(p[0], p[1]);
        }
    }
}

}  // namespace

moe_status launch_scatter(const moe_shape &s, const void *x, const int32_t *slot_of,
                          void *xe, int t0, int t1, hipStream_t st)
{
    if (t1 <= t0) return MOE_OK;
    const int elem = s.dtype == MOE_BF16 ? 2 : 4;
    const int max_rows = static_cast<int>(moe_max_rows(&s));
    const int vec = s.d_model * elem / 16;
    hipLaunchKernelGGL(scatter_rows_kernel, dim3(ceil_div(t1 - t0, kRowWaves)),
                       dim3(kRowThreads), 0, st, static_cast<const uint4 *>(x), slot_of,
                       static_cast<uint4 *>(xe), t0, t1, s.k, vec, max_rows);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status launch_combine(const moe_shape &s, const void *ye, const int32_t *slot_of,
                          const float *gate, float *y, void *y_act, int t0, int t1,
                          hipStream_t st, int64_t rows)
{
    if (t1 <= t0) return MOE_OK;
    const int vec = s.d_model * ye_elem_bytes(s) / 16;   // 16-byte vectors per row of ye
    const int max_rows = static_cast<int>(rows < 0 ? moe_max_rows(&s) : rows);
    const dim3 grid(ceil_div(t1 - t0, kRowWaves)), block(kRowThreads);
    const uint4 *ye4 = static_cast<const uint4 *>(ye);
#define MOE_COMBINE(TIN, AB)                                                                      \
    hipLaunchKernelGGL((combine_rows_kernel<TIN, AB>), grid, block, 0, st, ye4, slot_of, gate, y,  \
                       y_act, t0, t1, s.k, vec, max_rows)
    if (s.dtype == MOE_BF16) {
        if (y_act == nullptr) MOE_COMBINE(_Float16, 0); else MOE_COMBINE(_Float16, 2);
    } else {
        if (y_act == nullptr) MOE_COMBINE(float, 0); else MOE_COMBINE(float, 4);
    }
#undef MOE_COMBINE
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace moe
