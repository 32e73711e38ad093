// Row movers: pack tokens into the expert-major buffer (the payload of the first
// all-to-all, paper end of Sec. 2.1) and the gate-weighted unpack ("combine",
// Sec. 2.2 forward-pass timeline).  Both are bound by HBM bandwidth: one wavefront
// owns one token, every lane moves 16 bytes per step, a token's row is read once
// and written to each of its kept slots (pack) or its kept expert rows are read
// once and the weighted sum written once (unpack).
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

// y[t,:] = sum_j gate[t,j] * ye[slot_of[t*k+j],:] over kept j, ascending j.
// ACT_BYTES: element size of the optional copy in the activation dtype (0 = none).
template <int ACT_BYTES>
__global__ __launch_bounds__(kRowThreads) void combine_rows_kernel(
    const float4 *__restrict__ ye, const int32_t *__restrict__ slot_of,
    const float *__restrict__ gate, float4 *__restrict__ y, void *__restrict__ y_act,
    int t0, int t1, int k, int vec, int max_rows)
{
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
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        bool first = true;
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j) {
            if (j < k && slots[j] >= 0) {
                const float4 v = ye[static_cast<size_t>(slots[j]) * vec + c];
                if (first) {
                    acc = make_float4(g[j] * v.x, g[j] * v.y, g[j] * v.z, g[j] * v.w);
                    first = false;
                } else {
                    acc.x = __builtin_fmaf(g[j], v.x, acc.x);
                    acc.y = __builtin_fmaf(g[j], v.y, acc.y);
                    acc.z = __builtin_fmaf(g[j], v.z, acc.z);
                    acc.w = __builtin_fmaf(g[j], v.w, acc.w);
                }
            }
        }
        y[static_cast<size_t>(t) * vec + c] = acc;
        if constexpr (ACT_BYTES == 4) {
            static_cast<float4 *>(y_act)[static_cast<size_t>(t) * vec + c] = acc;
        } else if constexpr (ACT_BYTES == 2) {
            uint2 p;
            p.x = f32_to_bf16(acc.x) | (static_cast<uint32_t>(f32_to_bf16(acc.y)) << 16);
            p.y = f32_to_bf16(acc.z) | (static_cast<uint32_t>(f32_to_bf16(acc.w)) << 16);
            static_cast<uint2 *>(y_act)[static_cast<size_t>(t) * vec + c] = p;
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

moe_status launch_combine(const moe_shape &s, const float *ye, const int32_t *slot_of,
                          const float *gate, float *y, void *y_act, int t0, int t1,
                          hipStream_t st, int64_t rows)
{
    if (t1 <= t0) return MOE_OK;
    const int vec = s.d_model / 4;   // 16-byte vectors of fp32
    const int max_rows = static_cast<int>(rows < 0 ? moe_max_rows(&s) : rows);
    const dim3 grid(ceil_div(t1 - t0, kRowWaves)), block(kRowThreads);
    const float4 *ye4 = reinterpret_cast<const float4 *>(ye);
    float4 *y4 = reinterpret_cast<float4 *>(y);
    if (y_act == nullptr)
        hipLaunchKernelGGL(combine_rows_kernel<0>, grid, block, 0, st, ye4, slot_of, gate, y4,
                           y_act, t0, t1, s.k, vec, max_rows);
    else if (s.dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_rows_kernel<2>, grid, block, 0, st, ye4, slot_of, gate, y4,
                           y_act, t0, t1, s.k, vec, max_rows);
    else
        hipLaunchKernelGGL(combine_rows_kernel<4>, grid, block, 0, st, ye4, slot_of, gate, y4,
                           y_act, t0, t1, s.k, vec, max_rows);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace moe
