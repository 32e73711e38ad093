// Gate: logits, top-k selection and softmax gate weights (paper Sec. 2.1).
//
// The logit of (token, expert) is one fp32 accumulator walked over the model
// dimension in ascending order with fused multiply-adds, so that the top-k
// decision (an integer result) does not depend on a reduction tree.  The work is
// therefore plain fp32 vector arithmetic: a lane owns one token and EPT experts,
// the token's embedding comes from an LDS tile, and the gate matrix, which is
// uniform across the lanes of a wavefront, is fetched with scalar loads and fed
// to v_fma_f32 from scalar registers.
#include "common.h"

namespace moe {
namespace {

constexpr int kTok = 64;   // tokens per block (= lanes of one wavefront)
constexpr int kKC = 64;    // model-dimension chunk staged in LDS

__device__ __forceinline__ void load_row_vec(const float *p, float (&v)[8], int &n)
{
    const float4 q = *reinterpret_cast<const float4 *>(p);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    n = 4;
}
__device__ __forceinline__ void load_row_vec(const uint16_t *p, float (&v)[8], int &n)
{
    const uint4 q = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
    n = 8;
}

// Block = (EP / EPT) wavefronts over the same 64 tokens; wavefront w owns experts
// [w*EPT, (w+1)*EPT).  Wgp is the packed gate matrix: fp32 [d][EP], zero padded.
template <typename XT, int EPT>
__global__ __launch_bounds__(1024) void route_kernel(
    const XT *__restrict__ x, const float *__restrict__ Wgp,
    const float *__restrict__ bias, int bias_stride, int32_t *__restrict__ expert_idx,
    float *__restrict__ gate, int T, int d, int E, int EP, int k, int renorm)
{
    constexpr int VE = 16 / sizeof(XT);          // elements per 16-byte vector
    __shared__ float xs[kTok][kKC + 1];
    __shared__ float zs[kTok][kMaxExperts + 1];

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int e0 = wave * EPT;
    const int t0 = blockIdx.x * kTok;

    float acc[EPT];
#pragma unroll
    for (int q = 0; q < EPT; ++q) acc[q] = 0.0f;

    for (int k0 = 0; k0 < d; k0 += kKC) {
        const int kc = min(kKC, d - k0);
        __syncthreads();
        // stage x[t0 .. t0+63][k0 .. k0+kc) as fp32
        const int vec_per_row = kKC / VE;
        for (int v = threadIdx.x; v < kTok * vec_per_row; v += blockDim.x) {
            const int r = v / vec_per_row;
            const int c = (v % vec_per_row) * VE;
            if (c < kc) {
                const int t = min(t0 + r, T - 1);
                float vals[8];
                int n;
                load_row_vec(x + static_cast<size_t>(t) * d + k0 + c, vals, n);
#pragma unroll
                for (int i = 0; i < VE; ++i) xs[r][c + i] = vals[i];
            }
        }
        __syncthreads();
        const float *wrow = Wgp + static_cast<size_t>(k0) * EP + e0;
        if (kc == kKC) {
#pragma unroll 8
            for (int i = 0; i < kKC; ++i) {
                const float xv = xs[lane][i];
#pragma unroll
                for (int q = 0; q < EPT; ++q)
                    acc[q] = __builtin_fmaf(xv, wrow[static_cast<size_t>(i) * EP + q], acc[q]);
            }
        } else {
            for (int i = 0; i < kc; ++i) {
                const float xv = xs[lane][i];
#pragma unroll
                for (int q = 0; q < EPT; ++q)
                    acc[q] = __builtin_fmaf(xv, wrow[static_cast<size_t>(i) * EP + q], acc[q]);
            }
        }
    }

    const int t = t0 + lane;
#pragma unroll
    for (int q = 0; q < EPT; ++q) {
        const int e = e0 + q;
        if (e < E) {
            float z = acc[q];
            if (bias != nullptr && t < T)
                z = z + bias[static_cast<size_t>(t) * bias_stride + e];
            zs[lane][e] = z;
        }
    }
    __syncthreads();
    if (wave != 0 || t >= T) return;

    // softmax denominator over all E experts
    float zmax = zs[lane][0];
    for (int e = 1; e < E; ++e) zmax = fmaxf(zmax, zs[lane][e]);
    float denom = 0.0f;
    for (int e = 0; e < E; ++e) denom += expf(zs[lane][e] - zmax);

    float gsum = 1.0f;
    if (renorm) {
        gsum = 0.0f;
        uint64_t taken = 0;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            float bz = 0.0f;
            for (int e = 0; e < E; ++e) {
                if ((taken >> e) & 1ull) continue;
                const float zv = zs[lane][e];
                if (best < 0 || zv > bz) { best = e; bz = zv; }
            }
            taken |= 1ull << best;
            gsum += expf(bz - zmax) / denom;
        }
    }
    uint64_t taken = 0;
    for (int j = 0; j < k; ++j) {
        int best = -1;
        float bz = 0.0f;
        for (int e = 0; e < E; ++e) {
            if ((taken >> e) & 1ull) continue;
            const float zv = zs[lane][e];
            if (best < 0 || zv > bz) { best = e; bz = zv; }   // ties: lower index stays
        }
        taken |= 1ull << best;
        const float g = expf(bz - zmax) / denom;
        expert_idx[static_cast<size_t>(t) * k + j] = best;
        gate[static_cast<size_t>(t) * k + j] = renorm ? g / gsum : g;
    }
}

// Gate matrix [d][E] (fp32 or bf16) -> fp32 [d][EP], zero padded.
template <typename XT>
__global__ void pack_gate_kernel(const XT *__restrict__ Wg, float *__restrict__ Wgp,
                                 int d, int E, int EP)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= d * EP) return;
    const int i = idx / EP, e = idx % EP;
    float v = 0.0f;
    if (e < E) {
        if constexpr (sizeof(XT) == 2)
            v = bf16_to_f32(Wg[static_cast<size_t>(i) * E + e]);
        else
            v = Wg[static_cast<size_t>(i) * E + e];
    }
    Wgp[idx] = v;
}

int pow2_ceil(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

template <typename XT>
moe_status launch_route_t(const moe_shape &s, const XT *x, const float *Wgp,
                          const float *bias, int bias_stride, int32_t *expert_idx,
                          float *gate, hipStream_t st)
{
    const int EP = pow2_ceil(s.E);
    const int blocks = ceil_div(s.T, kTok);
    // Largest expert slice per lane that still leaves >= 1024 wavefronts in flight;
    // a block holds at most 16 wavefronts.
    int ept = 16;
    while (ept > 1 && (ept > EP || static_cast<long>(blocks) * (EP / ept) < 1024)) ept >>= 1;
    while (EP / ept > 16) ept <<= 1;
    const dim3 grid(blocks), block((EP / ept) * kWave);
#define MOE_ROUTE_CASE(N)                                                              \
    case N:                                                                            \
        hipLaunchKernelGGL((route_kernel<XT, N>), grid, block, 0, st, x, Wgp, bias,    \
                           bias_stride, expert_idx, gate, s.T, s.d_model, s.E, EP, s.k, \
                           s.renorm_topk);                                             \
        break;
    switch (ept) {
        MOE_ROUTE_CASE(1)
        MOE_ROUTE_CASE(2)
        MOE_ROUTE_CASE(4)
        MOE_ROUTE_CASE(8)
        MOE_ROUTE_CASE(16)
    default:
        set_error("route: internal error, expert slice %d", ept);
        return MOE_EINVAL;
    }
#undef MOE_ROUTE_CASE
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace

size_t packed_gate_bytes(const moe_shape &s)
{
    return static_cast<size_t>(s.d_model) * pow2_ceil(s.E) * sizeof(float);
}

moe_status launch_pack_gate(const moe_shape &s, const void *Wg, float *Wgp, hipStream_t st)
{
    const int EP = pow2_ceil(s.E);
    const int n = s.d_model * EP;
    const dim3 grid(ceil_div(n, 256)), block(256);
    if (s.dtype == MOE_BF16)
        hipLaunchKernelGGL(pack_gate_kernel<uint16_t>, grid, block, 0, st,
                           static_cast<const uint16_t *>(Wg), Wgp, s.d_model, s.E, EP);
    else
        hipLaunchKernelGGL(pack_gate_kernel<float>, grid, block, 0, st,
                           static_cast<const float *>(Wg), Wgp, s.d_model, s.E, EP);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status launch_route(const moe_shape &s, const void *x, const void *Wgp,
                        const float *bias, int bias_stride, int32_t *expert_idx,
                        float *gate, hipStream_t st)
{
    if (s.dtype == MOE_BF16)
        return launch_route_t<uint16_t>(s, static_cast<const uint16_t *>(x),
                                        static_cast<const float *>(Wgp), bias, bias_stride,
                                        expert_idx, gate, st);
    return launch_route_t<float>(s, static_cast<const float *>(x),
                                 static_cast<const float *>(Wgp), bias, bias_stride,
                                 expert_idx, gate, st);
}

}  // namespace moe
