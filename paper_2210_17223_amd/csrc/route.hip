// Gate: logits, top-k selection and softmax gate weights (paper Sec. 2.1).
//
// The logit of (token, expert) is one fp32 accumulator walked over the model
// dimension in ascending order with fused multiply-adds, so that the top-k
// decision (an integer result) does not depend on a reduction tree.  The work is
// therefore plain fp32 vector arithmetic: a lane owns one token and EPT experts,
// the token's embedding comes from a double-buffered LDS tile, and the gate matrix,
// which is uniform across the lanes of a wavefront, is fetched with scalar loads and
// fed to v_fma_f32 from scalar registers.
#include "common.h"

namespace moe {
namespace {

constexpr int kTok = 64;      // tokens per block (= lanes of one wavefront)
constexpr int kGatePad = 128; // the packed gate matrix pads the model dimension to this

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Model-dimension chunk staged in LDS per step: 16 vectors of 16 bytes per token row.
template <typename XT> struct Stage { static constexpr int kc = 256 / sizeof(XT); };

__device__ __forceinline__ void store_row_vec(float *dst, const u32x4 &q, float)
{
    *reinterpret_cast<f32x4 *>(dst) = __builtin_bit_cast(f32x4, q);
}
__device__ __forceinline__ void store_row_vec(float *dst, const u32x4 &q, uint16_t)
{
    f32x4 lo, hi;
    lo[0] = __uint_as_float(q[0] << 16); lo[1] = __uint_as_float(q[0] & 0xFFFF0000u);
    lo[2] = __uint_as_float(q[1] << 16); lo[3] = __uint_as_float(q[1] & 0xFFFF0000u);
    hi[0] = __uint_as_float(q[2] << 16); hi[1] = __uint_as_float(q[2] & 0xFFFF0000u);
    hi[2] = __uint_as_float(q[3] << 16); hi[3] = __uint_as_float(q[3] & 0xFFFF0000u);
    *reinterpret_cast<f32x4 *>(dst) = lo;
    *reinterpret_cast<f32x4 *>(dst + 4) = hi;
}

// Block = NW wavefronts over the same 64 tokens; wavefront w owns experts
// [w*EPT, (w+1)*EPT) and lane t owns token t0 + t.  Wgp is the packed gate matrix:
// fp32 [EP][dP], expert-major, zero padded, so that eight consecutive weights of one
// expert arrive with one scalar load.  The token tile is staged through LDS as fp32
// (double buffered, the next stage's global loads in flight during the FMAs).
template <typename XT, int EPT, int NW>
__global__ __launch_bounds__(NW * 64) void route_kernel(
    const XT *__restrict__ x, const float *__restrict__ Wgp,
    const float *__restrict__ bias, int bias_stride, int32_t *__restrict__ expert_idx,
    float *__restrict__ gate, int32_t *__restrict__ seg_cnt, int T, int d, int dP, int E, int k,
    int renorm)
{
    constexpr int KC = Stage<XT>::kc;            // 128 (bf16) or 64 (fp32)
    constexpr int VE = 16 / sizeof(XT);          // elements per 16-byte vector
    constexpr int LDX = KC + 4;                  // LDS row pitch in floats
    constexpr int NVEC = kTok * 16;              // 16-byte vectors per stage
    constexpr int VPT = 16 / NW;                 // vectors per thread per stage
    static_assert(NVEC == VPT * NW * kWave, "staging map");
    constexpr int PD = NW >= 8 ? 4 : (NW == 4 ? 2 : 1);   // stages of global loads kept in flight
    __shared__ __attribute__((aligned(16))) float xs[2][kTok][LDX];
    static_assert(sizeof(float) * 2 * kTok * LDX >= sizeof(float) * (kTok + 1) * (kMaxExperts + 1), "zs alias");
    float (*zs)[kMaxExperts + 1] = reinterpret_cast<float (*)[kMaxExperts + 1]>(&xs[0][0][0]);

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int e0 = wave * EPT;
    const int t0 = blockIdx.x * kTok;

    // staging map: vector v = row (v / 16), 16-byte column (v % 16)
    u32x4 pre[PD][VPT];
    const XT *src[VPT];
    int col[VPT];
    float *dst[2][VPT];
#pragma unroll
    for (int q = 0; q < VPT; ++q) {
        const int v = threadIdx.x + q * NW * kWave;
        const int r = v >> 4;
        col[q] = (v & 15) * VE;
        src[q] = x + static_cast<size_t>(min(t0 + r, T - 1)) * d + col[q];
        dst[0][q] = &xs[0][r][col[q]];
        dst[1][q] = &xs[1][r][col[q]];
    }
#define MOE_LOAD_STAGE(slot, k0)                                                      \
    _Pragma("unroll") for (int q = 0; q < VPT; ++q)                                   \
    {                                                                                 \
        const u32x4 zero = {0u, 0u, 0u, 0u};                                          \
        pre[slot][q] = zero;                                                          \
        if ((k0) + col[q] < d)                                                        \
            pre[slot][q] = *reinterpret_cast<const u32x4 *>(src[q] + (k0));           \
    }
#define MOE_STORE_STAGE(slot, buf)                                                    \
    _Pragma("unroll") for (int q = 0; q < VPT; ++q)                                   \
        store_row_vec(dst[buf][q], pre[slot][q], XT());

    float acc[EPT];
#pragma unroll
    for (int q = 0; q < EPT; ++q) acc[q] = 0.0f;

    const int nstage = dP / KC;
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (u < nstage) { MOE_LOAD_STAGE(u, u * KC) }
    for (int s0 = 0; s0 < nstage; s0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int s = s0 + u;
            if (s < nstage) {
                // PD is even or 1, so the LDS buffer of stage s is the compile-time u & 1
                // (for PD == 1 it alternates with s)
                const int buf = PD == 1 ? (s & 1) : (u & 1);
                if (buf) { MOE_STORE_STAGE(u, 1) } else { MOE_STORE_STAGE(u, 0) }
                __syncthreads();
                if (s + PD < nstage) { MOE_LOAD_STAGE(u, (s + PD) * KC) }
                const float *wbase = Wgp + static_cast<size_t>(e0) * dP + s * KC;
                const float *xrow = &xs[buf][lane][0];
#pragma unroll 2
                for (int ib = 0; ib < KC / 8; ++ib) {
                    float w[EPT][8];
#pragma unroll
                    for (int q = 0; q < EPT; ++q)
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            w[q][i] = wbase[static_cast<size_t>(q) * dP + ib * 8 + i];
                    const f32x4 xa = *reinterpret_cast<const f32x4 *>(xrow + ib * 8);
                    const f32x4 xb = *reinterpret_cast<const f32x4 *>(xrow + ib * 8 + 4);
                    const float xv[8] = {xa[0], xa[1], xa[2], xa[3], xb[0], xb[1], xb[2], xb[3]};
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int q = 0; q < EPT; ++q)
                            acc[q] = __builtin_fmaf(xv[i], w[q][i], acc[q]);
                }
            }
        }
    }
#undef MOE_LOAD_STAGE
#undef MOE_STORE_STAGE
    __syncthreads();           // every wavefront is done with the token tile: reuse it for logits

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
    if (wave != 0) return;
    // The first wavefront finishes the block's 64 tokens: top-k, softmax weights and, for the
    // layer call, the expert histogram of these tokens (one segment of the dispatch plan).
    // The histogram sits behind the logits in the reused token-tile memory.
    int32_t *cnt = reinterpret_cast<int32_t *>(&zs[kTok][0]);
    if (seg_cnt != nullptr) cnt[lane] = 0;
    __builtin_amdgcn_wave_barrier();
    if (t < T) {
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
        if (seg_cnt != nullptr) atomicAdd(&cnt[best], 1);
    }
    }
    if (seg_cnt != nullptr) {
        __builtin_amdgcn_wave_barrier();
        seg_cnt[static_cast<size_t>(blockIdx.x) * kMaxExperts + lane] = cnt[lane];
    }
}

// Gate matrix [d][E] (fp32 or bf16) -> fp32 [EP][dP], expert-major, zero padded.
template <typename XT>
__global__ void pack_gate_kernel(const XT *__restrict__ Wg, float *__restrict__ Wgp,
                                 int d, int dP, int E, int EP)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= dP * EP) return;
    const int e = idx / dP, i = idx % dP;
    float v = 0.0f;
    if (e < E && i < d) {
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

int padded_dim(int d) { return (d + kGatePad - 1) / kGatePad * kGatePad; }

template <typename XT>
moe_status launch_route_t(const moe_shape &s, const XT *x, const float *Wgp,
                          const float *bias, int bias_stride, int32_t *expert_idx,
                          float *gate, int32_t *seg_cnt, hipStream_t st)
{
    const int EP = pow2_ceil(s.E);
    const int dP = padded_dim(s.d_model);
    const int blocks = ceil_div(s.T, kTok);
    // Largest expert slice per lane (at most 4: the weights of a slice live in scalar
    // registers) that still leaves about four wavefronts per SIMD in flight; a block
    // holds at most 16 wavefronts.
    int ept = 4;
    while (ept > 1 && (ept > EP || static_cast<long>(blocks) * (EP / ept) < 4096)) ept >>= 1;
    while (EP / ept > 16) ept <<= 1;
    const int nw = EP / ept;
    const dim3 grid(blocks), block(nw * kWave);
#define MOE_ROUTE_CASE(EPT_, NW_)                                                            \
    if (ept == EPT_ && nw == NW_) {                                                          \
        hipLaunchKernelGGL((route_kernel<XT, EPT_, NW_>), grid, block, 0, st, x, Wgp, bias,  \
                           bias_stride, expert_idx, gate, seg_cnt, s.T, s.d_model, dP, s.E,  \
                           s.k, s.renorm_topk);                                              \
        launched = true;                                                                     \
    }
    bool launched = false;
    MOE_ROUTE_CASE(4, 16) MOE_ROUTE_CASE(4, 8) MOE_ROUTE_CASE(4, 4) MOE_ROUTE_CASE(4, 2) MOE_ROUTE_CASE(4, 1)
    MOE_ROUTE_CASE(2, 16) MOE_ROUTE_CASE(2, 8) MOE_ROUTE_CASE(2, 4) MOE_ROUTE_CASE(2, 2) MOE_ROUTE_CASE(2, 1)
    MOE_ROUTE_CASE(1, 16) MOE_ROUTE_CASE(1, 8) MOE_ROUTE_CASE(1, 4) MOE_ROUTE_CASE(1, 2) MOE_ROUTE_CASE(1, 1)
#undef MOE_ROUTE_CASE
    if (!launched) {
        set_error("route: internal error, expert slice %d x %d wavefronts", ept, nw);
        return MOE_EINVAL;
    }
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace

size_t packed_gate_bytes(const moe_shape &s)
{
    return static_cast<size_t>(padded_dim(s.d_model)) * pow2_ceil(s.E) * sizeof(float);
}

moe_status launch_pack_gate(const moe_shape &s, const void *Wg, float *Wgp, hipStream_t st)
{
    const int EP = pow2_ceil(s.E);
    const int dP = padded_dim(s.d_model);
    const int n = dP * EP;
    const dim3 grid(ceil_div(n, 256)), block(256);
    if (s.dtype == MOE_BF16)
        hipLaunchKernelGGL(pack_gate_kernel<uint16_t>, grid, block, 0, st,
                           static_cast<const uint16_t *>(Wg), Wgp, s.d_model, dP, s.E, EP);
    else
        hipLaunchKernelGGL(pack_gate_kernel<float>, grid, block, 0, st,
                           static_cast<const float *>(Wg), Wgp, s.d_model, dP, s.E, EP);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status launch_route(const moe_shape &s, const void *x, const void *Wgp,
                        const float *bias, int bias_stride, int32_t *expert_idx,
                        float *gate, int32_t *seg_cnt, hipStream_t st)
{
    if (s.dtype == MOE_BF16)
        return launch_route_t<uint16_t>(s, static_cast<const uint16_t *>(x),
                                        static_cast<const float *>(Wgp), bias, bias_stride,
                                        expert_idx, gate, seg_cnt, st);
    return launch_route_t<float>(s, static_cast<const float *>(x),
                                 static_cast<const float *>(Wgp), bias, bias_stride,
                                 expert_idx, gate, seg_cnt, st);
}

}  // namespace moe
