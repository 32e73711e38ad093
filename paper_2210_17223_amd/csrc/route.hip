// Gate: logits, top-k selection and softmax gate weights (paper Sec. 2.1).
//
// The logit of (token, expert) is one fp32 accumulator walked over the model
// dimension in ascending order with fused multiply-adds, so that the top-k
// decision (an integer result) does not depend on a reduction tree.  The work is
// therefore plain fp32 vector arithmetic on T x E independent chains.  A lane owns
// TPL tokens x EPL experts (a register block of chains, sized on the host so that the
// chip still has enough wavefronts); both operands come from LDS tiles of the token
// rows and of the packed gate matrix, 64 columns of the model dimension per stage,
// double buffered, with two or three further stages of global loads in flight in registers.
#include "common.h"

#include <algorithm>

namespace moe {
namespace {

constexpr int kGatePad = 128; // the packed gate matrix pads the model dimension to this
constexpr int kKC = 64;       // model-dimension columns per stage
constexpr int kLDX = kKC + 4; // LDS row pitch in floats: rows 4 banks apart, 16-byte aligned

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

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

// Top-k, softmax weights and the histogram of a block's tokens from their logits in LDS
// (zs[token][expert]; the histogram sits behind them), with LP lanes per token -- all 256
// lanes when the block has few tokens: lane `sub` of a token's group holds the logits of
// experts sub, sub + LP, ... (NQ of them) in registers; maxima, sums and the k selections
// are butterflies over the group.  Groups are aligned pieces of one wavefront.
template <int NQ>
__device__ __forceinline__ void route_tail(float (*zs)[kMaxExperts + 1], int32_t *__restrict__ expert_idx,
                                           float *__restrict__ gate, int32_t *__restrict__ seg_cnt,
                                           int t0, int T, int E, int TB, int LP, int k, int renorm)
{
    const int tid = threadIdx.x;
    int32_t *cnt = reinterpret_cast<int32_t *>(&zs[kWave][0]);
    if (seg_cnt != nullptr && tid < kMaxExperts) cnt[tid] = 0;
    const int tl = tid / LP, sub = tid % LP;
    const int t = t0 + tl;
    const bool live = tl < TB && t < T;
    float zl[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int e = sub + LP * q;
        zl[q] = (live && e < E) ? zs[tl][e] : -INFINITY;
    }
    if (seg_cnt != nullptr) __syncthreads();     // the histogram is cleared
    float zmax = zl[0];
#pragma unroll
    for (int q = 1; q < NQ; ++q) zmax = fmaxf(zmax, zl[q]);
    for (int m = 1; m < LP; m <<= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, m));
    float denom = 0.0f;
#pragma unroll
    for (int q = 0; q < NQ; ++q)
        if (sub + LP * q < E) denom += expf(zl[q] - zmax);
    for (int m = 1; m < LP; m <<= 1) denom += __shfl_xor(denom, m);

    constexpr int kNone = 0x7fffffff;            // "no candidate": never wins a comparison
    float sel_z[kMaxTopK];
    int sel_e[kMaxTopK];
    uint32_t taken = 0;                          // bit q: this lane's q-th expert is selected
    float gsum = 0.0f;
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
        sel_z[j] = 0.0f;
        sel_e[j] = 0;
        if (j < k) {
            float bz = -INFINITY;
            int be = kNone;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int e = sub + LP * q;      // ascending in q: a strict > keeps the lower index
                if (e < E && !((taken >> q) & 1u) && (be == kNone || zl[q] > bz)) {
                    bz = zl[q];
                    be = e;
                }
            }
            for (int m = 1; m < LP; m <<= 1) {
                const float oz = __shfl_xor(bz, m);
                const int oe = __shfl_xor(be, m);
                if (oe != kNone && (be == kNone || oz > bz || (oz == bz && oe < be))) {
                    bz = oz;
                    be = oe;
                }
            }
            if (be != kNone && be % LP == sub) taken |= 1u << (be / LP);
            sel_z[j] = bz;
            sel_e[j] = be;
            gsum += expf(bz - zmax) / denom;
        }
    }
    if (live && sub == 0) {
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j) {
            if (j < k) {
                const float g = expf(sel_z[j] - zmax) / denom;
                expert_idx[static_cast<size_t>(t) * k + j] = sel_e[j];
                gate[static_cast<size_t>(t) * k + j] = renorm ? g / gsum : g;
                if (seg_cnt != nullptr) atomicAdd(&cnt[sel_e[j]], 1);
            }
        }
    }
    if (seg_cnt != nullptr) {
        __syncthreads();
        if (tid < kMaxExperts)
            seg_cnt[static_cast<size_t>(blockIdx.x) * kMaxExperts + tid] = cnt[tid];
    }
}

// Block = TB tokens x EP experts (EP = E rounded up to a power of two), NG = EP / EPL
// expert groups x TB / TPL token groups of lanes.  Lane (tg, eg) owns tokens
// a * TG + tg and experts b * NG + eg (interleaved, so that the lanes of a wavefront read
// neighbouring LDS rows).  Wgp is the packed gate matrix: fp32 [EP][dP], expert-major,
// zero padded.  After the chains the logits go to LDS and the first wavefront finishes
// the block's tokens: top-k, softmax weights and, for the layer call, the expert
// histogram of these TB tokens (one segment of the dispatch plan).
template <typename XT, int TPL, int EPL>
__global__ __launch_bounds__(256, 2) void route_kernel(
    const XT *__restrict__ x, const float *__restrict__ Wgp,
    const float *__restrict__ bias, int bias_stride, int32_t *__restrict__ expert_idx,
    float *__restrict__ gate, int32_t *__restrict__ seg_cnt, int T, int d, int dP, int E, int EP,
    int TB, int k, int renorm)
{
    // register stages of global loads in flight: a stage of a large register block takes long
    // enough for two to cover the load latency
    constexpr int PD = TPL * EPL >= 4 ? 2 : 3;
    constexpr int UNR = PD == 2 ? 2 : 6;             // stages per unrolled trip: lcm(PD, 2)
    // LDS reads this many four-column steps ahead of the chain, in a register ring: a lane with
    // few chains has nothing else to cover their latency with
    constexpr int PF = TPL + EPL <= 2 ? 8 : TPL + EPL <= 4 ? 4 : 0;
    constexpr int VE = 16 / sizeof(XT);              // elements per 16-byte vector
    constexpr int XRV = kKC / VE;                    // 16-byte vectors per token row per stage
    constexpr int WRV = kKC / 4;                     // ... per gate-matrix row per stage
    constexpr int XV = 64 * XRV / 256;               // per thread, at most (TB <= 64, 256 threads)
    constexpr int WV = 64 * WRV / 256;               // per thread, at most (EP <= 64)
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float *xs = smem;                                // [2][TB][kLDX]
    float *ws = smem + 2 * TB * kLDX;                // [2][EP][kLDX]
    float (*zs)[kMaxExperts + 1] = reinterpret_cast<float (*)[kMaxExperts + 1]>(smem);

    const int tid = threadIdx.x, nthr = blockDim.x;
    const int NG = EP / EPL, TG = TB / TPL;
    // threads beyond NG * TG (few experts) only help to stage the tiles
    const bool active = tid < NG * TG;
    const int eg = tid % NG, tg = min(tid / NG, TG - 1);
    const int t0 = blockIdx.x * TB;

    // staging maps: x vector v = row (v / XRV), column (v % XRV) * VE; same for the matrix
    const int nxv = TB * XRV, nwv = EP * WRV;
    const XT *xsrc[XV];
    const float *wsrc[WV];
    int xdst[XV], wdst[WV], xcol[XV];
#pragma unroll
    for (int q = 0; q < XV; ++q) {
        const int v = min(tid + q * nthr, nxv - 1);
        const int r = v / XRV;
        xcol[q] = (v % XRV) * VE;
        xsrc[q] = x + static_cast<size_t>(min(t0 + r, T - 1)) * d + xcol[q];
        xdst[q] = r * kLDX + xcol[q];
    }
#pragma unroll
    for (int q = 0; q < WV; ++q) {
        const int v = min(tid + q * nthr, nwv - 1);
        const int r = v / WRV, c = (v % WRV) * 4;
        wsrc[q] = Wgp + static_cast<size_t>(r) * dP + c;
        wdst[q] = r * kLDX + c;
    }
    u32x4 xpre[PD][XV], wpre[PD][WV];
#define MOE_LOAD_STAGE(slot, k0)                                                      \
    {                                                                                 \
        _Pragma("unroll") for (int q = 0; q < XV; ++q)                                \
        {                                                                             \
            xpre[slot][q] = (u32x4){0u, 0u, 0u, 0u};                                  \
            if (tid + q * nthr < nxv && (k0) + xcol[q] < d)                           \
                xpre[slot][q] = *reinterpret_cast<const u32x4 *>(xsrc[q] + (k0));     \
        }                                                                             \
        _Pragma("unroll") for (int q = 0; q < WV; ++q)                                \
            if (tid + q * nthr < nwv)                                                 \
                wpre[slot][q] = *reinterpret_cast<const u32x4 *>(wsrc[q] + (k0));     \
    }
#define MOE_STORE_STAGE(slot, buf)                                                    \
    {                                                                                 \
        _Pragma("unroll") for (int q = 0; q < XV; ++q)                                \
            if (tid + q * nthr < nxv)                                                 \
                store_row_vec(xs + (buf) * TB * kLDX + xdst[q], xpre[slot][q], XT()); \
        _Pragma("unroll") for (int q = 0; q < WV; ++q)                                \
            if (tid + q * nthr < nwv)                                                 \
                *reinterpret_cast<u32x4 *>(ws + (buf) * EP * kLDX + wdst[q]) = wpre[slot][q]; \
    }

    float acc[TPL][EPL];
#pragma unroll
    for (int a = 0; a < TPL; ++a)
#pragma unroll
        for (int b = 0; b < EPL; ++b) acc[a][b] = 0.0f;

    const int nstage = dP / kKC;
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (u < nstage) MOE_LOAD_STAGE(u, u * kKC)
    for (int s0 = 0; s0 < nstage; s0 += UNR) {
        // unrolled so that the register slot (u % PD) and the LDS buffer (u & 1) of a stage
        // are compile-time
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int s = s0 + u;
            if (s < nstage) {
                const int buf = u & 1;
                MOE_STORE_STAGE(u % PD, buf)
                __syncthreads();
                if (s + PD < nstage) MOE_LOAD_STAGE(u % PD, (s + PD) * kKC)
                const float *xrow = xs + buf * TB * kLDX + tg * kLDX;
                const float *wrow = ws + buf * EP * kLDX + eg * kLDX;
                if constexpr (PF > 0) {
                    // a ring of PF four-column steps of operands in registers: the reads of step
                    // i + PF are issued right after step i's multiply-adds, so a read has PF
                    // steps of the chain to arrive (left alone, the compiler keeps one step ahead)
                    f32x4 xr[PF][TPL], wr[PF][EPL];
#pragma unroll
                    for (int p = 0; p < PF; ++p) {
#pragma unroll
                        for (int a = 0; a < TPL; ++a)
                            xr[p][a] = *reinterpret_cast<const f32x4 *>(xrow + a * TG * kLDX + p * 4);
#pragma unroll
                        for (int b = 0; b < EPL; ++b)
                            wr[p][b] = *reinterpret_cast<const f32x4 *>(wrow + b * NG * kLDX + p * 4);
                    }
#pragma unroll
                    for (int i4 = 0; i4 < kKC / 4; ++i4) {
                        const int slot = i4 % PF;
#pragma unroll
                        for (int c = 0; c < 4; ++c)
#pragma unroll
                            for (int a = 0; a < TPL; ++a)
#pragma unroll
                                for (int b = 0; b < EPL; ++b)
                                    acc[a][b] = __builtin_fmaf(xr[slot][a][c], wr[slot][b][c], acc[a][b]);
                        if (i4 + PF < kKC / 4) {
#pragma unroll
                            for (int a = 0; a < TPL; ++a)
                                xr[slot][a] = *reinterpret_cast<const f32x4 *>(xrow + a * TG * kLDX + (i4 + PF) * 4);
#pragma unroll
                            for (int b = 0; b < EPL; ++b)
                                wr[slot][b] = *reinterpret_cast<const f32x4 *>(wrow + b * NG * kLDX + (i4 + PF) * 4);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll 4
                for (int i4 = 0; i4 < kKC / 4; ++i4) {
                    f32x4 xv[TPL], wv[EPL];
#pragma unroll
                    for (int a = 0; a < TPL; ++a)
                        xv[a] = *reinterpret_cast<const f32x4 *>(xrow + a * TG * kLDX + i4 * 4);
#pragma unroll
                    for (int b = 0; b < EPL; ++b)
                        wv[b] = *reinterpret_cast<const f32x4 *>(wrow + b * NG * kLDX + i4 * 4);
#pragma unroll
                    for (int c = 0; c < 4; ++c)
#pragma unroll
                        for (int a = 0; a < TPL; ++a)
#pragma unroll
                            for (int b = 0; b < EPL; ++b)
                                acc[a][b] = __builtin_fmaf(xv[a][c], wv[b][c], acc[a][b]);
                }
                }
            }
        }
    }
#undef MOE_LOAD_STAGE
#undef MOE_STORE_STAGE
    __syncthreads();           // every wavefront is done with the tiles: reuse them for logits

#pragma unroll
    for (int a = 0; a < TPL; ++a) {
        const int tl = a * TG + tg;
        const int t = t0 + tl;
#pragma unroll
        for (int b = 0; b < EPL; ++b) {
            const int e = b * NG + eg;
            if (active && e < E) {
                float z = acc[a][b];
                if (bias != nullptr && t < T)
                    z = z + bias[static_cast<size_t>(t) * bias_stride + e];
                zs[tl][e] = z;
            }
        }
    }
    __syncthreads();
    const int LP = min(min(256 / TB, EP), kWave);      // lanes per token in the tail
    switch (EP / LP) {                                 // logits per lane: at most 16 (LP >= 4 when EP = 64)
    case 1: route_tail<1>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    case 2: route_tail<2>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    case 4: route_tail<4>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    case 8: route_tail<8>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    default: route_tail<16>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    }
}

// The gate for problems with few chains (one chain per lane, T * EP of them): there the
// chain of d dependent FMAs IS the time, so neither its operands nor the LDS pipe may make
// it wait.
//  * Operands: the tiles of a 64-column stage go from global memory straight into an LDS
//    ring of kChainStages stages (gfx950's 16-byte load-to-LDS: a wavefront's 64 lanes fill
//    1 KiB of consecutive LDS, so a stage is laid out in 1 KiB chunks and each lane fetches
//    whatever belongs at its place), several stages ahead of the chain, with an exact count
//    of the loads in flight; no registers, no LDS store phase, one barrier per stage.
//  * LDS pipe: a lane that reads both of its operands from LDS moves 32 bytes per four FMAs,
//    and the four wavefronts of a block then keep the pipe busier than the chains keep the
//    ALUs.  So a row of 16 lanes is one expert and its lanes are 16 tokens: every lane reads
//    its own token's 16 columns (storage type: 32 bytes of bf16), ONE 4-byte read per lane
//    brings the row's 16 gate-matrix values, and each FMA takes its value from the lane
//    that holds it through the DPP row broadcast -- about a third of the LDS traffic.
//  * The 16-byte pieces of both tiles are XOR-swizzled with their row, so that the 16
//    tokens (x) and the 4 experts (gate matrix) a wavefront reads at once fall into
//    different banks.
// Reads run two 16-column groups ahead of the chain, across stage boundaries (the barrier
// that publishes stage s + 1 sits in the middle of stage s).
// Shapes: d a multiple of 64, a stage of at most 8 KiB, EP * ceil(TB / 16) <= 16 rows.
constexpr int kChainStages = 8;

#define MOE_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// acc += w[lane J of this lane's row of 16] * xv.  FIRST: w may just have been written.
template <int J, bool FIRST>
__device__ __forceinline__ void fmac_row_bcast(float &acc, float w, float xv)
{
#if defined(__HIP_DEVICE_COMPILE__)
    if constexpr (FIRST)
        asm("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
            : "+v"(acc) : "v"(w), "v"(xv), "n"(J));
    else
        asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
            : "+v"(acc) : "v"(w), "v"(xv), "n"(J));
#endif
}

template <typename XT>
struct ChainGroup {                    // operands of 16 columns
    static constexpr int XQ = 16 * sizeof(XT) / 16;      // 16-byte pieces of the token row
    float w;
    uint4 xq[XQ];
};

template <typename XT, int CPW>
__global__ __launch_bounds__(256, 2) void route_chain_kernel(
    const XT *__restrict__ x, const float *__restrict__ Wgp, const float *__restrict__ bias,
    int bias_stride, int32_t *__restrict__ expert_idx, float *__restrict__ gate,
    int32_t *__restrict__ seg_cnt, int T, int d, int dP, int E, int EP, int TB, int k, int renorm)
{
#if defined(__HIP_DEVICE_COMPILE__)   // (the host pass needs the launch stub only)
    constexpr int NS = kChainStages;
    constexpr int XROWB = kKC * static_cast<int>(sizeof(XT));     // bytes of a token row per stage
    constexpr int WROWB = kKC * 4;                                // ... of a gate-matrix row
    constexpr int XQ = ChainGroup<XT>::XQ;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    char *ring = reinterpret_cast<char *>(smem);
    float (*zs)[kMaxExperts + 1] = reinterpret_cast<float (*)[kMaxExperts + 1]>(smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // row of 16 lanes = (expert, sixteen tokens); lane of the row = token
    const int TB16 = (TB + 15) >> 4;
    const int row_e = (tid >> 4) / TB16, tok = ((tid >> 4) % TB16) * 16 + (tid & 15);
    const bool active = row_e < EP && tok < TB;
    const int eg = min(row_e, EP - 1), tg = min(tok, TB - 1);     // idle lanes repeat a chain
    const int t0 = blockIdx.x * TB;
    const int xbytes = (TB * XROWB + 1023) / 1024 * 1024;         // a stage: token rows, then
    const int wbytes = (EP * WROWB + 1023) / 1024 * 1024;         // gate-matrix rows, in 1 KiB chunks
    const int stage_bytes = xbytes + wbytes;
    const int chunks = stage_bytes / 1024;
    // where piece v of a row's 16-byte pieces sits: v ^ swizzle(row)
    auto xswizzle = [](int row) { return sizeof(XT) == 2 ? ((row ^ (row >> 3)) & 7) : (row & 15); };

    // this lane's CPW loads per stage: chunk wave + 4 j (surplus loads repeat the last chunk)
    const char *gsrc[CPW];
    int gstep[CPW], cbyte[CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
        const int c = min(wave + 4 * j, chunks - 1);
        cbyte[j] = c * 1024;
        const int p = c * 1024 + lane * 16;                       // this lane's place in the stage
        if (p < xbytes) {
            const int row = min(p / XROWB, TB - 1), vec = ((p % XROWB) / 16) ^ xswizzle(row);
            gsrc[j] = reinterpret_cast<const char *>(x + static_cast<size_t>(min(t0 + row, T - 1)) * d) + vec * 16;
            gstep[j] = XROWB;
        } else {
            const int q = p - xbytes;
            const int row = min(q / WROWB, EP - 1), vec = ((q % WROWB) / 16) ^ (row & 15);
            gsrc[j] = reinterpret_cast<const char *>(Wgp + static_cast<size_t>(row) * dP) + vec * 16;
            gstep[j] = WROWB;
        }
    }
    // The load is written out rather than taken from the compiler's builtin: behind the
    // builtin every later LDS read is made to wait until NO load is in flight, which is the
    // one thing this kernel must not do.  M0 = the wavefront's place in LDS; lane l lands at
    // M0 + 16 l.  Completion is counted by hand below.
    const uint32_t ring_lds = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(MOE_LDS_PTR(ring)));
#define MOE_CHAIN_LOAD(s_)                                                                    \
    {                                                                                         \
        const uint32_t slot_ = ring_lds + ((s_) % NS) * stage_bytes;                          \
        _Pragma("unroll") for (int j = 0; j < CPW; ++j) {                                     \
            const char *g_ = gsrc[j] + static_cast<size_t>(s_) * gstep[j];                    \
            const uint32_t m_ = __builtin_amdgcn_readfirstlane(slot_ + cbyte[j]);             \
            uint32_t keep_;                                  /* M0 is handed back as found */ \
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\t"               \
                         "global_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"                 \
                         : "=&s"(keep_) : "v"(g_), "s"(m_) : "memory");                       \
        }                                                                                     \
    }
    // Stage s_ becomes readable: this wavefront's part of it has landed once at most the
    // loads of the NS - 3 stages behind it are in flight; after the barrier everybody's has,
    // and everybody has consumed stage s_ - 2, whose place the next loads take.  A plain
    // s_barrier: __syncthreads() would first wait for ALL loads into LDS in flight.
#define MOE_CHAIN_SYNC(s_)                                                                    \
    {                                                                                         \
        if ((s_) + NS - 3 <= nstage - 1)                                                      \
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 3) * CPW) : "memory");             \
        else                                                                                  \
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                  \
        __builtin_amdgcn_s_barrier();                                                         \
        asm volatile("" ::: "memory");                                                        \
        if ((s_) - 2 + NS < nstage) MOE_CHAIN_LOAD((s_) - 2 + NS)                             \
    }
    const int nstage = d / kKC;                       // (columns past d meet zeros of the matrix)
    for (int s = 0; s < NS - 2; ++s)
        if (s < nstage) MOE_CHAIN_LOAD(s)

    float acc = 0.0f;
    const int xoff = tg * XROWB, xswz = xswizzle(tg);
    const int woff = xbytes + eg * WROWB, wswz = eg & 15;
    const int wl = tid & 15;                          // the gate-matrix column this lane fetches
    ChainGroup<XT> grp[4];
    // group g_ of stage s_: columns 16 g_ .. 16 g_ + 15
#define MOE_CHAIN_READ(slot_, s_, g_)                                                         \
    {                                                                                         \
        const char *base_ = ring + ((s_) % NS) * stage_bytes;                                 \
        grp[slot_].w = *reinterpret_cast<const float *>(                                      \
            base_ + woff + ((((g_) * 4 + (wl >> 2)) ^ wswz) << 4) + ((wl & 3) << 2));         \
        _Pragma("unroll") for (int q = 0; q < XQ; ++q)                                        \
            grp[slot_].xq[q] = *reinterpret_cast<const uint4 *>(                              \
                base_ + xoff + ((((g_) * XQ + q) ^ xswz) << 4));                              \
    }
    auto compute = [&](const ChainGroup<XT> &g) {
        float xv[16];
#pragma unroll
        for (int q = 0; q < XQ; ++q) {
            const uint32_t u[4] = {g.xq[q].x, g.xq[q].y, g.xq[q].z, g.xq[q].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if constexpr (sizeof(XT) == 2) {
                    xv[q * 8 + 2 * c] = __uint_as_float(u[c] << 16);
                    xv[q * 8 + 2 * c + 1] = __uint_as_float(u[c] & 0xFFFF0000u);
                } else {
                    xv[q * 4 + c] = __uint_as_float(u[c]);
                }
            }
        }
        fmac_row_bcast<0, true>(acc, g.w, xv[0]);
        fmac_row_bcast<1, false>(acc, g.w, xv[1]);
        fmac_row_bcast<2, false>(acc, g.w, xv[2]);
        fmac_row_bcast<3, false>(acc, g.w, xv[3]);
        fmac_row_bcast<4, false>(acc, g.w, xv[4]);
        fmac_row_bcast<5, false>(acc, g.w, xv[5]);
        fmac_row_bcast<6, false>(acc, g.w, xv[6]);
        fmac_row_bcast<7, false>(acc, g.w, xv[7]);
        fmac_row_bcast<8, false>(acc, g.w, xv[8]);
        fmac_row_bcast<9, false>(acc, g.w, xv[9]);
        fmac_row_bcast<10, false>(acc, g.w, xv[10]);
        fmac_row_bcast<11, false>(acc, g.w, xv[11]);
        fmac_row_bcast<12, false>(acc, g.w, xv[12]);
        fmac_row_bcast<13, false>(acc, g.w, xv[13]);
        fmac_row_bcast<14, false>(acc, g.w, xv[14]);
        fmac_row_bcast<15, false>(acc, g.w, xv[15]);
    };
    // every kernel argument is in its registers before the loop: a scalar load still in
    // flight there would make each wait on an LDS read a wait for all of them
    asm volatile("" ::"s"(bias), "s"(seg_cnt), "s"(expert_idx), "s"(gate), "s"(bias_stride),
                 "s"(E), "s"(k), "s"(renorm), "s"(T));
    MOE_CHAIN_SYNC(0)
    MOE_CHAIN_READ(0, 0, 0)
    MOE_CHAIN_READ(1, 0, 1)
    // (every iteration issues the same reads, so that the counts of reads in flight are
    // static: behind the last stage they fetch a place of the ring that nobody consumes)
    for (int s = 0; s < nstage; ++s) {
        // (the fences keep the compiler from gathering the reads in one place, where it
        // would then wait for all of them)
        MOE_CHAIN_READ(2, s, 2)
        __builtin_amdgcn_sched_barrier(0);
        compute(grp[0]);
        __builtin_amdgcn_sched_barrier(0);
        MOE_CHAIN_READ(3, s, 3)
        __builtin_amdgcn_sched_barrier(0);
        compute(grp[1]);
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < nstage) MOE_CHAIN_SYNC(s + 1)
        MOE_CHAIN_READ(0, s + 1, 0)
        __builtin_amdgcn_sched_barrier(0);
        compute(grp[2]);
        __builtin_amdgcn_sched_barrier(0);
        MOE_CHAIN_READ(1, s + 1, 1)
        __builtin_amdgcn_sched_barrier(0);
        compute(grp[3]);
        __builtin_amdgcn_sched_barrier(0);
    }
#undef MOE_CHAIN_READ
#undef MOE_CHAIN_SYNC
#undef MOE_CHAIN_LOAD
    __syncthreads();                  // every wavefront is done with the ring: reuse it for logits
    {
        const int t = t0 + tg;
        if (active && eg < E) {
            float z = acc;
            if (bias != nullptr && t < T) z = z + bias[static_cast<size_t>(t) * bias_stride + eg];
            zs[tg][eg] = z;
        }
    }
    __syncthreads();
    const int LP = min(min(256 / TB, EP), kWave);
    switch (EP / LP) {
    case 1: route_tail<1>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    case 2: route_tail<2>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    case 4: route_tail<4>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    case 8: route_tail<8>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    default: route_tail<16>(zs, expert_idx, gate, seg_cnt, t0, T, E, TB, LP, k, renorm); break;
    }
#endif
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

// Register block of chains per lane and tokens per block for a layer shape: the largest
// block that still leaves about eight wavefronts per compute unit, a block of 256 lanes
// covering at most 64 tokens (the tail and the plan's segments are one wavefront wide).
struct RouteShape {
    int tpl, epl, tb;
};

RouteShape route_shape(const moe_shape &s)
{
    static const int cand[5][2] = {{4, 4}, {2, 4}, {2, 2}, {1, 2}, {1, 1}};
    const int EP = pow2_ceil(s.E);
    const long chains = static_cast<long>(s.T) * EP;
    for (int c = 0; c < 5; ++c) {
        const int tpl = cand[c][0], epl = cand[c][1];
        if (epl > EP) continue;
        const int ng = EP / epl;
        const int tb = std::min(64, 256 * tpl / ng);
        if (tb < tpl) continue;
        const bool last = c == 4;
        if (last || chains / (tpl * epl) >= 131072) {
            // a handful of tokens: fewer blocks than compute units -- spread them (the lanes
            // of a block share its LDS, and a chain is only as fast as its operands arrive)
            int few = tb;
            while (few > 8 && few > tpl && (s.T + few - 1) / few < 256) few /= 2;
            return {tpl, epl, few};
        }
    }
    return {1, 1, std::min(64, 256 / EP)};
}

template <typename XT>
moe_status launch_route_t(const moe_shape &s, const XT *x, const float *Wgp,
                          const float *bias, int bias_stride, int32_t *expert_idx,
                          float *gate, int32_t *seg_cnt, hipStream_t st)
{
    const int EP = pow2_ceil(s.E);
    const int dP = padded_dim(s.d_model);
    const RouteShape rs = route_shape(s);
    const int blocks = ceil_div(s.T, rs.tb);
    // one chain per lane and a small stage: the kernel that streams its operands through LDS
    {
        const int xrowb = kKC * static_cast<int>(sizeof(XT));
        const int stage = (rs.tb * xrowb + 1023) / 1024 * 1024 + (EP * kKC * 4 + 1023) / 1024 * 1024;
        const size_t logits = sizeof(float) * (kWave + 2) * (kMaxExperts + 1);
        if (rs.tpl == 1 && rs.epl == 1 && s.d_model % kKC == 0 && stage <= 8192 &&
            EP * ((rs.tb + 15) / 16) <= 16) {
            const int cpw = (stage / 1024 + 3) / 4;       // 1 or 2: a stage is at most 8 chunks
            const size_t lds = std::max(static_cast<size_t>(kChainStages) * stage, logits);
#define MOE_CHAIN_CASE(CPW_)                                                                  \
    if (cpw == CPW_) {                                                                        \
        auto kern = route_chain_kernel<XT, CPW_>;                                             \
        static PerDeviceOnce once;                                                            \
        once.raise_lds(reinterpret_cast<const void *>(kern), 72 * 1024);                              \
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, st, x, Wgp, bias, bias_stride, \
                           expert_idx, gate, seg_cnt, s.T, s.d_model, dP, s.E, EP, rs.tb,     \
                           s.k, s.renorm_topk);                                               \
    }
            MOE_CHAIN_CASE(1) MOE_CHAIN_CASE(2)
#undef MOE_CHAIN_CASE
            MOE_TRY_HIP(hipGetLastError());
            return MOE_OK;
        }
    }
    const size_t tiles = sizeof(float) * 2 * (rs.tb + EP) * kLDX;
    const size_t logits = sizeof(float) * (kWave + 2) * (kMaxExperts + 1);
    const size_t lds = std::max(tiles, logits);
#define MOE_ROUTE_CASE(TPL_, EPL_)                                                            \
    if (rs.tpl == TPL_ && rs.epl == EPL_) {                                                   \
        auto kern = route_kernel<XT, TPL_, EPL_>;                                             \
        static PerDeviceOnce once;                                                            \
        once.raise_lds(reinterpret_cast<const void *>(kern), 72 * 1024);                              \
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, st, x, Wgp, bias, bias_stride, \
                           expert_idx, gate, seg_cnt, s.T, s.d_model, dP, s.E, EP, rs.tb,     \
                           s.k, s.renorm_topk);                                               \
        launched = true;                                                                      \
    }
    bool launched = false;
    MOE_ROUTE_CASE(4, 4) MOE_ROUTE_CASE(2, 4) MOE_ROUTE_CASE(2, 2) MOE_ROUTE_CASE(1, 2) MOE_ROUTE_CASE(1, 1)
#undef MOE_ROUTE_CASE
    if (!launched) {
        set_error("route: internal error, register block %d x %d", rs.tpl, rs.epl);
        return MOE_EINVAL;
    }
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace

int route_segment_tokens(const moe_shape &s) { return route_shape(s).tb; }

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
