// Dispatch plan: per-expert histogram, stable token-order rank, capacity bound,
// exclusive scan, slot of every assignment -- the layout of the expert-major
// buffer that the first all-to-all would carry (paper, end of Sec. 2.1).
//
// Integer work only.  A wavefront ranks a segment of kSeg consecutive assignments,
// 64 at a time: lanes that chose the same expert find each other with six ballots
// (one per bit of the expert index), the rank inside the 64 is a popcount of the
// lower lanes, and the running per-expert count lives in LDS.
//   plan_count : per-segment expert histograms
//   plan_scan  : one block; exclusive scan over segments per expert, totals,
//                capacity clamp, offsets
//   plan_rank  : per-segment ranks -> slot_of / src_of
//   plan_tiles : row tiles of the grouped GEMM per chunk (binary search in src_of)
#include "common.h"

namespace moe {
namespace {

constexpr int kPlanWaves = 4;                    // wavefronts (segments) per block
constexpr int kPlanThreads = kPlanWaves * kWave;

// Mask of the lanes whose (valid) expert equals this lane's.
__device__ __forceinline__ uint64_t same_expert_lanes(int e, bool valid)
{
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        const bool bit = (e >> b) & 1;
        const uint64_t m = __ballot(bit);
        peers &= bit ? m : ~m;
    }
    return peers;
}

__device__ __forceinline__ uint64_t lanes_below(int lane)
{
    return (1ull << lane) - 1ull;
}

__device__ __forceinline__ int clamp_expert(int e, int E)
{
    return static_cast<unsigned>(e) < static_cast<unsigned>(E) ? e : E - 1;
}

__global__ __launch_bounds__(kPlanThreads) void plan_count_kernel(
    const int32_t *__restrict__ expert_idx, int32_t *__restrict__ seg_cnt, int n, int E)
{
    __shared__ int32_t run[kPlanWaves][kMaxExperts];
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int seg = blockIdx.x * kPlanWaves + wave;
    run[wave][lane] = 0;
    __builtin_amdgcn_wave_barrier();
    const int base = seg * kSeg;
    for (int off = 0; off < kSeg; off += kWave) {
        const int i = base + off + lane;
        const bool valid = i < n;
        const int e = valid ? clamp_expert(expert_idx[i], E) : 0;
        const uint64_t peers = same_expert_lanes(e, valid);
        const bool leader = valid && (peers & lanes_below(lane)) == 0;
        if (leader) run[wave][e] += __popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
    if (base < n) seg_cnt[static_cast<size_t>(seg) * kMaxExperts + lane] = run[wave][lane];
}

// One block of 16 groups x 64 experts.  seg_cnt[seg][e] becomes the number of
// assignments to e in all earlier segments.
__global__ __launch_bounds__(1024) void plan_scan_kernel(
    int32_t *__restrict__ seg_cnt, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int nseg, int E, int capacity)
{
    __shared__ int32_t gsum[16][kMaxExperts];
    __shared__ int32_t kept[kMaxExperts];
    const int e = threadIdx.x % kMaxExperts;
    const int g = threadIdx.x / kMaxExperts;
    const int per = ceil_div(nseg, 16);
    const int s0 = min(g * per, nseg), s1 = min(s0 + per, nseg);
    int32_t local = 0;
    for (int s = s0; s < s1; ++s) local += seg_cnt[static_cast<size_t>(s) * kMaxExperts + e];
    gsum[g][e] = local;
    __syncthreads();
    int32_t before = 0, total = 0;
    for (int gg = 0; gg < 16; ++gg) {
        const int32_t v = gsum[gg][e];
        if (gg < g) before += v;
        total += v;
    }
    int32_t running = before;
    for (int s = s0; s < s1; ++s) {
        const size_t at = static_cast<size_t>(s) * kMaxExperts + e;
        const int32_t c = seg_cnt[at];
        seg_cnt[at] = running;
        running += c;
    }
    if (g == 0) {
        if (e < E) counts[e] = total;
        kept[e] = e < E ? min(total, capacity) : 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t acc = 0;
        for (int ee = 0; ee < E; ++ee) {
            offsets[ee] = acc;
            acc += kept[ee];
        }
        offsets[E] = acc;
    }
}

__global__ __launch_bounds__(kPlanThreads) void plan_rank_kernel(
    const int32_t *__restrict__ expert_idx, const int32_t *__restrict__ seg_base,
    const int32_t *__restrict__ offsets, int32_t *__restrict__ slot_of,
    int32_t *__restrict__ src_of, int n, int E, int capacity)
{
    __shared__ int32_t run[kPlanWaves][kMaxExperts];
    __shared__ int32_t off_s[kMaxExperts];
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int seg = blockIdx.x * kPlanWaves + wave;
    const int base = seg * kSeg;
    if (threadIdx.x < kMaxExperts) off_s[threadIdx.x] = threadIdx.x < E ? offsets[threadIdx.x] : 0;
    run[wave][lane] = base < n ? seg_base[static_cast<size_t>(seg) * kMaxExperts + lane] : 0;
    __syncthreads();
    for (int off = 0; off < kSeg; off += kWave) {
        const int i = base + off + lane;
        const bool valid = i < n;
        const int e = valid ? clamp_expert(expert_idx[i], E) : 0;
        const uint64_t peers = same_expert_lanes(e, valid);
        const int rank = __popcll(peers & lanes_below(lane));
        const int32_t before = run[wave][e];
        __builtin_amdgcn_wave_barrier();
        if (valid && rank == 0) run[wave][e] = before + __popcll(peers);
        __builtin_amdgcn_wave_barrier();
        if (valid) {
            const int32_t pos = before + rank;
            const int32_t slot = pos < capacity ? off_s[e] + pos : -1;
            slot_of[i] = slot;
            if (slot >= 0) src_of[slot] = i;
        }
    }
}

// Row tiles of chunk c (block c): expert e's rows of the chunk are the slots whose
// source assignment lies in [t0*k, t1*k); src_of ascends inside an expert, so both
// ends are binary searches.  Lane e owns expert e.
__global__ __launch_bounds__(kWave) void plan_tiles_kernel(
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ src_of,
    RowTile *__restrict__ tiles, int32_t *__restrict__ ntiles, int T, int k, int E,
    int n_chunks, int tile_rows, int max_tiles)
{
    const int c = blockIdx.x;
    const int e = threadIdx.x;
    const long t0 = static_cast<long>(c) * T / n_chunks;
    const long t1 = static_cast<long>(c + 1) * T / n_chunks;
    int lo = 0, hi = 0;
    if (e < E) {
        const int b = offsets[e], end = offsets[e + 1];
        if (n_chunks == 1) {
            lo = b;
            hi = end;
        } else {
            const int keys[2] = {static_cast<int>(t0 * k), static_cast<int>(t1 * k)};
            int res[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                int l = b, r = end;             // first slot in [b,end) with src >= key
                while (l < r) {
                    const int m = (l + r) >> 1;
                    if (src_of[m] < keys[q]) l = m + 1; else r = m;
                }
                res[q] = l;
            }
            lo = res[0];
            hi = res[1];
        }
    }
    const int mine = ceil_div(hi - lo, tile_rows);
    // exclusive prefix sum over the 64 lanes
    int incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int v = __shfl_up(incl, d);
        if (e >= d) incl += v;
    }
    const int first = incl - mine;
    RowTile *out = tiles + static_cast<size_t>(c) * max_tiles;
    for (int q = 0; q < mine; ++q) {
        if (first + q < max_tiles) {
            RowTile rt;
            rt.expert = e;
            rt.row0 = lo + q * tile_rows;
            rt.row1 = min(hi, lo + (q + 1) * tile_rows);
            rt.pad = 0;
            out[first + q] = rt;
        }
    }
    if (e == kWave - 1) ntiles[c] = min(incl, max_tiles);
}

}  // namespace

moe_status launch_plan(const moe_shape &s, const int32_t *expert_idx, int32_t *counts,
                       int32_t *offsets, int32_t *slot_of, int32_t *src_of,
                       const Workspace &w, hipStream_t st)
{
    const int n = s.T * s.k;
    const int blocks = ceil_div(w.nseg, kPlanWaves);
    hipLaunchKernelGGL(plan_count_kernel, dim3(blocks), dim3(kPlanThreads), 0, st,
                       expert_idx, w.seg_cnt, n, s.E);
    hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(1024), 0, st, w.seg_cnt, counts,
                       offsets, w.nseg, s.E, s.capacity);
    hipLaunchKernelGGL(plan_rank_kernel, dim3(blocks), dim3(kPlanThreads), 0, st,
                       expert_idx, w.seg_cnt, offsets, slot_of, src_of, n, s.E, s.capacity);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status launch_tiles(const moe_shape &s, int n_chunks, const int32_t *offsets,
                        const int32_t *src_of, const Workspace &w, hipStream_t st)
{
    hipLaunchKernelGGL(plan_tiles_kernel, dim3(n_chunks), dim3(kWave), 0, st, offsets,
                       src_of, w.tiles, w.ntiles, s.T, s.k, s.E, n_chunks, w.tile_rows,
                       w.max_tiles);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace moe
