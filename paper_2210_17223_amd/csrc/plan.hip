// Dispatch plan: per-expert histogram, stable token-order rank, capacity bound,
// exclusive scan, slot of every assignment -- the layout of the expert-major
// buffer that the first all-to-all would carry (paper, end of Sec. 2.1).
//
// Integer work only.  A wavefront ranks one segment (the assignments of kSegTok
// consecutive tokens), 64 at a time: lanes that chose the same expert find each other
// with six ballots (one per bit of the expert index), the rank inside the 64 is a
// popcount of the lower lanes, and the running per-expert count lives in LDS.
//   plan_count : per-segment expert histograms (the layer call gets them from the
//                gate's top-k kernel instead)
//   plan_scan  : one block; exclusive scan over segments per expert, totals,
//                capacity clamp, offsets; for an unchunked layer also the work lists
//   plan_rank  : per-segment ranks -> slot_of / src_of
//   plan_rank_prefix : scan and rank in one launch when there are few segments
//   plan_items : work lists of the two expert GEMMs per chunk
#include "common.h"

namespace moe {
namespace {

constexpr int kPlanWaves = 4;                    // wavefronts (segments) per block
constexpr int kPrefixSegments = 512;             // plans up to this many segments: one launch
constexpr int kItemBlocks = 8;                   // ... whose work lists are built by this many blocks
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

// An index outside [0, E) names no expert (a padding marker such as -1): the assignment is
// left out of the counts, takes no slot and gets slot_of = -1.
__device__ __forceinline__ bool names_expert(int e, int E)
{
    return static_cast<unsigned>(e) < static_cast<unsigned>(E);
}

__device__ void build_items(const GemmPlan &gp, WorkItem *__restrict__ items,
                            int32_t *__restrict__ nitems_out, const int32_t *lo_s,
                            const int32_t *hi_s, int32_t *mt_s, int32_t *cum_s, int part,
                            int nparts);

__global__ __launch_bounds__(kPlanThreads) void plan_count_kernel(
    const int32_t *__restrict__ expert_idx, int32_t *__restrict__ seg_cnt, int n, int E,
    int seg_len)
{
    __shared__ int32_t run[kPlanWaves][kMaxExperts];
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int seg = blockIdx.x * kPlanWaves + wave;
    run[wave][lane] = 0;
    __builtin_amdgcn_wave_barrier();
    const int base = seg * seg_len;
    for (int off = 0; off < seg_len; off += kWave) {
        const int i = base + off + lane;
        const bool in_seg = i < n && off + lane < seg_len;
        const int e_raw = in_seg ? expert_idx[i] : 0;
        const bool valid = in_seg && names_expert(e_raw, E);
        const int e = valid ? e_raw : 0;
        const uint64_t peers = same_expert_lanes(e, valid);
        const bool leader = valid && (peers & lanes_below(lane)) == 0;
        if (leader) run[wave][e] += __popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
    if (base < n) seg_cnt[static_cast<size_t>(seg) * kMaxExperts + lane] = run[wave][lane];
}

// One block of 1024 lanes = G groups x EPs experts (EPs = E rounded up to a power of two),
// each group walking its contiguous share of the segments.  seg_cnt[seg][e] becomes the
// number of assignments to e in all earlier segments.
__global__ __launch_bounds__(1024) void plan_scan_kernel(
    int32_t *__restrict__ seg_cnt, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int nseg, int E, int EPs, int capacity, int with_items,
    WorkItem *__restrict__ items0, int32_t *__restrict__ nitems0, GemmPlan gp0,
    WorkItem *__restrict__ items1, int32_t *__restrict__ nitems1, GemmPlan gp1)
{
    __shared__ int32_t gsum[1024];                 // [G][EPs]
    __shared__ int32_t kept[kMaxExperts];
    __shared__ int32_t lo_s[kMaxExperts], hi_s[kMaxExperts], mt_s[kMaxExperts];
    __shared__ int32_t cum_s[kMaxExperts + 1];
    // groups: about four segments each, at least 16, at most what 1024 lanes hold
    const int G = min(1024 / EPs, max(16, nseg / 4));
    const int e = threadIdx.x % EPs;
    const int g = threadIdx.x / EPs;
    const int per = ceil_div(nseg, G);
    const int s0 = min(g * per, nseg), s1 = min(s0 + per, nseg);
    // The common case (at most eight segments per group) keeps the group's counts in
    // registers: one batch of loads instead of two dependent passes over global memory.
    constexpr int kKeep = 8;
    int32_t c[kKeep];
    int32_t local = 0;
    if (per <= kKeep) {
#pragma unroll
        for (int q = 0; q < kKeep; ++q)
            c[q] = s0 + q < s1 ? seg_cnt[static_cast<size_t>(s0 + q) * kMaxExperts + e] : 0;
#pragma unroll
        for (int q = 0; q < kKeep; ++q) local += c[q];
    } else {
        for (int s = s0; s < s1; ++s) local += seg_cnt[static_cast<size_t>(s) * kMaxExperts + e];
    }
    if (g < G) gsum[g * EPs + e] = local;
    if (threadIdx.x < kMaxExperts) kept[threadIdx.x] = 0;
    __syncthreads();
    int32_t before = 0, total = 0;
    for (int gg = 0; gg < G; ++gg) {
        const int32_t v = gsum[gg * EPs + e];
        if (gg < g) before += v;
        total += v;
    }
    int32_t running = before;
    if (per <= kKeep) {
#pragma unroll
        for (int q = 0; q < kKeep; ++q) {
            if (s0 + q < s1) seg_cnt[static_cast<size_t>(s0 + q) * kMaxExperts + e] = running;
            running += c[q];
        }
    } else {
        for (int s = s0; s < s1; ++s) {
            const size_t at = static_cast<size_t>(s) * kMaxExperts + e;
            const int32_t cc = seg_cnt[at];
            seg_cnt[at] = running;
            running += cc;
        }
    }
    if (g == 0 && e < E) {
        counts[e] = total;
        kept[e] = min(total, capacity);
    }
    __syncthreads();
    if (threadIdx.x < kWave) {                      // exclusive scan of kept[] by one wavefront
        const int ee = threadIdx.x;
        int incl = kept[ee];
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int v = __shfl_up(incl, d);
            if (ee >= d) incl += v;
        }
        lo_s[ee] = incl - kept[ee];
        hi_s[ee] = incl;
        if (ee < E) offsets[ee] = incl - kept[ee];
        if (ee == E - 1) offsets[E] = incl;
    }
    __syncthreads();
    if (with_items) {
        build_items(gp0, items0, nitems0, lo_s, hi_s, mt_s, cum_s, 0, 1);
        build_items(gp1, items1, nitems1, lo_s, hi_s, mt_s, cum_s, 0, 1);
    }
}

__global__ __launch_bounds__(kPlanThreads) void plan_rank_kernel(
    const int32_t *__restrict__ expert_idx, const int32_t *__restrict__ seg_base,
    const int32_t *__restrict__ offsets, int32_t *__restrict__ slot_of,
    int32_t *__restrict__ src_of, int n, int E, int capacity, int seg_len, int padded)
{
    __shared__ int32_t run[kPlanWaves][kMaxExperts];
    __shared__ int32_t off_s[kMaxExperts];
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int seg = blockIdx.x * kPlanWaves + wave;
    const int base = seg * seg_len;
    // padded layout: expert e owns the slots [e * capacity, (e + 1) * capacity)
    if (threadIdx.x < kMaxExperts)
        off_s[threadIdx.x] = static_cast<int>(threadIdx.x) >= E ? 0 : padded ? threadIdx.x * capacity : offsets[threadIdx.x];
    run[wave][lane] = base < n ? seg_base[static_cast<size_t>(seg) * kMaxExperts + lane] : 0;
    __syncthreads();
    for (int off = 0; off < seg_len; off += kWave) {
        const int i = base + off + lane;
        const bool in_seg = i < n && off + lane < seg_len;
        const int e_raw = in_seg ? expert_idx[i] : 0;
        const bool valid = in_seg && names_expert(e_raw, E);
        const int e = valid ? e_raw : 0;
        const uint64_t peers = same_expert_lanes(e, valid);
        const int rank = __popcll(peers & lanes_below(lane));
        const int32_t before = run[wave][e];
        __builtin_amdgcn_wave_barrier();
        if (valid && rank == 0) run[wave][e] = before + __popcll(peers);
        __builtin_amdgcn_wave_barrier();
        if (in_seg) {
            const int32_t pos = before + rank;
            const int32_t slot = valid && pos < capacity ? off_s[e] + pos : -1;
            slot_of[i] = slot;
            if (slot >= 0) src_of[slot] = i;
        }
    }
}

// Work list of one expert GEMM from the per-expert row ranges [lo_s[e], hi_s[e]) held in
// LDS (entries at or beyond E are empty).  An expert's rows are cut into row tiles of equal
// height (a multiple of 32, at most gp.bm), and its output tiles are listed panel by panel --
// `concurrent / row_tiles` column tiles wide, row tiles inside -- so that the blocks in
// flight on one XCD share both their weight and their activation tiles.  Called by every
// thread of the block; part `part` of `nparts` blocks emits its share of the entries.
__device__ void build_items(const GemmPlan &gp, WorkItem *__restrict__ items,
                            int32_t *__restrict__ nitems_out, const int32_t *lo_s,
                            const int32_t *hi_s, int32_t *mt_s, int32_t *cum_s, int part,
                            int nparts)
{
    if (threadIdx.x < kWave) {
        const int e = threadIdx.x;
        const int mt = ceil_div(hi_s[e] - lo_s[e], gp.bm);
        int incl = mt * gp.tiles_n;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int v = __shfl_up(incl, d);
            if (e >= d) incl += v;
        }
        mt_s[e] = mt;
        cum_s[e + 1] = incl;
        if (e == 0) cum_s[0] = 0;
    }
    __syncthreads();
    const int total = min(cum_s[kMaxExperts], gp.max_items);
    if (part == 0 && threadIdx.x == 0) *nitems_out = total;
    for (int L = part * blockDim.x + threadIdx.x; L < total; L += nparts * blockDim.x) {
        int e = 0;                                  // largest e with cum_s[e] <= L
#pragma unroll
        for (int step = kMaxExperts / 2; step > 0; step >>= 1)
            if (cum_s[e + step] <= L) e += step;
        const int l = L - cum_s[e];
        const int mt = mt_s[e];
        const int gn = min(gp.tiles_n, max(1, gp.concurrent / mt));
        const int panel = l / (mt * gn);
        const int within = l - panel * (mt * gn);
        const int width = min(gn, gp.tiles_n - panel * gn);
        const int m = within / width;
        const int nt = panel * gn + within % width;
        const int rows = hi_s[e] - lo_s[e];
        const int per_tile = min(gp.bm, ceil_div(ceil_div(rows, mt), 32) * 32);
        WorkItem it;
        it.expert = e;
        it.row0 = lo_s[e] + m * per_tile;
        it.row1 = min(hi_s[e], it.row0 + per_tile);
        it.n0 = nt * gp.bn;
        items[L] = it;
    }
    __syncthreads();
}

// Scan and rank in one launch, for plans of few segments: every block sums the raw
// per-segment counts itself (all of them for the totals, those before its first segment for
// its own base -- nseg * 256 bytes from L2 per block) instead of waiting for a scan kernel's
// launch.  The blocks beyond those that rank segments hold none: the last one writes counts
// and offsets, and for an unchunked layer they share the building of the work lists.
__global__ __launch_bounds__(kPlanThreads) void plan_rank_prefix_kernel(
    const int32_t *__restrict__ expert_idx, const int32_t *__restrict__ seg_cnt,
    int32_t *__restrict__ counts, int32_t *__restrict__ offsets, int32_t *__restrict__ slot_of,
    int32_t *__restrict__ src_of, int n, int E, int capacity, int seg_len, int nseg, int padded,
    int with_items, WorkItem *__restrict__ items0, int32_t *__restrict__ nitems0, GemmPlan gp0,
    WorkItem *__restrict__ items1, int32_t *__restrict__ nitems1, GemmPlan gp1,
    int spb, const uint4 *__restrict__ x, uint4 *__restrict__ xe, int vec, int k, int T)
{
    constexpr int kParts = kPlanWaves * 4;          // partial sums: 16-byte loads, 4 segments per wavefront load
    __shared__ int32_t part_before[kParts][kMaxExperts], part_total[kParts][kMaxExperts];
    __shared__ int32_t run[kPlanWaves][kMaxExperts];
    __shared__ int32_t slot_s[kSegTok * kMaxTopK];  // the segment's slots, for the packing below
    __shared__ int32_t off_s[kMaxExperts];
    __shared__ int32_t lo_s[kMaxExperts], hi_s[kMaxExperts], mt_s[kMaxExperts];
    __shared__ int32_t cum_s[kMaxExperts + 1];
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int first = min(static_cast<int>(blockIdx.x) * spb, nseg);
    {
        // lane = (segment of the load, four experts): part p = wave * 4 + lane / 16 walks the
        // segments p, p + 16, ...
        const int part = wave * 4 + lane / 16, e4 = (lane % 16) * 4;
        int4 before = make_int4(0, 0, 0, 0), total = before;
#pragma unroll 16
        for (int s = part; s < nseg; s += kParts) {
            const int4 c = *reinterpret_cast<const int4 *>(seg_cnt + static_cast<size_t>(s) * kMaxExperts + e4);
            total.x += c.x; total.y += c.y; total.z += c.z; total.w += c.w;
            if (s < first) { before.x += c.x; before.y += c.y; before.z += c.z; before.w += c.w; }
        }
        *reinterpret_cast<int4 *>(&part_before[part][e4]) = before;
        *reinterpret_cast<int4 *>(&part_total[part][e4]) = total;
    }
    __syncthreads();
    if (wave == 0) {
        int32_t before = 0, total = 0;
#pragma unroll
        for (int q = 0; q < kParts; ++q) {
            before += part_before[q][lane];
            total += part_total[q][lane];
        }
        const int32_t kept = lane < E ? min(total, capacity) : 0;
        int32_t incl = kept;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int v = __shfl_up(incl, d);
            if (lane >= d) incl += v;
        }
        off_s[lane] = lane >= E ? 0 : padded ? lane * capacity : incl - kept;
        lo_s[lane] = incl - kept;
        hi_s[lane] = incl;
        int32_t base = before;
#pragma unroll
        for (int q = 0; q < kPlanWaves; ++q) {
            run[q][lane] = base;
            if (q < spb && first + q < nseg)
                base += seg_cnt[static_cast<size_t>(first + q) * kMaxExperts + lane];
        }
        if (first == nseg && blockIdx.x == gridDim.x - 1) {   // one of the blocks without segments
            if (lane < E) {
                counts[lane] = total;
                offsets[lane] = incl - kept;
            }
            if (lane == E - 1) offsets[E] = incl;
        }
    }
    __syncthreads();
    if (first == nseg) {
        if (with_items) {
            // the kItemBlocks blocks without segments: even ones build the first GEMM's list,
            // odd ones the second's, each its share
            const int x = static_cast<int>(gridDim.x - 1 - blockIdx.x);
            if (x & 1)
                build_items(gp1, items1, nitems1, lo_s, hi_s, mt_s, cum_s, x >> 1, kItemBlocks / 2);
            else
                build_items(gp0, items0, nitems0, lo_s, hi_s, mt_s, cum_s, x >> 1, kItemBlocks / 2);
        }
        return;
    }
    const int seg = first + wave;
    const int base = seg * seg_len;
    const bool ranks = wave < spb && seg < nseg;
    if (!ranks && x == nullptr) return;
    if (ranks) {
        for (int off = 0; off < seg_len; off += kWave) {
            const int i = base + off + lane;
            const bool in_seg = i < n && off + lane < seg_len;
            const int e_raw = in_seg ? expert_idx[i] : 0;
            const bool valid = in_seg && names_expert(e_raw, E);
            const int e = valid ? e_raw : 0;
            const uint64_t peers = same_expert_lanes(e, valid);
            const int rank = __popcll(peers & lanes_below(lane));
            const int32_t before = run[wave][e];
            __builtin_amdgcn_wave_barrier();
            if (valid && rank == 0) run[wave][e] = before + __popcll(peers);
            __builtin_amdgcn_wave_barrier();
            int32_t slot = -1;
            if (in_seg) {
                const int32_t pos = before + rank;
                slot = valid && pos < capacity ? off_s[e] + pos : -1;
                slot_of[i] = slot;
                if (slot >= 0) src_of[slot] = i;
            }
            if (x != nullptr && off + lane < seg_len) slot_s[off + lane] = slot;
        }
    }
    if (x == nullptr) return;
    // Packing in the same launch (one segment per block: spb = 1): the block's wavefronts
    // copy the segment's token rows to their kept slots, two tokens per round.
    __syncthreads();
    const int seg_tok = seg_len / k;
    const int t_seg = first * seg_tok;
    for (int tt = wave; tt < seg_tok; tt += 2 * kPlanWaves) {
        const int ta = tt, tb = tt + kPlanWaves;
        const bool has_a = t_seg + ta < T, has_b = tb < seg_tok && t_seg + tb < T;
        int sa[kMaxTopK], sb[kMaxTopK];
        bool any_a = false, any_b = false;
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j) {
            sa[j] = has_a && j < k ? slot_s[ta * k + j] : -1;
            sb[j] = has_b && j < k ? slot_s[tb * k + j] : -1;
            any_a |= sa[j] >= 0;
            any_b |= sb[j] >= 0;
        }
        const uint4 *src_a = x + static_cast<size_t>(t_seg + ta) * vec;
        const uint4 *src_b = x + static_cast<size_t>(t_seg + tb) * vec;
        for (int c = lane; c < vec; c += kWave) {
            uint4 va = make_uint4(0, 0, 0, 0), vb = va;
            if (any_a) va = src_a[c];
            if (any_b) vb = src_b[c];
#pragma unroll
            for (int j = 0; j < kMaxTopK; ++j) {
                if (sa[j] >= 0) xe[static_cast<size_t>(sa[j]) * vec + c] = va;
                if (sb[j] >= 0) xe[static_cast<size_t>(sb[j]) * vec + c] = vb;
            }
        }
    }
}

// Work lists for FFN group f (blockIdx.x) and GEMM g (blockIdx.y).  Group f of n_groups is the
// run of chunks [f*n_chunks/n_groups, (f+1)*n_chunks/n_groups), i.e. the tokens [t0, t1) between
// those chunks' bounds.  Expert e's rows of the group are the slots whose source assignment
// lies in [t0*k, t1*k); src_of ascends inside an expert, so both ends are binary searches
// (lane e of the first wavefront owns expert e).
__global__ __launch_bounds__(256) void plan_items_kernel(
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ src_of,
    WorkItem *__restrict__ items0, int32_t *__restrict__ nitems0, GemmPlan gp0,
    WorkItem *__restrict__ items1, int32_t *__restrict__ nitems1, GemmPlan gp1, int T, int k,
    int E, int n_chunks, int n_groups)
{
    __shared__ int32_t lo_s[kMaxExperts], hi_s[kMaxExperts], mt_s[kMaxExperts];
    __shared__ int32_t cum_s[kMaxExperts + 1];
    const int c = blockIdx.x;
    const GemmPlan gp = blockIdx.y == 0 ? gp0 : gp1;
    WorkItem *items = (blockIdx.y == 0 ? items0 : items1) + static_cast<size_t>(c) * gp.max_items;
    int32_t *nitems = (blockIdx.y == 0 ? nitems0 : nitems1) + c;

    if (threadIdx.x < kWave) {
        const int e = threadIdx.x;
        const long c0 = static_cast<long>(c) * n_chunks / n_groups;
        const long c1 = static_cast<long>(c + 1) * n_chunks / n_groups;
        const long t0 = c0 * T / n_chunks;
        const long t1 = c1 * T / n_chunks;
        int lo = 0, hi = 0;
        if (e < E) {
            const int b = offsets[e], end = offsets[e + 1];
            if (n_groups == 1) {
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
        lo_s[e] = lo;
        hi_s[e] = hi;
    }
    __syncthreads();
    build_items(gp, items, nitems, lo_s, hi_s, mt_s, cum_s, blockIdx.z, gridDim.z);
}

// One work list per expert (list e holds expert e's output tiles only), for executing the
// experts one after the other: block (e, g) builds list e of GEMM g.
__global__ __launch_bounds__(256) void plan_items_expert_kernel(
    const int32_t *__restrict__ offsets, WorkItem *__restrict__ items0,
    int32_t *__restrict__ nitems0, GemmPlan gp0, WorkItem *__restrict__ items1,
    int32_t *__restrict__ nitems1, GemmPlan gp1, int E)
{
    __shared__ int32_t lo_s[kMaxExperts], hi_s[kMaxExperts], mt_s[kMaxExperts];
    __shared__ int32_t cum_s[kMaxExperts + 1];
    const int only = blockIdx.x;
    const GemmPlan gp = blockIdx.y == 0 ? gp0 : gp1;
    WorkItem *items = (blockIdx.y == 0 ? items0 : items1) + static_cast<size_t>(only) * gp.max_items;
    int32_t *nitems = (blockIdx.y == 0 ? nitems0 : nitems1) + only;
    if (threadIdx.x < kWave) {
        const int e = threadIdx.x;
        const bool mine = e == only && e < E;
        lo_s[e] = mine ? offsets[e] : 0;
        hi_s[e] = mine ? offsets[e + 1] : 0;
    }
    __syncthreads();
    build_items(gp, items, nitems, lo_s, hi_s, mt_s, cum_s, 0, 1);
}

// Work lists of the padded layout: micro-op m (blockIdx.x) covers, for every expert, the slot
// positions [m*C/n, (m+1)*C/n) of its C slots; only those below min(count, C) hold rows.
__global__ __launch_bounds__(256) void plan_items_padded_kernel(
    const int32_t *__restrict__ counts, WorkItem *__restrict__ items0,
    int32_t *__restrict__ nitems0, GemmPlan gp0, WorkItem *__restrict__ items1,
    int32_t *__restrict__ nitems1, GemmPlan gp1, int E, int capacity, int n_micro)
{
    __shared__ int32_t lo_s[kMaxExperts], hi_s[kMaxExperts], mt_s[kMaxExperts];
    __shared__ int32_t cum_s[kMaxExperts + 1];
    const int m = blockIdx.x;
    const GemmPlan gp = blockIdx.y == 0 ? gp0 : gp1;
    WorkItem *items = (blockIdx.y == 0 ? items0 : items1) + static_cast<size_t>(m) * gp.max_items;
    int32_t *nitems = (blockIdx.y == 0 ? nitems0 : nitems1) + m;
    if (threadIdx.x < kWave) {
        const int e = threadIdx.x;
        int lo = 0, hi = 0;
        if (e < E) {
            const int kept = min(counts[e], capacity);
            const int p0 = static_cast<int>(static_cast<long>(m) * capacity / n_micro);
            const int p1 = static_cast<int>(static_cast<long>(m + 1) * capacity / n_micro);
            lo = e * capacity + min(p0, kept);
            hi = e * capacity + min(p1, kept);
        }
        lo_s[e] = lo;
        hi_s[e] = hi;
    }
    __syncthreads();
    build_items(gp, items, nitems, lo_s, hi_s, mt_s, cum_s, blockIdx.z, gridDim.z);
}

}  // namespace

moe_status launch_items_padded(const moe_shape &s, int n_micro, const int32_t *counts,
                               const Workspace &w, hipStream_t st)
{
    hipLaunchKernelGGL(plan_items_padded_kernel, dim3(n_micro, 2, 4), dim3(256), 0, st, counts,
                       w.items[0], w.nitems[0], w.gp[0], w.items[1], w.nitems[1], w.gp[1], s.E,
                       s.capacity, n_micro);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status launch_items_per_expert(const moe_shape &s, const int32_t *offsets, const Workspace &w,
                                   hipStream_t st)
{
    hipLaunchKernelGGL(plan_items_expert_kernel, dim3(s.E, 2), dim3(256), 0, st, offsets, w.items[0],
                       w.nitems[0], w.gp[0], w.items[1], w.nitems[1], w.gp[1], s.E);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status launch_plan(const moe_shape &s, const int32_t *expert_idx, int32_t *counts,
                       int32_t *offsets, int32_t *slot_of, int32_t *src_of,
                       const Workspace &w, bool counted, int n_chunks, hipStream_t st, bool padded,
                       const void *x, void *xe, bool *packed)
{
    if (packed != nullptr) *packed = false;
    const int n = s.T * s.k;
    const int seg_len = w.seg_tok * s.k;
    int eps = 1;
    while (eps < s.E) eps <<= 1;
    const int blocks = ceil_div(w.nseg, kPlanWaves);
    if (!counted)
        hipLaunchKernelGGL(plan_count_kernel, dim3(blocks), dim3(kPlanThreads), 0, st,
                           expert_idx, w.seg_cnt, n, s.E, seg_len);
    if (w.nseg <= kPrefixSegments) {
        const bool with_items = n_chunks == 1 && !padded;
        // with the token rows at hand the same launch packs them: then one segment per block
        // (up to 64 MiB of token rows: beyond that the pack kernel's many more wavefronts in
        // flight are worth its launch -- measured at 134 MB: 89.9 us fused against 84.5)
        const int elem = s.dtype == MOE_BF16 ? 2 : 4;
        const bool pack = x != nullptr && xe != nullptr && packed != nullptr && !padded &&
                          static_cast<size_t>(s.T) * s.d_model * elem <= (64u << 20);
        const int spb = pack ? 1 : kPlanWaves;
        hipLaunchKernelGGL(plan_rank_prefix_kernel,
                           dim3(ceil_div(w.nseg, spb) + (with_items ? kItemBlocks : 1)),
                           dim3(kPlanThreads), 0, st,
                           expert_idx, w.seg_cnt, counts, offsets, slot_of, src_of, n, s.E,
                           s.capacity, seg_len, w.nseg, padded ? 1 : 0, with_items ? 1 : 0, w.items[0], w.nitems[0], w.gp[0],
                           w.items[1], w.nitems[1], w.gp[1], spb,
                           pack ? static_cast<const uint4 *>(x) : nullptr,
                           pack ? static_cast<uint4 *>(xe) : nullptr, s.d_model * elem / 16, s.k,
                           s.T);
        MOE_TRY_HIP(hipGetLastError());
        if (pack) *packed = true;
        return MOE_OK;
    }
    hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(1024), 0, st, w.seg_cnt, counts,
                       offsets, w.nseg, s.E, eps, s.capacity, n_chunks == 1 && !padded ? 1 : 0, w.items[0],
                       w.nitems[0], w.gp[0], w.items[1], w.nitems[1], w.gp[1]);
    hipLaunchKernelGGL(plan_rank_kernel, dim3(blocks), dim3(kPlanThreads), 0, st,
                       expert_idx, w.seg_cnt, offsets, slot_of, src_of, n, s.E, s.capacity,
                       seg_len, padded ? 1 : 0);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status launch_items(const moe_shape &s, int n_chunks, int n_groups, const int32_t *offsets,
                        const int32_t *src_of, const Workspace &w, hipStream_t st)
{
    hipLaunchKernelGGL(plan_items_kernel, dim3(n_groups, 2, 8), dim3(256), 0, st, offsets, src_of,
                       w.items[0], w.nitems[0], w.gp[0], w.items[1], w.nitems[1], w.gp[1], s.T,
                       s.k, s.E, n_chunks, n_groups);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // namespace moe
