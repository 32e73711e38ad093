// Popularity-based expert scheduling for inference (paper Sec. 5.2): sample-path tables,
// the per-batch popularity estimate in exact fixed-point arithmetic, Eq. (1),
// first-fit-decreasing packing and the two-phase check.  The table and estimate steps
// are integer kernels over tokens (HBM / atomic bound, a few bytes per token); the
// scheduling decisions are tiny and run on the host thread that owns the scheduler.
#include "common.h"
#include "moe_sched.h"

#include <algorithm>
#include <vector>

namespace moe {
namespace {

constexpr int kFix = 32;           // probabilities are floor(p * 2^32)
constexpr int64_t kMaxPaths = 1ll << 24;

int64_t path_count(const moe_path_shape *s)
{
    if (s == nullptr || s->E < 1 || s->E > kMaxExperts || s->l < 1 || s->k < 1 ||
        s->k > kMaxTopK || s->k > s->E)
        return 0;
    int64_t p = 1;
    for (int m = 0; m < s->l; ++m) {
        p *= s->E;
        if (p > kMaxPaths) return 0;
    }
    return p;
}

// Sample path of token t whose oldest layer starts at `hist` (layer stride = T*k entries):
// the l first choices as an l-digit number in base E, or -1 if one is not an expert.
__device__ __forceinline__ int path_of(const int32_t *__restrict__ hist, size_t layer_stride,
                                       int t, int k, int l, int E)
{
    int j = 0;
    for (int m = 0; m < l; ++m) {
        const int e = hist[m * layer_stride + static_cast<size_t>(t) * k];
        if (static_cast<unsigned>(e) >= static_cast<unsigned>(E)) return -1;
        j = j * E + e;
    }
    return j;
}

// One thread per (table a, token t): table a predicts layer a + l from layers a .. a+l-1.
__global__ __launch_bounds__(256) void path_profile_kernel(
    const int32_t *__restrict__ sel, uint32_t *__restrict__ counts, int T, int tables, int E,
    int k, int l, int paths)
{
    const long idx = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= static_cast<long>(tables) * T) return;
    const int a = static_cast<int>(idx / T), t = static_cast<int>(idx % T);
    const size_t layer_stride = static_cast<size_t>(T) * k;
    const int j = path_of(sel + a * layer_stride, layer_stride, t, k, l, E);
    if (j < 0) return;
    const int32_t *next = sel + (a + l) * layer_stride + static_cast<size_t>(t) * k;
    for (int c = 0; c < k; ++c)
        if (static_cast<unsigned>(next[c]) >= static_cast<unsigned>(E)) return;
    uint32_t *row = counts + (static_cast<size_t>(a) * paths + j) * E;
    for (int c = 0; c < k; ++c) atomicAdd(&row[next[c]], 1u);
}

// One thread per (table, path) row: row total, then k rounds of "largest remaining count,
// lowest index first".
__global__ __launch_bounds__(256) void path_finalize_kernel(
    const uint32_t *__restrict__ counts, int32_t *__restrict__ top_expert,
    unsigned long long *__restrict__ top_prob, long rows, int E, int k)
{
    const long r = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    const uint32_t *row = counts + r * E;
    unsigned long long tot = 0;
    for (int e = 0; e < E; ++e) tot += row[e];
    unsigned long long taken = 0;
    for (int c = 0; c < k; ++c) {
        int best = -1;
        uint32_t bc = 0;
        for (int e = 0; e < E; ++e) {
            if ((taken >> e) & 1ull) continue;
            if (row[e] > bc) { best = e; bc = row[e]; }      // count 0 never wins
        }
        unsigned long long q = 0;
        if (best >= 0) {
            taken |= 1ull << best;
            q = (static_cast<unsigned long long>(bc) << kFix) / tot;
        }
        top_expert[r * k + c] = best;
        top_prob[r * k + c] = q;
    }
}

__global__ void zero_u64_kernel(unsigned long long *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

// A block walks its share of the tokens, sums their contributions in LDS and adds them to
// S with one 64-bit atomic per expert (few blocks: the atomics of all blocks hit the same E
// addresses).  Integer sums: the result does not depend on the order.
__global__ __launch_bounds__(256) void popularity_estimate_kernel(
    const int32_t *__restrict__ hist, const int32_t *__restrict__ top_expert,
    const unsigned long long *__restrict__ top_prob, unsigned long long *__restrict__ S,
    int N_t, int E, int k, int l)
{
    __shared__ unsigned long long acc[kMaxExperts];
    if (threadIdx.x < kMaxExperts) acc[threadIdx.x] = 0ull;
    __syncthreads();
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < N_t; t += gridDim.x * blockDim.x) {
        const int j = path_of(hist, static_cast<size_t>(N_t) * k, t, k, l, E);
        if (j < 0) continue;
        for (int c = 0; c < k; ++c) {
            const int e = top_expert[static_cast<size_t>(j) * k + c];
            if (e >= 0) atomicAdd(&acc[e], top_prob[static_cast<size_t>(j) * k + c]);
        }
    }
    __syncthreads();
    if (static_cast<int>(threadIdx.x) < E && acc[threadIdx.x] != 0ull) atomicAdd(&S[threadIdx.x], acc[threadIdx.x]);
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

struct Schedule {
    std::vector<int32_t> replicas;
    std::vector<std::vector<int32_t>> hosted;
    int32_t used = 0;
};

// The packing of moe_schedule_experts on host vectors.
Schedule schedule_experts(int N, int E, const uint64_t *w, uint64_t W, const uint8_t *has,
                          int max_pack)
{
    Schedule out;
    out.replicas.assign(E, 0);
    out.hosted.assign(N, {});
    std::vector<std::vector<int32_t>> groups;     // experts of each asked-for device
    std::vector<int32_t> small;
    for (int e = 0; e < E; ++e) {
        if (!has[e]) continue;
        if (w[e] >= W) {
            // round half up of w / W, without forming 2w + W (which could overflow)
            const uint64_t q = w[e] / W, rem = w[e] % W;
            const uint64_t r = q + (rem >= W - rem ? 1 : 0);
            out.replicas[e] = static_cast<int32_t>(std::min<uint64_t>(r, N));   // never more than all devices
            for (int32_t i = 0; i < out.replicas[e]; ++i) groups.push_back({e});
        } else {
            small.push_back(e);
        }
    }
    std::stable_sort(small.begin(), small.end(),
                     [&](int32_t a, int32_t b) { return w[a] > w[b]; });   // index order kept on ties
    std::vector<std::vector<int32_t>> bins;
    std::vector<uint64_t> load;
    for (int32_t e : small) {
        size_t b = 0;
        for (; b < bins.size(); ++b)
            if (load[b] + w[e] <= W && static_cast<int>(bins[b].size()) < max_pack) break;
        if (b == bins.size()) {
            bins.push_back({});
            load.push_back(0);
        }
        bins[b].push_back(e);
        load[b] += w[e];
        out.replicas[e] = 1;
    }
    for (auto &b : bins) groups.push_back(b);
    const int64_t used = static_cast<int64_t>(groups.size());
    for (int64_t g = 0; g < used; ++g) {
        auto &dev = out.hosted[g % N];
        for (int32_t e : groups[g])
            if (std::find(dev.begin(), dev.end(), e) == dev.end()) dev.push_back(e);
    }
    const int64_t free_devs = N - used;
    int64_t m = 0;
    for (int e = 0; e < E; ++e) {
        if (has[e]) continue;
        const int64_t d = free_devs > 0 ? used + (m % free_devs) : e % N;
        out.hosted[d].push_back(e);
        out.replicas[e] = 1;
        ++m;
    }
    out.used = static_cast<int32_t>(std::min<int64_t>(used, N));
    return out;
}

moe_status check_schedule_args(int32_t N, int32_t E, const void *w_or_S, int32_t max_pack,
                               const int32_t *replicas, const int32_t *dev_count,
                               const int32_t *dev_experts, const int32_t *devices_used)
{
    if (N < 1 || E < 1 || E > kMaxExperts || max_pack < 1) {
        set_error("schedule: need N >= 1, 1 <= E <= %d, max_pack >= 1 (N=%d E=%d max_pack=%d)",
                  kMaxExperts, N, E, max_pack);
        return MOE_EINVAL;
    }
    if (w_or_S == nullptr || replicas == nullptr || dev_count == nullptr ||
        dev_experts == nullptr || devices_used == nullptr) {
        set_error("schedule: NULL argument");
        return MOE_EINVAL;
    }
    return MOE_OK;
}

void write_schedule(const Schedule &sc, int N, int E, int32_t *replicas, int32_t *dev_count,
                    int32_t *dev_experts, int32_t *devices_used)
{
    for (int e = 0; e < E; ++e) replicas[e] = sc.replicas[e];
    for (int d = 0; d < N; ++d) {
        // wrapping can put more than E entries' worth of groups on a device, never more
        // than E distinct experts
        dev_count[d] = static_cast<int32_t>(sc.hosted[d].size());
        for (int i = 0; i < E; ++i)
            dev_experts[static_cast<size_t>(d) * E + i] =
                i < dev_count[d] ? sc.hosted[d][i] : -1;
    }
    *devices_used = sc.used;
}

// The 2k (at most E) most popular experts, most popular first, ties to the lower index.
template <typename V>
std::vector<int32_t> top_list(int E, int m, const V *score)
{
    std::vector<int32_t> order(E);
    for (int e = 0; e < E; ++e) order[e] = e;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return score[a] > score[b]; });
    order.resize(m);
    return order;
}

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

int64_t moe_path_count(const moe_path_shape *s) { return path_count(s); }

moe_status moe_path_profile(const moe_path_shape *s, const int32_t *sel, int32_t T,
                            uint32_t *counts, void *stream)
{
    const int64_t paths = path_count(s);
    if (paths == 0 || s->L <= s->l) {
        set_error("path shape: need 1 <= E <= %d, 1 <= k <= min(E, %d), l >= 1, E^l <= 2^24, L > l",
                  kMaxExperts, kMaxTopK);
        return MOE_EINVAL;
    }
    if (T < 0 || sel == nullptr || counts == nullptr || !aligned(sel, 4) || !aligned(counts, 4)) {
        set_error("moe_path_profile: T < 0, or sel / counts NULL or misaligned");
        return MOE_EINVAL;
    }
    const int tables = s->L - s->l;
    const long n = static_cast<long>(tables) * T;
    if (n == 0) return MOE_OK;
    if (n > (1l << 40)) {
        set_error("moe_path_profile: %ld (table, token) pairs in one call", n);
        return MOE_EUNSUPPORTED;
    }
    hipLaunchKernelGGL(path_profile_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256),
                       0, static_cast<hipStream_t>(stream), sel, counts, T, tables, s->E, s->k,
                       s->l, static_cast<int>(paths));
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status moe_path_finalize(const moe_path_shape *s, const uint32_t *counts,
                             int32_t *top_expert, uint64_t *top_prob, void *stream)
{
    const int64_t paths = path_count(s);
    if (paths == 0 || s->L <= s->l) {
        set_error("path shape: need 1 <= E <= %d, 1 <= k <= min(E, %d), l >= 1, E^l <= 2^24, L > l",
                  kMaxExperts, kMaxTopK);
        return MOE_EINVAL;
    }
    if (counts == nullptr || top_expert == nullptr || top_prob == nullptr || !aligned(counts, 4) ||
        !aligned(top_expert, 4) || !aligned(top_prob, 8)) {
        set_error("moe_path_finalize: NULL or misaligned argument");
        return MOE_EINVAL;
    }
    const long rows = static_cast<long>(s->L - s->l) * paths;
    hipLaunchKernelGGL(path_finalize_kernel, dim3(static_cast<unsigned>((rows + 255) / 256)),
                       dim3(256), 0, static_cast<hipStream_t>(stream), counts, top_expert,
                       reinterpret_cast<unsigned long long *>(top_prob), rows, s->E, s->k);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

moe_status moe_popularity_estimate(const moe_path_shape *s, const int32_t *sel_hist,
                                   int32_t N_t, const int32_t *top_expert,
                                   const uint64_t *top_prob, uint64_t *S, void *stream)
{
    if (path_count(s) == 0) {
        set_error("path shape: need 1 <= E <= %d, 1 <= k <= min(E, %d), l >= 1, E^l <= 2^24",
                  kMaxExperts, kMaxTopK);
        return MOE_EINVAL;
    }
    if (N_t < 0 || sel_hist == nullptr || top_expert == nullptr || top_prob == nullptr ||
        S == nullptr || !aligned(sel_hist, 4) || !aligned(top_expert, 4) ||
        !aligned(top_prob, 8) || !aligned(S, 8)) {
        set_error("moe_popularity_estimate: N_t < 0, or a NULL or misaligned argument");
        return MOE_EINVAL;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned long long *Sd = reinterpret_cast<unsigned long long *>(S);
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(kMaxExperts), 0, st, Sd, s->E);
    if (N_t > 0)
        hipLaunchKernelGGL(popularity_estimate_kernel,
                           dim3(std::min(256, (N_t + 1023) / 1024)), dim3(256), 0, st,
                           sel_hist, top_expert,
                           reinterpret_cast<const unsigned long long *>(top_prob), Sd, N_t, s->E,
                           s->k, s->l);
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

double moe_devices_for_expert(uint64_t S_e, int32_t N_t, int32_t N)
{
    if (N_t < 1) return 0.0;
    return static_cast<double>(N) * (static_cast<double>(S_e) / 4294967296.0) /
           static_cast<double>(N_t);
}

moe_status moe_schedule_experts(int32_t N, int32_t E, const uint64_t *w, uint64_t W,
                                const uint8_t *has, int32_t max_pack, int32_t *replicas,
                                int32_t *dev_count, int32_t *dev_experts, int32_t *devices_used)
{
    const moe_status st =
        check_schedule_args(N, E, w, max_pack, replicas, dev_count, dev_experts, devices_used);
    if (st != MOE_OK) return st;
    if (has == nullptr || W < 1) {
        set_error("moe_schedule_experts: has is NULL or W < 1");
        return MOE_EINVAL;
    }
    const Schedule sc = schedule_experts(N, E, w, W, has, max_pack);
    write_schedule(sc, N, E, replicas, dev_count, dev_experts, devices_used);
    return MOE_OK;
}

int32_t moe_top_lists_identical(int32_t E, int32_t k, const uint64_t *S, const int32_t *counts)
{
    if (E < 1 || E > kMaxExperts || k < 1 || S == nullptr || counts == nullptr) return 0;
    const int m = std::min(2 * k, E);
    return top_list(E, m, S) == top_list(E, m, counts) ? 1 : 0;
}

moe_status moe_schedule_layer(int32_t N, int32_t E, int32_t k, int32_t N_t, const uint64_t *S,
                              const int32_t *counts, int32_t max_pack, int32_t *replicas,
                              int32_t *dev_count, int32_t *dev_experts, int32_t *devices_used,
                              int32_t *rescheduled)
{
    const moe_status st =
        check_schedule_args(N, E, S, max_pack, replicas, dev_count, dev_experts, devices_used);
    if (st != MOE_OK) return st;
    if (counts == nullptr || rescheduled == nullptr || k < 1 || N_t < 1) {
        set_error("moe_schedule_layer: counts / rescheduled NULL, or k < 1, or N_t < 1");
        return MOE_EINVAL;
    }
    // N * S[e] <= N * N_t * 2^32 must fit 64 bits
    if (static_cast<uint64_t>(N) * static_cast<uint64_t>(N_t) >= (1ull << 31)) {
        set_error("moe_schedule_layer: N * N_t = %llu does not fit the fixed-point weights",
                  static_cast<unsigned long long>(N) * static_cast<unsigned long long>(N_t));
        return MOE_EUNSUPPORTED;
    }
    uint64_t w[kMaxExperts];
    uint8_t has[kMaxExperts];
    *rescheduled = 0;
    if (moe_top_lists_identical(E, k, S, counts)) {
        for (int e = 0; e < E; ++e) {
            w[e] = static_cast<uint64_t>(N) * S[e];
            has[e] = S[e] > 0;
        }
        write_schedule(schedule_experts(N, E, w, static_cast<uint64_t>(N_t) << kFix, has, max_pack),
                       N, E, replicas, dev_count, dev_experts, devices_used);
    } else {
        for (int e = 0; e < E; ++e) {
            w[e] = static_cast<uint64_t>(N) * static_cast<uint64_t>(counts[e] < 0 ? 0 : counts[e]);
            has[e] = counts[e] > 0;
        }
        write_schedule(schedule_experts(N, E, w, static_cast<uint64_t>(N_t) * k, has, max_pack),
                       N, E, replicas, dev_count, dev_experts, devices_used);
        *rescheduled = 1;
    }
    return MOE_OK;
}

}  // extern "C"
