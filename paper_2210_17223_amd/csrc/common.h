// Shared declarations of libmoe's translation units (host helpers, device
// conversions, kernel launch prototypes).  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "moe.h"

namespace moe {

constexpr int kWave = 64;          // wavefront width on CDNA
constexpr int kMaxExperts = 64;    // one ballot bit / one lane per expert
constexpr int kMaxTopK = 8;
constexpr int kSegTok = 64;        // most tokens per plan segment (= tokens per gate block)
constexpr int kMaxChunks = 64;

// ---- host side -------------------------------------------------------------
void set_error(const char *fmt, ...);
moe_status hip_fail(hipError_t e, const char *what);

#define MOE_TRY_HIP(expr)                                             \
    do {                                                              \
        hipError_t e_ = (expr);                                       \
        if (e_ != hipSuccess) return ::moe::hip_fail(e_, #expr);      \
    } while (0)

// Raises a kernel's dynamic-LDS limit once per kernel and per device.  Any host thread may be
// the first to launch a kernel: the flag word is atomic, and a thread that arrives while
// another is still setting the attribute waits for it instead of launching too early.
struct PerDeviceOnce {
    std::atomic<uint64_t> done{0};           // bit per device ordinal (up to 64 devices)
    std::mutex setting;
    void raise_lds(const void *kernel, int bytes)
    {
        int dev = 0;
        (void)hipGetDevice(&dev);
        const uint64_t bit = 1ull << (dev & 63);
        if (done.load(std::memory_order_acquire) & bit) return;
        std::lock_guard<std::mutex> lock(setting);
        if (done.load(std::memory_order_relaxed) & bit) return;
        (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        done.fetch_or(bit, std::memory_order_release);
    }
};

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// One output tile of a grouped GEMM: rows [row0, row1) of the expert-major buffer, all
// owned by `expert`, output columns [n0, n0 + tile width).
struct WorkItem {
    int32_t expert;
    int32_t row0;
    int32_t row1;
    int32_t n0;
};

// Tile shape and work-list bounds of one of the two expert GEMMs.
struct GemmPlan {
    int32_t bm, bn;          // rows / columns per output tile
    int32_t tiles_n;         // column tiles
    int32_t max_row_tiles;   // upper bound of row tiles per chunk
    int32_t max_items;       // upper bound of work items per chunk
    int32_t concurrent;      // work items in flight per XCD (sets the panel width)
};
GemmPlan choose_gemm_plan(const moe_shape &s, int which, int n_chunks);
void expert_gemm_kernel_name(const moe_shape &s, int which, int n_chunks, char *name, size_t len);

// Where each piece of the caller's workspace lives.
struct Workspace {
    int32_t *seg_cnt;      // [nseg][kMaxExperts] per-segment expert counts -> bases
    WorkItem *items[2];    // per GEMM: [n_chunks][gp.max_items]
    int32_t *nitems[2];    // per GEMM: [n_chunks]
    void *hidden;          // [max_rows][d_ff] hidden activations
    GemmPlan gp[2];
    int32_t nseg;
    int32_t seg_tok;       // tokens per segment (route_segment_tokens)
    size_t bytes;
};
bool layout_workspace(const moe_shape &s, int n_chunks, void *base, Workspace *w);

// Optional per-stage timing (moe_profile_enable): when a stage is enabled, its
// launches are bracketed by a pair of timing events on the stream they run on.
enum Stage { kStageRoute = 0, kStagePlan, kStageTiles, kStageScatter, kStageGemm1, kStageGemm2,
             kStageCombine,
             // backward pass: the five GEMMs (each one kernel), and everything else
             kStageBwdRecompute, kStageBwdDP, kStageBwdDxe, kStageBwdWgrad2, kStageBwdWgrad1,
             kStageBwdOther, kNumStages };
// Tokens per block of the gate kernel for this shape = tokens per segment of the plan.
int route_segment_tokens(const moe_shape &s);
void prof_begin(int stage, hipStream_t st);
void prof_end(int stage, hipStream_t st);
// For a stage that is one kernel: the pair of events to attach to that kernel's own
// dispatch (hipExtLaunchKernelGGL), which then carry the kernel's begin and end
// timestamps without the launch gaps around it.  Both null when the stage is not timed.
void prof_kernel_events(int stage, hipEvent_t *start, hipEvent_t *stop);

// ---- kernel launchers (each only enqueues on `st`) ---------------------------
// when seg_cnt is not NULL the per-segment expert histogram of the dispatch plan is
// produced in the same pass
moe_status launch_route(const moe_shape &s, const void *x, const void *Wg,
                        const float *bias, int bias_stride, int32_t *expert_idx,
                        float *gate, int32_t *seg_cnt, hipStream_t st);
// counted = the per-segment histogram is already in w.seg_cnt (launch_route made it);
// n_chunks == 1 also builds the GEMM work lists (otherwise launch_items does, after the ranks)
// padded: slot = e * capacity + rank (the equal-split layout) instead of offsets[e] + rank;
// offsets still receives the compact scan, and no work lists are built
// x, xe, packed: when all three are given and the plan is short enough for one launch, that
// launch also copies every token row to its kept slots (what launch_scatter does for all
// tokens) and sets *packed; otherwise *packed = false and the caller runs launch_scatter
moe_status launch_plan(const moe_shape &s, const int32_t *expert_idx, int32_t *counts,
                       int32_t *offsets, int32_t *slot_of, int32_t *src_of,
                       const Workspace &w, bool counted, int n_chunks, hipStream_t st,
                       bool padded = false, const void *x = nullptr, void *xe = nullptr,
                       bool *packed = nullptr);
// work lists of the padded layout, one per micro-op (slot positions [m*C/n, (m+1)*C/n))
moe_status launch_items_padded(const moe_shape &s, int n_micro, const int32_t *counts,
                               const Workspace &w, hipStream_t st);
// one pair of work lists per FFN group (a run of consecutive chunks, ffn_groups() of them)
moe_status launch_items(const moe_shape &s, int n_chunks, int n_groups, const int32_t *offsets,
                        const int32_t *src_of, const Workspace &w, hipStream_t st);
// How many expert-FFN launches a layer cut into n_chunks gets.  Every FFN launch streams the
// weights of all experts once, so a launch needs enough rows per expert to pay for that.
int ffn_groups(const moe_shape &s, int n_chunks);
// w.items[g] / w.nitems[g] sized for E lists: list e = the output tiles of expert e alone
moe_status launch_items_per_expert(const moe_shape &s, const int32_t *offsets, const Workspace &w,
                                   hipStream_t st);
moe_status launch_scatter(const moe_shape &s, const void *x, const int32_t *slot_of,
                          void *xe, int t0, int t1, hipStream_t st);
// rows: rows of ye (slots at or beyond it are never followed); < 0 = moe_max_rows
// ye: the expert outputs in their stored type (fp16 for bf16 layers, fp32 for fp32 layers)
moe_status launch_combine(const moe_shape &s, const void *ye, const int32_t *slot_of,
                          const float *gate, float *y, void *y_act, int t0, int t1,
                          hipStream_t st, int64_t rows = -1);
// pre: NULL, or fp16 [rows, d_ff] receiving the pre-activations of the first GEMM (bf16 layers)
// row_src: NULL, or the dispatch plan's src_of: `xe` is then the token matrix x itself and the
// first GEMM gathers slot i's row from token src_of[i] / k (bf16 layers)
moe_status launch_ffn(const moe_shape &s, const void *xe, const void *W1p,
                      const float *b1, const void *W2p, const float *b2, void *ye,
                      const Workspace &w, int chunk, hipStream_t st, void *pre = nullptr,
                      const int32_t *row_src = nullptr);
// bytes per element of the expert outputs ye
inline int ye_elem_bytes(const moe_shape &s) { return s.dtype == MOE_BF16 ? 2 : 4; }
moe_status launch_pack(const moe_shape &s, const void *W1, const void *W2, void *W1p,
                       void *W2p, hipStream_t st);

// ---- device helpers --------------------------------------------------------
#if defined(__HIPCC__)
__device__ __forceinline__ float bf16_to_f32(uint16_t b)
{
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// round to nearest, ties to even; finite inputs
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}
__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
#endif

}  // namespace moe
