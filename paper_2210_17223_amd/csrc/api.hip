// C-ABI entry points of libmoe: argument checks, workspace layout, and the order in
// which the kernels are enqueued.  No arithmetic of the layer happens here.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "common.h"
#include "moe_train.h"

namespace moe {

size_t packed_gate_bytes(const moe_shape &s);
moe_status launch_pack_gate(const moe_shape &s, const void *Wg, float *Wgp, hipStream_t st);

namespace {
thread_local char g_error[512] = "";
}

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

moe_status hip_fail(hipError_t e, const char *what)
{
    set_error("HIP error %d (%s) in %s", static_cast<int>(e), hipGetErrorString(e), what);
    return MOE_EHIP;
}

// ---- optional per-stage timing ------------------------------------------------
namespace {
struct Profiler {
    uint32_t mask = 0;
    int cap = 0;
    int n[kNumStages] = {};
    hipEvent_t *start[kNumStages] = {};
    hipEvent_t *stop[kNumStages] = {};
};
Profiler g_prof;

// Destroys every event and array of the profiler and switches it off (entries never created
// are null and skipped).
void prof_release()
{
    g_prof.mask = 0;
    for (int st = 0; st < kNumStages; ++st) {
        for (int i = 0; i < g_prof.cap; ++i) {
            if (g_prof.start[st] && g_prof.start[st][i]) (void)hipEventDestroy(g_prof.start[st][i]);
            if (g_prof.stop[st] && g_prof.stop[st][i]) (void)hipEventDestroy(g_prof.stop[st][i]);
        }
        delete[] g_prof.start[st];
        delete[] g_prof.stop[st];
        g_prof.start[st] = g_prof.stop[st] = nullptr;
        g_prof.n[st] = 0;
    }
    g_prof.cap = 0;
}
}  // namespace

void prof_begin(int stage, hipStream_t st)
{
    if (!((g_prof.mask >> stage) & 1u) || g_prof.n[stage] >= g_prof.cap) return;
    (void)hipEventRecord(g_prof.start[stage][g_prof.n[stage]], st);
}

void prof_end(int stage, hipStream_t st)
{
    if (!((g_prof.mask >> stage) & 1u) || g_prof.n[stage] >= g_prof.cap) return;
    (void)hipEventRecord(g_prof.stop[stage][g_prof.n[stage]], st);
    g_prof.n[stage] += 1;
}

void prof_kernel_events(int stage, hipEvent_t *start, hipEvent_t *stop)
{
    *start = *stop = nullptr;
    if (!((g_prof.mask >> stage) & 1u) || g_prof.n[stage] >= g_prof.cap) return;
    *start = g_prof.start[stage][g_prof.n[stage]];
    *stop = g_prof.stop[stage][g_prof.n[stage]];
    g_prof.n[stage] += 1;
}

namespace {

int elem_bytes(const moe_shape &s) { return s.dtype == MOE_BF16 ? 2 : 4; }

bool check_shape(const moe_shape *s)
{
    if (s == nullptr) {
        set_error("shape is NULL");
        return false;
    }
    if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) {
        set_error("dtype %d is neither MOE_F32 nor MOE_BF16", s->dtype);
        return false;
    }
    if (s->act < MOE_ACT_GELU_ERF || s->act > MOE_ACT_IDENTITY) {
        set_error("unknown activation %d", s->act);
        return false;
    }
    if (s->T < 1 || s->d_model < 1 || s->d_ff < 1 || s->E < 1 || s->k < 1 || s->capacity < 1) {
        set_error("T, d_model, d_ff, E, k, capacity must all be >= 1");
        return false;
    }
    if (s->k > s->E) {
        set_error("k = %d exceeds E = %d", s->k, s->E);
        return false;
    }
    if (static_cast<int64_t>(s->T) * s->k >= (1ll << 31)) {
        set_error("T*k = %lld does not fit 31 bits", static_cast<long long>(s->T) * s->k);
        return false;
    }
    if (static_cast<int64_t>(s->E) * s->capacity >= (1ll << 40)) {
        set_error("E*capacity = %lld is not below 2^40", static_cast<long long>(s->E) * s->capacity);
        return false;
    }
    return true;
}

// MOE_OK, or MOE_EUNSUPPORTED with the reason recorded.
moe_status check_supported(const moe_shape &s)
{
    if (s.E > kMaxExperts) {
        set_error("E = %d: at most %d experts are supported", s.E, kMaxExperts);
        return MOE_EUNSUPPORTED;
    }
    if (s.k > kMaxTopK) {
        set_error("k = %d: at most %d experts per token are supported", s.k, kMaxTopK);
        return MOE_EUNSUPPORTED;
    }
    const int eb = elem_bytes(s);
    if ((s.d_model * eb) % 16 != 0 || (s.d_ff * eb) % 16 != 0) {
        set_error("row sizes must be multiples of 16 bytes (d_model=%d, d_ff=%d, %d-byte elements)",
                  s.d_model, s.d_ff, eb);
        return MOE_EUNSUPPORTED;
    }
    return MOE_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define MOE_REQUIRE_PTR(p)                                          \
    do {                                                            \
        if ((p) == nullptr || !aligned16(p)) {                      \
            set_error(#p " is NULL or not 16-byte aligned");        \
            return MOE_EINVAL;                                      \
        }                                                           \
    } while (0)
#define MOE_OPTIONAL_PTR(p)                                         \
    do {                                                            \
        if ((p) != nullptr && !aligned16(p)) {                      \
            set_error(#p " is not 16-byte aligned");                \
            return MOE_EINVAL;                                      \
        }                                                           \
    } while (0)
#define MOE_TIMED(stage, stream, expr)        \
    do {                                     \
        prof_begin(stage, stream);           \
        moe_status st_ = (expr);             \
        prof_end(stage, stream);             \
        if (st_ != MOE_OK) return st_;       \
    } while (0)
#define MOE_TRY(expr)                        \
    do {                                     \
        moe_status st_ = (expr);             \
        if (st_ != MOE_OK) return st_;       \
    } while (0)

moe_status check_common(const moe_shape *s)
{
    if (!check_shape(s)) return MOE_EINVAL;
    return check_supported(*s);
}

moe_status check_bias(const moe_shape &s, const float *gate_bias, int32_t stride)
{
    if (gate_bias != nullptr && stride != 0 && stride != s.E) {
        set_error("bias_token_stride must be 0 or E (= %d), got %d", s.E, stride);
        return MOE_EINVAL;
    }
    return MOE_OK;
}

// Side streams and events of moe_layer_chunked, created on first use per device and
// kept until the process ends.
struct ChunkResources {
    bool ready = false;
    std::mutex enqueue;        // held while a call enqueues on the side streams
    hipStream_t pack = nullptr, unpack = nullptr;
    hipEvent_t planned = nullptr, unpacked = nullptr;
    hipEvent_t packed[kMaxChunks] = {};
    hipEvent_t computed[kMaxChunks] = {};
};
std::mutex g_res_mutex;
ChunkResources g_res[16];

moe_status chunk_resources(ChunkResources **out)
{
    int dev = 0;
    MOE_TRY_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16) {
        set_error("device index %d out of range", dev);
        return MOE_EUNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_res_mutex);
    ChunkResources &r = g_res[dev];
    if (!r.ready) {
        MOE_TRY_HIP(hipStreamCreateWithFlags(&r.pack, hipStreamNonBlocking));
        MOE_TRY_HIP(hipStreamCreateWithFlags(&r.unpack, hipStreamNonBlocking));
        MOE_TRY_HIP(hipEventCreateWithFlags(&r.planned, hipEventDisableTiming));
        MOE_TRY_HIP(hipEventCreateWithFlags(&r.unpacked, hipEventDisableTiming));
        for (int c = 0; c < kMaxChunks; ++c) {
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.packed[c], hipEventDisableTiming));
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.computed[c], hipEventDisableTiming));
        }
        r.ready = true;
    }
    *out = &r;
    return MOE_OK;
}

// ---- scratch of the entry point that allocates nothing ---------------------------
// moe_dispatch_static keeps the dispatch plan's per-segment expert counts here instead of in
// a caller's workspace.  In host code the array's NAME is only a stand-in for the symbol: the
// memory is reached through the address hipGetSymbolAddress returns, looked up once per
// device (every GPU holds its own copy of the array at its own address).
constexpr size_t kScratchBytes = size_t(4) << 20;
__device__ __align__(256) unsigned char scratch[kScratchBytes];
std::mutex g_scratch_mutex;
void *g_scratch_ptr[16] = {};

moe_status scratch_address(void **out)
{
    int dev = 0;
    MOE_TRY_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16) {
        set_error("device index %d out of range", dev);
        return MOE_EUNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        MOE_TRY_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr) {
            set_error("hipGetSymbolAddress returned a null address for the scratch array");
            return MOE_EHIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}

}  // namespace

// The expert FFN of a chunked layer runs once per GROUP of consecutive chunks.  A launch
// reads every expert's two weight matrices from HBM once whatever its row count, and is bound
// by the matrix cores only with several hundred rows per expert (2*rows flops per 2-byte
// weight against ~1 PFLOP/s over ~3.5 TB/s of HBM put the break-even near 300 rows; measured
// at 512 rows per expert and launch the two GEMMs still take 16 % longer than in one launch):
// groups are sized to hold at least 2048 rows per expert on average.  Packing and unpacking
// keep the caller's n_chunks.
std::atomic<int32_t> g_group_rows{2048};

int ffn_groups(const moe_shape &s, int n_chunks)
{
    const int64_t rows_per_expert = moe_max_rows(&s) / s.E;
    int64_t g = rows_per_expert / g_group_rows.load(std::memory_order_relaxed);
    if (g < 1) g = 1;
    return static_cast<int>(g < n_chunks ? g : n_chunks);
}

bool layout_workspace(const moe_shape &s, int n_chunks, void *base, Workspace *w)
{
    if (n_chunks < 1 || n_chunks > kMaxChunks) return false;
    const int64_t n = static_cast<int64_t>(s.T) * s.k;
    const int64_t max_rows = moe_max_rows(&s);
    (void)n;
    w->seg_tok = route_segment_tokens(s);
    w->nseg = (s.T + w->seg_tok - 1) / w->seg_tok;
    char *p = static_cast<char *>(base);
    size_t off = 0;
    w->seg_cnt = reinterpret_cast<int32_t *>(p + off);
    off += align_up(static_cast<size_t>(w->nseg) * kMaxExperts * sizeof(int32_t), 256);
    for (int g = 0; g < 2; ++g) {
        w->gp[g] = choose_gemm_plan(s, g, n_chunks);
        w->items[g] = reinterpret_cast<WorkItem *>(p + off);
        off += align_up(static_cast<size_t>(n_chunks) * w->gp[g].max_items * sizeof(WorkItem), 256);
        w->nitems[g] = reinterpret_cast<int32_t *>(p + off);
        off += align_up(static_cast<size_t>(n_chunks) * sizeof(int32_t), 256);
    }
    w->hidden = p + off;
    const size_t hidden_elem = s.dtype == MOE_BF16 ? 2 : 4;
    off += align_up(static_cast<size_t>(max_rows) * s.d_ff * hidden_elem, 256);
    w->bytes = off;
    return true;
}

}  // namespace moe

using namespace moe;

extern "C" {

int64_t moe_capacity(int32_t T, int32_t E, int32_t k, double cf)
{
    if (T < 1 || E < 1 || k < 1) return 0;
    if (!(cf > 0.0)) return T;
    // the product and the quotient in double, left to right, then the ceiling: a value that
    // comes out above an integer by any amount rounds up
    const double v = cf * static_cast<double>(k) * static_cast<double>(T) / static_cast<double>(E);
    const int64_t c = static_cast<int64_t>(std::ceil(v));
    return c < 1 ? 1 : c;
}

int64_t moe_max_rows(const moe_shape *s)
{
    if (s == nullptr) return 0;
    const int64_t a = static_cast<int64_t>(s->T) * s->k;
    const int64_t b = static_cast<int64_t>(s->E) * s->capacity;
    return a < b ? a : b;
}

size_t moe_workspace_bytes(const moe_shape *s, int32_t n_chunks)
{
    if (check_common(s) != MOE_OK) return 0;
    if (n_chunks < 1 || n_chunks > kMaxChunks) {
        set_error("n_chunks must be in 1..%d, got %d", kMaxChunks, n_chunks);
        return 0;
    }
    // the same buffer serves every call with up to n_chunks chunks (a chunked layer lays its
    // work lists out for its number of FFN groups, which is at most n_chunks)
    size_t bytes = 0;
    for (int c = 1; c <= n_chunks; ++c) {
        Workspace w;
        layout_workspace(*s, c, nullptr, &w);
        if (w.bytes > bytes) bytes = w.bytes;
    }
    return bytes;
}

const char *moe_last_error(void) { return g_error; }

moe_status moe_profile_enable(uint32_t stage_mask, int32_t max_samples)
{
    if (max_samples < 0 || stage_mask >= (1u << kNumStages)) {
        set_error("moe_profile_enable: bad stage mask or sample count");
        return MOE_EINVAL;
    }
    prof_release();
    if (stage_mask == 0 || max_samples == 0) return MOE_OK;
    g_prof.cap = max_samples;       // prof_release walks this many entries per enabled stage
    for (int st = 0; st < kNumStages; ++st) {
        if (!((stage_mask >> st) & 1u)) continue;
        g_prof.start[st] = new hipEvent_t[max_samples]();
        g_prof.stop[st] = new hipEvent_t[max_samples]();
        for (int i = 0; i < max_samples; ++i) {
            hipError_t e = hipEventCreate(&g_prof.start[st][i]);
            if (e == hipSuccess) e = hipEventCreate(&g_prof.stop[st][i]);
            if (e != hipSuccess) {      // give back what was created so far, stay switched off
                prof_release();
                return hip_fail(e, "hipEventCreate (moe_profile_enable)");
            }
        }
    }
    g_prof.mask = stage_mask;
    return MOE_OK;
}

int32_t moe_profile_read(int32_t stage, float *ms, int32_t cap)
{
    if (stage < 0 || stage >= kNumStages || ms == nullptr) return 0;
    const int n = g_prof.n[stage] < cap ? g_prof.n[stage] : cap;
    for (int i = 0; i < n; ++i) {
        ms[i] = -1.0f;
        if (hipEventSynchronize(g_prof.stop[stage][i]) != hipSuccess) continue;
        (void)hipEventElapsedTime(&ms[i], g_prof.start[stage][i], g_prof.stop[stage][i]);
    }
    g_prof.n[stage] = 0;
    return n;
}

size_t moe_packed_weight_bytes(const moe_shape *s)
{
    if (check_common(s) != MOE_OK) return 0;
    return static_cast<size_t>(s->E) * s->d_model * s->d_ff * elem_bytes(*s);
}

size_t moe_packed_gate_bytes(const moe_shape *s)
{
    if (check_common(s) != MOE_OK) return 0;
    return packed_gate_bytes(*s);
}

moe_status moe_pack_weights(const moe_shape *s, const void *W1, const void *W2, void *W1p,
                            void *W2p, void *stream)
{
    MOE_TRY(check_common(s));
    MOE_REQUIRE_PTR(W1);
    MOE_REQUIRE_PTR(W2);
    MOE_REQUIRE_PTR(W1p);
    MOE_REQUIRE_PTR(W2p);
    return launch_pack(*s, W1, W2, W1p, W2p, static_cast<hipStream_t>(stream));
}

moe_status moe_pack_gate(const moe_shape *s, const void *Wg, float *Wgp, void *stream)
{
    MOE_TRY(check_common(s));
    MOE_REQUIRE_PTR(Wg);
    MOE_REQUIRE_PTR(Wgp);
    return launch_pack_gate(*s, Wg, Wgp, static_cast<hipStream_t>(stream));
}

moe_status moe_route(const moe_shape *s, const void *x, const float *Wgp,
                     const float *gate_bias, int32_t bias_token_stride, int32_t *expert_idx,
                     float *gate, void *stream)
{
    MOE_TRY(check_common(s));
    MOE_REQUIRE_PTR(x);
    MOE_REQUIRE_PTR(Wgp);
    MOE_REQUIRE_PTR(expert_idx);
    MOE_REQUIRE_PTR(gate);
    MOE_TRY(check_bias(*s, gate_bias, bias_token_stride));
    hipStream_t st = static_cast<hipStream_t>(stream);
    MOE_TIMED(kStageRoute, st, launch_route(*s, x, Wgp, gate_bias, bias_token_stride, expert_idx,
                                            gate, nullptr, st));
    return MOE_OK;
}

moe_status moe_dispatch(const moe_shape *s, const void *x, const int32_t *expert_idx,
                        int32_t *counts, int32_t *offsets, int32_t *slot_of, int32_t *src_of,
                        void *xe, void *workspace, void *stream)
{
    MOE_TRY(check_common(s));
    MOE_REQUIRE_PTR(x);
    MOE_REQUIRE_PTR(expert_idx);
    MOE_REQUIRE_PTR(counts);
    MOE_REQUIRE_PTR(offsets);
    MOE_REQUIRE_PTR(slot_of);
    MOE_REQUIRE_PTR(src_of);
    MOE_REQUIRE_PTR(xe);
    MOE_REQUIRE_PTR(workspace);
    Workspace w;
    layout_workspace(*s, 1, workspace, &w);
    hipStream_t st = static_cast<hipStream_t>(stream);
    bool packed = false;
    MOE_TIMED(kStagePlan, st, launch_plan(*s, expert_idx, counts, offsets, slot_of, src_of, w,
                                          false, 0, st, false, x, xe, &packed));
    if (!packed) MOE_TIMED(kStageScatter, st, launch_scatter(*s, x, slot_of, xe, 0, s->T, st));
    return MOE_OK;
}

int32_t moe_tune_ffn_group_rows(int32_t rows)
{
    const int32_t before = g_group_rows.load(std::memory_order_relaxed);
    if (rows >= 1) g_group_rows.store(rows, std::memory_order_relaxed);
    return before;
}

size_t moe_dispatch_static_limit(void) { return kScratchBytes; }

moe_status moe_dispatch_static(const moe_shape *s, const void *x, const int32_t *expert_idx,
                               int32_t *counts, int32_t *offsets, int32_t *slot_of,
                               int32_t *src_of, void *xe, void *stream)
{
    MOE_TRY(check_common(s));
    MOE_REQUIRE_PTR(x);
    MOE_REQUIRE_PTR(expert_idx);
    MOE_REQUIRE_PTR(counts);
    MOE_REQUIRE_PTR(offsets);
    MOE_REQUIRE_PTR(slot_of);
    MOE_REQUIRE_PTR(src_of);
    MOE_REQUIRE_PTR(xe);
    Workspace w = {};
    w.seg_tok = route_segment_tokens(*s);
    w.nseg = (s->T + w.seg_tok - 1) / w.seg_tok;
    const size_t need = static_cast<size_t>(w.nseg) * kMaxExperts * sizeof(int32_t);
    if (need > kScratchBytes) {
        set_error("moe_dispatch_static: this shape's plan needs %zu bytes of scratch (%d segments "
                  "of %d tokens), the static array holds %zu; use moe_dispatch with a workspace",
                  need, w.nseg, w.seg_tok, kScratchBytes);
        return MOE_EUNSUPPORTED;
    }
    void *ptr = nullptr;
    MOE_TRY(scratch_address(&ptr));
    w.seg_cnt = static_cast<int32_t *>(ptr);
    hipStream_t st = static_cast<hipStream_t>(stream);
    bool packed = false;
    // n_chunks = 0: no work lists (they are the expert FFN's, which builds its own)
    MOE_TIMED(kStagePlan, st, launch_plan(*s, expert_idx, counts, offsets, slot_of, src_of, w,
                                          false, 0, st, false, x, xe, &packed));
    if (!packed) MOE_TIMED(kStageScatter, st, launch_scatter(*s, x, slot_of, xe, 0, s->T, st));
    return MOE_OK;
}

moe_status moe_expert_ffn(const moe_shape *s, const void *xe, const int32_t *offsets,
                          const void *W1p, const float *b1, const void *W2p, const float *b2,
                          void *ye, void *workspace, void *stream)
{
    MOE_TRY(check_common(s));
    MOE_REQUIRE_PTR(xe);
    MOE_REQUIRE_PTR(offsets);
    MOE_REQUIRE_PTR(W1p);
    MOE_REQUIRE_PTR(W2p);
    MOE_OPTIONAL_PTR(b1);
    MOE_OPTIONAL_PTR(b2);
    MOE_REQUIRE_PTR(ye);
    MOE_REQUIRE_PTR(workspace);
    Workspace w;
    layout_workspace(*s, 1, workspace, &w);
    hipStream_t st = static_cast<hipStream_t>(stream);
    MOE_TIMED(kStageTiles, st, launch_items(*s, 1, 1, offsets, nullptr, w, st));
    return launch_ffn(*s, xe, W1p, b1, W2p, b2, ye, w, 0, st);
}

moe_status moe_combine(const moe_shape *s, const void *ye, const int32_t *slot_of,
                       const float *gate, float *y, void *y_act, void *stream)
{
    MOE_TRY(check_common(s));
    MOE_REQUIRE_PTR(ye);
    MOE_REQUIRE_PTR(slot_of);
    MOE_REQUIRE_PTR(gate);
    MOE_REQUIRE_PTR(y);
    MOE_OPTIONAL_PTR(y_act);
    hipStream_t st = static_cast<hipStream_t>(stream);
    MOE_TIMED(kStageCombine, st, launch_combine(*s, ye, slot_of, gate, y, y_act, 0, s->T, st));
    return MOE_OK;
}

}  // extern "C"

namespace {

// The layer call; pre != NULL (one chunk only) keeps the first GEMM's pre-activations.
moe_status layer_forward(const moe_shape *s, int32_t n_chunks, const void *x,
                         const float *Wgp, const float *gate_bias,
                         int32_t bias_token_stride, const void *W1p, const float *b1,
                         const void *W2p, const float *b2, int32_t *expert_idx, float *gate,
                         int32_t *counts, int32_t *offsets, int32_t *slot_of,
                         int32_t *src_of, void *xe, void *ye, void *pre, void *hid, float *y,
                         void *y_act, void *workspace, void *stream)
{
    MOE_TRY(check_common(s));
    if (n_chunks < 1 || n_chunks > kMaxChunks) {
        set_error("n_chunks must be in 1..%d, got %d", kMaxChunks, n_chunks);
        return MOE_EINVAL;
    }
    MOE_REQUIRE_PTR(x);
    MOE_REQUIRE_PTR(Wgp);
    MOE_REQUIRE_PTR(W1p);
    MOE_REQUIRE_PTR(W2p);
    MOE_OPTIONAL_PTR(b1);
    MOE_OPTIONAL_PTR(b2);
    MOE_REQUIRE_PTR(expert_idx);
    MOE_REQUIRE_PTR(gate);
    MOE_REQUIRE_PTR(counts);
    MOE_REQUIRE_PTR(offsets);
    MOE_REQUIRE_PTR(slot_of);
    MOE_REQUIRE_PTR(src_of);
    MOE_REQUIRE_PTR(xe);
    MOE_REQUIRE_PTR(ye);
    MOE_REQUIRE_PTR(y);
    MOE_OPTIONAL_PTR(y_act);
    MOE_REQUIRE_PTR(workspace);
    MOE_TRY(check_bias(*s, gate_bias, bias_token_stride));
    if (n_chunks > s->T) n_chunks = s->T;
    // FFN launches: one per group of consecutive chunks; a layer whose FFN would run as one
    // group anyway is run unchunked (same outputs, one launch less per chunk)
    const int n_groups = ffn_groups(*s, n_chunks);
    if (n_groups == 1) n_chunks = 1;

    Workspace w;
    layout_workspace(*s, n_groups, workspace, &w);
    if (hid != nullptr) w.hidden = hid;       // the hidden activations go where the caller keeps them
    hipStream_t st = static_cast<hipStream_t>(stream);

    MOE_TIMED(kStageRoute, st,
              launch_route(*s, x, Wgp, gate_bias, bias_token_stride, expert_idx, gate,
                           w.seg_cnt, st));
    bool packed = false;       // an unchunked layer's plan launch packs the token rows as well
    MOE_TIMED(kStagePlan, st,
              launch_plan(*s, expert_idx, counts, offsets, slot_of, src_of, w, true, n_chunks, st,
                          false, n_chunks == 1 ? x : nullptr, xe, &packed));
    if (n_chunks > 1)
        MOE_TIMED(kStageTiles, st, launch_items(*s, n_chunks, n_groups, offsets, src_of, w, st));

    // bf16 layers: the first expert GEMM gathers its rows from the token matrix through
    // src_of, so it does not wait for the pack; xe (the first all-to-all's payload) is then
    // written beside it on a side stream.  fp32 layers multiply the packed buffer.
    const bool gather = s->dtype == MOE_BF16;
    const void *ffn_in = gather ? x : xe;
    const int32_t *row_src = gather ? src_of : nullptr;

    if (n_chunks == 1 && (packed || !gather)) {
        if (!packed)
            MOE_TIMED(kStageScatter, st, launch_scatter(*s, x, slot_of, xe, 0, s->T, st));
        MOE_TRY(launch_ffn(*s, ffn_in, W1p, b1, W2p, b2, ye, w, 0, st, pre, row_src));
        MOE_TIMED(kStageCombine, st,
                  launch_combine(*s, ye, slot_of, gate, y, y_act, 0, s->T, st));
        return MOE_OK;
    }

    // pack stream: chunk after chunk; caller's stream: expert FFN of a group of chunks (fp32
    // layers: once the group is packed); unpack stream: combine of a chunk once its group's FFN
    // is done.  An unchunked bf16 layer takes this path with one chunk and one group: its pack
    // runs beside the FFN.
    ChunkResources *r = nullptr;
    MOE_TRY(chunk_resources(&r));
    // One call at a time enqueues on this device's side streams: two threads' records and
    // waits on the shared events must not interleave.
    std::lock_guard<std::mutex> enqueue(r->enqueue);
    MOE_TRY_HIP(hipEventRecord(r->planned, st));
    MOE_TRY_HIP(hipStreamWaitEvent(r->pack, r->planned, 0));
    if (n_chunks > 1) MOE_TRY_HIP(hipStreamWaitEvent(r->unpack, r->planned, 0));
    auto bound = [&](int c) { return static_cast<int>(static_cast<int64_t>(c) * s->T / n_chunks); };
    auto enqueue_chunks = [&]() -> moe_status {
        for (int c = 0; c < n_chunks; ++c) {
            MOE_TIMED(kStageScatter, r->pack,
                      launch_scatter(*s, x, slot_of, xe, bound(c), bound(c + 1), r->pack));
            if (!gather) MOE_TRY_HIP(hipEventRecord(r->packed[c], r->pack));
        }
        for (int f = 0; f < n_groups; ++f) {
            // group f = chunks [c0, c1)
            const int c0 = static_cast<int>(static_cast<int64_t>(f) * n_chunks / n_groups);
            const int c1 = static_cast<int>(static_cast<int64_t>(f + 1) * n_chunks / n_groups);
            if (!gather) MOE_TRY_HIP(hipStreamWaitEvent(st, r->packed[c1 - 1], 0));
            MOE_TRY(launch_ffn(*s, ffn_in, W1p, b1, W2p, b2, ye, w, f, st, pre, row_src));
            if (n_chunks == 1) {
                MOE_TIMED(kStageCombine, st,
                          launch_combine(*s, ye, slot_of, gate, y, y_act, 0, s->T, st));
                continue;
            }
            MOE_TRY_HIP(hipEventRecord(r->computed[f], st));
            MOE_TRY_HIP(hipStreamWaitEvent(r->unpack, r->computed[f], 0));
            for (int c = c0; c < c1; ++c)
                MOE_TIMED(kStageCombine, r->unpack,
                          launch_combine(*s, ye, slot_of, gate, y, y_act, bound(c), bound(c + 1),
                                         r->unpack));
        }
        return MOE_OK;
    };
    const moe_status rc = enqueue_chunks();
    // Join the side streams back into the caller's stream, also after a failure part-way:
    // whatever was enqueued there must not outlive the call unobserved.
    hipError_t je = hipEventRecord(r->packed[0], r->pack);
    if (je == hipSuccess) je = hipStreamWaitEvent(st, r->packed[0], 0);
    if (je == hipSuccess && n_chunks > 1) je = hipEventRecord(r->unpacked, r->unpack);
    if (je == hipSuccess && n_chunks > 1) je = hipStreamWaitEvent(st, r->unpacked, 0);
    if (rc != MOE_OK) return rc;
    if (je != hipSuccess) return hip_fail(je, "joining the side streams");
    return MOE_OK;
}

}  // namespace

extern "C" {

moe_status moe_layer_chunked(const moe_shape *s, int32_t n_chunks, const void *x,
                             const float *Wgp, const float *gate_bias,
                             int32_t bias_token_stride, const void *W1p, const float *b1,
                             const void *W2p, const float *b2, int32_t *expert_idx, float *gate,
                             int32_t *counts, int32_t *offsets, int32_t *slot_of,
                             int32_t *src_of, void *xe, void *ye, float *y, void *y_act,
                             void *workspace, void *stream)
{
    return layer_forward(s, n_chunks, x, Wgp, gate_bias, bias_token_stride, W1p, b1, W2p, b2,
                         expert_idx, gate, counts, offsets, slot_of, src_of, xe, ye, nullptr,
                         nullptr, y, y_act, workspace, stream);
}

moe_status moe_layer_forward_keep(const moe_shape *s, const void *x, const float *Wgp,
                                  const float *gate_bias, int32_t bias_token_stride,
                                  const void *W1p, const float *b1, const void *W2p,
                                  const float *b2, int32_t *expert_idx, float *gate,
                                  int32_t *counts, int32_t *offsets, int32_t *slot_of,
                                  int32_t *src_of, void *xe, void *ye, void *pre, void *hid,
                                  float *y, void *workspace, void *stream)
{
    MOE_TRY(check_common(s));
    if (s->dtype != MOE_BF16) {
        set_error("moe_layer_forward_keep: bf16 layers only");
        return MOE_EUNSUPPORTED;
    }
    MOE_REQUIRE_PTR(pre);
    MOE_REQUIRE_PTR(hid);
    return layer_forward(s, 1, x, Wgp, gate_bias, bias_token_stride, W1p, b1, W2p, b2, expert_idx,
                         gate, counts, offsets, slot_of, src_of, xe, ye, pre, hid, y, nullptr,
                         workspace, stream);
}

}  // extern "C"
