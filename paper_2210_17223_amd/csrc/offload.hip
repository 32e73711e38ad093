// Expert FFN with host-resident expert weights (paper Sec. 4.2 "Expert packing":
// DRAM-offloading; Sec. 6.2: packed experts are loaded and computed one at a time).
// Expert e's packed weights travel host -> staging slot e % resident on a copy stream
// while earlier experts are computed; the two GEMMs of expert e then run on the caller's
// stream from a work list that holds expert e's tiles only.  Bound by the host link:
// 2 d h element bytes per expert against a few microseconds of matrix-core work per row.
#include "common.h"
#include "moe_offload.h"

#include <mutex>

namespace moe {
namespace {

struct OffloadResources {
    hipStream_t copy = nullptr;
    hipEvent_t ready[kMaxExperts] = {};     // slot filled
    hipEvent_t freed[kMaxExperts] = {};     // slot's expert computed
    hipEvent_t begin = nullptr;
    bool ok = false;
    std::mutex enqueue;                     // held while a call enqueues on the copy stream
};
OffloadResources g_res[16];
std::mutex g_res_mutex;

moe_status resources(OffloadResources **out)
{
    int dev = 0;
    MOE_TRY_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16) {
        set_error("device ordinal %d is outside the supported range", dev);
        return MOE_EUNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_res_mutex);
    OffloadResources &r = g_res[dev];
    if (!r.ok) {
        MOE_TRY_HIP(hipStreamCreateWithFlags(&r.copy, hipStreamNonBlocking));
        MOE_TRY_HIP(hipEventCreateWithFlags(&r.begin, hipEventDisableTiming));
        for (int i = 0; i < kMaxExperts; ++i) {
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.ready[i], hipEventDisableTiming));
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.freed[i], hipEventDisableTiming));
        }
        r.ok = true;
    }
    *out = &r;
    return MOE_OK;
}

bool supported(const moe_shape *s)
{
    return s != nullptr && s->dtype == MOE_BF16 && s->T >= 1 && s->E >= 1 && s->E <= kMaxExperts &&
           s->k >= 1 && s->k <= kMaxTopK && s->k <= s->E && s->capacity >= 1 && s->d_model >= 8 &&
           s->d_ff >= 8 && s->d_model % 8 == 0 && s->d_ff % 8 == 0;
}

size_t expert_bytes(const moe_shape &s) { return static_cast<size_t>(s.d_model) * s.d_ff * 2; }

void layout(const moe_shape &s, void *base, Workspace *w)
{
    char *p = static_cast<char *>(base);
    size_t off = 0;
    *w = Workspace{};
    for (int g = 0; g < 2; ++g) {
        w->gp[g] = choose_gemm_plan(s, g, 1);            // the resident path's tile shapes
        w->items[g] = reinterpret_cast<WorkItem *>(p + off);
        off += align_up(static_cast<size_t>(s.E) * w->gp[g].max_items * sizeof(WorkItem), 256);
        w->nitems[g] = reinterpret_cast<int32_t *>(p + off);
        off += align_up(static_cast<size_t>(s.E) * sizeof(int32_t), 256);
    }
    w->hidden = p + off;
    off += align_up(static_cast<size_t>(moe_max_rows(&s)) * s.d_ff * 2, 256);
    w->bytes = off;
}

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

size_t moe_offload_staging_bytes(const moe_shape *s, int32_t resident)
{
    if (!supported(s) || resident < 1) return 0;
    return static_cast<size_t>(resident > s->E ? s->E : resident) * 2 * align_up(expert_bytes(*s), 256);
}

size_t moe_offload_workspace_bytes(const moe_shape *s)
{
    if (!supported(s)) return 0;
    Workspace w;
    layout(*s, reinterpret_cast<void *>(static_cast<uintptr_t>(256)), &w);
    return w.bytes;
}

moe_status moe_expert_ffn_offloaded(const moe_shape *s, const void *xe, const int32_t *offsets,
                                    const void *W1p_host, const void *W2p_host, const float *b1,
                                    const float *b2, void *ye, void *staging, int32_t resident,
                                    void *workspace, void *stream)
{
    if (!supported(s)) {
        set_error("moe_expert_ffn_offloaded: bf16 layers, E <= %d, k <= %d, d_model and d_ff "
                  "multiples of 8", kMaxExperts, kMaxTopK);
        return s == nullptr ? MOE_EINVAL : MOE_EUNSUPPORTED;
    }
    if (resident < 1) {
        set_error("resident = %d: at least one expert slot is needed", resident);
        return MOE_EINVAL;
    }
    const void *need[] = {xe, offsets, W1p_host, W2p_host, ye, staging, workspace};
    for (const void *p : need) {
        if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) != 0) {
            set_error("moe_expert_ffn_offloaded: a required pointer is NULL or not 16-byte aligned");
            return MOE_EINVAL;
        }
    }
    if (resident > s->E) resident = s->E;
    OffloadResources *r = nullptr;
    const moe_status rs = resources(&r);
    if (rs != MOE_OK) return rs;
    // one call at a time enqueues on this device's copy stream and shared events
    std::lock_guard<std::mutex> enqueue(r->enqueue);
    Workspace w;
    layout(*s, workspace, &w);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t eb = expert_bytes(*s), slot_bytes = align_up(eb, 256);
    char *stage = static_cast<char *>(staging);
    const char *h1 = static_cast<const char *>(W1p_host), *h2 = static_cast<const char *>(W2p_host);

    moe_status rc = launch_items_per_expert(*s, offsets, w, st);
    if (rc != MOE_OK) return rc;
    // the copy stream may not touch the staging area before what the caller enqueued earlier
    // (possibly a previous call's GEMMs reading it) has finished
    MOE_TRY_HIP(hipEventRecord(r->begin, st));
    MOE_TRY_HIP(hipStreamWaitEvent(r->copy, r->begin, 0));
    for (int e = 0; e < s->E; ++e) {
        const int slot = e % resident;
        char *d1 = stage + static_cast<size_t>(slot) * 2 * slot_bytes, *d2 = d1 + slot_bytes;
        if (e >= resident) MOE_TRY_HIP(hipStreamWaitEvent(r->copy, r->freed[slot], 0));
        MOE_TRY_HIP(hipMemcpyAsync(d1, h1 + static_cast<size_t>(e) * eb, eb, hipMemcpyHostToDevice, r->copy));
        MOE_TRY_HIP(hipMemcpyAsync(d2, h2 + static_cast<size_t>(e) * eb, eb, hipMemcpyHostToDevice, r->copy));
        MOE_TRY_HIP(hipEventRecord(r->ready[slot], r->copy));
        MOE_TRY_HIP(hipStreamWaitEvent(st, r->ready[slot], 0));
        // The GEMM kernel addresses expert e's weights as base + e * d * h elements: hand it
        // a base that lands on the slot.  Only [slot, slot + eb) is ever dereferenced, since
        // list e holds expert e's tiles only.
        const char *f1 = d1 - static_cast<size_t>(e) * eb, *f2 = d2 - static_cast<size_t>(e) * eb;
        rc = launch_ffn(*s, xe, f1, b1, f2, b2, ye, w, e, st);
        if (rc != MOE_OK) return rc;
        MOE_TRY_HIP(hipEventRecord(r->freed[slot], st));
    }
    return MOE_OK;
}

}  // extern "C"
