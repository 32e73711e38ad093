// Padded equal-split layout, all-to-all micro-ops pipelined with the expert FFN, and the
// communication scheduler that gives all-to-all micro-ops the link before allreduce
// micro-ops (paper Sec. 4.2, Sec. 6.1) -- on one GPU, with a copy kernel of a few
// workgroups on its own stream standing in for the network link.
//
//   link_copy_kernel   one micro-op: rows [r0, r1) of every slab, send -> receive buffer
//   pack_padded_kernel the slot rows of one micro-op: a kept slot receives its token's row,
//                      an empty slot zeros (an equal-split all-to-all carries those too)
//   Comm               the scheduler: operations cut into micro-ops, two ready queues, one
//                      thread that keeps at most `depth` micro-ops on the link and picks
//                      the next one by the policy
//   moe_layer_padded   gate, padded plan, pack, and per micro-op: first all-to-all, FFN,
//                      second all-to-all; combine at the end
#include "common.h"
#include "moe_comm.h"

#include <chrono>
#include <condition_variable>
#include <deque>
#include <map>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

#define MOE_TRY(expr)                        \
    do {                                     \
        moe_status st_ = (expr);             \
        if (st_ != MOE_OK) return st_;       \
    } while (0)

namespace moe {
namespace {

// ---------------------------------------------------------------- kernels
// Vector i of the micro-op is vector (i % nvec) of slab (i / nvec)'s rows [r0, r1); four
// loads in flight per lane.
__global__ __launch_bounds__(256) void link_copy_kernel(
    const uint4 *__restrict__ src, uint4 *__restrict__ dst, long long slab_vecs, long long v0,
    long long nvec, long long total)
{
    const long long stride = static_cast<long long>(gridDim.x) * 256;
    long long i = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
    for (; i + 3 * stride < total; i += 4 * stride) {
        long long at[4];
        uint4 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const long long j = i + q * stride;
            at[q] = (j / nvec) * slab_vecs + v0 + j % nvec;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = src[at[q]];
#pragma unroll
        for (int q = 0; q < 4; ++q) dst[at[q]] = v[q];
    }
    for (; i < total; i += stride) {
        const long long at = (i / nvec) * slab_vecs + v0 + i % nvec;
        dst[at] = src[at];
    }
}

// One wavefront per slot row: row r of the micro-op is position p0 + r % np of expert r / np.
__global__ __launch_bounds__(256) void pack_padded_kernel(
    const uint4 *__restrict__ x, const int32_t *__restrict__ src_of,
    const int32_t *__restrict__ counts, uint4 *__restrict__ xs, int capacity, int p0, int np,
    int E, int k, int n_assign, int vec)
{
    const int lane = lane_id();
    const int r = blockIdx.x * 4 + threadIdx.x / kWave;
    if (r >= E * np) return;
    const int e = r / np, p = p0 + r % np;
    const size_t slot = static_cast<size_t>(e) * capacity + p;
    uint4 *out = xs + slot * vec;
    if (p < min(counts[e], capacity)) {
        const int i = min(max(src_of[slot], 0), n_assign - 1);
        const uint4 *in = x + static_cast<size_t>(i / k) * vec;
        for (int c = lane; c < vec; c += kWave) out[c] = in[c];
    } else {
        for (int c = lane; c < vec; c += kWave) out[c] = make_uint4(0u, 0u, 0u, 0u);
    }
}

void launch_link_copy(const void *src, void *dst, int64_t slabs, int64_t rows, int64_t row_bytes,
                      int64_t r0, int64_t r1, int blocks, hipStream_t st)
{
    const long long row_vecs = row_bytes / 16;
    const long long nvec = (r1 - r0) * row_vecs;
    const long long total = slabs * nvec;
    if (total <= 0) return;
    const long long need = (total + 255) / 256;
    const int grid = static_cast<int>(need < blocks ? need : blocks);
    hipLaunchKernelGGL(link_copy_kernel, dim3(grid), dim3(256), 0, st,
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), rows * row_vecs,
                       r0 * row_vecs, nvec, total);
}

// ---------------------------------------------------------------- scheduler
struct MicroOp {
    int state = 0;                 // 0 announced, 1 posted (ready queue), 2 on the link, 3 done
    hipEvent_t ready = nullptr;    // shared by the micro-ops of one post
    hipEvent_t done = nullptr;     // what consumers' streams wait for
    bool data_seen = false;        // its ready event was found complete: no wait needed on the link
    int64_t ready_seq = 0;
    int64_t posted_ns = 0;
    int64_t log_index = -1;        // position of its record in the log (counted from the first ever)
};

struct Op {
    int64_t id = 0;
    int kind = 0;
    const char *src = nullptr;
    char *dst = nullptr;
    int64_t slabs = 0, rows = 0, row_bytes = 0;
    int n = 0;
    std::vector<MicroOp> m;
    std::vector<hipEvent_t> post_events;   // in post order; the first is the operation's start
    int issued = 0, completed = 0;
    bool released = false;
};

using Clock = std::chrono::steady_clock;

}  // namespace
}  // namespace moe

using namespace moe;

struct moe_comm {
    int device = 0;
    int policy = 0, blocks = 1, depth = 1;
    hipStream_t link = nullptr;
    std::thread thread;
    std::mutex mu;
    std::condition_variable cv_work;    // the thread sleeps here when it has nothing to do
    std::condition_variable cv_state;   // callers sleep here for "on the link" / "done"
    std::map<int64_t, std::unique_ptr<Op>> ops;
    int64_t next_id = 1;
    std::deque<std::pair<Op *, int>> ready[2];   // per kind under the priority policy; [0] alone otherwise
    std::deque<std::pair<Op *, int>> on_link;
    int a2a_on_link = 0;
    bool hold = false, paused = false, stop = false;
    int64_t seq = 0;
    std::deque<moe_comm_record> log;
    int64_t log_dropped = 0;            // records that fell off the front of the log
    Clock::time_point t0 = Clock::now();
    std::vector<hipEvent_t> pool;
    hipError_t failed = hipSuccess;     // first HIP error met by the thread

    int64_t now_ns() const
    {
        return std::chrono::duration_cast<std::chrono::nanoseconds>(Clock::now() - t0).count();
    }

    void add_record(const moe_comm_record &rec)
    {
        log.push_back(rec);
        if (log.size() > 65536) {
            log.pop_front();
            log_dropped += 1;
        }
    }

    hipEvent_t take_event()
    {
        if (!pool.empty()) {
            hipEvent_t e = pool.back();
            pool.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }

    void recycle(Op *op)
    {
        for (hipEvent_t e : op->post_events) pool.push_back(e);
        for (MicroOp &mo : op->m)
            if (mo.done != nullptr) pool.push_back(mo.done);
        ops.erase(op->id);
    }

    // Waits for a micro-op to leave the link by polling its event: a blocking host wait
    // holds the event's lock in the runtime for as long as it lasts, and a consumer's
    // hipStreamWaitEvent on the same event would then block the consumer's thread until the
    // micro-op has finished.  Polls flat out for a short while (a micro-op of a few MiB is
    // shorter than a sleeping thread's wake-up), then with naps in between.
    static hipError_t wait_for(hipEvent_t ev)
    {
        const auto spin_until = Clock::now() + std::chrono::microseconds(200);
        hipError_t e = hipEventQuery(ev);
        while (e == hipErrorNotReady) {
            if (Clock::now() >= spin_until) std::this_thread::sleep_for(std::chrono::microseconds(50));
            e = hipEventQuery(ev);
        }
        (void)hipGetLastError();            // "not ready" is not an error to report later
        return e;
    }

    // The next micro-op by the policy, or false.  Called with the lock held.
    bool choose(std::pair<Op *, int> *out)
    {
        if (paused) return false;
        if (!ready[0].empty()) {
            *out = ready[0].front();
            ready[0].pop_front();
            return true;
        }
        if (policy == MOE_COMM_PRIORITY && !ready[1].empty() && !hold && a2a_on_link == 0) {
            *out = ready[1].front();
            ready[1].pop_front();
            return true;
        }
        return false;
    }

    void run()
    {
        (void)hipSetDevice(device);
        std::unique_lock<std::mutex> lock(mu);
        for (;;) {
            std::pair<Op *, int> next;
            if (static_cast<int>(on_link.size()) < depth && failed == hipSuccess && choose(&next)) {
                Op *op = next.first;
                MicroOp &mo = op->m[next.second];
                const int64_t r0 = static_cast<int64_t>(next.second) * op->rows / op->n;
                const int64_t r1 = static_cast<int64_t>(next.second + 1) * op->rows / op->n;
                hipError_t e = hipSuccess;
                if (!mo.data_seen) {
                    if (hipEventQuery(mo.ready) == hipSuccess) {
                        // (its neighbours of the same post need not ask again)
                        for (MicroOp &other : op->m)
                            if (other.ready == mo.ready) other.data_seen = true;
                    } else {
                        (void)hipGetLastError();
                        e = hipStreamWaitEvent(link, mo.ready, 0);
                    }
                }
                if (e == hipSuccess) {
                    launch_link_copy(op->src, op->dst, op->slabs, op->rows, op->row_bytes, r0, r1,
                                     blocks, link);
                    e = hipGetLastError();
                }
                if (e == hipSuccess) e = hipEventRecord(mo.done, link);
                if (e != hipSuccess) failed = e;
                mo.state = 2;
                op->issued += 1;
                if (op->kind == MOE_COMM_ALL_TO_ALL) a2a_on_link += 1;
                on_link.push_back(next);
                moe_comm_record rec;
                rec.op = op->id;
                rec.micro = next.second;
                rec.kind = op->kind;
                rec.bytes = op->slabs * (r1 - r0) * op->row_bytes;
                rec.ready_seq = mo.ready_seq;
                rec.issue_seq = seq++;
                rec.posted_ns = mo.posted_ns;
                rec.launched_ns = now_ns();
                rec.done_ns = 0;
                mo.log_index = log_dropped + static_cast<int64_t>(log.size());
                add_record(rec);
                cv_state.notify_all();
                continue;
            }
            if (!on_link.empty()) {
                // wait for the oldest micro-op on the link without holding the lock
                const std::pair<Op *, int> front = on_link.front();
                hipEvent_t done = front.first->m[front.second].done;
                lock.unlock();
                const hipError_t e = wait_for(done);
                lock.lock();
                if (e != hipSuccess && failed == hipSuccess) failed = e;
                on_link.pop_front();
                Op *op = front.first;
                const int64_t at = op->m[front.second].log_index - log_dropped;
                if (at >= 0 && at < static_cast<int64_t>(log.size())) log[at].done_ns = now_ns();
                op->m[front.second].state = 3;
                op->completed += 1;
                if (op->kind == MOE_COMM_ALL_TO_ALL) a2a_on_link -= 1;
                if (op->released && op->completed == op->n) recycle(op);
                cv_state.notify_all();
                continue;
            }
            if (stop) break;
            cv_work.wait(lock);
        }
    }
};

namespace {

moe_status comm_failed(moe_comm *c)
{
    set_error("the scheduler thread met HIP error %d (%s)", static_cast<int>(c->failed),
              hipGetErrorString(c->failed));
    return MOE_EHIP;
}

Op *find_op(moe_comm *c, int64_t id)
{
    auto it = c->ops.find(id);
    return it == c->ops.end() ? nullptr : it->second.get();
}

// Side stream and events of moe_layer_padded's own link, per device, kept for the process.
struct PaddedResources {
    bool ready = false;
    std::mutex enqueue;        // held while a call enqueues on the link stream
    hipStream_t link = nullptr;
    hipEvent_t packed[kMaxChunks] = {}, arrived[kMaxChunks] = {}, computed[kMaxChunks] = {};
    hipEvent_t returned = nullptr;
};
std::mutex g_padded_mutex;
PaddedResources g_padded[16];

moe_status padded_resources(PaddedResources **out)
{
    int dev = 0;
    MOE_TRY_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16) {
        set_error("device index %d out of range", dev);
        return MOE_EUNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_padded_mutex);
    PaddedResources &r = g_padded[dev];
    if (!r.ready) {
        MOE_TRY_HIP(hipStreamCreateWithFlags(&r.link, hipStreamNonBlocking));
        MOE_TRY_HIP(hipEventCreateWithFlags(&r.returned, hipEventDisableTiming));
        for (int c = 0; c < kMaxChunks; ++c) {
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.packed[c], hipEventDisableTiming));
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.arrived[c], hipEventDisableTiming));
            MOE_TRY_HIP(hipEventCreateWithFlags(&r.computed[c], hipEventDisableTiming));
        }
        r.ready = true;
    }
    *out = &r;
    return MOE_OK;
}

// Workspace of the padded layer: the plan's scratch, the compact offsets nobody outside
// needs, per micro-op work lists, and the hidden activations of all E*C slots.
struct PaddedWorkspace {
    Workspace w;
    int32_t *offsets = nullptr;
    size_t bytes = 0;
};

bool padded_shape_ok(const moe_shape *s, int n_micro)
{
    if (moe_workspace_bytes(s, 1) == 0) return false;            // the common shape checks
    if (static_cast<int64_t>(s->E) * s->capacity >= (1ll << 31)) {
        set_error("E * capacity does not fit 31 bits");
        return false;
    }
    if (n_micro < 1 || n_micro > kMaxChunks || n_micro > s->capacity) {
        set_error("n_micro must be in 1..min(capacity, %d), got %d", kMaxChunks, n_micro);
        return false;
    }
    return true;
}

void layout_padded(const moe_shape &s, int n_micro, void *base, PaddedWorkspace *pw)
{
    Workspace &w = pw->w;
    w = Workspace{};
    w.seg_tok = route_segment_tokens(s);
    w.nseg = (s.T + w.seg_tok - 1) / w.seg_tok;
    char *p = static_cast<char *>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *at = p + off;
        off += align_up(bytes, 256);
        return at;
    };
    w.seg_cnt = reinterpret_cast<int32_t *>(take(static_cast<size_t>(w.nseg) * kMaxExperts * 4));
    pw->offsets = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (s.E + 1)));
    const int per_micro = (s.capacity + n_micro - 1) / n_micro;   // slot positions, at most
    for (int g = 0; g < 2; ++g) {
        GemmPlan gp = choose_gemm_plan(s, g, n_micro);
        gp.max_row_tiles = s.E * ((per_micro + gp.bm - 1) / gp.bm);
        gp.max_items = gp.max_row_tiles * gp.tiles_n;
        w.gp[g] = gp;
        w.items[g] = reinterpret_cast<WorkItem *>(take(sizeof(WorkItem) * n_micro * gp.max_items));
        w.nitems[g] = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * n_micro));
    }
    const size_t hidden_elem = s.dtype == MOE_BF16 ? 2 : 4;
    w.hidden = take(static_cast<size_t>(s.E) * s.capacity * s.d_ff * hidden_elem);
    w.bytes = pw->bytes = off;
}

}  // namespace

extern "C" {

// ---------------------------------------------------------------- scheduler ABI
moe_status moe_comm_create(moe_comm **out, moe_comm_policy policy, int32_t link_blocks, int32_t depth)
{
    if (out == nullptr || (policy != MOE_COMM_ARRIVAL_ORDER && policy != MOE_COMM_PRIORITY) ||
        link_blocks < 1 || link_blocks > 1024 || depth < 1 || depth > 4) {
        set_error("moe_comm_create: policy 0 or 1, link_blocks 1..1024, depth 1..4");
        return MOE_EINVAL;
    }
    std::unique_ptr<moe_comm> c(new moe_comm);
    MOE_TRY_HIP(hipGetDevice(&c->device));
    c->policy = policy;
    c->blocks = link_blocks;
    c->depth = depth;
    MOE_TRY_HIP(hipStreamCreateWithFlags(&c->link, hipStreamNonBlocking));
    moe_comm *raw = c.release();
    raw->thread = std::thread([raw] { raw->run(); });
    *out = raw;
    return MOE_OK;
}

moe_status moe_comm_destroy(moe_comm *c)
{
    if (c == nullptr) return MOE_OK;
    {
        std::lock_guard<std::mutex> lock(c->mu);
        c->stop = true;
        c->paused = false;
        c->hold = false;
    }
    c->cv_work.notify_all();
    c->thread.join();          // the thread leaves once both queues and the link are empty
    (void)hipStreamSynchronize(c->link);
    for (auto &kv : c->ops) {
        for (hipEvent_t e : kv.second->post_events) (void)hipEventDestroy(e);
        for (MicroOp &mo : kv.second->m)
            if (mo.done != nullptr) (void)hipEventDestroy(mo.done);
    }
    for (hipEvent_t e : c->pool) (void)hipEventDestroy(e);
    (void)hipStreamDestroy(c->link);
    delete c;
    return MOE_OK;
}

moe_status moe_comm_submit(moe_comm *c, moe_comm_kind kind, const void *src, void *dst,
                           int64_t slabs, int64_t rows, int64_t row_bytes, int32_t n_micro,
                           int64_t *op_out)
{
    if (c == nullptr || op_out == nullptr || src == nullptr || dst == nullptr ||
        (kind != MOE_COMM_ALL_TO_ALL && kind != MOE_COMM_ALLREDUCE) || slabs < 1 || rows < 1 ||
        row_bytes < 16 || row_bytes % 16 != 0 || n_micro < 1 || n_micro > 4096 || n_micro > rows ||
        ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) != 0) {
        set_error("moe_comm_submit: NULL or misaligned pointer, or slabs/rows < 1, row_bytes not a "
                  "multiple of 16, n_micro outside 1..min(rows, 4096)");
        return MOE_EINVAL;
    }
    std::lock_guard<std::mutex> lock(c->mu);
    if (c->failed != hipSuccess) return comm_failed(c);
    std::unique_ptr<Op> op(new Op);
    op->id = c->next_id++;
    op->kind = kind;
    op->src = static_cast<const char *>(src);
    op->dst = static_cast<char *>(dst);
    op->slabs = slabs;
    op->rows = rows;
    op->row_bytes = row_bytes;
    op->n = n_micro;
    op->m.resize(n_micro);
    for (MicroOp &mo : op->m) {
        mo.done = c->take_event();
        if (mo.done == nullptr) {
            for (MicroOp &back : op->m)
                if (back.done != nullptr) c->pool.push_back(back.done);
            set_error("moe_comm_submit: could not create an event");
            return MOE_EHIP;
        }
    }
    *op_out = op->id;
    c->ops[op->id] = std::move(op);
    return MOE_OK;
}

moe_status moe_comm_post(moe_comm *c, int64_t id, int32_t first, int32_t count, void *producer_stream)
{
    if (c == nullptr) {
        set_error("moe_comm_post: NULL scheduler");
        return MOE_EINVAL;
    }
    std::lock_guard<std::mutex> lock(c->mu);
    if (c->failed != hipSuccess) return comm_failed(c);
    Op *op = find_op(c, id);
    if (op == nullptr || op->released || first < 0 || count < 1 || first + count > op->n) {
        set_error("moe_comm_post: unknown operation or micro-ops [%d, %d) out of range", first,
                  first + count);
        return MOE_EINVAL;
    }
    for (int i = first; i < first + count; ++i) {
        if (op->m[i].state != 0) {
            set_error("moe_comm_post: micro-op %d was posted before", i);
            return MOE_EINVAL;
        }
    }
    hipEvent_t ev = c->take_event();
    if (ev == nullptr) {
        set_error("moe_comm_post: could not create an event");
        return MOE_EHIP;
    }
    const hipError_t e = hipEventRecord(ev, static_cast<hipStream_t>(producer_stream));
    if (e != hipSuccess) {
        c->pool.push_back(ev);
        return hip_fail(e, "hipEventRecord(ready)");
    }
    // An event recorded on an idle stream may sit in the runtime's batch until something
    // forces it out -- which would be the link's own wait, possibly much later: its time
    // stamp would then say when it was looked at, not when the data was ready.  A query
    // sends it on its way (and "not ready" is no error).
    (void)hipEventQuery(ev);
    (void)hipGetLastError();
    op->post_events.push_back(ev);
    const int64_t ready_seq = c->seq++;
    const int64_t posted_ns = c->now_ns();
    const int q = c->policy == MOE_COMM_PRIORITY ? op->kind : 0;
    for (int i = first; i < first + count; ++i) {
        op->m[i].state = 1;
        op->m[i].posted_ns = posted_ns;
        op->m[i].ready = ev;
        op->m[i].ready_seq = ready_seq;
        c->ready[q].push_back({op, i});
    }
    c->cv_work.notify_all();
    return MOE_OK;
}

moe_status moe_comm_wait(moe_comm *c, int64_t id, int32_t micro, void *consumer_stream,
                         int32_t timeout_ms)
{
    if (c == nullptr) {
        set_error("moe_comm_wait: NULL scheduler");
        return MOE_EINVAL;
    }
    std::unique_lock<std::mutex> lock(c->mu);
    Op *op = find_op(c, id);
    if (op == nullptr || op->released || micro < -1 || micro >= op->n) {
        set_error("moe_comm_wait: unknown operation or micro-op %d out of range", micro);
        return MOE_EINVAL;
    }
    const int last = micro < 0 ? op->n - 1 : micro;
    const auto until = Clock::now() + std::chrono::milliseconds(timeout_ms < 0 ? 0 : timeout_ms);
    // (micro-ops of one operation go to the link in the order of their posts; waiting for all
    // of them means waiting for each)
    auto launched = [&] {
        if (c->failed != hipSuccess) return true;
        if (micro >= 0) return op->m[micro].state >= 2;
        return op->issued == op->n;
    };
    if (!c->cv_state.wait_until(lock, until, launched)) {
        set_error("moe_comm_wait: micro-op %d of operation %lld was not launched within %d ms "
                  "(%d of %d launched, %zu + %zu ready, %zu on the link, hold %d, paused %d)",
                  micro, static_cast<long long>(id), timeout_ms, op->issued, op->n,
                  c->ready[0].size(), c->ready[1].size(), c->on_link.size(), c->hold ? 1 : 0,
                  c->paused ? 1 : 0);
        return MOE_EHIP;
    }
    if (c->failed != hipSuccess) return comm_failed(c);
    hipStream_t st = static_cast<hipStream_t>(consumer_stream);
    if (micro >= 0) {
        MOE_TRY_HIP(hipStreamWaitEvent(st, op->m[last].done, 0));
    } else {
        for (int i = 0; i < op->n; ++i) MOE_TRY_HIP(hipStreamWaitEvent(st, op->m[i].done, 0));
    }
    return MOE_OK;
}

moe_status moe_comm_hold(moe_comm *c, int32_t on)
{
    if (c == nullptr) {
        set_error("moe_comm_hold: NULL scheduler");
        return MOE_EINVAL;
    }
    std::lock_guard<std::mutex> lock(c->mu);
    c->hold = on != 0;
    moe_comm_record rec;
    rec.op = -1;
    rec.micro = on != 0 ? 1 : 0;
    rec.kind = 2;
    rec.bytes = 0;
    rec.ready_seq = rec.issue_seq = c->seq++;
    rec.posted_ns = rec.launched_ns = rec.done_ns = c->now_ns();
    c->add_record(rec);
    c->cv_work.notify_all();
    return MOE_OK;
}

moe_status moe_comm_pause(moe_comm *c, int32_t on)
{
    if (c == nullptr) {
        set_error("moe_comm_pause: NULL scheduler");
        return MOE_EINVAL;
    }
    std::lock_guard<std::mutex> lock(c->mu);
    c->paused = on != 0;
    c->cv_work.notify_all();
    return MOE_OK;
}

moe_status moe_comm_release(moe_comm *c, int64_t id)
{
    if (c == nullptr) {
        set_error("moe_comm_release: NULL scheduler");
        return MOE_EINVAL;
    }
    std::lock_guard<std::mutex> lock(c->mu);
    Op *op = find_op(c, id);
    if (op == nullptr || op->released) {
        set_error("moe_comm_release: unknown operation");
        return MOE_EINVAL;
    }
    for (const MicroOp &mo : op->m) {
        if (mo.state == 0) {
            set_error("moe_comm_release: the operation has micro-ops that were never posted");
            return MOE_EINVAL;
        }
    }
    op->released = true;
    if (op->completed == op->n) c->recycle(op);
    return MOE_OK;
}

moe_status moe_comm_finish(moe_comm *c, int64_t id, int32_t timeout_ms, float *gpu_ms)
{
    if (c == nullptr) {
        set_error("moe_comm_finish: NULL scheduler");
        return MOE_EINVAL;
    }
    std::unique_lock<std::mutex> lock(c->mu);
    Op *op = find_op(c, id);
    if (op == nullptr || op->released) {
        set_error("moe_comm_finish: unknown operation");
        return MOE_EINVAL;
    }
    const auto until = Clock::now() + std::chrono::milliseconds(timeout_ms < 0 ? 0 : timeout_ms);
    if (!c->cv_state.wait_until(lock, until, [&] {
            return c->failed != hipSuccess || op->completed == op->n;
        })) {
        set_error("moe_comm_finish: operation %lld not complete within %d ms (%d of %d micro-ops "
                  "done, %d launched)", static_cast<long long>(id), timeout_ms, op->completed,
                  op->n, op->issued);
        return MOE_EHIP;
    }
    if (c->failed != hipSuccess) return comm_failed(c);
    moe_status rc = MOE_OK;
    if (gpu_ms != nullptr) {
        const hipError_t e = hipEventElapsedTime(gpu_ms, op->post_events.front(), op->m[op->n - 1].done);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventElapsedTime(operation)");
    }
    c->recycle(op);
    return rc;
}

int32_t moe_comm_log(moe_comm *c, moe_comm_record *out, int32_t cap)
{
    if (c == nullptr || out == nullptr || cap < 1) return 0;
    std::lock_guard<std::mutex> lock(c->mu);
    const size_t n = c->log.size() < static_cast<size_t>(cap) ? c->log.size() : static_cast<size_t>(cap);
    const size_t from = c->log.size() - n;
    for (size_t i = 0; i < n; ++i) out[i] = c->log[from + i];
    return static_cast<int32_t>(n);
}

// ---------------------------------------------------------------- padded layer ABI
size_t moe_padded_workspace_bytes(const moe_shape *s, int32_t n_micro)
{
    if (s == nullptr || !padded_shape_ok(s, n_micro)) return 0;
    PaddedWorkspace pw;
    layout_padded(*s, n_micro, nullptr, &pw);
    return pw.bytes;
}

moe_status moe_layer_padded(const moe_shape *s, int32_t n_micro, moe_comm *link,
                            int32_t link_blocks, const void *x, const float *Wgp,
                            const float *gate_bias, int32_t bias_token_stride, const void *W1p,
                            const float *b1, const void *W2p, const float *b2,
                            int32_t *expert_idx, float *gate, int32_t *counts, int32_t *slot_of,
                            int32_t *src_of, void *xs, void *xr, void *ys, void *yr, float *y,
                            void *workspace, void *stream)
{
    if (s == nullptr || !padded_shape_ok(s, n_micro)) return s == nullptr ? MOE_EINVAL : MOE_EUNSUPPORTED;
    if (link == nullptr && (link_blocks < 1 || link_blocks > 1024)) {
        set_error("moe_layer_padded: link_blocks must be in 1..1024");
        return MOE_EINVAL;
    }
    if (gate_bias != nullptr && bias_token_stride != 0 && bias_token_stride != s->E) {
        set_error("bias_token_stride must be 0 or E");
        return MOE_EINVAL;
    }
    const void *need[] = {x, Wgp, W1p, W2p, expert_idx, gate, counts, slot_of, src_of, xs, xr, ys, yr,
                          y, workspace};
    for (const void *p : need) {
        if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) != 0) {
            set_error("moe_layer_padded: a required pointer is NULL or not 16-byte aligned");
            return MOE_EINVAL;
        }
    }
    const int E = s->E, C = s->capacity, d = s->d_model;
    const int elem = s->dtype == MOE_BF16 ? 2 : 4;
    const int vec = d * elem / 16;
    const int64_t slots = static_cast<int64_t>(E) * C;
    PaddedWorkspace pw;
    layout_padded(*s, n_micro, workspace, &pw);
    hipStream_t st = static_cast<hipStream_t>(stream);

    MOE_TRY(launch_route(*s, x, Wgp, gate_bias, bias_token_stride, expert_idx, gate, pw.w.seg_cnt, st));
    MOE_TRY(launch_plan(*s, expert_idx, counts, pw.offsets, slot_of, src_of, pw.w, true, 1, st, true));
    MOE_TRY(launch_items_padded(*s, n_micro, counts, pw.w, st));

    auto pack = [&](int m) {
        const int p0 = static_cast<int>(static_cast<int64_t>(m) * C / n_micro);
        const int p1 = static_cast<int>(static_cast<int64_t>(m + 1) * C / n_micro);
        const int rows = E * (p1 - p0);
        if (rows > 0)
            hipLaunchKernelGGL(pack_padded_kernel, dim3(ceil_div(rows, 4)), dim3(256), 0, st,
                               static_cast<const uint4 *>(x), src_of, counts, static_cast<uint4 *>(xs),
                               C, p0, p1 - p0, E, s->k, s->T * s->k, vec);
    };

    if (link != nullptr) {
        // both all-to-alls as operations of the caller's scheduler
        int64_t first = 0, second = 0;
        MOE_TRY(moe_comm_submit(link, MOE_COMM_ALL_TO_ALL, xs, xr, E, C, static_cast<int64_t>(d) * elem,
                                n_micro, &first));
        moe_status rc = moe_comm_submit(link, MOE_COMM_ALL_TO_ALL, ys, yr, E, C,
                                        static_cast<int64_t>(d) * ye_elem_bytes(*s), n_micro, &second);
        const int timeout_ms = 20000;
        int posted1 = 0, posted2 = 0;
        for (int m = 0; rc == MOE_OK && m < n_micro; ++m) {
            pack(m);
            rc = moe_comm_post(link, first, m, 1, st);
            if (rc == MOE_OK) posted1 = m + 1;
        }
        for (int m = 0; rc == MOE_OK && m < n_micro; ++m) {
            rc = moe_comm_wait(link, first, m, st, timeout_ms);
            if (rc == MOE_OK) rc = launch_ffn(*s, xr, W1p, b1, W2p, b2, ys, pw.w, m, st);
            if (rc == MOE_OK) rc = moe_comm_post(link, second, m, 1, st);
            if (rc == MOE_OK) posted2 = m + 1;
        }
        if (rc == MOE_OK) rc = moe_comm_wait(link, second, -1, st, timeout_ms);
        if (rc == MOE_OK) rc = launch_combine(*s, yr, slot_of, gate, y, nullptr, 0, s->T, st, slots);
        // An operation must be fully posted before it can be let go: after an error post the
        // rest (the data is then meaningless, but every micro-op still leaves the link).
        char msg[512];
        snprintf(msg, sizeof(msg), "%s", moe_last_error());
        if (posted1 < n_micro) (void)moe_comm_post(link, first, posted1, n_micro - posted1, st);
        if (posted2 < n_micro) (void)moe_comm_post(link, second, posted2, n_micro - posted2, st);
        (void)moe_comm_release(link, first);
        (void)moe_comm_release(link, second);
        if (rc != MOE_OK) set_error("%s", msg);
        return rc;
    }

    PaddedResources *r = nullptr;
    MOE_TRY(padded_resources(&r));
    // one call at a time enqueues on this device's link stream and shared events
    std::lock_guard<std::mutex> enqueue(r->enqueue);
    auto range = [&](int m, int64_t *r0, int64_t *r1) {
        *r0 = static_cast<int64_t>(m) * C / n_micro;
        *r1 = static_cast<int64_t>(m + 1) * C / n_micro;
    };
    auto send_first = [&](int m) -> moe_status {
        int64_t r0, r1;
        range(m, &r0, &r1);
        MOE_TRY_HIP(hipStreamWaitEvent(r->link, r->packed[m], 0));
        launch_link_copy(xs, xr, E, C, static_cast<int64_t>(d) * elem, r0, r1, link_blocks, r->link);
        MOE_TRY_HIP(hipEventRecord(r->arrived[m], r->link));
        return MOE_OK;
    };
    for (int m = 0; m < n_micro; ++m) {
        pack(m);
        MOE_TRY_HIP(hipEventRecord(r->packed[m], st));
    }
    MOE_TRY(send_first(0));
    for (int m = 0; m < n_micro; ++m) {
        MOE_TRY_HIP(hipStreamWaitEvent(st, r->arrived[m], 0));
        MOE_TRY(launch_ffn(*s, xr, W1p, b1, W2p, b2, ys, pw.w, m, st));
        MOE_TRY_HIP(hipEventRecord(r->computed[m], st));
        if (m + 1 < n_micro) MOE_TRY(send_first(m + 1));
        int64_t r0, r1;
        range(m, &r0, &r1);
        MOE_TRY_HIP(hipStreamWaitEvent(r->link, r->computed[m], 0));
        launch_link_copy(ys, yr, E, C, static_cast<int64_t>(d) * ye_elem_bytes(*s), r0, r1, link_blocks, r->link);
    }
    MOE_TRY_HIP(hipEventRecord(r->returned, r->link));
    MOE_TRY_HIP(hipStreamWaitEvent(st, r->returned, 0));
    MOE_TRY(launch_combine(*s, yr, slot_of, gate, y, nullptr, 0, s->T, st, slots));
    MOE_TRY_HIP(hipGetLastError());
    return MOE_OK;
}

}  // extern "C"
