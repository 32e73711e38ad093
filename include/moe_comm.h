/*
 * libmoe -- the padded equal-split layout, all-to-all micro-ops pipelined with the expert
 * FFN, and the communication scheduler that prioritises them over allreduce micro-ops
 * (paper Sec. 4, "Prioritizing All-to-All in Training": Sec. 4.2 tensor partitioning,
 * micro-ops and their pipelining; Sec. 6.1, "Communication scheduler"), on ONE GPU.
 *
 * One GPU has no peer to exchange tokens with, so the network is replaced by a stand-in
 * link: a copy kernel confined to `link_blocks` workgroups that moves a micro-op's bytes
 * from a send buffer to a receive buffer of the same device, one micro-op after the other
 * on one stream (the link is a serial resource; its rate grows with link_blocks).  What is
 * exercised at real shape is everything around the wire: the padded layout, the cut into
 * micro-ops, the FFN that starts after each micro-op, and the order in which micro-ops of
 * competing operations get the link.
 *
 * Padded layout (the equal-split all-to-all of training, Sec. 6.2 contrasts it with the
 * unequal split of inference): expert e owns the C = capacity slots [e*C, (e+1)*C) of an
 * [E*C, d_model] buffer; the assignment with rank p among those that chose e (token-major
 * order, as in moe_dispatch) sits in slot e*C + p if p < C and is dropped otherwise; slots
 * at or beyond min(count[e], C) are zero rows.  Micro-op m of n covers the slot positions
 * [floor(m*C/n), floor((m+1)*C/n)) of EVERY expert (the tensor is cut along the token
 * dimension, Sec. 6.1).
 *
 * Conventions as in moe.h (device pointers, caller-owned buffers, status codes,
 * moe_last_error).  Calls that take a moe_comm block the calling thread where stated.
 */
#ifndef MOE_COMM_H
#define MOE_COMM_H

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------ scheduler */

typedef struct moe_comm moe_comm;

typedef enum { MOE_COMM_ALL_TO_ALL = 0, MOE_COMM_ALLREDUCE = 1 } moe_comm_kind;

typedef enum {
    /* micro-ops get the link in the order in which they became ready, whatever their kind:
     * what happens when both operations are simply handed to the network (Sec. 2.2) */
    MOE_COMM_ARRIVAL_ORDER = 0,
    /* Sec. 4.2 / 6.1: a ready all-to-all micro-op always goes first; an allreduce micro-op
     * is launched only while no all-to-all micro-op is ready or on the link and the caller
     * has not announced one (moe_comm_hold) */
    MOE_COMM_PRIORITY = 1
} moe_comm_policy;

/*
 * A scheduler instance: one link (stream + copy kernel of link_blocks workgroups, 1..1024)
 * on the current device and one scheduler thread (Sec. 6.1: "runs a single thread").
 * depth (1..4) = micro-ops the thread keeps on the link at once: 1 lets a newly ready
 * all-to-all micro-op wait for at most one allreduce micro-op, 2 hides the host's
 * launch latency behind the running micro-op at the price of a second one.
 */
moe_status moe_comm_create(moe_comm **c, moe_comm_policy policy, int32_t link_blocks,
                           int32_t depth);

/* Waits until every submitted micro-op has left the link, stops the thread, frees all. */
moe_status moe_comm_destroy(moe_comm *c);

/*
 * Announces an operation that moves [slabs][rows][row_bytes] bytes (contiguous, same layout
 * on both sides, row_bytes a multiple of 16, both pointers 16-byte aligned) from src to dst,
 * cut into n_micro micro-ops (1 <= n_micro <= min(rows, 4096)): micro-op m moves rows
 * [floor(m*rows/n_micro), floor((m+1)*rows/n_micro)) of every slab.  A gradient of B bytes
 * cut into chunks of about S bytes is slabs = 1, rows = B/16, row_bytes = 16,
 * n_micro = ceil(B/S); chunks of different gradients never share a micro-op because every
 * gradient is its own operation.  Nothing moves until its micro-ops are posted.
 * *op receives the handle.
 */
moe_status moe_comm_submit(moe_comm *c, moe_comm_kind kind, const void *src, void *dst,
                           int64_t slabs, int64_t rows, int64_t row_bytes, int32_t n_micro,
                           int64_t *op);

/*
 * Micro-ops [first, first + count) of `op` are ready once the work enqueued so far on
 * `producer_stream` has run (an event is recorded there).  Every micro-op is posted once.
 */
moe_status moe_comm_post(moe_comm *c, int64_t op, int32_t first, int32_t count,
                         void *producer_stream);

/*
 * Makes `consumer_stream` wait for micro-op `micro` of `op` (-1: for the whole operation).
 * BLOCKS the calling thread until the scheduler thread has put that micro-op on the link
 * (at most `timeout_ms`, then MOE_EHIP with the state in moe_last_error); the wait for
 * its completion is the stream's, not the host's.
 */
moe_status moe_comm_wait(moe_comm *c, int64_t op, int32_t micro, void *consumer_stream,
                         int32_t timeout_ms);

/* Sec. 6.1: the caller knows an all-to-all is imminent (the combine computation of the
 * backward pass has started): while on != 0 no further allreduce micro-op is launched. */
moe_status moe_comm_hold(moe_comm *c, int32_t on);

/* While on != 0 the scheduler thread launches nothing at all (micro-ops already on the link
 * finish): lets a caller hand over a batch of operations whose order on the link then
 * depends on the policy alone. */
moe_status moe_comm_pause(moe_comm *c, int32_t on);

/* Forgets `op` without waiting: its events are recycled once its last micro-op has left the
 * link (all of its micro-ops must have been posted).  The handle is invalid afterwards. */
moe_status moe_comm_release(moe_comm *c, int64_t op);

/*
 * BLOCKS until every micro-op of `op` has left the link (posting all of them is the
 * caller's duty; at most timeout_ms), then forgets the operation.  gpu_ms (nullable)
 * receives the time on the device from the moment the operation's first posted micro-op
 * was ready to the end of its last micro-op -- the operation's completion time as the
 * paper measures it.
 */
moe_status moe_comm_finish(moe_comm *c, int64_t op, int32_t timeout_ms, float *gpu_ms);

/* One entry per micro-op put on the link, in link order, and one per moe_comm_hold call. */
typedef struct {
    int64_t op;          /* -1 for a hold entry */
    int32_t micro;       /* hold entry: the `on` value */
    int32_t kind;        /* moe_comm_kind, or 2 for a hold entry */
    int64_t bytes;
    int64_t ready_seq;   /* position of its post among all posts and holds of this instance */
    int64_t issue_seq;   /* position of its launch in the same count: everything with a
                            smaller number had happened when the thread chose it */
    /* host clock, nanoseconds since moe_comm_create: when it was posted, when the thread
     * launched it, and when the thread saw it finished (0 while it is still on the link) */
    int64_t posted_ns, launched_ns, done_ns;
} moe_comm_record;

/* Copies the newest records (at most cap, oldest first) to `out` (host), returns how many;
 * the instance keeps the last 65536. */
int32_t moe_comm_log(moe_comm *c, moe_comm_record *out, int32_t cap);

/* ------------------------------------------------------------------ padded layer */

/* Bytes of workspace moe_layer_padded needs (0 if the shape is invalid). */
size_t moe_padded_workspace_bytes(const moe_shape *s, int32_t n_micro);

/*
 * The layer of moe_layer_chunked in the padded layout, with both all-to-alls carried over
 * the stand-in link in n_micro micro-ops each (1 <= n_micro <= min(capacity, 64)):
 *   gate, plan, pack into xs (zero rows included)                  -- caller's stream
 *   first all-to-all: micro-op m copies xs -> xr                   -- link
 *   expert FFN of micro-op m on xr -> ys, as soon as m has arrived -- caller's stream
 *   second all-to-all: micro-op m copies ys -> yr                  -- link
 *   combine from yr once the last micro-op is in                   -- caller's stream
 * link = NULL: the micro-ops go to a link of `link_blocks` workgroups owned by the library
 * in a fixed order (first(0), first(1), second(0), first(2), second(1), ...); the call only
 * enqueues.  link != NULL: the micro-ops are submitted to that scheduler as two all-to-all
 * operations and share its link with whatever else was submitted there; the call then
 * blocks while it waits for micro-ops to be launched, and link_blocks is ignored.
 *   expert_idx, gate [T*k], counts [E]: as in moe_layer_chunked
 *   slot_of [T*k]: e*C + rank, -1 if dropped;  src_of [E*C]: written for kept slots only
 *   xs, xr [E*C, d_model] in `dtype`;  ys, yr [E*C, d_model] as moe_expert_ffn's ye (fp16 for
 *   MOE_BF16 layers, fp32 for MOE_F32);  y [T, d_model] fp32
 * Rows of ys / yr at or beyond an expert's min(count, C) are left untouched in ys and
 * copied as they are.  y equals moe_layer_chunked's y bit for bit.
 */
moe_status moe_layer_padded(const moe_shape *s, int32_t n_micro, moe_comm *link,
                            int32_t link_blocks, const void *x, const float *Wgp,
                            const float *gate_bias, int32_t bias_token_stride,
                            const void *W1p, const float *b1, const void *W2p,
                            const float *b2, int32_t *expert_idx, float *gate,
                            int32_t *counts, int32_t *slot_of, int32_t *src_of, void *xs,
                            void *xr, void *ys, void *yr, float *y, void *workspace,
                            void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_COMM_H */
