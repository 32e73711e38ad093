/*
 * libmoe -- one-GPU forward pass of a Mixture-of-Experts layer for AMD gfx950.
 *
 * The layer is the one the paper states in Sec. 2.1: a gating network multiplies
 * every token embedding by its trainable matrix and sends the token to its top-k
 * experts; each expert is a two-layer fully connected network; the output is the
 * gate-weighted sum of the selected experts' outputs.  Between gate and experts
 * the tokens are packed into an expert-major buffer, and unpacked afterwards:
 * these are the payloads of the two all-to-all exchanges of expert parallelism
 * (end of Sec. 2.1, Sec. 2.2), here built for one GPU's share with no network.
 * moe_layer_chunked splits the token stream into equal parts and overlaps the
 * packing of part i+1 with the expert computation of part i, the one-GPU analogue
 * of the paper's all-to-all micro-ops pipelined with the expert FFN (Sec. 4.2,
 * "Pipelining micro-ops"; Sec. 6.1).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers unless a comment says "host".
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Calls only enqueue work; they never synchronise the host with the device,
 *     never allocate or free device memory, and never copy results to the host.
 *   - The caller owns every buffer, including `workspace`
 *     (size from moe_workspace_bytes), and keeps it alive until the enqueued
 *     work has finished.  Buffers must be 16-byte aligned and must not overlap.
 *   - Matrices are row-major and dense.  Row lengths in bytes (d_model, d_ff
 *     times the element size) must be multiples of 16.
 *   - Return value: MOE_OK, or an error code; moe_last_error() then describes the
 *     problem (thread-local string).  Argument errors (MOE_EINVAL,
 *     MOE_EUNSUPPORTED) are found before anything is enqueued.  MOE_EHIP means a
 *     HIP runtime call failed part-way: work enqueued before it stays enqueued,
 *     the library's side streams are joined back into `stream` before the call
 *     returns, and the outputs are unspecified.
 *     No C++ exception crosses this boundary.
 *   - Threads: any host thread may call any entry point.  Calls that use the
 *     library's own side streams on one device (moe_layer_chunked with
 *     n_chunks > 1) take a per-device lock for the time they enqueue, so two
 *     threads' calls do not interleave on those streams; their work then runs
 *     one call after the other.  Two calls that write the same buffers race as
 *     any two writers do.  The measurement aid at the end of this file is the
 *     exception: one thread, no call in progress.
 *   - Inputs are assumed finite.
 *
 * Element types.  `dtype` is the storage type of x, Wg, W1, W2, xe.  Gate logits,
 * softmax and gate weights are fp32.  MOE_BF16 layers: the hidden activations and
 * the expert outputs ye are stored in fp16 (the payload of the second all-to-all is
 * then two bytes per element, as the first one's); the weighted sum over the selected
 * experts is accumulated in fp32 and the layer output y is fp32 (a 16-bit y would
 * spend the whole error budget on its own rounding of the largest elements).
 * MOE_F32 layers: everything fp32.
 */
#ifndef MOE_H
#define MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_EINVAL = 1,       /* null / misaligned pointer, inconsistent sizes */
    MOE_EUNSUPPORTED = 2, /* a size or option outside what the kernels handle */
    MOE_EWORKSPACE = 3,   /* reserved */
    MOE_EHIP = 4          /* a HIP runtime call failed */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

typedef enum {
    MOE_ACT_GELU_ERF = 0, /* 0.5 v (1 + erf(v / sqrt 2)) */
    MOE_ACT_GELU_TANH = 1,
    MOE_ACT_RELU = 2,     /* the activation the paper names in Sec. 2.1 */
    MOE_ACT_IDENTITY = 3
} moe_act;

/* Shape of one layer.  T tokens, E experts (1..64), k experts per token
 * (1..min(E,8)), capacity = slots per expert (>= 1; pass T for "never drop"). */
typedef struct {
    int32_t T;
    int32_t d_model;
    int32_t E;
    int32_t d_ff;
    int32_t k;
    int32_t capacity;
    int32_t dtype;       /* moe_dtype */
    int32_t act;         /* moe_act */
    int32_t renorm_topk; /* 0: gate weight = softmax probability;
                            1: divided by the sum over the k selected experts */
} moe_shape;

/* Host, pure.  ceil(cf * k * T / E) evaluated in double; cf <= 0 returns T. */
int64_t moe_capacity(int32_t T, int32_t E, int32_t k, double cf);

/* Host, pure.  Upper bound of kept assignments: min(T*k, E*capacity).
 * xe, ye and src_of must hold this many rows / entries. */
int64_t moe_max_rows(const moe_shape *s);

/* Host, pure.  Bytes of `workspace` the calls below need for this shape and up to
 * n_chunks chunks (the same buffer serves all of them).  0 on an invalid shape. */
size_t moe_workspace_bytes(const moe_shape *s, int32_t n_chunks);

/* Host.  Description of the last error on the calling thread ("" if none). */
const char *moe_last_error(void);

/* Host, pure.  Bytes of each packed weight buffer (W1p and W2p have equal size). */
size_t moe_packed_weight_bytes(const moe_shape *s);

/* One-time re-layout of the expert weights for the FFN kernels (like loading a
 * checkpoint; not part of the timed path).
 *   W1 [E, d_model, d_ff], W2 [E, d_ff, d_model]: canonical layout, `dtype`.
 *   W1p, W2p: moe_packed_weight_bytes each.
 * MOE_BF16: W1p = bf16 [E, d_ff, d_model] (each expert transposed so that the
 * contraction index is contiguous); W2p = fp16 [E, d_model, d_ff].  The hidden
 * activations are held in fp16 (three more mantissa bits than bf16 at the same
 * matrix-core rate); every bf16 weight of magnitude in [2^-17, 65504] converts
 * exactly, smaller ones round to the nearest multiple of 2^-24.
 * MOE_F32: plain copies. */
moe_status moe_pack_weights(const moe_shape *s, const void *W1, const void *W2,
                            void *W1p, void *W2p, void *stream);

/* Host, pure.  Bytes of the packed gate matrix. */
size_t moe_packed_gate_bytes(const moe_shape *s);

/* One-time re-layout of the gating network's matrix (Sec. 2.1: "its trainable
 * matrix"): Wg [d_model, E] in `dtype` -> Wgp fp32 [EP][dP], expert-major:
 * Wgp[e*dP + i] = Wg[i, e], EP = E rounded up to a power of two, dP = d_model
 * rounded up to a multiple of 128, zeros elsewhere (moe_packed_gate_bytes =
 * EP*dP*4).  Every bf16 value converts exactly.  Treat the buffer as opaque:
 * build it with this call, not by hand. */
moe_status moe_pack_gate(const moe_shape *s, const void *Wg, float *Wgp, void *stream);

/* Gate (Sec. 2.1).  z[t,e] = sum_i x[t,i] Wg[i,e] accumulated in fp32 in
 * ascending i with fused multiply-adds, then + gate_bias.  The k experts of a
 * token are its k largest logits (in order of decreasing logit, ties: lower index
 * first); gate[t,j] = softmax(z[t,:])[expert j] (optionally renormalised).
 *   x [T, d_model] in `dtype`; Wgp from moe_pack_gate.
 *   gate_bias: NULL, or fp32 [E] (bias_token_stride 0) or [T,E] (stride E).
 *   expert_idx int32 [T*k], gate fp32 [T*k]: outputs. */
moe_status moe_route(const moe_shape *s, const void *x, const float *Wgp,
                     const float *gate_bias, int32_t bias_token_stride,
                     int32_t *expert_idx, float *gate, void *stream);

/* Dispatch = pack for the first all-to-all (end of Sec. 2.1).  Assignment
 * i = t*k + j is kept iff fewer than `capacity` assignments with a smaller i chose
 * the same expert; kept assignments of expert e fill slots
 * [offsets[e], offsets[e+1]) in ascending i.
 * An expert_idx entry outside [0, E) names no expert (a padding marker): that
 * assignment is in no count, takes no slot, and gets slot_of = -1.
 *   counts int32 [E]: assignments per expert before the capacity bound.
 *   offsets int32 [E+1]: exclusive scan of min(counts, capacity).
 *   slot_of int32 [T*k]: slot of assignment i, -1 if dropped.
 *   src_of int32 [moe_max_rows]: assignment held by each slot < offsets[E].
 *   xe [moe_max_rows, d_model] `dtype`: xe[slot,:] = x[t,:]; rows at or beyond
 *   offsets[E] are left untouched. */
moe_status moe_dispatch(const moe_shape *s, const void *x, const int32_t *expert_idx,
                        int32_t *counts, int32_t *offsets, int32_t *slot_of,
                        int32_t *src_of, void *xe, void *workspace, void *stream);

/* moe_dispatch for callers that cannot allocate device memory or have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and results as moe_dispatch
 * minus `workspace`; the plan's scratch (256 bytes per plan segment; a segment
 * is 4 to 64 tokens by shape) lives in an array of
 * moe_dispatch_static_limit() = 4 MiB inside the library's device image, which
 * every GPU the library runs on holds until the process ends.  The call
 * allocates and frees nothing (its first call on a device looks the array's
 * address up once).  A shape whose plan needs more scratch than the array holds
 * is refused with MOE_EUNSUPPORTED before anything is enqueued.  All calls on
 * one GPU share that GPU's array, whatever their stream or thread: two calls
 * whose work overlaps in time on one GPU race on it; serialise them (one
 * stream, or events).  Nothing in the array has to start at zero: every call
 * overwrites the part it reads. */
size_t moe_dispatch_static_limit(void);
moe_status moe_dispatch_static(const moe_shape *s, const void *x,
                               const int32_t *expert_idx, int32_t *counts,
                               int32_t *offsets, int32_t *slot_of, int32_t *src_of,
                               void *xe, void *stream);

/* Expert FFN (Sec. 2.1): for slot r of expert e,
 *   ye[r,:] = act(xe[r,:] W1[e] + b1[e]) W2[e] + b2[e].
 *   W1p, W2p from moe_pack_weights; b1 fp32 [E,d_ff] and b2 fp32 [E,d_model] may
 *   be NULL; ye [moe_max_rows, d_model], fp16 for MOE_BF16 layers and fp32 for MOE_F32
 *   layers.  Experts with no rows read no weights.  Rows at or beyond offsets[E] are
 *   left untouched. */
moe_status moe_expert_ffn(const moe_shape *s, const void *xe, const int32_t *offsets,
                          const void *W1p, const float *b1, const void *W2p,
                          const float *b2, void *ye, void *workspace, void *stream);

/* Combine = unpack after the second all-to-all (Sec. 2.2, forward-pass timeline):
 *   y[t,:] = sum over kept j of gate[t,j] * ye[slot_of[t*k+j],:]  (fp32, ascending j),
 * zero for a token with no kept assignment.
 *   ye as moe_expert_ffn writes it (fp16 / fp32 by dtype); y fp32 [T, d_model].  y_act: NULL, or [T, d_model] in `dtype` receiving y
 *   rounded to nearest-even (the next layer's input in a stack). */
moe_status moe_combine(const moe_shape *s, const void *ye, const int32_t *slot_of,
                       const float *gate, float *y, void *y_act, void *stream);

/* The whole layer with the token stream cut into n_chunks contiguous parts
 * (chunk c = tokens [floor(c*T/n), floor((c+1)*T/n)); 1 <= n_chunks <= 64).
 * Routing and the dispatch plan are computed once over all T tokens, so every
 * output is identical for every n_chunks (Sec. 7.1: the scheduling does not change
 * what is computed).  Packing of chunk c+1 and unpacking of chunk c-1 run on side
 * streams concurrently with the expert FFN of chunk c (Sec. 4.2).  In MOE_BF16 layers
 * the first expert GEMM reads its rows straight from x through src_of (the tokens are
 * already in this GPU's memory), so no FFN launch waits for the pack: xe, the payload
 * the first all-to-all would carry, is written beside it -- also when n_chunks = 1.
 * The expert FFN runs once per GROUP of consecutive chunks: every FFN launch streams
 * all experts' weights from HBM once, so a launch is given at least
 * moe_tune_ffn_group_rows() (default 2048) rows per expert on average --
 * groups = min(n_chunks, (moe_max_rows / E) / that), at least 1; packing and unpacking
 * keep n_chunks.  With one group the call runs as n_chunks = 1.
 * Arguments as in the calls above; all outputs are written.  The side streams
 * and events are created on the first chunked call on a device and kept. */
moe_status moe_layer_chunked(const moe_shape *s, int32_t n_chunks, const void *x,
                             const float *Wgp, const float *gate_bias,
                             int32_t bias_token_stride, const void *W1p,
                             const float *b1, const void *W2p, const float *b2,
                             int32_t *expert_idx, float *gate, int32_t *counts,
                             int32_t *offsets, int32_t *slot_of, int32_t *src_of,
                             void *xe, void *ye, float *y, void *y_act,
                             void *workspace, void *stream);

/* Tuning knob, process-wide: the average rows per expert an FFN launch of a chunked
 * layer must hold (see moe_layer_chunked).  rows >= 1 sets it; any other value only
 * reads.  Returns the value before the call.  1 gives one FFN launch per chunk. */
int32_t moe_tune_ffn_group_rows(int32_t rows);

/* Measurement aid, off by default (not part of the layer).  Stage numbers:
 * 0 gate, 1 dispatch plan, 2 row-tile table, 3 pack (scatter), 4 first expert GEMM
 * (+ activation), 5 second expert GEMM, 6 combine; backward pass (moe_train.h): 7 recomputed
 * pre-activation GEMM, 8 hidden-gradient GEMM, 9 input-gradient GEMM, 10 and 11 the weight
 * gradient GEMMs of the second and first layer, 12 all its other kernels together.
 * An unchunked layer (and moe_dispatch) whose plan fits one launch packs the rows in
 * that launch: stage 3 then records nothing and stage 1 covers both.
 * moe_profile_enable: for every stage whose bit is set in stage_mask, the next
 * max_samples launches of that stage are bracketed by a pair of timing events
 * recorded on the stream the stage runs on.  (0, 0) switches it off and frees the
 * events.  Host; creates events; not thread-safe; call it while no libmoe call is
 * in progress.
 * moe_profile_read: waits for the recorded events of `stage`, writes the elapsed
 * milliseconds of each bracket to ms[0..n) (host pointer, -1 where a read failed),
 * returns n <= cap and forgets the samples. */
moe_status moe_profile_enable(uint32_t stage_mask, int32_t max_samples);
int32_t moe_profile_read(int32_t stage, float *ms, int32_t cap);

/* Calibration of the two roofs the measurements are quoted against (measurement aid,
 * not part of the layer; the caller times the calls with events on `stream`).
 * moe_calib_copy: dst[0..bytes) = src[0..bytes) by a plain copy kernel (16 bytes per
 *   lane and step); bytes and both pointers multiples of 16.  Reads `bytes` and writes
 *   `bytes`: the HBM rate it reaches on buffers far larger than the caches is the
 *   measured memory roof, and its reading under the profiler's FETCH_SIZE / WRITE_SIZE
 *   counters fixes their unit.
 * moe_calib_mfma: 256 x waves_per_simd blocks of four wavefronts, each wavefront
 *   issuing iters x 8 independent 32x32x16 bf16 matrix instructions on register
 *   operands (random_operands != 0: operand bits differ per lane; 0: all ones, which
 *   draws less power and holds a higher clock).  sink: fp32 [256*waves_per_simd*256].
 *   moe_calib_mfma_flops gives the launch's floating-point operations.
 * moe_calib_gemm: the 256 x 256 expert-GEMM kernel alone, on operands and a work list
 *   the caller makes: A bf16 [rows, K], W bf16 [E, N, K], C fp16 [rows, N] (written),
 *   items int32 [max_items][4] = {expert, row0, row1, first column} with row1 - row0 in
 *   1..256 and the first column a multiple of 256, *n_items <= max_items (device).
 *   variant 0 is the kernel as the layer runs it; other variants leave parts of it out to
 *   show what each costs (bit 0: no matrix instructions; bit 1: no LDS fragment reads
 *   after the first step; bit 2: no global loads and LDS writes in the loop; bit 3: no
 *   output stores; built: 0, 1, 2, 4, 6, 7, 8) -- their outputs are wrong by
 *   construction.  K a multiple of 64, N * K * 2 and 256 * K * 2 below 2^31.
 * moe_expert_gemm_kernel: which kernel an unchunked bf16 layer of shape s launches for its
 *   expert GEMM `which` (0: first, xe W1; 1: second, H W2), written to name (host, len
 *   bytes, always terminated) as "<kernel> <tile rows>x<tile columns>", so that a
 *   measurement can say which kernel it timed.  MOE_EINVAL for which outside {0, 1}, a
 *   null name or len == 0, an unsupported shape or an fp32 layer (one kernel there). */
moe_status moe_expert_gemm_kernel(const moe_shape *s, int32_t which, char *name, size_t len);
moe_status moe_calib_copy(void *dst, const void *src, size_t bytes, void *stream);
moe_status moe_calib_gemm(const void *A, const void *W, void *C, const int32_t *items,
                          const int32_t *n_items, int32_t max_items, int32_t N, int32_t K,
                          int32_t variant, int32_t gelu, void *stream);
moe_status moe_calib_mfma(float *sink, int32_t waves_per_simd, int32_t iters,
                          int32_t random_operands, void *stream);
double moe_calib_mfma_flops(int32_t waves_per_simd, int32_t iters);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H */
