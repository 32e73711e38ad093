/*
 * libmoe -- backward pass of the one-GPU MoE layer (the training half of the paper:
 * Sec. 2.1's layer is trained, and Sec. 2.2 / Sec. 4 schedule its backward pass).
 *
 * The gradients are the chain rule of the forward definition in moe.h for a loss L whose
 * gradient with respect to the layer output y is given as dy:
 *
 *   dye[slot]  = g[t,j] * dy[t]                 for every kept assignment (t, j)
 *   dgate[t,j] = <ye[slot], dy[t]>              (0 for dropped assignments)
 *   dP         = (dye . W2[e]^T) * act'(P)      P = xe . W1[e]: kept by the forward call
 *                                               below, else recomputed here
 *   dW2[e]     = act(P)^T . dye                 rows of expert e; act(P) kept by the forward
 *                                               call below (fp16, rounded to bf16 as an
 *                                               operand), else recomputed
 *   dW1[e]     = xe^T . dP
 *   dxe        = dP . W1[e]^T
 *   dz[t,:]    = p * (dgfull - <p, dgfull>)     p = softmax of the token's logits,
 *                                               dgfull[e] = dgate[t,j] where e = e(t,j)
 *   dx[t]      = sum_j kept dxe[slot(t,j)] + dz[t,:] . Wg^T
 *   dWg        = x^T . dz
 *
 * Routing (which experts, which slots, what is dropped) is piecewise constant and carries
 * no gradient.  bf16 layers only; no FFN biases; renorm_topk must be 0.  The contractions
 * run on bf16 MFMA with fp32 accumulation: dye, dP and the recomputed act(P) are rounded to
 * bf16 as GEMM operands, every returned gradient is fp32.
 *
 * Conventions as in moe.h: device pointers, enqueue only, caller-owned buffers, status
 * codes, moe_last_error.
 */
#ifndef MOE_TRAIN_H
#define MOE_TRAIN_H

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The forward pass of a training step: moe_layer_chunked with one chunk (same arguments,
 * same outputs bit for bit, no y_act) that also keeps the first expert GEMM's result
 * before the activation, which the backward pass would otherwise compute again.
 *   pre  [moe_max_rows, d_ff] fp16, output: pre[slot,:] = xe[slot,:] W1[e] + b1[e], rounded
 *        from the fp32 accumulator; rows at or beyond offsets[E] are left untouched
 *   hid  [moe_max_rows, d_ff] fp16, output: act(pre) as the second GEMM reads it -- the
 *        hidden activations, which otherwise live in the workspace; same rows
 * bf16 layers only.
 */
moe_status moe_layer_forward_keep(const moe_shape *s, const void *x, const float *Wgp,
                                  const float *gate_bias, int32_t bias_token_stride,
                                  const void *W1p, const float *b1, const void *W2p,
                                  const float *b2, int32_t *expert_idx, float *gate,
                                  int32_t *counts, int32_t *offsets, int32_t *slot_of,
                                  int32_t *src_of, void *xe, void *ye, void *pre, void *hid,
                                  float *y, void *workspace, void *stream);

/* Bytes of workspace moe_layer_backward needs for this shape (0 if unsupported). */
size_t moe_backward_workspace_bytes(const moe_shape *s);

/*
 * All gradients of one layer.
 *   forward inputs   x [T,d]; Wgp the packed gate matrix of moe_pack_gate; gate_bias,
 *                    bias_token_stride as given to moe_route; W1 [E,d,h], W2 [E,h,d] in their
 *                    canonical layouts; W1p the packed W1 of moe_pack_weights
 *   forward outputs  expert_idx, gate, offsets, slot_of, src_of, xe, ye exactly as the
 *                    forward call left them
 *   pre, hid         both NULL, or the buffers moe_layer_forward_keep filled in that forward call
 *                    (the backward pass of a layer with FFN biases is not supported either way)
 *   dy               [T,d] fp32
 *   dx [T,d], dWg [d,E], dW1 [E,d,h], dW2 [E,h,d], dgate [T*k]: fp32, overwritten (weight
 *                    gradients of an expert without rows are zero)
 */
moe_status moe_layer_backward(const moe_shape *s, const void *x, const void *Wgp,
                              const float *gate_bias, int32_t bias_token_stride,
                              const void *W1, const void *W2, const void *W1p,
                              const int32_t *expert_idx, const float *gate,
                              const int32_t *offsets, const int32_t *slot_of,
                              const int32_t *src_of, const void *xe, const void *ye,
                              const void *pre, const void *hid, const float *dy, float *dx,
                              float *dWg, float *dW1, float *dW2, float *dgate, void *workspace,
                              void *stream);

/* moe_layer_backward with the token stream cut into n_chunks contiguous parts (1..64), the
 * backward pass's counterpart of moe_layer_chunked (Sec. 2.2: the backward pass has two
 * all-to-alls of its own; Sec. 4.2: they are cut into micro-ops along the token dimension).
 * Gradient rows are dispatched to the expert-major order chunk by chunk on a side stream, the
 * two input-gradient GEMMs run once per group of consecutive chunks (the same grouping rule as
 * the forward's FFN launches, moe_tune_ffn_group_rows) as soon as the group's last chunk is
 * there, and the rows that come back are folded into dx chunk by chunk on a second side
 * stream while the caller's stream goes on with the next group and the weight gradients.
 * Every gradient is the same bits for every n_chunks.  With one group the call runs as
 * n_chunks = 1.  Side streams and events are created on the first chunked call on a device. */
moe_status moe_layer_backward_chunked(const moe_shape *s, int32_t n_chunks, const void *x,
                                      const void *Wgp, const float *gate_bias,
                                      int32_t bias_token_stride, const void *W1, const void *W2,
                                      const void *W1p, const int32_t *expert_idx,
                                      const float *gate, const int32_t *offsets,
                                      const int32_t *slot_of, const int32_t *src_of,
                                      const void *xe, const void *ye, const void *pre,
                                      const void *hid, const float *dy, float *dx, float *dWg,
                                      float *dW1, float *dW2, float *dgate, void *workspace,
                                      void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_TRAIN_H */
