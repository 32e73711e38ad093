/*
 * libmoe -- expert FFN with the expert weights resident in host memory.
 *
 * The paper keeps expert parameters that are not in use in host DRAM when GPU memory is
 * short (Sec. 4.2, end of "Expert packing": DRAM-offloading) and, in inference, has a
 * device that hosts several experts load them one at a time, compute, and move on to the
 * next packed expert (Sec. 6.2, "Expert packing"; "Resource scheduler": every device
 * keeps the weights of all experts in its host DRAM).  moe_expert_ffn_offloaded is that
 * execution order on one GPU: experts are processed in index order; at most `resident`
 * experts' weights are on the device at a time; the copy of the next expert's weights
 * runs on its own stream while the current expert is computed.
 *
 * The result is the one moe_expert_ffn gives for the same packed weights, bit for bit
 * (same kernels, same tiles; only the order of the experts' launches differs).
 *
 * Conventions as in moe.h, except where a pointer is marked "host".
 */
#ifndef MOE_OFFLOAD_H
#define MOE_OFFLOAD_H

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Device bytes of the staging area for `resident` expert slots (0 if unsupported or
 * resident < 1).  resident >= 2 lets copy and compute overlap. */
size_t moe_offload_staging_bytes(const moe_shape *s, int32_t resident);

/* Device bytes of workspace (per-expert work lists and the hidden activations). */
size_t moe_offload_workspace_bytes(const moe_shape *s);

/*
 * ye[r, :] = act(xe[r, :] . W1[e] + b1[e]) . W2[e] + b2[e] for the rows of every expert e,
 * as moe_expert_ffn, with
 *   W1p_host, W2p_host  host: the packed weights of moe_pack_weights (moe_packed_weight_bytes
 *                       each), in page-locked host memory so that the copies are asynchronous;
 *                       they must stay unchanged until the enqueued work has finished
 *   staging             device, moe_offload_staging_bytes(s, resident)
 *   workspace           device, moe_offload_workspace_bytes(s)
 * bf16 layers.  Creates, once per process and device, one copy stream and 2 * 64 events.
 * Overlapping calls that share a staging area race.
 */
moe_status moe_expert_ffn_offloaded(const moe_shape *s, const void *xe, const int32_t *offsets,
                                    const void *W1p_host, const void *W2p_host, const float *b1,
                                    const float *b2, void *ye, void *staging, int32_t resident,
                                    void *workspace, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_OFFLOAD_H */
