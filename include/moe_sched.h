/*
 * libmoe -- popularity-based expert scheduling for MoE inference (paper Sec. 5.2,
 * "Popularity based Scheduling"; Sec. 6.2, "Resource scheduler").
 *
 * The paper observes that a token's expert choices in consecutive MoE layers follow a
 * pattern, profiles it offline, and uses it to estimate -- before a layer's gate has
 * run -- how popular each expert of that layer will be for the batch at hand, so that
 * popular experts can be replicated and unpopular ones packed onto shared devices:
 *
 *   profiling   tokens are grouped by their sample path j, the experts they selected in
 *               the last l layers; per path the distribution Psi_j of the experts
 *               selected in the NEXT layer is recorded      (moe_path_profile,
 *               moe_path_finalize)
 *   estimate    for a batch, every token contributes the probabilities of the top-k
 *               experts of its path's distribution; the sum over the batch divided by
 *               the batch size is the estimated popularity  (moe_popularity_estimate)
 *   Eq. (1)     n_e = N * estimated popularity of e = devices expert e should get
 *               (moe_devices_for_expert)
 *   phase 1     experts are replicated / packed first-fit-decreasing onto the N devices
 *               (moe_schedule_experts)
 *   phase 2     once the gate has selected, the overall top-2k experts of estimate and
 *               actual selection are compared; if the lists differ the schedule is
 *               recomputed from the actual popularity      (moe_top_lists_identical,
 *               moe_schedule_layer)
 *
 * Selections.  sel[i][t][j] (int32) is the j-th choice of token t in MoE layer i, j = 0
 * the first choice -- the expert_idx output of moe_route, one layer after the other.
 * The sample path of a token ending at layer i is the l first choices of layers
 * i-l+1 .. i, read as an l-digit number in base E, oldest layer first; with k > 1 the
 * path follows the first choice only (the paper's inference runs use k = 1), while all k
 * choices of the next layer count in Psi.
 *
 * Exact arithmetic.  Probabilities are held in 2^-32 fixed point,
 * floor(count * 2^32 / row total), and summed in 64-bit integers, so an estimate does not
 * depend on the order in which tokens are added, and every decision taken from it
 * (rankings, packing) is an integer decision.  A path's row total must stay below 2^32.
 *
 * Device calls follow the conventions of moe.h (device pointers, enqueue only, caller
 * owns all buffers, status codes, moe_last_error).  Calls marked "host" take host
 * pointers, run on the calling thread and touch no GPU.
 */
#ifndef MOE_SCHED_H
#define MOE_SCHED_H

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t L; /* MoE layers in the model (profiling needs L > l) */
    int32_t E; /* experts per layer, 1 .. 64 */
    int32_t k; /* experts selected per token, 1 .. min(E, 8) */
    int32_t l; /* sample-path length (Sec. 7.1 uses 3) */
} moe_path_shape;

/* host.  Number of sample paths E^l, or 0 if the shape is invalid or E^l > 2^24. */
int64_t moe_path_count(const moe_path_shape *s);

/*
 * Profiling stage (Sec. 5.2, "Estimating expert popularity"): adds the selections of T
 * profiled tokens to the tables.  For every layer i = l-1 .. L-2 and token t,
 * counts[i-(l-1)][path(t, i)][sel[i+1][t][j]] += 1 for j < k.
 *   sel     [L][T][k] int32; a token with an expert outside [0, E) in a layer is skipped
 *           for the tables that layer takes part in
 *   counts  [(L-l)][E^l][E] uint32, accumulated (the caller zeroes it before the first
 *           batch); several calls add up
 */
moe_status moe_path_profile(const moe_path_shape *s, const int32_t *sel, int32_t T,
                            uint32_t *counts, void *stream);

/*
 * Turns the counts into what the estimate looks up: per layer and path the top-k experts
 * of Psi_j (largest count first, ties to the lower index, experts with count 0 not listed)
 * and their probabilities in 2^-32 fixed point.
 *   top_expert  [(L-l)][E^l][k] int32, -1 where nothing is listed
 *   top_prob    [(L-l)][E^l][k] uint64, 0 where nothing is listed
 */
moe_status moe_path_finalize(const moe_path_shape *s, const uint32_t *counts,
                             int32_t *top_expert, uint64_t *top_prob, void *stream);

/*
 * Estimate for one layer and one batch (the sum of Eq. (1) before the division by N_t):
 * S[e] = sum over the batch's tokens of P_{j(t)}(e), 2^-32 fixed point.
 *   sel_hist    [l][N_t][k] int32: the batch's selections in the l layers before the one
 *               estimated (oldest first); tokens with an invalid expert contribute nothing
 *   top_expert, top_prob   the [E^l][k] slices of that layer from moe_path_finalize
 *   S           [E] uint64, overwritten.  Expert e is in some token's top-k list iff
 *               S[e] > 0.
 */
moe_status moe_popularity_estimate(const moe_path_shape *s, const int32_t *sel_hist,
                                   int32_t N_t, const int32_t *top_expert,
                                   const uint64_t *top_prob, uint64_t *S, void *stream);

/* host.  Eq. (1): n_e = N * (S_e / 2^32) / N_t. */
double moe_devices_for_expert(uint64_t S_e, int32_t N_t, int32_t N);

/*
 * host.  Phase-1 scheduling from integer weights: expert e should get w[e] / W devices
 * (w = N * S, W = N_t * 2^32 for the estimate; w = N * count, W = N_t * k for the actual
 * popularity).  What the paper leaves open is fixed as follows:
 *   - an expert with w >= W is replicated on round-half-up(w / W) devices of its own
 *     (at most N);
 *   - the others are packed first-fit-decreasing (weight descending, then expert index)
 *     into devices of capacity W holding at most max_pack experts (Sec. 7.1: 4);
 *   - experts with has[e] == 0 (no estimate) go round-robin, in index order, onto the
 *     devices left free; if none is free expert e goes to device e mod N (deterministic
 *     stand-in for the paper's random choice);
 *   - if more than N devices are asked for, device numbers wrap modulo N.
 *   replicas     [E]   devices hosting e (>= 1 for every expert on return)
 *   dev_count    [N]   experts hosted by device d
 *   dev_experts  [N*E] row d holds dev_count[d] expert ids, then -1
 *   devices_used       devices that host estimated experts (at most N)
 * Requires N >= 1, 1 <= E <= 64, W >= 1, max_pack >= 1 and N * max(w) below 2^63.
 */
moe_status moe_schedule_experts(int32_t N, int32_t E, const uint64_t *w, uint64_t W,
                                const uint8_t *has, int32_t max_pack, int32_t *replicas,
                                int32_t *dev_count, int32_t *dev_experts,
                                int32_t *devices_used);

/* host.  Phase-2 check: 1 if the 2k most popular experts by S and by counts are the same
 * list (same experts in the same order; ties rank the lower index first), else 0. */
int32_t moe_top_lists_identical(int32_t E, int32_t k, const uint64_t *S, const int32_t *counts);

/*
 * host.  Both phases for one layer: schedules from the estimate S; if the top-2k lists of
 * S and of the gate's histogram `counts` differ, schedules again from the actual
 * popularity.  Outputs as for moe_schedule_experts, for the schedule that stands at the
 * end; *rescheduled is 1 if phase 2 recomputed it.
 */
moe_status moe_schedule_layer(int32_t N, int32_t E, int32_t k, int32_t N_t, const uint64_t *S,
                              const int32_t *counts, int32_t max_pack, int32_t *replicas,
                              int32_t *dev_count, int32_t *dev_experts, int32_t *devices_used,
                              int32_t *rescheduled);

#ifdef __cplusplus
}
#endif
#endif /* MOE_SCHED_H */
