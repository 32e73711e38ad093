/*
 * CPU oracle of the MoE-layer forward pass -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-pass statement of what the layer computes, used by the
 * tests, the smoke check and the benchmark's cpu_baseline leg.  It shares no
 * code with the GPU library and must never be called from the product path.
 *
 * The layer (paper Sec. 2.1): a gating network multiplies each token embedding
 * by its trainable matrix and sends the token to a small number of experts;
 * every expert is a two-layer fully connected network; the layer's output is
 * the weighted sum of the selected experts' outputs.  Tokens are first moved
 * into an expert-major buffer (the payload of the first all-to-all, end of
 * Sec. 2.1 and Sec. 2.2) and moved back afterwards (the second all-to-all, then
 * "combine": Sec. 2.2 and the caption of its forward-pass timeline figure).
 *
 * Arithmetic: gate logits in fp32 with one accumulator walked over the model
 * dimension in ascending order (fused multiply-add), because the top-k decision
 * is an integer result that both sides must take in the same precision.
 * Everything else that is floating point accumulates in fp64.
 *
 * All arrays are host arrays, row-major, float unless stated.
 * Parity status: every function here is pinned by tests/test_oracle_*.py
 * against closed forms, invariants, brute force or a library routine.
 * Absolute y values on the five benchmark configurations have no external
 * reference (the paper prints no worked example): they are pinned only through
 * the dense special case plus the invariants.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the parallel loops below will use. */
int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

enum { ACT_GELU_ERF = 0, ACT_GELU_TANH = 1, ACT_RELU = 2, ACT_IDENTITY = 3 };

/* Gate logits, Sec. 2.1 ("multiplies them with its trainable matrix").
 * z[t,e] = (((0 + x[t,0]*Wg[0,e]) + x[t,1]*Wg[1,e]) + ...) + bias, each step one
 * fp32 fused multiply-add; the bias is added last with one fp32 addition.
 * bias may be NULL; bias_stride is 0 (one bias row for all tokens) or E. */
void oracle_gate_logits(const float *x, const float *Wg, const float *bias,
                        int bias_stride, int T, int d, int E, float *z)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            float acc = 0.0f;
            for (int i = 0; i < d; ++i)
                acc = fmaf(x[(size_t)t * d + i], Wg[(size_t)i * E + e], acc);
            if (bias)
                acc = acc + bias[(size_t)t * bias_stride + e];
            z[(size_t)t * E + e] = acc;
        }
    }
}

/* Expert selection and gate weights, Sec. 2.1 ("dispatches the token to a small
 * number of experts ... weighted sum").  The k experts of a token are its k
 * largest logits, ties going to the lower expert index; the weight of a selected
 * expert is its softmax probability over all E experts (fp64 evaluation, stored
 * fp32).  With renorm != 0 the k weights are divided by their sum. */
void oracle_topk_softmax(const float *z, int T, int E, int k, int renorm,
                         int32_t *expert_idx, float *gate)
{
    for (int t = 0; t < T; ++t) {
        const float *zt = z + (size_t)t * E;
        int32_t *sel = expert_idx + (size_t)t * k;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                int taken = 0;
                for (int jj = 0; jj < j; ++jj)
                    if (sel[jj] == e) taken = 1;
                if (taken) continue;
                if (best < 0 || zt[e] > zt[best]) best = e;
            }
            sel[j] = best;
        }
        double zmax = zt[0];
        for (int e = 1; e < E; ++e)
            if (zt[e] > zmax) zmax = zt[e];
        double denom = 0.0;
        for (int e = 0; e < E; ++e) denom += exp((double)zt[e] - zmax);
        double gsum = 0.0;
        double g[64];
        for (int j = 0; j < k; ++j) {
            g[j] = exp((double)zt[sel[j]] - zmax) / denom;
            gsum += g[j];
        }
        for (int j = 0; j < k; ++j)
            gate[(size_t)t * k + j] = (float)(renorm ? g[j] / gsum : g[j]);
    }
}

/* Slots per expert for a capacity factor cf: the smallest integer that is not
 * below cf*k*T/E, the product and the quotient evaluated in double from left to
 * right (the paper names no capacity; this is the usual rule of the MoE layer
 * it builds on, Sec. 2.1, and the benchmark configurations are stated by cf). */
int64_t oracle_capacity(int T, int E, int k, double cf)
{
    return (int64_t)ceil(cf * (double)k * (double)T / (double)E);
}

/* Dispatch plan: per-expert histogram, token-order rank, capacity bound,
 * exclusive scan, slot of every assignment.  Flat assignment index i = t*k + j;
 * an assignment is kept iff fewer than C earlier assignments (smaller i) chose
 * the same expert.  Kept rows of expert e occupy slots [off[e], off[e+1]) in
 * ascending i.  slot_of[i] = -1 for dropped assignments; src_of[slot] = i.
 * An index outside [0, E) names no expert (a padding marker): that assignment is
 * dispatched nowhere -- it is in no count, takes no slot, and has slot_of = -1.
 * Returns A = off[E], the number of kept assignments. */
int oracle_plan(const int32_t *expert_idx, int T, int k, int E, int C,
                int32_t *count, int32_t *off, int32_t *slot_of, int32_t *src_of)
{
    int n = T * k;
    for (int e = 0; e < E; ++e) count[e] = 0;
    for (int i = 0; i < n; ++i)
        if (expert_idx[i] >= 0 && expert_idx[i] < E) count[expert_idx[i]] += 1;
    off[0] = 0;
    for (int e = 0; e < E; ++e)
        off[e + 1] = off[e] + (count[e] < C ? count[e] : C);
    int32_t *run = (int32_t *)calloc(64, sizeof(int32_t));
    for (int i = 0; i < n; ++i) {
        int e = expert_idx[i];
        if (e < 0 || e >= E) {
            slot_of[i] = -1;
            continue;
        }
        int pos = run[e];
        run[e] += 1;
        if (pos < C) {
            slot_of[i] = off[e] + pos;
            src_of[off[e] + pos] = i;
        } else {
            slot_of[i] = -1;
        }
    }
    free(run);
    return off[E];
}

/* Pack: xe[slot,:] = x[t,:] for every kept assignment (first all-to-all payload). */
void oracle_scatter(const float *x, const int32_t *slot_of, int T, int k, int d,
                    float *xe)
{
    for (int i = 0; i < T * k; ++i) {
        if (slot_of[i] < 0) continue;
        memcpy(xe + (size_t)slot_of[i] * d, x + (size_t)(i / k) * d,
               (size_t)d * sizeof(float));
    }
}

static double act_fn(double v, int act)
{
    switch (act) {
    case ACT_GELU_ERF:
        return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));
    case ACT_GELU_TANH:
        return 0.5 * v * (1.0 + tanh(sqrt(2.0 / M_PI) * (v + 0.044715 * v * v * v)));
    case ACT_RELU:
        return v > 0.0 ? v : 0.0;
    default:
        return v;
    }
}

double oracle_act(double v, int act) { return act_fn(v, act); }

/* Expert FFN on a list of slot rows (Sec. 2.1: two-layer fully connected expert;
 * Sec. 4.2: the FFN works per token, so any subset of rows stands alone).
 * For row r owned by expert e (off[e] <= r < off[e+1]):
 *   H = act(xe[r,:] . W1[e] + b1[e]),  ye[r,:] = H . W2[e] + b2[e]
 * W1 is [E,d,h], W2 is [E,h,d]; b1 [E,h] and b2 [E,d] may be NULL.
 * All sums in fp64, nothing rounded in between.  ye_rows[q,:] (double) receives
 * the output of rows[q]. */
void oracle_ffn_rows(const float *xe, const int32_t *off, int E, int d, int h,
                     const float *W1, const float *b1, const float *W2,
                     const float *b2, int act, const int32_t *rows, int nrows,
                     double *ye_rows)
{
#pragma omp parallel
    {
        double *hid = (double *)malloc((size_t)h * sizeof(double));
#pragma omp for schedule(dynamic, 4)
        for (int q = 0; q < nrows; ++q) {
            int r = rows[q];
            int e = 0;
            while (e < E && !(off[e] <= r && r < off[e + 1])) ++e;
            double *out = ye_rows + (size_t)q * d;
            if (e == E) { /* row beyond off[E]: not a valid slot */
                for (int c = 0; c < d; ++c) out[c] = NAN;
                continue;
            }
            const float *w1 = W1 + (size_t)e * d * h;
            const float *w2 = W2 + (size_t)e * h * d;
            for (int j = 0; j < h; ++j) hid[j] = b1 ? (double)b1[(size_t)e * h + j] : 0.0;
            for (int i = 0; i < d; ++i) {
                double xv = xe[(size_t)r * d + i];
                const float *w = w1 + (size_t)i * h;
                for (int j = 0; j < h; ++j) hid[j] += xv * (double)w[j];
            }
            for (int j = 0; j < h; ++j) hid[j] = act_fn(hid[j], act);
            for (int c = 0; c < d; ++c) out[c] = b2 ? (double)b2[(size_t)e * d + c] : 0.0;
            for (int j = 0; j < h; ++j) {
                double hv = hid[j];
                const float *w = w2 + (size_t)j * d;
                for (int c = 0; c < d; ++c) out[c] += hv * (double)w[c];
            }
        }
        free(hid);
    }
}

/* Combine (Sec. 2.2, caption of the forward-pass timeline figure): y[t,:] = sum over kept choices j (ascending) of
 * gate[t,j] * ye[slot_of[t*k+j],:], zero when no choice was kept; fp64 sums,
 * stored fp32.  ye is the full [A,d] fp64 buffer. */
void oracle_combine(const double *ye, const int32_t *slot_of, const float *gate,
                    int T, int k, int d, float *y)
{
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j) {
                int s = slot_of[(size_t)t * k + j];
                if (s < 0) continue;
                acc += (double)gate[(size_t)t * k + j] * ye[(size_t)s * d + c];
            }
            y[(size_t)t * d + c] = (float)acc;
        }
    }
}
