/*
 * CPU oracle for one Mixture-of-Experts layer's local computation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it,
 * and it shares no code with the GPU sources.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg use it.
 *
 * What it computes (paper: Section 1 and Figure 1 for the layer -- a routing
 * function that sends every token to exactly one expert FFN; Section 3,
 * steps 3-7 of Figure 3 for the order routing -> exchange -> expert FFN
 * shard -> exchange back; Section 2.4 for the FFN being a pair of consecutive
 * fully connected layers split Megatron-style, of which one GPU owns f of the
 * 4h inner columns and therefore produces a partial sum).
 *
 * The paper leaves the routing function's form, the capacity rule and the
 * activation open.  The readings taken here:
 *   - gate logits  L = X Wg  (no bias), accumulated in double, stored as fp32;
 *   - expert of a token = lowest index attaining the row maximum of the fp32
 *     logits (comparison on float values, so -0 == +0);
 *   - gate probability = softmax over the E logits, evaluated in double with
 *     the row maximum subtracted, rounded to fp32;
 *   - capacity C is given; a token's slot is the number of earlier tokens
 *     (smaller index) routed to the same expert; it is kept iff slot < C;
 *   - dispatch copies kept tokens to D[e, slot, :], other rows of D are zero;
 *   - expert FFN: Z = D_e W1_e, H = GeLU(Z), Y = H W2_e  (no biases);
 *   - combine: out[t] = p_t * Y[e_t, slot_t] for kept tokens, 0 for dropped.
 * Backward is the exact derivative of the above with e_t and slot_t constant.
 *
 * All floating point accumulation is in double.  Inputs are fp32 arrays (for
 * bf16 workloads they hold bf16-representable values).  No blocking, no
 * fusion: each function is the definition written out; OpenMP only splits the
 * outermost independent loop.
 *
 * Pins: see tests/test_oracle_*.py (brute force routing, one-hot cumsum
 * formulation, library matmul/softmax/GeLU in fp64, autograd through a dense
 * one-hot formulation, finite differences, the paper's 4-token example; for the optimizer step at
 * the end of this file: a library AdamW in fp64, closed forms of the first step, tiling invariance;
 * for duplicate token dropping: strided array slices, the round trip, every row in exactly one share,
 * and the two-rank picture of the paper's Figure 5).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_ACT_GELU_ERF 0
#define ORC_ACT_GELU_TANH 1

static double act_fwd(double x, int act) {
    if (act == ORC_ACT_GELU_TANH) {
        double u = sqrt(2.0 / M_PI) * (x + 0.044715 * x * x * x);
        return 0.5 * x * (1.0 + tanh(u));
    }
    return 0.5 * x * (1.0 + erf(x / sqrt(2.0)));
}

static double act_grad(double x, int act) {
    if (act == ORC_ACT_GELU_TANH) {
        double c = sqrt(2.0 / M_PI);
        double u = c * (x + 0.044715 * x * x * x);
        double th = tanh(u);
        double du = c * (1.0 + 3.0 * 0.044715 * x * x);
        return 0.5 * (1.0 + th) + 0.5 * x * (1.0 - th * th) * du;
    }
    return 0.5 * (1.0 + erf(x / sqrt(2.0))) + x * exp(-0.5 * x * x) / sqrt(2.0 * M_PI);
}

/* scalar access for the GeLU pins */
double orc_act(double x, int act) { return act_fwd(x, act); }
double orc_act_grad(double x, int act) { return act_grad(x, act); }
/* the same derivative over an array (what a backward pass may keep instead of z) */
void orc_act_grad_array(int64_t n, const double *z, double *g, int act) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) g[i] = act_grad(z[i], act);
}

/* Routing function, linear part: L[t,j] = sum_k X[t,k] Wg[k,j]. */
void orc_gate_logits(int64_t T, int32_t h, int32_t E, const float *x, const float *wg, float *logits) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int32_t j = 0; j < E; ++j) {
            double acc = 0.0;
            for (int32_t k = 0; k < h; ++k) acc += (double)x[t * h + k] * (double)wg[(int64_t)k * E + j];
            logits[t * E + j] = (float)acc;
        }
    }
}

/* Top-1 choice and softmax over the stored fp32 logits. probs may be NULL. */
void orc_top1_softmax(int64_t T, int32_t E, const float *logits, int32_t *expert, float *gate_p, float *probs) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const float *row = logits + t * E;
        int32_t best = 0;
        for (int32_t j = 1; j < E; ++j)
            if (row[j] > row[best]) best = j; /* strict: first maximum wins */
        double m = (double)row[best];
        double denom = 0.0;
        for (int32_t j = 0; j < E; ++j) denom += exp((double)row[j] - m);
        expert[t] = best;
        gate_p[t] = (float)(1.0 / denom);
        if (probs)
            for (int32_t j = 0; j < E; ++j) probs[t * E + j] = (float)(exp((double)row[j] - m) / denom);
    }
}

/* Capacity-limited slot assignment in arrival (token index) order.
 * token_of_slot [E*C] may be NULL; unfilled entries are -1. */
void orc_route(int64_t T, int32_t E, int64_t C, const int32_t *expert, int32_t *slot, int32_t *counts,
               int32_t *kept, int32_t *token_of_slot) {
    for (int32_t e = 0; e < E; ++e) counts[e] = 0;
    if (token_of_slot)
        for (int64_t i = 0; i < (int64_t)E * C; ++i) token_of_slot[i] = -1;
    for (int64_t t = 0; t < T; ++t) {
        int32_t e = expert[t];
        int64_t s = counts[e]++;
        if (s < C) {
            slot[t] = (int32_t)s;
            if (token_of_slot) token_of_slot[(int64_t)e * C + s] = (int32_t)t;
        } else {
            slot[t] = -1;
        }
    }
    for (int32_t e = 0; e < E; ++e) kept[e] = counts[e] < C ? counts[e] : (int32_t)C;
}

/* D[e_t, slot_t, :] = X[t, :] for kept tokens; every other row of D is zero. */
void orc_dispatch(int64_t T, int32_t h, int32_t E, int64_t C, const float *x, const int32_t *expert,
                  const int32_t *slot, float *D) {
    memset(D, 0, sizeof(float) * (size_t)E * (size_t)C * (size_t)h);
    for (int64_t t = 0; t < T; ++t) {
        if (slot[t] < 0) continue;
        float *dst = D + ((int64_t)expert[t] * C + slot[t]) * h;
        for (int32_t k = 0; k < h; ++k) dst[k] = x[t * h + k];
    }
}

/* Duplicate token dropping (paper Section 5.1, Figure 5).  The G ranks of a tensor-parallel group hold the same
 * expert chunks; before the all-to-all each rank "drops" all rows but its own share, so that every row
 * leaves the group exactly once and the messages shrink by the factor G; after the all-to-all an all-gather
 * among the G ranks puts the shares together again.  The paper does not say which rows a rank keeps; the
 * reading here: rank r keeps rows s with s mod G == r, in order (row s becomes row s / G of its share).
 *   drop:    share[e, j, :] = buf[e, j*G + r, :]   for j*G + r < C, zero rows beyond   (share is [E, Cg, w], Cg = ceil(C/G))
 *   gather:  buf[e, s, :]   = shares[s mod G][e, s / G, :]                              (shares is [G, E, Cg, w])
 * Works on float arrays of row width w (activations or their gradients: the backward swaps the two steps). */
void orc_dtd_drop(int32_t E, int64_t C, int32_t w, int32_t G, int32_t r, const float *buf, float *share) {
    const int64_t Cg = (C + G - 1) / G;
    for (int32_t e = 0; e < E; ++e)
        for (int64_t j = 0; j < Cg; ++j) {
            const int64_t s = j * G + r;
            float *dst = share + ((int64_t)e * Cg + j) * w;
            for (int32_t k = 0; k < w; ++k) dst[k] = s < C ? buf[((int64_t)e * C + s) * w + k] : 0.0f;
        }
}

void orc_dtd_gather(int32_t E, int64_t C, int32_t w, int32_t G, const float *shares, float *buf) {
    const int64_t Cg = (C + G - 1) / G;
    for (int32_t e = 0; e < E; ++e)
        for (int64_t s = 0; s < C; ++s) {
            const float *src = shares + (((int64_t)(s % G) * E + e) * Cg + s / G) * w;
            float *dst = buf + ((int64_t)e * C + s) * w;
            for (int32_t k = 0; k < w; ++k) dst[k] = src[k];
        }
}

/* One expert's FFN on `rows` rows: Z = D W1, H = act(Z), Y = H W2.
 * D [rows,h], W1 [h,f], W2 [f,h] fp32; Z,H [rows,f], Y [rows,h] double. */
void orc_ffn_fwd(int64_t rows, int32_t h, int32_t f, int32_t act, const float *D, const float *W1,
                 const float *W2, double *Z, double *H, double *Y) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double *z = Z + r * f, *hh = H + r * f, *y = Y + r * h;
        for (int32_t n = 0; n < f; ++n) z[n] = 0.0;
        for (int32_t k = 0; k < h; ++k) {
            double a = (double)D[r * h + k];
            const float *w = W1 + (int64_t)k * f;
            for (int32_t n = 0; n < f; ++n) z[n] += a * (double)w[n];
        }
        for (int32_t n = 0; n < f; ++n) hh[n] = act_fwd(z[n], act);
        for (int32_t j = 0; j < h; ++j) y[j] = 0.0;
        for (int32_t n = 0; n < f; ++n) {
            double a = hh[n];
            const float *w = W2 + (int64_t)n * h;
            for (int32_t j = 0; j < h; ++j) y[j] += a * (double)w[j];
        }
    }
}

/* out[t,:] = p_t * Y[e_t, slot_t, :] if kept else 0.  Y is [E,C,h] double. */
void orc_combine(int64_t T, int32_t h, int64_t C, const double *Y, const int32_t *expert, const int32_t *slot,
                 const float *gate_p, double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        double *o = out + t * h;
        if (slot[t] < 0) {
            for (int32_t j = 0; j < h; ++j) o[j] = 0.0;
        } else {
            const double *y = Y + ((int64_t)expert[t] * C + slot[t]) * h;
            double p = (double)gate_p[t];
            for (int32_t j = 0; j < h; ++j) o[j] = p * y[j];
        }
    }
}

/* Backward of combine: dY[e_t,slot_t,:] = p_t dOut[t,:]; dp_t = <dOut[t,:], Y[e_t,slot_t,:]>.
 * Unfilled rows of dY are zero; dp of dropped tokens is zero. */
void orc_combine_bwd(int64_t T, int32_t h, int32_t E, int64_t C, const float *d_out, const double *Y,
                     const int32_t *expert, const int32_t *slot, const float *gate_p, double *dY, double *dp) {
    memset(dY, 0, sizeof(double) * (size_t)E * (size_t)C * (size_t)h);
    for (int64_t t = 0; t < T; ++t) {
        dp[t] = 0.0;
        if (slot[t] < 0) continue;
        int64_t row = (int64_t)expert[t] * C + slot[t];
        double p = (double)gate_p[t], acc = 0.0;
        for (int32_t j = 0; j < h; ++j) {
            double g = (double)d_out[t * h + j];
            dY[row * h + j] = p * g;
            acc += g * Y[row * h + j];
        }
        dp[t] = acc;
    }
}

/* Backward of one expert's FFN on `rows` rows.
 *   dH = dY W2^T ; dZ = dH * act'(Z) ; dW2 = H^T dY ; dW1 = D^T dZ ; dD = dZ W1^T
 * dY [rows,h], Z,H [rows,f] double; D,W1,W2 fp32.
 * Outputs dD [rows,h], dW1 [h,f], dW2 [f,h], dZ [rows,f] (all double). */
void orc_ffn_bwd(int64_t rows, int32_t h, int32_t f, int32_t act, const double *dY, const float *D,
                 const double *Z, const double *H, const float *W1, const float *W2, double *dD, double *dW1,
                 double *dW2, double *dZ) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int32_t n = 0; n < f; ++n) {
            double acc = 0.0;
            const float *w = W2 + (int64_t)n * h;
            for (int32_t j = 0; j < h; ++j) acc += dY[r * h + j] * (double)w[j];
            dZ[r * f + n] = acc * act_grad(Z[r * f + n], act);
        }
    }
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < f; ++n) {
        double *g = dW2 + (int64_t)n * h;
        for (int32_t j = 0; j < h; ++j) g[j] = 0.0;
        for (int64_t r = 0; r < rows; ++r) {
            double a = H[r * f + n];
            for (int32_t j = 0; j < h; ++j) g[j] += a * dY[r * h + j];
        }
    }
#pragma omp parallel for schedule(static)
    for (int32_t k = 0; k < h; ++k) {
        double *g = dW1 + (int64_t)k * f;
        for (int32_t n = 0; n < f; ++n) g[n] = 0.0;
        for (int64_t r = 0; r < rows; ++r) {
            double a = (double)D[r * h + k];
            for (int32_t n = 0; n < f; ++n) g[n] += a * dZ[r * f + n];
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int32_t k = 0; k < h; ++k) {
            double acc = 0.0;
            const float *w = W1 + (int64_t)k * f;
            for (int32_t n = 0; n < f; ++n) acc += dZ[r * f + n] * (double)w[n];
            dD[r * h + k] = acc;
        }
    }
}

/* Backward of dispatch: dX[t,:] = dD[e_t, slot_t, :] if kept else 0.  dD is [E,C,h]. */
void orc_dispatch_bwd(int64_t T, int32_t h, int64_t C, const double *dD, const int32_t *expert,
                      const int32_t *slot, double *dX) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int32_t k = 0; k < h; ++k)
            dX[t * h + k] = slot[t] < 0 ? 0.0 : dD[((int64_t)expert[t] * C + slot[t]) * h + k];
    }
}

/* Backward of the gate (softmax top-1 probability and the linear map).
 *   dL[t,j] = dp_t * p_t * ([j == e_t] - P[t,j])      (softmax Jacobian row e_t)
 *   dWg     = X^T dL ;  dX_gate = dL Wg^T
 * probs [T,E] fp32 (P), dp [T] double.  Outputs double: dL [T,E], dWg [h,E], dXg [T,h]. */
void orc_gate_bwd(int64_t T, int32_t h, int32_t E, const double *dp, const float *probs, const int32_t *expert,
                  const float *x, const float *wg, double *dL, double *dWg, double *dXg) {
    for (int64_t t = 0; t < T; ++t) {
        double pe = (double)probs[t * E + expert[t]];
        for (int32_t j = 0; j < E; ++j) {
            double delta = (j == expert[t]) ? 1.0 : 0.0;
            dL[t * E + j] = dp[t] * pe * (delta - (double)probs[t * E + j]);
        }
    }
#pragma omp parallel for schedule(static)
    for (int32_t k = 0; k < h; ++k) {
        for (int32_t j = 0; j < E; ++j) {
            double acc = 0.0;
            for (int64_t t = 0; t < T; ++t) acc += (double)x[t * h + k] * dL[t * E + j];
            dWg[(int64_t)k * E + j] = acc;
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int32_t k = 0; k < h; ++k) {
            double acc = 0.0;
            for (int32_t j = 0; j < E; ++j) acc += dL[t * E + j] * (double)wg[(int64_t)k * E + j];
            dXg[t * h + k] = acc;
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Tiled mixed-precision AdamW step (paper: Section 4 -- the optimizer up-casts the 16-bit
 * gradients of the expert parameter group to 32 bit before the update; done for the whole group
 * at once this needs a temporary of 4 bytes per parameter, so the group is cut into tiles of ts
 * parameters that are processed one after the other, and the temporary of 4*ts bytes is reused
 * by every tile.  The optimizer is AdamW: experimental set-up, Section 6).
 *
 * Per tile, in the paper's order:
 *   1. up-cast: staging[j] = fp32(grad[i0 + j]) * grad_mult        (fp32 storage, ts floats)
 *   2. update from staging, element by element (decoupled weight decay, bias-corrected moments):
 *        m <- b1 m + (1 - b1) g            v <- b2 v + (1 - b2) g^2
 *        mhat = m / (1 - b1^t)             vhat = v / (1 - b2^t)
 *        w <- w - lr * ( mhat / (sqrt(vhat) + eps) + wd * w )
 *      evaluated in double from the fp32 values of g, m, v, w; m, v, w are stored as fp32 (the
 *      optimizer states of mixed precision training are 32 bit);
 *   3. the 16-bit copy of the parameter is the fp32 master value rounded to nearest even bf16
 *      (round_bf16 != 0) or the fp32 value itself.
 * Readings the paper leaves open: the decay term is scaled by lr (the form every framework the
 * paper builds on uses); grad_mult is the inverse loss scale (1 for bf16); t counts from 1.
 *
 * staging must hold ts floats and nothing else is used as temporary, which is the memory bound
 * of Section 4; touched_hi (optional) receives the highest staging index written + 1.
 * ------------------------------------------------------------------------------------------ */
static float round_to_bf16(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return x;            /* NaN stays NaN */
    uint32_t keep = u >> 16, rest = u & 0xffffu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1u;
    u = keep << 16;
    float y;
    memcpy(&y, &u, 4);
    return y;
}

void orc_adamw_tiled(int64_t n, int64_t ts, double lr, double beta1, double beta2, double eps, double wd,
                     int32_t step, double grad_mult, const float *grad, float *master, float *exp_avg,
                     float *exp_avg_sq, float *param, int32_t round_bf16, float *staging, int64_t *touched_hi) {
    const double bc1 = 1.0 - pow(beta1, (double)step);
    const double bc2 = 1.0 - pow(beta2, (double)step);
    int64_t hi = 0;
    for (int64_t i0 = 0; i0 < n; i0 += ts) {
        const int64_t len = (n - i0 < ts) ? (n - i0) : ts;
        for (int64_t j = 0; j < len; ++j) staging[j] = (float)((double)grad[i0 + j] * grad_mult);
        if (len > hi) hi = len;
        for (int64_t j = 0; j < len; ++j) {
            const int64_t i = i0 + j;
            const double g = (double)staging[j];
            const double m = beta1 * (double)exp_avg[i] + (1.0 - beta1) * g;
            const double v = beta2 * (double)exp_avg_sq[i] + (1.0 - beta2) * g * g;
            const double mhat = m / bc1, vhat = v / bc2;
            const double w0 = (double)master[i];
            const double w = w0 - lr * (mhat / (sqrt(vhat) + eps) + wd * w0);
            exp_avg[i] = (float)m;
            exp_avg_sq[i] = (float)v;
            master[i] = (float)w;
            param[i] = round_bf16 ? round_to_bf16(master[i]) : master[i];
        }
    }
    if (touched_hi) *touched_hi = hi;
}

int orc_max_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
