/*
 * Switch FFN layer -- CPU oracle (TEST INFRASTRUCTURE, not a product path).
 *
 * A plain, slow, fp64 evaluation of the layer's definition, written from the
 * paper (arXiv 2101.03961).  The T tokens form n_groups routing groups of
 * T / n_groups consecutive tokens each (the appendix listing's num_cores;
 * capacity, position and the auxiliary loss are taken per group, the experts
 * are shared); n_groups = 1 is one group holding all tokens.  It is the
 * thing the GPU library is compared against; it shares no code, header or
 * table with that library and must never be called from it.
 *
 * Conventions
 *   - Tensors arrive as float arrays holding the exact values the GPU sees
 *     (bf16 and fp32 both widen to float without rounding); every arithmetic
 *     step is done in double.  Integer routing results are int32 / uint8.
 *   - Row-major:  x[T][d], W_r[d][E], W_in[E][d][f], W_out[E][f][d].
 *   - Loops run in the order the definition is written (k ascending inside a
 *     dot product, tokens in sequence order); there is no blocking or fusion.
 *     OpenMP is used only across independent tokens / output elements, which
 *     does not change any summation order.
 *
 * Readings of the paper taken here (each also listed in the design notes):
 *   - capacity = floor(T / E * capacity_factor), evaluated in double (Eq. 3
 *     leaves the rounding open).
 *   - position_in_expert is the 0-based count of earlier tokens (sequence
 *     order) that chose the same expert; a token is kept iff position <
 *     capacity, so an expert keeps exactly min(count, capacity) tokens
 *     (Fig. 3; the appendix listing's 1-based cumsum with a strict compare
 *     would keep capacity-1 and is read as an off-by-one).
 *   - arg max ties go to the lowest expert index.
 *   - f_i in the auxiliary loss counts arg max decisions over ALL tokens,
 *     before any capacity truncation (Eq. 5), and is a constant under
 *     differentiation; P_i is differentiable (Sec. 2.2).
 *   - with several groups the loss is the mean over groups of the one-group
 *     loss (the listing's mean over [num_cores, num_experts] times N^2), and
 *     the capacity is floor(T_group / E * capacity_factor).
 *   - training-time noise (optional, off by default; swo_noise):
 *       input jitter (App. C: multiplicative jitter on the router's incoming representation;
 *       the appendix listing instead adds the noise to the logits -- the text is followed):
 *       the router sees x[t][k] * m, m uniform in [1 - eps, 1 + eps), the experts see x;
 *       expert dropout (Sec. 2.4): the hidden activation ReLU(h) of every expert is dropped
 *       with the given rate (rounded down to a multiple of 2^-16) and the survivors are
 *       scaled by 1 / (1 - that rate).
 *     The random numbers come from a counter-based generator defined here (swo_mix): a
 *     32-bit mixing function of (seed, stream, element index), so that any implementation
 *     can reproduce every draw from the element's coordinates alone.
 *   - expert FFN variants (ffn_kind): 0 = the ReLU FFN of Sec. 5's review, ReLU(x W_in) W_out;
 *     1 = the gated-GELU FFN that App. "Switch models" / Tab. 9 marks as FFN_GEGLU (the
 *     expansion matrix replaced by two sets of weights combined non-linearly, after Shazeer
 *     2020): (GELU(x W_g) (.) (x W_l)) W_out with the exact GELU(u) = u Phi(u); W_in then holds
 *     [W_g | W_l] side by side, [d][2 f].  Expert dropout acts on the combined hidden
 *     activation.
 *   - No-Token-Left-Behind (App. B), optional: see swo_ntlb.  A re-routed token's output is
 *     scaled by the router probability of the expert that processes it; the auxiliary loss
 *     keeps counting the arg max decisions.
 *   - the residual connection is outside the layer: a dropped token's output
 *     row is zero.
 *   - ReLU'(0) = 0.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Storage type of the incoming tensors.  float by default (holds every bf16 and
 * fp32 value exactly).  The finite-difference tests build a second copy of this
 * file with -DSWO_IN_T=double so that inputs can be perturbed by 1e-6; the
 * arithmetic below is the same either way (every operand is widened to double
 * before use). */
#ifndef SWO_IN_T
#define SWO_IN_T float
#endif
typedef SWO_IN_T in_t;

/* ---- training-time noise ------------------------------------------------- */
typedef struct {
    float expert_dropout; /* rate in [0, 1): 0 = off                          */
    float jitter_eps;     /* eps in [0, 1): 0 = off                           */
    uint64_t seed;
} swo_noise;

/* 32 random bits for element `idx` (wrapping 32-bit index) of stream `stream`:
 * multiply / xor-shift rounds over idx, with the two halves of the seed and the stream
 * number folded in. */
uint32_t swo_mix(uint32_t idx, uint32_t stream, uint64_t seed) {
    uint32_t z = idx ^ (uint32_t)seed;
    z *= 0x9E3779B1u;
    z ^= z >> 15;
    z += (uint32_t)(seed >> 32) + stream * 0x7F4A7C15u;
    z *= 0x85EBCA77u;
    z ^= z >> 13;
    z *= 0xC2B2AE3Du;
    z ^= z >> 16;
    return z;
}
enum { SWO_STREAM_JITTER = 1, SWO_STREAM_DROPOUT = 2 };

/* jitter multiplier of x[t][k]: (1 - eps) + 2 eps u with u = (top 24 bits) 2^-24, evaluated
 * in fp32 with one fused multiply-add (so that an fp32 implementation gets the same m) */
static double jitter_mult(const swo_noise *nz, int64_t t, int64_t d, int64_t k) {
    if (!nz || nz->jitter_eps <= 0.0f) return 1.0;
    uint32_t z = swo_mix((uint32_t)((uint64_t)t * (uint64_t)d + (uint64_t)k), SWO_STREAM_JITTER,
                         nz->seed);
    float u = (float)(z >> 8) * 0x1p-24f;
    return (double)fmaf(2.0f * nz->jitter_eps, u, 1.0f - nz->jitter_eps);
}
/* dropout factor of hidden unit j of token t: 0 (dropped) or 1 / (1 - rate'), rate' = the
 * rate rounded down to a multiple of 2^-16.  Element idx = t f + j (wrapping 32-bit) takes 16
 * of the 32 bits drawn for the pair idx / 2 -- the low half if idx is even, the high half if
 * odd -- and is dropped iff they are below rate' 2^16; survivors are scaled so that the
 * expectation is exactly the undropped value. */
static double dropout_factor(const swo_noise *nz, int64_t t, int64_t f, int64_t j) {
    if (!nz || nz->expert_dropout <= 0.0f) return 1.0;
    uint32_t thr = (uint32_t)floor((double)nz->expert_dropout * 65536.0);
    uint32_t idx = (uint32_t)((uint64_t)t * (uint64_t)f + (uint64_t)j);
    uint32_t z = swo_mix(idx >> 1, SWO_STREAM_DROPOUT, nz->seed);
    uint32_t h = (idx & 1u) ? z >> 16 : z & 0xFFFFu;
    return h >= thr ? 65536.0 / (65536.0 - (double)thr) : 0.0;
}
/* exported for the tests */
double swo_jitter_mult(const swo_noise *nz, int64_t t, int64_t d, int64_t k) {
    return jitter_mult(nz, t, d, k);
}
double swo_dropout_factor(const swo_noise *nz, int64_t t, int64_t f, int64_t j) {
    return dropout_factor(nz, t, f, j);
}

/* ---- Eq. 3: expert capacity -------------------------------------------- */
int64_t swo_capacity(int64_t T, int64_t E, double capacity_factor) {
    double c = (double)T / (double)E * capacity_factor;
    return (int64_t)floor(c);
}

/* ---- Sec. 2.1: router logits h(x) = W_r . x (+ optional bias) ----------- */
void swo_logits(int64_t T, int64_t d, int64_t E, const in_t *x, const in_t *W_r,
                const in_t *b_r /* may be NULL */, const swo_noise *nz /* may be NULL */,
                double *h /* [T][E] */) {
#pragma omp parallel
    {
        double *xr = (double *)malloc(sizeof(double) * (size_t)(d > 0 ? d : 1));
#pragma omp for schedule(static)
        for (int64_t t = 0; t < T; ++t) {
            /* the router's view of the token: x_t, jittered if asked for */
            for (int64_t k = 0; k < d; ++k)
                xr[k] = (double)x[t * d + k] * jitter_mult(nz, t, d, k);
            for (int64_t i = 0; i < E; ++i) {
                double s = 0.0;
                for (int64_t k = 0; k < d; ++k) s += xr[k] * (double)W_r[k * E + i];
                if (b_r) s += (double)b_r[i];
                h[t * E + i] = s;
            }
        }
        free(xr);
    }
}

/* ---- Eq. 1: p_i = exp(h_i) / sum_j exp(h_j), max-shifted ---------------- */
void swo_softmax(int64_t T, int64_t E, const double *h, double *p) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double *ht = h + t * E;
        double m = ht[0];
        for (int64_t i = 1; i < E; ++i)
            if (ht[i] > m) m = ht[i];
        double z = 0.0;
        for (int64_t i = 0; i < E; ++i) z += exp(ht[i] - m);
        for (int64_t i = 0; i < E; ++i) p[t * E + i] = exp(ht[i] - m) / z;
    }
}

/* ---- Switch routing (k = 1): expert = arg max, gate = its probability --- */
void swo_top1(int64_t T, int64_t E, const double *h, const double *p,
              int32_t *expert_index, double *gate) {
    for (int64_t t = 0; t < T; ++t) {
        int64_t best = 0;
        for (int64_t i = 1; i < E; ++i)
            if (h[t * E + i] > h[t * E + best]) best = i; /* strict: lowest index wins ties */
        expert_index[t] = (int32_t)best;
        gate[t] = p[t * E + best];
    }
}

/* ---- Eqs. 4-6: loss = alpha * N * sum_i f_i P_i, averaged over the groups ---
 * counts [E]: arg max decisions per expert over all tokens.  counts_g, f_out,
 * P_out: [n_groups][E] (each may be NULL): per-group counts, f and P. */
double swo_aux_loss(int64_t T, int64_t E, int64_t n_groups, const int32_t *expert_index,
                    const double *p, double alpha, int64_t *counts, int64_t *counts_g,
                    double *f_out, double *P_out) {
    for (int64_t i = 0; i < E; ++i) counts[i] = 0;
    for (int64_t t = 0; t < T; ++t) counts[expert_index[t]] += 1;
    const int64_t Tg = T / n_groups;
    double total = 0.0;
    for (int64_t g = 0; g < n_groups; ++g) {
        double loss = 0.0;
        for (int64_t i = 0; i < E; ++i) {
            int64_t cnt = 0;
            double P_i = 0.0;
            for (int64_t t = g * Tg; t < (g + 1) * Tg; ++t) {
                cnt += (expert_index[t] == i);
                P_i += p[t * E + i];
            }
            /* empty batch: both fractions are empty sums; the loss is taken as 0 */
            double f_i = Tg > 0 ? (double)cnt / (double)Tg : 0.0;
            P_i = Tg > 0 ? P_i / (double)Tg : 0.0;
            if (counts_g) counts_g[g * E + i] = cnt;
            if (f_out) f_out[g * E + i] = f_i;
            if (P_out) P_out[g * E + i] = P_i;
            loss += f_i * P_i;
        }
        total += alpha * (double)E * loss;
    }
    return total / (double)n_groups;
}

/* ---- position in expert, sequence order inside the token's group; overflow is
 * dropped.  C is the per-group capacity; kept: [n_groups][E]. ---------------- */
void swo_positions(int64_t T, int64_t E, int64_t C, int64_t n_groups,
                   const int32_t *expert_index, int32_t *position_in_expert, uint8_t *dropped,
                   int64_t *kept) {
    int64_t *seen = (int64_t *)calloc((size_t)E, sizeof(int64_t));
    const int64_t Tg = T / n_groups;
    for (int64_t g = 0; g < n_groups; ++g) {
        for (int64_t i = 0; i < E; ++i) {
            seen[i] = 0;
            kept[g * E + i] = 0;
        }
        for (int64_t t = g * Tg; t < (g + 1) * Tg; ++t) {
            int32_t e = expert_index[t];
            int64_t pos = seen[e]++;
            position_in_expert[t] = (int32_t)pos;
            dropped[t] = (uint8_t)(pos >= C);
            if (pos < C) kept[g * E + e] += 1;
        }
    }
    free(seen);
}

/* ---- No-Token-Left-Behind (App. B): after the Switch routing above (stage 1), `rounds`
 * further stages re-route the tokens that are still without a slot.  In stage r + 1 every
 * such token, in sequence order inside its group, asks for its next-best expert -- experts
 * ranked by logit, highest first, equal logits by lower index; softmax is monotone, so this
 * is the ranking by router probability -- and gets that expert's next free slot if the
 * group's capacity is not used up; otherwise it stays without one (and may try again in
 * the next stage).  Inputs: the stage-1 result (expert_index, position_in_expert, dropped,
 * kept as left by swo_positions).  choice_override ([T][rounds], may be NULL): the expert a
 * token asks for in stage r + 1 instead of the ranking's.
 * Outputs, for tokens that found a slot in a later stage: expert_index = that expert,
 * position_in_expert = its slot number within the (group, expert) capacity, dropped = 0; all
 * other entries are left as they are.  choices ([T][rounds], may be NULL) records what each
 * token asked for (-1: it already had a slot, or no expert was left to ask). */
void swo_ntlb(int64_t T, int64_t E, int64_t C, int64_t n_groups, int64_t rounds,
              const double *logits /* [T][E] */, const int32_t *choice_override,
              int32_t *expert_index, int32_t *position_in_expert, uint8_t *dropped,
              int64_t *kept /* [n_groups][E] */, int32_t *choices) {
    const int64_t Tg = T / n_groups;
    int32_t *asked = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    for (int64_t t = 0; t < T; ++t) asked[t] = expert_index[t];   /* the last expert asked */
    for (int64_t r = 0; r < rounds; ++r) {
        for (int64_t t = 0; t < T; ++t) {
            if (choices) choices[t * rounds + r] = -1;
            if (!dropped[t]) continue;
            const int64_t g = t / Tg;
            const double *h = logits + t * E;
            int32_t next = -1;
            if (choice_override) {
                next = choice_override[t * rounds + r];
            } else if (asked[t] >= 0) {
                /* the best expert that ranks strictly after the one asked last */
                const int32_t a = asked[t];
                for (int32_t i = 0; i < (int32_t)E; ++i) {
                    const int after = h[i] < h[a] || (h[i] == h[a] && i > a);
                    if (after && (next < 0 || h[i] > h[next])) next = i;
                }
            }
            asked[t] = next;
            if (choices) choices[t * rounds + r] = next;
            if (next < 0) continue;
            if (kept[g * E + next] < C) {
                expert_index[t] = next;
                position_in_expert[t] = (int32_t)kept[g * E + next];
                dropped[t] = 0;
                kept[g * E + next] += 1;
            }
        }
    }
    free(asked);
}

/* Work sharing.  The expert part is evaluated token by token, in sequence
 * order; inside one token the independent output elements (columns of h, of o,
 * rows of the weight gradients) are split over the OpenMP team.  Every element
 * is still produced by one thread, with its sum taken in ascending index order,
 * so the arithmetic does not depend on the number of threads. */
static void my_range(int64_t n, int64_t *lo, int64_t *hi) {
    int64_t nt = omp_get_num_threads(), id = omp_get_thread_num();
    *lo = n * id / nt;
    *hi = n * (id + 1) / nt;
}

enum { SWO_FFN_RELU = 0, SWO_FFN_GEGLU = 1 };

/* Phi(u), the standard normal distribution function, and GELU(u) = u Phi(u) with its derivative
 * Phi(u) + u phi(u). */
static double norm_cdf(double u) { return 0.5 * erfc(-u * 0.70710678118654752440); }
static double gelu(double u) { return u * norm_cdf(u); }
static double gelu_deriv(double u) {
    return norm_cdf(u) + u * 0.39894228040143267794 * exp(-0.5 * u * u);
}

/* One token through one expert (Sec. 5, review of the FFN layer): h = x W_in, the hidden
 * activation a from h, o = a W_out.  ReLU FFN: W_in is [d][f], a = ReLU(h).  Gated-GELU FFN:
 * W_in is [d][2 f], a_j = GELU(h_j) h_{f+j}.  hpre has room for 2 f values.  Called by every
 * thread of the team. */
static void ffn_token(int kind, int64_t d, int64_t f, const in_t *xt, const in_t *Wi,
                      const in_t *Wo, const swo_noise *nz, int64_t t, double *hpre, double *a,
                      double *o) {
    const int64_t f1 = kind == SWO_FFN_GEGLU ? 2 * f : f;
    int64_t c0, c1, j0, j1, i0, i1;
    my_range(f1, &c0, &c1);
    my_range(f, &j0, &j1);
    my_range(d, &i0, &i1);
    for (int64_t j = c0; j < c1; ++j) hpre[j] = 0.0;
    for (int64_t k = 0; k < d; ++k) {
        double xk = (double)xt[k];
        const in_t *row = Wi + k * f1;
        for (int64_t j = c0; j < c1; ++j) hpre[j] += xk * (double)row[j];
    }
#pragma omp barrier
    for (int64_t j = j0; j < j1; ++j) {
        double act = kind == SWO_FFN_GEGLU ? gelu(hpre[j]) * hpre[f + j]
                                           : (hpre[j] > 0.0 ? hpre[j] : 0.0);
        a[j] = act != 0.0 ? act * dropout_factor(nz, t, f, j) : 0.0;
    }
#pragma omp barrier
    for (int64_t i = i0; i < i1; ++i) o[i] = 0.0;
    for (int64_t j = 0; j < f; ++j) {
        double aj = a[j];
        const in_t *row = Wo + j * d;
        for (int64_t i = i0; i < i1; ++i) o[i] += aj * (double)row[i];
    }
#pragma omp barrier
}

/* ---- layer output: y_t = gate_t * FFN_{e_t}(x_t) for kept tokens, 0 for
 * dropped ones (Fig. 2 caption; Sec. 2.2 on dropped tokens).
 * token_sel (may be NULL = all): tokens with token_sel[t] == 0 are skipped and
 * their rows are filled with NaN ("not computed"). */
void swo_expert_ffn(int64_t T, int64_t d, int64_t f, int64_t E, const in_t *x,
                    const in_t *W_in, const in_t *W_out, const int32_t *expert_index,
                    const uint8_t *dropped, const double *gate, const uint8_t *token_sel,
                    const swo_noise *nz /* may be NULL */, int64_t ffn_kind,
                    double *y /* [T][d] */) {
    const int64_t f1 = ffn_kind == SWO_FFN_GEGLU ? 2 * f : f;
    double *hpre = (double *)malloc(sizeof(double) * (size_t)f1);
    double *a = (double *)malloc(sizeof(double) * (size_t)f);
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp parallel
    {
        int64_t i0, i1;
        my_range(d, &i0, &i1);
        for (int64_t t = 0; t < T; ++t) {
            int32_t e = expert_index[t];
            double *yt = y + t * d;
            if (token_sel && !token_sel[t]) {
                for (int64_t i = i0; i < i1; ++i) yt[i] = NAN;
                continue;
            }
            if (dropped[t]) {
                for (int64_t i = i0; i < i1; ++i) yt[i] = 0.0;
                continue;
            }
            ffn_token((int)ffn_kind, d, f, x + t * d, W_in + (int64_t)e * d * f1,
                      W_out + (int64_t)e * f * d, nz, t, hpre, a, o);
            for (int64_t i = i0; i < i1; ++i) yt[i] = gate[t] * o[i];
#pragma omp barrier
        }
    }
    free(hpre);
    free(a);
    free(o);
    (void)E;
}

/* ---- hidden units whose ReLU decision an fp32 evaluation may take the other way ----
 * For every evaluated kept token t (token_sel as above) and hidden unit j with
 *     |h_tj| <= rel_eps * RMS_j(h_t),
 * (t, j, h_tj) is recorded (up to max_out entries; the return value is the number found).
 * The layer is discontinuous in its inputs there: an implementation that accumulates h in
 * fp32 gets the sign of such a sum from its rounding errors.  Tokens are shared out over
 * the OpenMP threads (each token's sums are taken by one thread, k ascending); the entries
 * come out in no particular order. */
int64_t swo_hidden_near_zero(int64_t T, int64_t d, int64_t f, const in_t *x, const in_t *W_in,
                             const int32_t *expert_index, const uint8_t *dropped,
                             const uint8_t *token_sel, double rel_eps, int64_t max_out,
                             int64_t *out_t, int64_t *out_j, double *out_h) {
    int64_t found = 0;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)f);
#pragma omp for schedule(dynamic, 16)
        for (int64_t t = 0; t < T; ++t) {
            if ((token_sel && !token_sel[t]) || dropped[t]) continue;
            const in_t *Wi = W_in + (int64_t)expert_index[t] * d * f;
            const in_t *xt = x + t * d;
            for (int64_t j = 0; j < f; ++j) h[j] = 0.0;
            for (int64_t k = 0; k < d; ++k) {
                double xk = (double)xt[k];
                const in_t *row = Wi + k * f;
                for (int64_t j = 0; j < f; ++j) h[j] += xk * (double)row[j];
            }
            double ss = 0.0;
            for (int64_t j = 0; j < f; ++j) ss += h[j] * h[j];
            double bound = rel_eps * sqrt(ss / (double)f);
            for (int64_t j = 0; j < f; ++j)
                if (fabs(h[j]) <= bound) {
#pragma omp critical(swo_near_zero)
                    {
                        if (found < max_out) {
                            out_t[found] = t;
                            out_j[found] = j;
                            out_h[found] = h[j];
                        }
                        ++found;
                    }
                }
        }
        free(h);
    }
    return found;
}

/* ---- backward ------------------------------------------------------------
 * Scalar objective  L = sum_t <dy_t, y_t> + d_aux * aux_loss.
 * Chain rule through y_t = k_t g_t o_t, o = a W_out, a = ReLU(h), h = x W_in,
 * g_t = p[t, e_t], p = softmax(x W_r + b_r), aux = mean over groups g of
 * alpha E sum_i f_gi P_gi with f held constant (T_g tokens per group, n groups):
 *   do_t  = k_t g_t dy_t                 dg_t = k_t <dy_t, o_t>
 *   dW_out[e] += a_t^T do_t              da_t = do_t W_out[e]^T
 *   dh_t  = da_t * 1[h_t > 0]            dW_in[e] += x_t^T dh_t
 *   dx_t  = dh_t W_in[e]^T  (expert part)
 *   dp[t,i]  = dg_t 1[i = e_t] + d_aux alpha E f_gi / (n T_g)      (t in group g)
 *   dl[t,j]  = p[t,j] (dp[t,j] - sum_i p[t,i] dp[t,i])         (softmax)
 *   dW_r = x^T dl,  db_r = sum_t dl_t,  dx_t += dl_t W_r^T
 * With noise: the router's input is x (.) m (jitter multipliers, constants), so x is replaced
 * by x (.) m in dW_r and the router's share of dx_t is (dl_t W_r^T) (.) m_t; the hidden
 * activation is ReLU(h) (.) q with q in {0, 1 / (1 - rate)}, so dh_t carries the same q.
 * Gated-GELU FFN (h = [u | v], a = GELU(u) (.) v (.) q): with da_t = dout_t W_out[e]^T,
 *   du_t = da_t (.) q (.) v (.) GELU'(u),  dv_t = da_t (.) q (.) GELU(u),  dh_t = [du_t | dv_t],
 * and dW_in, dx_t as above with the [d][2 f] matrix.
 *
 * Partial evaluation (for sampled checks on large layers):
 *   token_sel[t] == 0 (token_sel may be NULL = all selected): the token's expert
 *     FFN is not evaluated; its dgate is taken as 0 in the router part (exact
 *     only if dy is zero on that token) and its dx row is NaN.
 *   sel_slot[e] >= 0 (sel_slot may be NULL = slot e for every expert): expert
 *     e's weight gradients are accumulated into slot sel_slot[e] of dW_in_sel /
 *     dW_out_sel -- complete only if every kept token of e is selected.
 * ReLU decisions taken the other way: for the n_flip pairs (flip_t[q], flip_j[q]) the gate
 *   1[h > 0] is inverted (see swo_hidden_near_zero; the tests use it to follow an fp32
 *   implementation's decision on pre-activations that are zero to rounding).
 */
void swo_backward(int64_t T, int64_t d, int64_t f, int64_t E, const in_t *x, const in_t *W_r,
                  const in_t *W_in, const in_t *W_out, const in_t *dy, double d_aux,
                  double alpha, const int32_t *expert_index, const uint8_t *dropped,
                  const double *gate, const double *p /* [T][E] */, int64_t n_groups,
                  const int64_t *counts_g /* [n_groups][E] */,
                  const int32_t *sel_slot /* [E] or NULL */,
                  const uint8_t *token_sel /* [T] or NULL */, int64_t n_flip,
                  const int64_t *flip_t, const int64_t *flip_j,
                  const swo_noise *nz /* may be NULL */, int64_t ffn_kind,
                  double *dx /* [T][d] */,
                  double *dW_r /* [d][E] */, double *db_r /* [E] */,
                  double *dW_in_sel /* [nsel][d][f1] */, double *dW_out_sel /* [nsel][f][d] */,
                  double *dgate /* [T] */, double *dlogits /* [T][E] */) {
    /* expert part: tokens in sequence order, see "Work sharing" above */
    const int64_t f1 = ffn_kind == SWO_FFN_GEGLU ? 2 * f : f;   /* columns of W_in */
    double *hpre = (double *)malloc(sizeof(double) * (size_t)f1);
    double *a = (double *)malloc(sizeof(double) * (size_t)f);
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    double *dout = (double *)malloc(sizeof(double) * (size_t)d);
    double *dh = (double *)malloc(sizeof(double) * (size_t)f1);
#pragma omp parallel
    {
        int64_t j0, j1, k0, k1;
        my_range(f, &j0, &j1);
        my_range(d, &k0, &k1);
        for (int64_t e = 0; e < E; ++e) {
            int64_t slot = sel_slot ? sel_slot[e] : e;
            if (slot < 0) continue;
            double *gWi = dW_in_sel + slot * d * f1;
            double *gWo = dW_out_sel + slot * f * d;
            for (int64_t k = k0; k < k1; ++k)
                for (int64_t j = 0; j < f1; ++j) gWi[k * f1 + j] = 0.0;
            for (int64_t j = j0; j < j1; ++j)
                for (int64_t i = 0; i < d; ++i) gWo[j * d + i] = 0.0;
        }
#pragma omp barrier
        for (int64_t t = 0; t < T; ++t) {
            int64_t e = expert_index[t];
            int64_t slot = sel_slot ? sel_slot[e] : e;
            double *dxt = dx + t * d;
            if ((token_sel && !token_sel[t]) || dropped[t]) {
                double fill = (token_sel && !token_sel[t]) ? NAN : 0.0;
                for (int64_t k = k0; k < k1; ++k) dxt[k] = fill;
                if (omp_get_thread_num() == 0) dgate[t] = 0.0;
                continue;
            }
            const in_t *Wi = W_in + e * d * f1;
            const in_t *Wo = W_out + e * f * d;
            double *gWi = slot >= 0 ? dW_in_sel + slot * d * f1 : NULL;
            double *gWo = slot >= 0 ? dW_out_sel + slot * f * d : NULL;
            const in_t *xt = x + t * d;
            const in_t *dyt = dy + t * d;
            ffn_token((int)ffn_kind, d, f, xt, Wi, Wo, nz, t, hpre, a, o);
            /* gate gradient: a short dot product, taken whole by every thread */
            double dg = 0.0;
            for (int64_t i = 0; i < d; ++i) dg += (double)dyt[i] * o[i];
            if (omp_get_thread_num() == 0) dgate[t] = dg;
            for (int64_t i = k0; i < k1; ++i) dout[i] = gate[t] * (double)dyt[i];
#pragma omp barrier
            for (int64_t j = j0; j < j1; ++j) {
                const in_t *row = Wo + j * d;
                double aj = a[j], s = 0.0;
                if (gWo) {
                    double *grow = gWo + j * d;
                    for (int64_t i = 0; i < d; ++i) grow[i] += aj * dout[i];
                }
                for (int64_t i = 0; i < d; ++i) s += dout[i] * (double)row[i];
                if (ffn_kind == SWO_FFN_GEGLU) {
                    double sq = s * dropout_factor(nz, t, f, j);
                    dh[j] = sq * hpre[f + j] * gelu_deriv(hpre[j]);
                    dh[f + j] = sq * gelu(hpre[j]);
                    continue;
                }
                int on = hpre[j] > 0.0;
                for (int64_t q = 0; q < n_flip; ++q)
                    if (flip_t[q] == t && flip_j[q] == j) on = !on;
                dh[j] = on ? s * dropout_factor(nz, t, f, j) : 0.0;
            }
#pragma omp barrier
            for (int64_t k = k0; k < k1; ++k) {
                const in_t *row = Wi + k * f1;
                double xk = (double)xt[k], s = 0.0;
                if (gWi) {
                    double *grow = gWi + k * f1;
                    for (int64_t j = 0; j < f1; ++j) grow[j] += xk * dh[j];
                }
                for (int64_t j = 0; j < f1; ++j) s += dh[j] * (double)row[j];
                dxt[k] = s;
            }
#pragma omp barrier
        }
    }
    free(hpre);
    free(a);
    free(o);
    free(dout);
    free(dh);

    /* router part: softmax backward per token */
#pragma omp parallel
    {
        double *dp = (double *)malloc(sizeof(double) * (size_t)E);
#pragma omp for schedule(static)
        for (int64_t t = 0; t < T; ++t) {
            const double *pt = p + t * E;
            double s = 0.0;
            for (int64_t i = 0; i < E; ++i) {
                const int64_t Tg = T / n_groups;
                const int64_t g = t / Tg;
                double f_i = (double)counts_g[g * E + i] / (double)Tg;
                dp[i] = d_aux * alpha * (double)E * f_i / ((double)n_groups * (double)Tg);
                if (i == expert_index[t]) dp[i] += dgate[t];
                s += pt[i] * dp[i];
            }
            for (int64_t j = 0; j < E; ++j) dlogits[t * E + j] = pt[j] * (dp[j] - s);
            double *dxt = dx + t * d;
            for (int64_t k = 0; k < d; ++k) {
                double r = 0.0;
                for (int64_t j = 0; j < E; ++j) r += dlogits[t * E + j] * (double)W_r[k * E + j];
                dxt[k] += r * jitter_mult(nz, t, d, k);   /* the router saw x[t][k] * m */
            }
        }
        free(dp);
    }
    /* dW_r[k][j] = sum_t x[t][k] dl[t][j], t ascending for every element; a
     * thread owns whole rows k, so no element is shared between threads. */
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < d; ++k) {
        double *row = dW_r + k * E;
        for (int64_t j = 0; j < E; ++j) row[j] = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double xk = (double)x[t * d + k] * jitter_mult(nz, t, d, k);
            const double *dl = dlogits + t * E;
            for (int64_t j = 0; j < E; ++j) row[j] += xk * dl[j];
        }
    }
    for (int64_t j = 0; j < E; ++j) {
        double s = 0.0;
        for (int64_t t = 0; t < T; ++t) s += dlogits[t * E + j];
        db_r[j] = s;
    }
}
