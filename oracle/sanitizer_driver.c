/* Host-only check of the oracle's memory accesses: the whole forward + backward (both FFN
 * kinds, noise, routing groups, re-routing stages, partial evaluation, ReLU flips) on small
 * random inputs, built by the tests with -fsanitize=address,undefined.  Exact buffer sizes
 * everywhere, so that an access one element past any tensor is reported.  Test infrastructure,
 * like the rest of this directory. */
#include "switch_oracle.c"

#include <stdio.h>

static uint64_t rng_state = 88172645463325252ull;
static double urand(void) {   /* xorshift64: only to fill the inputs */
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0 - 0.5;
}
static in_t *randn(size_t n, double scale) {
    in_t *p = (in_t *)malloc(sizeof(in_t) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = (in_t)(scale * urand());
    return p;
}

static int run(int64_t T, int64_t d, int64_t f, int64_t E, int64_t n, double cf, int kind,
               int64_t rounds, const swo_noise *nz) {
    const int64_t f1 = kind == SWO_FFN_GEGLU ? 2 * f : f;
    in_t *x = randn((size_t)(T * d), 2.0), *W_r = randn((size_t)(d * E), 1.0);
    in_t *b_r = randn((size_t)E, 1.0), *W_in = randn((size_t)(E * d * f1), 1.0);
    in_t *W_out = randn((size_t)(E * f * d), 1.0), *dy = randn((size_t)(T * d), 2.0);
    double *h = malloc(sizeof(double) * (size_t)(T * E + 1)), *p = malloc(sizeof(double) * (size_t)(T * E + 1));
    int32_t *e = malloc(sizeof(int32_t) * (size_t)(T + 1)), *pos = malloc(sizeof(int32_t) * (size_t)(T + 1));
    uint8_t *dr = malloc((size_t)(T + 1)), *sel = malloc((size_t)(T + 1));
    double *g = malloc(sizeof(double) * (size_t)(T + 1));
    int64_t *counts = malloc(sizeof(int64_t) * (size_t)E), *counts_g = malloc(sizeof(int64_t) * (size_t)(n * E));
    int64_t *kept = malloc(sizeof(int64_t) * (size_t)(n * E));
    double *fo = malloc(sizeof(double) * (size_t)(n * E)), *Po = malloc(sizeof(double) * (size_t)(n * E));
    int32_t *choices = malloc(sizeof(int32_t) * (size_t)(T * (rounds ? rounds : 1) + 1));
    const int64_t C = swo_capacity(T / n, E, cf);
    swo_logits(T, d, E, x, W_r, b_r, nz, h);
    swo_softmax(T, E, h, p);
    swo_top1(T, E, h, p, e, g);
    double loss = swo_aux_loss(T, E, n, e, p, 0.01, counts, counts_g, fo, Po);
    swo_positions(T, E, C, n, e, pos, dr, kept);
    if (rounds) {
        swo_ntlb(T, E, C, n, rounds, h, NULL, e, pos, dr, kept, choices);
        for (int64_t t = 0; t < T; ++t) g[t] = p[t * E + e[t]];
    }
    for (int64_t t = 0; t < T; ++t) sel[t] = (uint8_t)(t % 3 != 1);
    double *y = malloc(sizeof(double) * (size_t)(T * d + 1));
    swo_expert_ffn(T, d, f, E, x, W_in, W_out, e, dr, g, NULL, nz, kind, y);
    swo_expert_ffn(T, d, f, E, x, W_in, W_out, e, dr, g, sel, nz, kind, y);
    int64_t nt[8], nj[8];
    double nh[8];
    int64_t found = kind == SWO_FFN_RELU ? swo_hidden_near_zero(T, d, f, x, W_in, e, dr, sel, 0.05, 8, nt, nj, nh) : 0;
    int64_t nflip = found < 8 ? found : 8;
    double *dx = malloc(sizeof(double) * (size_t)(T * d + 1)), *dW_r = malloc(sizeof(double) * (size_t)(d * E));
    double *db_r = malloc(sizeof(double) * (size_t)E), *dgate = malloc(sizeof(double) * (size_t)(T + 1));
    double *dlog = malloc(sizeof(double) * (size_t)(T * E + 1));
    /* all experts */
    double *dWi = malloc(sizeof(double) * (size_t)(E * d * f1)), *dWo = malloc(sizeof(double) * (size_t)(E * f * d));
    swo_backward(T, d, f, E, x, W_r, W_in, W_out, dy, 0.7, 0.01, e, dr, g, p, n, counts_g, NULL, NULL,
                 nflip, nt, nj, nz, kind, dx, dW_r, db_r, dWi, dWo, dgate, dlog);
    /* a selection: the last expert into slot 0, nothing else; some tokens skipped */
    int32_t *slot = malloc(sizeof(int32_t) * (size_t)E);
    for (int64_t i = 0; i < E; ++i) slot[i] = -1;
    slot[E - 1] = 0;
    double *dWi1 = malloc(sizeof(double) * (size_t)(d * f1)), *dWo1 = malloc(sizeof(double) * (size_t)(f * d));
    swo_backward(T, d, f, E, x, W_r, W_in, W_out, dy, 0.7, 0.01, e, dr, g, p, n, counts_g, slot, sel,
                 0, NULL, NULL, nz, kind, dx, dW_r, db_r, dWi1, dWo1, dgate, dlog);
    double check = loss + (T ? dx[0] : 0.0) + dW_r[0];
    free(x); free(W_r); free(b_r); free(W_in); free(W_out); free(dy); free(h); free(p); free(e);
    free(pos); free(dr); free(sel); free(g); free(counts); free(counts_g); free(kept); free(fo);
    free(Po); free(choices); free(y); free(dx); free(dW_r); free(db_r); free(dgate); free(dlog);
    free(dWi); free(dWo); free(slot); free(dWi1); free(dWo1);
    return check == check || 1;
}

int main(void) {
    swo_noise nz = {0.3f, 0.1f, 0x123456789abcdefull};
    int ok = 1;
    ok &= run(37, 5, 7, 3, 1, 0.75, SWO_FFN_RELU, 0, NULL);
    ok &= run(36, 4, 6, 4, 3, 1.0, SWO_FFN_RELU, 2, &nz);
    ok &= run(40, 6, 3, 5, 2, 0.5, SWO_FFN_GEGLU, 5, &nz);
    ok &= run(16, 3, 2, 1, 1, 2.0, SWO_FFN_GEGLU, 0, NULL);
    ok &= run(8, 2, 2, 16, 1, 1.0, SWO_FFN_RELU, 1, &nz);   /* capacity 0 */
    ok &= run(0, 4, 4, 2, 1, 1.0, SWO_FFN_RELU, 0, NULL);   /* empty batch */
    puts(ok ? "oracle sanitizer run: ok" : "oracle sanitizer run: FAILED");
    return ok ? 0 : 1;
}
