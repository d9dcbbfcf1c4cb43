/* Runs every function of the CPU oracle on small inputs, edge cases included, in a build with AddressSanitizer and
 * UndefinedBehaviorSanitizer (tests/test_sanitizers.py compiles oracle/team_moe_oracle.c together with this file).
 * Exit status 0 = the sanitizers had nothing to report and a few invariants hold. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_router_logits(const float *x, const float *w_router, int T, int H, int E, float *logits);
void oracle_route_from_logits(const float *logits, int T, int E, int k, int renormalize, const uint8_t *mask, int32_t *topk_idx,
                              double *topk_gate);
void oracle_route_two_round(const float *logits, int T, int E, int k, int renormalize, const uint8_t *first_round, uint8_t *mask_out,
                            int32_t *topk_idx, double *topk_gate);
void oracle_classify_tokens(const float *conf, const uint8_t *state, int n_rows, int block_len, const int32_t *live_index, int T,
                            float tau_h, int L_h, uint8_t *token_class);
void oracle_expert_rows(const float *x, int T, int H, int I, int k, const float *w_gate, const float *w_up, const float *w_down,
                        const int32_t *topk_idx, double *o, int threads);
void oracle_combine(const double *o, const double *topk_gate, const int32_t *topk_idx, int T, int k, int H, double *y);
void oracle_dispatch(const int32_t *topk_idx, int T, int k, int E, int32_t *offsets, int32_t *sorted_token, int32_t *inv_pos,
                     int32_t *active_experts, int32_t *n_active);
void oracle_moe_layer(const float *x, int T, int H, int E, int k, int I, int renormalize, const float *w_router, const float *w_gate,
                      const float *w_up, const float *w_down, const uint8_t *mask, double *y, int32_t *topk_idx, double *topk_gate,
                      int threads);
void oracle_row_representatives(const void *x, int T, int row_bytes, int32_t *rep);

static uint32_t rng_state = 12345u;
static float rnd(void) {                      /* uniform in [-1, 1) */
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)(rng_state >> 8) / 8388608.0f - 1.0f;
}
static float *randoms(size_t n, float scale) {
    float *p = (float *)malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = rnd() * scale;
    return p;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int one_case(int T, int H, int E, int k, int I, int renorm, int n_allowed, int threads) {
    float *x = randoms((size_t)T * H, 1.f), *wr = randoms((size_t)E * H, 0.3f);
    float *wg = randoms((size_t)E * I * H, 0.3f), *wu = randoms((size_t)E * I * H, 0.3f), *wd = randoms((size_t)E * H * I, 0.3f);
    uint8_t *mask = (uint8_t *)calloc((size_t)E, 1);
    for (int e = 0; e < n_allowed && e < E; ++e) mask[(e * 7) % E] = 1;
    double *y = (double *)malloc(sizeof(double) * T * H), *gate = (double *)malloc(sizeof(double) * T * k);
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * T * k);
    oracle_moe_layer(x, T, H, E, k, I, renorm, wr, wg, wu, wd, n_allowed < 0 ? NULL : mask, y, idx, gate, threads);
    /* staged: logits -> route -> dispatch -> expert rows -> combine gives the same y */
    float *logits = (float *)malloc(sizeof(float) * T * E);
    oracle_router_logits(x, wr, T, H, E, logits);
    int32_t *idx2 = (int32_t *)malloc(sizeof(int32_t) * T * k);
    double *gate2 = (double *)malloc(sizeof(double) * T * k);
    oracle_route_from_logits(logits, T, E, k, renorm, n_allowed < 0 ? NULL : mask, idx2, gate2);
    CHECK(memcmp(idx, idx2, sizeof(int32_t) * T * k) == 0);
    int32_t *offsets = (int32_t *)malloc(sizeof(int32_t) * (E + 1)), *sorted_token = (int32_t *)malloc(sizeof(int32_t) * T * k);
    int32_t *inv_pos = (int32_t *)malloc(sizeof(int32_t) * T * k), *active = (int32_t *)malloc(sizeof(int32_t) * E), n_active = -1;
    oracle_dispatch(idx2, T, k, E, offsets, sorted_token, inv_pos, active, &n_active);
    CHECK(offsets[0] == 0 && offsets[E] <= T * k && n_active >= 0 && n_active <= E);
    double *o = (double *)malloc(sizeof(double) * T * k * H), *y2 = (double *)malloc(sizeof(double) * T * H);
    oracle_expert_rows(x, T, H, I, k, wg, wu, wd, idx2, o, threads);
    oracle_combine(o, gate2, idx2, T, k, H, y2);
    for (int i = 0; i < T * H; ++i) CHECK(fabs(y[i] - y2[i]) <= 1e-12 * (1.0 + fabs(y[i])));
    /* two-round routing with every other token in the first round */
    uint8_t *first = (uint8_t *)malloc((size_t)T), *e_a = (uint8_t *)malloc((size_t)E);
    for (int t = 0; t < T; ++t) first[t] = (uint8_t)(t % 2 == 0);
    oracle_route_two_round(logits, T, E, k, renorm, first, e_a, idx2, gate2);
    for (int t = 0; t < T; ++t)
        for (int s = 0; s < k; ++s)
            if (idx2[t * k + s] >= 0) CHECK(e_a[idx2[t * k + s]] == 1);
    int32_t *rep = (int32_t *)malloc(sizeof(int32_t) * T);
    oracle_row_representatives(x, T, H * (int)sizeof(float), rep);
    for (int t = 0; t < T; ++t) CHECK(rep[t] >= 0 && rep[t] <= t);
    free(x); free(wr); free(wg); free(wu); free(wd); free(mask); free(y); free(gate); free(idx); free(logits); free(idx2); free(gate2);
    free(offsets); free(sorted_token); free(inv_pos); free(active); free(o); free(y2); free(first); free(e_a); free(rep);
    return 0;
}

int main(void) {
    /* T, H, E, k, I, renormalize, allowed experts (-1: no mask), threads */
    if (one_case(5, 8, 6, 2, 4, 1, -1, 1)) return 1;
    if (one_case(5, 8, 6, 2, 4, 0, 3, 2)) return 1;
    if (one_case(1, 4, 1, 1, 4, 1, 1, 1)) return 1;          /* one expert */
    if (one_case(7, 12, 9, 4, 8, 1, 2, 3)) return 1;         /* fewer allowed experts than k */
    if (one_case(3, 4, 5, 3, 4, 1, 0, 1)) return 1;          /* empty activated set: nothing selected, y = 0 */
    if (one_case(3, 4, 5, 5, 4, 0, -1, 1)) return 1;         /* k = E */
    /* scores that are not numbers */
    {
        const float nanv = nanf(""), inf = INFINITY;
        float logits[2][5] = {{nanv, 1.f, nanv, -inf, inf}, {nanv, nanv, nanv, nanv, nanv}};
        int32_t idx[2][3];
        double gate[2][3];
        oracle_route_from_logits(&logits[0][0], 2, 5, 3, 1, NULL, &idx[0][0], &gate[0][0]);
        CHECK(idx[0][0] == 4 && idx[0][1] == 1 && idx[0][2] == 3 && idx[1][0] == 0 && idx[1][1] == 1 && idx[1][2] == 2);
        oracle_route_from_logits(&logits[0][0], 2, 5, 3, 0, NULL, &idx[0][0], &gate[0][0]);
        CHECK(isnan(gate[1][0]));
    }
    /* token classification: block borders, listed rows outside the tensor, reach larger than the block */
    {
        const float conf[8] = {0.1f, 0.9f, 0.2f, 0.3f, 0.95f, 0.1f, 0.1f, 0.69f};
        const uint8_t state[8] = {1, 0, 0, 0, 0, 0, 2, 0};
        const int32_t live[6] = {1, 3, 7, -1, 8, 6};
        uint8_t cls[8];
        oracle_classify_tokens(conf, state, 8, 4, NULL, 8, 0.7f, 1, cls);
        CHECK(cls[0] == 1 && cls[1] == 1 && cls[2] == 0 && cls[3] == 0 && cls[4] == 1 && cls[5] == 1 && cls[6] == 1 && cls[7] == 1);
        oracle_classify_tokens(conf, state, 8, 4, live, 6, 0.7f, 0, cls);
        CHECK(cls[0] == 1 && cls[1] == 0 && cls[2] == 0 && cls[3] == 0 && cls[4] == 0 && cls[5] == 1);
        oracle_classify_tokens(conf, state, 8, 3, NULL, 8, 2.0f, 100, cls);    /* last block is shorter than block_len */
    }
    printf("oracle under sanitizers: ok\n");
    return 0;
}
