/*
 * CPU oracle for the TEAM MoE-layer hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition the HIP kernels are checked against.  It is used by the tests,
 * by the smoke check and by the benchmark's CPU-baseline leg; the product path never calls it and shares
 * no code, header, table or constant with it.
 *
 * What it computes (paper: Algorithm 1 "Limited Activation for cold tokens" and its prose in Section
 * "Limited Activation for Cold Tokens (LAC)"; Section "Mixture-of-Experts" of Related Work for the
 * per-token gating of a MoE layer): for every token of a diffusion block, independently,
 *
 *   logit[e] = sum_h x[h] * W_r[e][h]                        router score of expert e
 *   S        = experts allowed by the activated-expert mask  (Router(C, E_A): routing confined to E_A)
 *   sel      = the k_eff = min(k,|S|) experts of S with the largest logit, ties to the lower id
 *   gate     = softmax over the selected logits              (renormalised top-k gates), or, without
 *              renormalisation, the selected entries of the softmax over all experts
 *   y        = sum_s gate[s] * W_d[sel_s] ( silu(W_g[sel_s] x) * (W_u[sel_s] x) ),  silu(z) = z/(1+exp(-z))
 *
 * and the grouping of (token, slot) assignments by expert that the GPU path needs as an intermediate
 * (counts, exclusive offsets, rows of one expert ordered by token id).
 *
 * Arithmetic: inputs are fp32 values (bf16-stored tensors are widened exactly before they get here);
 * every sum is accumulated in double, in ascending index order, with no blocking or reordering.  The one
 * place floating point decides an integer - which experts are selected - is decided on the logit rounded
 * to fp32, the precision the kernels select in.
 *
 * oracle_route_two_round is Algorithm 1 itself (first-round tokens over all experts, E_A = union of their picks,
 * cold tokens inside E_A); oracle_classify_tokens is its step 1 (hot/cold classification, Eq. 4).
 * oracle_row_representatives names, for every row of a call, the first row with exactly the same stored bytes (candidate
 * branches of Section "Speculative Exploration for Hot Tokens (SEH)" repeat most rows of the base branch); a layer that
 * computes each distinct row once must return what oracle_moe_layer returns for all rows.
 *
 * Pins (tests/test_oracle_pins.py): hand-worked example (tests/golden), dense-SwiGLU special case,
 * mask-free top-k MoE written separately, brute-force subset enumeration, superset invariance from
 * Algorithm 1, sub-model equivalence, permutation equivariance, closed forms, and an independent NumPy
 * implementation.  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double silu(double z) { return z / (1.0 + exp(-z)); }

static double dot(const float *a, const float *b, int n) {
    double acc = 0.0;
    for (int i = 0; i < n; ++i) acc += (double)a[i] * (double)b[i];
    return acc;
}

/* logits[t,e] for all tokens; each rounded once to fp32. */
void oracle_router_logits(const float *x, const float *w_router, int T, int H, int E, float *logits) {
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e) logits[(size_t)t * E + e] = (float)dot(x + (size_t)t * H, w_router + (size_t)e * H, H);
}

/* Order of the selection: a larger logit ranks first; a NaN logit ranks below every number, -infinity included (the paper
 * says nothing about non-finite scores; with this reading a NaN is taken only when fewer than k_eff numbers are allowed, and
 * the token's gates then come out NaN by the arithmetic below, so a broken input shows in the output instead of vanishing).
 * Equal logits (+0 and -0 are equal) and two NaNs do not rank before each other: the caller keeps the lower id. */
static int ranks_before(float a, float b) {
    if (isnan(b)) return !isnan(a);
    return a > b;
}

/* Selection and gates of ONE token from its fp32 logits.
 * idx[k]: selected expert ids in order (logit descending, id ascending), -1 padded.
 * gate[k]: routing weights in the same order, 0 padded.  Returns k_eff.
 * Non-finite logits: the formulas are evaluated as they stand in IEEE arithmetic (exp(inf - inf) and anything with a NaN
 * give NaN gates for the token). */
static int route_token(const float *logit, int E, int k, int renormalize, const uint8_t *mask, int32_t *idx, double *gate) {
    int n_allowed = 0;
    for (int e = 0; e < E; ++e) n_allowed += (mask == NULL || mask[e] != 0);
    int k_eff = k < n_allowed ? k : n_allowed;
    for (int s = 0; s < k; ++s) { idx[s] = -1; gate[s] = 0.0; }
    for (int s = 0; s < k_eff; ++s) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            if (mask != NULL && mask[e] == 0) continue;
            int taken = 0;
            for (int j = 0; j < s; ++j) taken |= (idx[j] == e);
            if (taken) continue;
            if (best < 0 || ranks_before(logit[e], logit[best])) best = e;   /* strict order keeps the lower id on ties */
        }
        idx[s] = best;
    }
    if (k_eff == 0) return 0;
    if (renormalize) {
        double m = (double)logit[idx[0]], den = 0.0;
        for (int s = 0; s < k_eff; ++s) den += exp((double)logit[idx[s]] - m);
        for (int s = 0; s < k_eff; ++s) gate[s] = exp((double)logit[idx[s]] - m) / den;
    } else {
        double m = (double)logit[0], den = 0.0;
        for (int e = 1; e < E; ++e) if ((double)logit[e] > m) m = (double)logit[e];
        for (int e = 0; e < E; ++e) den += exp((double)logit[e] - m);
        for (int s = 0; s < k_eff; ++s) gate[s] = exp((double)logit[idx[s]] - m) / den;
    }
    return k_eff;
}

/* Routing of all tokens from given logits. */
void oracle_route_from_logits(const float *logits, int T, int E, int k, int renormalize, const uint8_t *mask,
                              int32_t *topk_idx, double *topk_gate) {
    for (int t = 0; t < T; ++t)
        route_token(logits + (size_t)t * E, E, k, renormalize, mask, topk_idx + (size_t)t * k, topk_gate + (size_t)t * k);
}

/* Two-round routing (Algorithm 1, "Limited Activation for cold tokens").
 * Round 1: tokens with first_round[t] != 0 (newly accepted tokens D_a and hot tokens H) are routed over all experts E_0.
 * E_A = union over those tokens of their selected experts (mask_out[e] = 1 for e in E_A, else 0).
 * Round 2: the remaining (cold) tokens are routed inside E_A.  W = Concat(W_1, W_2): one row per token, in token order. */
void oracle_route_two_round(const float *logits, int T, int E, int k, int renormalize, const uint8_t *first_round,
                            uint8_t *mask_out, int32_t *topk_idx, double *topk_gate) {
    for (int e = 0; e < E; ++e) mask_out[e] = 0;
    for (int t = 0; t < T; ++t) {
        if (!first_round[t]) continue;
        route_token(logits + (size_t)t * E, E, k, renormalize, NULL, topk_idx + (size_t)t * k, topk_gate + (size_t)t * k);
        for (int s = 0; s < k; ++s)
            if (topk_idx[(size_t)t * k + s] >= 0) mask_out[topk_idx[(size_t)t * k + s]] = 1;
    }
    for (int t = 0; t < T; ++t) {
        if (first_round[t]) continue;
        route_token(logits + (size_t)t * E, E, k, renormalize, mask_out, topk_idx + (size_t)t * k, topk_gate + (size_t)t * k);
    }
}

/* Classification of the live tokens of a step (Algorithm 1, step 1; hot tokens as in Eq. 4 of Section "Speculative Exploration
 * for Hot Tokens"; its distance condition is read with Section "Experimental Setup": a masked token is hot if its confidence
 * exceeds tau_h or if some decoded token of its block lies within L_h positions, L_h included).
 *   state[p]: 0 masked, 1 decoded in an earlier step, 2 newly accepted in the previous step; conf[p]: confidence of the
 *   current decoding attempt (used for masked positions only); positions p of one block are the rows
 *   [b*block_len, (b+1)*block_len) and distances are taken inside a block.
 *   token_class[t] for the live row p = live_index[t] (or p = t when live_index is NULL):
 *     1 = takes part in the first routing round (newly accepted, or masked and hot; a row decoded earlier that is listed
 *         anyway is routed freely as well), 0 = cold. */
void oracle_classify_tokens(const float *conf, const uint8_t *state, int n_rows, int block_len, const int32_t *live_index, int T,
                            float tau_h, int L_h, uint8_t *token_class) {
    for (int t = 0; t < T; ++t) {
        int p = live_index ? live_index[t] : t;
        if (p < 0 || p >= n_rows) { token_class[t] = 0; continue; }     /* not a row: nothing to route freely */
        if (state[p] != 0) { token_class[t] = 1; continue; }
        int hot = conf[p] > tau_h;
        int b0 = (p / block_len) * block_len, b1 = b0 + block_len;
        if (b1 > n_rows) b1 = n_rows;
        for (int j = b0; j < b1 && !hot; ++j)
            if (state[j] != 0) {
                int d = p > j ? p - j : j - p;
                if (d <= L_h) hot = 1;
            }
        token_class[t] = (uint8_t)hot;
    }
}

/* Output of one expert for one token: out[H] = W_d ( silu(W_g x) * (W_u x) ); hbuf is I doubles of scratch. */
static void expert_ffn_token(const float *x, int H, int I, const float *w_gate, const float *w_up, const float *w_down,
                             double *hbuf, double *out) {
    for (int i = 0; i < I; ++i) {
        double g = dot(w_gate + (size_t)i * H, x, H);
        double u = dot(w_up + (size_t)i * H, x, H);
        hbuf[i] = silu(g) * u;
    }
    for (int h = 0; h < H; ++h) {
        double acc = 0.0;
        const float *row = w_down + (size_t)h * I;
        for (int i = 0; i < I; ++i) acc += (double)row[i] * hbuf[i];
        out[h] = acc;
    }
}

/* Expert outputs per (token, slot): o[t,s,:] for the given selection; rows of padded slots are zero. */
void oracle_expert_rows(const float *x, int T, int H, int I, int k, const float *w_gate, const float *w_up,
                        const float *w_down, const int32_t *topk_idx, double *o, int threads) {
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#endif
    (void)threads;
#pragma omp parallel
    {
        double *hbuf = (double *)malloc(sizeof(double) * (size_t)I);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < T * k; ++r) {
            int t = r / k;
            int e = topk_idx[r];
            double *out = o + (size_t)r * H;
            if (e < 0) { memset(out, 0, sizeof(double) * (size_t)H); continue; }
            size_t we = (size_t)e * I * H;
            expert_ffn_token(x + (size_t)t * H, H, I, w_gate + we, w_up + we, w_down + we, hbuf, out);
        }
        free(hbuf);
    }
}

/* y[t,:] = sum over slots s ascending of gate[t,s] * o[t,s,:]. */
void oracle_combine(const double *o, const double *topk_gate, const int32_t *topk_idx, int T, int k, int H, double *y) {
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int s = 0; s < k; ++s)
                if (topk_idx[(size_t)t * k + s] >= 0) acc += topk_gate[(size_t)t * k + s] * o[((size_t)t * k + s) * H + h];
            y[(size_t)t * H + h] = acc;
        }
}

/* Grouping of assignments by expert: counts -> exclusive offsets[E+1]; rows of expert e are its tokens in
 * ascending token id; inv_pos[t,s] is the row of assignment (t,s) (-1 for padded slots); active_experts lists
 * the experts with at least one row in ascending id, padded with -1 up to E. */
void oracle_dispatch(const int32_t *topk_idx, int T, int k, int E, int32_t *offsets, int32_t *sorted_token,
                     int32_t *inv_pos, int32_t *active_experts, int32_t *n_active) {
    for (int e = 0; e <= E; ++e) offsets[e] = 0;
    for (int r = 0; r < T * k; ++r) { inv_pos[r] = -1; sorted_token[r] = -1; }
    for (int r = 0; r < T * k; ++r)
        if (topk_idx[r] >= 0) offsets[topk_idx[r] + 1] += 1;
    for (int e = 0; e < E; ++e) offsets[e + 1] += offsets[e];
    int na = 0;
    for (int e = 0; e < E; ++e) {
        int pos = offsets[e];
        for (int t = 0; t < T; ++t)
            for (int s = 0; s < k; ++s)
                if (topk_idx[(size_t)t * k + s] == e) { sorted_token[pos] = t; inv_pos[(size_t)t * k + s] = pos; ++pos; }
        if (offsets[e + 1] > offsets[e]) active_experts[na++] = e;
    }
    for (int i = na; i < E; ++i) active_experts[i] = -1;
    *n_active = na;
}

/* The whole layer, token by token, straight from the definition (no grouping). */
void oracle_moe_layer(const float *x, int T, int H, int E, int k, int I, int renormalize, const float *w_router,
                      const float *w_gate, const float *w_up, const float *w_down, const uint8_t *mask,
                      double *y, int32_t *topk_idx, double *topk_gate, int threads) {
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#endif
    (void)threads;
#pragma omp parallel
    {
        float *logit = (float *)malloc(sizeof(float) * (size_t)E);
        double *hbuf = (double *)malloc(sizeof(double) * (size_t)I);
        double *out = (double *)malloc(sizeof(double) * (size_t)H);
#pragma omp for schedule(dynamic, 1)
        for (int t = 0; t < T; ++t) {
            const float *xt = x + (size_t)t * H;
            for (int e = 0; e < E; ++e) logit[e] = (float)dot(xt, w_router + (size_t)e * H, H);
            int32_t *idx = topk_idx + (size_t)t * k;
            double *gate = topk_gate + (size_t)t * k;
            int k_eff = route_token(logit, E, k, renormalize, mask, idx, gate);
            double *yt = y + (size_t)t * H;
            for (int h = 0; h < H; ++h) yt[h] = 0.0;
            for (int s = 0; s < k_eff; ++s) {
                size_t we = (size_t)idx[s] * I * H;
                expert_ffn_token(xt, H, I, w_gate + we, w_up + we, w_down + we, hbuf, out);
                for (int h = 0; h < H; ++h) yt[h] += gate[s] * out[h];
            }
        }
        free(logit); free(hbuf); free(out);
    }
}

/* Section "Speculative Exploration for Hot Tokens (SEH)" / "Aligned Token Candidates in SEH": the extra branches are the
 * base block with one or two more positions accepted, so a call over several branches may hold the same row more than
 * once.  rep[t] = the smallest j <= t whose row consists of exactly the same row_bytes bytes as row t (stored bits, so
 * +0 and -0 differ and equal NaN patterns match). */
void oracle_row_representatives(const void *x, int T, int row_bytes, int32_t *rep) {
    const unsigned char *rows = (const unsigned char *)x;
    for (int t = 0; t < T; ++t) {
        rep[t] = t;
        for (int j = 0; j < t; ++j) {
            if (memcmp(rows + (size_t)j * row_bytes, rows + (size_t)t * row_bytes, (size_t)row_bytes) == 0) {
                rep[t] = j;
                break;
            }
        }
    }
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
