/*
 * team_moe.h - C ABI of the MI355X (gfx950) MoE-layer forward used by TEAM-style block-diffusion decoding.
 *
 * One call of team_moe_layer_forward is one MoE layer of one denoising step over the live tokens of a
 * diffusion block (and of its speculative branches), with expert routing confined to a per-step
 * activated-expert set E_A.  The operation is the one TEAM's Algorithm 1 ("Limited Activation for cold
 * tokens") hands to the model: Router(tokens, E_A) -> routing weights W, then the experts of E_A applied to
 * their tokens and summed with W (Section "Limited Activation for Cold Tokens (LAC)"; the per-token top-k
 * gating of a MoE layer is the standard one the paper assumes in Section "Related work / Mixture-of-Experts").
 * The paper targets the memory-bound regime of block decoding (Section "Delayed Caching for Decoded Tokens")
 * where each activated expert serves few tokens (Section "Speculative Exploration for Hot Tokens"), so the
 * cost of a call is the bytes of the experts that receive at least one token; experts outside E_A, and
 * experts of E_A no token selects, are never read.
 *
 * Conventions for every entry point
 *   - `cfg` and `bytes` are HOST pointers.  Every other pointer is a DEVICE pointer owned by the caller
 *     (hipMalloc / PyTorch-ROCm storage), 16-byte aligned.  The library never allocates, frees or keeps
 *     them.  Scratch comes from the caller's `workspace` (>= team_moe_workspace_size bytes, 256-B aligned).
 *   - `stream` is a hipStream_t (NULL = default stream).  Calls only enqueue kernels and return; there is no
 *     host synchronisation and no host read of device data.
 *   - Tensors are row-major and dense.  x [T,H], w_router [E,H], w_gate and w_up [E,I,H], w_down [E,H,I],
 *     y [T,H]: all in cfg->dtype (TEAM_BF16: bfloat16 bit patterns; TEAM_F32: float).  Accumulation, router
 *     logits, gates and expert_out are always float.
 *   - Return value is a team_status.  Arguments are validated on the host before anything is launched:
 *     NULL required pointer, T < 1, T > cfg->max_tokens, sizes out of range -> TEAM_ERR_INVALID_ARG;
 *     shapes the kernels do not tile -> TEAM_ERR_UNSUPPORTED; workspace too small -> TEAM_ERR_WORKSPACE;
 *     a launch the runtime rejects -> TEAM_ERR_HIP.  On error nothing has been enqueued.
 *   - Results are deterministic: same inputs give bit-identical outputs (no floating-point atomics).
 *   - Calls that share a workspace must be ordered on one stream (or otherwise serialised).
 *   - One expert-FFN launch per device at a time.  team_moe_expert_ffn and every team_moe_layer_forward* call run one
 *     persistent kernel whose grid fills the whole device and whose workgroups wait for each other (the down projection of an
 *     expert starts when its gate/up projection is complete).  Two such kernels in flight on one device at once - calls on
 *     different streams, or from different processes - can keep each other's workgroups off the compute units they need.
 *     The waits are bounded (about 0.1 s): a wait that gives up marks the workspace (team_moe_workspace_status), and the
 *     rows it could not compute are stored as NaN, so the failure cannot pass for a result.  Order such calls on one stream,
 *     or serialise them, and they never wait longer than the producers take to run.
 *   - Router scores that are not numbers.  The paper leaves them undefined; here a NaN score ranks below every number (ties
 *     by the lower expert id, as for equal numbers), so it is selected only when fewer than top_k numbers are allowed, and
 *     the gates are the softmax formulas evaluated in IEEE arithmetic: a token that selects a NaN or an infinite score gets
 *     NaN gates and a NaN row of y; with renormalize == 0 a NaN score anywhere in the token's row does the same.
 *
 * Limits: 1 <= top_k <= 16, top_k <= num_experts <= 256, max_tokens <= 1024.
 *   TEAM_BF16: hidden in {256,512,1024,2048}, inter a multiple of 128 with inter <= 1024.
 *   TEAM_F32 : hidden and inter multiples of 4.
 */
#ifndef TEAM_MOE_H
#define TEAM_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TEAM_OK = 0,
    TEAM_ERR_INVALID_ARG = -1,
    TEAM_ERR_UNSUPPORTED = -2,
    TEAM_ERR_WORKSPACE = -3,
    TEAM_ERR_HIP = -4,
    TEAM_ERR_TIMEOUT = -5        /* only from team_moe_workspace_status: a wait inside a kernel gave up */
} team_status;

typedef enum { TEAM_F32 = 0, TEAM_BF16 = 1 } team_dtype;

typedef struct {
    int32_t hidden;       /* H */
    int32_t inter;        /* I, SwiGLU intermediate size of one expert */
    int32_t num_experts;  /* E = |E_0| */
    int32_t top_k;        /* k, experts per token */
    int32_t dtype;        /* team_dtype of x, weights and y */
    int32_t renormalize;  /* 1: gates = softmax over the selected logits (sum to 1);
                             0: gates = the selected entries of the softmax over all E experts */
    int32_t max_tokens;   /* largest T any call with this cfg will pass (sizes the workspace) */
    int32_t reserved;     /* must be 0 */
} team_moe_config;

/* Bytes of workspace that team_moe_layer_forward (and every other entry point) needs for `cfg`.  The contents of a
 * workspace need no initialisation. */
int team_moe_workspace_size(const team_moe_config* cfg, size_t* bytes);

/*
 * Has a kernel that used `workspace` given up a wait for another workgroup since the last call of this function?  (See
 * "One expert-FFN launch per device at a time" above; in correct use the answer is always no.)
 * Unlike every other entry point this one SYNCHRONISES: it waits for the work queued on `stream` (a hipStream_t), reads
 * the first bytes of the workspace (its status area, the same for every configuration: ws_bytes >= 256), and, if it finds
 * the failure mark, removes it.  Returns TEAM_OK (no failure), TEAM_ERR_TIMEOUT (a wait gave up: the outputs of that call
 * hold NaN in the rows that could not be computed; the mark is removed, so a failure is reported once),
 * TEAM_ERR_WORKSPACE (bad pointer or size) or TEAM_ERR_HIP (the copy failed).  It does not allocate.
 * workspace == NULL asks about the static array that team_moe_layer_forward_static uses on the current device.
 * A workspace that was never passed to a kernel holds arbitrary bytes; they are not mistaken for the mark (a 64-bit pattern).
 */
int team_moe_workspace_status(void* workspace, size_t ws_bytes, void* stream);

/*
 * Router restricted to the activated-expert set (Algorithm 1, "Router(C, E_A)"; with expert_mask == NULL it
 * is the first-round router over all experts E_0).
 *   logit[t,e] = sum_h x[t,h] * w_router[e,h]               (float accumulation)
 *   S = { e : expert_mask == NULL or expert_mask[e] != 0 },  k_eff = min(top_k, |S|)
 *   topk_idx[t, 0..k_eff)  = the k_eff experts of S with the largest logit, largest first, ties to the lower
 *                            id; remaining slots are -1
 *   topk_gate[t, s]        = routing weight of slot s (see cfg->renormalize); 0 in padded slots
 *   logits_out [T,E]       = the logits, if the caller wants them; with NULL they are kept in `workspace`
 *                            (required then: team_moe_workspace_size bytes; may be NULL when logits_out is given)
 * An all-zero mask gives topk_idx = -1 and gates 0 everywhere.  Scores that are not numbers: see the conventions above.
 * The signature has two arguments more than the five-call outline of the layer (workspace, ws_bytes): the selection kernel
 * reads the scores back, so they need a place when the caller does not ask for them.
 */
int team_moe_route(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router,
                   const uint8_t* expert_mask /* [E] bytes or NULL */, int32_t* topk_idx /* [T,k] */,
                   float* topk_gate /* [T,k] */, float* logits_out /* [T,E] or NULL */, void* workspace,
                   size_t ws_bytes, void* stream);

/*
 * Token-to-expert grouping of the routing table.  The paper leaves this step implicit; Section "Speculative Exploration
 * for Hot Tokens (SEH)" describes its result, a handful of tokens per activated expert.  Integer only, bit-exact.
 *   expert_offsets[E+1]  exclusive prefix sum of the number of (token,slot) pairs assigned to each expert
 *   sorted_token[T*k]    token id of every row, rows of one expert contiguous and in ascending token id;
 *                        entries beyond expert_offsets[E] are -1
 *   inv_pos[T,k]         row of pair (t,s) in that order, -1 for padded slots
 *   active_experts[E]    ids of the experts with at least one row, ascending, padded with -1
 *   n_active[1]          their number
 * Entries of topk_idx outside [0,E) are treated as padding.
 * `workspace` / `ws_bytes` are not used (the grouping works in on-chip memory only); pass NULL / 0 or anything else.
 */
int team_moe_build_dispatch(const team_moe_config* cfg, const int32_t* topk_idx, int32_t T,
                            int32_t* expert_offsets, int32_t* sorted_token, int32_t* inv_pos,
                            int32_t* active_experts, int32_t* n_active, void* workspace, size_t ws_bytes,
                            void* stream);

/*
 * Grouped SwiGLU expert FFN over the experts listed in active_experts only: the step whose cost the paper's method
 * reduces.  Section "Delayed Caching for Decoded Tokens" places block decoding in the memory-bound regime and Section
 * "Speculative Exploration for Hot Tokens (SEH)" attributes the latency to the feed-forward layers, each activated expert
 * serving few tokens: the time of this call is the time to read the listed experts' weights once.
 * For every row p in [expert_offsets[e], expert_offsets[e+1]) of an active expert e, with t = sorted_token[p]:
 *   g = w_gate[e] x[t],  u = w_up[e] x[t],  h = silu(g) * u  (silu(z) = z / (1 + exp(-z))),
 *   expert_out[p,:] = w_down[e] h                              (float, [T*k, H]; rows >= expert_offsets[E]
 *                                                               are left untouched)
 * TEAM_BF16: products on bf16 MFMA with float accumulation; h is rounded to bf16 between the two GEMMs.
 * Weights of experts that are not listed are not read.
 * `workspace`: team_moe_workspace_size bytes (the call uses its first part: status area, control block, h).  The call
 * is self-contained: it prepares what it needs in the workspace itself and may be repeated, or follow any other call.
 * If a wait inside the kernel gives up (see the conventions), the rows of expert_out it could not compute are NaN.
 */
int team_moe_expert_ffn(const team_moe_config* cfg, const void* x, int32_t T, const int32_t* expert_offsets,
                        const int32_t* sorted_token, const int32_t* active_experts, const int32_t* n_active,
                        const void* w_gate, const void* w_up, const void* w_down, float* expert_out,
                        void* workspace, size_t ws_bytes, void* stream);

/*
 * Gate-weighted combine with the routing weights W that Algorithm 1 returns (Concat(W_1, W_2)): y[t,:] = sum_{s ascending, inv_pos[t,s] >= 0} topk_gate[t,s] * expert_out[inv_pos[t,s],:]
 * in float, then cast to cfg->dtype (round to nearest even).  Tokens with no valid slot get y = 0.
 */
int team_moe_combine(const team_moe_config* cfg, const float* expert_out, const float* topk_gate,
                     const int32_t* inv_pos, int32_t T, void* y, void* stream);

/*
 * The whole layer on one stream: route -> build_dispatch -> expert_ffn -> combine, all intermediates in
 * `workspace`.  y [T,H] in cfg->dtype.  This is the MoE layer of one denoising step with routing confined to the
 * activated set: Algorithm 1's "Router(C, E_A)" followed by the experts of E_A weighted with W (Section "Limited
 * Activation for Cold Tokens (LAC)"); expert_mask == NULL is the unrestricted layer of the baseline decoder.
 */
int team_moe_layer_forward(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router,
                           const void* w_gate, const void* w_up, const void* w_down,
                           const uint8_t* expert_mask, void* y, void* workspace, size_t ws_bytes, void* stream);

/*
 * team_moe_layer_forward for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The intermediates live in a static array of
 * TEAM_MOE_STATIC_SCRATCH_BYTES bytes of device memory that is part of the library's code object (every GPU the library runs
 * on holds its own copy until the process ends); the call allocates and frees nothing.  Same arguments, results and errors as
 * team_moe_layer_forward, except: a configuration whose team_moe_workspace_size exceeds TEAM_MOE_STATIC_SCRATCH_BYTES is
 * rejected with TEAM_ERR_WORKSPACE (the 32-token and 128-token configurations of a 2048 x 768 x 128-expert layer fit; 256
 * tokens do not), and failing to locate the array on the current device gives TEAM_ERR_HIP.  All calls on one GPU share the
 * array: calls that overlap in time on one GPU (different streams or threads) race on it and must be serialised by the caller.
 * Nothing in the array has to survive from one call to the next.
 */
#define TEAM_MOE_STATIC_SCRATCH_BYTES (16u << 20)
int team_moe_layer_forward_static(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router,
                                  const void* w_gate, const void* w_up, const void* w_down,
                                  const uint8_t* expert_mask, void* y, void* stream);

/*
 * Step 1 of Algorithm 1: classification of the live tokens of a denoising step (Eq. 4 of Section "Speculative Exploration for
 * Hot Tokens (SEH)"; where Eq. 4's strict, universally quantified distance condition and the wording of Section "Experimental
 * Setup" differ, the latter is followed: some decoded row within L_h positions, L_h itself included).
 *   conf  [n_rows] float : confidence c_k of the current decoding attempt of every row (read for masked rows only)
 *   state [n_rows] bytes : 0 = masked, 1 = decoded in an earlier step, 2 = newly accepted in the previous step (D_a)
 *   rows [b*block_len, (b+1)*block_len) form one block (or one speculative branch of it); distances are taken inside a block
 *   live_index [T] int32 : the rows that are computed in this step (masked and newly accepted ones), or NULL for rows 0..T-1
 *   token_class [T] bytes: 1 = first-round token: newly accepted, or masked and hot, i.e. conf > tau_h (strictly) or a row of
 *                          its block with state != 0 at distance <= L_h; 0 = cold token.  A listed row that was decoded earlier
 *                          is classed 1 (routed freely); a listed index outside [0, n_rows) is classed 0.
 * The output is what team_moe_route_two_round / team_moe_layer_forward_two_round take as token_class.
 * Needs no cfg and no workspace.  n_rows, block_len, T >= 1, L_h >= 0, tau_h not NaN, else TEAM_ERR_INVALID_ARG.
 */
int team_moe_classify_tokens(const float* conf, const uint8_t* state, int32_t n_rows, int32_t block_len,
                             const int32_t* live_index /* [T] or NULL */, int32_t T, float tau_h, int32_t L_h,
                             uint8_t* token_class /* [T] */, void* stream);

/*
 * Two-round routing of Algorithm 1 ("Limited Activation for cold tokens") in one call.
 *   token_class [T] bytes: non-zero = first-round token (a newly accepted token of D_a or a hot token of H, which may
 *                          activate experts); zero = cold token of C.
 *   first round: every first-round token is routed over all experts E_0 exactly as team_moe_route with expert_mask == NULL;
 *   E_A     = the union of the experts those tokens selected;
 *   second round: every cold token is routed exactly as team_moe_route with expert_mask = E_A.
 *   topk_idx / topk_gate [T,k]: W = Concat(W_1, W_2), one row per token in token order, same conventions as
 *                               team_moe_route (cold tokens have min(k, |E_A|) valid slots).
 *   activated_mask_out [E] bytes (1 = in E_A) and n_activated_out [1] (= |E_A|): optional, may be NULL.
 *   logits_out [T,E]: optional as in team_moe_route.
 * With no first-round token E_A is empty and every cold token gets topk_idx = -1, gate 0.
 * `workspace` is required (team_moe_workspace_size bytes, 256-byte aligned): it holds E_A while it is being built.
 */
int team_moe_route_two_round(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router,
                             const uint8_t* token_class /* [T] */, uint8_t* activated_mask_out /* [E] or NULL */,
                             int32_t* n_activated_out /* [1] or NULL */, int32_t* topk_idx /* [T,k] */,
                             float* topk_gate /* [T,k] */, float* logits_out /* [T,E] or NULL */, void* workspace,
                             size_t ws_bytes, void* stream);

/*
 * team_moe_layer_forward with the routing step replaced by team_moe_route_two_round: the MoE layer of one denoising
 * step under Algorithm 1, E_A decided on the device from the tokens' classes.  Only experts of E_A can be read.
 */
int team_moe_layer_forward_two_round(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router,
                                     const void* w_gate, const void* w_up, const void* w_down,
                                     const uint8_t* token_class /* [T] */, uint8_t* activated_mask_out /* [E] or NULL */,
                                     int32_t* n_activated_out /* [1] or NULL */, void* y, void* workspace,
                                     size_t ws_bytes, void* stream);

/*
 * The layer over the live rows of larger tensors, without a gather by the caller (Section "Delayed Caching for Decoded
 * Tokens": a step computes the masked rows and the rows accepted one step earlier; rows decoded before that keep what was
 * cached for them).
 *   x_rows, y_rows [n_rows, H] in cfg->dtype; row_index [T] int32 lists the rows this call computes: token t of the call
 *   reads x_rows[row_index[t]] and writes y_rows[row_index[t]].  Rows that are not listed are neither read nor written.
 *   Entries outside [0, n_rows) are clamped into that range on the device; if a row is listed twice, which of the two equal
 *   results is stored last is not defined.
 * Routing: with token_class == NULL as in team_moe_layer_forward (expert_mask may be NULL), otherwise as in
 * team_moe_layer_forward_two_round (expert_mask must then be NULL); token_class, like every per-token table, is indexed by
 * the position t in row_index.  activated_mask_out / n_activated_out are written in the two-round mode only (optional).
 * T <= cfg->max_tokens; n_rows is only bounded by the tensors.
 */
int team_moe_layer_forward_rows(const team_moe_config* cfg, const void* x_rows, void* y_rows, int32_t n_rows,
                                const int32_t* row_index /* [T] */, int32_t T, const void* w_router, const void* w_gate,
                                const void* w_up, const void* w_down, const uint8_t* expert_mask /* [E] or NULL */,
                                const uint8_t* token_class /* [T] or NULL */, uint8_t* activated_mask_out /* [E] or NULL */,
                                int32_t* n_activated_out /* [1] or NULL */, void* workspace, size_t ws_bytes, void* stream);

/*
 * team_moe_layer_forward for calls that hold the same row more than once (Section "Speculative Exploration for Hot Tokens
 * (SEH)" and "Aligned Token Candidates in SEH": the extra branches are the base block with one or two more positions
 * accepted, so where rows do not yet depend on each other most rows of a multi-branch call repeat the base branch).
 * Every distinct row is routed and run through its experts once; repeated rows receive a copy of that result.
 *   Two rows are the same when all their stored bytes are equal (so +0 and -0 differ).  The router finds them on the
 *   device: a hash per row, then a byte-wise comparison of rows whose hashes match.
 *   row_rep_out [T] int32 or NULL: row_rep_out[t] = the first token whose row equals token t's (t itself if none before).
 *   n_unique_out [1] int32 or NULL: number of distinct rows.
 * y is what team_moe_layer_forward returns for the same arguments, up to the rounding differences between the kernel
 * variants the two calls may choose (the choice depends on the number of rows per expert); y[t] and y[row_rep[t]] are
 * bit-identical.  Routing is single-round (expert_mask may be NULL).
 */
int team_moe_layer_forward_unique_rows(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router,
                                       const void* w_gate, const void* w_up, const void* w_down,
                                       const uint8_t* expert_mask /* [E] or NULL */, void* y,
                                       int32_t* row_rep_out /* [T] or NULL */, int32_t* n_unique_out /* [1] or NULL */,
                                       void* workspace, size_t ws_bytes, void* stream);

/*
 * 8-bit expert weights (a variant outside the paper: it halves the bytes the memory-bound path of Section "Delayed Caching for
 * Decoded Tokens" / "Speculative Exploration for Hot Tokens (SEH)" has to read).  Storage: w_*_q hold OCP E4M3 codes (1 sign,
 * 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest magnitude 448) in the layouts of the bf16 weights
 * ([E,I,H], [E,I,H], [E,H,I]); scale_gate [E,I], scale_up [E,I], scale_down [E,H] hold one float per matrix row; the weight a
 * code stands for is (value of the code) x (scale of its row).  x, h, the router weights and y stay as in the bf16 configuration
 * (cfg->dtype must be TEAM_BF16; hidden 1024 or 2048, inter a multiple of 256); products are formed on bf16 operands (every
 * E4M3 value is a bf16 value) with float accumulation, and the row scale multiplies the finished sum.
 *
 * team_moe_expert_ffn_w8 / team_moe_layer_forward_w8: as team_moe_expert_ffn / team_moe_layer_forward, with these weights.
 * team_moe_dequantize_w8: out[r, c] = value(codes[r, c]) * scale[r] as float, for a [rows, cols] matrix (cols a multiple of 16;
 *   codes and out 16-byte aligned) - the conversion the expert FFN applies to its operands, exposed for checking a quantiser.
 */
int team_moe_expert_ffn_w8(const team_moe_config* cfg, const void* x, int32_t T, const int32_t* expert_offsets,
                           const int32_t* sorted_token, const int32_t* active_experts, const int32_t* n_active,
                           const uint8_t* w_gate_q, const uint8_t* w_up_q, const uint8_t* w_down_q, const float* scale_gate,
                           const float* scale_up, const float* scale_down, float* expert_out, void* workspace,
                           size_t ws_bytes, void* stream);
int team_moe_layer_forward_w8(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router,
                              const uint8_t* w_gate_q, const uint8_t* w_up_q, const uint8_t* w_down_q,
                              const float* scale_gate, const float* scale_up, const float* scale_down,
                              const uint8_t* expert_mask /* [E] or NULL */, void* y, void* workspace, size_t ws_bytes,
                              void* stream);
int team_moe_dequantize_w8(const uint8_t* codes, const float* scale, int64_t rows, int64_t cols, float* out, void* stream);

/*
 * One denoising step's MoE layer with the variants above combined, as the decoding loop of the paper uses them together
 * (Sections "Delayed Caching for Decoded Tokens", "Limited Activation for Cold Tokens (LAC)" / Algorithm 1, and "Speculative
 * Exploration for Hot Tokens (SEH)"): live rows of the block's tensors, the activated set from a mask or from the tokens'
 * classes on the device, bf16 or 8-bit expert weights, repeated rows computed once.  All pointers are device pointers unless
 * stated; every field that a variant does not use must be NULL / 0.
 */
typedef struct {
    const void* x;                  /* [T,H], or [n_rows,H] when row_index is given */
    void* y;                        /* same shape as x; only the rows of the call are written */
    int32_t T;                      /* tokens of the call */
    int32_t n_rows;                 /* rows of x and y when row_index is given, else 0 */
    const int32_t* row_index;       /* [T] rows of x / y that the call computes, or NULL: rows 0..T-1 (team_moe_layer_forward_rows) */
    const void* w_router;           /* [E,H] in cfg->dtype */
    const void* w_gate;             /* [E,I,H] in cfg->dtype, or E4M3 codes when the scales are given */
    const void* w_up;               /* [E,I,H] */
    const void* w_down;             /* [E,H,I] */
    const float* scale_gate;        /* [E,I]; all three scale tables or none (team_moe_layer_forward_w8) */
    const float* scale_up;          /* [E,I] */
    const float* scale_down;        /* [E,H] */
    const uint8_t* expert_mask;     /* [E] or NULL; must be NULL when token_class is given */
    const uint8_t* token_class;     /* [T] or NULL: two-round routing (team_moe_layer_forward_two_round) */
    uint8_t* activated_mask_out;    /* [E] or NULL; written in the two-round mode */
    int32_t* n_activated_out;       /* [1] or NULL; written in the two-round mode */
    int32_t unique_rows;            /* 1: compute repeated rows once (team_moe_layer_forward_unique_rows).  With row_index the rows
                                       compared are the live rows, and row_rep_out holds positions in the call (0..T-1), not rows
                                       of x.  With token_class every first-round token, repeated or not, contributes its picks to
                                       the activated set, so each token's result is the one it gets without the search (a row's
                                       first occurrence may be cold and a later one first-round: the picks of that row then lie
                                       inside the set, and routing confined to the set equals free routing for it) */
    int32_t reserved;               /* must be 0 */
    int32_t* row_rep_out;           /* [T] or NULL; written when unique_rows */
    int32_t* n_unique_out;          /* [1] or NULL; written when unique_rows */
    void* workspace;                /* team_moe_workspace_size(cfg) bytes, 256-byte aligned */
    size_t ws_bytes;
    void* stream;                   /* hipStream_t */
    void* ffn_begin_event;          /* both NULL, or two hipEvent_t created by the caller: recorded on `stream` directly before and */
    void* ffn_end_event;            /* after the expert FFN kernel of this call, so that a caller can time that kernel inside the layer */
} team_moe_layer_args;

/* `args` is a host pointer and is not retained.  Returns a team_status; unsupported combinations: TEAM_ERR_INVALID_ARG. */
int team_moe_layer_forward_ex(const team_moe_config* cfg, const team_moe_layer_args* args);

/* Static, NUL-terminated description of a team_status value. */
const char* team_moe_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TEAM_MOE_H */
