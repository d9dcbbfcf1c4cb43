// Host-side launchers of the MoE-layer kernels (internal; the public boundary is include/team_moe.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace team {

struct Dims {
    int T, H, I, E, k;
    int bf16;          // 1: bf16 storage, 0: float storage
    int renormalize;
    // Token t of the call lives in row row_index[t] of the caller's x and y tensors, which have n_rows rows
    // (row_index == nullptr: row t; the call's tensors are dense [T,H]).  The router's logits kernel reads x through the
    // index and leaves a dense [T,H] copy of the live rows in x_dense for the expert FFN; the combine kernel writes y
    // through the index.
    const int32_t* row_index = nullptr;
    int n_rows = 0;
    void* x_dense = nullptr;
    // Repeated rows (row_rep != nullptr): row_rep[t] is the first token whose row holds the same bytes as token t's.  Only
    // tokens with row_rep[t] == t are routed and computed; the combine kernel gives every token the result of row_rep[t].
    const int32_t* row_rep = nullptr;
};

// Search for repeated rows inside the router (hash == nullptr: off).  The logits kernel writes a 64-bit hash of every row and
// clears *n_unique; the selection kernel of token t compares hashes with the tokens before it, confirms a match byte by byte,
// writes rep[t], counts the tokens that are their own representative and leaves the routing table of the others empty.
// With a live-row index the rows compared are those of the dense copy (Dims::x_dense).  Under two-round routing a repeated
// first-round row still contributes its picks to E_A, so the result of every token is the one it would get without the search.
struct RowDedup {
    unsigned long long* hash = nullptr;   // [T]
    int32_t* rep = nullptr;               // [T]
    int32_t* n_unique = nullptr;          // [1]
    unsigned long long hash_mask = ~0ull; // bits of the hash that are compared (fewer bits: more byte-wise confirmations)
};

// The first WS_STATUS_BYTES of a workspace are its status area.  Word 0 is the failure mark: a kernel whose bounded wait
// for another workgroup gives up stores WS_FAIL_MARK there (and fills the outputs it could not compute with NaN); nothing
// but team_moe_workspace_status ever resets it, so the mark survives later calls.  A workspace that was never used holds
// arbitrary bytes there; the mark is a 64-bit pattern so that such bytes are not mistaken for it.
constexpr size_t WS_STATUS_BYTES = 256;
constexpr unsigned long long WS_FAIL_MARK = 0x5445414d4641494cull;

// Words of the FFN control block that must be zero before an FFN launch: `header` leading words, then one word
// every `stride` words for each of the E expert slots.
struct CtrlZero {
    int32_t* words;     // nullptr: nothing to clear
    int header, stride;
};
// logits: [T,E] floats, required (scratch of the selection kernel and, for the caller, the router scores).
// ctrl: control block the selection kernel also clears for an expert FFN that follows without a dispatch kernel.
hipError_t launch_route(const Dims& d, const void* x, const void* w_router, const uint8_t* mask, int32_t* topk_idx,
                        float* topk_gate, float* logits, CtrlZero ctrl, hipStream_t s, RowDedup dedup = RowDedup());
// Two-round routing (Algorithm 1): tokens with token_class != 0 are routed over all experts, E_A = union of their picks,
// the other tokens are routed inside E_A.  state: 256 bytes of device memory (cleared by the call); mask_out [E] bytes and
// n_activated_out [1] may be null.  T <= 1024.
hipError_t launch_route_two_round(const Dims& d, const void* x, const void* w_router, const uint8_t* token_class, uint8_t* mask_out,
                                  int32_t* n_activated_out, int32_t* topk_idx, float* topk_gate, float* logits, void* state,
                                  CtrlZero ctrl, hipStream_t s, RowDedup dedup = RowDedup());
// Hot/cold classification of live tokens (Algorithm 1 step 1, Eq. 4): token_class[t] = 1 first-round, 0 cold.
hipError_t launch_classify_tokens(const float* conf, const uint8_t* state, int n_rows, int block_len, const int32_t* live_index, int T,
                                  float tau_h, int L_h, uint8_t* token_class, hipStream_t s);
// ctrl: control block the dispatch kernel also clears for the expert FFN that follows (words == nullptr: none).
hipError_t launch_dispatch(const Dims& d, const int32_t* topk_idx, int32_t* offsets, int32_t* sorted_token,
                           int32_t* inv_pos, int32_t* active, int32_t* n_active, CtrlZero ctrl, hipStream_t s);
hipError_t launch_combine(const Dims& d, const float* expert_out, const float* gate, const int32_t* inv_pos, void* y,
                          hipStream_t s);
// fp32 storage: plain-ALU grouped FFN.
hipError_t launch_ffn_f32(const Dims& d, const float* x, const int32_t* offsets, const int32_t* sorted_token,
                          const int32_t* active, const int32_t* n_active, const float* wg, const float* wu,
                          const float* wd, float* h_ws, float* expert_out, hipStream_t s);
// bf16 storage: MFMA grouped FFN streaming the weights of the active experts.
// ctrl: ffn_ctrl_bytes() of scratch for the kernel's per-expert counters; the words ffn_ctrl_zero() names must be
// zero when the kernel starts (the dispatch kernel clears them).
// 8-bit weights: E4M3 codes in the same [E,I,H] / [E,H,I] layouts plus one float scale per matrix row (w = code value x scale).
struct W8Scales {
    const float* gate;   // [E,I]
    const float* up;     // [E,I]
    const float* down;   // [E,H]
};
bool ffn_w8_supported(int H, int I);
// codes [rows, cols] (cols a multiple of 16), scale [rows] -> out [rows, cols] floats; the conversion the FFN kernel uses.
hipError_t launch_dequantize_w8(const uint8_t* codes, const float* scale, long long rows, long long cols, float* out, hipStream_t s);
bool ffn_bf16_supported(int H, int I);
size_t ffn_ctrl_bytes();
CtrlZero ffn_ctrl_zero(void* ctrl);
// fail_mark: the workspace's failure mark (see WS_FAIL_MARK).
hipError_t launch_ffn_bf16(const Dims& d, const uint16_t* x, const int32_t* offsets, const int32_t* sorted_token,
                           const int32_t* active, const int32_t* n_active, const void* wg, const void* wu,
                           const void* wd, void* ctrl, unsigned long long* fail_mark, uint16_t* h_ws, float* expert_out, hipStream_t s,
                           const W8Scales* w8 = nullptr);
// Clears the words ffn_ctrl_zero() names with a one-workgroup launch of its own (the staged team_moe_expert_ffn: no other
// kernel of that call runs before the FFN kernel).
hipError_t launch_ffn_ctrl_clear(void* ctrl, int E, hipStream_t s);
// Whole-layer form for small calls: the FFN kernel groups the routing table (topk_idx) itself and writes inv_pos for
// the combine kernel; no dispatch kernel is needed.  ffn_bf16_groups_itself says whether a call qualifies.
bool ffn_bf16_groups_itself(const Dims& d);
hipError_t launch_ffn_bf16_from_routing(const Dims& d, const uint16_t* x, const int32_t* topk_idx, int32_t* inv_pos_out,
                                        const void* wg, const void* wu, const void* wd, void* ctrl, unsigned long long* fail_mark,
                                        uint16_t* h_ws, float* expert_out, hipStream_t s, const W8Scales* w8 = nullptr);

}  // namespace team
