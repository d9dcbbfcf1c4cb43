// C-ABI boundary of the MoE layer (declared in include/team_moe.h): argument validation on the host,
// workspace carving, and kernel launches on the caller's stream.  No allocation, no synchronisation.
#include "../../include/team_moe.h"

#include "kernels.hpp"
#include "tuning.hpp"

#include <stdio.h>
#include <stdlib.h>

#include <atomic>

namespace {

using team::Dims;

constexpr int MAX_TOKENS = 1024;
constexpr int MAX_EXPERTS = 256;
constexpr int MAX_TOPK = 16;

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_cfg(const team_moe_config* c) {
    if (!c) return TEAM_ERR_INVALID_ARG;
    if (c->dtype != TEAM_F32 && c->dtype != TEAM_BF16) return TEAM_ERR_INVALID_ARG;
    if (c->reserved != 0) return TEAM_ERR_INVALID_ARG;
    if (c->renormalize != 0 && c->renormalize != 1) return TEAM_ERR_INVALID_ARG;
    if (c->hidden < 1 || c->inter < 1 || c->num_experts < 1 || c->top_k < 1 || c->max_tokens < 1) return TEAM_ERR_INVALID_ARG;
    if (c->top_k > c->num_experts) return TEAM_ERR_INVALID_ARG;
    if (c->top_k > MAX_TOPK || c->num_experts > MAX_EXPERTS || c->max_tokens > MAX_TOKENS) return TEAM_ERR_UNSUPPORTED;
    if (c->dtype == TEAM_BF16) {
        if (!team::ffn_bf16_supported(c->hidden, c->inter)) return TEAM_ERR_UNSUPPORTED;
    } else {
        if (c->hidden % 4 != 0 || c->inter % 4 != 0) return TEAM_ERR_UNSUPPORTED;
    }
    return TEAM_OK;
}

int check_T(const team_moe_config* c, int32_t T) { return (T < 1 || T > c->max_tokens) ? TEAM_ERR_INVALID_ARG : TEAM_OK; }

Dims dims_of(const team_moe_config* c, int32_t T) {
    Dims d;
    d.T = T; d.H = c->hidden; d.I = c->inter; d.E = c->num_experts; d.k = c->top_k;
    d.bf16 = c->dtype == TEAM_BF16;
    d.renormalize = c->renormalize;
    return d;
}

// Workspace layout, sized for max_tokens.  The status area comes first (team_moe_workspace_status reads it without knowing
// the configuration), then the expert FFN's scratch (control block, h), so that team_moe_expert_ffn and
// team_moe_layer_forward agree on where it is.
struct Layout {
    size_t status, ctrl, h, logits, topk_idx, topk_gate, offsets, sorted_token, inv_pos, active, n_active, expert_out, two_round, x_dense, row_hash, row_rep, n_unique, total;
};
Layout layout_of(const team_moe_config* c) {
    const size_t A = (size_t)c->max_tokens * c->top_k;
    const size_t elem = c->dtype == TEAM_BF16 ? 2 : 4;
    Layout L;
    size_t off = 0;
    L.status = off;       off += team::WS_STATUS_BYTES;
    L.ctrl = off;         off += align256(team::ffn_ctrl_bytes());
    L.h = off;            off += align256(A * c->inter * elem);
    L.logits = off;       off += align256((size_t)c->max_tokens * c->num_experts * 4);
    L.topk_idx = off;     off += align256(A * 4);
    L.topk_gate = off;    off += align256(A * 4);
    L.offsets = off;      off += align256(((size_t)c->num_experts + 1) * 4);
    L.sorted_token = off; off += align256(A * 4);
    L.inv_pos = off;      off += align256(A * 4);
    L.active = off;       off += align256((size_t)c->num_experts * 4);
    L.n_active = off;     off += 256;
    L.expert_out = off;   off += align256(A * c->hidden * 4);
    L.two_round = off;    off += 256;                       // bit set E_A of two-round routing (calls of more than 256 tokens)
    L.x_dense = off;      off += align256((size_t)c->max_tokens * c->hidden * elem);   // live rows gathered by the router (row-index calls)
    L.row_hash = off;     off += align256((size_t)c->max_tokens * 8);                  // repeated-row search of the router
    L.row_rep = off;      off += align256((size_t)c->max_tokens * 4);
    L.n_unique = off;     off += 256;
    L.total = off;
    return L;
}

// Launch errors are read with hipGetLastError(), which also reports errors left behind by earlier, unrelated
// runtime calls of the process; every entry point clears that state before its first launch.
inline void clear_stale_error() { (void)hipGetLastError(); }
inline int hip_status(hipError_t e) {
    if (e == hipSuccess) return TEAM_OK;
    if (getenv("TEAM_MOE_DEBUG")) fprintf(stderr, "team_moe: HIP error %d (%s)\n", (int)e, hipGetErrorString(e));
    return TEAM_ERR_HIP;
}

int run_ffn(const team_moe_config* cfg, const Dims& d, const void* x, const int32_t* offsets, const int32_t* sorted_token,
            const int32_t* active, const int32_t* n_active, const void* wg, const void* wu, const void* wd, float* expert_out,
            void* ctrl, unsigned long long* fail_mark, void* h_ws, hipStream_t s, const team::W8Scales* w8 = nullptr) {
    if (cfg->dtype == TEAM_BF16)
        return hip_status(team::launch_ffn_bf16(d, (const uint16_t*)x, offsets, sorted_token, active, n_active, wg, wu, wd, ctrl,
                                                fail_mark, (uint16_t*)h_ws, expert_out, s, w8));
    if (w8) return TEAM_ERR_UNSUPPORTED;
    return hip_status(team::launch_ffn_f32(d, (const float*)x, offsets, sorted_token, active, n_active, (const float*)wg,
                                           (const float*)wu, (const float*)wd, (float*)h_ws, expert_out, s));
}

}  // namespace

extern "C" {

int team_moe_workspace_size(const team_moe_config* cfg, size_t* bytes) {
    if (!bytes) return TEAM_ERR_INVALID_ARG;
    int st = check_cfg(cfg);
    if (st != TEAM_OK) return st;
    *bytes = layout_of(cfg).total;
    return TEAM_OK;
}

int team_moe_route(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router, const uint8_t* expert_mask,
                   int32_t* topk_idx, float* topk_gate, float* logits_out, void* workspace, size_t ws_bytes, void* stream) {
    int st = check_cfg(cfg);
    if (st != TEAM_OK) return st;
    if ((st = check_T(cfg, T)) != TEAM_OK) return st;
    if (!x || !w_router || !topk_idx || !topk_gate) return TEAM_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_router)) return TEAM_ERR_INVALID_ARG;
    if (cfg->hidden % (cfg->dtype == TEAM_BF16 ? 8 : 4) != 0) return TEAM_ERR_UNSUPPORTED;
    float* logits = logits_out;
    if (!logits) {                       // the scores live in the workspace when the caller does not want them
        const Layout L = layout_of(cfg);
        if (!workspace || !aligned16(workspace) || ws_bytes < L.topk_idx) return TEAM_ERR_WORKSPACE;
        logits = (float*)((char*)workspace + L.logits);
    } else if (!aligned16(logits)) {
        return TEAM_ERR_INVALID_ARG;
    }
    clear_stale_error();
    return hip_status(team::launch_route(dims_of(cfg, T), x, w_router, expert_mask, topk_idx, topk_gate, logits,
                                         team::CtrlZero{nullptr, 0, 0}, (hipStream_t)stream));
}

int team_moe_build_dispatch(const team_moe_config* cfg, const int32_t* topk_idx, int32_t T, int32_t* expert_offsets,
                            int32_t* sorted_token, int32_t* inv_pos, int32_t* active_experts, int32_t* n_active, void* workspace,
                            size_t ws_bytes, void* stream) {
    int st = check_cfg(cfg);
    if (st != TEAM_OK) return st;
    if ((st = check_T(cfg, T)) != TEAM_OK) return st;
    if (!topk_idx || !expert_offsets || !sorted_token || !inv_pos || !active_experts || !n_active) return TEAM_ERR_INVALID_ARG;
    (void)workspace;                     // the grouping needs no scratch outside LDS
    (void)ws_bytes;
    clear_stale_error();
    return hip_status(team::launch_dispatch(dims_of(cfg, T), topk_idx, expert_offsets, sorted_token, inv_pos, active_experts, n_active,
                                            team::CtrlZero{nullptr, 0, 0}, (hipStream_t)stream));
}

namespace {
int check_w8(const team_moe_config* cfg, const team::W8Scales& w8) {
    if (!w8.gate || !w8.up || !w8.down) return TEAM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(w8.gate) | reinterpret_cast<uintptr_t>(w8.up) | reinterpret_cast<uintptr_t>(w8.down)) & 3u)
        return TEAM_ERR_INVALID_ARG;
    if (cfg->dtype != TEAM_BF16 || !team::ffn_w8_supported(cfg->hidden, cfg->inter)) return TEAM_ERR_UNSUPPORTED;
    return TEAM_OK;
}

int expert_ffn(const team_moe_config* cfg, const void* x, int32_t T, const int32_t* expert_offsets,
               const int32_t* sorted_token, const int32_t* active_experts, const int32_t* n_active, const void* w_gate,
               const void* w_up, const void* w_down, float* expert_out, void* workspace, size_t ws_bytes, void* stream,
               const team::W8Scales* w8) {
    int st = check_cfg(cfg);
    if (st != TEAM_OK) return st;
    if ((st = check_T(cfg, T)) != TEAM_OK) return st;
    if (w8 && (st = check_w8(cfg, *w8)) != TEAM_OK) return st;
    if (!x || !expert_offsets || !sorted_token || !active_experts || !n_active || !w_gate || !w_up || !w_down || !expert_out)
        return TEAM_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) || !aligned16(expert_out))
        return TEAM_ERR_INVALID_ARG;
    const Layout L = layout_of(cfg);
    if (!workspace || !aligned16(workspace) || ws_bytes < L.logits /* = end of the control block + h segments */) return TEAM_ERR_WORKSPACE;
    clear_stale_error();
    // The kernel's per-expert counters start from zero: cleared here by a small launch of its own, so that the call depends on
    // nothing that ran before it (inside team_moe_layer_forward the router's selection kernel does it on the way).
    if (cfg->dtype == TEAM_BF16 &&
        (st = hip_status(team::launch_ffn_ctrl_clear((char*)workspace + L.ctrl, cfg->num_experts, (hipStream_t)stream))) != TEAM_OK)
        return st;
    return run_ffn(cfg, dims_of(cfg, T), x, expert_offsets, sorted_token, active_experts, n_active, w_gate, w_up, w_down, expert_out,
                   (char*)workspace + L.ctrl, (unsigned long long*)((char*)workspace + L.status), (char*)workspace + L.h,
                   (hipStream_t)stream, w8);
}
}  // namespace

int team_moe_expert_ffn(const team_moe_config* cfg, const void* x, int32_t T, const int32_t* expert_offsets,
                        const int32_t* sorted_token, const int32_t* active_experts, const int32_t* n_active, const void* w_gate,
                        const void* w_up, const void* w_down, float* expert_out, void* workspace, size_t ws_bytes, void* stream) {
    return expert_ffn(cfg, x, T, expert_offsets, sorted_token, active_experts, n_active, w_gate, w_up, w_down, expert_out, workspace,
                      ws_bytes, stream, nullptr);
}

int team_moe_expert_ffn_w8(const team_moe_config* cfg, const void* x, int32_t T, const int32_t* expert_offsets,
                           const int32_t* sorted_token, const int32_t* active_experts, const int32_t* n_active, const uint8_t* w_gate_q,
                           const uint8_t* w_up_q, const uint8_t* w_down_q, const float* scale_gate, const float* scale_up,
                           const float* scale_down, float* expert_out, void* workspace, size_t ws_bytes, void* stream) {
    const team::W8Scales w8{scale_gate, scale_up, scale_down};
    return expert_ffn(cfg, x, T, expert_offsets, sorted_token, active_experts, n_active, w_gate_q, w_up_q, w_down_q, expert_out, workspace,
                      ws_bytes, stream, &w8);
}

int team_moe_dequantize_w8(const uint8_t* codes, const float* scale, int64_t rows, int64_t cols, float* out, void* stream) {
    if (!codes || !scale || !out) return TEAM_ERR_INVALID_ARG;
    if (rows < 1 || cols < 16 || cols % 16 != 0) return TEAM_ERR_INVALID_ARG;
    if (!aligned16(codes) || !aligned16(out)) return TEAM_ERR_INVALID_ARG;
    clear_stale_error();
    return hip_status(team::launch_dequantize_w8(codes, scale, rows, cols, out, (hipStream_t)stream));
}

int team_moe_combine(const team_moe_config* cfg, const float* expert_out, const float* topk_gate, const int32_t* inv_pos, int32_t T,
                     void* y, void* stream) {
    int st = check_cfg(cfg);
    if (st != TEAM_OK) return st;
    if ((st = check_T(cfg, T)) != TEAM_OK) return st;
    if (!expert_out || !topk_gate || !inv_pos || !y) return TEAM_ERR_INVALID_ARG;
    if (!aligned16(expert_out) || !aligned16(y)) return TEAM_ERR_INVALID_ARG;
    clear_stale_error();
    return hip_status(team::launch_combine(dims_of(cfg, T), expert_out, topk_gate, inv_pos, y, (hipStream_t)stream));
}

int team_moe_route_two_round(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router, const uint8_t* token_class,
                             uint8_t* activated_mask_out, int32_t* n_activated_out, int32_t* topk_idx, float* topk_gate,
                             float* logits_out, void* workspace, size_t ws_bytes, void* stream) {
    int st = check_cfg(cfg);
    if (st != TEAM_OK) return st;
    if ((st = check_T(cfg, T)) != TEAM_OK) return st;
    if (!x || !w_router || !token_class || !topk_idx || !topk_gate) return TEAM_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_router) || (logits_out && !aligned16(logits_out))) return TEAM_ERR_INVALID_ARG;
    if (cfg->hidden % (cfg->dtype == TEAM_BF16 ? 8 : 4) != 0) return TEAM_ERR_UNSUPPORTED;
    const Layout L = layout_of(cfg);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || ws_bytes < L.total) return TEAM_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    float* logits = logits_out ? logits_out : (float*)(ws + L.logits);
    clear_stale_error();
    return hip_status(team::launch_route_two_round(dims_of(cfg, T), x, w_router, token_class, activated_mask_out, n_activated_out,
                                                   topk_idx, topk_gate, logits, ws + L.two_round, team::CtrlZero{nullptr, 0, 0},
                                                   (hipStream_t)stream));
}

int team_moe_classify_tokens(const float* conf, const uint8_t* state, int32_t n_rows, int32_t block_len, const int32_t* live_index,
                             int32_t T, float tau_h, int32_t L_h, uint8_t* token_class, void* stream) {
    if (!conf || !state || !token_class) return TEAM_ERR_INVALID_ARG;
    if (n_rows < 1 || block_len < 1 || T < 1 || L_h < 0) return TEAM_ERR_INVALID_ARG;
    if (!(tau_h == tau_h)) return TEAM_ERR_INVALID_ARG;                 // NaN threshold
    if (!live_index && T > n_rows) return TEAM_ERR_INVALID_ARG;
    clear_stale_error();
    return hip_status(team::launch_classify_tokens(conf, state, n_rows, block_len, live_index, T, tau_h, L_h, token_class,
                                                   (hipStream_t)stream));
}

namespace {

// The whole layer; the routing step is either the single-round router confined to expert_mask (token_class == nullptr) or
// the two-round router driven by token_class.
int layer_forward(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router, const void* w_gate, const void* w_up,
                  const void* w_down, const uint8_t* expert_mask, const uint8_t* token_class, uint8_t* activated_mask_out,
                  int32_t* n_activated_out, void* y, void* workspace, size_t ws_bytes, void* stream,
                  const int32_t* row_index = nullptr, int32_t n_rows = 0, bool unique_rows = false, int32_t* row_rep_out = nullptr,
                  int32_t* n_unique_out = nullptr, const team::W8Scales* w8 = nullptr, hipEvent_t ffn_begin = nullptr,
                  hipEvent_t ffn_end = nullptr) {
    int st = check_cfg(cfg);
    if (st != TEAM_OK) return st;
    if ((st = check_T(cfg, T)) != TEAM_OK) return st;
    if (w8 && (st = check_w8(cfg, *w8)) != TEAM_OK) return st;
    if (!x || !w_router || !w_gate || !w_up || !w_down || !y) return TEAM_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_router) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) || !aligned16(y))
        return TEAM_ERR_INVALID_ARG;
    const Layout L = layout_of(cfg);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || ws_bytes < L.total) return TEAM_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    int32_t* topk_idx = (int32_t*)(ws + L.topk_idx);
    float* topk_gate = (float*)(ws + L.topk_gate);
    int32_t* offsets = (int32_t*)(ws + L.offsets);
    int32_t* sorted_token = (int32_t*)(ws + L.sorted_token);
    int32_t* inv_pos = (int32_t*)(ws + L.inv_pos);
    int32_t* active = (int32_t*)(ws + L.active);
    int32_t* n_active = (int32_t*)(ws + L.n_active);
    float* expert_out = (float*)(ws + L.expert_out);
    float* logits = (float*)(ws + L.logits);
    const void* x_ffn = x;
    Dims d = dims_of(cfg, T);
    d.row_index = row_index;
    d.n_rows = n_rows;
    if (row_index) {                     // the router gathers the live rows once; the expert FFN reads the dense copy
        d.x_dense = ws + L.x_dense;
        x_ffn = d.x_dense;
    }
    team::RowDedup dedup;
    if (unique_rows) {                   // the router finds repeated rows; only the first of each is routed and computed
        dedup.hash = (unsigned long long*)(ws + L.row_hash);
        dedup.rep = row_rep_out ? row_rep_out : (int32_t*)(ws + L.row_rep);
        dedup.n_unique = n_unique_out ? n_unique_out : (int32_t*)(ws + L.n_unique);
        const int nb = team::tuning().row_hash_bits.load();            // (tests compare fewer bits to force collisions)
        dedup.hash_mask = nb >= 64 ? ~0ull : (nb <= 0 ? 0ull : ((1ull << nb) - 1ull));
        d.row_rep = dedup.rep;
    }
    hipStream_t s = (hipStream_t)stream;
    clear_stale_error();
    // Small calls (the block-decoding regime): route -> expert FFN -> combine.  The FFN kernel groups the routing table itself
    // (every workgroup, in LDS) and writes inv_pos; the selection kernel clears the FFN's control block.  Otherwise a dispatch
    // kernel groups the table and clears the control block.
    const bool short_path = team::ffn_bf16_groups_itself(d);
    const team::CtrlZero none{nullptr, 0, 0};
    const team::CtrlZero cz = cfg->dtype == TEAM_BF16 ? team::ffn_ctrl_zero(ws + L.ctrl) : none;
    if (token_class)
        st = hip_status(team::launch_route_two_round(d, x, w_router, token_class, activated_mask_out, n_activated_out, topk_idx,
                                                     topk_gate, logits, ws + L.two_round, short_path ? cz : none, s, dedup));
    else
        st = hip_status(team::launch_route(d, x, w_router, expert_mask, topk_idx, topk_gate, logits, short_path ? cz : none, s, dedup));
    if (st != TEAM_OK) return st;
    unsigned long long* fail_mark = (unsigned long long*)(ws + L.status);
    if (!short_path &&
        (st = hip_status(team::launch_dispatch(d, topk_idx, offsets, sorted_token, inv_pos, active, n_active, cz, s))) != TEAM_OK)
        return st;
    if (ffn_begin && (st = hip_status(hipEventRecord(ffn_begin, s))) != TEAM_OK) return st;
    if (short_path)
        st = hip_status(team::launch_ffn_bf16_from_routing(d, (const uint16_t*)x_ffn, topk_idx, inv_pos, w_gate, w_up, w_down, ws + L.ctrl,
                                                           fail_mark, (uint16_t*)(ws + L.h), expert_out, s, w8));
    else
        st = run_ffn(cfg, d, x_ffn, offsets, sorted_token, active, n_active, w_gate, w_up, w_down, expert_out, ws + L.ctrl, fail_mark,
                     ws + L.h, s, w8);
    if (st != TEAM_OK) return st;
    if (ffn_end && (st = hip_status(hipEventRecord(ffn_end, s))) != TEAM_OK) return st;
    return hip_status(team::launch_combine(d, expert_out, topk_gate, inv_pos, y, s));
}

}  // namespace

int team_moe_layer_forward(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router, const void* w_gate,
                           const void* w_up, const void* w_down, const uint8_t* expert_mask, void* y, void* workspace,
                           size_t ws_bytes, void* stream) {
    return layer_forward(cfg, x, T, w_router, w_gate, w_up, w_down, expert_mask, nullptr, nullptr, nullptr, y, workspace, ws_bytes,
                         stream);
}

// ---- the layer for callers that cannot allocate: the workspace is a static device array ----------------------------------
namespace {

constexpr size_t STATIC_SCRATCH_BYTES = (size_t)TEAM_MOE_STATIC_SCRATCH_BYTES;
constexpr int STATIC_MAX_DEVICES = 64;
// One copy of this array exists on every GPU the library runs on, from the moment its code object is loaded there until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
std::atomic<void*> g_scratch_ptr[STATIC_MAX_DEVICES];      // per device: where that device's copy of `scratch` lives

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return TEAM_ERR_HIP;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_status(e == hipSuccess ? hipErrorInvalidSymbol : e);
        g_scratch_ptr[dev].store(p, std::memory_order_release);      // (two first callers store the same address)
    }
    *out = p;
    return TEAM_OK;
}

}  // namespace

int team_moe_layer_forward_static(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router, const void* w_gate,
                                  const void* w_up, const void* w_down, const uint8_t* expert_mask, void* y, void* stream) {
    int st = check_cfg(cfg);
    if (st != TEAM_OK) return st;
    if (layout_of(cfg).total > STATIC_SCRATCH_BYTES) return TEAM_ERR_WORKSPACE;     // this configuration needs more than the array holds
    void* ws = nullptr;
    if ((st = static_scratch(&ws)) != TEAM_OK) return st;
    return layer_forward(cfg, x, T, w_router, w_gate, w_up, w_down, expert_mask, nullptr, nullptr, nullptr, y, ws, STATIC_SCRATCH_BYTES,
                         stream);
}

int team_moe_layer_forward_two_round(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router, const void* w_gate,
                                     const void* w_up, const void* w_down, const uint8_t* token_class, uint8_t* activated_mask_out,
                                     int32_t* n_activated_out, void* y, void* workspace, size_t ws_bytes, void* stream) {
    if (!token_class) return TEAM_ERR_INVALID_ARG;
    return layer_forward(cfg, x, T, w_router, w_gate, w_up, w_down, nullptr, token_class, activated_mask_out, n_activated_out, y,
                         workspace, ws_bytes, stream);
}

int team_moe_layer_forward_rows(const team_moe_config* cfg, const void* x_rows, void* y_rows, int32_t n_rows, const int32_t* row_index,
                                int32_t T, const void* w_router, const void* w_gate, const void* w_up, const void* w_down,
                                const uint8_t* expert_mask, const uint8_t* token_class, uint8_t* activated_mask_out,
                                int32_t* n_activated_out, void* workspace, size_t ws_bytes, void* stream) {
    if (!row_index || n_rows < 1) return TEAM_ERR_INVALID_ARG;
    if (expert_mask && token_class) return TEAM_ERR_INVALID_ARG;       // one routing mode per call
    return layer_forward(cfg, x_rows, T, w_router, w_gate, w_up, w_down, expert_mask, token_class, activated_mask_out, n_activated_out,
                         y_rows, workspace, ws_bytes, stream, row_index, n_rows);
}

int team_moe_layer_forward_unique_rows(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router, const void* w_gate,
                                       const void* w_up, const void* w_down, const uint8_t* expert_mask, void* y, int32_t* row_rep_out,
                                       int32_t* n_unique_out, void* workspace, size_t ws_bytes, void* stream) {
    return layer_forward(cfg, x, T, w_router, w_gate, w_up, w_down, expert_mask, nullptr, nullptr, nullptr, y, workspace, ws_bytes,
                         stream, nullptr, 0, true, row_rep_out, n_unique_out);
}

int team_moe_layer_forward_w8(const team_moe_config* cfg, const void* x, int32_t T, const void* w_router, const uint8_t* w_gate_q,
                              const uint8_t* w_up_q, const uint8_t* w_down_q, const float* scale_gate, const float* scale_up,
                              const float* scale_down, const uint8_t* expert_mask, void* y, void* workspace, size_t ws_bytes,
                              void* stream) {
    const team::W8Scales w8{scale_gate, scale_up, scale_down};
    return layer_forward(cfg, x, T, w_router, w_gate_q, w_up_q, w_down_q, expert_mask, nullptr, nullptr, nullptr, y, workspace, ws_bytes,
                         stream, nullptr, 0, false, nullptr, nullptr, &w8);
}

int team_moe_layer_forward_ex(const team_moe_config* cfg, const team_moe_layer_args* a) {
    if (!a || a->reserved != 0) return TEAM_ERR_INVALID_ARG;
    const bool rows = a->row_index != nullptr;
    if (rows ? a->n_rows < 1 : a->n_rows != 0) return TEAM_ERR_INVALID_ARG;
    if (a->expert_mask && a->token_class) return TEAM_ERR_INVALID_ARG;                // one routing mode per call
    if (a->unique_rows != 0 && a->unique_rows != 1) return TEAM_ERR_INVALID_ARG;
    if (!a->unique_rows && (a->row_rep_out || a->n_unique_out)) return TEAM_ERR_INVALID_ARG;
    if (!a->token_class && (a->activated_mask_out || a->n_activated_out)) return TEAM_ERR_INVALID_ARG;
    if ((a->ffn_begin_event == nullptr) != (a->ffn_end_event == nullptr)) return TEAM_ERR_INVALID_ARG;      // both events or none
    const bool any_scale = a->scale_gate || a->scale_up || a->scale_down;
    const team::W8Scales w8{a->scale_gate, a->scale_up, a->scale_down};
    return layer_forward(cfg, a->x, a->T, a->w_router, a->w_gate, a->w_up, a->w_down, a->expert_mask, a->token_class,
                         a->activated_mask_out, a->n_activated_out, a->y, a->workspace, a->ws_bytes, a->stream, a->row_index, a->n_rows,
                         a->unique_rows != 0, a->row_rep_out, a->n_unique_out, any_scale ? &w8 : nullptr, (hipEvent_t)a->ffn_begin_event,
                         (hipEvent_t)a->ffn_end_event);
}

int team_moe_workspace_status(void* workspace, size_t ws_bytes, void* stream) {
    void* ws = workspace;
    if (!ws) {                                         // the static array of team_moe_layer_forward_static on the current device
        int st = static_scratch(&ws);
        if (st != TEAM_OK) return st;
    } else if (!aligned16(ws) || ws_bytes < team::WS_STATUS_BYTES) {
        return TEAM_ERR_WORKSPACE;
    }
    hipStream_t s = (hipStream_t)stream;
    clear_stale_error();
    unsigned long long mark = 0ull;
    hipError_t e = hipMemcpyAsync(&mark, ws, sizeof(mark), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_status(e);
    if (mark != team::WS_FAIL_MARK) return TEAM_OK;
    const unsigned long long zero = 0ull;              // reported once: the mark is taken off again
    e = hipMemcpyAsync(ws, &zero, sizeof(zero), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_status(e);
    return TEAM_ERR_TIMEOUT;
}

const char* team_moe_status_string(int status) {
    switch (status) {
        case TEAM_OK: return "ok";
        case TEAM_ERR_INVALID_ARG: return "invalid argument";
        case TEAM_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case TEAM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case TEAM_ERR_HIP: return "HIP runtime rejected a launch";
        case TEAM_ERR_TIMEOUT: return "a wait inside a kernel gave up; the affected outputs hold NaN";
        default: return "unknown status";
    }
}

}  // extern "C"
