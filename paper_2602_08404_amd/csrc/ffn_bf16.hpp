// Internal declarations shared by the host side (ffn_bf16.hip) and the kernel instantiations
// (ffn_bf16_kernel.hip, compiled once per hidden size) of the bf16 grouped expert FFN.
#pragma once
#include "device_utils.hpp"
#include "kernels.hpp"

namespace team {

constexpr int FFN_THREADS = 256;
constexpr int FFN_WAVES = 4;
constexpr int FFN_MAX_E = 256;
constexpr int FFN_LAYER_MAX_TOKENS = 128;    // up to this many tokens (and FFN_LAYER_MAX_ROWS pairs) the kernel can group the routing table itself
constexpr int FFN_LAYER_MAX_ROWS = 1024;
static_assert(FFN_THREADS == FFN_MAX_E && FFN_LAYER_MAX_ROWS % FFN_THREADS == 0, "the in-kernel grouping maps one thread to one expert");
constexpr int FFN_MAX_DEVICES = 64;      // devices the per-device launch tables hold
constexpr int FFN_DONE_STRIDE = 64;      // one counter per 256 bytes: polled counters sit in different memory channels

// Control block of one FFN launch (in the caller's workspace); must be all zero when the kernel starts (the words
// ffn_ctrl_zero() names: a kernel earlier in the same call clears them).
struct FfnCtrl {
    int32_t reserved[16];
    int32_t done[FFN_MAX_E][FFN_DONE_STRIDE];   // [slot][0]: gate/up items of the slot that have published their part of h
};

struct FfnArgs {
    const uint16_t* x;
    const int32_t* offsets;
    const int32_t* sorted_token;
    const int32_t* active;
    const int32_t* n_active;
    const void* wg;             // bf16 elements, or E4M3 codes when sg / su / sd are given
    const void* wu;
    const void* wd;
    const float* sg = nullptr;  // 8-bit weights: one scale per row of w_gate [E,I], w_up [E,I], w_down [E,H]
    const float* su = nullptr;
    const float* sd = nullptr;
    uint16_t* h;
    float* out;
    FfnCtrl* ctrl;
    const int32_t* topk_idx;    // non-null: group this routing table in the kernel (offsets .. n_active are then unused)
    int32_t* inv_pos_out;       // with topk_idx: [T,k] rows of the pairs, written for the combine kernel
    int T, k, E;
    int device;                 // current device (index into the per-device tables of the launchers)
    int n_cu;                   // compute units of that device
    int grid_override;          // > 0: use a smaller grid than the resident maximum (tuning aid)
    int spin_limit;
    int cooperative;            // measurement aid: launch through hipLaunchCooperativeKernel
    int skip_publish;           // tests only: gate/up items do not publish, so every wait for them gives up
    unsigned long long* fail_mark;   // workspace word that receives WS_FAIL_MARK when a wait gives up (see kernels.hpp)
    int tiled_min_avg_rows;     // > 0: switch to the streaming variant when the call averages at least this many rows per expert
    int wide_min_avg_rows;      // streaming variant: above this many rows per expert on average, two token tiles per wavefront
    int expert_major;           // 1: shares that would cross expert boundaries are replaced by whole workgroups per expert (see the kernel)
    hipStream_t stream;
};

// KSA = hidden / 128; dispatches on ksb = inter / 128.
template <int KSA>
hipError_t launch_ffn_fused_ksa(const FfnArgs& p, int ksb);

extern template hipError_t launch_ffn_fused_ksa<2>(const FfnArgs&, int);
extern template hipError_t launch_ffn_fused_ksa<4>(const FfnArgs&, int);
extern template hipError_t launch_ffn_fused_ksa<8>(const FfnArgs&, int);
extern template hipError_t launch_ffn_fused_ksa<16>(const FfnArgs&, int);
// 8-bit weights (hidden 1024 or 2048; inter a multiple of 256): same dispatch.
template <int KSA>
hipError_t launch_ffn_fused_w8_ksa(const FfnArgs& p, int ksb);
extern template hipError_t launch_ffn_fused_w8_ksa<8>(const FfnArgs&, int);
extern template hipError_t launch_ffn_fused_w8_ksa<16>(const FfnArgs&, int);

}  // namespace team
