// Host side of the bf16 grouped expert FFN: shape support, control-block layout, launch.
#include "ffn_bf16.hpp"

#include <stddef.h>

#include <atomic>

#include "tuning.hpp"

namespace team {

// Compute units of a device, asked once per device.
static int compute_units(int dev) {
    static std::atomic<int> n_cu_of[FFN_MAX_DEVICES];
    int n_cu = n_cu_of[dev].load(std::memory_order_relaxed);
    if (n_cu == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess) n_cu = prop.multiProcessorCount;
        if (n_cu <= 0) n_cu = 256;
        n_cu_of[dev].store(n_cu, std::memory_order_relaxed);
    }
    return n_cu;
}

size_t ffn_ctrl_bytes() { return sizeof(FfnCtrl); }
CtrlZero ffn_ctrl_zero(void* ctrl) { return CtrlZero{(int32_t*)ctrl, 16, FFN_DONE_STRIDE}; }
static_assert(offsetof(FfnCtrl, done) == 16 * sizeof(int32_t), "header of the control block is 16 words");

bool ffn_bf16_supported(int H, int I) {
    const bool h_ok = H == 256 || H == 512 || H == 1024 || H == 2048;
    const bool i_ok = I % 128 == 0 && I >= 128 && I <= 1024;
    return h_ok && i_ok;
}

bool ffn_w8_supported(int H, int I) { return (H == 1024 || H == 2048) && I % 256 == 0 && I >= 256 && I <= 1024; }

bool ffn_bf16_groups_itself(const Dims& d) {
    return d.bf16 && d.T <= FFN_LAYER_MAX_TOKENS && d.T * d.k <= FFN_LAYER_MAX_ROWS && d.E <= FFN_MAX_E && ffn_bf16_supported(d.H, d.I);
}

static hipError_t launch_common(const Dims& d, FfnArgs& p, hipStream_t s) {
    p.T = d.T; p.k = d.k; p.E = d.E;
    if (!p.fail_mark) return hipErrorInvalidValue;
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= FFN_MAX_DEVICES) return hipErrorInvalidDevice;
    p.device = dev;
    p.n_cu = compute_units(dev);
    const Tuning& tn = tuning();
    p.grid_override = tn.ffn_grid.load();             // tuning aid only; never raises the grid above what is resident
    p.spin_limit = tn.ffn_spin_limit.load();          // ~0.1 s of polling by default; see the waits in the kernel
    p.skip_publish = tn.ffn_skip_publish.load();
    p.cooperative = tn.ffn_cooperative.load();
    // With at most 32 tokens per call an expert has at most 32 rows: one pass of the register-resident token operand, which is
    // reused across the expert's items.  Beyond that the kernel decides on the device from the average number of rows per expert.
    p.tiled_min_avg_rows = d.T > 32 ? tn.ffn_tiled_rows.load() : 0;
    p.wide_min_avg_rows = tn.ffn_wide_rows.load();
    p.expert_major = tn.ffn_shares.load() == 0 ? 0 : (tn.ffn_shares.load() == 2 ? 2 : 1);
    p.stream = s;
    if (p.sg) {                       // 8-bit weights
        if (!p.su || !p.sd || !ffn_w8_supported(d.H, d.I)) return hipErrorInvalidValue;
        return d.H == 2048 ? launch_ffn_fused_w8_ksa<16>(p, d.I / 128) : launch_ffn_fused_w8_ksa<8>(p, d.I / 128);
    }
    switch (d.H / 128) {
        case 2: return launch_ffn_fused_ksa<2>(p, d.I / 128);
        case 4: return launch_ffn_fused_ksa<4>(p, d.I / 128);
        case 8: return launch_ffn_fused_ksa<8>(p, d.I / 128);
        case 16: return launch_ffn_fused_ksa<16>(p, d.I / 128);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_ffn_bf16(const Dims& d, const uint16_t* x, const int32_t* offsets, const int32_t* sorted_token, const int32_t* active,
                           const int32_t* n_active, const void* wg, const void* wu, const void* wd, void* ctrl,
                           unsigned long long* fail_mark, uint16_t* h_ws, float* expert_out, hipStream_t s, const W8Scales* w8) {
    if (!ffn_bf16_supported(d.H, d.I) || d.E > FFN_MAX_E) return hipErrorInvalidValue;
    FfnArgs p;
    if (w8) { p.sg = w8->gate; p.su = w8->up; p.sd = w8->down; }
    p.x = x; p.offsets = offsets; p.sorted_token = sorted_token; p.active = active; p.n_active = n_active;
    p.wg = wg; p.wu = wu; p.wd = wd; p.h = h_ws; p.out = expert_out; p.ctrl = (FfnCtrl*)ctrl; p.fail_mark = fail_mark;
    p.topk_idx = nullptr; p.inv_pos_out = nullptr;
    return launch_common(d, p, s);
}

hipError_t launch_ffn_bf16_from_routing(const Dims& d, const uint16_t* x, const int32_t* topk_idx, int32_t* inv_pos_out,
                                        const void* wg, const void* wu, const void* wd, void* ctrl, unsigned long long* fail_mark,
                                        uint16_t* h_ws, float* expert_out, hipStream_t s, const W8Scales* w8) {
    if (!ffn_bf16_groups_itself(d)) return hipErrorInvalidValue;
    FfnArgs p;
    if (w8) { p.sg = w8->gate; p.su = w8->up; p.sd = w8->down; }
    p.x = x; p.offsets = nullptr; p.sorted_token = nullptr; p.active = nullptr; p.n_active = nullptr;
    p.wg = wg; p.wu = wu; p.wd = wd; p.h = h_ws; p.out = expert_out; p.ctrl = (FfnCtrl*)ctrl; p.fail_mark = fail_mark;
    p.topk_idx = topk_idx; p.inv_pos_out = inv_pos_out;
    return launch_common(d, p, s);
}

// ---- control block cleared by a launch of its own (staged calls, where no other kernel of the call precedes the FFN kernel)
__global__ __launch_bounds__(FFN_MAX_E) void ffn_ctrl_clear_kernel(CtrlZero cz, int E) {
    const int tid = threadIdx.x;
    if (tid < cz.header) cz.words[tid] = 0;
    if (tid < E) cz.words[cz.header + tid * cz.stride] = 0;
}

hipError_t launch_ffn_ctrl_clear(void* ctrl, int E, hipStream_t s) {
    if (E < 1 || E > FFN_MAX_E) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ffn_ctrl_clear_kernel, dim3(1), dim3(FFN_MAX_E), 0, s, ffn_ctrl_zero(ctrl), E);
    return hipGetLastError();
}

// ---- the 8-bit weight format as this library reads it (also what the FFN kernel's operands are widened with)
__global__ __launch_bounds__(256) void dequantize_w8_kernel(const uint8_t* __restrict__ codes, const float* __restrict__ scale,
                                                            long long rows, long long cols, float* __restrict__ out) {
    const long long chunks_per_row = cols / 16;
    const long long c = (long long)blockIdx.x * 256 + threadIdx.x;
    if (c >= rows * chunks_per_row) return;
    const long long row = c / chunks_per_row;
    const bf16x8_t raw = *reinterpret_cast<const bf16x8_t*>(codes + c * 16);
    bf16x8_t lo, hi;
    widen_e4m3(raw, lo, hi);
    const float sc = scale[row];
    float* o = out + c * 16;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        o[i] = (float)lo[i] * sc;
        o[8 + i] = (float)hi[i] * sc;
    }
}

hipError_t launch_dequantize_w8(const uint8_t* codes, const float* scale, long long rows, long long cols, float* out, hipStream_t s) {
    if (rows < 1 || cols < 16 || cols % 16 != 0) return hipErrorInvalidValue;
    const long long chunks = rows * (cols / 16);
    const long long blocks = (chunks + 255) / 256;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dequantize_w8_kernel, dim3((unsigned)blocks), dim3(256), 0, s, codes, scale, rows, cols, out);
    return hipGetLastError();
}

}  // namespace team
