// Grouped SwiGLU expert FFN for float storage (the small fp32 configuration): plain fused-multiply-add dot
// products, one wavefront per output element, float accumulation in a fixed order.  The bf16 configurations
// use the MFMA kernels in ffn_bf16.hip; this file exists so the fp32 configuration is computed in fp32.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace team {

constexpr int F32_THREADS = 256;
constexpr int F32_WAVES = F32_THREADS / WAVE;

__device__ __forceinline__ float dot_f32_wave(const float* __restrict__ a, const float* __restrict__ b, int n, int lane) {
    float acc = 0.f;
    for (int c = lane; c < n / 4; c += WAVE) {
        float av[4], bv[4];
        load4(a + 4 * c, av);
        load4(b + 4 * c, bv);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = fmaf(av[j], bv[j], acc);
    }
    return wave_sum(acc);
}

// Rows [r0,r1) of active slot a, clipped to the table; false if the slot is unused or its entry is not an expert id.
__device__ __forceinline__ bool slot_rows(const int32_t* __restrict__ offsets, const int32_t* __restrict__ active,
                                          const int32_t* __restrict__ n_active, int a, int E, int A, int& e, int& r0, int& r1) {
    if (a >= *n_active) return false;
    e = active[a];
    if (e < 0 || e >= E) return false;
    r0 = max(offsets[e], 0);
    r1 = min(offsets[e + 1], A);
    return r1 > r0;
}

// Phase A: h[p,i] = silu(w_gate[e,i,:].x[t]) * (w_up[e,i,:].x[t]) for the rows p of active slot blockIdx.y
__global__ __launch_bounds__(F32_THREADS) void ffn_f32_gate_up(const float* __restrict__ x, const int32_t* __restrict__ offsets,
                                                               const int32_t* __restrict__ sorted_token, const int32_t* __restrict__ active,
                                                               const int32_t* __restrict__ n_active, const float* __restrict__ wg,
                                                               const float* __restrict__ wu, float* __restrict__ h, int T, int k, int H,
                                                               int I, int E) {
    int e, r0, r1;
    if (!slot_rows(offsets, active, n_active, blockIdx.y, E, T * k, e, r0, r1)) return;
    const int lane = threadIdx.x & (WAVE - 1);
    const int i = blockIdx.x * F32_WAVES + threadIdx.x / WAVE;
    if (i >= I) return;
    for (int p = r0; p < r1; ++p) {
        const int t = sorted_token[p];
        if (t < 0 || t >= T) continue;
        const float* xt = x + (size_t)t * H;
        float g = dot_f32_wave(wg + ((size_t)e * I + i) * H, xt, H, lane);
        float u = dot_f32_wave(wu + ((size_t)e * I + i) * H, xt, H, lane);
        if (lane == 0) h[(size_t)p * I + i] = silu_f32(g) * u;
    }
}

// Phase B: expert_out[p,j] = w_down[e,j,:].h[p,:]
__global__ __launch_bounds__(F32_THREADS) void ffn_f32_down(const int32_t* __restrict__ offsets, const int32_t* __restrict__ sorted_token,
                                                            const int32_t* __restrict__ active, const int32_t* __restrict__ n_active,
                                                            const float* __restrict__ wd, const float* __restrict__ h,
                                                            float* __restrict__ out, int T, int k, int H, int I, int E) {
    int e, r0, r1;
    if (!slot_rows(offsets, active, n_active, blockIdx.y, E, T * k, e, r0, r1)) return;
    const int lane = threadIdx.x & (WAVE - 1);
    const int j = blockIdx.x * F32_WAVES + threadIdx.x / WAVE;
    if (j >= H) return;
    for (int p = r0; p < r1; ++p) {
        const int t = sorted_token[p];
        if (t < 0 || t >= T) continue;
        float v = dot_f32_wave(wd + ((size_t)e * H + j) * I, h + (size_t)p * I, I, lane);
        if (lane == 0) out[(size_t)p * H + j] = v;
    }
}

hipError_t launch_ffn_f32(const Dims& d, const float* x, const int32_t* offsets, const int32_t* sorted_token, const int32_t* active,
                          const int32_t* n_active, const float* wg, const float* wu, const float* wd, float* h_ws, float* expert_out,
                          hipStream_t s) {
    hipLaunchKernelGGL(ffn_f32_gate_up, dim3((d.I + F32_WAVES - 1) / F32_WAVES, d.E), dim3(F32_THREADS), 0, s, x, offsets, sorted_token,
                       active, n_active, wg, wu, h_ws, d.T, d.k, d.H, d.I, d.E);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(ffn_f32_down, dim3((d.H + F32_WAVES - 1) / F32_WAVES, d.E), dim3(F32_THREADS), 0, s, offsets, sorted_token, active,
                       n_active, wd, h_ws, expert_out, d.T, d.k, d.H, d.I, d.E);
    return hipGetLastError();
}

}  // namespace team
