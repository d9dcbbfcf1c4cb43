// Gate-weighted combine of the expert outputs: y[t,:] = sum_s gate[t,s] * expert_out[inv_pos[t,s],:].
// These gates are the routing weights W that Algorithm 1 returns.  Slots are summed in ascending order in
// float by one thread per output element group, so the result does not depend on scheduling.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace team {

constexpr int COMBINE_THREADS = 256;
constexpr int C_MAX_K = 16;      // top_k limit of the library

template <bool BF16>
__global__ __launch_bounds__(COMBINE_THREADS) void combine_kernel(const float* __restrict__ expert_out, const float* __restrict__ gate,
                                                                  const int32_t* __restrict__ inv_pos, void* __restrict__ y, int H, int k,
                                                                  const int32_t* __restrict__ row_index, int n_rows,
                                                                  const int32_t* __restrict__ row_rep) {
    const int t = blockIdx.y;
    const int src = row_rep ? row_rep[t] : t;           // token whose expert rows and gates this token's result is made of
    const size_t yrow = (size_t)token_row(row_index, n_rows, t);
    const int h4 = (blockIdx.x * COMBINE_THREADS + threadIdx.x) * 4;
    if (h4 >= H) return;
    // all slot indices and gates first, then all expert rows, then the sum in slot order: the loads of the
    // k rows are in flight together
    int p[C_MAX_K];
    float g[C_MAX_K];
    float4 o[C_MAX_K];
#pragma unroll
    for (int s = 0; s < C_MAX_K; ++s) {
        p[s] = s < k ? inv_pos[(size_t)src * k + s] : -1;
        g[s] = s < k ? gate[(size_t)src * k + s] : 0.f;
    }
#pragma unroll
    for (int s = 0; s < C_MAX_K; ++s)
        o[s] = p[s] >= 0 ? *reinterpret_cast<const float4*>(expert_out + (size_t)p[s] * H + h4) : make_float4(0.f, 0.f, 0.f, 0.f);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int s = 0; s < C_MAX_K; ++s) {
        if (p[s] < 0) continue;
        acc.x = fmaf(g[s], o[s].x, acc.x); acc.y = fmaf(g[s], o[s].y, acc.y); acc.z = fmaf(g[s], o[s].z, acc.z); acc.w = fmaf(g[s], o[s].w, acc.w);
    }
    if (BF16) {
        uint2 packed;
        packed.x = f32_to_bf16_bits(acc.x) | (f32_to_bf16_bits(acc.y) << 16);
        packed.y = f32_to_bf16_bits(acc.z) | (f32_to_bf16_bits(acc.w) << 16);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(y) + yrow * H + h4) = packed;
    } else {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(y) + yrow * H + h4) = acc;
    }
}

hipError_t launch_combine(const Dims& d, const float* expert_out, const float* gate, const int32_t* inv_pos, void* y, hipStream_t s) {
    dim3 grid((d.H / 4 + COMBINE_THREADS - 1) / COMBINE_THREADS, d.T), block(COMBINE_THREADS);
    if (d.bf16)
        hipLaunchKernelGGL(combine_kernel<true>, grid, block, 0, s, expert_out, gate, inv_pos, y, d.H, d.k, d.row_index, d.n_rows, d.row_rep);
    else
        hipLaunchKernelGGL(combine_kernel<false>, grid, block, 0, s, expert_out, gate, inv_pos, y, d.H, d.k, d.row_index, d.n_rows, d.row_rep);
    return hipGetLastError();
}

}  // namespace team
