// Router restricted to the activated-expert set: logits, masked top-k, gates.
// Paper: Algorithm 1, "Router(C, E_A)" (second-round routing confined to the necessary experts) and, with no
// mask, the first-round router over E_0.  One workgroup per token: every wavefront scores a share of the
// experts (dot products reduced across lanes), then wavefront 0 selects the k best allowed experts with
// cross-lane arg-max and turns the selected logits into gates with a cross-lane softmax.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace team {

constexpr int ROUTE_THREADS = 512;
constexpr int ROUTE_WAVES = ROUTE_THREADS / WAVE;
constexpr int MAX_E = 256;

template <typename ST> struct Chunk;
template <> struct Chunk<uint16_t> { static constexpr int N = 8; };
template <> struct Chunk<float> { static constexpr int N = 4; };

template <typename ST>
__device__ __forceinline__ void load_chunk(const ST* p, float* out);
template <> __device__ __forceinline__ void load_chunk<uint16_t>(const uint16_t* p, float* out) { load8(p, out); }
template <> __device__ __forceinline__ void load_chunk<float>(const float* p, float* out) { load4(p, out); }

// Lexicographic "better" for selection: larger logit wins, equal logits go to the lower expert id.
__device__ __forceinline__ bool better(float va, int ia, float vb, int ib) { return va > vb || (va == vb && ia < ib); }

template <typename ST>
__global__ __launch_bounds__(ROUTE_THREADS) void route_kernel(const ST* __restrict__ x, const ST* __restrict__ w_router,
                                                              const uint8_t* __restrict__ mask, int32_t* __restrict__ topk_idx,
                                                              float* __restrict__ topk_gate, float* __restrict__ logits_out,
                                                              int H, int E, int k, int renormalize) {
    constexpr int CN = Chunk<ST>::N;
    __shared__ float s_logit[MAX_E];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x / WAVE;
    const int n_chunks = H / CN;                 // chunks of CN consecutive elements; lane takes chunk lane, lane+64, ...
    const ST* xt = x + (size_t)t * H;

    // ---- logits: fixed summation order (per lane ascending, then butterfly) -> deterministic
    for (int e = wave; e < E; e += ROUTE_WAVES) {
        const ST* wr = w_router + (size_t)e * H;
        float acc = 0.f;
        for (int c = lane; c < n_chunks; c += WAVE) {
            float xv[CN], wv[CN];
            load_chunk<ST>(xt + (size_t)c * CN, xv);
            load_chunk<ST>(wr + (size_t)c * CN, wv);
#pragma unroll
            for (int j = 0; j < CN; ++j) acc = fmaf(xv[j], wv[j], acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) {
            s_logit[e] = acc;
            if (logits_out) logits_out[(size_t)t * E + e] = acc;
        }
    }
    __syncthreads();
    if (wave != 0) return;

    // ---- selection by wavefront 0: lane owns experts lane, lane+64, lane+128, lane+192
    constexpr int PER_LANE = MAX_E / WAVE;
    float v[PER_LANE];
    bool ok[PER_LANE];
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) {
        int e = lane + j * WAVE;
        ok[j] = e < E && (mask == nullptr || mask[e] != 0);
        v[j] = e < E ? s_logit[e] : 0.f;
    }
    float full_max = 0.f, full_den = 1.f;
    if (!renormalize) {                         // softmax denominator over all E experts
        float m = -INFINITY;
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j) if (lane + j * WAVE < E) m = fmaxf(m, v[j]);
        m = wave_max(m);
        float dsum = 0.f;
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j) if (lane + j * WAVE < E) dsum += expf(v[j] - m);
        full_max = m;
        full_den = wave_sum(dsum);
    }
    float my_sel_logit = 0.f;     // lane s keeps the logit of slot s
    int my_sel_idx = -1;
    int k_eff = 0;
    for (int s = 0; s < k; ++s) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j)
            if (ok[j] && better(v[j], lane + j * WAVE, bv, bi)) { bv = v[j]; bi = lane + j * WAVE; }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            float ov = __shfl_xor(bv, off, WAVE);
            int oi = __shfl_xor(bi, off, WAVE);
            if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        if (bi == 0x7fffffff) break;            // allowed set exhausted: k_eff = |S| < k
        ++k_eff;
        if (lane == s) { my_sel_logit = bv; my_sel_idx = bi; }
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j) if (lane + j * WAVE == bi) ok[j] = false;
    }
    // ---- gates
    float gate = 0.f;
    if (renormalize) {
        float m = __shfl(my_sel_logit, 0, WAVE);
        float w = lane < k_eff ? expf(my_sel_logit - m) : 0.f;
        float den = wave_sum(w);
        gate = lane < k_eff ? w / den : 0.f;
    } else {
        gate = lane < k_eff ? expf(my_sel_logit - full_max) / full_den : 0.f;
    }
    if (lane < k) {
        topk_idx[(size_t)t * k + lane] = lane < k_eff ? my_sel_idx : -1;
        topk_gate[(size_t)t * k + lane] = gate;
    }
}

hipError_t launch_route(const Dims& d, const void* x, const void* w_router, const uint8_t* mask, int32_t* topk_idx,
                        float* topk_gate, float* logits_out, hipStream_t s) {
    dim3 grid(d.T), block(ROUTE_THREADS);
    if (d.bf16)
        hipLaunchKernelGGL(route_kernel<uint16_t>, grid, block, 0, s, (const uint16_t*)x, (const uint16_t*)w_router, mask,
                           topk_idx, topk_gate, logits_out, d.H, d.E, d.k, d.renormalize);
    else
        hipLaunchKernelGGL(route_kernel<float>, grid, block, 0, s, (const float*)x, (const float*)w_router, mask, topk_idx,
                           topk_gate, logits_out, d.H, d.E, d.k, d.renormalize);
    return hipGetLastError();
}

}  // namespace team
