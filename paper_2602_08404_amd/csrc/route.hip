// Router restricted to the activated-expert set: logits, masked top-k, gates.
// Paper: Algorithm 1, "Router(C, E_A)" (second-round routing confined to the necessary experts) and, with no
// mask, the first-round router over E_0.  One workgroup per token: every wavefront scores a share of the
// experts (dot products reduced across lanes; the loads of a group of experts are issued together so the
// kernel pays the memory latency once per group, not once per expert), then wavefront 0 selects the k best
// allowed experts with cross-lane arg-max and turns the selected logits into gates with a cross-lane softmax.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace team {

constexpr int ROUTE_THREADS = 512;
constexpr int ROUTE_WAVES = ROUTE_THREADS / WAVE;
constexpr int MAX_E = 256;

template <typename ST> struct Chunk;
template <> struct Chunk<uint16_t> { static constexpr int N = 8; };
template <> struct Chunk<float> { static constexpr int N = 4; };

// 16 packed bytes (8 bf16 or 4 floats) -> floats
template <typename ST>
__device__ __forceinline__ void unpack_chunk(const uint4& v, float* out);
template <> __device__ __forceinline__ void unpack_chunk<uint16_t>(const uint4& v, float* out) {
    out[0] = __uint_as_float(v.x << 16); out[1] = __uint_as_float(v.x & 0xffff0000u);
    out[2] = __uint_as_float(v.y << 16); out[3] = __uint_as_float(v.y & 0xffff0000u);
    out[4] = __uint_as_float(v.z << 16); out[5] = __uint_as_float(v.z & 0xffff0000u);
    out[6] = __uint_as_float(v.w << 16); out[7] = __uint_as_float(v.w & 0xffff0000u);
}
template <> __device__ __forceinline__ void unpack_chunk<float>(const uint4& v, float* out) {
    out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y); out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
}

// Selection key: larger logit wins, equal logits go to the lower expert id.  The float is mapped to an
// unsigned integer with the same order; the id is stored complemented in the low word; 0 = no candidate.
__device__ __forceinline__ unsigned long long select_key(float v, int e) {
    const uint32_t b = __float_as_uint(v + 0.f);      // -0 and +0 compare equal: both become +0
    const uint32_t ord = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return ((unsigned long long)ord << 32) | (uint32_t)(0xffffffffu - (uint32_t)e);
}
__device__ __forceinline__ int key_expert(unsigned long long key) { return (int)(0xffffffffu - (uint32_t)key); }

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

    // ---- logits: fixed summation order (per lane ascending, then butterfly) -> deterministic.
    // Wavefront w scores experts w, w+8, ...; EG of them per pass with all their loads in flight together.
    constexpr int EG = 8;          // experts per pass
    constexpr int XC = 4;          // chunks of the token row per lane per block of 256 chunks
    for (int e0 = wave; e0 < E; e0 += ROUTE_WAVES * EG) {
        float acc[EG];
#pragma unroll
        for (int g = 0; g < EG; ++g) acc[g] = 0.f;
        for (int cb = 0; cb < n_chunks; cb += WAVE * XC) {
            // 16-byte packed chunks stay packed in registers until they are multiplied
            uint4 xp[XC], wp[EG][XC];
#pragma unroll
            for (int j = 0; j < XC; ++j) {
                const int c = cb + j * WAVE + lane;
                xp[j] = c < n_chunks ? *reinterpret_cast<const uint4*>(xt + (size_t)c * CN) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int g = 0; g < EG; ++g) {
                const int e = e0 + g * ROUTE_WAVES;
                const ST* wr = w_router + (size_t)(e < E ? e : 0) * H;
#pragma unroll
                for (int j = 0; j < XC; ++j) {
                    const int c = cb + j * WAVE + lane;
                    wp[g][j] = (c < n_chunks && e < E) ? *reinterpret_cast<const uint4*>(wr + (size_t)c * CN) : make_uint4(0u, 0u, 0u, 0u);
                }
            }
#pragma unroll
            for (int j = 0; j < XC; ++j) {
                float xv[CN];
                unpack_chunk<ST>(xp[j], xv);
#pragma unroll
                for (int g = 0; g < EG; ++g) {
                    float wv[CN];
                    unpack_chunk<ST>(wp[g][j], wv);
#pragma unroll
                    for (int i = 0; i < CN; ++i) acc[g] = fmaf(xv[i], wv[i], acc[g]);
                }
            }
        }
#pragma unroll
        for (int g = 0; g < EG; ++g) {
            const float v = wave_sum(acc[g]);
            const int e = e0 + g * ROUTE_WAVES;
            if (lane == 0 && e < E) {
                s_logit[e] = v;
                if (logits_out) logits_out[(size_t)t * E + e] = v;
            }
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
        unsigned long long best = 0;                     // NaN logits are never selected (their key is not formed)
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j)
            if (ok[j] && v[j] == v[j]) {
                const unsigned long long key = select_key(v[j], lane + j * WAVE);
                best = key > best ? key : best;
            }
        best = wave_max_u64(best);
        if (best == 0) break;                            // allowed set exhausted: k_eff = |S| < k
        const int bi = key_expert(best);
        ++k_eff;
        if (lane == s) { my_sel_logit = s_logit[bi]; my_sel_idx = bi; }
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j) if (lane + j * WAVE == bi) ok[j] = false;
    }
    // ---- gates
    float gate = 0.f;
    if (renormalize) {
        const float m = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_sel_logit), 0));
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
