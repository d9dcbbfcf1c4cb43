// Router restricted to the activated-expert set: logits, masked top-k, gates.
// Paper: Algorithm 1, "Router(C, E_A)" (second-round routing confined to the necessary experts) and, with no
// mask, the first-round router over E_0.  Two small latency-bound kernels:
//   logits : one workgroup per (token, group of 32 experts); a wavefront scores 8 experts with all their loads
//            in flight together (one memory round trip), fp32 FMA, cross-lane sums without LDS traffic.
//            Splitting the experts of a token over several compute units keeps the router matrix traffic per
//            compute unit small (the whole matrix through one compute unit costs more than the rest together).
//   select : one workgroup per token, one thread per expert.  The slot of an expert is its rank = the number of
//            allowed experts that beat it (larger logit, or equal logit and lower id): every thread counts its
//            own rank against the logits in LDS, so there is no serial arg-max loop; experts with rank < k write
//            themselves into their slot.  One wavefront then turns the selected logits into gates.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace team {

constexpr int LOGIT_THREADS = 256;
constexpr int LOGIT_WAVES = LOGIT_THREADS / WAVE;
constexpr int EG = 8;                                   // experts per wavefront
constexpr int LOGIT_GROUP = LOGIT_WAVES * EG;           // experts per workgroup
constexpr int MAX_E = 256;
constexpr int SELECT_THREADS = MAX_E;

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

template <typename ST>
__global__ __launch_bounds__(LOGIT_THREADS) void route_logits_kernel(const ST* __restrict__ x, const ST* __restrict__ w_router,
                                                                     float* __restrict__ logits, int H, int E) {
    constexpr int CN = Chunk<ST>::N;
    constexpr int XC = 4;          // chunks of the token row per lane per block of 256 chunks
    const int t = blockIdx.y;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x / WAVE;
    const int n_chunks = H / CN;   // chunks of CN consecutive elements; lane takes chunk lane, lane+64, ...
    const ST* xt = x + (size_t)t * H;
    const int e0 = blockIdx.x * LOGIT_GROUP + wave;     // this wavefront: experts e0, e0+4, ..., e0+28

    // fixed summation order (per lane ascending, then the cross-lane tree) -> deterministic
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
            const int e = e0 + g * LOGIT_WAVES;
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
        const int e = e0 + g * LOGIT_WAVES;
        if (lane == 0 && e < E) logits[(size_t)t * E + e] = v;
    }
}

// Selection key: larger logit wins, equal logits go to the lower expert id.  The float is mapped to an unsigned
// integer with the same order; the id is stored complemented in the low word; 0 = not a candidate.
__device__ __forceinline__ unsigned long long select_key(float v, int e) {
    const uint32_t b = __float_as_uint(v);
    const uint32_t ord = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return ((unsigned long long)ord << 32) | (uint32_t)(0xffffffffu - (uint32_t)e);
}

__global__ __launch_bounds__(SELECT_THREADS) void route_select_kernel(const float* __restrict__ logits, const uint8_t* __restrict__ mask,
                                                                      int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate,
                                                                      int E, int k, int renormalize, CtrlZero ctrl) {
    __shared__ __attribute__((aligned(16))) unsigned long long s_key[MAX_E];   // 0 for experts that are not candidates
    __shared__ float s_all[MAX_E];                                              // every logit (for the full softmax)
    __shared__ float s_sel_logit[16];
    __shared__ int32_t s_sel_idx[16];
    __shared__ int32_t s_count[SELECT_THREADS / WAVE];
    const int t = blockIdx.x;
    const int e = threadIdx.x;
    const int lane = e & (WAVE - 1);
    if (ctrl.words && t == 0) {                     // control block of an expert FFN that follows without a dispatch kernel
        if (e < ctrl.header) ctrl.words[e] = 0;
        if (e < E) ctrl.words[ctrl.header + e * ctrl.stride] = 0;
    }
    float v = 0.f;
    bool ok = false;
    if (e < E) {
        v = logits[(size_t)t * E + e] + 0.f;                         // -0 -> +0 so that equal logits compare equal
        ok = (mask == nullptr || mask[e] != 0) && v == v;            // a NaN logit is never selected
    }
    const unsigned long long my_key = ok ? select_key(v, e) : 0ull;
    if (e < 16) { s_sel_idx[e] = -1; s_sel_logit[e] = 0.f; }
    s_all[e] = e < E ? v : -INFINITY;
    s_key[e] = my_key;
    const unsigned long long ok_lanes = __ballot(ok);
    if (lane == 0) s_count[e / WAVE] = __popcll(ok_lanes);
    __syncthreads();
    if (ok) {                                                         // rank = number of candidates that beat this one
        int rank = 0;
        const int n2 = (E + 1) / 2;
#pragma unroll 8
        for (int j2 = 0; j2 < n2; ++j2) {
            const ulonglong2 o = *reinterpret_cast<const ulonglong2*>(s_key + 2 * j2);   // same address in all lanes: broadcast
            rank += (o.x > my_key) + (o.y > my_key);
        }
        if (rank < k) { s_sel_idx[rank] = e; s_sel_logit[rank] = v; }
    }
    __syncthreads();
    if (e >= WAVE) return;
    // ---- gates by wavefront 0: lane s owns slot s
    int n_allowed = 0;
#pragma unroll
    for (int w = 0; w < SELECT_THREADS / WAVE; ++w) n_allowed += s_count[w];
    const int k_eff = min(k, n_allowed);
    const float my_logit = lane < 16 ? s_sel_logit[lane] : 0.f;
    float gate = 0.f;
    if (renormalize) {
        const float m = s_sel_logit[0];
        const float w = lane < k_eff ? expf(my_logit - m) : 0.f;
        const float den = wave_sum(w);
        gate = lane < k_eff ? w / den : 0.f;
    } else {                                                         // selected entries of the softmax over all E experts
        float m = -INFINITY;
        for (int j = lane; j < E; j += WAVE) m = fmaxf(m, s_all[j]);
        m = wave_max(m);
        float dsum = 0.f;
        for (int j = lane; j < E; j += WAVE) dsum += expf(s_all[j] - m);
        const float den = wave_sum(dsum);
        gate = lane < k_eff ? expf(my_logit - m) / den : 0.f;
    }
    if (lane < k) {
        topk_idx[(size_t)t * k + lane] = lane < k_eff ? s_sel_idx[lane] : -1;
        topk_gate[(size_t)t * k + lane] = gate;
    }
}

hipError_t launch_route(const Dims& d, const void* x, const void* w_router, const uint8_t* mask, int32_t* topk_idx,
                        float* topk_gate, float* logits, CtrlZero ctrl, hipStream_t s) {
    dim3 grid((d.E + LOGIT_GROUP - 1) / LOGIT_GROUP, d.T), block(LOGIT_THREADS);
    if (d.bf16)
        hipLaunchKernelGGL(route_logits_kernel<uint16_t>, grid, block, 0, s, (const uint16_t*)x, (const uint16_t*)w_router, logits, d.H, d.E);
    else
        hipLaunchKernelGGL(route_logits_kernel<float>, grid, block, 0, s, (const float*)x, (const float*)w_router, logits, d.H, d.E);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(route_select_kernel, dim3(d.T), dim3(SELECT_THREADS), 0, s, logits, mask, topk_idx, topk_gate, d.E, d.k,
                       d.renormalize, ctrl);
    return hipGetLastError();
}

}  // namespace team
