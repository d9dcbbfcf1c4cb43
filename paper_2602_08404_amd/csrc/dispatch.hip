// Token-to-expert grouping of the routing table, integer only and bit-exact.
// The paper leaves the grouping implicit (each activated expert serves a small number of tokens; Section
// "Speculative Exploration for Hot Tokens"); the expert FFN needs, per expert, the list of its tokens.
// One workgroup, everything in LDS: a token bitset per expert (a token selects an expert at most once, so the
// rank of token t inside expert e is the number of set bits below t), popcount histogram, prefix sum over the
// experts, then every (token,slot) pair computes its own row.  No ordering depends on thread scheduling.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace team {

constexpr int DISPATCH_THREADS = 1024;
constexpr int D_MAX_E = 256;
constexpr int D_MAX_WORDS = 32;          // 32 words x 32 bits = 1024 tokens
constexpr int D_MAX_STRIDE = D_MAX_WORDS + 1;

__global__ __launch_bounds__(DISPATCH_THREADS) void dispatch_kernel(const int32_t* __restrict__ topk_idx, int T, int k, int E,
                                                                    int32_t* __restrict__ offsets, int32_t* __restrict__ sorted_token,
                                                                    int32_t* __restrict__ inv_pos, int32_t* __restrict__ active,
                                                                    int32_t* __restrict__ n_active, CtrlZero ctrl) {
    __shared__ uint32_t s_bits[D_MAX_E * D_MAX_STRIDE];
    __shared__ unsigned long long s_scan[2][D_MAX_E];   // low 32 bits: rows, high 32 bits: 1 if the expert has rows
    __shared__ int32_t s_off[D_MAX_E + 1];
    const int tid = threadIdx.x;
    const int words = (T + 31) / 32;
    // Bitsets are stored with an odd number of words from one expert to the next: threads that work on different experts (one
    // thread per expert in the histogram, one per pair in the rank computation) then read different LDS banks.  With a stride
    // of 32 words all 64 lanes of a wavefront hit one bank, and 1024 tokens took 47 us in this kernel.
    const int stride = words | 1;
    const int A = T * k;

    if (ctrl.words) {                           // control block of the expert FFN that follows
        if (tid < ctrl.header) ctrl.words[tid] = 0;
        if (tid < E) ctrl.words[ctrl.header + tid * ctrl.stride] = 0;
    }
    for (int i = tid; i < E * stride; i += DISPATCH_THREADS) s_bits[i] = 0u;
    __syncthreads();
    for (int r = tid; r < A; r += DISPATCH_THREADS) {
        int e = topk_idx[r];
        int t = r / k;
        if (e >= 0 && e < E) atomicOr(&s_bits[e * stride + (t >> 5)], 1u << (t & 31));
    }
    __syncthreads();
    // histogram + inclusive scan (Hillis-Steele over E <= 256 entries, ping-pong buffers)
    if (tid < D_MAX_E) {
        unsigned long long c = 0;
        if (tid < E) {
            unsigned n = 0;
            for (int w = 0; w < words; ++w) n += __popc(s_bits[tid * stride + w]);
            c = (unsigned long long)n | ((unsigned long long)(n > 0) << 32);
        }
        s_scan[0][tid] = c;
    }
    __syncthreads();
    int cur = 0;
    for (int step = 1; step < D_MAX_E; step <<= 1) {
        if (tid < D_MAX_E) {
            unsigned long long v = s_scan[cur][tid];
            if (tid >= step) v += s_scan[cur][tid - step];
            s_scan[cur ^ 1][tid] = v;
        }
        cur ^= 1;
        __syncthreads();
    }
    if (tid < E) {
        unsigned long long incl = s_scan[cur][tid];
        unsigned long long excl = tid ? s_scan[cur][tid - 1] : 0ull;
        int rows_before = (int)(excl & 0xffffffffull);
        int act_before = (int)(excl >> 32);
        s_off[tid] = rows_before;
        offsets[tid] = rows_before;
        if ((incl >> 32) != (excl >> 32)) active[act_before] = tid;
        if (tid == E - 1) {
            int total = (int)(incl & 0xffffffffull);
            s_off[E] = total;
            offsets[E] = total;
            *n_active = (int)(incl >> 32);
        }
    }
    __syncthreads();
    const int total = s_off[E];
    const int n_act = (int)(s_scan[cur][E - 1] >> 32);
    for (int i = n_act + tid; i < E; i += DISPATCH_THREADS) active[i] = -1;
    for (int i = total + tid; i < A; i += DISPATCH_THREADS) sorted_token[i] = -1;
    for (int r = tid; r < A; r += DISPATCH_THREADS) {
        int e = topk_idx[r];
        int t = r / k;
        int pos = -1;
        if (e >= 0 && e < E) {
            const uint32_t* b = s_bits + e * stride;
            int rank = 0;
            for (int w = 0; w < (t >> 5); ++w) rank += __popc(b[w]);
            rank += __popc(b[t >> 5] & ((1u << (t & 31)) - 1u));
            pos = s_off[e] + rank;
            sorted_token[pos] = t;
        }
        inv_pos[r] = pos;
    }
}

hipError_t launch_dispatch(const Dims& d, const int32_t* topk_idx, int32_t* offsets, int32_t* sorted_token, int32_t* inv_pos,
                           int32_t* active, int32_t* n_active, CtrlZero ctrl, hipStream_t s) {
    hipLaunchKernelGGL(dispatch_kernel, dim3(1), dim3(DISPATCH_THREADS), 0, s, topk_idx, d.T, d.k, d.E, offsets, sorted_token,
                       inv_pos, active, n_active, ctrl);
    return hipGetLastError();
}

}  // namespace team
