// Classification of the live tokens of a denoising step into first-round tokens and cold tokens.
// Paper: Algorithm 1 step 1 and Eq. 4 (Section "Speculative Exploration for Hot Tokens"): a masked token is hot if its
// confidence exceeds tau_h or if some decoded token of its block lies within L_h positions, L_h included (where Eq. 4 and
// Section "Experimental Setup" differ on the distance condition, the latter is followed); newly accepted tokens and hot tokens take part in the first routing round, the rest are cold.
// One thread per live token, a scan of at most 2*L_h+1 neighbours; integer and one float comparison, no arithmetic.
#include "kernels.hpp"

namespace team {

__global__ __launch_bounds__(256) void classify_tokens_kernel(const float* __restrict__ conf, const uint8_t* __restrict__ state,
                                                              int n_rows, int block_len, const int32_t* __restrict__ live_index, int T,
                                                              float tau_h, int L_h, uint8_t* __restrict__ token_class) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const int p = live_index ? live_index[t] : t;
    if (p < 0 || p >= n_rows) {            // not a row: nothing to route freely
        token_class[t] = 0;
        return;
    }
    if (state[p] != 0) {                   // newly accepted (or decoded earlier and listed anyway): routed over all experts
        token_class[t] = 1;
        return;
    }
    bool hot = conf[p] > tau_h;
    if (!hot) {
        const int b0 = (p / block_len) * block_len;
        const int b1 = min(b0 + block_len, n_rows);
        const int lo = max(b0, p - min(L_h, block_len)), hi = min(b1 - 1, p + min(L_h, block_len));
        for (int j = lo; j <= hi && !hot; ++j) hot = state[j] != 0;
    }
    token_class[t] = hot ? 1 : 0;
}

hipError_t launch_classify_tokens(const float* conf, const uint8_t* state, int n_rows, int block_len, const int32_t* live_index, int T,
                                  float tau_h, int L_h, uint8_t* token_class, hipStream_t s) {
    hipLaunchKernelGGL(classify_tokens_kernel, dim3((T + 255) / 256), dim3(256), 0, s, conf, state, n_rows, block_len, live_index, T, tau_h,
                       L_h, token_class);
    return hipGetLastError();
}

}  // namespace team
