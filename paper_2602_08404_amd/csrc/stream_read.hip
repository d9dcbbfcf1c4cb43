// A plain read-only streaming kernel (include/team_moe_internal.h: team_moe_internal_stream_read): every workgroup reads
// contiguous 64 KB pieces of a buffer with 16-byte non-temporal loads, the way the expert FFN reads weights, and keeps only an
// exclusive-or of what it read.  The benchmark times it on buffers of the sizes the expert FFN streams, as the practical
// ceiling of a read-only stream on the device the numbers are taken on.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/team_moe.h"
#include "../../include/team_moe_internal.h"

namespace {

constexpr int SR_THREADS = 256;
constexpr int SR_UNROLL = 16;                                   // 16-byte loads in flight per lane: 64 KB per workgroup
constexpr size_t SR_PIECE = (size_t)SR_THREADS * SR_UNROLL * 16;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ __launch_bounds__(SR_THREADS) void stream_read_kernel(const u32x4* __restrict__ src, size_t n_vec, uint32_t* __restrict__ sink) {
    const size_t pieces = (n_vec * 16 + SR_PIECE - 1) / SR_PIECE;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t p = blockIdx.x; p < pieces; p += gridDim.x) {
        const size_t base = p * (SR_PIECE / 16) + threadIdx.x;
        u32x4 v[SR_UNROLL];
#pragma unroll
        for (int j = 0; j < SR_UNROLL; ++j) {
            const size_t i = base + (size_t)j * SR_THREADS;
            v[j] = i < n_vec ? __builtin_nontemporal_load(src + i) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int j = 0; j < SR_UNROLL; ++j) acc ^= v[j];
    }
    const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (x == 0x9e3779b9u) sink[blockIdx.x] = x;                   // (keeps the loads alive; practically never taken)
}

}  // namespace

extern "C" int team_moe_internal_stream_read(const void* src, size_t bytes, uint32_t* sink, int32_t workgroups, void* stream) {
    if (!src || !sink || bytes < 16 || bytes % 16 != 0 || workgroups < 1 || workgroups > 65536) return TEAM_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(src) & 15u) return TEAM_ERR_INVALID_ARG;
    (void)hipGetLastError();
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)workgroups), dim3(SR_THREADS), 0, (hipStream_t)stream, (const u32x4*)src,
                       bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? TEAM_OK : TEAM_ERR_HIP;
}
