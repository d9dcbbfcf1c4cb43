// Grouped SwiGLU expert FFN over the activated experts, bf16 storage, gfx950 MFMA, HBM-streaming design.
//
// Paper context: block-level decoding is memory-bound (Section "Delayed Caching for Decoded Tokens"), latency
// is dominated by the feed-forward layers and every activated expert serves only a few tokens (Section
// "Speculative Exploration for Hot Tokens").  So the cost of this step is reading the weights of the experts
// that received tokens, once, at HBM speed; the arithmetic rides along on the matrix cores.
//
// Two kernels, both persistent (a fixed grid walks a contiguous range of work items computed on the device
// from n_active, so experts without tokens cost nothing and the host never reads device data):
//   gate/up : item = (active expert, 8 consecutive intermediate indices) = 8 rows of w_gate + 8 rows of
//             w_up, all H columns.  h = silu(g) * u is formed in the epilogue and stored as bf16.
//   down    : item = (active expert, 16*RB consecutive output rows of w_down), all I columns; fp32 out.
// Inside a workgroup the reduction dimension is split over the 4 wavefronts.  Each wavefront pulls its
// slice of the item's weight rows HBM -> LDS with 16-byte-per-lane direct-to-LDS loads (lanes consecutive
// along the contiguous dimension), keeps the whole slice in flight at once, then feeds v_mfma_f32_16x16x32
// bf16 with the weights as the 16-row operand and up to 32 token rows as the 16-column operand.  The token
// operand lives in registers and is reused for every item of the same expert.  Partial sums of the 4
// wavefronts are added in a fixed order through LDS (deterministic, no atomics).
//
// LDS slice layout: a wavefront's slice of a 16-row sub-tile is 16 rows x C chunks of 16 bytes
// (C = 4 * K-steps).  Chunk (r, c) sits at position r*C + (c ^ (r >> (4 - V))), V = min(4, ctz(C)), which
// makes the 16 rows of one MFMA operand read hit 16 different 16-byte bank groups.
#include "device_utils.hpp"
#include "kernels.hpp"

#include <stdlib.h>
#include <string.h>

namespace team {

constexpr int FFN_THREADS = 256;
constexpr int FFN_WAVES = 4;
constexpr int NT = 2;                    // token tiles of 16 rows handled per pass (32 tokens)

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// 64 lanes x 16 bytes, each lane from its own global address, land contiguously at lds_base + lane*16.
__device__ __forceinline__ void slab_load(const void* gsrc, char* lds_base_uniform) {
    __builtin_amdgcn_global_load_lds((gptr_t)gsrc, (lptr_t)lds_base_uniform, 16, 0, 0);
}
__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

constexpr int ctz_cap4(int c) { return (c % 16 == 0) ? 4 : (c % 8 == 0) ? 3 : (c % 4 == 0) ? 2 : (c % 2 == 0) ? 1 : 0; }

template <int KS>
struct Slice {
    static constexpr int C = 4 * KS;                  // 16-byte chunks per row of the wavefront's slice
    static constexpr int V = ctz_cap4(C);
    static constexpr int SLABS = KS;                  // 1 KB slabs per 16-row sub-tile
    static constexpr int BYTES = 16 * C * 16;         // bytes of one 16-row sub-tile slice
    __device__ static __forceinline__ int phys(int r, int c) { return r * C + (c ^ (r >> (4 - V))); }
};

struct Rows {
    int e, r0, m;
};
// Rows of active slot a, clipped to the table; m = 0 if the slot holds no valid expert.
__device__ __forceinline__ Rows rows_of_slot(const int32_t* __restrict__ offsets, const int32_t* __restrict__ active, int a, int E, int A) {
    Rows r;
    r.e = active[a];
    r.r0 = 0;
    r.m = 0;
    if (r.e >= 0 && r.e < E) {
        int lo = max(offsets[r.e], 0), hi = min(offsets[r.e + 1], A);
        r.r0 = lo;
        r.m = max(hi - lo, 0);
    }
    return r;
}

// ---------------------------------------------------------------------------------------------- gate/up
// KS = H / 128: MFMA K-steps (of 32) per wavefront.
template <int KS>
__global__ __launch_bounds__(FFN_THREADS, 2) void ffn_gate_up_kernel(const uint16_t* __restrict__ x, const int32_t* __restrict__ offsets,
                                                                     const int32_t* __restrict__ sorted_token,
                                                                     const int32_t* __restrict__ active, const int32_t* __restrict__ n_active,
                                                                     const uint16_t* __restrict__ wg, const uint16_t* __restrict__ wu,
                                                                     uint16_t* __restrict__ h, int T, int k, int I, int E) {
    using S = Slice<KS>;
    constexpr int H = KS * 128;
    constexpr int KSLICE = KS * 32;                       // columns per wavefront
    __shared__ __attribute__((aligned(1024))) char s_w[FFN_WAVES * S::BYTES];
    __shared__ f32x4_t s_red[FFN_WAVES][NT][WAVE];

    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, q = lane >> 4;
    const int A = T * k;
    const int tiles = I / 8;
    const int n_act = min(max(*n_active, 0), E);
    const long long total = (long long)n_act * tiles;
    const int begin = (int)(total * blockIdx.x / gridDim.x);
    const int end = (int)(total * (blockIdx.x + 1) / gridDim.x);
    char* region = s_w + wave * S::BYTES;

    bf16x8_t xr[NT][KS];
    int cur_a = -1;
    for (int item = begin; item < end; ++item) {
        const int a = item / tiles, it = item - a * tiles;
        const Rows rw = rows_of_slot(offsets, active, a, E, A);
        if (rw.m == 0) continue;                           // uniform over the workgroup
        // ---- stream this wavefront's slice of the 16 weight rows into LDS (all slabs in flight)
        {
            const size_t ebase = (size_t)rw.e * I;
#pragma unroll
            for (int j = 0; j < S::SLABS; ++j) {
                const int P = 64 * j + lane;
                const int r = P / S::C, cp = P % S::C;
                const int c = cp ^ (r >> (4 - S::V));
                // MFMA row r = 4*qq + j2: j2 in {0,1} -> gate rows, {2,3} -> up rows of intermediate index 2*qq + (j2 & 1)
                const uint16_t* mat = (r & 2) ? wu : wg;
                const int irow = it * 8 + 2 * (r >> 2) + (r & 1);
                slab_load(mat + (ebase + irow) * H + wave * KSLICE + c * 8, region + j * 1024);
            }
        }
        const int chunks = (rw.m + 16 * NT - 1) / (16 * NT);
        for (int ch = 0; ch < chunks; ++ch) {
            const int row_base = ch * 16 * NT;
            if (a != cur_a || chunks > 1) {                // token operand: registers, reused across items of one expert
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int row = row_base + nt * 16 + n;
                    int tok = row < rw.m ? sorted_token[rw.r0 + row] : -1;
                    if (tok >= T) tok = -1;
                    const uint16_t* xp = x + (size_t)(tok < 0 ? 0 : tok) * H + wave * KSLICE + q * 8;
#pragma unroll
                    for (int s = 0; s < KS; ++s) {
                        bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(xp + s * 32);
                        if (tok < 0) v = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                        xr[nt][s] = v;
                    }
                }
            }
            cur_a = a;
            wait_all_loads();
            const bool two = rw.m - row_base > 16;
            f32x4_t acc[NT] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const bf16x8_t wv = *reinterpret_cast<const bf16x8_t*>(region + S::phys(n, 4 * s + q) * 16);
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, xr[0][s], acc[0], 0, 0, 0);
                if (two) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, xr[1][s], acc[1], 0, 0, 0);
            }
            s_red[wave][0][lane] = acc[0];
            s_red[wave][1][lane] = acc[1];
            __syncthreads();
            if (wave < NT && (wave == 0 || two)) {        // wavefront nt finishes token tile nt
                f32x4_t v = s_red[0][wave][lane];
#pragma unroll
                for (int w = 1; w < FFN_WAVES; ++w) v += s_red[w][wave][lane];
                const int row = row_base + wave * 16 + n;
                if (row < rw.m) {
                    // lane holds (g_a, g_b, u_a, u_b) of intermediate indices ia = it*8 + 2*q, ia+1 for token row `row`
                    const float h0 = silu_f32(v[0]) * v[2];
                    const float h1 = silu_f32(v[1]) * v[3];
                    const uint32_t packed = f32_to_bf16_bits(h0) | (f32_to_bf16_bits(h1) << 16);
                    *reinterpret_cast<uint32_t*>(h + (size_t)(rw.r0 + row) * I + it * 8 + 2 * q) = packed;
                }
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------- down
// KS = I / 128 K-steps per wavefront; RB 16-row sub-tiles of w_down per item.
template <int KS, int RB>
__global__ __launch_bounds__(FFN_THREADS, 2) void ffn_down_kernel(const uint16_t* __restrict__ hbuf, const int32_t* __restrict__ offsets,
                                                                  const int32_t* __restrict__ sorted_token, const int32_t* __restrict__ active,
                                                                  const int32_t* __restrict__ n_active, const uint16_t* __restrict__ wd,
                                                                  float* __restrict__ out, int T, int k, int H, int E) {
    using S = Slice<KS>;
    constexpr int I = KS * 128;
    constexpr int KSLICE = KS * 32;
    __shared__ __attribute__((aligned(1024))) char s_w[FFN_WAVES * RB * S::BYTES];
    __shared__ f32x4_t s_red[FFN_WAVES][RB][NT][WAVE];

    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, q = lane >> 4;
    const int A = T * k;
    const int tiles = H / (16 * RB);
    const int n_act = min(max(*n_active, 0), E);
    const long long total = (long long)n_act * tiles;
    const int begin = (int)(total * blockIdx.x / gridDim.x);
    const int end = (int)(total * (blockIdx.x + 1) / gridDim.x);
    char* region = s_w + wave * (RB * S::BYTES);

    bf16x8_t hr[NT][KS];
    int cur_a = -1;
    for (int item = begin; item < end; ++item) {
        const int a = item / tiles, it = item - a * tiles;
        const Rows rw = rows_of_slot(offsets, active, a, E, A);
        if (rw.m == 0) continue;
        {
            const size_t ebase = (size_t)rw.e * H + (size_t)it * 16 * RB;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int j = 0; j < S::SLABS; ++j) {
                    const int P = 64 * j + lane;
                    const int r = P / S::C, cp = P % S::C;
                    const int c = cp ^ (r >> (4 - S::V));
                    slab_load(wd + (ebase + rb * 16 + r) * I + wave * KSLICE + c * 8, region + rb * S::BYTES + j * 1024);
                }
        }
        const int chunks = (rw.m + 16 * NT - 1) / (16 * NT);
        for (int ch = 0; ch < chunks; ++ch) {
            const int row_base = ch * 16 * NT;
            if (a != cur_a || chunks > 1) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int row = row_base + nt * 16 + n;
                    const bool valid = row < rw.m && sorted_token[rw.r0 + row] >= 0;
                    const uint16_t* hp = hbuf + (size_t)(valid ? rw.r0 + row : 0) * I + wave * KSLICE + q * 8;
#pragma unroll
                    for (int s = 0; s < KS; ++s) {
                        bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(hp + s * 32);
                        if (!valid) v = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                        hr[nt][s] = v;
                    }
                }
            }
            cur_a = a;
            wait_all_loads();
            const bool two = rw.m - row_base > 16;
            f32x4_t acc[RB][NT];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[rb][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    const bf16x8_t wv = *reinterpret_cast<const bf16x8_t*>(region + rb * S::BYTES + S::phys(n, 4 * s + q) * 16);
                    acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, hr[0][s], acc[rb][0], 0, 0, 0);
                    if (two) acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, hr[1][s], acc[rb][1], 0, 0, 0);
                }
            }
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) s_red[wave][rb][nt][lane] = acc[rb][nt];
            __syncthreads();
            // (rb, nt) pairs are finished by wavefronts round-robin, partial sums added in wavefront order
            for (int pair = wave; pair < RB * NT; pair += FFN_WAVES) {
                const int rb = pair / NT, nt = pair % NT;
                const int row = row_base + nt * 16 + n;
                if (row < rw.m) {
                    f32x4_t v = s_red[0][rb][nt][lane];
#pragma unroll
                    for (int w = 1; w < FFN_WAVES; ++w) v += s_red[w][rb][nt][lane];
                    // lane holds output rows it*16*RB + rb*16 + 4*q + (0..3) of token row `row`
                    *reinterpret_cast<f32x4_t*>(out + (size_t)(rw.r0 + row) * H + it * 16 * RB + rb * 16 + 4 * q) = v;
                }
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------- host side
static int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    int x = atoi(v);
    return x > 0 ? x : dflt;
}

static int persistent_grid(const char* env_name, int per_cu) {
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n_cu = prop.multiProcessorCount;
        if (n_cu <= 0) n_cu = 256;
    }
    return env_int(env_name, n_cu * per_cu);
}

bool ffn_bf16_supported(int H, int I) {
    const bool h_ok = H == 256 || H == 512 || H == 1024 || H == 2048;
    const bool i_ok = I % 128 == 0 && I >= 128 && I <= 1024;
    return h_ok && i_ok;
}

constexpr int DOWN_RB = 2;

template <int KS>
static void launch_gate_up(int grid, hipStream_t s, const Dims& d, const uint16_t* x, const int32_t* offsets, const int32_t* sorted_token,
                           const int32_t* active, const int32_t* n_active, const uint16_t* wg, const uint16_t* wu, uint16_t* h) {
    hipLaunchKernelGGL(ffn_gate_up_kernel<KS>, dim3(grid), dim3(FFN_THREADS), 0, s, x, offsets, sorted_token, active, n_active, wg, wu, h,
                       d.T, d.k, d.I, d.E);
}
template <int KS>
static void launch_down(int grid, hipStream_t s, const Dims& d, const uint16_t* h, const int32_t* offsets, const int32_t* sorted_token,
                        const int32_t* active, const int32_t* n_active, const uint16_t* wd, float* out) {
    hipLaunchKernelGGL((ffn_down_kernel<KS, DOWN_RB>), dim3(grid), dim3(FFN_THREADS), 0, s, h, offsets, sorted_token, active, n_active, wd,
                       out, d.T, d.k, d.H, d.E);
}

hipError_t launch_ffn_bf16(const Dims& d, const uint16_t* x, const int32_t* offsets, const int32_t* sorted_token, const int32_t* active,
                           const int32_t* n_active, const uint16_t* wg, const uint16_t* wu, const uint16_t* wd, uint16_t* h_ws,
                           float* expert_out, hipStream_t s) {
    if (!ffn_bf16_supported(d.H, d.I)) return hipErrorInvalidValue;
    const int grid_a = persistent_grid("TEAM_MOE_GRID_GATE_UP", 2);
    const int grid_b = persistent_grid("TEAM_MOE_GRID_DOWN", 2);
#define GU(KS) launch_gate_up<KS>(grid_a, s, d, x, offsets, sorted_token, active, n_active, wg, wu, h_ws)
    switch (d.H / 128) {
        case 2: GU(2); break;
        case 4: GU(4); break;
        case 8: GU(8); break;
        case 16: GU(16); break;
        default: return hipErrorInvalidValue;
    }
#undef GU
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
#define DN(KS) launch_down<KS>(grid_b, s, d, h_ws, offsets, sorted_token, active, n_active, wd, expert_out)
    switch (d.I / 128) {
        case 1: DN(1); break;
        case 2: DN(2); break;
        case 3: DN(3); break;
        case 4: DN(4); break;
        case 5: DN(5); break;
        case 6: DN(6); break;
        case 7: DN(7); break;
        case 8: DN(8); break;
        default: return hipErrorInvalidValue;
    }
#undef DN
    return hipGetLastError();
}

}  // namespace team
