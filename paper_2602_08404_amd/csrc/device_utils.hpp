// Small device helpers shared by the gfx950 kernels of the MoE layer (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace team {

constexpr int WAVE = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// bfloat16 bit pattern <-> float.  Widening is exact; narrowing rounds to nearest even (finite values).
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Cross-lane moves inside a row of 16 lanes (data-parallel primitives, no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
constexpr int DPP_XOR1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i <-> 7-i inside 8 lanes
constexpr int DPP_MIRROR = 0x140;       // lane i <-> 15-i inside 16 lanes

// Sum over the 64 lanes, returned in every lane.  Fixed order: pairs, quads, 8, 16 lanes, then the four rows.
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<DPP_XOR1>(v);
    v += dpp_f32<DPP_XOR2>(v);
    v += dpp_f32<DPP_HALF_MIRROR>(v);
    v += dpp_f32<DPP_MIRROR>(v);
    const float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (a + b) + (c + d);
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<DPP_XOR1>(v));
    v = fmaxf(v, dpp_f32<DPP_XOR2>(v));
    v = fmaxf(v, dpp_f32<DPP_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_f32<DPP_MIRROR>(v));
    const float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return fmaxf(fmaxf(a, b), fmaxf(c, d));
}
// Maximum of a 64-bit key over the 64 lanes, returned in every lane.
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long key) {
    uint32_t hi = (uint32_t)(key >> 32), lo = (uint32_t)key;
#define TEAM_STEP(CTRL)                                                              \
    {                                                                                \
        const uint32_t ohi = dpp_u32<CTRL>(hi), olo = dpp_u32<CTRL>(lo);             \
        const bool take = ohi > hi || (ohi == hi && olo > lo);                       \
        hi = take ? ohi : hi;                                                        \
        lo = take ? olo : lo;                                                        \
    }
    TEAM_STEP(DPP_XOR1)
    TEAM_STEP(DPP_XOR2)
    TEAM_STEP(DPP_HALF_MIRROR)
    TEAM_STEP(DPP_MIRROR)
#undef TEAM_STEP
    unsigned long long best = 0;
#pragma unroll
    for (int r = 0; r < 64; r += 16) {
        const unsigned long long k = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)hi, r) << 32) |
                                     (uint32_t)__builtin_amdgcn_readlane((int)lo, r);
        best = k > best ? k : best;
    }
    return best;
}

// Element loaders: N consecutive elements of storage type -> float.
__device__ __forceinline__ void load8(const uint16_t* p, float* out) {   // 8 bf16 = 16 bytes
    uint4 v = *reinterpret_cast<const uint4*>(p);
    out[0] = __uint_as_float(v.x << 16); out[1] = __uint_as_float(v.x & 0xffff0000u);
    out[2] = __uint_as_float(v.y << 16); out[3] = __uint_as_float(v.y & 0xffff0000u);
    out[4] = __uint_as_float(v.z << 16); out[5] = __uint_as_float(v.z & 0xffff0000u);
    out[6] = __uint_as_float(v.w << 16); out[7] = __uint_as_float(v.w & 0xffff0000u);
}
__device__ __forceinline__ void load4(const float* p, float* out) {      // 4 floats = 16 bytes
    float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}

// 16 E4M3 codes (as read from LDS) -> two MFMA operands of 8 bf16: codes 0-7 and codes 8-15.  Every E4M3 value is a bf16 value.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ void widen_e4m3(const bf16x8_t& raw, bf16x8_t& first, bf16x8_t& second) {
    const u32x4_t r = __builtin_bit_cast(u32x4_t, raw);
    union {
        bf16x2_t p[4];
        bf16x8_t v;
    } a, b;
    a.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[0], 1.0f, false);
    a.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[0], 1.0f, true);
    a.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[1], 1.0f, false);
    a.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[1], 1.0f, true);
    b.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[2], 1.0f, false);
    b.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[2], 1.0f, true);
    b.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[3], 1.0f, false);
    b.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[3], 1.0f, true);
    first = a.v;
    second = b.v;
}
__device__ __forceinline__ float silu_f32(float z) { return z / (1.0f + expf(-z)); }

// Row of the caller's x / y tensors that holds token t of the call: t itself, or row_index[t] clamped into [0, n_rows).
__device__ __forceinline__ int token_row(const int32_t* __restrict__ row_index, int n_rows, int t) {
    if (!row_index) return t;
    const int r = row_index[t];
    return r < 0 ? 0 : (r >= n_rows ? n_rows - 1 : r);
}

}  // namespace team
