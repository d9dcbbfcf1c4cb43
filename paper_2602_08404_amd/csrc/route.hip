// Router restricted to the activated-expert set: logits, masked top-k, gates.
// Paper: Algorithm 1, "Router(C, E_A)" (second-round routing confined to the necessary experts) and, with no
// mask, the first-round router over E_0.  Two small latency-bound kernels:
//   logits : one workgroup per (token, group of 32 experts); a wavefront scores 8 experts with all their loads
//            in flight together (one memory round trip), fp32 FMA, cross-lane sums without LDS traffic.
//            Splitting the experts of a token over several compute units keeps the router matrix traffic per
//            compute unit small (the whole matrix through one compute unit costs more than the rest together).
//            Calls of 64 tokens or more (bf16): 16 x 16 tiles on the matrix cores instead, so that a router row is read
//            once per 16 tokens.
//   select : one workgroup per token, one thread per expert.  The slot of an expert is its rank = the number of
//            allowed experts that beat it (larger logit, or equal logit and lower id): every thread counts its
//            own rank against the logits in LDS, so there is no serial arg-max loop; experts with rank < k write
//            themselves into their slot.  One wavefront then turns the selected logits into gates.
//   repeated rows : optionally the logits kernel also hashes every row and the selection kernel of a token looks for an
//            earlier token with the same row (hash match, then a byte-wise comparison); such a token gets an empty
//            routing table and later the result of the earlier one (candidate branches of Section "Speculative
//            Exploration for Hot Tokens (SEH)" repeat most rows of the base branch).
//   two-round select : Algorithm 1 in one launch.
//            Calls of at most 256 tokens (a block, or a few): no workgroup depends on another.  Every workgroup rebuilds E_A itself:
//            a wavefront finds the k picks of a first-round token with k rounds of a cross-lane maximum over the same
//            (logit, id) keys the selection uses, four tokens at a time, which is cheaper than one exchange through memory.
//            Larger calls: two launches of one kernel, so that no workgroup ever waits for another.  The first routes the
//            first-round tokens (newly accepted and hot) over all experts and ORs their picks into a bit set E_A in device
//            memory; the second routes the cold tokens inside that set.
// Scores that are not numbers: a NaN ranks below every number (ties by the lower id, as for equal numbers), so it is selected
// only when fewer than k numbers are allowed; the gates are the softmax formulas in IEEE arithmetic, so a token that selects a
// NaN or an infinite score gets NaN gates and a NaN output row.
#include "tuning.hpp"

#include "device_utils.hpp"
#include "kernels.hpp"

namespace team {

constexpr int LOGIT_THREADS = 256;
constexpr int LOGIT_WAVES = LOGIT_THREADS / WAVE;
constexpr int EG = 8;                                   // experts per wavefront
constexpr int LOGIT_GROUP = LOGIT_WAVES * EG;           // experts per workgroup
constexpr int MAX_E = 256;
constexpr int SELECT_THREADS = MAX_E;
constexpr int MAX_TOKENS_2R = 1024;                     // tokens of one two-round call (class bit set in LDS)
constexpr int TWO_ROUND_MASK_WORDS = MAX_E / 32;
constexpr int TWO_ROUND_STATE_WORDS = 64;               // 256 bytes of device state, cleared by the logits kernel

struct TwoRound {
    const uint8_t* token_class;    // [T] non-zero: first-round token
    uint32_t* mask_bits;           // E_A as a bit set, built with device-scope atomics by the first launch
    uint8_t* mask_out;             // [E] or null
    int32_t* n_activated_out;      // [1] or null
    int phase;                     // 0: the launch that routes the first-round tokens; 1: the one that routes the cold tokens
};

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

// Hash of one 16-byte chunk and its position in the row (multiply / shift-xor mixing).  Rows with equal bytes have equal
// hashes; the converse is confirmed byte by byte where it matters.
__device__ __forceinline__ unsigned long long chunk_hash(const uint4& v, uint32_t pos) {
    unsigned long long a = ((unsigned long long)v.y << 32 | v.x) + 0x9E3779B97F4A7C15ull * (pos + 1u);
    unsigned long long b = ((unsigned long long)v.w << 32 | v.z) ^ 0xC2B2AE3D27D4EB4Full;
    a ^= a >> 31; a *= 0xBF58476D1CE4E5B9ull;
    b ^= b >> 29; b *= 0x94D049BB133111EBull;
    unsigned long long h = a ^ (b + (a << 7) + (a >> 3));
    h ^= h >> 32; h *= 0xD6E8FEB86659FD93ull; h ^= h >> 29;
    return h;
}
__device__ __forceinline__ uint32_t wave_xor_u32(uint32_t v) {
    v ^= dpp_u32<DPP_XOR1>(v);
    v ^= dpp_u32<DPP_XOR2>(v);
    v ^= dpp_u32<DPP_HALF_MIRROR>(v);
    v ^= dpp_u32<DPP_MIRROR>(v);
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) ^ (uint32_t)__builtin_amdgcn_readlane((int)v, 16) ^
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) ^ (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

__device__ __forceinline__ void clear_select_state(uint32_t* __restrict__ zero_words, int n_zero, uint32_t* __restrict__ zero_count) {
    if (blockIdx.x != 0 || blockIdx.y != 0) return;
    if (zero_words && (int)threadIdx.x < n_zero) zero_words[threadIdx.x] = 0u;
    if (zero_count && threadIdx.x == 0) *zero_count = 0u;
}

template <typename ST>
__global__ __launch_bounds__(LOGIT_THREADS) void route_logits_kernel(const ST* __restrict__ x, const ST* __restrict__ w_router,
                                                                     float* __restrict__ logits, int H, int E,
                                                                     uint32_t* __restrict__ zero_words, int n_zero,
                                                                     uint32_t* __restrict__ zero_count,
                                                                     const int32_t* __restrict__ row_index, int n_rows,
                                                                     ST* __restrict__ x_dense,
                                                                     unsigned long long* __restrict__ row_hash) {
    constexpr int CN = Chunk<ST>::N;
    // state the selection kernel that follows starts from (two-round routing: bit set and arrival counter; repeated-row
    // search: the count of distinct rows)
    clear_select_state(zero_words, n_zero, zero_count);
    constexpr int XC = 4;          // chunks of the token row per lane per block of 256 chunks
    const int t = blockIdx.y;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x / WAVE;
    const int n_chunks = H / CN;   // chunks of CN consecutive elements; lane takes chunk lane, lane+64, ...
    const ST* xt = x + (size_t)token_row(row_index, n_rows, t) * H;
    const int e0 = blockIdx.x * LOGIT_GROUP + wave;     // this wavefront: experts e0, e0+4, ..., e0+28

    // fixed summation order (per lane ascending, then the cross-lane tree) -> deterministic
    float acc[EG];
#pragma unroll
    for (int g = 0; g < EG; ++g) acc[g] = 0.f;
    const bool first_wave_of_token = blockIdx.x == 0 && wave == 0;
    unsigned long long hash = 0ull;
    for (int cb = 0; cb < n_chunks; cb += WAVE * XC) {
        // 16-byte packed chunks stay packed in registers until they are multiplied
        uint4 xp[XC], wp[EG][XC];
#pragma unroll
        for (int j = 0; j < XC; ++j) {
            const int c = cb + j * WAVE + lane;
            xp[j] = c < n_chunks ? *reinterpret_cast<const uint4*>(xt + (size_t)c * CN) : make_uint4(0u, 0u, 0u, 0u);
            // dense copy of the live rows for the kernels that follow (one wavefront per token writes it)
            if (x_dense && first_wave_of_token && c < n_chunks)
                *reinterpret_cast<uint4*>(x_dense + (size_t)t * H + (size_t)c * CN) = xp[j];
            if (row_hash && first_wave_of_token && c < n_chunks) hash ^= chunk_hash(xp[j], (uint32_t)c);
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
    if (row_hash && first_wave_of_token) {              // exclusive-or of the chunk hashes: any order gives the same value
        const uint32_t lo = wave_xor_u32((uint32_t)hash), hi = wave_xor_u32((uint32_t)(hash >> 32));
        if (lane == 0) row_hash[t] = ((unsigned long long)hi << 32) | lo;
    }
}

// The same scores on the matrix cores (bf16 storage, calls of LOGIT_MFMA_MIN_TOKENS tokens or more): a workgroup computes a 16 x 16 tile (experts x tokens), its
// four wavefronts each a quarter of the reduction, operands loaded straight from global memory in MFMA layout (lane (n, q) of
// K-step s holds 8 consecutive columns 32 s + 8 q .. of row n), partial sums added in wavefront order through LDS.  A row of the
// router matrix is then read once per 16 tokens instead of once per token (T = 256 tokens over 256 experts: 32 MB from L2
// instead of 256 MB).  bf16 products are exact in fp32; only the order of the fp32 sums differs from the kernel above.
constexpr int LOGIT_TILE = 16;
constexpr int LOGIT_MFMA_MIN_TOKENS = 64;
__global__ __launch_bounds__(LOGIT_THREADS) void route_logits_mfma_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router,
                                                                          float* __restrict__ logits, int T, int H, int E,
                                                                          uint32_t* __restrict__ zero_words, int n_zero,
                                                                          uint32_t* __restrict__ zero_count,
                                                                          const int32_t* __restrict__ row_index, int n_rows,
                                                                          uint16_t* __restrict__ x_dense,
                                                                          unsigned long long* __restrict__ row_hash) {
    clear_select_state(zero_words, n_zero, zero_count);
    __shared__ f32x4_t s_part[LOGIT_WAVES][WAVE];
    __shared__ unsigned long long s_hash[LOGIT_WAVES][LOGIT_TILE];
    static_assert(LOGIT_WAVES == 4, "four partial sums and four partial hashes per tile");
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    const int n = lane & 15, q = lane >> 4;
    const int e0 = blockIdx.x * LOGIT_TILE, t0 = blockIdx.y * LOGIT_TILE;
    const int kw = H / LOGIT_WAVES;                                  // columns per wavefront, a multiple of 32
    // rows beyond the last expert / token repeat the last one; their results are not stored
    const int t_mine = min(t0 + n, T - 1);
    const int col0 = wave * kw + q * 8;
    const uint16_t* wp = w_router + (size_t)min(e0 + n, E - 1) * H + col0;
    const uint16_t* xp = x + (size_t)token_row(row_index, n_rows, t_mine) * H + col0;
    // the workgroups of the first expert tile also leave the dense copy of the live rows and the row hashes, as the kernel
    // above does (same chunk numbering; the exclusive-or of the chunk hashes does not depend on the order)
    const bool side_work = blockIdx.x == 0 && t0 + n < T;
    unsigned long long hash = 0ull;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    constexpr int STEPS = 16;                                        // K-steps whose loads are in flight together (one round trip for H = 2048)
    for (int k0 = 0; k0 < kw; k0 += 32 * STEPS) {
        bf16x8_t a[STEPS], b[STEPS];
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int k = min(k0 + 32 * s, kw - 32);                 // (a short last group re-reads its last step and skips it below)
            a[s] = *reinterpret_cast<const bf16x8_t*>(wp + k);
            b[s] = *reinterpret_cast<const bf16x8_t*>(xp + k);
        }
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            if (k0 + 32 * s >= kw) break;
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s], b[s], acc, 0, 0, 0);
            if (side_work) {
                const int col = col0 + k0 + 32 * s;
                if (x_dense) *reinterpret_cast<bf16x8_t*>(x_dense + (size_t)t_mine * H + col) = b[s];
                if (row_hash) hash ^= chunk_hash(__builtin_bit_cast(uint4, b[s]), (uint32_t)(col / 8));
            }
        }
    }
    s_part[wave][lane] = acc;
    if (row_hash && blockIdx.x == 0) {                               // a row's chunks sit in the four lanes n, n + 16, n + 32, n + 48
        uint32_t lo = (uint32_t)hash, hi = (uint32_t)(hash >> 32);
        lo ^= __shfl_xor(lo, 16); hi ^= __shfl_xor(hi, 16);
        lo ^= __shfl_xor(lo, 32); hi ^= __shfl_xor(hi, 32);
        if (q == 0) s_hash[wave][n] = ((unsigned long long)hi << 32) | lo;
    }
    __syncthreads();
    if (wave == 0) {
        f32x4_t v = s_part[0][lane];
#pragma unroll
        for (int w = 1; w < LOGIT_WAVES; ++w) v += s_part[w][lane];
        // lane holds experts e0 + 4 q + (0..3) of token t0 + n
        const int t = t0 + n, e = e0 + 4 * q;
        if (t < T) {
            float* dst = logits + (size_t)t * E + e;
            if (e + 3 < E && (E & 3) == 0) {
                *reinterpret_cast<f32x4_t*>(dst) = v;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (e + j < E) dst[j] = v[j];
            }
            if (row_hash && blockIdx.x == 0 && q == 0) row_hash[t] = s_hash[0][n] ^ s_hash[1][n] ^ s_hash[2][n] ^ s_hash[3][n];
        }
    }
}

// Selection key: larger logit wins, equal logits go to the lower expert id.  The float is mapped to an unsigned
// integer with the same order (minus infinity maps to 0x007fffff, the smallest image of a number); a NaN maps to 1, below
// every number; the id is stored complemented in the low word; 0 = not a candidate.
__device__ __forceinline__ unsigned long long select_key(float v, int e) {
    const uint32_t b = __float_as_uint(v);
    uint32_t ord = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    if (v != v) ord = 1u;
    return ((unsigned long long)ord << 32) | (uint32_t)(0xffffffffu - (uint32_t)e);
}

struct SelectLds {
    __attribute__((aligned(16))) unsigned long long key[MAX_E];   // 0 for experts that are not candidates
    float all[MAX_E];                                              // every logit (for the full softmax)
    float sel_logit[16];
    int32_t sel_idx[16];
    int32_t count[SELECT_THREADS / WAVE];
};

// Thread e ranks expert e among the candidates; on return (after a workgroup barrier) LDS holds the k selected experts in
// slot order and the number of candidates.  Returns whether expert e is one of the selected.  Threads e >= SELECT_THREADS of a
// larger workgroup only take part in the barriers (ok must be false for them).
__device__ __forceinline__ bool select_rank(SelectLds& sm, float v, bool ok, int e, int E, int k) {
    const int lane = e & (WAVE - 1);
    const unsigned long long my_key = ok ? select_key(v, e) : 0ull;
    if (e < 16) { sm.sel_idx[e] = -1; sm.sel_logit[e] = 0.f; }
    if (e < SELECT_THREADS) {
        sm.all[e] = e < E ? v : -INFINITY;
        sm.key[e] = my_key;
        const unsigned long long ok_lanes = __ballot(ok);
        if (lane == 0) sm.count[e / WAVE] = __popcll(ok_lanes);
    }
    __syncthreads();
    bool selected = false;
    if (ok) {                                                         // rank = number of candidates that beat this one
        int rank = 0;
        const int n2 = (E + 1) / 2;
#pragma unroll 8
        for (int j2 = 0; j2 < n2; ++j2) {
            const ulonglong2 o = *reinterpret_cast<const ulonglong2*>(sm.key + 2 * j2);   // same address in all lanes: broadcast
            rank += (o.x > my_key) + (o.y > my_key);
        }
        if (rank < k) { sm.sel_idx[rank] = e; sm.sel_logit[rank] = v; selected = true; }
    }
    __syncthreads();
    return selected;
}

// Gates of token t from the selection in LDS; called by wavefront 0 only, lane s owns slot s.
__device__ __forceinline__ void write_gates(const SelectLds& sm, int t, int lane, int E, int k, int renormalize,
                                            int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate) {
    int n_allowed = 0;
#pragma unroll
    for (int w = 0; w < SELECT_THREADS / WAVE; ++w) n_allowed += sm.count[w];
    const int k_eff = min(k, n_allowed);
    const float my_logit = lane < 16 ? sm.sel_logit[lane] : 0.f;
    float gate = 0.f;
    if (renormalize) {
        const float m = sm.sel_logit[0];
        const float w = lane < k_eff ? expf(my_logit - m) : 0.f;
        const float den = wave_sum(w);
        gate = lane < k_eff ? w / den : 0.f;
    } else {                                                         // selected entries of the softmax over all E experts
        float m = -INFINITY;
        for (int j = lane; j < E; j += WAVE) m = fmaxf(m, sm.all[j]);
        m = wave_max(m);
        float dsum = 0.f;
        for (int j = lane; j < E; j += WAVE) dsum += expf(sm.all[j] - m);
        const float den = wave_sum(dsum);
        gate = lane < k_eff ? expf(my_logit - m) / den : 0.f;
    }
    if (lane < k) {
        topk_idx[(size_t)t * k + lane] = lane < k_eff ? sm.sel_idx[lane] : -1;
        topk_gate[(size_t)t * k + lane] = gate;
    }
}

__device__ __forceinline__ void clear_ffn_ctrl(const CtrlZero& ctrl, int tid, int E) {
    if (tid < ctrl.header) ctrl.words[tid] = 0;
    if (tid < E) ctrl.words[ctrl.header + tid * ctrl.stride] = 0;
}

// First token j < t whose row holds the same row_bytes bytes as token t's (t itself if there is none); all threads of the
// workgroup take part and get the result.  Candidates are the tokens with the same (masked) hash, in ascending order; each is
// confirmed by comparing the rows.
template <int THREADS>
__device__ __forceinline__ int first_equal_row(const RowDedup& dd, const unsigned char* __restrict__ x, int row_bytes, int t, int tid) {
    __shared__ int s_best;
    const unsigned long long my_hash = dd.hash[t] & dd.hash_mask;
    const uint4* mine = reinterpret_cast<const uint4*>(x + (size_t)t * row_bytes);
    int after = -1;                                      // candidates up to here have been looked at
    while (true) {
        if (tid == 0) s_best = t;
        __syncthreads();
        for (int j = after + 1 + tid; j < t; j += THREADS)
            if ((dd.hash[j] & dd.hash_mask) == my_hash) { atomicMin(&s_best, j); break; }
        __syncthreads();
        const int cand = s_best;
        if (cand >= t) return t;
        const uint4* other = reinterpret_cast<const uint4*>(x + (size_t)cand * row_bytes);
        bool same = true;
        for (int c = tid; c < row_bytes / 16; c += THREADS) {
            const uint4 a = mine[c], b = other[c];
            same = same && a.x == b.x && a.y == b.y && a.z == b.z && a.w == b.w;
        }
        if (__syncthreads_and(same)) return cand;        // (also orders this round's reads of s_best before the next write)
        after = cand;
    }
}

// Repeated-row search for token t (all THREADS threads of the workgroup): writes rep[t], counts the tokens that are their own
// representative, and for a token that is not leaves its row of the routing table empty (it takes no part in the expert FFN:
// its result is its representative's).  Returns whether t is its own representative.
template <int THREADS>
__device__ __forceinline__ bool own_representative(const RowDedup& dd, const unsigned char* __restrict__ x, int row_bytes, int t, int tid,
                                                   int k, int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate) {
    const int rep = first_equal_row<THREADS>(dd, x, row_bytes, t, tid);
    if (tid == 0) {
        dd.rep[t] = rep;
        if (rep == t) atomicAdd(dd.n_unique, 1);
    }
    if (rep != t && tid < k) { topk_idx[(size_t)t * k + tid] = -1; topk_gate[(size_t)t * k + tid] = 0.f; }
    return rep == t;
}

__global__ __launch_bounds__(SELECT_THREADS) void route_select_kernel(const float* __restrict__ logits, const uint8_t* __restrict__ mask,
                                                                      int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate,
                                                                      int E, int k, int renormalize, CtrlZero ctrl, RowDedup dd,
                                                                      const unsigned char* __restrict__ x, int row_bytes) {
    __shared__ SelectLds sm;
    const int t = blockIdx.x;
    const int e = threadIdx.x;
    if (ctrl.words && t == 0) clear_ffn_ctrl(ctrl, e, E);   // control block of an expert FFN that follows without a dispatch kernel
    if (dd.hash && !own_representative<SELECT_THREADS>(dd, x, row_bytes, t, e, k, topk_idx, topk_gate)) return;
    float v = 0.f;
    bool ok = false;
    if (e < E) {
        v = logits[(size_t)t * E + e] + 0.f;                         // -0 -> +0 so that equal logits compare equal
        ok = mask == nullptr || mask[e] != 0;
    }
    select_rank(sm, v, ok, e, E, k);
    if (e < WAVE) write_gates(sm, t, e, E, k, renormalize, topk_idx, topk_gate);
}

// ---- two-round routing (Algorithm 1) -------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t load_agent(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

__global__ __launch_bounds__(SELECT_THREADS) void route_select_two_round_kernel(const float* __restrict__ logits, TwoRound tr,
                                                                                int32_t* __restrict__ topk_idx,
                                                                                float* __restrict__ topk_gate, int T, int E, int k,
                                                                                int renormalize, CtrlZero ctrl, RowDedup dd,
                                                                                const unsigned char* __restrict__ x, int row_bytes) {
    __shared__ SelectLds sm;
    __shared__ unsigned long long s_cls[MAX_TOKENS_2R / WAVE];   // bit t: token t is a first-round token
    __shared__ uint32_t s_bits[TWO_ROUND_MASK_WORDS];
    const int b = blockIdx.x;
    const int e = threadIdx.x;
    const int lane = e & (WAVE - 1);
    const int wave = e / WAVE;
    if (ctrl.words && b == 0 && tr.phase == 0) clear_ffn_ctrl(ctrl, e, E);

    // ---- which token is this workgroup's: the b-th in the order (first-round tokens ascending, then cold tokens ascending)
#pragma unroll
    for (int j = 0; j < MAX_TOKENS_2R / SELECT_THREADS; ++j) {
        const int tok = j * SELECT_THREADS + e;
        const bool first = tok < T && tr.token_class[tok] != 0;
        const unsigned long long bal = __ballot(first);
        if (lane == 0) s_cls[j * (SELECT_THREADS / WAVE) + wave] = bal;
    }
    __syncthreads();
    int n_first = 0, t = 0;
    {
        constexpr int NW = MAX_TOKENS_2R / WAVE;
        const int n_words = (T + WAVE - 1) / WAVE;
        int c1[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) { c1[w] = w < n_words ? __popcll(s_cls[w]) : 0; n_first += c1[w]; }
        const bool want_first = b < n_first;
        int target = want_first ? b : b - n_first;
        unsigned long long bits = 0ull;
        int word = 0;
        bool found = false;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const int left = T - w * WAVE;                                             // tokens of this word that exist
            const unsigned long long valid = left >= WAVE ? ~0ull : (left > 0 ? ((1ull << left) - 1ull) : 0ull);
            const unsigned long long cand = want_first ? s_cls[w] : (~s_cls[w] & valid);
            const int c = __popcll(cand);
            if (!found) {
                if (target < c) { found = true; word = w; bits = cand; }
                else target -= c;
            }
        }
        for (int i = 0; i < target; ++i) bits &= bits - 1ull;                          // drop the lower set bits
        t = word * WAVE + (bits ? __builtin_ctzll(bits) : 0);
    }
    const bool is_first = b < n_first;
    // ---- the launch this workgroup has nothing to route in: workgroup 0 publishes E_A where it is known, the others leave
    if (is_first != (tr.phase == 0)) {
        if (b == 0) {                                  // phase 0 without first-round tokens: E_A is empty; phase 1: E_A is complete
            if (e < TWO_ROUND_MASK_WORDS) s_bits[e] = tr.phase == 0 ? 0u : load_agent(tr.mask_bits + e);
            __syncthreads();
            if (tr.mask_out && e < E) tr.mask_out[e] = (uint8_t)((s_bits[e >> 5] >> (e & 31)) & 1u);
            if (tr.n_activated_out && e == 0) {
                int n = 0;
#pragma unroll
                for (int w = 0; w < TWO_ROUND_MASK_WORDS; ++w) n += __popc(s_bits[w]);
                *tr.n_activated_out = n;
            }
        }
        return;
    }
    // A repeated row is routed and computed once, for its first occurrence.  As a first-round token it still adds its picks to
    // E_A (its first occurrence may be a cold token; the picks then lie inside E_A, so that token's restricted routing is the
    // free one and serves both); as a cold token it has nothing left to do.
    bool keeps_row = true;
    if (dd.hash) {
        keeps_row = own_representative<SELECT_THREADS>(dd, x, row_bytes, t, e, k, topk_idx, topk_gate);
        if (!keeps_row && !is_first) return;
    }

    float v = 0.f;
    bool ok = false;
    if (e < E) {
        v = logits[(size_t)t * E + e] + 0.f;
        ok = true;
    }
    if (!is_first) {
        // ---- cold token: E_A is complete (the launch that built it has ended); route inside it
        if (e < TWO_ROUND_MASK_WORDS) s_bits[e] = load_agent(tr.mask_bits + e);
        __syncthreads();
        ok = ok && ((s_bits[e >> 5] >> (e & 31)) & 1u);
    }
    const bool selected = select_rank(sm, v, ok, e, E, k);
    if (is_first) {
        // ---- first-round token: E_A |= picks
        const unsigned long long sel_lanes = __ballot(selected);
        if (lane == 0) {
            const uint32_t lo = (uint32_t)sel_lanes, hi = (uint32_t)(sel_lanes >> 32);
            if (lo) __hip_atomic_fetch_or(tr.mask_bits + 2 * wave, lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (hi) __hip_atomic_fetch_or(tr.mask_bits + 2 * wave + 1, hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (keeps_row && e < WAVE) write_gates(sm, t, e, E, k, renormalize, topk_idx, topk_gate);
}

// ---- two-round routing for calls of at most LOCAL_2R_MAX_TOKENS tokens: E_A is rebuilt by every workgroup -------------------
constexpr int LOCAL_2R_MAX_TOKENS = 256;             // (beyond that the redundant first-round work per workgroup outgrows one exchange through memory)
constexpr int LOCAL_2R_THREADS = 1024;                 // 16 wavefronts share the first-round tokens; the first 4 then select

__global__ __launch_bounds__(LOCAL_2R_THREADS) void route_select_two_round_local_kernel(const float* __restrict__ logits,
                                                                                        const uint8_t* __restrict__ token_class,
                                                                                        uint8_t* __restrict__ mask_out,
                                                                                        int32_t* __restrict__ n_activated_out,
                                                                                        int32_t* __restrict__ topk_idx,
                                                                                        float* __restrict__ topk_gate, int T, int E, int k,
                                                                                        int renormalize, CtrlZero ctrl, RowDedup dd,
                                                                                        const unsigned char* __restrict__ x, int row_bytes) {
    __shared__ SelectLds sm;
    __shared__ uint32_t s_bits[TWO_ROUND_MASK_WORDS];
    const int t = blockIdx.x;
    const int e = threadIdx.x;
    const int lane = e & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(e / WAVE);
    if (ctrl.words && t == 0 && e < SELECT_THREADS) clear_ffn_ctrl(ctrl, e, E);
    // A repeated row is routed once, for its first occurrence (token 0 is always one, so the outputs below are written).  E_A is
    // built from every first-round token, repeated or not: a cold first occurrence of a first-round row finds that row's free
    // picks inside E_A, and its restricted routing is the free one.
    if (dd.hash && !own_representative<LOCAL_2R_THREADS>(dd, x, row_bytes, t, e, k, topk_idx, topk_gate)) return;
    if (e < TWO_ROUND_MASK_WORDS) s_bits[e] = 0u;
    // one memory round trip: the token classes (every wavefront builds the bit set of first-round tokens for itself) and
    // this token's own logits
    constexpr int WORDS = LOCAL_2R_MAX_TOKENS / WAVE;
    bool lane_first[WORDS];
#pragma unroll
    for (int w = 0; w < WORDS; ++w) lane_first[w] = lane + WAVE * w < T && token_class[lane + WAVE * w] != 0;
    float v = 0.f;
    if (e < E) v = logits[(size_t)t * E + e] + 0.f;
    unsigned long long first_set[WORDS];
    int n_first = 0;
    bool is_first = false;
#pragma unroll
    for (int w = 0; w < WORDS; ++w) {
        first_set[w] = __ballot(lane_first[w]);
        n_first += __popcll(first_set[w]);
        if ((t >> 6) == w) is_first = (first_set[w] >> (t & 63)) & 1ull;
    }
    __syncthreads();                                   // s_bits is cleared
    // ---- E_A = union of the picks of the first-round tokens.  Needed by cold tokens, and by workgroup 0 for the outputs.
    // Wavefront w takes the w-th, (w+16)-th, ... first-round token: k rounds of a cross-lane maximum over the selection keys.
    if ((!is_first || t == 0) && n_first > 0) {
        int ordinal = 0;                               // first-round tokens seen so far (every wavefront walks the whole set)
#pragma unroll
        for (int w = 0; w < WORDS; ++w)
        for (unsigned long long rest = first_set[w]; rest != 0ull; rest &= rest - 1ull, ++ordinal) {
            if (ordinal % (LOCAL_2R_THREADS / WAVE) != wave) continue;
            const int tok = WAVE * w + __builtin_ctzll(rest);
            const float* row = logits + (size_t)tok * E;
            unsigned long long key[MAX_E / WAVE];        // expert lane + 64 i
#pragma unroll
            for (int i = 0; i < MAX_E / WAVE; ++i) {
                const int ex = lane + WAVE * i;
                const float lv = ex < E ? row[ex] + 0.f : 0.f;
                key[i] = ex < E ? select_key(lv, ex) : 0ull;
            }
            for (int r = 0; r < k; ++r) {
                unsigned long long mine = key[0];
#pragma unroll
                for (int i = 1; i < MAX_E / WAVE; ++i) mine = key[i] > mine ? key[i] : mine;
                const unsigned long long best = wave_max_u64(mine);
                if (best == 0ull) break;                 // fewer than k experts
                if (mine == best) {                      // keys are distinct: exactly one lane, one of its slots
                    const int ex = (int)(0xffffffffu - (uint32_t)best);
                    atomicOr(&s_bits[ex >> 5], 1u << (ex & 31));
#pragma unroll
                    for (int i = 0; i < MAX_E / WAVE; ++i)
                        if (key[i] == best) key[i] = 0ull;
                }
            }
        }
    }
    __syncthreads();
    if (t == 0) {
        if (mask_out && e < E) mask_out[e] = (uint8_t)((s_bits[e >> 5] >> (e & 31)) & 1u);
        if (n_activated_out && e == 0) {
            int n = 0;
#pragma unroll
            for (int w = 0; w < TWO_ROUND_MASK_WORDS; ++w) n += __popc(s_bits[w]);
            *n_activated_out = n;
        }
    }
    // ---- this token's own selection: over all experts (first round) or inside E_A (cold)
    const bool ok = e < E && (is_first || ((s_bits[e >> 5] >> (e & 31)) & 1u));
    select_rank(sm, v, ok, e, E, k);
    if (e < WAVE) write_gates(sm, t, e, E, k, renormalize, topk_idx, topk_gate);
}

static hipError_t launch_logits(const Dims& d, const void* x, const void* w_router, float* logits, uint32_t* zero_words, int n_zero,
                                hipStream_t s, const RowDedup& dedup = RowDedup()) {
    unsigned long long* row_hash = dedup.hash;
    uint32_t* zero_count = dedup.hash ? (uint32_t*)dedup.n_unique : nullptr;
    // bf16, a hidden size the four wavefronts can split into K-steps, and enough tokens to fill tiles: the matrix-core kernel
    // (with one block of 32 tokens it has only 16 workgroups and is 0.5-1 us slower than the kernel above; with 128 tokens it
    // is 1.3 us faster, with 256 tokens over 256 experts 14 us)
    const int force = tuning().logits_kernel.load();                // tuning aid: 1 / 2 = the per-token / the matrix-core kernel for every token count
    const bool many_tokens = force ? force == 2 : d.T >= LOGIT_MFMA_MIN_TOKENS;
    if (d.bf16 && d.H % (32 * LOGIT_WAVES) == 0 && many_tokens) {
        dim3 tiles((d.E + LOGIT_TILE - 1) / LOGIT_TILE, (d.T + LOGIT_TILE - 1) / LOGIT_TILE);
        hipLaunchKernelGGL(route_logits_mfma_kernel, tiles, dim3(LOGIT_THREADS), 0, s, (const uint16_t*)x, (const uint16_t*)w_router, logits,
                           d.T, d.H, d.E, zero_words, n_zero, zero_count, d.row_index, d.n_rows, (uint16_t*)d.x_dense, row_hash);
        return hipGetLastError();
    }
    dim3 grid((d.E + LOGIT_GROUP - 1) / LOGIT_GROUP, d.T), block(LOGIT_THREADS);
    if (d.bf16)
        hipLaunchKernelGGL(route_logits_kernel<uint16_t>, grid, block, 0, s, (const uint16_t*)x, (const uint16_t*)w_router, logits, d.H,
                           d.E, zero_words, n_zero, zero_count, d.row_index, d.n_rows, (uint16_t*)d.x_dense, row_hash);
    else
        hipLaunchKernelGGL(route_logits_kernel<float>, grid, block, 0, s, (const float*)x, (const float*)w_router, logits, d.H, d.E,
                           zero_words, n_zero, zero_count, d.row_index, d.n_rows, (float*)d.x_dense, row_hash);
    return hipGetLastError();
}

// The repeated-row search compares the rows of the call: the caller's dense x, or the dense copy of the live rows the logits
// kernel has just written.
static bool dedup_args_ok(const Dims& d, const RowDedup& dedup, int row_bytes) {
    if (!dedup.hash) return true;
    return row_bytes % 16 == 0 && dedup.rep && dedup.n_unique && (!d.row_index || d.x_dense);
}
static const unsigned char* searched_rows(const Dims& d, const void* x) {
    return (const unsigned char*)(d.row_index ? d.x_dense : x);
}

hipError_t launch_route(const Dims& d, const void* x, const void* w_router, const uint8_t* mask, int32_t* topk_idx,
                        float* topk_gate, float* logits, CtrlZero ctrl, hipStream_t s, RowDedup dedup) {
    const int row_bytes = d.H * (d.bf16 ? 2 : 4);
    if (!dedup_args_ok(d, dedup, row_bytes)) return hipErrorInvalidValue;
    hipError_t err = launch_logits(d, x, w_router, logits, nullptr, 0, s, dedup);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(route_select_kernel, dim3(d.T), dim3(SELECT_THREADS), 0, s, logits, mask, topk_idx, topk_gate, d.E, d.k,
                       d.renormalize, ctrl, dedup, searched_rows(d, x), row_bytes);
    return hipGetLastError();
}

hipError_t launch_route_two_round(const Dims& d, const void* x, const void* w_router, const uint8_t* token_class, uint8_t* mask_out,
                                  int32_t* n_activated_out, int32_t* topk_idx, float* topk_gate, float* logits, void* state,
                                  CtrlZero ctrl, hipStream_t s, RowDedup dedup) {
    if (d.T > MAX_TOKENS_2R || d.E > 32 * TWO_ROUND_MASK_WORDS) return hipErrorInvalidValue;
    const int row_bytes = d.H * (d.bf16 ? 2 : 4);
    if (!dedup_args_ok(d, dedup, row_bytes)) return hipErrorInvalidValue;
    uint32_t* words = (uint32_t*)state;                 // [0..7] bit set E_A
    if (d.T <= LOCAL_2R_MAX_TOKENS) {                   // every workgroup rebuilds E_A itself, nothing is exchanged
        hipError_t err = launch_logits(d, x, w_router, logits, nullptr, 0, s, dedup);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(route_select_two_round_local_kernel, dim3(d.T), dim3(LOCAL_2R_THREADS), 0, s, logits, token_class, mask_out,
                           n_activated_out, topk_idx, topk_gate, d.T, d.E, d.k, d.renormalize, ctrl, dedup, searched_rows(d, x), row_bytes);
        return hipGetLastError();
    }
    hipError_t err = launch_logits(d, x, w_router, logits, words, TWO_ROUND_STATE_WORDS, s, dedup);
    if (err != hipSuccess) return err;
    TwoRound tr;
    tr.token_class = token_class; tr.mask_bits = words; tr.mask_out = mask_out; tr.n_activated_out = n_activated_out;
    for (tr.phase = 0; tr.phase < 2; ++tr.phase) {
        hipLaunchKernelGGL(route_select_two_round_kernel, dim3(d.T), dim3(SELECT_THREADS), 0, s, logits, tr, topk_idx, topk_gate, d.T,
                           d.E, d.k, d.renormalize, ctrl, dedup, searched_rows(d, x), row_bytes);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    return hipSuccess;
}

}  // namespace team
