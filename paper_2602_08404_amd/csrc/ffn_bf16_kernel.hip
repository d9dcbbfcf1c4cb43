// Grouped SwiGLU expert FFN over the activated experts, bf16 storage, gfx950 MFMA, HBM-streaming design.
//
// Paper context: block-level decoding is memory-bound (Section "Delayed Caching for Decoded Tokens"), latency
// is dominated by the feed-forward layers and every activated expert serves only a few tokens (Section
// "Speculative Exploration for Hot Tokens").  So the cost of this step is reading the weights of the experts
// that received tokens, once, at HBM speed; the arithmetic rides along on the matrix cores.
//
// ONE persistent kernel does both GEMMs.  Work items:
//   gate/up items : (active expert, 8 consecutive intermediate indices) = 8 rows of w_gate + 8 rows of w_up,
//                   all H columns; h = silu(g) * u is formed in the epilogue and stored as bf16;
//   down items    : (active expert, 16*RB consecutive output rows of w_down), all I columns; fp32 out.
// The grid is exactly the number of workgroups the device holds at once.  Workgroup b owns the b-th of G
// contiguous shares (equal up to one item) of the gate/up item list and then the b-th share of the down item list (lists in
// expert-major order, computed on the device from n_active, so experts without tokens cost nothing and the
// host never reads device data).  Consecutive items of a share belong to the same expert, so the token
// operand stays in registers; and because both lists are cut at the same fractions, the down items of a
// workgroup belong to the expert(s) whose gate/up items it and its neighbours have just finished.  A down
// item waits (bounded spin on a per-expert counter) until every gate/up item of its expert has published h.
// Gate/up items never wait and every workgroup is resident (the host sizes the grid from the occupancy the
// runtime reports), so every wait ends.
//
// Inside a workgroup the reduction dimension is split over the 4 wavefronts.  Each wavefront pulls its slice of the
// item's weight rows HBM -> LDS with 16-byte-per-lane direct-to-LDS loads into a region of its own, as one continuous
// stream: the slice is cut into stages of two MFMA K-steps, and as soon as a stage has been read the same stage of the
// NEXT item is requested into the same bytes, so a wavefront's loads never stop - not during the reduction or the
// epilogue, not at item boundaries (only a publication of h drains them).  The loads carry the non-temporal hint.
// v_mfma_f32_16x16x32 bf16 takes the weights as the 16-row operand and up to 32 token rows as the 16-column operand
// (held in registers).  Partial sums of the 4 wavefronts are added in a fixed order through LDS (deterministic, no
// float atomics).  h of a run of gate/up items is kept in LDS and stored in one go when the run is published, because
// a store between weight loads holds up the in-order load pipeline until it is acknowledged.
//
// Weights may also be stored as 8-bit E4M3 codes with one float scale per matrix row (template parameter WB = bytes per
// weight).  The stream, the LDS layout and the waits are the same with half the bytes; a 16-byte LDS read then carries the
// operands of two MFMA K-steps, which are widened to bf16 in registers (exactly), the token operand is laid out to match,
// and the row scales multiply the fp32 sums in the epilogues.
//
// Two more things happen in this kernel.  (1) For small calls (at most 128 tokens and 1024 routed rows) started by
// team_moe_layer_forward, every workgroup groups the routing table itself in LDS during its prologue (the same
// bitset / popcount / prefix-sum method as the dispatch kernel, which is then not launched).  (2) When a call
// averages many rows per expert, all workgroups switch to the streaming body in ffn_bf16_tiled.hpp.
#include <atomic>

#include "ffn_bf16.hpp"
#include "ffn_bf16_tiled.hpp"

namespace team {

namespace {

constexpr int NT = 2;                    // token tiles of 16 rows handled per pass (32 tokens)
constexpr int H_BUF_ITEMS = 7;           // gate/up items whose h is held back in LDS (what is left of the workgroup's 80 KB)

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// 64 lanes x 16 bytes, each lane from its own global address, land contiguously at lds_base + lane*16.  The loads carry the
// non-temporal hint: weights are read exactly once per call, and without the hint the stream pushes the small reused data
// (token rows, h, the output rows being written) out of L2 over and over, which costs far more than those bytes suggest.
__device__ __forceinline__ void slab_load(const void* gsrc, char* lds_base_uniform) {
    __builtin_amdgcn_global_load_lds((gptr_t)gsrc, (lptr_t)lds_base_uniform, 16, 0, /*nt*/ 2);
}
// Waits until every outstanding vector-memory operation of this wavefront (loads, direct-to-LDS loads and
// stores: one counter on this architecture) has completed.
__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// h travels between workgroups that may sit on different XCDs (each with its own L2) inside one launch.
// Both sides use device-scope accesses (the stores write through to the device-coherent level, the loads do
// not use possibly stale cache lines), so no cache-wide write-back or invalidate is needed around the
// per-expert counter: those cost far more than the item they would guard.
__device__ __forceinline__ void store_coherent(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16 bytes of h at byte offset `off` of the buffer `rsrc` describes, as one device-scope load (a buffer load can carry the
// scope in its cache-policy bits; 16 is the device-scope bit of this architecture's encoding).  Offsets beyond the
// descriptor's size read as zero.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_bits;
__device__ __forceinline__ bf16x8_t load_coherent_16(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
    const u32x4_bits v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, /*sc1*/ 16);
    return __builtin_bit_cast(bf16x8_t, v);
}
// Returns v, but opaque to the optimiser: values derived from the result are recomputed where they are used
// instead of being hoisted out of the item loop and kept in registers (the token operand needs those registers).
__device__ __forceinline__ int opaque(int v) {
    asm volatile("" : "+v"(v));
    return v;
}

// One 32-bit load at (uniform base + per-lane byte offset), complete on return.
// The five idle cycles in front of the load are required, not tuning: under register pressure the compiler keeps the base
// pointer in lanes of a vector register and moves it back into scalar registers (v_readlane) directly in front of this
// statement.  A scalar register written by a vector instruction may only be read as a memory instruction's base address five
// cycles later; the compiler keeps that distance for loads it emits itself but cannot see into this one, and a load issued
// too early uses a stale base: an access to an arbitrary address.
__device__ __forceinline__ int global_read_i32(const int32_t* base_uniform, uint32_t byte_off) {
    int v;
    asm volatile("s_nop 4\n\tglobal_load_dword %0, %1, %2\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(byte_off), "s"(base_uniform) : "memory");
    return v;
}
__device__ __forceinline__ int lds_read_u16(uint32_t a) {
    int v;
    asm volatile("ds_read_u16 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a) : "memory");
    return v;
}
__device__ __forceinline__ uint32_t lds_read_u32(uint32_t a) {
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a) : "memory");
    return v;
}
__device__ __forceinline__ void lds_write_u32(uint32_t a, uint32_t v) { asm volatile("ds_write_b32 %0, %1" ::"v"(a), "v"(v) : "memory"); }
// LDS accesses and the workgroup barrier as explicit instructions (see the item loop for why).
// 16-byte accesses with a constant byte offset in the instruction: the partial sums of the four wavefronts sit at fixed
// distances from one per-lane address, so one address register serves all of them.
template <int OFF>
__device__ __forceinline__ void lds_write_f4_at(uint32_t a, const f32x4_t& v) {
    asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(a), "v"(v), "n"(OFF) : "memory");
}
template <int OFF>
__device__ __forceinline__ f32x4_t lds_read_f4_at(uint32_t a) {
    f32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a), "n"(OFF) : "memory");
    return v;
}
// Sum of the four wavefronts' partial sums, STRIDE bytes apart, added in wavefront order.
template <int STRIDE>
__device__ __forceinline__ f32x4_t lds_sum4(uint32_t a) {
    static_assert(FFN_WAVES == 4 && 3 * STRIDE + 16 <= 65536, "four partial sums within the instruction's offset range");
    f32x4_t v = lds_read_f4_at<0>(a);
    v += lds_read_f4_at<STRIDE>(a);
    v += lds_read_f4_at<2 * STRIDE>(a);
    v += lds_read_f4_at<3 * STRIDE>(a);
    return v;
}
// A matrix instruction's result may only be read by a memory instruction a number of cycles after it was issued.  The compiler
// inserts that distance for instructions it knows, not for the explicit LDS writes above, so the accumulators pass through this
// first: it is ordered after the matrix instructions that produce them (operands) and idles for longer than any of them needs.
template <int N>
__device__ __forceinline__ void settle_accumulators(f32x4_t (&acc)[N]) {
    if constexpr (N == 2) asm volatile("s_nop 15\n\ts_nop 7" : "+v"(acc[0]), "+v"(acc[1]));
    else asm volatile("s_nop 15\n\ts_nop 7" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]));
}
// Every LDS operation of this wavefront has completed, then all wavefronts of the workgroup meet.  Vector-memory
// operations in flight are NOT waited for.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

constexpr int cmax(int a, int b) { return a > b ? a : b; }

// LDS layout of a wavefront's slice of a 16-row weight sub-tile (KS K-steps of 32 columns = C chunks of 16 bytes per row).
// The slice is cut into stages of two K-steps: a stage is 16 rows x 8 chunks = 2 KB = two direct-to-LDS slabs (rows 0-7 and
// 8-15), lane l of a slab fetching row l/8, so every row contributes a 128-byte segment.  Inside a row of a stage chunk c sits
// at slot c ^ ((row >> 1) & 7), which spreads the 16 rows of one MFMA operand read over the LDS banks.  A stage can be consumed
// as soon as its two slabs have arrived and refilled as soon as it has been read.
template <int KS>
struct Staged {
    static constexpr int C = 4 * KS;                  // chunks per row of the slice
    static constexpr int S = (KS + 1) / 2;            // stages per sub-tile
    static constexpr int BYTES = S * 2048;            // LDS bytes of one sub-tile slice
    __device__ static __forceinline__ int swz(int row) { return (row >> 1) & 7; }
    // lane ln of slab `half` of stage st: the row it fetches and the chunk of that row (may be >= C in the last stage of an
    // odd KS: such lanes fetch nothing)
    __device__ static __forceinline__ int slab_row(int half, int ln) { return 8 * half + (ln >> 3); }
    __device__ static __forceinline__ int slab_chunk(int st, int half, int ln) { return 8 * st + ((ln & 7) ^ swz(slab_row(half, ln))); }
    // byte offset inside the sub-tile slice of the operand of K-step 2*st + u for MFMA lane (n, q)
    __device__ static __forceinline__ int read_off(int n, int st, int u, int q) {
        return st * 2048 + (n >> 3) * 1024 + (((n & 7) * 8) + ((4 * u + q) ^ swz(n))) * 16;
    }
};

// Waits until at most n (even, 0..46) vector-memory operations of this wavefront are outstanding; n is a constant after
// unrolling, so the switch folds to one instruction.  Anything else waits for all of them.
__device__ __forceinline__ void wait_outstanding(int n) {
#define TEAM_WAIT_CASE(N) \
    case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
    switch (n) {
        TEAM_WAIT_CASE(2) TEAM_WAIT_CASE(4) TEAM_WAIT_CASE(6) TEAM_WAIT_CASE(8) TEAM_WAIT_CASE(10) TEAM_WAIT_CASE(12)
        TEAM_WAIT_CASE(14) TEAM_WAIT_CASE(16) TEAM_WAIT_CASE(18) TEAM_WAIT_CASE(20) TEAM_WAIT_CASE(22) TEAM_WAIT_CASE(24)
        TEAM_WAIT_CASE(26) TEAM_WAIT_CASE(28) TEAM_WAIT_CASE(30) TEAM_WAIT_CASE(32) TEAM_WAIT_CASE(34) TEAM_WAIT_CASE(36)
        TEAM_WAIT_CASE(38) TEAM_WAIT_CASE(40) TEAM_WAIT_CASE(42) TEAM_WAIT_CASE(44) TEAM_WAIT_CASE(46)
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
#undef TEAM_WAIT_CASE
}
// Two / one 16-byte LDS reads, complete on return (explicit instructions: see the item loop).
__device__ __forceinline__ void lds_read2(uint32_t a0, uint32_t a1, bf16x8_t& w0, bf16x8_t& w1) {
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)" : "=&v"(w0), "=&v"(w1) : "v"(a0), "v"(a1) : "memory");
}
__device__ __forceinline__ void lds_read1(uint32_t a0, bf16x8_t& w0) {
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(w0) : "v"(a0) : "memory");
}

// Row scales are read through the scalar cache (same address in every lane; the tables are never written by the kernel): that
// path has its own counter, so waiting for a scale does not wait for the weight loads in flight.
typedef const __attribute__((address_space(4))) float* const_f32_ptr;
template <int N>
__device__ __forceinline__ void load_uniform(const float* base_uniform, float (&v)[N]) {
    const_f32_ptr p = (const_f32_ptr)base_uniform;
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = p[i];
}
// v[4*q + j] for a lane-dependent q in 0..3 out of 16 uniform values
[[maybe_unused]] __device__ __forceinline__ float pick4(const float (&v)[16], int q, int j) {
    const float lo = q == 0 ? v[j] : v[4 + j], hi = q == 2 ? v[8 + j] : v[12 + j];
    return q < 2 ? lo : hi;
}

// A use of every operand register, placed in the branch that has just loaded them: the compiler's wait for those loads then
// sits in that branch, and not in front of the first matrix instruction of every item, where it would also wait for all the
// weights in flight.
template <int KS, int KSM_>
__device__ __forceinline__ void settle(bf16x8_t (&opr)[NT][KSM_]) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(opr[nt][s]));
}

// Products of one item (one pass over up to 32 token rows) for one wavefront, stage by stage.
// The item's weights may still be arriving: before stage g the wavefront waits until at most the loads issued after that
// stage are outstanding.  Loads complete in issue order, so that is a count: the later stages of this item, plus, when
// PREFETCH, the stages of the next item already requested (two slabs per stage, g of them by then).  Other loads or stores
// issued after the stage only make the wait stricter than needed.
//   PREFETCH : right after stage g has been read, next_stage(g) requests stage g of the next item into the same LDS bytes
//              (it must issue exactly two slab loads).
//   WB == 1  : KS counts 64-byte units of E4M3 codes; a unit is two K-steps (see widen_e4m3 and the token operand's layout).
template <class ST, int KS, int RBN, bool PREFETCH, bool TWO, int WB, int KSM_, class NextStage>
__device__ __forceinline__ void stream_item(uint32_t region, int n, int q, const bf16x8_t (&opr)[NT][KSM_], f32x4_t (&acc)[RBN][NT],
                                            NextStage&& next_stage) {
    constexpr int NST = RBN * ST::S;
#pragma unroll
    for (int g = 0; g < NST; ++g) {
        const int rb = g / ST::S, st = g % ST::S;
        wait_outstanding(PREFETCH ? 2 * (NST - 1) : 2 * (NST - 1 - g));
        const bool second = 2 * st + 1 < KS;
        bf16x8_t w0, w1;
        const uint32_t base = region + rb * ST::BYTES;
        if (second) lds_read2(base + ST::read_off(n, st, 0, q), base + ST::read_off(n, st, 1, q), w0, w1);
        else lds_read1(base + ST::read_off(n, st, 0, q), w0);
        if (PREFETCH) next_stage(g);
        if constexpr (WB == 2) {
            acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w0, opr[0][2 * st], acc[rb][0], 0, 0, 0);
            if (TWO) acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w0, opr[1][2 * st], acc[rb][1], 0, 0, 0);
            if (second) {
                acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1, opr[0][2 * st + 1], acc[rb][0], 0, 0, 0);
                if (TWO) acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1, opr[1][2 * st + 1], acc[rb][1], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (u == 1 && !second) break;
                bf16x8_t wa, wb;
                widen_e4m3(u == 0 ? w0 : w1, wa, wb);
                const int s0 = 4 * st + 2 * u;                 // K-steps of unit 2*st + u
                acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, opr[0][s0], acc[rb][0], 0, 0, 0);
                if (TWO) acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, opr[1][s0], acc[rb][1], 0, 0, 0);
                acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, opr[0][s0 + 1], acc[rb][0], 0, 0, 0);
                if (TWO) acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, opr[1][s0 + 1], acc[rb][1], 0, 0, 0);
            }
        }
    }
}

}  // namespace

// KSA = H / 128 and KSB = I / 128: MFMA K-steps (of 32) per wavefront in the two GEMMs; RB = 16-row sub-tiles
// of w_down per down item; WB = bytes per weight (2: bf16; 1: E4M3 codes with the row scales sg, su, sd).
template <int KSA, int KSB, int RB, int WB>
__global__ __launch_bounds__(FFN_THREADS, 2) void ffn_fused_kernel(const uint16_t* __restrict__ x, const int32_t* __restrict__ offsets,
                                                                   const int32_t* __restrict__ sorted_token,
                                                                   const int32_t* __restrict__ active, const int32_t* __restrict__ n_active,
                                                                   const unsigned char* __restrict__ wg, const unsigned char* __restrict__ wu,
                                                                   const unsigned char* __restrict__ wd, uint16_t* __restrict__ h,
                                                                   float* __restrict__ out, FfnCtrl* __restrict__ ctrl, int T, int k, int E,
                                                                   int spin_limit, int skip_publish, unsigned long long* __restrict__ fail_mark,
                                                                   int tiled_min_avg_rows, int expert_major_ok, int wide_min_avg_rows,
                                                                   const int32_t* __restrict__ topk_idx, int32_t* __restrict__ inv_pos_out,
                                                                   const float* __restrict__ sg, const float* __restrict__ su,
                                                                   const float* __restrict__ sd) {
    static_assert(WB == 2 || (WB == 1 && KSA % 2 == 0 && KSB % 2 == 0), "8-bit weights: whole 64-byte units per wavefront");
    constexpr int UA = KSA * WB / 2, UB = KSB * WB / 2;           // 64-byte units of a weight row per wavefront
    using SA = Staged<UA>;
    using SB = Staged<UB>;
    constexpr int H = KSA * 128, I = KSB * 128;
    constexpr int KSLICE_A = KSA * 32, KSLICE_B = KSB * 32;       // columns per wavefront
    constexpr int KSM = cmax(KSA, KSB);
    constexpr int W_A = FFN_WAVES * SA::BYTES, W_B = FFN_WAVES * RB * SB::BYTES;
    constexpr int RED_A = FFN_WAVES * NT * WAVE * 16, RED_B = FFN_WAVES * RB * NT * WAVE * 16;
    constexpr int LDS_BYTES = cmax(cmax(W_A + RED_A, W_B + RED_B), tiled::RING_BYTES);   // the streaming variant reuses s_mem
    constexpr int TILES_A = I / 8, TILES_B = H / (16 * RB);
    __shared__ __attribute__((aligned(1024))) char s_mem[LDS_BYTES];
    __shared__ int32_t s_slot_e[FFN_MAX_E];
    __shared__ int32_t s_off[FFN_MAX_E + 1];
    __shared__ uint16_t s_sorted[FFN_LAYER_MAX_ROWS];    // token of every row (0xffff: none), when the table fits
    __shared__ uint32_t s_hbuf[H_BUF_ITEMS][NT][WAVE];   // h of the gate/up items of the current slot run, until it is published
    __shared__ int32_t s_nact;
    __shared__ uint32_t s_wait_failed;                   // set by thread 0 when a wait for another workgroup gave up

    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int A = T * k;
    const int G = gridDim.x;

    if (tid == 0) s_wait_failed = 0u;                    // (a workgroup barrier follows in every path before the first wait)
    int n_act;
    const bool own_tables = topk_idx != nullptr;
    // the token of every row sits in LDS when the table fits (always, when the kernel groups the routing table itself)
    const bool lds_tokens = own_tables || A <= FFN_LAYER_MAX_ROWS;
    if (!own_tables) {
        // ---- tables into LDS (one global round trip)
        n_act = min(max(*n_active, 0), E);
        for (int i = tid; i < E; i += FFN_THREADS) s_slot_e[i] = active[i];
        for (int i = tid; i <= E; i += FFN_THREADS) s_off[i] = min(max(offsets[i], 0), A);
        if (lds_tokens)
            for (int i = tid; i < A; i += FFN_THREADS) {
                const int t = sorted_token[i];
                s_sorted[i] = (t >= 0 && t < T) ? (uint16_t)t : (uint16_t)0xffffu;
            }
    } else {
        // ---- small calls (T <= FFN_LAYER_MAX_TOKENS, at most FFN_LAYER_MAX_ROWS pairs): every workgroup groups the routing table itself,
        // in LDS, instead of waiting for a separate grouping kernel.  Same method and same result as that kernel: a token
        // bitset per expert, popcount histogram, prefix sum, and the row of a pair = offset + number of lower tokens.
        constexpr int BW = FFN_LAYER_MAX_TOKENS / 32;                                     // words of a token bitset
        constexpr int BS = BW | 1;                // words from one expert's bitset to the next: odd, so that threads working on
                                                  // different experts read different LDS banks
        static_assert(BS * FFN_MAX_E * 4 + 16 <= LDS_BYTES, "prologue tables fit the weight area");
        uint32_t* bits = reinterpret_cast<uint32_t*>(s_mem);                              // [E][BW]
        uint32_t* wave_total = reinterpret_cast<uint32_t*>(s_mem + BS * FFN_MAX_E * 4);   // [4]
        // the table is requested first; clearing the bitsets and the barrier pass while it is on its way
        int my_e[FFN_LAYER_MAX_ROWS / FFN_THREADS];
#pragma unroll
        for (int j = 0; j < FFN_LAYER_MAX_ROWS / FFN_THREADS; ++j) {
            const int r = tid + j * FFN_THREADS;
            int e = r < A ? topk_idx[r] : -1;
            if (e >= E) e = -1;
            my_e[j] = e;
        }
        for (int i = tid; i < BS * E; i += FFN_THREADS) bits[i] = 0u;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < FFN_LAYER_MAX_ROWS / FFN_THREADS; ++j) {
            const int r = tid + j * FFN_THREADS;
            if (my_e[j] >= 0) {
                const int t = r / k;
                atomicOr(&bits[BS * my_e[j] + (t >> 5)], 1u << (t & 31));
            }
        }
        __syncthreads();
        // Prefix sums over the experts (thread = expert) of (rows, 1 if the expert has rows), packed as rows | flag << 16 (at most
        // FFN_LAYER_MAX_ROWS rows and FFN_MAX_E experts in total, so neither field overflows): inside each wavefront with
        // cross-lane moves, then the totals of the lower wavefronts through LDS.  One barrier instead of one per doubling step.
        static_assert(FFN_LAYER_MAX_ROWS < 65536 && FFN_MAX_E < 65536 && FFN_THREADS == FFN_MAX_E && FFN_THREADS == 4 * WAVE,
                      "packed prefix sum: one thread per expert, four wavefronts");
        uint32_t c = 0;
        if (tid < E) {
            unsigned cnt = 0;
#pragma unroll
            for (int w = 0; w < BW; ++w) cnt += __popc(bits[BS * tid + w]);
            c = cnt | ((cnt > 0 ? 1u : 0u) << 16);
        }
        uint32_t incl = c;
#pragma unroll
        for (int d = 1; d < WAVE; d <<= 1) {
            const uint32_t below = __shfl_up(incl, d, WAVE);
            if (lane >= d) incl += below;
        }
        if (lane == WAVE - 1) wave_total[wave] = incl;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < 3; ++w)
            if (w < wave) incl += wave_total[w];
        const uint32_t excl = incl - c;
        if (tid < E) {
            s_off[tid] = (int)(excl & 0xffffu);
            if ((incl >> 16) != (excl >> 16)) s_slot_e[(int)(excl >> 16)] = tid;
            if (tid == E - 1) {
                s_off[E] = (int)(incl & 0xffffu);
                s_nact = (int)(incl >> 16);
            }
        }
        __syncthreads();
        n_act = s_nact;
#pragma unroll
        for (int j = 0; j < FFN_LAYER_MAX_ROWS / FFN_THREADS; ++j) {
            const int r = tid + j * FFN_THREADS;
            if (r >= A) continue;
            const int e = my_e[j];
            int pos = -1;
            if (e >= 0) {
                const int t = r / k;
                int rank = 0;                                       // tokens of this expert below t
#pragma unroll
                for (int w = 0; w < BW; ++w) {
                    const uint32_t b = bits[BS * e + w];
                    rank += w < (t >> 5) ? __popc(b) : (w == (t >> 5) ? __popc(b & ((1u << (t & 31)) - 1u)) : 0);
                }
                pos = s_off[e] + rank;
                s_sorted[pos] = (uint16_t)t;
            }
            if (blockIdx.x == 0) inv_pos_out[r] = pos;         // the combine kernel that follows needs the rows of every pair
        }
        __syncthreads();                                        // s_mem is handed to the weight stream from here on
    }
    if (tiled_min_avg_rows > 0) {
        // Many rows per expert on average: the register-resident token operand below would have to be re-gathered for
        // every item; pipeline both operands instead (weights through an LDS ring, tokens through registers, several items
        // per token pass).  The decision depends on the tables only, so every workgroup of the launch takes the same branch.
        __syncthreads();
        const int total_rows = s_off[E];
        if (n_act > 0 && (long long)total_rows >= (long long)tiled_min_avg_rows * n_act) {
            // More than wide_min_avg_rows rows per expert on average: two token tiles per wavefront (128 rows per pass), so that
            // most experts take one pass over their weights instead of two (bf16 weights; uniform over the launch).
            bool wide = false;
            if constexpr (WB == 2) wide = wide_min_avg_rows > 0 && (long long)total_rows > (long long)wide_min_avg_rows * n_act;
            if constexpr (WB == 2) {
                if (wide) {
                    tiled::ffn_tiled_body<tiled::RING_STAGES, tiled::X_AHEAD, WB, 2>(s_mem, s_slot_e, s_off, lds_tokens ? s_sorted : nullptr, n_act, x,
                                                                                     sorted_token, wg, wu, wd, h, out, ctrl, T, E, H, I, spin_limit,
                                                                                     expert_major_ok, sg, su, sd, skip_publish, fail_mark,
                                                                                     tiled::lds_addr(&s_wait_failed));
                    return;
                }
            }
            tiled::ffn_tiled_body<tiled::RING_STAGES, tiled::X_AHEAD, WB, 1>(s_mem, s_slot_e, s_off, lds_tokens ? s_sorted : nullptr, n_act, x,
                                                                             sorted_token, wg, wu, wd, h, out, ctrl, T, E, H, I, spin_limit,
                                                                             expert_major_ok, sg, su, sd, skip_publish, fail_mark,
                                                                             tiled::lds_addr(&s_wait_failed));
            return;
        }
    }
    const uint32_t total_a = (uint32_t)n_act * TILES_A, total_b = (uint32_t)n_act * TILES_B;   // (at most 256 experts x 128 items)
    // Contiguous shares of floor(total / G) items; the remainder goes, one item each, to the lowest-numbered workgroups.  Those are
    // placed first, one per compute unit, and run ahead of the second workgroup of their unit by about one item over a launch
    // (measured), so the extra item is absorbed instead of extending the phase (with shares that alternate between n and n + 1
    // items every unit ends up with a straggler).
    const int bx = (int)blockIdx.x;
    const uint32_t Gu = (uint32_t)G;
    const int base_a = (int)(total_a / Gu), rem_a = (int)(total_a % Gu), base_b = (int)(total_b / Gu), rem_b = (int)(total_b % Gu);
    const int a_begin = bx * base_a + min(bx, rem_a), a_end = a_begin + base_a + (bx < rem_a ? 1 : 0);
    const int b_begin = bx * base_b + min(bx, rem_b), b_end = b_begin + base_b + (bx < rem_b ? 1 : 0);
    const int n_a = a_end - a_begin, n_mine = n_a + (b_end - b_begin);
    __syncthreads();

    bf16x8_t opr[NT][KSM];                   // token operand (x rows for gate/up items, h rows for down items)
    int cur_key = -1;                        // (phase, slot) the operand registers hold; -1: nothing
    int ready_slot = -1;                     // slot whose h this workgroup has already acquired
    int pend = 0;                            // finished gate/up items of the current slot not yet published
    int held = 0, held_it0 = 0;              // items whose h is still in s_hbuf, and the tile index of the first of them
    bool wait_failed = false;                // a wait of this workgroup gave up: its down items from then on store NaN
    const uint32_t hbuf_base = tiled::lds_addr(s_hbuf);

    // While direct-to-LDS loads of the NEXT item are in flight, every LDS read below is written as explicit
    // instructions: the compiler would otherwise wait for all outstanding direct-to-LDS loads before any LDS read it
    // can see, and so would the fence of __syncthreads().
    const uint32_t tab_e = tiled::lds_addr(s_slot_e), tab_off = tiled::lds_addr(s_off), tab_sorted = tiled::lds_addr(s_sorted);
    struct Item {
        bool is_a;
        int li, a, it, e, r0, m;
    };
    // Token of a row (-1: no such row).  A token that comes from global memory is only usable after every load
    // issued before it, the weights included; that wait stays inside the branch that needs it.
    auto token_of_row = [&](int r0, int m, int row) {
        int tok = -1;
        if (row < m) {
            if (lds_tokens) tok = lds_read_u16(tab_sorted + 2 * (r0 + row));
            else tok = global_read_i32(sorted_token, 4u * (uint32_t)(r0 + row));
        }
        return tok >= T ? -1 : tok;
    };
    // First column (relative to the lane's base column) of the 8 token elements that meet the weights of K-step s.
    // bf16 weights: lane q of K-step s holds weight columns 32 s + 8 q .. + 7.  E4M3 weights: a lane's 16-byte LDS read holds
    // columns 64 j + 16 q .. + 15 of unit j, used as K-steps 2 j (first 8) and 2 j + 1 (last 8); any assignment of columns
    // to K-steps is a valid order of the sum as long as both operands use the same one.
    auto kstep_col = [](int s) { return WB == 2 ? s * 32 : (s >> 1) * 64 + (s & 1) * 8; };
    auto item_at = [&](int step) {
        Item t;
        t.is_a = step < n_a;
        t.li = t.is_a ? a_begin + step : b_begin + (step - n_a);
        const int tiles = t.is_a ? TILES_A : TILES_B;
        t.a = t.li / tiles;
        t.it = t.li - t.a * tiles;
        t.e = __builtin_amdgcn_readfirstlane(tiled::lds_read_i32(tab_e + 4 * t.a));
        const bool ok = t.e >= 0 && t.e < E;
        t.r0 = ok ? __builtin_amdgcn_readfirstlane(tiled::lds_read_i32(tab_off + 4 * t.e)) : 0;
        t.m = ok ? max(__builtin_amdgcn_readfirstlane(tiled::lds_read_i32(tab_off + 4 * t.e + 4)) - t.r0, 0) : 0;
        return t;
    };
    // Stage g of an item's weights into this wavefront's private LDS region: exactly two slab loads.
    auto issue_stage_a = [&](const Item& t, int g) {
        const int ln = opaque(lane);
        char* dst = s_mem + wave * SA::BYTES + g * 2048;
        const size_t ebase = (size_t)t.e * I;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int r = SA::slab_row(half, ln), c = SA::slab_chunk(g, half, ln);
            // MFMA row r = 4*qq + j2: j2 in {0,1} -> gate rows, {2,3} -> up rows of intermediate index 2*qq + (j2 & 1)
            const unsigned char* mat = (r & 2) ? wu : wg;
            const int irow = t.it * 8 + 2 * (r >> 2) + (r & 1);
            if (SA::C % 8 == 0 || c < SA::C) slab_load(mat + ((ebase + irow) * H + wave * KSLICE_A) * WB + c * 16, dst + half * 1024);
        }
    };
    auto issue_stage_b = [&](const Item& t, int g) {
        const int ln = opaque(lane);
        const int rb = g / SB::S, st = g % SB::S;
        char* dst = s_mem + wave * (RB * SB::BYTES) + g * 2048;
        const size_t ebase = (size_t)t.e * H + (size_t)t.it * 16 * RB + rb * 16;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int r = SB::slab_row(half, ln), c = SB::slab_chunk(st, half, ln);
            if (SB::C % 8 == 0 || c < SB::C) slab_load(wd + ((ebase + r) * I + wave * KSLICE_B) * WB + c * 16, dst + half * 1024);
        }
    };
    // All stages of an item at once (nothing of it has been requested yet).
    auto issue_loads = [&](const Item& t) {
        if (t.m <= 0) return;
        if (t.is_a) {
#pragma unroll
            for (int g = 0; g < SA::S; ++g) issue_stage_a(t, g);
        } else {
#pragma unroll
            for (int g = 0; g < RB * SB::S; ++g) issue_stage_b(t, g);
        }
    };
    const uint32_t red_base = tiled::lds_addr(s_mem + LDS_BYTES - RED_A);     // red_a; red_b ends at the same address
    const uint32_t redb_base = tiled::lds_addr(s_mem + LDS_BYTES - RED_B);

    // h as a buffer (raw, no swizzle, 32-bit data format), for its device-scope gather in the down phase
    const __amdgpu_buffer_rsrc_t h_rsrc = __builtin_amdgcn_make_buffer_rsrc(h, 0, (int)min((size_t)A * I * 2, (size_t)0x7fffffff), 0x00020000);

    Item cur{};
    if (n_mine > 0) cur = item_at(0);
    bool ahead = false;                      // the current item's weights were requested during the previous item
    for (int step = 0; step < n_mine; ++step) {   // this workgroup's gate/up items, then its down items
        const bool has_next = step + 1 < n_mine;
        const Item nxt = item_at(has_next ? step + 1 : step);
        // First down item of an expert with nothing requested yet (the publication of this workgroup's own h has just drained
        // its loads): thread 0 looks at the expert's counter BEFORE the item's weights are requested.  Loads return in
        // order, so behind the weights the first look would take as long as the weights do; on its own it is one round trip,
        // and in most launches it already finds the expert complete.
        bool seen_complete = false;
        if (!cur.is_a && cur.a != ready_slot && !ahead && tid == 0)
            seen_complete = __hip_atomic_load(&ctrl->done[cur.a][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= TILES_A;
        if (!ahead) issue_loads(cur);
        ahead = false;
        const bool is_a = cur.is_a;
        const int li = cur.li, a = cur.a, it = cur.it, r0 = cur.r0, m = cur.m;
        const int key = (is_a ? 0 : 0x10000) | a;
        const int ln = opaque(lane);
        const int n = ln & 15, q = ln >> 4;
        const int chunks = (m + 16 * NT - 1) / (16 * NT);
        if (is_a) {
            // =============================================================== gate/up item
            const uint32_t region = tiled::lds_addr(s_mem + wave * SA::BYTES);
            // Items of one slot are published together after the last of them; that one waits for its h stores.
            const bool publish_now = step + 1 >= n_a || (li + 1) / TILES_A != a;
            float sc_g[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f}, sc_u[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
            if constexpr (WB == 1) {     // scales of this item's 8 gate rows and 8 up rows (requested now, needed in the epilogue)
                if (m > 0) {
                    load_uniform(sg + (size_t)cur.e * I + it * 8, sc_g);
                    load_uniform(su + (size_t)cur.e * I + it * 8, sc_u);
                }
            }
            for (int ch = 0; ch < chunks; ++ch) {
                const int row_base = ch * 16 * NT;
                const bool last_chunk = ch + 1 == chunks;
                if (key != cur_key || chunks > 1) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const int tok = token_of_row(r0, m, row_base + nt * 16 + n);
                        const uint16_t* xp = x + (size_t)(tok < 0 ? 0 : tok) * H + wave * KSLICE_A + q * (16 / WB);
                        if (tok >= 0) {
#pragma unroll
                            for (int s = 0; s < KSA; ++s) opr[nt][s] = *reinterpret_cast<const bf16x8_t*>(xp + kstep_col(s));
                        } else {
#pragma unroll
                            for (int s = 0; s < KSA; ++s) opr[nt][s] = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                        }
                    }
                    settle<KSA>(opr);
                    cur_key = chunks > 1 ? -1 : key;
                }
                const bool two = m - row_base > 16;
                f32x4_t acc[1][NT] = {{{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}};
                // Stage by stage: wait for the stage, read it, and (in the item's last pass, unless a publication follows)
                // request the same stage of the next item, so this wavefront's loads never stop.  One branch per item.
                const bool prefetch = last_chunk && has_next && !publish_now && nxt.m > 0;
                auto next_stage = [&](int g) { issue_stage_a(nxt, g); };
                if (prefetch) {
                    if (two) stream_item<SA, UA, 1, true, true, WB, KSM>(region, n, q, opr, acc, next_stage);
                    else stream_item<SA, UA, 1, true, false, WB, KSM>(region, n, q, opr, acc, next_stage);
                    ahead = true;
                } else {
                    if (two) stream_item<SA, UA, 1, false, true, WB, KSM>(region, n, q, opr, acc, next_stage);
                    else stream_item<SA, UA, 1, false, false, WB, KSM>(region, n, q, opr, acc, next_stage);
                }
                settle_accumulators(acc[0]);
                const uint32_t red_mine = red_base + (uint32_t)(wave * NT * WAVE + ln) * 16;
                lds_write_f4_at<0>(red_mine, acc[0][0]);
                lds_write_f4_at<WAVE * 16>(red_mine, acc[0][1]);
                lds_barrier();
                if (chunks == 1 && held == 0) held_it0 = it;
                if (wave < NT && (wave == 0 || two)) {        // wavefront nt finishes token tile nt
                    f32x4_t v = lds_sum4<NT * WAVE * 16>(red_base + (uint32_t)(wave * WAVE + ln) * 16);
                    const int row = row_base + wave * 16 + n;
                    // lane holds (g_a, g_b, u_a, u_b) of intermediate indices it*8 + 2*q, +1 for token row `row`
                    if constexpr (WB == 1) {
                        // (the lane's group index is made opaque here so that the selections are not moved in front of the
                        // stream, where their results would occupy registers the stream needs)
                        const int qs = opaque(q);
                        const float g0 = qs == 0 ? sc_g[0] : qs == 1 ? sc_g[2] : qs == 2 ? sc_g[4] : sc_g[6];
                        const float g1 = qs == 0 ? sc_g[1] : qs == 1 ? sc_g[3] : qs == 2 ? sc_g[5] : sc_g[7];
                        const float u0 = qs == 0 ? sc_u[0] : qs == 1 ? sc_u[2] : qs == 2 ? sc_u[4] : sc_u[6];
                        const float u1 = qs == 0 ? sc_u[1] : qs == 1 ? sc_u[3] : qs == 2 ? sc_u[5] : sc_u[7];
                        v[0] *= g0; v[1] *= g1; v[2] *= u0; v[3] *= u1;
                    }
                    const float h0 = silu_f32(v[0]) * v[2];
                    const float h1 = silu_f32(v[1]) * v[3];
                    const uint32_t packed = f32_to_bf16_bits(h0) | (f32_to_bf16_bits(h1) << 16);
                    uint32_t* hrow = reinterpret_cast<uint32_t*>(h + (size_t)(r0 + (row < m ? row : 0)) * I + 2 * q);
                    if (chunks > 1) {
                        if (row < m) store_coherent(hrow + it * 4, packed);
                    } else {
                        // A store between the weight loads holds up this wavefront's load pipeline until it is acknowledged
                        // (loads and stores complete in order), and an item's h is only needed once the whole slot run is
                        // published: keep it in LDS (every lane re-reads only what it wrote) and store the run in one go.
                        lds_write_u32(hbuf_base + ((held * NT + wave) * WAVE + ln) * 4, packed);
                        if (publish_now || held + 1 == H_BUF_ITEMS) {
                            for (int j = 0; j <= held; ++j) {
                                const uint32_t pv = lds_read_u32(hbuf_base + ((j * NT + wave) * WAVE + ln) * 4);
                                if (row < m) store_coherent(hrow + (held_it0 + j) * 4, pv);
                            }
                        }
                    }
                }
                if (chunks == 1) held = (publish_now || held + 1 == H_BUF_ITEMS) ? 0 : held + 1;
                // vmcnt counts stores too.  Before a publication every h store of this workgroup must have been
                // acknowledged; nothing else is in flight then (the next item's weights are not requested before a
                // publication), so this waits for exactly those stores.
                if (publish_now && last_chunk) wait_all_loads();
                lds_barrier();            // partial-sum buffer is free; with the wait above, h of this workgroup is complete
            }
            // publish finished gate/up items, once per run of items of one slot.  The h stores are device-coherent
            // write-through stores and every wavefront has waited for its own before the barrier.
            ++pend;
            if (publish_now) {
                if (tid == 0 && !skip_publish) __hip_atomic_fetch_add(&ctrl->done[a][0], pend, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                pend = 0;
            }
        } else {
            // =============================================================== down item
            const uint32_t region = tiled::lds_addr(s_mem + wave * (RB * SB::BYTES));
            float sc_d[16] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
            if constexpr (WB == 1) {     // scales of the 16 output rows this wavefront finishes (pair = wave: sub-tile wave / NT)
                if (m > 0 && wave < RB * NT) load_uniform(sd + (size_t)cur.e * H + it * 16 * RB + (wave / NT) * 16, sc_d);
            }
            if (a != ready_slot) {       // wait until every gate/up item of this expert has published h
                if (tid == 0 && !seen_complete) {
                    int spins = 0;
                    while (__hip_atomic_load(&ctrl->done[a][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < TILES_A) {
                        __builtin_amdgcn_s_sleep(8);      // ~0.2 us between polls; the counters sit in different memory channels
                        // Giving up: only when the producers cannot run (another launch holds the compute units they need) or
                        // the control block was not cleared.  The workspace gets its failure mark, and this workgroup stores
                        // NaN instead of products of an incomplete h from here on.
                        if (++spins > spin_limit) {
                            // (the mark is put together behind an opaque value, inside this branch: as a plain constant the
                            // compiler loads it into registers in front of the item loop and keeps it there)
                            __hip_atomic_store(fail_mark, WS_FAIL_MARK + (unsigned long long)opaque(0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            lds_write_u32(tiled::lds_addr(&s_wait_failed), 1u);
                            break;
                        }
                    }
                }
                lds_barrier();
                ready_slot = a;
                wait_failed = wait_failed || __builtin_amdgcn_readfirstlane((int)lds_read_u32(tiled::lds_addr(&s_wait_failed))) != 0;
            }
            for (int ch = 0; ch < chunks; ++ch) {
                const int row_base = ch * 16 * NT;
                const bool last_chunk = ch + 1 == chunks;
                if (key != cur_key || chunks > 1) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const int row = row_base + nt * 16 + n;
                        const bool valid = token_of_row(r0, m, row) >= 0;
                        const uint32_t hoff = (uint32_t)(((valid ? r0 + row : 0) * I + wave * KSLICE_B + q * (16 / WB)) * 2);
                        if (valid) {
#pragma unroll
                            for (int s = 0; s < KSB; ++s) opr[nt][s] = load_coherent_16(h_rsrc, hoff + 2u * (uint32_t)kstep_col(s));
                        } else {
#pragma unroll
                            for (int s = 0; s < KSB; ++s) opr[nt][s] = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                        }
                    }
                    settle<KSB>(opr);
                    cur_key = chunks > 1 ? -1 : key;
                }
                const bool two = m - row_base > 16;
                f32x4_t acc[RB][NT];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[rb][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                const bool prefetch = last_chunk && has_next && nxt.m > 0;     // the next item is a down item too
                auto next_stage = [&](int g) { issue_stage_b(nxt, g); };
                if (prefetch) {
                    if (two) stream_item<SB, UB, RB, true, true, WB, KSM>(region, n, q, opr, acc, next_stage);
                    else stream_item<SB, UB, RB, true, false, WB, KSM>(region, n, q, opr, acc, next_stage);
                    ahead = true;
                } else {
                    if (two) stream_item<SB, UB, RB, false, true, WB, KSM>(region, n, q, opr, acc, next_stage);
                    else stream_item<SB, UB, RB, false, false, WB, KSM>(region, n, q, opr, acc, next_stage);
                }
                settle_accumulators(reinterpret_cast<f32x4_t(&)[RB * NT]>(acc));
                const uint32_t redb_mine = redb_base + (uint32_t)(wave * RB * NT * WAVE + ln) * 16;
                static_assert(NT == 2 && (RB == 1 || RB == 2), "partial sums are written out one by one");
                lds_write_f4_at<0>(redb_mine, acc[0][0]);
                lds_write_f4_at<WAVE * 16>(redb_mine, acc[0][1]);
                if constexpr (RB == 2) {
                    lds_write_f4_at<2 * WAVE * 16>(redb_mine, acc[1][0]);
                    lds_write_f4_at<3 * WAVE * 16>(redb_mine, acc[1][1]);
                }
                lds_barrier();
                // (rb, nt) pairs are finished by wavefronts round-robin, partial sums added in wavefront order
                for (int pair = wave; pair < RB * NT; pair += FFN_WAVES) {
                    const int rb = pair / NT, nt = pair % NT;
                    const int row = row_base + nt * 16 + n;
                    if (row < m) {
                        f32x4_t v = lds_sum4<RB * NT * WAVE * 16>(redb_base + (uint32_t)((rb * NT + nt) * WAVE + ln) * 16);
                        // lane holds output rows it*16*RB + rb*16 + 4*q + (0..3) of token row `row`
                        if constexpr (WB == 1) {
                            const int qs = opaque(q);       // as in the gate/up epilogue
                            v[0] *= pick4(sc_d, qs, 0); v[1] *= pick4(sc_d, qs, 1); v[2] *= pick4(sc_d, qs, 2); v[3] *= pick4(sc_d, qs, 3);
                        }
                        if (wait_failed) v = f32x4_t{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), __builtin_nanf("")};
                        *reinterpret_cast<f32x4_t*>(out + (size_t)(r0 + row) * H + it * 16 * RB + rb * 16 + 4 * q) = v;
                    }
                }
                lds_barrier();
            }
        }
        cur = nxt;
    }
}


// The kernel's waits need every workgroup of the grid to be resident at once, so the grid is what the runtime
// says fits: (workgroups per compute unit for this instantiation) x (compute units), never more.
template <int KSA, int KSB, int WB>
hipError_t launch_ffn_fused(const FfnArgs& p) {
    constexpr int RB = KSB <= 6 ? 2 : 1;      // two sub-tiles per down item while the partial sums fit the register budget
    // Workgroups of this instantiation that fit one compute unit of the current device, asked once per device.
    static std::atomic<int> per_cu_of[FFN_MAX_DEVICES];
    if (p.device < 0 || p.device >= FFN_MAX_DEVICES) return hipErrorInvalidDevice;
    int per_cu = per_cu_of[p.device].load(std::memory_order_relaxed);
    if (per_cu == 0) {
        hipError_t err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, ffn_fused_kernel<KSA, KSB, RB, WB>, FFN_THREADS, 0);
        if (err != hipSuccess) return err;
        if (per_cu < 1) return hipErrorLaunchOutOfResources;
        per_cu_of[p.device].store(per_cu, std::memory_order_relaxed);      // (two first callers store the same value)
    }
    const int resident = per_cu * p.n_cu;
    const int grid = p.grid_override > 0 && p.grid_override < resident ? p.grid_override : resident;
    if (p.cooperative) {
        // Measurement aid: the same launch through the runtime's cooperative path, which refuses a grid that cannot be resident
        // at once.  (It does not reserve the device either: workgroups of a kernel from another stream can still hold compute units.)
        const uint16_t* x = p.x; const int32_t *offsets = p.offsets, *sorted_token = p.sorted_token, *active = p.active, *n_active = p.n_active;
        const unsigned char *wg = (const unsigned char*)p.wg, *wu = (const unsigned char*)p.wu, *wd = (const unsigned char*)p.wd;
        uint16_t* h = p.h; float* out = p.out; FfnCtrl* ctrl = p.ctrl; int T = p.T, k = p.k, E = p.E, spin_limit = p.spin_limit;
        int skip_publish = p.skip_publish; unsigned long long* fail_mark = p.fail_mark;
        int tiled_rows = p.tiled_min_avg_rows, expert_major = p.expert_major, wide_rows = p.wide_min_avg_rows;
        const int32_t* topk_idx = p.topk_idx; int32_t* inv_pos_out = p.inv_pos_out; const float *sg = p.sg, *su = p.su, *sd = p.sd;
        void* args[] = {&x, &offsets, &sorted_token, &active, &n_active, &wg, &wu, &wd, &h, &out, &ctrl, &T, &k, &E, &spin_limit, &skip_publish,
                        &fail_mark, &tiled_rows, &expert_major, &wide_rows, &topk_idx, &inv_pos_out, &sg, &su, &sd};
        return hipLaunchCooperativeKernel(reinterpret_cast<const void*>(&ffn_fused_kernel<KSA, KSB, RB, WB>), dim3(grid), dim3(FFN_THREADS), args, 0,
                                          p.stream);
    }
    hipLaunchKernelGGL((ffn_fused_kernel<KSA, KSB, RB, WB>), dim3(grid), dim3(FFN_THREADS), 0, p.stream, p.x, p.offsets, p.sorted_token,
                       p.active, p.n_active, (const unsigned char*)p.wg, (const unsigned char*)p.wu, (const unsigned char*)p.wd, p.h, p.out,
                       p.ctrl, p.T, p.k, p.E, p.spin_limit, p.skip_publish, p.fail_mark, p.tiled_min_avg_rows, p.expert_major,
                       p.wide_min_avg_rows, p.topk_idx, p.inv_pos_out, p.sg, p.su, p.sd);
    return hipGetLastError();
}

#ifndef FFN_KSA_THIS_FILE
#error "compile with -DFFN_KSA_THIS_FILE=<hidden/128> (and -DFFN_W8_THIS_FILE for the 8-bit weight kernels of that hidden size)"
#endif
#ifndef FFN_W8_THIS_FILE
template <int KSA>
hipError_t launch_ffn_fused_ksa(const FfnArgs& p, int ksb) {
    switch (ksb) {
        case 1: return launch_ffn_fused<KSA, 1, 2>(p);
        case 2: return launch_ffn_fused<KSA, 2, 2>(p);
        case 3: return launch_ffn_fused<KSA, 3, 2>(p);
        case 4: return launch_ffn_fused<KSA, 4, 2>(p);
        case 5: return launch_ffn_fused<KSA, 5, 2>(p);
        case 6: return launch_ffn_fused<KSA, 6, 2>(p);
        case 7: return launch_ffn_fused<KSA, 7, 2>(p);
        case 8: return launch_ffn_fused<KSA, 8, 2>(p);
        default: return hipErrorInvalidValue;
    }
}
template hipError_t launch_ffn_fused_ksa<FFN_KSA_THIS_FILE>(const FfnArgs& p, int ksb);
#else
template <int KSA>
hipError_t launch_ffn_fused_w8_ksa(const FfnArgs& p, int ksb) {
    switch (ksb) {
        case 2: return launch_ffn_fused<KSA, 2, 1>(p);
        case 4: return launch_ffn_fused<KSA, 4, 1>(p);
        case 6: return launch_ffn_fused<KSA, 6, 1>(p);
        case 8: return launch_ffn_fused<KSA, 8, 1>(p);
        default: return hipErrorInvalidValue;
    }
}
template hipError_t launch_ffn_fused_w8_ksa<FFN_KSA_THIS_FILE>(const FfnArgs& p, int ksb);
#endif

}  // namespace team
