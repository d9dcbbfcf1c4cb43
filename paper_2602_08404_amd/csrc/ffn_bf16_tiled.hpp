// Grouped SwiGLU expert FFN, bf16, gfx950 MFMA: the variant for calls with many tokens per expert
// (speculative branches and batched blocks: tens to hundreds of rows per activated expert).  Included by
// ffn_bf16_kernel.hip; the persistent kernel switches to this body when the call averages many rows per expert.
//
// Same work decomposition, same per-expert h hand-over and same deterministic results as ffn_bf16_kernel.hip,
// but the token operand is not kept in registers across items: with more than 32 rows per expert it would have to
// be re-gathered for every item, with the weight stream standing still meanwhile.  Here both operands are
// software-pipelined:
//
//   item     gate/up: (expert, 16 intermediate indices) = 16 rows of w_gate + 16 rows of w_up, all H columns
//            down   : (expert, 32 output rows of w_down), all I columns
//   segment  up to TILES consecutive items of a workgroup's share that belong to one expert, worked on together: the token
//            rows are fetched once per segment, not once per item (that traffic, from L2, is otherwise twice the weights')
//   pass     64 token rows of the expert (4 token tiles, one per wavefront), or 128 in the instance with two token tiles per
//            wavefront (calls with many rows per expert); experts with more rows take several passes over the same weight
//            rows (served by the caches after the first pass)
//   stage    64 reduction columns of a segment: 32 weight rows x 128 B = 4 KB per item
// Weights: a ring of RING_STAGES stages in LDS; every wavefront issues one 1 KB direct-to-LDS load per item and stage (8
// weight rows), RING_STAGES-1 stages (up to 48 KB per workgroup) ahead of the stage being multiplied, also across segment
// boundaries.  Tokens: a wavefront owns one or two token tiles and loads its own MFMA operands of a stage (16 bytes per lane,
// tile and K-step, straight from the L2-resident x or h rows) into registers, X_AHEAD stages ahead.  It multiplies them with
// both 16-row weight tiles of every item of the segment: no reduction across wavefronts, sums in a fixed order.
// Shares: the phase's item list is cut contiguously over the workgroups, or, where a share is a single segment and such a
// cut would cross expert boundaries, the workgroups are dealt out to the experts (see ffn_tiled_body).
//
// LDS stage layout: rows of 128 B (8 chunks of 16 B); chunk c of row r is stored at chunk c ^ ((r >> 1) & 7),
// which spreads the 16 rows of an MFMA operand read over all 16 bank groups.  The swizzle is applied to the
// global address a lane fetches, because a direct-to-LDS load writes the lanes of a wavefront contiguously.
//
// The loop issues all of its loads as explicit instructions, counts them, and waits with s_waitcnt vmcnt(N), N = the
// loads issued after the ones a stage needs (loads complete in issue order); it reads LDS with explicit instructions too.
// The compiler cannot do this: it turns every wait for an ordinary load into a wait for all loads while a direct-to-LDS
// load it knows of is in flight, treats such loads as aliasing every LDS read, and gives up counting across a loop's back edge.
#pragma once
#include <type_traits>
#include <utility>

#include "ffn_bf16.hpp"

namespace team {

namespace tiled {

constexpr int KC = 64;                 // reduction columns per stage with bf16 weights (128 bytes of a weight row; 128 columns of E4M3 codes)
constexpr int MT = 64;                 // token rows per pass
constexpr int W_ROWS = 32;             // weight rows per item
constexpr int ROW_BYTES = KC * 2;      // 128
constexpr int W_BYTES = W_ROWS * ROW_BYTES;
constexpr int TILES = 4;               // items of a segment (measured: 2 and 3 are slower, 6 is no faster)
constexpr int STAGE_BYTES = TILES * W_BYTES;   // only the weights pass through LDS

typedef __attribute__((address_space(3))) void* lptr_t;

// Streaming direct-to-LDS load (non-temporal: weights are read once and must not displace the small reused data from L2).
// M0 holds the LDS address; one idle cycle between writing M0 and the load that reads it; M0 is restored, as the compiler
// does not expect it to change.
__device__ __forceinline__ void slab_load_stream_explicit(const void* gsrc, uint32_t lds_addr_uniform) {
    uint32_t saved_m0;
    lds_addr_uniform = __builtin_amdgcn_readfirstlane(lds_addr_uniform);   // (a scalar register also where the compiler cannot prove uniformity)
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, off nt\n\t"
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0"
        : "=&s"(saved_m0)
        : "v"(gsrc), "s"(lds_addr_uniform)
        : "memory");
}
// 16 bytes per lane into registers, asynchronously: `dst` is only valid after a wait for at most N outstanding loads with
// N = the loads issued since.  Until then the compiler believes the value is there already, so nothing may touch it: its only
// use is as an operand of the matrix instructions, which depend on the LDS reads that follow that wait (explicit statements
// keep their order).  A copy of such a register in the generated code would read it too early;
// tests/test_generated_code.py looks for that.
// DEVICE: device-scope load (h written by other workgroups of this launch).
template <bool DEVICE, int BYTE_OFFSET>
__device__ __forceinline__ void request_tokens(bf16x8_t& dst, const uint16_t* p) {
    if constexpr (DEVICE) asm volatile("global_load_dwordx4 %0, %1, off offset:%2 sc1" : "=v"(dst) : "v"(p), "n"(BYTE_OFFSET) : "memory");
    else asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(dst) : "v"(p), "n"(BYTE_OFFSET) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_outstanding() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wg_barrier() {
    asm volatile("s_barrier" ::: "memory");
}
__device__ __forceinline__ void store_coherent(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(lptr_t)p;
}
__device__ __forceinline__ int lds_read_u16(uint32_t a) {
    int v;
    asm volatile("ds_read_u16 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a) : "memory");
    return v;
}
// One 32-bit LDS read at byte address a.
__device__ __forceinline__ int lds_read_i32(uint32_t a) {
    int v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a) : "memory");
    return v;
}

// f(integral_constant<int, 0>), f(<1>), ... in turn, until one returns false.
template <class F, int... U>
__device__ __forceinline__ void for_each_slot(F&& f, std::integer_sequence<int, U...>) {
    (void)(f(std::integral_constant<int, U>{}) && ...);
}

// Row scales of 8-bit weights: 16 consecutive floats at a wave-uniform address, read through the scalar cache (the tables are
// never written by the kernel).  That path has its own counter, so the loads neither join the queue the loop counts nor make the
// compiler wait for the weight stream.
typedef const __attribute__((address_space(4))) float* const_f32_ptr;
__device__ __forceinline__ void load_scales(const float* base_uniform, float (&v)[16]) {
    const_f32_ptr p = (const_f32_ptr)base_uniform;
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = p[i];
}
// v[first + stride * q] for a lane-dependent q in 0..3
__device__ __forceinline__ float pick_q(const float (&v)[16], int first, int stride, int q) {
    const float lo = q == 0 ? v[first] : v[first + stride], hi = q == 2 ? v[first + 2 * stride] : v[first + 3 * stride];
    return q < 2 ? lo : hi;
}

struct Seg {                   // one (segment, pass) of a workgroup's share
    int li;                    // first item of the segment in the expert-major list of the phase
    int nw;                    // items in the segment (1..TILES)
    int a, it, e, r0, m, pass;
    bool valid;
};

constexpr int RING_STAGES = 4;
constexpr int RING_BYTES = RING_STAGES * STAGE_BYTES;
constexpr int X_AHEAD = 4;
constexpr int MAX_COUNTED = 24;        // largest wait count used: (RING_STAGES - 1) stages of TILES + 2 loads, rounded up

// Waits until at most n vector-memory operations of this wavefront are outstanding (n uniform; above MAX_COUNTED: until none).
// The count is an immediate of the wait instruction, so a run-time count selects one of MAX_COUNTED + 1 instructions: a jump into
// a table of (wait, branch to the end) pairs of 8 bytes each.  (Written as a switch, the compiler emitted a chain of some 60
// scalar instructions and taken branches per call, a fifth of the time of a stage.)
__device__ __forceinline__ void wait_outstanding_rt(int n) {
    static_assert(MAX_COUNTED == 24, "the table below has entries 0 .. 24");
    n = __builtin_amdgcn_readfirstlane(n);
    const int entry = (unsigned)n > (unsigned)MAX_COUNTED ? 0 : n;
    int offset;
    asm volatile(
        "s_getpc_b64 vcc\n"
        ".Lteam_wait_pc%=:\n\t"
        "s_lshl_b32 %0, %1, 3\n\t"
        "s_add_u32 %0, %0, .Lteam_wait_table%=-.Lteam_wait_pc%=\n\t"
        "s_add_u32 vcc_lo, vcc_lo, %0\n\t"
        "s_addc_u32 vcc_hi, vcc_hi, 0\n\t"
        "s_setpc_b64 vcc\n"
        ".Lteam_wait_table%=:\n\t"
        "s_waitcnt vmcnt(0)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(1)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(2)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(3)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(4)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(5)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(6)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(7)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(8)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(9)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(10)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(11)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(12)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(13)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(14)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(15)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(16)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(17)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(18)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(19)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(20)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(21)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(22)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(23)\n\ts_branch .Lteam_wait_end%=\n\t"
        "s_waitcnt vmcnt(24)\n"
        ".Lteam_wait_end%=:"
        : "=&s"(offset)
        : "s"(entry)
        : "vcc", "scc", "memory");
}
// The four weight operands of an item's stage (two 16-row tiles x two K-steps) at byte addresses a0..a3.
__device__ __forceinline__ void lds_read4(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, bf16x8_t& w0, bf16x8_t& w1, bf16x8_t& w2,
                                          bf16x8_t& w3) {
    asm volatile(
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %5\n\t"
        "ds_read_b128 %2, %6\n\t"
        "ds_read_b128 %3, %7\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(w0), "=&v"(w1), "=&v"(w2), "=&v"(w3)
        : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
        : "memory");
}

// Body of the streaming variant; runs inside the persistent FFN kernel (all workgroups take it or none does).
// s_ring: RING_BYTES of LDS, 1 KB aligned; s_slot_e / s_off: the kernel's tables (active list, clipped offsets); s_sorted: its
// LDS copy of the grouped token list (0xffff: no token), or null when the list did not fit.
// WB = bytes per weight: 2 (bf16) or 1 (E4M3 codes with one float scale per matrix row: sg, su [E,I], sd [E,H]).  With codes a
// stage holds 128 reduction columns (the same 128 bytes per weight row), a 16-byte LDS read carries the operands of two K-steps
// (widened to bf16 in registers), a lane's token operand of a stage is 4 x 16 bytes, and the row scales multiply the sums in
// the epilogues.
template <int DW, int DX, int WB, int NT>
__device__ __forceinline__ void ffn_tiled_body(char* s_ring, const int32_t* s_slot_e, const int32_t* s_off, const uint16_t* s_sorted, int n_act,
                                               const uint16_t* __restrict__ x, const int32_t* __restrict__ sorted_token,
                                               const unsigned char* __restrict__ wg, const unsigned char* __restrict__ wu,
                                               const unsigned char* __restrict__ wd, uint16_t* __restrict__ h, float* __restrict__ out,
                                               FfnCtrl* __restrict__ ctrl, int T, int E, int H, int I, int spin_limit, int expert_major_ok,
                                               const float* __restrict__ sg, const float* __restrict__ su, const float* __restrict__ sd,
                                               int skip_publish, unsigned long long* __restrict__ fail_mark, uint32_t fail_addr) {
    asm volatile("; team_tiled_body_begin" ::: "memory");   // (marks for the checks of the generated code: a kernel holds two instances)
    constexpr int KCOL = ROW_BYTES / WB;          // reduction columns per stage
    // NT token tiles per wavefront: a pass covers MTT = NT x 64 rows of the expert (tile j of wavefront w: rows 64 j + 16 w ..).
    // With two tiles an expert of 65 to 128 rows takes one pass instead of two, at about 1.3 times the cost of a stage.
    constexpr int MTT = MT * NT;
    static_assert(NT == 1 || (NT == 2 && WB == 2), "two token tiles per wavefront: bf16 weights only (registers)");
    constexpr int XL = 2 * (2 / WB);              // 16-byte token loads per lane and stage = K-steps per stage
    // The tokens of a stage are requested before its weights (DX >= DW), so "everything up to the weights of the stage" is
    // what a stage waits for.
    static_assert(DX >= DW && (DW - 1) * (TILES + NT * XL) <= MAX_COUNTED, "token requests lead the weight requests; wait counts fit");
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, q = lane >> 4;
    const int G = gridDim.x;
    const int tiles_a = I / 16, tiles_b = H / W_ROWS;
    bool wait_failed = false;             // a wait of this workgroup gave up: the down results it stores from then on are NaN

    // ---- lane constants
    // weight loads: lane fetches row (l / 8) of an 8-row slab, stored chunk (l % 8)
    const int ld_row = lane >> 3, ld_cs = lane & 7;
    // weight reads: MFMA operand row n of tile rt, chunk 4*ks + q, un-swizzled on the fly
    const uint32_t ring0 = lds_addr(s_ring);
    const uint32_t tab_e = lds_addr(s_slot_e), tab_off = lds_addr(s_off);
    uint32_t rd_w[2][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const int r = 16 * rt + n;
            rd_w[rt][ks] = r * ROW_BYTES + (((4 * ks + q) ^ ((r >> 1) & 7)) << 4);
        }

    // (decided once for both phases, from the gate/up list, so that a workgroup's down items belong to the expert whose
    // gate/up items it and its neighbours have just finished)
    bool expert_major = false;
    if (expert_major_ok && n_act > 0 && n_act <= G) {
        const uint32_t total_a = (uint32_t)n_act * (uint32_t)tiles_a;
        const int need = (int)((total_a + (uint32_t)G - 1u) / (uint32_t)G);
        expert_major = need <= TILES && (tiles_a % need != 0 || total_a % (uint32_t)G != 0u);
    }

    for (int phase = 0; phase < 2; ++phase) {
        const int tiles = phase == 0 ? tiles_a : tiles_b;
        const int nks = (phase == 0 ? H : I) / KCOL;               // stages per (segment, pass)
        const uint32_t total = (uint32_t)n_act * (uint32_t)tiles;   // (at most FFN_MAX_E experts x 128 items: 32-bit arithmetic)
        // contiguous shares; the remainder goes to the lowest-numbered workgroups (see the register-operand body)
        const int share = (int)(total / (uint32_t)G), extra = (int)(total % (uint32_t)G), bx = (int)blockIdx.x;
        int li_begin = bx * share + min(bx, extra), li_end = li_begin + share + (bx < extra ? 1 : 0);
        // A share that crosses from one expert into the next costs its workgroup a second, short segment: as many stages again
        // for a fraction of the bytes, and those stages are bound by latency, not by bytes (a segment of one item keeps 12 KB in
        // flight).  That workgroup then finishes late, and with it both experts it has a part of.  Where a share is a single
        // segment, the workgroups are therefore dealt out to the experts instead (G / n_act each, one more for the first
        // G % n_act), and an expert's items are cut evenly among its workgroups: shares differ by one item, none crosses.
        if (expert_major && (phase == 0 || expert_major_ok == 1)) {
            const int q_wg = G / n_act, r_wg = G % n_act, big = r_wg * (q_wg + 1);
            int a, j, wgs;
            if (bx < big) {
                a = bx / (q_wg + 1); j = bx - a * (q_wg + 1); wgs = q_wg + 1;
            } else {
                a = r_wg + (bx - big) / q_wg; j = (bx - big) - (a - r_wg) * q_wg; wgs = q_wg;
            }
            li_begin = a * tiles + j * tiles / wgs;
            li_end = a * tiles + (j + 1) * tiles / wgs;
        }
        const size_t tile_stride = (phase == 0 ? (size_t)16 * H : (size_t)W_ROWS * I) * WB;   // bytes between the weight rows of adjacent items

        auto load_seg = [&](Seg& s) {                               // segment that starts at item s.li; skips experts without rows
            s.valid = false;
            while (s.li < li_end) {
                s.a = s.li / tiles;
                s.it = s.li - s.a * tiles;
                s.nw = min(min(TILES, li_end - s.li), tiles - s.it);
                s.e = __builtin_amdgcn_readfirstlane(lds_read_i32(tab_e + 4 * s.a));
                const bool ok = s.e >= 0 && s.e < E;
                s.r0 = ok ? __builtin_amdgcn_readfirstlane(lds_read_i32(tab_off + 4 * s.e)) : 0;
                s.m = ok ? max(__builtin_amdgcn_readfirstlane(lds_read_i32(tab_off + 4 * s.e + 4)) - s.r0, 0) : 0;
                s.pass = 0;
                if (s.m > 0) {
                    s.valid = true;
                    return;
                }
                s.li += s.nw;
            }
        };
        auto next_seg = [&](Seg& s) {
            if ((s.pass + 1) * MTT < s.m) {
                ++s.pass;
            } else {
                s.li += s.nw;
                load_seg(s);
            }
        };

        int issued = 0;                   // vector-memory loads this wavefront has issued in this phase

        // ---------------------------------------------------------------- weight producer: one 1 KB slab per item and stage
        Seg pw;
        pw.li = li_begin;
        load_seg(pw);
        int pw_ks = 0, w_issued = 0;
        const unsigned char* src_w = nullptr;  // rows 8*wave .. 8*wave+7 of the segment's first item
        int mark_w[DW];                   // `issued` right after the weight requests of the stage in that ring slot
        auto pw_enter = [&]() {
            const int r = 8 * wave + ld_row;                       // weight row of the item this lane fetches
            const int c = ld_cs ^ ((r >> 1) & 7);                  // global chunk that belongs at the stored chunk
            if (phase == 0) {
                const int i = r & 15;
                const int iidx = pw.it * 16 + (r >> 4) * 8 + 2 * (i >> 2) + (i & 1);   // rows 4q+{0,1}: gate, 4q+{2,3}: up
                const unsigned char* mat = (i & 2) ? wu : wg;
                src_w = mat + ((size_t)pw.e * I + iidx) * H * WB + c * 16;
            } else {
                src_w = wd + ((size_t)pw.e * H + (size_t)pw.it * W_ROWS + r) * I * WB + c * 16;
            }
        };
        auto produce_w = [&](int& slot_mark) {                      // (only while pw.valid)
            const uint32_t dst = ring0 + (w_issued % DW) * STAGE_BYTES + wave * 8 * ROW_BYTES;
            const unsigned char* p = src_w + pw_ks * ROW_BYTES;
#pragma unroll
            for (int t = 0; t < TILES; ++t)
                if (t < pw.nw) slab_load_stream_explicit(p + t * tile_stride, dst + t * W_BYTES);
            issued += pw.nw;
            slot_mark = issued;
            ++w_issued;
            if (++pw_ks == nks) {
                pw_ks = 0;
                next_seg(pw);
                if (pw.valid) pw_enter();
            }
        };

        // ---------------------------------------------------------------- token producer: this lane's operand of a stage, in registers
        Seg px = pw;                      // (the three cursors start at the same segment: looked up once)
        int px_ks = 0;
        const uint16_t* src_x[NT];        // per token tile: row 64*j + 16*wave + n of the pass, columns 8*q .. (bf16 weights) or 16*q .. (codes)
#pragma unroll
        for (int j = 0; j < NT; ++j) src_x[j] = nullptr;
        int px_key = -1;                  // (slot, pass) src_x was built for
        int ready_slot = -1;              // down phase: slot whose h is known to be complete
        auto px_enter = [&]() {           // new (segment, pass): uniform control flow
            if (phase == 1 && px.a != ready_slot) {                // wait until every gate/up item of this expert has published h
                if (tid == 0) {
                    int spins = 0;
                    while (__hip_atomic_load(&ctrl->done[px.a][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < tiles_a) {
                        __builtin_amdgcn_s_sleep(8);
                        if (++spins > spin_limit) {                  // giving up: see the same wait in ffn_bf16_kernel.hip
                            int zero = 0;
                            asm volatile("" : "+v"(zero));             // (keeps the constant below out of the loop's registers)
                            __hip_atomic_store(fail_mark, WS_FAIL_MARK + (unsigned long long)zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            asm volatile("ds_write_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" ::"v"(fail_addr), "v"(1u) : "memory");
                            break;
                        }
                    }
                }
                wg_barrier();
                wait_failed = wait_failed || __builtin_amdgcn_readfirstlane(lds_read_i32(fail_addr)) != 0;
                ready_slot = px.a;
            }
            const int key = px.a * 64 + px.pass;
            if (key != px_key) {
                px_key = key;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    int row = px.pass * MTT + j * MT + 16 * wave + n;
                    if (row >= px.m) row = px.pass * MTT;              // rows beyond the expert's last: a valid row, result unused
                    if (phase == 0) {
                        // (from the kernel's LDS copy when there is one; a load from global memory waits for every load in flight)
                        int tok = s_sorted ? lds_read_u16(lds_addr(s_sorted) + 2 * (px.r0 + row)) : sorted_token[px.r0 + row];
                        tok = min(max(tok, 0), T - 1);
                        src_x[j] = x + (size_t)tok * H + q * (16 / WB);
                    } else {
                        src_x[j] = h + (size_t)(px.r0 + row) * I + q * (16 / WB);
                    }
                }
            }
        };
        // Token operands of the next DX stages.  K-step s of a stage meets, in lane group q, the 8 columns 32 s + 8 q .. (bf16
        // weights) or 64 (s / 2) + 16 q + 8 (s % 2) .. (codes: a lane's 16-byte LDS read holds 16 consecutive columns, used as two
        // K-steps); any assignment of columns to K-steps is a valid order of the sum as long as both operands use it.
        bf16x8_t xq[DX][NT][XL];
        auto produce_x = [&](bf16x8_t (&dst)[NT][XL]) {             // (only while px.valid)
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const uint16_t* p = src_x[j] + px_ks * KCOL;
                if constexpr (WB == 2) {
                    if (phase == 0) {
                        request_tokens<false, 0>(dst[j][0], p);
                        request_tokens<false, 64>(dst[j][1], p);
                    } else {
                        request_tokens<true, 0>(dst[j][0], p);
                        request_tokens<true, 64>(dst[j][1], p);
                    }
                } else {
                    if (phase == 0) {
                        request_tokens<false, 0>(dst[j][0], p);
                        request_tokens<false, 16>(dst[j][1], p);
                        request_tokens<false, 128>(dst[j][2], p);
                        request_tokens<false, 144>(dst[j][3], p);
                    } else {
                        request_tokens<true, 0>(dst[j][0], p);
                        request_tokens<true, 16>(dst[j][1], p);
                        request_tokens<true, 128>(dst[j][2], p);
                        request_tokens<true, 144>(dst[j][3], p);
                    }
                }
            }
            issued += NT * XL;
            if (++px_ks == nks) {
                px_ks = 0;
                next_seg(px);
                if (px.valid) px_enter();
            }
        };

        // ---------------------------------------------------------------- consumer
        Seg cs = pw;
        int c_ks = 0;                     // stage inside the segment
        int pend = 0;                     // finished gate/up items of the current run (one slot) not yet published
        int pub_slot = -1, pub_cnt = 0, pub_mark = 0;   // run whose publication waits for its h stores to be acknowledged
        f32x4_t acc[TILES][NT][2];
#pragma unroll
        for (int t = 0; t < TILES; ++t)
#pragma unroll
            for (int j = 0; j < NT; ++j) acc[t][j][0] = acc[t][j][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        // Requests in front of the loop: the tokens of the first DX stages and the weights of the first DW - 1.  Gate/up phase:
        // tokens first, as inside the loop.  Down phase: the weights first, because the tokens (h) have to wait for other
        // workgroups and the weights do not; its first DW - 1 stages then wait for all of these requests.
        if (phase == 0) {
            if (px.valid) px_enter();
#pragma unroll
            for (int u = 0; u < DX; ++u)
                if (px.valid) produce_x(xq[u]);
        }
        if (pw.valid) pw_enter();
#pragma unroll
        for (int i = 0; i < DW; ++i) mark_w[i] = 0;
#pragma unroll
        for (int i = 0; i < DW - 1; ++i)
            if (pw.valid) produce_w(mark_w[i]);
        if (phase == 1) {
            if (px.valid) px_enter();
#pragma unroll
            for (int u = 0; u < DX; ++u)
                if (px.valid) produce_x(xq[u]);
#pragma unroll
            for (int i = 0; i < DW - 1; ++i) mark_w[i] = issued;
        }

        while (cs.valid) {
            for_each_slot([&](auto slot_index) -> bool {
                constexpr int u = decltype(slot_index)::value;      // token registers of this stage; its ring slot is u % DW
                static_assert(DX % DW == 0, "the ring slot of a stage follows from its token registers");
                if (!cs.valid) return false;
                // (1) this stage's tokens and weights have landed: everything up to the weight requests of this stage
                wait_outstanding_rt(issued - mark_w[u % DW]);
                wg_barrier();
                // (2) a run of gate/up items whose h stores are older than loads that have completed is complete in every
                //     wavefront (operations complete in issue order): publish it
                if (pub_slot >= 0 && mark_w[u % DW] > pub_mark) {
                    if (tid == 0 && !skip_publish) __hip_atomic_fetch_add(&ctrl->done[pub_slot][0], pub_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    pub_slot = -1;
                }
                // (3) refill the ring slot that the previous iteration has finished reading
                if (pw.valid) produce_w(mark_w[(u + DW - 1) % DW]);
                // (4) multiply
                const uint32_t slot = ring0 + (u % DW) * STAGE_BYTES;
#pragma unroll
                for (int t = 0; t < TILES; ++t) {
                    if (t < cs.nw) {
                        const uint32_t wt = slot + t * W_BYTES;
                        bf16x8_t w00, w10, w01, w11;
                        lds_read4(wt + rd_w[0][0], wt + rd_w[1][0], wt + rd_w[0][1], wt + rd_w[1][1], w00, w10, w01, w11);
                        if constexpr (WB == 2) {
#pragma unroll
                            for (int j = 0; j < NT; ++j) {
                                acc[t][j][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w00, xq[u][j][0], acc[t][j][0], 0, 0, 0);
                                acc[t][j][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w10, xq[u][j][0], acc[t][j][1], 0, 0, 0);
                            }
#pragma unroll
                            for (int j = 0; j < NT; ++j) {
                                acc[t][j][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w01, xq[u][j][1], acc[t][j][0], 0, 0, 0);
                                acc[t][j][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w11, xq[u][j][1], acc[t][j][1], 0, 0, 0);
                            }
                        } else {                                    // each read: the codes of two K-steps
                            bf16x8_t a0, a1, b0, b1;
                            widen_e4m3(w00, a0, a1);
                            widen_e4m3(w10, b0, b1);
                            acc[t][0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, xq[u][0][0], acc[t][0][0], 0, 0, 0);
                            acc[t][0][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b0, xq[u][0][0], acc[t][0][1], 0, 0, 0);
                            acc[t][0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, xq[u][0][1], acc[t][0][0], 0, 0, 0);
                            acc[t][0][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b1, xq[u][0][1], acc[t][0][1], 0, 0, 0);
                            widen_e4m3(w01, a0, a1);
                            widen_e4m3(w11, b0, b1);
                            acc[t][0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, xq[u][0][2], acc[t][0][0], 0, 0, 0);
                            acc[t][0][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b0, xq[u][0][2], acc[t][0][1], 0, 0, 0);
                            acc[t][0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, xq[u][0][3], acc[t][0][0], 0, 0, 0);
                            acc[t][0][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b1, xq[u][0][3], acc[t][0][1], 0, 0, 0);
                        }
                    }
                }
                // (5) request this lane's tokens of the stage DX ahead into the registers just used
                if (px.valid) produce_x(xq[u]);
                if (++c_ks < nks) return true;
                // (6) last stage of the (segment, pass): epilogue for this wavefront's token tile
                c_ks = 0;
#pragma unroll
                for (int t = 0; t < TILES; ++t) {
#pragma unroll
                  for (int j = 0; j < NT; ++j) {
                    const int row = cs.pass * MTT + j * MT + 16 * wave + n;
                    f32x4_t (&ac)[2] = acc[t][j];
                    if (t < cs.nw && row < cs.m) {
                        const int it = cs.it + t;
                        if constexpr (WB == 1) {                    // row scales of the item (read through the scalar cache: see load_scales)
                            if (phase == 0) {
                                float g16[16], u16[16];             // scales of intermediate indices it*16 .. +15
                                load_scales(sg + (size_t)cs.e * I + it * 16, g16);
                                load_scales(su + (size_t)cs.e * I + it * 16, u16);
#pragma unroll
                                for (int rt = 0; rt < 2; ++rt) {
                                    ac[rt][0] *= pick_q(g16, 8 * rt, 2, q);
                                    ac[rt][1] *= pick_q(g16, 8 * rt + 1, 2, q);
                                    ac[rt][2] *= pick_q(u16, 8 * rt, 2, q);
                                    ac[rt][3] *= pick_q(u16, 8 * rt + 1, 2, q);
                                }
                            } else {
#pragma unroll
                                for (int rt = 0; rt < 2; ++rt) {
                                    float d16[16];                  // scales of output rows it*32 + rt*16 .. +15
                                    load_scales(sd + (size_t)cs.e * H + it * W_ROWS + rt * 16, d16);
#pragma unroll
                                    for (int c = 0; c < 4; ++c) ac[rt][c] *= pick_q(d16, c, 4, q);
                                }
                            }
                        }
                        if (phase == 0) {
#pragma unroll
                            for (int rt = 0; rt < 2; ++rt) {
                                // lane holds (g_a, g_b, u_a, u_b) of intermediate indices it*16 + rt*8 + 2*q, +1 for token row `row`
                                const float h0 = silu_f32(ac[rt][0]) * ac[rt][2];
                                const float h1 = silu_f32(ac[rt][1]) * ac[rt][3];
                                const uint32_t packed = f32_to_bf16_bits(h0) | (f32_to_bf16_bits(h1) << 16);
                                store_coherent(reinterpret_cast<uint32_t*>(h + (size_t)(cs.r0 + row) * I + it * 16 + rt * 8 + 2 * q), packed);
                            }
                        } else {
#pragma unroll
                            for (int rt = 0; rt < 2; ++rt) { // lane holds output rows it*32 + rt*16 + 4*q + (0..3) of token row `row`
                                const float nan = __builtin_nanf("");
                                *reinterpret_cast<f32x4_t*>(out + (size_t)(cs.r0 + row) * H + it * W_ROWS + rt * 16 + 4 * q) =
                                    wait_failed ? f32x4_t{nan, nan, nan, nan} : ac[rt];
                            }
                        }
                    }
                    ac[0] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    ac[1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                  }
                }
                const int prev_a = cs.a, prev_li = cs.li, prev_nw = cs.nw;
                next_seg(cs);
                if (phase == 0 && (!cs.valid || cs.li != prev_li)) {   // the segment is finished (all passes)
                    pend += prev_nw;
                    if (!cs.valid || cs.a != prev_a) {                  // and so is the run of items of this slot
                        if (pub_slot >= 0) {                            // an older run is still waiting (only with very few stages per
                            wait_outstanding<0>();                      // item): acknowledge everything now and publish it at once
                            wg_barrier();
                            if (tid == 0 && !skip_publish)
                                __hip_atomic_fetch_add(&ctrl->done[pub_slot][0], pub_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                        pub_slot = prev_a;
                        pub_cnt = pend;
                        pub_mark = issued;
                        pend = 0;
                    }
                }
                return true;
            }, std::make_integer_sequence<int, DX>{});
        }
        // ---- end of phase: everything this workgroup stored is acknowledged, then the last run is published
        wait_outstanding<0>();
        wg_barrier();
        if (pub_slot >= 0 && tid == 0 && !skip_publish)
            __hip_atomic_fetch_add(&ctrl->done[pub_slot][0], pub_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("; team_tiled_body_end" ::: "memory");
}

}  // namespace tiled

}  // namespace team
