// Grouped SwiGLU expert FFN, bf16, gfx950 MFMA: the variant for calls with many tokens per expert
// (speculative branches and batched blocks: tens to hundreds of rows per activated expert).  Included by
// ffn_bf16_kernel.hip; the persistent kernel switches to this body when the call averages many rows per expert.
//
// Same work decomposition, same per-expert h hand-over and same deterministic results as ffn_bf16_kernel.hip,
// but both operands stream through LDS in a software pipeline instead of keeping the token operand in
// registers: with more than 32 rows per expert the register-resident operand has to be re-gathered for every
// item, and that gather (16 bytes per lane, rows 4 KB apart) costs more than the weights it is used with.
//
//   item     gate/up: (expert, 16 intermediate indices) = 16 rows of w_gate + 16 rows of w_up, all H columns
//            down   : (expert, 32 output rows of w_down), all I columns
//   pass     64 token rows of the expert (4 token tiles, one per wavefront); experts with more rows take
//            several passes over the same weight rows (served by the caches after the first pass)
//   stage    64 reduction columns: 32 weight rows x 128 B (4 KB) + 64 token rows x 128 B (8 KB)
// A ring of D stages lives in LDS.  Every wavefront issues three 1 KB direct-to-LDS loads per stage (8 weight
// rows, and the two halves of its own token tile), D-1 stages ahead of the stage being multiplied, so weight
// bytes are in flight all the time, also across item boundaries.  A wavefront owns a token tile and
// multiplies it with both 16-row weight tiles: no reduction across wavefronts, sums in a fixed order.
//
// LDS stage layout: rows of 128 B (8 chunks of 16 B); chunk c of row r is stored at chunk c ^ ((r >> 1) & 7),
// which spreads the 16 rows of an MFMA operand read over all 16 bank groups.  The swizzle is applied to the
// global address a lane fetches, because a direct-to-LDS load writes the lanes of a wavefront contiguously.
//
// The loop counts its own outstanding loads (s_waitcnt vmcnt(N) with a constant N per wavefront) and reads LDS
// with explicit instructions: the compiler's automatic waits treat every direct-to-LDS load as aliasing every
// LDS read and would drain the pipeline at each stage.
#pragma once
#include "ffn_bf16.hpp"

namespace team {

namespace tiled {

constexpr int KC = 64;                 // reduction columns per stage
constexpr int MT = 64;                 // token rows per pass
constexpr int W_ROWS = 32;             // weight rows per item
constexpr int ROW_BYTES = KC * 2;      // 128
constexpr int W_BYTES = W_ROWS * ROW_BYTES;
constexpr int X_BYTES = MT * ROW_BYTES;
constexpr int STAGE_BYTES = W_BYTES + X_BYTES;
constexpr int LOADS_PER_STAGE = 3;     // per wavefront

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int AUX>
__device__ __forceinline__ void slab_load(const void* gsrc, char* lds_base_uniform) {
    __builtin_amdgcn_global_load_lds((gptr_t)gsrc, (lptr_t)lds_base_uniform, 16, 0, AUX);
}
constexpr int AUX_NONE = 0;
constexpr int AUX_STREAM = 2;          // nt: read once, do not displace the small reused data (tokens, h, out) from L2
constexpr int AUX_DEVICE_SCOPE = 16;   // sc1: the load does not use possibly stale lines of this XCD's L2

template <int N>
__device__ __forceinline__ void wait_outstanding() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wg_barrier() {
    asm volatile("s_barrier" ::: "memory");
}
// Three 16-byte LDS reads (two weight tiles, one token tile) at byte addresses a0, a1, a2.
__device__ __forceinline__ void lds_read3(uint32_t a0, uint32_t a1, uint32_t a2, bf16x8_t& w0, bf16x8_t& w1, bf16x8_t& xt) {
    asm volatile(
        "ds_read_b128 %0, %3\n\t"
        "ds_read_b128 %1, %4\n\t"
        "ds_read_b128 %2, %5\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(w0), "=&v"(w1), "=&v"(xt)
        : "v"(a0), "v"(a1), "v"(a2)
        : "memory");
}
__device__ __forceinline__ void store_coherent(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(lptr_t)p;
}
// One 32-bit LDS read at byte address a (explicit for the same reason as lds_read3).
__device__ __forceinline__ int lds_read_i32(uint32_t a) {
    int v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a) : "memory");
    return v;
}

struct Seg {                   // one (item, pass) of a workgroup's share
    int li;                    // item index in the expert-major list of the phase
    int a, it, e, r0, m, pass;
    bool valid;
};

constexpr int RING_STAGES = 6;
constexpr int RING_BYTES = RING_STAGES * STAGE_BYTES;

// Body of the streaming variant; runs inside the persistent FFN kernel (all workgroups take it or none does).
// s_ring: RING_BYTES of LDS, 1 KB aligned; s_slot_e / s_off: the kernel's tables (active list, clipped offsets).
template <int D>
__device__ __forceinline__ void ffn_tiled_body(char* s_ring, const int32_t* s_slot_e, const int32_t* s_off, int n_act,
                                               const uint16_t* __restrict__ x, const int32_t* __restrict__ sorted_token,
                                               const uint16_t* __restrict__ wg, const uint16_t* __restrict__ wu,
                                               const uint16_t* __restrict__ wd, uint16_t* __restrict__ h, float* __restrict__ out,
                                               FfnCtrl* __restrict__ ctrl, int T, int E, int H, int I, int spin_limit) {
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, q = lane >> 4;
    const int G = gridDim.x;
    const int tiles_a = I / 16, tiles_b = H / W_ROWS;

    // ---- lane constants
    // loads: lane fetches row (l / 8) of an 8-row slab, stored chunk (l % 8)
    const int ld_row = lane >> 3, ld_cs = lane & 7;
    // reads: MFMA operand row n, chunk 4*ks + q, un-swizzled on the fly
    const uint32_t ring0 = lds_addr(s_ring);
    const uint32_t tab_e = lds_addr(s_slot_e), tab_off = lds_addr(s_off);
    uint32_t rd_w[2][2], rd_x[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const int r = 16 * rt + n;
            rd_w[rt][ks] = r * ROW_BYTES + (((4 * ks + q) ^ ((r >> 1) & 7)) << 4);
        }
        const int r = 16 * wave + n;
        rd_x[ks] = W_BYTES + r * ROW_BYTES + (((4 * ks + q) ^ ((r >> 1) & 7)) << 4);
    }

    for (int phase = 0; phase < 2; ++phase) {
        const int tiles = phase == 0 ? tiles_a : tiles_b;
        const int nks = (phase == 0 ? H : I) / KC;                 // stages per (item, pass)
        const long long total = (long long)n_act * tiles;
        // contiguous shares; the remainder goes to the lowest-numbered workgroups (see the register-operand body)
        const int share = (int)(total / G), extra = (int)(total % G), bx = (int)blockIdx.x;
        const int li_begin = bx * share + min(bx, extra), li_end = li_begin + share + (bx < extra ? 1 : 0);

        auto load_item = [&](Seg& s) {                              // fills a, it, e, r0, m of item s.li; skips items without rows
            s.valid = false;
            while (s.li < li_end) {
                s.a = s.li / tiles;
                s.it = s.li - s.a * tiles;
                s.e = __builtin_amdgcn_readfirstlane(lds_read_i32(tab_e + 4 * s.a));
                const bool ok = s.e >= 0 && s.e < E;
                s.r0 = ok ? __builtin_amdgcn_readfirstlane(lds_read_i32(tab_off + 4 * s.e)) : 0;
                s.m = ok ? max(__builtin_amdgcn_readfirstlane(lds_read_i32(tab_off + 4 * s.e + 4)) - s.r0, 0) : 0;
                s.pass = 0;
                if (s.m > 0) {
                    s.valid = true;
                    return;
                }
                ++s.li;
            }
        };
        auto next_seg = [&](Seg& s) {
            if ((s.pass + 1) * MT < s.m) {
                ++s.pass;
            } else {
                ++s.li;
                load_item(s);
            }
        };

        // ---------------------------------------------------------------- producer: per-lane source pointers of the three slabs
        Seg ps;
        ps.li = li_begin;
        load_item(ps);
        int p_ks = 0;
        int p_issued = 0;                 // stages issued so far in this phase
        const uint16_t* src_w = nullptr;  // weight slab: rows 8*wave .. 8*wave+7 of the item
        const uint16_t* src_x0 = nullptr; // token slabs: rows 16*wave .. +7 and +8 .. +15 of the pass
        const uint16_t* src_x1 = nullptr;
        int p_key = -1;                   // (slot, pass) the token pointers were built for
        int ready_slot = -1;              // down phase: slot whose h is known to be complete

        auto producer_enter = [&]() {     // new (item, pass): rebuild the source pointers (uniform control flow)
            const int r = 8 * wave + ld_row;                       // weight row of the item this lane fetches
            const int c = ld_cs ^ ((r >> 1) & 7);                  // global chunk that belongs at the stored chunk
            if (phase == 0) {
                const int i = r & 15;
                const int iidx = ps.it * 16 + (r >> 4) * 8 + 2 * (i >> 2) + (i & 1);   // rows 4q+{0,1}: gate, 4q+{2,3}: up
                const uint16_t* mat = (i & 2) ? wu : wg;
                src_w = mat + ((size_t)ps.e * I + iidx) * H + c * 8;
            } else {
                src_w = wd + ((size_t)ps.e * H + (size_t)ps.it * W_ROWS + r) * I + c * 8;
            }
            const int key = ps.a * 64 + ps.pass;
            if (phase == 1 && ps.a != ready_slot) {                // wait until every gate/up item of this expert has published h
                if (tid == 0) {
                    int spins = 0;
                    while (__hip_atomic_load(&ctrl->done[ps.a][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < tiles_a) {
                        __builtin_amdgcn_s_sleep(8);
                        if (++spins > spin_limit) {                  // cannot happen with a control block zeroed before the launch
                            ctrl->error = 1;
                            break;
                        }
                    }
                }
                wg_barrier();
                ready_slot = ps.a;
            }
            if (key != p_key) {
                p_key = key;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int tr = 16 * wave + 8 * j + ld_row;     // token row of the pass
                    const int cx = ld_cs ^ ((tr >> 1) & 7);
                    int row = ps.pass * MT + tr;
                    if (row >= ps.m) row = ps.pass * MT;           // rows beyond the expert's last: fetch a valid row, result unused
                    const uint16_t* p;
                    if (phase == 0) {
                        int tok = sorted_token[ps.r0 + row];
                        tok = min(max(tok, 0), T - 1);
                        p = x + (size_t)tok * H + cx * 8;
                    } else {
                        p = h + (size_t)(ps.r0 + row) * I + cx * 8;
                    }
                    if (j == 0) src_x0 = p; else src_x1 = p;
                }
            }
        };
        auto produce_stage = [&]() {      // issue the three loads of the producer's current stage, then advance it
            char* slot = s_ring + (p_issued % D) * STAGE_BYTES;
            const int koff = p_ks * KC;
            slab_load<AUX_STREAM>(src_w + koff, slot + wave * 8 * ROW_BYTES);
            if (phase == 0) {
                slab_load<AUX_NONE>(src_x0 + koff, slot + W_BYTES + (16 * wave) * ROW_BYTES);
                slab_load<AUX_NONE>(src_x1 + koff, slot + W_BYTES + (16 * wave + 8) * ROW_BYTES);
            } else {
                slab_load<AUX_DEVICE_SCOPE>(src_x0 + koff, slot + W_BYTES + (16 * wave) * ROW_BYTES);
                slab_load<AUX_DEVICE_SCOPE>(src_x1 + koff, slot + W_BYTES + (16 * wave + 8) * ROW_BYTES);
            }
            ++p_issued;
            if (++p_ks == nks) {
                p_ks = 0;
                next_seg(ps);
                if (ps.valid) producer_enter();
            }
        };

        // ---------------------------------------------------------------- consumer
        Seg cs;
        cs.li = li_begin;
        load_item(cs);
        int c_ks = 0, c_done = 0;         // stage inside the segment; stages consumed so far in this phase
        int pend = 0;                     // finished gate/up items of the current run (one slot) not yet published
        int pub_slot = -1, pub_cnt = 0, pub_at = 0;   // run whose publication waits for its h stores to be acknowledged
        f32x4_t acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};

        if (ps.valid) producer_enter();
        for (int i = 0; i < D - 1 && ps.valid; ++i) produce_stage();

        while (cs.valid) {
            // (1) this stage's loads have landed: all but the loads of the D-2 stages issued after it
            if (p_issued - c_done - 1 == D - 2) wait_outstanding<LOADS_PER_STAGE*(D - 2)>(); else wait_outstanding<0>();
            wg_barrier();
            // (2) a run of gate/up items whose h stores are D-1 stages old is complete in every wavefront: publish it
            if (pub_slot >= 0 && c_done >= pub_at) {
                if (tid == 0) __hip_atomic_fetch_add(&ctrl->done[pub_slot][0], pub_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                pub_slot = -1;
            }
            // (3) refill the slot that the previous iteration has finished reading
            if (ps.valid) produce_stage();
            // (4) multiply
            const uint32_t slot = ring0 + (c_done % D) * STAGE_BYTES;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                bf16x8_t w0, w1, xt;
                lds_read3(slot + rd_w[0][ks], slot + rd_w[1][ks], slot + rd_x[ks], w0, w1, xt);
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w0, xt, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1, xt, acc[1], 0, 0, 0);
            }
            ++c_done;
            if (++c_ks < nks) continue;
            // (5) last stage of the (item, pass): epilogue for this wavefront's token tile
            c_ks = 0;
            const int row = cs.pass * MT + 16 * wave + n;
            if (row < cs.m) {
                if (phase == 0) {
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt) {
                        // lane holds (g_a, g_b, u_a, u_b) of intermediate indices it*16 + rt*8 + 2*q, +1 for token row `row`
                        const float h0 = silu_f32(acc[rt][0]) * acc[rt][2];
                        const float h1 = silu_f32(acc[rt][1]) * acc[rt][3];
                        const uint32_t packed = f32_to_bf16_bits(h0) | (f32_to_bf16_bits(h1) << 16);
                        store_coherent(reinterpret_cast<uint32_t*>(h + (size_t)(cs.r0 + row) * I + cs.it * 16 + rt * 8 + 2 * q), packed);
                    }
                } else {
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt)   // lane holds output rows it*32 + rt*16 + 4*q + (0..3) of token row `row`
                        *reinterpret_cast<f32x4_t*>(out + (size_t)(cs.r0 + row) * H + cs.it * W_ROWS + rt * 16 + 4 * q) = acc[rt];
                }
            }
            acc[0] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            acc[1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            const int prev_a = cs.a, prev_li = cs.li;
            next_seg(cs);
            if (phase == 0 && (!cs.valid || cs.li != prev_li)) {   // the item is finished (all passes)
                ++pend;
                if (!cs.valid || cs.a != prev_a) {                  // and so is the run of items of this slot
                    if (pub_slot >= 0) {                            // an older run is still waiting (only with very few stages per
                        wait_outstanding<0>();                      // item): acknowledge everything now and publish it at once
                        wg_barrier();
                        if (tid == 0)
                            __hip_atomic_fetch_add(&ctrl->done[pub_slot][0], pub_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    pub_slot = prev_a;
                    pub_cnt = pend;
                    pub_at = c_done + D - 1;
                    pend = 0;
                }
            }
        }
        // ---- end of phase: everything this workgroup stored is acknowledged, then the last run is published
        wait_outstanding<0>();
        wg_barrier();
        if (pub_slot >= 0 && tid == 0) __hip_atomic_fetch_add(&ctrl->done[pub_slot][0], pub_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}  // namespace tiled

}  // namespace team
