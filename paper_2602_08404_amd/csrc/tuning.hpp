// Tuning and testing knobs of the library (internal).  Every knob is read from its environment variable once, when the
// library is first used, and can afterwards be changed through team_moe_internal_set (include/team_moe_internal.h): no
// entry point reads the environment on its launch path.
#pragma once
#include <atomic>

namespace team {

struct Tuning {
    std::atomic<int> ffn_grid{0};            // TEAM_MOE_FFN_GRID: > 0: a smaller FFN grid than the resident maximum
    std::atomic<int> ffn_tiled_rows{18};     // TEAM_MOE_FFN_TILED_ROWS: streaming body from this many rows per expert on average (calls of more than 32 tokens)
    std::atomic<int> ffn_wide_rows{56};      // TEAM_MOE_FFN_WIDE_ROWS: two token tiles per wavefront above this many rows per expert
    std::atomic<int> ffn_shares{1};          // TEAM_MOE_FFN_SHARES: 0 contiguous shares only, 1 workgroups dealt out to experts where a share would cross (2: gate/up phase only)
    std::atomic<int> logits_kernel{0};       // TEAM_MOE_LOGITS_KERNEL: 0 by token count, 1 per-token kernel, 2 matrix-core kernel
    std::atomic<int> row_hash_bits{64};      // TEAM_MOE_ROW_HASH_BITS: bits of the row hashes the repeated-row search compares (tests force collisions with fewer)
    std::atomic<int> ffn_spin_limit{1 << 16};// TEAM_MOE_FFN_SPIN_LIMIT: polls before a wait inside the FFN kernel gives up (about 0.1 s by default)
    std::atomic<int> ffn_cooperative{0};     // TEAM_MOE_FFN_COOPERATIVE: 1: launch the FFN kernel through hipLaunchCooperativeKernel (measurement aid)
    std::atomic<int> ffn_skip_publish{0};    // tests only: gate/up items do not announce their results, so every wait for them gives up
};

Tuning& tuning();

}  // namespace team
