// Tuning and testing knobs (see tuning.hpp) and their C entry points (include/team_moe_internal.h).
#include "tuning.hpp"

#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "../../include/team_moe.h"
#include "../../include/team_moe_internal.h"

namespace team {

namespace {

int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    return atoi(v);
}

std::atomic<int>* knob(Tuning& t, const char* key) {
    if (!key) return nullptr;
    if (!strcmp(key, "ffn_grid")) return &t.ffn_grid;
    if (!strcmp(key, "ffn_tiled_rows")) return &t.ffn_tiled_rows;
    if (!strcmp(key, "ffn_wide_rows")) return &t.ffn_wide_rows;
    if (!strcmp(key, "ffn_shares")) return &t.ffn_shares;
    if (!strcmp(key, "logits_kernel")) return &t.logits_kernel;
    if (!strcmp(key, "row_hash_bits")) return &t.row_hash_bits;
    if (!strcmp(key, "ffn_spin_limit")) return &t.ffn_spin_limit;
    if (!strcmp(key, "ffn_skip_publish")) return &t.ffn_skip_publish;
    if (!strcmp(key, "ffn_cooperative")) return &t.ffn_cooperative;
    return nullptr;
}

}  // namespace

Tuning& tuning() {
    static Tuning t;
    static std::once_flag once;
    std::call_once(once, [] {
        t.ffn_grid = env_int("TEAM_MOE_FFN_GRID", 0);
        t.ffn_tiled_rows = env_int("TEAM_MOE_FFN_TILED_ROWS", 18);
        t.ffn_wide_rows = env_int("TEAM_MOE_FFN_WIDE_ROWS", 56);
        const char* shares = getenv("TEAM_MOE_FFN_SHARES");            // "contiguous" | "all" | (default) expert-major where it pays
        t.ffn_shares = shares && shares[0] == 'c' ? 0 : (shares && shares[0] == 'a' ? 2 : 1);
        const char* lk = getenv("TEAM_MOE_LOGITS_KERNEL");             // "plain" | "mfma"
        t.logits_kernel = lk && lk[0] == 'p' ? 1 : (lk && lk[0] == 'm' ? 2 : 0);
        t.row_hash_bits = env_int("TEAM_MOE_ROW_HASH_BITS", 64);
        t.ffn_spin_limit = env_int("TEAM_MOE_FFN_SPIN_LIMIT", 1 << 16);
        t.ffn_cooperative = env_int("TEAM_MOE_FFN_COOPERATIVE", 0);
    });
    return t;
}

}  // namespace team

extern "C" {

int team_moe_internal_set(const char* key, int value) {
    std::atomic<int>* k = team::knob(team::tuning(), key);
    if (!k) return TEAM_ERR_INVALID_ARG;
    k->store(value);
    return TEAM_OK;
}

int team_moe_internal_get(const char* key, int* value) {
    std::atomic<int>* k = team::knob(team::tuning(), key);
    if (!k || !value) return TEAM_ERR_INVALID_ARG;
    *value = k->load();
    return TEAM_OK;
}

}  // extern "C"
