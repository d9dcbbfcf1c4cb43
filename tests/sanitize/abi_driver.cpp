// Calls the host side of the C ABI (include/team_moe.h) the way a confused caller would - NULL and misaligned pointers, sizes
// out of range, bad configurations, unknown knobs - in a build whose host code carries AddressSanitizer and
// UndefinedBehaviorSanitizer (tests/test_sanitizers.py).  Every call must be rejected before anything touches a GPU, so the
// program runs on a machine without one.  Exit status 0 = all statuses as expected and nothing for the sanitizers to report.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/team_moe.h"
#include "../../include/team_moe_internal.h"

#define EXPECT(call, status)                                                                      \
    do {                                                                                          \
        const int got_ = (call);                                                                  \
        if (got_ != (status)) {                                                                   \
            fprintf(stderr, "line %d: %s returned %d, expected %d\n", __LINE__, #call, got_, (int)(status)); \
            return 1;                                                                             \
        }                                                                                         \
    } while (0)

int main() {
    team_moe_config cfg = {2048, 768, 128, 8, TEAM_BF16, 1, 32, 0};
    void* fake = (void*)(uintptr_t)0x1000;       // aligned, never dereferenced: every call fails validation first
    void* odd = (void*)(uintptr_t)0x1004;
    size_t bytes = 0;
    EXPECT(team_moe_workspace_size(&cfg, &bytes), TEAM_OK);
    if (bytes < (size_t)32 * 8 * 2048 * 4 || bytes % 256 != 0) return 1;
    EXPECT(team_moe_workspace_size(nullptr, &bytes), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_workspace_size(&cfg, nullptr), TEAM_ERR_INVALID_ARG);
    // configurations: every field at and beyond its limits
    const int32_t bad[][8] = {{2048, 768, 128, 0, 1, 1, 32, 0},   {2048, 768, 4, 8, 1, 1, 32, 0},     {2048, 768, 512, 8, 1, 1, 32, 0},
                              {2048, 768, 128, 32, 1, 1, 32, 0},  {2000, 768, 128, 8, 1, 1, 32, 0},   {2048, 700, 128, 8, 1, 1, 32, 0},
                              {2048, 768, 128, 8, 1, 1, 4096, 0}, {2048, 768, 128, 8, 1, 1, 0, 0},    {2048, 768, 128, 8, 7, 1, 32, 0},
                              {2048, 768, 128, 8, 1, 2, 32, 0},   {2048, 768, 128, 8, 1, 1, 32, 9},   {-2048, 768, 128, 8, 1, 1, 32, 0},
                              {2048, 768, 128, 8, 1, 1, 2147483647, 0}, {2147483644, 2147483644, 256, 16, 0, 1, 1024, 0}};
    for (const auto& b : bad) {
        team_moe_config c;
        memcpy(&c, b, sizeof(c));
        const int st = team_moe_workspace_size(&c, &bytes);
        if (c.hidden == 2147483644) {                     // the largest float configuration the limits admit: size arithmetic must not overflow
            if (st != TEAM_OK || bytes < (size_t)1024 * 16 * 2147483644ull * 4) return 1;
            continue;
        }
        if (st != TEAM_ERR_INVALID_ARG && st != TEAM_ERR_UNSUPPORTED) {
            fprintf(stderr, "bad configuration accepted (hidden %d)\n", c.hidden);
            return 1;
        }
    }
    EXPECT(team_moe_route(&cfg, nullptr, 8, fake, nullptr, (int32_t*)fake, (float*)fake, nullptr, nullptr, 0, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_route(&cfg, fake, 0, fake, nullptr, (int32_t*)fake, (float*)fake, nullptr, nullptr, 0, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_route(&cfg, fake, 33, fake, nullptr, (int32_t*)fake, (float*)fake, nullptr, nullptr, 0, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_route(&cfg, odd, 8, fake, nullptr, (int32_t*)fake, (float*)fake, nullptr, nullptr, 0, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_route(&cfg, fake, 8, fake, nullptr, (int32_t*)fake, (float*)fake, nullptr, nullptr, 0, nullptr), TEAM_ERR_WORKSPACE);
    EXPECT(team_moe_route(&cfg, fake, 8, fake, nullptr, (int32_t*)fake, (float*)fake, nullptr, fake, 64, nullptr), TEAM_ERR_WORKSPACE);
    EXPECT(team_moe_build_dispatch(&cfg, nullptr, 8, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, nullptr, 0, nullptr),
           TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_expert_ffn(&cfg, fake, 8, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, fake, fake, nullptr, (float*)fake, fake,
                               (size_t)1 << 30, nullptr),
           TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_expert_ffn(&cfg, fake, 8, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, fake, fake, fake, (float*)fake, fake, 16,
                               nullptr),
           TEAM_ERR_WORKSPACE);
    EXPECT(team_moe_combine(&cfg, (float*)fake, (float*)fake, nullptr, 8, fake, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_layer_forward(&cfg, fake, 8, fake, fake, fake, fake, nullptr, nullptr, fake, (size_t)1 << 30, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_layer_forward(&cfg, fake, 8, fake, fake, fake, fake, nullptr, fake, nullptr, 0, nullptr), TEAM_ERR_WORKSPACE);
    EXPECT(team_moe_layer_forward(&cfg, fake, 8, fake, fake, fake, fake, nullptr, fake, fake, 1024, nullptr), TEAM_ERR_WORKSPACE);
    EXPECT(team_moe_layer_forward(&cfg, fake, 8, fake, fake, fake, fake, nullptr, fake, odd, (size_t)1 << 30, nullptr), TEAM_ERR_WORKSPACE);
    EXPECT(team_moe_route_two_round(&cfg, fake, 8, fake, nullptr, nullptr, nullptr, (int32_t*)fake, (float*)fake, nullptr, fake, (size_t)1 << 30, nullptr),
           TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_classify_tokens((float*)fake, (uint8_t*)fake, 32, 0, nullptr, 32, 0.7f, 3, (uint8_t*)fake, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_classify_tokens((float*)fake, (uint8_t*)fake, 32, 32, nullptr, 33, 0.7f, 3, (uint8_t*)fake, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_layer_forward_rows(&cfg, fake, fake, 0, (int32_t*)fake, 8, fake, fake, fake, fake, nullptr, nullptr, nullptr, nullptr, fake,
                                       (size_t)1 << 30, nullptr),
           TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_dequantize_w8((uint8_t*)fake, (float*)fake, 4, 40, (float*)fake, nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_workspace_status(fake, 128, nullptr), TEAM_ERR_WORKSPACE);
    EXPECT(team_moe_workspace_status(odd, (size_t)1 << 20, nullptr), TEAM_ERR_WORKSPACE);
    team_moe_config big = {2048, 512, 256, 8, TEAM_BF16, 1, 256, 0};
    EXPECT(team_moe_layer_forward_static(&big, fake, 256, fake, fake, fake, fake, nullptr, fake, nullptr), TEAM_ERR_WORKSPACE);
    team_moe_layer_args a;
    memset(&a, 0, sizeof(a));
    EXPECT(team_moe_layer_forward_ex(&cfg, nullptr), TEAM_ERR_INVALID_ARG);
    a.x = fake; a.y = fake; a.T = 8; a.w_router = a.w_gate = a.w_up = a.w_down = fake; a.workspace = fake; a.ws_bytes = (size_t)1 << 30;
    a.unique_rows = 2;
    EXPECT(team_moe_layer_forward_ex(&cfg, &a), TEAM_ERR_INVALID_ARG);
    a.unique_rows = 0; a.ffn_begin_event = fake;
    EXPECT(team_moe_layer_forward_ex(&cfg, &a), TEAM_ERR_INVALID_ARG);
    a.ffn_begin_event = nullptr; a.expert_mask = (uint8_t*)fake; a.token_class = (uint8_t*)fake;
    EXPECT(team_moe_layer_forward_ex(&cfg, &a), TEAM_ERR_INVALID_ARG);
    int v = 0;
    EXPECT(team_moe_internal_set("no_such_knob", 1), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_internal_set(nullptr, 1), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_internal_get("ffn_spin_limit", nullptr), TEAM_ERR_INVALID_ARG);
    EXPECT(team_moe_internal_get("row_hash_bits", &v), TEAM_OK);
    for (int s = -6; s <= 1; ++s)
        if (!team_moe_status_string(s) || !team_moe_status_string(s)[0]) return 1;
    printf("host side of the C ABI under sanitizers: ok\n");
    return 0;
}
