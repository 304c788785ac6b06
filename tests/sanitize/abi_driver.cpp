// Host side of libswapmoe under AddressSanitizer / UndefinedBehaviorSanitizer: the handle life
// cycle, every argument check, the maps, the update policies and the offline profile run here
// with the kernel launchers replaced by stubs (no GPU is touched; the HIP runtime calls that the
// checks make fail cleanly without a device and are turned into status codes).  Built and run by
// tests/test_sanitizers_cpu.py: the run must end with "ok" and no sanitizer report.
#include <cstdio>
#include <vector>

#include "smoe_internal.h"
#include "swapmoe_profile.h"

// ---- launcher stubs (the real ones live in the kernel translation units)
int smoe_launch_route(const smoe_layer*, const void*, int, int32_t*, float*, int32_t*, float*, float*, int32_t*, hipStream_t) { return 0; }
int smoe_launch_route_rank_small(const smoe_layer*, const void*, int, int32_t*, float*, int32_t*, float*, float*, int32_t*,
                                 float*, float*, int, int32_t*, int32_t*, int32_t*, hipStream_t) { return 0; }
bool smoe_decode_first_applies(const smoe_layer*, int) { return false; }
int smoe_launch_decode_first(const smoe_layer*, const void*, int, int32_t*, float*, int32_t*, float*, float*, int32_t*, float*, float*,
                             int, int32_t*, int32_t*, int32_t*, hipStream_t, hipEvent_t, hipEvent_t) { return 0; }
bool smoe_ffn_dense_path(const smoe_layer*, int) { return false; }
int smoe_launch_ffn_bf16_dense_second(const smoe_layer*, const int32_t*, const float*, const uint16_t*, int, uint16_t*, hipStream_t) { return 0; }
int smoe_launch_rank_importance(const smoe_layer*, const int32_t*, const float*, const float*, const int32_t*, int, int32_t*,
                                float*, float*, int, int32_t*, int32_t*, int32_t*, hipStream_t) { return 0; }
int smoe_launch_ffn_bf16_fused(const smoe_layer*, const uint16_t*, const int32_t*, const int32_t*, const int32_t*, const float*,
                               const uint16_t*, int, uint16_t*, hipStream_t) { return 0; }
int smoe_launch_importance(const smoe_layer*, const int32_t*, const float*, const float*, int, int32_t*, float*, float*, int,
                           hipStream_t) { return 0; }
int smoe_launch_permute(const smoe_layer*, const void*, const int32_t*, int, void*, int32_t*, int32_t*, int32_t*, hipStream_t) { return 0; }
int smoe_static_max_tokens() { return 65536; }
int smoe_launch_permute_static(const smoe_config&, const void*, const int32_t*, int, void*, int32_t*, int32_t*, int32_t*,
                               hipStream_t) { return 0; }
int smoe_launch_ffn_f32(const smoe_layer*, const float*, const int32_t*, int, float*, hipStream_t) { return 0; }
int smoe_launch_ffn_bf16(const smoe_layer*, const uint16_t*, const int32_t*, int, uint16_t*, hipStream_t) { return 0; }
int smoe_describe_ffn_bf16(const smoe_layer*, int, int, char* out, size_t n) { snprintf(out, n, "stub | stub"); return 0; }
int smoe_launch_combine(const smoe_layer*, const void*, const int32_t*, const float*, const void*, int, void*, hipStream_t) { return 0; }
int smoe_launch_pack_slot(const smoe_layer*, int, const void*, const void*, hipStream_t, int, int, int, int*) { return 0; }
int smoe_launch_set_map(const smoe_layer*, int, int, int, int, hipStream_t) { return 0; }
int smoe_launch_expert_norm(const smoe_layer*, const void*, const void*, int, float*, hipStream_t) { return 0; }
int smoe_launch_clear_maps(const smoe_layer*, hipStream_t) { return 0; }
int smoe_launch_split_router(const smoe_layer*, hipStream_t) { return 0; }
int smoe_launch_stream_read(const smoe_layer*, int, hipStream_t) { return 0; }
int smoe_launch_update_on_device(const smoe_layer*, const float*, const void*, const void*, hipStream_t) { return 0; }

#define EXPECT(call, want) do { int rc_ = (call); if (rc_ != (want)) { printf("line %d: got %d, want %d (%s)\n", __LINE__, rc_, (int)(want), smoe_last_error()); return 1; } } while (0)

int main() {
    void* fake = (void*)0x10000;
    smoe_layer_t* h = nullptr;
    smoe_config ok{8, 3, 64, 256, 128, SMOE_BF16, SMOE_GATE_FULL, 1};
    for (int bad = 0; bad < 7; ++bad) {
        smoe_config c = ok;
        if (bad == 0) c.E = 0; if (bad == 1) c.K = 9; if (bad == 2) c.d_model = 48; if (bad == 3) c.dtype = 5;
        if (bad == 4) c.gate_mode = 3; if (bad == 5) c.spare_slots = 9; if (bad == 6) c.max_tokens = 0;
        EXPECT(smoe_create(&c, &h), SMOE_EINVAL);
    }
    EXPECT(smoe_create(&ok, &h), SMOE_OK);
    if (smoe_workspace_bytes(h) == 0 || smoe_slot_weight_bytes(h) != (size_t)4 * 64 * 256 * 2) return 2;
    EXPECT(smoe_route(h, fake, 4, (int32_t*)fake, (float*)fake, (int32_t*)fake, (float*)fake, (float*)fake, nullptr), SMOE_ESTATE);
    EXPECT(smoe_bind(h, nullptr, fake, fake, (float*)fake, fake), SMOE_EINVAL);
    EXPECT(smoe_bind(h, (float*)fake, (char*)fake + 64, fake, (float*)fake, fake), SMOE_EINVAL);
    EXPECT(smoe_bind(h, (float*)fake, fake, fake, (float*)fake, fake), SMOE_OK);
    EXPECT(smoe_set_resident(h, 3, 0, fake, fake, nullptr), SMOE_EINVAL);
    EXPECT(smoe_set_resident(h, 0, 8, fake, fake, nullptr), SMOE_EINVAL);
    EXPECT(smoe_set_resident(h, 0, 0, fake, fake, nullptr), SMOE_EINVAL);      // not GPU-readable memory: refused
    EXPECT(smoe_expert_norm(h, fake, fake, 2, (float*)fake, nullptr), SMOE_EINVAL);
    EXPECT(smoe_route(h, fake, 4, (int32_t*)fake, (float*)fake, (int32_t*)fake, (float*)fake, (float*)fake, nullptr), SMOE_ESTATE);
    EXPECT(smoe_permute(h, fake, (int32_t*)fake, 129, fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, nullptr), SMOE_EINVAL);
    EXPECT(smoe_permute(h, fake, (int32_t*)fake, 4, fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, nullptr), SMOE_OK);
    EXPECT(smoe_permute_static(h, fake, (int32_t*)fake, 4, fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, nullptr), SMOE_OK);
    EXPECT(smoe_importance(h, (int32_t*)fake, (float*)fake, (float*)fake, 4, (int32_t*)fake, (float*)fake, (float*)fake, 2, nullptr), SMOE_EINVAL);
    EXPECT(smoe_combine(h, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr), SMOE_OK);
    EXPECT(smoe_forward(h, fake, 4, nullptr, fake, 0, (int32_t*)fake, (float*)fake, (int32_t*)fake, (float*)fake, (float*)fake,
                        (int32_t*)fake, (float*)fake, (float*)fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, nullptr), SMOE_ESTATE);
    // maps and policies
    std::vector<int32_t> s2e(3), e2s(8), cs(3), ce(3), count = {5, 0, 9, 9, 1, 2, 0, 0};
    std::vector<float> score = {0.5f, 0.f, 2.f, 0.1f, 3.f, 0.2f, 0.f, 0.f}, en(8, 1.f), rank(8);
    EXPECT(smoe_get_maps(h, s2e.data(), e2s.data()), SMOE_OK);
    for (int policy = 0; policy < 3; ++policy) EXPECT(smoe_policy_scores(policy, 8, count.data(), score.data(), en.data(), rank.data()), SMOE_OK);
    EXPECT(smoe_policy_scores(3, 8, count.data(), score.data(), en.data(), rank.data()), SMOE_EINVAL);
    EXPECT(smoe_select_resident(h, score.data(), cs.data(), ce.data()), 3);
    std::vector<int32_t> oe = {3, 4, 5, 6, 6, 1};
    EXPECT(smoe_on_demand_plan(h, oe.data(), (int)oe.size(), cs.data(), ce.data()), 3);
    EXPECT(smoe_on_demand_plan(h, oe.data(), 0, cs.data(), ce.data()), 0);
    oe[0] = 99;
    EXPECT(smoe_on_demand_plan(h, oe.data(), (int)oe.size(), cs.data(), ce.data()), SMOE_EINVAL);
    EXPECT(smoe_update_begin(h, score.data()), SMOE_ESTATE);                   // slots are not filled
    EXPECT(smoe_update_on_device(h, (float*)fake, fake, fake, nullptr), SMOE_ESTATE);   // slots are not filled
    EXPECT(smoe_update_tick(h, fake, fake, nullptr, nullptr), SMOE_EINVAL);    // banks are not GPU-readable memory
    EXPECT(smoe_update_pending(h), 0);
    // offline profile
    smoe_memory_profile m;
    EXPECT(smoe_profile_memory(&ok, &m), SMOE_OK);
    if (m.resident_bytes != 4 * m.expert_bytes || m.bank_bytes != 8 * m.expert_bytes) return 3;
    float lat[5] = {40.f, 41.f, 43.f, 50.f, 80.f}, us = 0.f;
    EXPECT(smoe_period_inflection(lat, 5, 0.1f), 2);
    EXPECT(smoe_period_inflection(lat, 0, 0.1f), SMOE_EINVAL);
    EXPECT(smoe_profile_end(h, nullptr, &us), SMOE_ESTATE);
    char buf[128];
    EXPECT(smoe_describe_ffn(h, 4, 1, buf, sizeof buf), SMOE_OK);
    EXPECT(smoe_profile_stream_read(h, 2, nullptr), SMOE_EINVAL);
    EXPECT(smoe_profile_stream_read(h, 1, nullptr), SMOE_OK);
    EXPECT(smoe_destroy(h), SMOE_OK);
    EXPECT(smoe_destroy(nullptr), SMOE_EINVAL);
    printf("ok\n");
    return 0;
}
