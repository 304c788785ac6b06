// Host side of the scheduling policies that SwapMoE's evaluation compares
// (Section 4.1 baselines, Section 4.5 ablation) and of the offline profile
// (Section 3.3, Appendix A.1): which numbers rank the experts at an update,
// the load-on-miss baseline, the memory model, an event bracket that measures
// the latency side, and the search for the update period (Section 3.4.1).
// No kernel lives here; everything works on host arrays and the handle.

#include <algorithm>
#include <cstdio>
#include <numeric>

#include "smoe_internal.h"
#include "swapmoe_profile.h"

extern "C" {

int smoe_policy_scores(int policy, int E, const int32_t* count, const float* score, const float* expert_norm,
                       float* rank) {
    if (E < 1 || !rank) return smoe_fail(SMOE_EINVAL, "smoe_policy_scores: bad E or null output");
    const void* src = policy == SMOE_POLICY_IMPORTANCE ? (const void*)score
                    : policy == SMOE_POLICY_COUNT ? (const void*)count
                    : policy == SMOE_POLICY_MAGNITUDE ? (const void*)expert_norm : nullptr;
    if (policy < SMOE_POLICY_IMPORTANCE || policy > SMOE_POLICY_MAGNITUDE)
        return smoe_fail(SMOE_EINVAL, "smoe_policy_scores: unknown policy %d", policy);
    if (!src) return smoe_fail(SMOE_EINVAL, "smoe_policy_scores: the array policy %d ranks by is null", policy);
    for (int e = 0; e < E; ++e)
        rank[e] = policy == SMOE_POLICY_COUNT ? (float)count[e] : policy == SMOE_POLICY_IMPORTANCE ? score[e] : expert_norm[e];
    return SMOE_OK;
}

int smoe_on_demand_plan(smoe_layer_t* L, const int32_t* orig_expert, int T, int32_t* changed_slots,
                        int32_t* changed_experts) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_on_demand_plan: null handle");
    const int E = L->cfg.E, K = L->cfg.K;
    if (T < 0 || (T > 0 && !orig_expert) || !changed_slots || !changed_experts)
        return smoe_fail(SMOE_EINVAL, "smoe_on_demand_plan: bad T or null argument");
    if (int rc = smoe_refresh_maps(L)) return rc;
    // host maps only: an empty slot has never been used and is the first to be filled
    if ((int)L->last_use.size() != K) L->last_use.assign(K, 0);
    const int64_t now = ++L->use_clock;
    std::vector<int> wanted(E, 0);
    for (int t = 0; t < T; ++t) {
        const int e = orig_expert[t];
        if (e < 0 || e >= E) return smoe_fail(SMOE_EINVAL, "smoe_on_demand_plan: orig_expert[%d] = %d outside [0,%d)", t, e, E);
        const int s = L->expert_to_slot[e];
        if (s >= 0) L->last_use[s] = now;           // a hit: the slot was used by this batch
        else wanted[e] += 1;                         // a miss: the expert was asked for and is not there
    }
    std::vector<int> missed, victims;
    for (int e = 0; e < E; ++e) if (wanted[e]) missed.push_back(e);
    std::stable_sort(missed.begin(), missed.end(), [&](int a, int b) { return wanted[a] > wanted[b]; });
    for (int s = 0; s < K; ++s) if (L->last_use[s] < now) victims.push_back(s);
    std::stable_sort(victims.begin(), victims.end(), [&](int a, int b) { return L->last_use[a] < L->last_use[b]; });
    const int n = (int)std::min(missed.size(), victims.size());
    for (int i = 0; i < n; ++i) {
        changed_slots[i] = victims[i];
        changed_experts[i] = missed[i];
        L->last_use[victims[i]] = now;               // what has just been loaded counts as used now
    }
    return n;
}

int smoe_profile_memory(const smoe_config* cfg, smoe_memory_profile* out) {
    if (!cfg || !out) return smoe_fail(SMOE_EINVAL, "smoe_profile_memory: null argument");
    smoe_layer_t* tmp = nullptr;
    int rc = smoe_create(cfg, &tmp);                 // validates the shape
    if (rc) return rc;
    const smoe_config& c = *cfg;
    out->expert_bytes = (uint64_t)2 * c.d_model * c.d_ff * smoe_elem_size(c.dtype);
    out->resident_bytes = (uint64_t)(c.K + c.spare_slots) * out->expert_bytes;
    out->workspace_bytes = smoe_workspace_bytes(tmp);
    out->bank_bytes = (uint64_t)c.E * out->expert_bytes;
    out->router_bytes = (uint64_t)c.E * c.d_model * 4;
    smoe_destroy(tmp);
    return SMOE_OK;
}

int smoe_profile_begin(smoe_layer_t* L, void* stream) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_profile_begin: null handle");
    for (int i = 0; i < 2; ++i)
        if (!L->bracket[i]) {
            int rc = smoe_check_hip(hipEventCreate(&L->bracket[i]), "smoe_profile_begin: event");
            if (rc) return rc;
        }
    L->bracket_open = true;
    return smoe_check_hip(hipEventRecord(L->bracket[0], (hipStream_t)stream), "smoe_profile_begin: record");
}

int smoe_profile_stream_read(smoe_layer_t* L, int which, void* stream) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_profile_stream_read: null handle");
    if (which != 0 && which != 1) return smoe_fail(SMOE_EINVAL, "smoe_profile_stream_read: which=%d is neither 0 nor 1", which);
    if (!L->workspace) return smoe_fail(SMOE_ESTATE, "smoe_profile_stream_read: smoe_bind has not been called");
    return smoe_launch_stream_read(L, which, (hipStream_t)stream);
}

int smoe_profile_end(smoe_layer_t* L, void* stream, float* elapsed_us) {
    if (!L || !elapsed_us) return smoe_fail(SMOE_EINVAL, "smoe_profile_end: null argument");
    if (!L->bracket_open) return smoe_fail(SMOE_ESTATE, "smoe_profile_end: no smoe_profile_begin before it");
    L->bracket_open = false;
    int rc = smoe_check_hip(hipEventRecord(L->bracket[1], (hipStream_t)stream), "smoe_profile_end: record");
    if (!rc) rc = smoe_check_hip(hipEventSynchronize(L->bracket[1]), "smoe_profile_end: wait");
    float ms = 0.f;
    if (!rc) rc = smoe_check_hip(hipEventElapsedTime(&ms, L->bracket[0], L->bracket[1]), "smoe_profile_end: elapsed");
    if (rc) return rc;
    *elapsed_us = ms * 1000.f;
    return SMOE_OK;
}

int smoe_describe_ffn(const smoe_layer_t* L, int T, int fused, char* out, size_t n) {
    if (!L || !out || n == 0) return smoe_fail(SMOE_EINVAL, "smoe_describe_ffn: null argument");
    if (T < 1 || T > L->cfg.max_tokens) return smoe_fail(SMOE_EINVAL, "smoe_describe_ffn: T=%d outside [1,%d]", T, L->cfg.max_tokens);
    if (L->cfg.dtype != SMOE_BF16) { snprintf(out, n, "ffn_f32_kernel | ffn_f32_kernel"); return SMOE_OK; }
    return smoe_describe_ffn_bf16(L, T, fused, out, n);
}

int smoe_period_inflection(const float* latency_us, int n, float tolerance) {
    if (!latency_us || n < 1) return smoe_fail(SMOE_EINVAL, "smoe_period_inflection: empty sweep");
    if (!(tolerance >= 0.f)) return smoe_fail(SMOE_EINVAL, "smoe_period_inflection: negative tolerance");
    float floor_us = latency_us[0];
    for (int i = 1; i < n; ++i) {
        if (latency_us[i] > (1.f + tolerance) * floor_us) return i - 1;   // the last point of the flat part
        floor_us = std::min(floor_us, latency_us[i]);
    }
    return n - 1;
}

}  // extern "C"
