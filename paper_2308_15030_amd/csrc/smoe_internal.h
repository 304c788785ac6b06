// Internal declarations shared by the translation units of libswapmoe.
// Nothing here is part of the C ABI (see include/swapmoe.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>

#include "swapmoe.h"

// Tokens handled by one workgroup of the sort kernels (histogram + ranking).
constexpr int SMOE_SORT_BLOCK = 1024;
// Upper bound on d_ff tiles / token tiles is derived from the config at bind time.

struct smoe_layer {
    smoe_config cfg;
    bool bound = false;
    int slots_set = 0;                       // number of slots that hold an expert
    std::vector<int32_t> slot_to_expert;     // host copies of the maps
    std::vector<int32_t> expert_to_slot;
    std::vector<int32_t> phys;               // virtual slot -> physical weight slot (host copy)
    std::vector<int32_t> free_phys;          // physical slots no virtual slot maps to

    // asynchronous update: the plan, and one record per load in flight
    struct Staged {
        int slot = -1, expert = -1, phys = -1, stage = -1;
        hipEvent_t done = nullptr;           // recorded on the load stream after the pack
    };
    std::vector<std::pair<int, int>> plan;   // (slot, expert) changes not started yet, in order
    std::vector<Staged> staged;              // loads in flight
    std::vector<hipEvent_t> event_pool;      // spare events, owned by the handle
    std::vector<int> free_stage;             // staging areas (one per spare slot) not in use
    char* d_stage = nullptr;                 // [spare_slots][2 matrices], bank layout: landing area of host-bank copies
    std::vector<hipEvent_t> released;        // per physical slot: compute-stream event after which it may be overwritten
    const void* bank_seen[2] = {nullptr, nullptr};   // banks smoe_update_tick has validated
    bool bank_is_host = false;               // ... and whether they are pinned host memory
    int ffn_variant[2] = {-1, -1};           // SMOE_FFN_VARIANT read at smoe_create (tuning aid); -1: built-in choice

    // caller-owned device buffers
    const float* router_w = nullptr;
    void* slot_w1 = nullptr;
    void* slot_w2 = nullptr;
    const float* expert_norm = nullptr;
    char* workspace = nullptr;

    // carved out of the workspace (device)
    int32_t* d_expert_to_slot = nullptr;     // [E]
    int32_t* d_slot_to_expert = nullptr;     // [K]
    int32_t* d_phys = nullptr;               // [K] physical weight slot of each virtual slot
    int32_t* d_plan = nullptr;               // [1 + 2K] smoe_update_on_device: number of loads, their slots, their experts
    int32_t* d_sort_hist = nullptr;          // [sort blocks, K]
    int32_t* d_hist32 = nullptr;             // fused path: [ceil(max_tokens/32), K] from the router
    void* d_hidden = nullptr;                // [max_tokens, d_ff] activations of the FFN
    float* d_partial = nullptr;              // small-T FFN: split partial sums
    float* d_norm_partial = nullptr;         // smoe_expert_norm: [E][64] partial sums of squares
    bool ws_ready = false;                   // device maps and counters initialised since the bind
    // smoe_update_on_device changes the device maps without the host: the host copies are then
    // stale until a call that needs them has fetched the device's (after waiting for that stream)
    bool maps_stale = false;
    hipStream_t maps_stream = nullptr;
    const void* dev_update_seen[3] = {nullptr, nullptr, nullptr};   // pointers smoe_update_on_device has checked
    void* d_router_split = nullptr;          // bf16 path: router weights split in three, MFMA order
    bool router_split_done = false;          // made by the first smoe_route after a bind

    hipEvent_t prof_ev[4] = {nullptr, nullptr, nullptr, nullptr};   // one-shot FFN profiling events
    hipEvent_t bracket[2] = {nullptr, nullptr};                     // smoe_profile_begin / _end
    bool bracket_open = false;

    // load-on-miss baseline: when each slot's expert was last some token's own choice
    std::vector<int64_t> last_use;
    int64_t use_clock = 0;
};

struct smoe_ws_layout {
    size_t e2s, s2e, phys, dplan, hist, hist32, hidden, partial, rsplit, norm, stage, total;
};
smoe_ws_layout smoe_ws_plan(const smoe_config& c);

int smoe_fail(int code, const char* fmt, ...);
int smoe_check_hip(hipError_t e, const char* what);

inline size_t smoe_elem_size(int dtype) { return dtype == SMOE_BF16 ? 2 : 4; }
inline int smoe_sort_blocks(int T) { return (T + SMOE_SORT_BLOCK - 1) / SMOE_SORT_BLOCK; }

// Kernel launchers, one per translation unit.  All validate nothing: the ABI
// layer has done that.  Each returns a smoe_status.
// hist32 (nullable): tokens per slot for every block of 32 tokens, [ceil(T/32)][K]
int smoe_launch_route(const smoe_layer* L, const void* x, int T, int32_t* orig_expert,
                      float* orig_gate, int32_t* slot, float* gate, float* xnorm, int32_t* hist32,
                      hipStream_t s);
int smoe_launch_route_rank_small(const smoe_layer* L, const void* x, int T, int32_t* orig_expert,
                                 float* orig_gate, int32_t* slot, float* gate, float* xnorm, int32_t* count,
                                 float* gsum, float* score, int accumulate, int32_t* perm, int32_t* inv_perm,
                                 int32_t* offsets, hipStream_t s);
bool smoe_decode_first_applies(const smoe_layer* L, int T);
int smoe_launch_decode_first(const smoe_layer* L, const void* x, int T, int32_t* orig_expert, float* orig_gate,
                             int32_t* slot, float* gate, float* xnorm, int32_t* count, float* gsum, float* score,
                             int accumulate, int32_t* perm, int32_t* inv_perm, int32_t* offsets, hipStream_t s,
                             hipEvent_t e0, hipEvent_t e1);
// true when the FFN of a T-token batch takes the one-tile-per-slot kernels (no sorted tiles)
// True when the expert slots of all layers alive in this process (both matrices, spare slots
// included) exceed what the 256 MB Infinity Cache can hold between two steps: the decode
// kernels then mark their weight loads non-temporal.  Measured with 16 slots of 768 x 3072:
// one layer (151 MB, stays cached from step to step) is 15 % slower with such loads, six
// layers (906 MB, never cached) are 7 % faster.
bool smoe_weights_outgrow_cache();
// plain read of the first K slots of slot_w1 (which = 0) or slot_w2 (1): see smoe_profile_stream_read
int smoe_launch_stream_read(const smoe_layer* L, int which, hipStream_t s);
bool smoe_ffn_dense_path(const smoe_layer* L, int T);
int smoe_launch_ffn_bf16_dense_second(const smoe_layer* L, const int32_t* slot_of, const float* gate,
                                      const uint16_t* residual, int T, uint16_t* out, hipStream_t s);
int smoe_launch_rank_importance(const smoe_layer* L, const int32_t* orig_expert, const float* orig_gate,
                                const float* xnorm, const int32_t* slot, int T, int32_t* count, float* gsum,
                                float* score, int accumulate, int32_t* perm, int32_t* inv_perm,
                                int32_t* offsets, hipStream_t s);
int smoe_launch_ffn_bf16_fused(const smoe_layer* L, const uint16_t* x, const int32_t* slot_of,
                               const int32_t* perm, const int32_t* offsets, const float* gate,
                               const uint16_t* residual, int T, uint16_t* out, hipStream_t s);
int smoe_launch_importance(const smoe_layer* L, const int32_t* orig_expert, const float* orig_gate,
                           const float* xnorm, int T, int32_t* count, float* gsum, float* score,
                           int accumulate, hipStream_t s);
int smoe_launch_permute(const smoe_layer* L, const void* x, const int32_t* slot, int T, void* x_perm,
                        int32_t* perm, int32_t* inv_perm, int32_t* offsets, hipStream_t s);
// smoe_permute without a workspace: block histograms in the library's own fixed device array
int smoe_static_max_tokens();
int smoe_launch_permute_static(const smoe_config& c, const void* x, const int32_t* slot, int T, void* x_perm,
                               int32_t* perm, int32_t* inv_perm, int32_t* offsets, hipStream_t s);
int smoe_launch_ffn_f32(const smoe_layer* L, const float* x_perm, const int32_t* offsets, int T,
                        float* y_perm, hipStream_t s);
int smoe_launch_ffn_bf16(const smoe_layer* L, const uint16_t* x_perm, const int32_t* offsets, int T,
                         uint16_t* y_perm, hipStream_t s);
int smoe_describe_ffn_bf16(const smoe_layer* L, int T, int fused, char* out, size_t n);
int smoe_launch_combine(const smoe_layer* L, const void* y_perm, const int32_t* inv_perm,
                        const float* gate, const void* residual, int T, void* out, hipStream_t s);
// packs / copies one expert's two matrices into physical slot `phys`
int smoe_launch_pack_slot(const smoe_layer* L, int slot, const void* w1_src, const void* w2_src, hipStream_t s,
                          int map_slot = -1, int expert = -1, int old_expert = -1, int* map_done = nullptr);
// slot now serves `expert` from physical slot `phys` (old_expert, if any, leaves the maps)
int smoe_launch_set_map(const smoe_layer* L, int slot, int expert, int old_expert, int phys, hipStream_t s);
int smoe_launch_expert_norm(const smoe_layer* L, const void* w1, const void* w2, int n, float* out,
                            hipStream_t s);
int smoe_launch_clear_maps(const smoe_layer* L, hipStream_t s);
// update rule on the device from score [E] (device), then the planned loads from a device-readable bank
int smoe_launch_update_on_device(const smoe_layer* L, const float* score, const void* bank_w1, const void* bank_w2,
                                 hipStream_t s);
// brings the host copies of the maps up to date after smoe_update_on_device (waits for its stream)
int smoe_refresh_maps(smoe_layer* L);
int smoe_launch_split_router(const smoe_layer* L, hipStream_t s);

// Kernel launch that, when a pair of events is given, attaches them to the
// dispatch itself (start and end of the kernel's execution).
template <typename K, typename... Args>
inline void smoe_launch_timed(K kernel, dim3 grid, dim3 block, hipStream_t s, hipEvent_t e0, hipEvent_t e1,
                              Args... args) {
    if (e0 && e1) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, e0, e1, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
}

// bf16 <-> fp32 on the device.  Widening is exact; narrowing rounds to
// nearest, ties to even (inputs are finite by contract).
// 16-byte load of data that is read once per launch (the decode path's weight streams): marked
// non-temporal, so the caches do not keep it at the expense of data that is read again.
__device__ __forceinline__ uint4 smoe_load_stream(const uint4* p) {
    typedef unsigned int smoe_u32x4 __attribute__((ext_vector_type(4)));
    const smoe_u32x4 v = __builtin_nontemporal_load((const smoe_u32x4*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ float smoe_bf16_to_f32(uint16_t b) {
    return __uint_as_float((uint32_t)b << 16);
}
__device__ __forceinline__ uint16_t smoe_f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
