// C ABI of libswapmoe: handle life cycle, argument validation, the host side
// of the slot<->expert maps (the Virtual-Expert bookkeeping of SwapMoE,
// abstract and Section 3.2) and the update policy.  No kernel lives here.

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <atomic>
#include <new>
#include <numeric>

#include "smoe_internal.h"
#include "swapmoe_profile.h"

namespace {
thread_local char g_err[512] = "";

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

hipStream_t as_stream(void* s) { return (hipStream_t)s; }

bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }

// A weight source or bank is read by a kernel (or by the copy engines): it must be memory the
// GPU can reach -- a device allocation, managed memory or pinned host memory.  A pageable host
// pointer (malloc, a numpy array) would fault on the GPU, so it is turned away here, before
// any launch.  *is_host (optional) tells pinned host memory from the rest.
int check_gpu_readable(const void* p, const char* who, const char* what, bool* is_host = nullptr) {
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();                   // the failed query must not surface in a later call
        return smoe_fail(SMOE_EINVAL, "%s: %s is not device, managed or pinned host memory (%s)", who, what,
                         hipGetErrorString(e));
    }
    if (at.type != hipMemoryTypeDevice && at.type != hipMemoryTypeHost && at.type != hipMemoryTypeManaged)
        return smoe_fail(SMOE_EINVAL, "%s: %s is not device, managed or pinned host memory", who, what);
    if (is_host) *is_host = at.type == hipMemoryTypeHost;
    return SMOE_OK;
}
}  // namespace

int smoe_fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int smoe_check_hip(hipError_t e, const char* what) {
    if (e == hipSuccess) return SMOE_OK;
    return smoe_fail(SMOE_EHIP, "%s: %s", what, hipGetErrorString(e));
}

smoe_ws_layout smoe_ws_plan(const smoe_config& c) {
    smoe_ws_layout w{};
    size_t off = 0;
    w.e2s = off;     off = align_up(off + (size_t)c.E * 4, 256);
    w.s2e = off;     off = align_up(off + (size_t)c.K * 4, 256);
    w.phys = off;    off = align_up(off + (size_t)c.K * 4, 256);
    w.dplan = off;   off = align_up(off + (size_t)(1 + 2 * c.K) * 4, 256);
    w.hist = off;    off = align_up(off + (size_t)smoe_sort_blocks(c.max_tokens) * c.K * 4, 256);
    w.hist32 = off;  off = align_up(off + (size_t)((c.max_tokens + 31) / 32) * c.K * 4, 256);
    // hidden activations: every segment is re-based to a multiple of 32 rows
    w.hidden = off;  off = align_up(off + ((size_t)c.max_tokens + 32 * (size_t)c.K) * c.d_ff * smoe_elem_size(c.dtype), 256);
    w.partial = off; off = align_up(off, 256);
    // bf16 path: three bf16 pieces of every router weight, experts padded to a multiple of 32
    w.rsplit = off;
    if (c.dtype == SMOE_BF16) off = align_up(off + (size_t)((c.E + 31) / 32 * 32) * c.d_model * 2 * 3, 256);
    w.norm = off;    off = align_up(off + (size_t)c.E * 64 * 4, 256);      // smoe_expert_norm partial sums
    // asynchronous loads from a host bank land here (copy engine) before they are packed into a slot
    w.stage = off;   off = align_up(off + (size_t)c.spare_slots * 2 * c.d_model * c.d_ff * smoe_elem_size(c.dtype), 256);
    w.total = off;
    return w;
}

// slot bytes of every live layer (see smoe_weights_outgrow_cache)
static std::atomic<long long> g_live_slot_bytes{0};
static long long layer_slot_bytes(const smoe_config& c) {
    return 2ll * (c.K + c.spare_slots) * c.d_model * c.d_ff * (long long)smoe_elem_size(c.dtype);
}

bool smoe_weights_outgrow_cache() {
    constexpr long long kCacheable = 192ll << 20;          // three quarters of the 256 MB Infinity Cache
    return g_live_slot_bytes.load(std::memory_order_relaxed) > kCacheable;
}

int smoe_refresh_maps(smoe_layer* L) {
    if (!L->maps_stale) return SMOE_OK;
    // the stream the update ran on may be gone by now: then the whole device is waited for
    hipError_t e = hipStreamSynchronize(L->maps_stream);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        e = hipDeviceSynchronize();
    }
    int rc = smoe_check_hip(e, "maps: wait for the device-side update");
    if (!rc) rc = smoe_check_hip(hipMemcpy(L->slot_to_expert.data(), L->d_slot_to_expert, (size_t)L->cfg.K * 4, hipMemcpyDeviceToHost),
                                 "maps: read-back");
    if (!rc) rc = smoe_check_hip(hipMemcpy(L->expert_to_slot.data(), L->d_expert_to_slot, (size_t)L->cfg.E * 4, hipMemcpyDeviceToHost),
                                 "maps: read-back");
    if (rc) return rc;
    L->maps_stale = false;
    return SMOE_OK;
}

extern "C" {

const char* smoe_last_error(void) { return g_err; }

int smoe_create(const smoe_config* cfg, smoe_layer_t** out) {
    if (out) *out = nullptr;
    if (!cfg || !out) return smoe_fail(SMOE_EINVAL, "smoe_create: null argument");
    const smoe_config& c = *cfg;
    if (c.E < 1 || c.E > 256) return smoe_fail(SMOE_EINVAL, "smoe_create: E=%d outside [1,256]", c.E);
    if (c.K < 1 || c.K > c.E)
        return smoe_fail(SMOE_EINVAL, "smoe_create: K=%d outside [1,E]", c.K);
    if (c.d_model < 1 || c.d_ff < 1 || c.d_model > (1 << 16) || c.d_ff > (1 << 18))
        return smoe_fail(SMOE_EINVAL, "smoe_create: d_model=%d d_ff=%d out of range", c.d_model, c.d_ff);
    if (c.max_tokens < 1 || c.max_tokens > (1 << 24))
        return smoe_fail(SMOE_EINVAL, "smoe_create: max_tokens=%d outside [1,2^24]", c.max_tokens);
    if (c.dtype != SMOE_F32 && c.dtype != SMOE_BF16)
        return smoe_fail(SMOE_EINVAL, "smoe_create: unknown dtype %d", c.dtype);
    if (c.gate_mode != SMOE_GATE_FULL && c.gate_mode != SMOE_GATE_RENORM)
        return smoe_fail(SMOE_EINVAL, "smoe_create: unknown gate_mode %d", c.gate_mode);
    if (c.spare_slots < 0 || c.spare_slots > 8)
        return smoe_fail(SMOE_EINVAL, "smoe_create: spare_slots=%d outside [0,8]", c.spare_slots);
    if (c.dtype == SMOE_BF16 && (c.d_model % 32 || c.d_ff % 32))
        return smoe_fail(SMOE_EINVAL, "smoe_create: bf16 needs d_model and d_ff to be multiples of 32");
    if (c.dtype == SMOE_F32 && (c.d_model % 4 || c.d_ff % 4))
        return smoe_fail(SMOE_EINVAL, "smoe_create: fp32 needs d_model and d_ff to be multiples of 4");
    smoe_layer* L = new (std::nothrow) smoe_layer();
    if (!L) return smoe_fail(SMOE_ENOMEM, "smoe_create: out of host memory");
    L->cfg = c;
    L->slot_to_expert.assign(c.K, -1);
    L->expert_to_slot.assign(c.E, -1);
    // tuning aid, read once here and never on a hot call: SMOE_FFN_VARIANT="v1,v2" fixes the tile
    // shapes of the two FFN products (indices checked by the launcher; anything else is ignored)
    if (const char* env = getenv("SMOE_FFN_VARIANT")) {
        int a = -1, b = -1;
        if (sscanf(env, "%d,%d", &a, &b) == 2 && a >= 0 && b >= 0) { L->ffn_variant[0] = a; L->ffn_variant[1] = b; }
    }
    g_live_slot_bytes += layer_slot_bytes(c);
    *out = L;
    return SMOE_OK;
}

int smoe_destroy(smoe_layer_t* layer) {
    if (!layer) return smoe_fail(SMOE_EINVAL, "smoe_destroy: null handle");
    g_live_slot_bytes -= layer_slot_bytes(layer->cfg);
    for (auto& st : layer->staged) if (st.done) (void)hipEventDestroy(st.done);
    for (hipEvent_t e : layer->event_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : layer->released) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : layer->bracket) if (e) (void)hipEventDestroy(e);
    delete layer;
    return SMOE_OK;
}

size_t smoe_workspace_bytes(const smoe_layer_t* layer) {
    return layer ? smoe_ws_plan(layer->cfg).total : 0;
}

size_t smoe_slot_weight_bytes(const smoe_layer_t* layer) {
    if (!layer) return 0;
    const smoe_config& c = layer->cfg;
    return (size_t)(c.K + c.spare_slots) * c.d_model * c.d_ff * smoe_elem_size(c.dtype);
}

int smoe_bind(smoe_layer_t* L, const float* router_w, void* slot_w1, void* slot_w2,
              const float* expert_norm, void* workspace) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_bind: null handle");
    if (!router_w || !slot_w1 || !slot_w2 || !expert_norm || !workspace)
        return smoe_fail(SMOE_EINVAL, "smoe_bind: null buffer");
    if (misaligned(slot_w1, 256) || misaligned(slot_w2, 256) || misaligned(workspace, 256))
        return smoe_fail(SMOE_EINVAL, "smoe_bind: slot arrays and workspace must be 256-byte aligned");
    if (misaligned(router_w, 16))
        return smoe_fail(SMOE_EINVAL, "smoe_bind: router_w must be 16-byte aligned");
    if (misaligned(expert_norm, 4))
        return smoe_fail(SMOE_EINVAL, "smoe_bind: expert_norm must be 4-byte aligned");
    smoe_ws_layout w = smoe_ws_plan(L->cfg);
    L->router_w = router_w;
    L->slot_w1 = slot_w1;
    L->slot_w2 = slot_w2;
    L->expert_norm = expert_norm;
    L->workspace = (char*)workspace;
    L->d_expert_to_slot = (int32_t*)(L->workspace + w.e2s);
    L->d_slot_to_expert = (int32_t*)(L->workspace + w.s2e);
    L->d_phys = (int32_t*)(L->workspace + w.phys);
    L->d_plan = (int32_t*)(L->workspace + w.dplan);
    L->maps_stale = false;
    L->d_stage = L->workspace + w.stage;
    L->d_sort_hist = (int32_t*)(L->workspace + w.hist);
    L->d_hist32 = (int32_t*)(L->workspace + w.hist32);
    L->d_hidden = L->workspace + w.hidden;
    L->d_partial = (float*)(L->workspace + w.partial);
    L->d_router_split = L->workspace + w.rsplit;
    L->router_split_done = false;
    L->ws_ready = false;
    L->d_norm_partial = (float*)(L->workspace + w.norm);
    std::fill(L->slot_to_expert.begin(), L->slot_to_expert.end(), -1);
    std::fill(L->expert_to_slot.begin(), L->expert_to_slot.end(), -1);
    L->phys.resize(L->cfg.K);
    std::iota(L->phys.begin(), L->phys.end(), 0);
    L->free_phys.clear();
    for (int p = L->cfg.K + L->cfg.spare_slots - 1; p >= L->cfg.K; --p) L->free_phys.push_back(p);
    L->free_stage.clear();
    for (int i = L->cfg.spare_slots - 1; i >= 0; --i) L->free_stage.push_back(i);
    L->plan.clear();
    L->bank_seen[0] = L->bank_seen[1] = nullptr;
    L->last_use.assign(L->cfg.K, 0);
    L->use_clock = 0;
    for (auto& st : L->staged) L->event_pool.push_back(st.done);   // loads of the old binding are forgotten
    L->staged.clear();
    L->slots_set = 0;
    L->bound = true;
    return SMOE_OK;
}

int smoe_get_maps(const smoe_layer_t* L, int32_t* slot_to_expert, int32_t* expert_to_slot) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_get_maps: null handle");
    if (int rc = smoe_refresh_maps(const_cast<smoe_layer*>(L))) return rc;
    if (slot_to_expert) std::memcpy(slot_to_expert, L->slot_to_expert.data(), (size_t)L->cfg.K * 4);
    if (expert_to_slot) std::memcpy(expert_to_slot, L->expert_to_slot.data(), (size_t)L->cfg.E * 4);
    return SMOE_OK;
}

int smoe_expert_norm(smoe_layer_t* L, const void* w1, const void* w2, int n, float* out, void* stream) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_expert_norm: null handle");
    if (n < 0 || n > L->cfg.E) return smoe_fail(SMOE_EINVAL, "smoe_expert_norm: n=%d outside [0,E]", n);
    if (n == 0) return SMOE_OK;
    if (!w1 || !w2 || !out) return smoe_fail(SMOE_EINVAL, "smoe_expert_norm: null buffer");
    if (misaligned(w1, 16) || misaligned(w2, 16))
        return smoe_fail(SMOE_EINVAL, "smoe_expert_norm: weights must be 16-byte aligned");
    if (!L->bound) return smoe_fail(SMOE_ESTATE, "smoe_expert_norm: call smoe_bind first");
    int rc = check_gpu_readable(w1, "smoe_expert_norm", "w1");
    if (!rc) rc = check_gpu_readable(w2, "smoe_expert_norm", "w2");
    if (rc) return rc;
    return smoe_launch_expert_norm(L, w1, w2, n, out, as_stream(stream));
}

// First stream work after a bind: the device maps and counters in the workspace
// are uninitialised memory until this has run.
static int ensure_workspace(smoe_layer* L, hipStream_t s) {
    if (L->ws_ready) return SMOE_OK;
    int rc = smoe_launch_clear_maps(L, s);
    if (rc) return rc;
    L->ws_ready = true;
    return SMOE_OK;
}

int smoe_set_resident(smoe_layer_t* L, int slot, int expert, const void* w1_src, const void* w2_src,
                      void* stream) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_set_resident: null handle");
    if (!L->bound) return smoe_fail(SMOE_ESTATE, "smoe_set_resident: call smoe_bind first");
    const smoe_config& c = L->cfg;
    if (slot < 0 || slot >= c.K) return smoe_fail(SMOE_EINVAL, "smoe_set_resident: slot %d outside [0,%d)", slot, c.K);
    if (expert < 0 || expert >= c.E)
        return smoe_fail(SMOE_EINVAL, "smoe_set_resident: expert %d outside [0,%d)", expert, c.E);
    if (!w1_src || !w2_src) return smoe_fail(SMOE_EINVAL, "smoe_set_resident: null weight source");
    if (misaligned(w1_src, 16) || misaligned(w2_src, 16))
        return smoe_fail(SMOE_EINVAL, "smoe_set_resident: weight sources must be 16-byte aligned");
    if (int rc = smoe_refresh_maps(L)) return rc;
    int cur = L->expert_to_slot[expert];
    if (cur >= 0 && cur != slot)
        return smoe_fail(SMOE_ESTATE, "smoe_set_resident: expert %d is already resident in slot %d", expert, cur);
    for (const auto& st : L->staged)
        if (st.slot == slot || st.expert == expert)
            return smoe_fail(SMOE_ESTATE, "smoe_set_resident: slot %d / expert %d has an asynchronous load in flight",
                             st.slot, st.expert);
    int rc0 = check_gpu_readable(w1_src, "smoe_set_resident", "w1_src");
    if (!rc0) rc0 = check_gpu_readable(w2_src, "smoe_set_resident", "w2_src");
    if (rc0) return rc0;
    hipStream_t s = as_stream(stream);
    rc0 = ensure_workspace(L, s);
    if (rc0) return rc0;
    int old = L->slot_to_expert[slot];
    int map_done = 0;
    int rc = smoe_launch_pack_slot(L, L->phys[slot], w1_src, w2_src, s, slot, expert, old, &map_done);
    if (rc) return rc;
    if (!map_done) {
        rc = smoe_launch_set_map(L, slot, expert, old, L->phys[slot], s);
        if (rc) return rc;
    }
    if (old >= 0) L->expert_to_slot[old] = -1; else L->slots_set += 1;
    L->slot_to_expert[slot] = expert;
    L->expert_to_slot[expert] = slot;
    return SMOE_OK;
}

// The update rule: the new resident set is the K best-scored experts (higher
// score first, lower id first among equals); experts that stay keep their slot;
// the freed slots, in ascending order, receive the newcomers in descending score.
// s2e / e2s are the maps the plan starts from.  Returns the number of changes, -1
// if the maps are inconsistent.
static int plan_changes(const smoe_config& c, const float* score, const std::vector<int32_t>& s2e,
                        const std::vector<int32_t>& e2s, int32_t* changed_slots, int32_t* changed_experts) {
    const int E = c.E, K = c.K;
    std::vector<int> rank(E);
    std::iota(rank.begin(), rank.end(), 0);
    std::sort(rank.begin(), rank.end(), [&](int a, int b) {
        return score[a] != score[b] ? score[a] > score[b] : a < b;
    });
    std::vector<char> wanted(E, 0);
    for (int i = 0; i < K; ++i) wanted[rank[i]] = 1;
    // walk the free slots upwards and the newcomers downwards in score
    int n = 0, ri = 0;
    for (int s = 0; s < K; ++s) {
        int cur = s2e[s];
        if (cur >= 0 && wanted[cur]) continue;
        while (ri < K && e2s[rank[ri]] >= 0) ++ri;
        if (ri >= K) return -1;
        changed_slots[n] = s;
        changed_experts[n] = rank[ri++];
        ++n;
    }
    return n;
}

int smoe_select_resident(const smoe_layer_t* L, const float* score, int32_t* changed_slots,
                         int32_t* changed_experts) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_select_resident: null handle");
    if (!score || !changed_slots || !changed_experts)
        return smoe_fail(SMOE_EINVAL, "smoe_select_resident: null argument");
    if (int rc = smoe_refresh_maps(const_cast<smoe_layer*>(L))) return rc;
    int n = plan_changes(L->cfg, score, L->slot_to_expert, L->expert_to_slot, changed_slots, changed_experts);
    if (n < 0) return smoe_fail(SMOE_ESTATE, "smoe_select_resident: inconsistent maps");
    return n;
}

// ---- update without the host ------------------------------------------------

int smoe_update_on_device(smoe_layer_t* L, const float* score, const void* bank_w1, const void* bank_w2, void* stream) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_update_on_device: null handle");
    if (!L->bound) return smoe_fail(SMOE_ESTATE, "smoe_update_on_device: call smoe_bind first");
    if (L->cfg.dtype != SMOE_BF16) return smoe_fail(SMOE_EINVAL, "smoe_update_on_device: bf16 layers only");
    if (!score || !bank_w1 || !bank_w2) return smoe_fail(SMOE_EINVAL, "smoe_update_on_device: null argument");
    if (misaligned(score, 4) || misaligned(bank_w1, 16) || misaligned(bank_w2, 16))
        return smoe_fail(SMOE_EINVAL, "smoe_update_on_device: score must be 4-byte, the banks 16-byte aligned");
    if (L->slots_set != L->cfg.K) return smoe_fail(SMOE_ESTATE, "smoe_update_on_device: not every slot holds an expert");
    if (!L->plan.empty() || !L->staged.empty())
        return smoe_fail(SMOE_ESTATE, "smoe_update_on_device: an asynchronous update is pending");
    // score and banks are read by kernels: checked once per triple of pointers
    if (score != L->dev_update_seen[0] || bank_w1 != L->dev_update_seen[1] || bank_w2 != L->dev_update_seen[2]) {
        int rc = check_gpu_readable(score, "smoe_update_on_device", "score");
        if (!rc) rc = check_gpu_readable(bank_w1, "smoe_update_on_device", "bank_w1");
        if (!rc) rc = check_gpu_readable(bank_w2, "smoe_update_on_device", "bank_w2");
        if (rc) return rc;
        L->dev_update_seen[0] = score; L->dev_update_seen[1] = bank_w1; L->dev_update_seen[2] = bank_w2;
    }
    hipStream_t s = as_stream(stream);
    int rc = ensure_workspace(L, s);
    if (rc) return rc;
    // The host copies must be current before the device changes the maps again only if somebody
    // reads them; they are marked stale and fetched on demand.
    rc = smoe_launch_update_on_device(L, score, bank_w1, bank_w2, s);
    if (rc) return rc;
    L->maps_stale = true;
    L->maps_stream = s;
    return SMOE_OK;
}

// ---- asynchronous, amortized update ----------------------------------------

int smoe_update_begin(smoe_layer_t* L, const float* score) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_update_begin: null handle");
    if (!L->bound) return smoe_fail(SMOE_ESTATE, "smoe_update_begin: call smoe_bind first");
    if (L->cfg.spare_slots < 1) return smoe_fail(SMOE_ESTATE, "smoe_update_begin: the layer has no spare slot");
    if (!score) return smoe_fail(SMOE_EINVAL, "smoe_update_begin: null score");
    if (L->slots_set != L->cfg.K) return smoe_fail(SMOE_ESTATE, "smoe_update_begin: not every slot holds an expert");
    if (int rc = smoe_refresh_maps(L)) return rc;
    // loads in flight count as done
    std::vector<int32_t> s2e = L->slot_to_expert, e2s = L->expert_to_slot;
    for (const auto& st : L->staged) {
        e2s[s2e[st.slot]] = -1;
        s2e[st.slot] = st.expert;
        e2s[st.expert] = st.slot;
    }
    std::vector<int32_t> cs(L->cfg.K), ce(L->cfg.K);
    int n = plan_changes(L->cfg, score, s2e, e2s, cs.data(), ce.data());
    if (n < 0) return smoe_fail(SMOE_ESTATE, "smoe_update_begin: inconsistent maps");
    // A slot whose load in flight is no longer wanted gets its new occupant after that load has
    // been committed: the entry stays in the plan and smoe_update_tick holds it back until then.
    L->plan.clear();
    for (int i = 0; i < n; ++i) L->plan.emplace_back(cs[i], ce[i]);
    return (int)L->plan.size();
}

int smoe_update_pending(const smoe_layer_t* L) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_update_pending: null handle");
    return (int)(L->plan.size() + L->staged.size());
}

int smoe_update_tick(smoe_layer_t* L, const void* bank_w1, const void* bank_w2, void* load_stream,
                     void* compute_stream) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_update_tick: null handle");
    if (!L->bound) return smoe_fail(SMOE_ESTATE, "smoe_update_tick: call smoe_bind first");
    if (L->cfg.spare_slots < 1) return smoe_fail(SMOE_ESTATE, "smoe_update_tick: the layer has no spare slot");
    if (!bank_w1 || !bank_w2) return smoe_fail(SMOE_EINVAL, "smoe_update_tick: null bank");
    if (misaligned(bank_w1, 16) || misaligned(bank_w2, 16))
        return smoe_fail(SMOE_EINVAL, "smoe_update_tick: banks must be 16-byte aligned");
    // the banks are read by a kernel or by the copy engines: checked once per pair of pointers
    if (bank_w1 != L->bank_seen[0] || bank_w2 != L->bank_seen[1]) {
        bool h1 = false, h2 = false;
        int rc = check_gpu_readable(bank_w1, "smoe_update_tick", "bank_w1", &h1);
        if (!rc) rc = check_gpu_readable(bank_w2, "smoe_update_tick", "bank_w2", &h2);
        if (rc) return rc;
        if (h1 != h2) return smoe_fail(SMOE_EINVAL, "smoe_update_tick: both banks must live in the same kind of memory");
        L->bank_seen[0] = bank_w1;
        L->bank_seen[1] = bank_w2;
        L->bank_is_host = h1;
    }
    hipStream_t ls = as_stream(load_stream), cs = as_stream(compute_stream);
    const smoe_config& c = L->cfg;
    if (L->released.empty()) L->released.assign(c.K + c.spare_slots, nullptr);
    int commits = 0;
    // (1) commit what has arrived
    for (size_t i = 0; i < L->staged.size();) {
        smoe_layer::Staged st = L->staged[i];
        hipError_t q = hipEventQuery(st.done);
        if (q == hipErrorNotReady) { ++i; continue; }
        if (q != hipSuccess) return smoe_check_hip(q, "smoe_update_tick: load event");
        // the load has completed, so work submitted from now on sees its writes: no stream wait needed
        int rc = SMOE_OK;
        const int old_expert = L->slot_to_expert[st.slot], old_phys = L->phys[st.slot];
        rc = smoe_launch_set_map(L, st.slot, st.expert, old_expert, st.phys, cs);
        if (rc) return rc;
        // work enqueued before this point may still read the physical slot that was just unmapped
        if (!L->released[old_phys]) {
            rc = smoe_check_hip(hipEventCreateWithFlags(&L->released[old_phys], hipEventDisableTiming),
                                "smoe_update_tick: event");
            if (rc) return rc;
        }
        rc = smoe_check_hip(hipEventRecord(L->released[old_phys], cs), "smoe_update_tick: release event");
        if (rc) return rc;
        L->expert_to_slot[old_expert] = -1;
        L->slot_to_expert[st.slot] = st.expert;
        L->expert_to_slot[st.expert] = st.slot;
        L->phys[st.slot] = st.phys;
        L->free_phys.push_back(old_phys);
        L->free_stage.push_back(st.stage);
        L->event_pool.push_back(st.done);
        L->staged.erase(L->staged.begin() + i);
        ++commits;
    }
    // (2) start the next loads
    const size_t per = (size_t)c.d_model * c.d_ff * smoe_elem_size(c.dtype);   // bytes per matrix
    // A bank in host memory is brought over by the copy engines into the staging area and packed from
    // there: a kernel that reads host memory directly fills every CU's memory pipeline with slow PCIe
    // reads and slows the forward pass it is meant to overlap with.
    // The plan is walked in order; a change whose slot still has a load in flight waits for that
    // load's commit (it stays in the plan) and the later changes go ahead of it.
    for (size_t pi = 0; pi < L->plan.size() && !L->free_phys.empty() && !L->free_stage.empty();) {
        const int slot = L->plan[pi].first, expert = L->plan[pi].second;
        bool busy = false;
        for (const auto& st : L->staged) busy |= st.slot == slot;
        if (busy) { ++pi; continue; }
        L->plan.erase(L->plan.begin() + pi);
        if (L->expert_to_slot[expert] >= 0) continue;          // became resident by another route
        smoe_layer::Staged st;
        st.slot = slot;
        st.expert = expert;
        st.phys = L->free_phys.back();
        st.stage = L->free_stage.back();
        if (!L->event_pool.empty()) {
            st.done = L->event_pool.back();
            L->event_pool.pop_back();
        } else {
            int rc = smoe_check_hip(hipEventCreateWithFlags(&st.done, hipEventDisableTiming), "smoe_update_tick: event");
            if (rc) return rc;
        }
        int rc = SMOE_OK;
        if (L->released[st.phys])
            rc = smoe_check_hip(hipStreamWaitEvent(ls, L->released[st.phys], 0), "smoe_update_tick: stream order");
        const char* src1 = (const char*)bank_w1 + (size_t)expert * per;
        const char* src2 = (const char*)bank_w2 + (size_t)expert * per;
        if (!rc && L->bank_is_host) {
            char* s1 = L->d_stage + (size_t)st.stage * 2 * per;
            rc = smoe_check_hip(hipMemcpyAsync(s1, src1, per, hipMemcpyHostToDevice, ls), "smoe_update_tick: copy");
            if (!rc) rc = smoe_check_hip(hipMemcpyAsync(s1 + per, src2, per, hipMemcpyHostToDevice, ls),
                                         "smoe_update_tick: copy");
            src1 = s1;
            src2 = s1 + per;
        }
        if (!rc) rc = smoe_launch_pack_slot(L, st.phys, src1, src2, ls);
        if (!rc) rc = smoe_check_hip(hipEventRecord(st.done, ls), "smoe_update_tick: load event");
        if (rc) {
            L->event_pool.push_back(st.done);
            return rc;
        }
        L->free_phys.pop_back();
        L->free_stage.pop_back();
        L->staged.push_back(st);
    }
    return commits;
}

// ---- the hot calls: validate, then hand over to the launchers -------------

static int check_hot(const smoe_layer* L, int T, const char* who, bool need_full) {
    if (!L) return smoe_fail(SMOE_EINVAL, "%s: null handle", who);
    if (!L->bound) return smoe_fail(SMOE_ESTATE, "%s: call smoe_bind first", who);
    if (T < 0 || T > L->cfg.max_tokens)
        return smoe_fail(SMOE_EINVAL, "%s: T=%d outside [0,%d]", who, T, L->cfg.max_tokens);
    if (need_full && L->slots_set != L->cfg.K)
        return smoe_fail(SMOE_ESTATE, "%s: only %d of %d slots hold an expert", who, L->slots_set, L->cfg.K);
    return SMOE_OK;
}

int smoe_route(smoe_layer_t* L, const void* x, int T, int32_t* orig_expert, float* orig_gate,
               int32_t* slot, float* gate, float* xnorm, void* stream) {
    int rc = check_hot(L, T, "smoe_route", true);
    if (rc) return rc;
    if (T == 0) return SMOE_OK;
    if (!x || !orig_expert || !orig_gate || !slot || !gate || !xnorm)
        return smoe_fail(SMOE_EINVAL, "smoe_route: null buffer");
    if (misaligned(x, 16)) return smoe_fail(SMOE_EINVAL, "smoe_route: x must be 16-byte aligned");
    if (L->cfg.dtype == SMOE_BF16 && !L->router_split_done) {
        rc = smoe_launch_split_router(L, as_stream(stream));
        if (rc) return rc;
        L->router_split_done = true;
    }
    return smoe_launch_route(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, nullptr, as_stream(stream));
}

int smoe_importance(smoe_layer_t* L, const int32_t* orig_expert, const float* orig_gate,
                    const float* xnorm, int T, int32_t* count, float* gsum, float* score,
                    int accumulate, void* stream) {
    int rc = check_hot(L, T, "smoe_importance", false);
    if (rc) return rc;
    if (accumulate != 0 && accumulate != 1)
        return smoe_fail(SMOE_EINVAL, "smoe_importance: accumulate must be 0 or 1");
    if (!count || !gsum || !score) return smoe_fail(SMOE_EINVAL, "smoe_importance: null output");
    if (T > 0 && (!orig_expert || !orig_gate || !xnorm))
        return smoe_fail(SMOE_EINVAL, "smoe_importance: null input");
    if (T == 0 && accumulate == 1) return SMOE_OK;
    return smoe_launch_importance(L, orig_expert, orig_gate, xnorm, T, count, gsum, score, accumulate,
                                  as_stream(stream));
}

int smoe_permute(smoe_layer_t* L, const void* x, const int32_t* slot, int T, void* x_perm,
                 int32_t* perm, int32_t* inv_perm, int32_t* offsets, void* stream) {
    int rc = check_hot(L, T, "smoe_permute", false);
    if (rc) return rc;
    if (!offsets) return smoe_fail(SMOE_EINVAL, "smoe_permute: null offsets");
    if (T > 0 && (!x || !slot || !x_perm || !perm || !inv_perm))
        return smoe_fail(SMOE_EINVAL, "smoe_permute: null buffer");
    if (T > 0 && (misaligned(x, 16) || misaligned(x_perm, 16)))
        return smoe_fail(SMOE_EINVAL, "smoe_permute: x and x_perm must be 16-byte aligned");
    return smoe_launch_permute(L, x, slot, T, x_perm, perm, inv_perm, offsets, as_stream(stream));
}

int smoe_permute_static(smoe_layer_t* L, const void* x, const int32_t* slot, int T, void* x_perm,
                        int32_t* perm, int32_t* inv_perm, int32_t* offsets, void* stream) {
    // needs the handle's shape only: no bound workspace, so an unbound handle is fine
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_permute_static: null handle");
    if (T < 0 || T > L->cfg.max_tokens)
        return smoe_fail(SMOE_EINVAL, "smoe_permute_static: T=%d outside [0,%d]", T, L->cfg.max_tokens);
    if (T > smoe_static_max_tokens())
        return smoe_fail(SMOE_EINVAL, "smoe_permute_static: T=%d exceeds the %d tokens the library's fixed scratch "
                         "array is sized for; use smoe_permute with a bound workspace", T, smoe_static_max_tokens());
    if (!offsets) return smoe_fail(SMOE_EINVAL, "smoe_permute_static: null offsets");
    if (T > 0 && (!x || !slot || !x_perm || !perm || !inv_perm))
        return smoe_fail(SMOE_EINVAL, "smoe_permute_static: null buffer");
    if (T > 0 && (misaligned(x, 16) || misaligned(x_perm, 16)))
        return smoe_fail(SMOE_EINVAL, "smoe_permute_static: x and x_perm must be 16-byte aligned");
    return smoe_launch_permute_static(L->cfg, x, slot, T, x_perm, perm, inv_perm, offsets, as_stream(stream));
}

int smoe_expert_ffn(smoe_layer_t* L, const void* x_perm, const int32_t* offsets, int T, void* y_perm,
                    void* stream) {
    int rc = check_hot(L, T, "smoe_expert_ffn", true);
    if (rc) return rc;
    if (T == 0) return SMOE_OK;
    if (!x_perm || !offsets || !y_perm) return smoe_fail(SMOE_EINVAL, "smoe_expert_ffn: null buffer");
    if (misaligned(x_perm, 16) || misaligned(y_perm, 16))
        return smoe_fail(SMOE_EINVAL, "smoe_expert_ffn: x_perm and y_perm must be 16-byte aligned");
    if (L->cfg.dtype == SMOE_F32)
        rc = smoe_launch_ffn_f32(L, (const float*)x_perm, offsets, T, (float*)y_perm, as_stream(stream));
    else
        rc = smoe_launch_ffn_bf16(L, (const uint16_t*)x_perm, offsets, T, (uint16_t*)y_perm, as_stream(stream));
    L->prof_ev[0] = L->prof_ev[1] = L->prof_ev[2] = L->prof_ev[3] = nullptr;
    return rc;
}

int smoe_forward(smoe_layer_t* L, const void* x, int T, const void* residual, void* out, int accumulate,
                 int32_t* orig_expert, float* orig_gate, int32_t* slot, float* gate, float* xnorm,
                 int32_t* count, float* gsum, float* score, int32_t* perm, int32_t* inv_perm,
                 int32_t* offsets, void* stream) {
    int rc = check_hot(L, T, "smoe_forward", true);
    if (rc) return rc;
    if (L->cfg.dtype != SMOE_BF16)
        return smoe_fail(SMOE_EINVAL, "smoe_forward: only bf16 layers have the fused path; use the six calls");
    if (accumulate != 0 && accumulate != 1)
        return smoe_fail(SMOE_EINVAL, "smoe_forward: accumulate must be 0 or 1");
    if (T == 0) {   // what the separate calls leave behind for an empty batch: offsets = 0, and zeroed sums when overwriting
        if (offsets) {
            rc = smoe_launch_permute(L, nullptr, nullptr, 0, nullptr, nullptr, nullptr, offsets, as_stream(stream));
            if (rc) return rc;
        }
        if (accumulate == 0 && count && gsum && score)
            rc = smoe_launch_importance(L, nullptr, nullptr, nullptr, 0, count, gsum, score, 0, as_stream(stream));
        return rc;
    }
    if (!x || !out || !orig_expert || !orig_gate || !slot || !gate || !xnorm || !count || !gsum || !score ||
        !perm || !inv_perm || !offsets)
        return smoe_fail(SMOE_EINVAL, "smoe_forward: null buffer");
    if (misaligned(x, 16) || misaligned(out, 16) || (residual && misaligned(residual, 16)))
        return smoe_fail(SMOE_EINVAL, "smoe_forward: x, residual and out must be 16-byte aligned");
    if (x == out) return smoe_fail(SMOE_EINVAL, "smoe_forward: out must not alias x");
    hipStream_t s = as_stream(stream);
    if (!L->router_split_done) {
        rc = smoe_launch_split_router(L, s);
        if (rc) return rc;
        L->router_split_done = true;
    }
    if (smoe_decode_first_applies(L, T) && smoe_ffn_dense_path(L, T)) {
        // decode step in two launches: the router (with its ranking tail) next to the first product
        // of every slot, then the second product of the slots that got tokens
        rc = smoe_launch_decode_first(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, count, gsum, score, accumulate,
                                      perm, inv_perm, offsets, s, L->prof_ev[0], L->prof_ev[1]);
        if (!rc) rc = smoe_launch_ffn_bf16_dense_second(L, slot, gate, (const uint16_t*)residual, T, (uint16_t*)out, s);
        L->prof_ev[0] = L->prof_ev[1] = L->prof_ev[2] = L->prof_ev[3] = nullptr;
        return rc;
    }
    if (T <= 32) {   // decode-sized batch: the router's one workgroup ranks and accumulates as well
        rc = smoe_launch_route_rank_small(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, count, gsum, score,
                                          accumulate, perm, inv_perm, offsets, s);
        if (rc) return rc;
    } else {
        rc = smoe_launch_route(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, L->d_hist32, s);
        if (rc) return rc;
        rc = smoe_launch_rank_importance(L, orig_expert, orig_gate, xnorm, slot, T, count, gsum, score, accumulate,
                                         perm, inv_perm, offsets, s);
        if (rc) return rc;
    }
    rc = smoe_launch_ffn_bf16_fused(L, (const uint16_t*)x, slot, perm, offsets, gate, (const uint16_t*)residual,
                                    T, (uint16_t*)out, s);
    L->prof_ev[0] = L->prof_ev[1] = L->prof_ev[2] = L->prof_ev[3] = nullptr;
    return rc;
}

int smoe_set_profile_events(smoe_layer_t* L, void* g1_begin, void* g1_end, void* g2_begin, void* g2_end) {
    if (!L) return smoe_fail(SMOE_EINVAL, "smoe_set_profile_events: null handle");
    bool none = !g1_begin && !g1_end && !g2_begin && !g2_end, all = g1_begin && g1_end && g2_begin && g2_end;
    if (!none && !all) return smoe_fail(SMOE_EINVAL, "smoe_set_profile_events: pass four events or four NULLs");
    L->prof_ev[0] = (hipEvent_t)g1_begin;
    L->prof_ev[1] = (hipEvent_t)g1_end;
    L->prof_ev[2] = (hipEvent_t)g2_begin;
    L->prof_ev[3] = (hipEvent_t)g2_end;
    return SMOE_OK;
}

int smoe_combine(smoe_layer_t* L, const void* y_perm, const int32_t* inv_perm, const float* gate,
                 const void* residual, int T, void* out, void* stream) {
    int rc = check_hot(L, T, "smoe_combine", false);
    if (rc) return rc;
    if (T == 0) return SMOE_OK;
    if (!y_perm || !inv_perm || !gate || !out) return smoe_fail(SMOE_EINVAL, "smoe_combine: null buffer");
    if (misaligned(y_perm, 16) || misaligned(out, 16) || (residual && misaligned(residual, 16)))
        return smoe_fail(SMOE_EINVAL, "smoe_combine: y_perm, residual and out must be 16-byte aligned");
    return smoe_launch_combine(L, y_perm, inv_perm, gate, residual, T, out, as_stream(stream));
}

}  // extern "C"
