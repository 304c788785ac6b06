/*
 * libswapmoe -- the Virtual-Expert top-1 MoE layer of SwapMoE on one MI355X.
 *
 * One Switch-style MoE layer whose router may only pick from a small resident
 * set of K "Virtual Experts" out of E (SwapMoE, Section 3.1 "Masked Gating",
 * Figure 4(b)).  The forward pass is six calls, all enqueued on the caller's
 * HIP stream, none of which allocates, synchronises or reads back:
 *
 *   smoe_route       router product, softmax, original and masked top-1, |x|
 *   smoe_importance  per-expert importance accumulators (Eq. 1)
 *   smoe_permute     stable sort of the tokens by resident slot
 *   smoe_expert_ffn  grouped FFN  ReLU(x W1_k) W2_k  over the sorted rows
 *   smoe_combine     y = G(x)_i E_i(x) back in token order
 *   smoe_set_resident  load one expert's weights into a slot (Section 3.2)
 *
 * Conventions
 *   - Plain C ABI.  Every call returns SMOE_OK (0) or a negative smoe_status;
 *     smoe_last_error() gives a thread-local message for the last failure.
 *     Arguments are validated before anything is launched.
 *   - Unless marked "host", every pointer is a DEVICE pointer owned by the
 *     caller, who keeps it alive until the stream work that uses it is done.
 *     The library owns only the opaque handle (host memory, plus one HIP
 *     event per spare slot once smoe_update_tick has been used).
 *   - All matrices are row-major and dense.  Activations and expert weights
 *     have the dtype given in smoe_config (fp32, or bf16 stored as uint16 bit
 *     patterns); router weights, gates, norms and scores are fp32; indices and
 *     counts are int32.
 *   - T is a host integer, 0 <= T <= max_tokens; T = 0 is a legal no-op.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Calls on one handle must be issued from one thread at a time, and stream
 *     work of consecutive calls on one handle must be ordered (same stream, or
 *     event dependencies), because they share the bound workspace.
 *   - NaN / Inf inputs give undefined results.
 */
#ifndef SWAPMOE_H
#define SWAPMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SMOE_OK = 0,
    SMOE_EINVAL = -1,   /* bad argument: null pointer, size out of range, unknown enum   */
    SMOE_ESTATE = -2,   /* call not legal in the handle's state (unbound, slots unset, ...) */
    SMOE_EHIP = -3,     /* the HIP runtime reported an error; text in smoe_last_error()  */
    SMOE_ENOMEM = -4    /* host allocation for the handle failed                         */
} smoe_status;

enum { SMOE_F32 = 0, SMOE_BF16 = 1 };
enum { SMOE_GATE_FULL = 0, SMOE_GATE_RENORM = 1 };

typedef struct smoe_layer smoe_layer_t;

/* Layer shape.  E experts in the full bank, K resident slots (1 <= K <= E),
 * d_model -> d_ff -> ReLU -> d_model experts without biases.  dtype is the
 * storage type of activations AND expert weights (SMOE_F32 or SMOE_BF16).
 * gate_mode: SMOE_GATE_FULL  gate = softmax over all E, read at the served expert;
 *            SMOE_GATE_RENORM the same divided by the resident experts' total.
 * spare_slots: physical weight slots beyond K that smoe_update_tick loads into while the
 *            K mapped ones keep serving (see the asynchronous update calls below).
 * Limits: E <= 256; K <= E; for SMOE_BF16, d_model and d_ff must be
 * multiples of 32 (the MFMA fragment width); max_tokens >= 1. */
typedef struct {
    int32_t E, K, d_model, d_ff, max_tokens;
    int32_t dtype;
    int32_t gate_mode;
    int32_t spare_slots;   /* extra physical slots for asynchronous loading, 0..8 (0: synchronous updates only) */
} smoe_config;

/* Creates a handle (host memory only; no HIP call is made).  *out is set to
 * NULL on failure.  Initially no slot holds an expert. */
int smoe_create(const smoe_config* cfg /*host*/, smoe_layer_t** out /*host*/);
int smoe_destroy(smoe_layer_t* layer);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char* smoe_last_error(void);

/* Bytes of device workspace smoe_bind() needs (maps, sort histograms, the
 * FFN's hidden activations for max_tokens rows).  0 if layer is NULL. */
size_t smoe_workspace_bytes(const smoe_layer_t* layer);

/* Bytes of ONE of the two slot weight arrays (slot_w1 or slot_w2) for all
 * K + spare_slots physical slots.  The arrays are opaque to the caller: for
 * SMOE_BF16 the library keeps each slot in a tiled order that feeds the matrix
 * cores with contiguous loads (see smoe_set_resident), so they can only be
 * filled through smoe_set_resident / smoe_update_tick.
 * Equals (K + spare_slots) * d_model * d_ff * sizeof(dtype): always size the
 * arrays with this call, never with K alone. */
size_t smoe_slot_weight_bytes(const smoe_layer_t* layer);

/* Binds the caller-owned device buffers the layer works on.
 *   router_w    [E, d_model] fp32, the router G's weight (no bias); the first
 *               smoe_route after a bind may keep a re-formatted copy in the
 *               workspace, so re-bind after changing the router's weights
 *   slot_w1/2   smoe_slot_weight_bytes() each, 256-byte aligned, contents
 *               written only by smoe_set_resident
 *   expert_norm [E] fp32, |E_i| of Eq. 1 for every expert of the bank
 *               (e.g. from smoe_expert_norm); read by smoe_importance
 *   workspace   smoe_workspace_bytes() bytes, 256-byte aligned
 * Rebinding is allowed and marks every slot empty again. */
int smoe_bind(smoe_layer_t* layer, const float* router_w, void* slot_w1, void* slot_w2,
              const float* expert_norm, void* workspace);

/* |E_i| of Eq. 1 for n <= E experts stored in bank layout (the layer must be
 * bound: partial sums use its workspace): w1 [n, d_model, d_ff],
 * w2 [n, d_ff, d_model] in the layer's dtype -> out [n] fp32, the Frobenius
 * norm of all of the expert's parameters, sqrt(|W1_i|^2 + |W2_i|^2).  The same
 * magnitude ranks experts in the paper's "Pruning" baseline (Section 4.1). */
int smoe_expert_norm(smoe_layer_t* layer, const void* w1, const void* w2, int n, float* out,
                     void* stream);

/* Virtual-Expert update (Section 3.2): puts `expert` into `slot`.  Reads the
 * expert's weights in bank layout, w1_src [d_model, d_ff] and w2_src
 * [d_ff, d_model] (device memory, managed memory, or pinned host memory mapped
 * into the device; pageable host memory is refused with SMOE_EINVAL before
 * anything is launched), and writes them into the slot arrays in the library's
 * tiled order;
 * updates the slot<->expert maps on the host and, in stream order, on the
 * device.  The previous occupant of the slot stops being resident.
 * Errors: slot outside [0,K) or expert outside [0,E) -> SMOE_EINVAL; expert
 * already resident in a DIFFERENT slot -> SMOE_ESTATE (same slot = refresh). */
int smoe_set_resident(smoe_layer_t* layer, int slot, int expert, const void* w1_src,
                      const void* w2_src, void* stream);

/* Host copies of the maps: slot_to_expert [K] (-1 = empty), expert_to_slot [E]
 * (-1 = not resident).  Either pointer may be NULL.  After smoe_update_on_device
 * the call first waits for that update and fetches the device's maps. */
int smoe_get_maps(const smoe_layer_t* layer, int32_t* slot_to_expert /*host*/,
                  int32_t* expert_to_slot /*host*/);

/* Update policy (Section 3.2: important experts in, unimportant out), host
 * only: given score [E] (host), the new resident set is the K highest-scoring
 * experts (ties: lower expert id); experts that stay keep their slot; freed
 * slots in ascending order receive incoming experts in descending score
 * order.  Nothing is changed in the handle: the (slot, expert) pairs to load
 * are written to changed_slots / changed_experts (host, capacity K) and their
 * number is returned (>= 0), or a negative smoe_status.  The caller then calls
 * smoe_set_resident for each pair, in the order given. */
int smoe_select_resident(const smoe_layer_t* layer, const float* score /*host*/,
                         int32_t* changed_slots /*host*/, int32_t* changed_experts /*host*/);

/* The same update with nobody waiting for anybody (bf16 layers): the rule above
 * is applied ON THE DEVICE to score [E] (device; what smoe_importance or
 * smoe_forward leaves, or any other ranking), the device maps are switched, and
 * the changed slots are loaded from the bank -- bank_w1 [E, d_model, d_ff],
 * bank_w2 [E, d_ff, d_model], bf16 bit patterns in device or pinned host
 * memory, indexed by expert id -- all enqueued on `stream` behind the work
 * already there, with no read-back: the host learns the new maps only when it
 * asks (smoe_get_maps and the other calls that consult the maps then wait for
 * that stream once).  With the whole bank in GPU memory (288 GB hold every
 * expert of the paper's models) this takes the controller's round trip out of
 * the decode loop.  SMOE_ESTATE until every slot holds an expert, and while an
 * asynchronous update (smoe_update_begin) is pending. */
int smoe_update_on_device(smoe_layer_t* layer, const float* score /*device*/, const void* bank_w1,
                          const void* bank_w2, void* stream);

/* What ranks the experts at an update, for smoe_select_resident / smoe_update_begin:
 *   SMOE_POLICY_IMPORTANCE  the Eq. 1 score (SwapMoE's own scheduling)
 *   SMOE_POLICY_COUNT       the number of tokens routed to the expert, the "simple
 *                           scheduling" of the ablation (Section 4.5)
 *   SMOE_POLICY_MAGNITUDE   |E_i|, constant over time: the "Pruning" baseline of the
 *                           evaluation (Section 4.1) keeps the K largest experts and never swaps
 * Writes rank[e] (host, [E]) from the host copies of the layer's accumulators
 * (count, score as smoe_importance leaves them) or of expert_norm; only the
 * array the policy reads must be non-NULL. */
enum { SMOE_POLICY_IMPORTANCE = 0, SMOE_POLICY_COUNT = 1, SMOE_POLICY_MAGNITUDE = 2 };
int smoe_policy_scores(int policy, int E, const int32_t* count /*host*/, const float* score /*host*/,
                       const float* expert_norm /*host*/, float* rank /*host*/);

/* The "On demand" baseline (Section 4.1; the caching the paper's Section 2.1
 * measures): after a batch, every expert that a token asked for and that was
 * not resident is loaded, into the slots that have gone unused the longest.
 * Reading (the paper gives no rule): given the batch's orig_expert [T] (host),
 * slots whose expert was some token's own choice are stamped as used now; the
 * missed experts, most requested first (ties: lower id), are paired with the
 * slots not used by this batch, least recently used first (ties: lower slot),
 * until either list ends.  The pairs are written to changed_slots /
 * changed_experts (host, capacity K) and their number is returned; the caller
 * loads them with smoe_set_resident.  The use stamps live in the handle and
 * start afresh at smoe_bind. */
int smoe_on_demand_plan(smoe_layer_t* layer, const int32_t* orig_expert /*host*/, int T,
                        int32_t* changed_slots /*host*/, int32_t* changed_experts /*host*/);

/* Router (Background section: with k = 1 only the expert with the largest G(x)_i runs)
 * and Masked Gating (Section 3.1).  For each token t of x [T, d_model]:
 *   logit = x_t . router_w^T (fp32), p = softmax(logit) over all E;
 *   orig_expert[t] = argmax_e logit (lowest id on a tie), orig_gate[t] = p[orig];
 *   s = argmax over RESIDENT experts of the same logits;
 *   slot[t] = slot holding s, gate[t] per gate_mode; xnorm[t] = |x_t|_2.
 * SMOE_ESTATE until every slot has been filled by smoe_set_resident. */
int smoe_route(smoe_layer_t* layer, const void* x, int T, int32_t* orig_expert, float* orig_gate,
               int32_t* slot, float* gate, float* xnorm, void* stream);

/* Importance accumulation (Eq. 1), over X_i = tokens whose ORIGINAL choice is i:
 *   count[i] (+)= |X_i|                      the "simple scheduling" score (Section 4.5)
 *   gsum[i]  (+)= sum_{t in X_i} orig_gate[t]
 *   score[i] (+)= expert_norm[i] * sum_{t in X_i} xnorm[t] * orig_gate[t]   (Eq. 1)
 * for all i in [0,E).  accumulate = 0 overwrites, 1 adds to the arrays'
 * current contents.  Deterministic: no atomics, fixed summation order. */
int smoe_importance(smoe_layer_t* layer, const int32_t* orig_expert, const float* orig_gate,
                    const float* xnorm, int T, int32_t* count, float* gsum, float* score,
                    int accumulate, void* stream);

/* Stable counting sort of the tokens by slot (each token goes to exactly one
 * resident expert, no capacity limit, no dropping): segments in slot order,
 * ascending token index inside a segment.
 *   offsets[k] = #tokens with slot < k, k in [0,K]; perm[pos] = token;
 *   inv_perm[token] = pos; x_perm[pos, :] = x[perm[pos], :].
 * slot values must lie in [0,K) (as smoe_route writes them). */
int smoe_permute(smoe_layer_t* layer, const void* x, const int32_t* slot, int T, void* x_perm,
                 int32_t* perm, int32_t* inv_perm, int32_t* offsets, void* stream);

/* smoe_permute for callers that cannot allocate device memory and have no
 * workspace to bind -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results bit for bit,
 * but the sort's per-block histograms (its only device memory beyond inputs
 * and outputs) live in a fixed 64-KiB array inside the library image, one copy
 * per GPU for the life of the process; the handle need not be bound.  The call
 * allocates nothing and synchronises nothing.
 * Limit: T <= 65536 (and T <= max_tokens); more is refused with SMOE_EINVAL.
 * Every call on a GPU shares that GPU's array: calls whose stream work may
 * overlap on one GPU (different streams, no ordering) race and must be
 * serialised by the caller.  Nothing in the array needs clearing between
 * calls -- each call overwrites every entry it later reads. */
int smoe_permute_static(smoe_layer_t* layer, const void* x, const int32_t* slot, int T, void* x_perm,
                        int32_t* perm, int32_t* inv_perm, int32_t* offsets, void* stream);

/* Grouped expert FFN, E_i(x) of the Background section: rows
 * [offsets[k], offsets[k+1]) of x_perm [T, d_model] belong to slot k and get
 *   y_perm[r, :] = ReLU(x_perm[r, :] . W1_k) . W2_k          (no biases)
 * bf16: matrix-core products with fp32 accumulation, the hidden activations
 * are rounded to bf16 between the two products.  offsets is the device array
 * smoe_permute wrote (non-decreasing, offsets[0] = 0, offsets[K] = T). */
int smoe_expert_ffn(smoe_layer_t* layer, const void* x_perm, const int32_t* offsets, int T,
                    void* y_perm, void* stream);

/* The whole layer in one call (bf16 layers): the same results as smoe_route,
 * smoe_importance, smoe_permute, smoe_expert_ffn and smoe_combine issued in that
 * order on the same buffers -- bit for bit -- in four launches instead of nine:
 * the router also counts tokens per slot, one launch ranks the tokens and
 * reduces the importance sums, the first FFN product reads its rows from x
 * through perm (x_perm is never written) and the second writes
 * gate * y (+ residual) straight to out in token order (y_perm is never
 * written).  A decode-sized batch (at most 32 tokens, a few per slot, at most
 * 64 experts) takes two launches: the router, which then also ranks the tokens
 * and adds the importance sums, runs as one workgroup of the launch whose other
 * workgroups compute the first product for every slot and every token of the
 * batch (it does not wait for the routing; the weights of slots that turn out
 * empty are streamed for nothing), and the second product picks each token's
 * row from its slot.  All the per-token and per-expert outputs of the individual
 * calls are produced: orig_expert, orig_gate, slot, gate, xnorm [T]; count, gsum,
 * score [E] (accumulate as in smoe_importance); perm, inv_perm [T];
 * offsets [K+1].  residual may be NULL and may alias x; out must not alias x.
 * T = 0 leaves what the separate calls leave: offsets = 0 and, with
 * accumulate = 0, zeroed count / gsum / score. */
int smoe_forward(smoe_layer_t* layer, const void* x, int T, const void* residual, void* out,
                 int accumulate, int32_t* orig_expert, float* orig_gate, int32_t* slot, float* gate,
                 float* xnorm, int32_t* count, float* gsum, float* score, int32_t* perm,
                 int32_t* inv_perm, int32_t* offsets, void* stream);

/* ---- Asynchronous, amortized resident-set update (Section 3.2 "Seamless ...
 * Update"; Figure 5(ii)) ---------------------------------------------------
 * Needs spare_slots >= 1.  The K virtual slots map onto K of the K+spare
 * physical weight slots; a new expert is packed into a free physical slot on
 * a separate stream while the forward pass keeps using the mapped ones, and
 * the maps are switched between two hot calls once the load has finished.
 * At most `spare_slots` loads are in flight, so an update of many experts is
 * spread over as many steps as it needs instead of stalling one step.
 *
 * smoe_update_begin: host policy.  From the E importance scores (host array)
 *   it plans the changes with the rule of smoe_select_resident, taking loads
 *   already in flight as done, and replaces any earlier plan not yet started.
 *   Returns the number of planned changes (>= 0) or a negative status.
 * smoe_update_tick: call between two steps.  (1) Every in-flight load whose
 *   copy has finished (event query; never waits) is committed: the slot and
 *   expert maps and the slot's physical index change on compute_stream, so
 *   the next hot call enqueued there serves the new expert, and the physical
 *   slot it leaves becomes free once the work already enqueued has drained.
 *   (2) While a physical slot is free and the plan is not empty, the next
 *   expert's weights are packed from the bank on load_stream.  bank_w1 /
 *   bank_w2 hold all E experts contiguously ([E][d_model][d_ff] and
 *   [E][d_ff][d_model], the layer's dtype) in device memory or in pinned host
 *   memory (then the copy engines bring the expert into a staging area of the
 *   workspace first); they must stay valid until the load is done.  Pageable
 *   host memory is refused with SMOE_EINVAL before anything is launched.
 *   A planned change whose slot still has an earlier load in flight waits
 *   for that load's commit; the other changes go ahead of it.
 *   load_stream must differ from compute_stream for any overlap to happen.
 *   Returns the number of commits made by this call (>= 0) or a negative status.
 * smoe_update_pending: planned changes not yet committed (in flight included). */
int smoe_update_begin(smoe_layer_t* layer, const float* score /*host, [E]*/);
int smoe_update_tick(smoe_layer_t* layer, const void* bank_w1, const void* bank_w2, void* load_stream,
                     void* compute_stream);
int smoe_update_pending(const smoe_layer_t* layer);

/* Gate-weighted combine, y = G(x)_i E_i(x) in token order:
 *   out[t, :] = gate[t] * y_perm[inv_perm[t], :]  (+ residual[t, :] if not NULL)
 * computed in fp32 and rounded once to the layer's dtype. */
int smoe_combine(smoe_layer_t* layer, const void* y_perm, const int32_t* inv_perm, const float* gate,
                 const void* residual, int T, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SWAPMOE_H */
