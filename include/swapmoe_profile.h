/*
 * libswapmoe -- the offline side of SwapMoE as far as it can be measured on
 * the layer itself: the per-expert profile of Section 3.3 / Appendix A.1
 * (memory footprint, inference latency, loading time) and the search for the
 * update period of Section 3.4.1.  The accuracy model and the genetic search
 * over per-layer expert counts need the paper's datasets and trained weights
 * and are not here.  Also: a per-kernel timing hook used by the benchmark.
 * Conventions as in swapmoe.h; nothing here is on the hot path.
 */
#ifndef SWAPMOE_PROFILE_H
#define SWAPMOE_PROFILE_H

#include "swapmoe.h"

#ifdef __cplusplus
extern "C" {
#endif

/* E_memory of Appendix A.1: memory is the sum over the resident experts, plus
 * what the layer needs besides them.  All in bytes, from the shape alone:
 *   expert_bytes     one expert's two matrices, 2 * d_model * d_ff * sizeof(dtype)
 *   resident_bytes   (K + spare_slots) * expert_bytes, the slot arrays in GPU memory
 *   workspace_bytes  smoe_workspace_bytes() for this shape
 *   bank_bytes       E * expert_bytes, the full bank kept in external memory
 *   router_bytes     E * d_model * 4                                           */
typedef struct {
    uint64_t expert_bytes, resident_bytes, workspace_bytes, bank_bytes, router_bytes;
} smoe_memory_profile;
int smoe_profile_memory(const smoe_config* cfg /*host*/, smoe_memory_profile* out /*host*/);

/* E_latency and the loading time of Appendix A.1 are measured, not modelled:
 * a bracket of two HIP events owned by the handle.  smoe_profile_begin records
 * the first on `stream`; the caller enqueues what is to be timed (n layer
 * passes at a given K, or n expert loads); smoe_profile_end records the
 * second, WAITS for it (the only synchronising call of the library besides
 * smoe_destroy) and returns the elapsed time in microseconds.
 * SMOE_ESTATE if end is called without a begin. */
int smoe_profile_begin(smoe_layer_t* layer, void* stream);
int smoe_profile_end(smoe_layer_t* layer, void* stream, float* elapsed_us /*host*/);

/* Update-period search (Section 3.4.1): the step latency is measured for update
 * frequencies from low to high (latency_us[0] belongs to the LONGEST period)
 * and the search stops where the latency inflects.  Reading: the inflection is
 * the first point whose latency exceeds the lowest latency seen so far by more
 * than `tolerance` (relative, e.g. 0.1); the index of the point BEFORE it --
 * the highest update frequency still on the flat part -- is returned (n - 1 if
 * the curve never rises).  Host arrays; negative return = smoe_status. */
int smoe_period_inflection(const float* latency_us /*host*/, int n, float tolerance);

/* Calibration for the rooflines this library is measured against (not part of
 * the paper's method): enqueues a kernel that does nothing but read the first K
 * slots of the first (which = 0) or second (which = 1) slot array once --
 * K * d_model * d_ff * sizeof(dtype) bytes, the bytes the weight-streaming
 * kernels of a decode step read when every slot is active -- with plain
 * coalesced loads.  Bracket it with smoe_profile_begin / _end: the elapsed time
 * is what a launch that moves these bytes costs on this GPU with no arithmetic
 * at all.  SMOE_ESTATE before smoe_bind. */
int smoe_profile_stream_read(smoe_layer_t* layer, int which, void* stream);

/* Measurement aid (not part of the paper's method): HIP events for the NEXT
 * smoe_expert_ffn (or smoe_forward) call on this handle.  The call attaches
 * them to its two product kernels' own dispatches: g1_begin / g1_end take the
 * start and end of the first product's execution, g2_begin / g2_end those of
 * the second, so hipEventElapsedTime(g1_begin, g1_end) is that kernel's
 * duration with no launch gap in it.  The events are caller-owned hipEvent_t
 * values passed as void*; they are used once and then forgotten.  Pass four
 * NULLs to cancel. */
int smoe_set_profile_events(smoe_layer_t* layer, void* g1_begin, void* g1_end, void* g2_begin, void* g2_end);

/* Names of the two kernel instances that the expert FFN of a T-token batch
 * runs on this layer (fused != 0: inside smoe_forward), written as a profiler
 * prints them, "first | second", into out (host, n bytes).  Lets a benchmark
 * check that a stored counter summary belongs to the kernels it has timed. */
int smoe_describe_ffn(const smoe_layer_t* layer, int T, int fused, char* out /*host*/, size_t n);

#ifdef __cplusplus
}
#endif
#endif /* SWAPMOE_PROFILE_H */
