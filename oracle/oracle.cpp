// CPU oracle for the Virtual-Expert (masked-gating) top-1 MoE layer of SwapMoE.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
// library is checked against.  Only the tests, the smoke check and the
// benchmark's cpu_baseline leg may build or call it; the product path never
// does.  It shares no code, header, table or helper with the HIP sources.
//
// Everything is written as the paper states the layer, one step after the
// other, with plain loops and double accumulation:
//   * sparse top-1 MoE output  y = G(x)_i * E_i(x), i = argmax G(x)
//     (Background and Motivation, first paragraph);
//   * Masked Gating: every token is served by a Virtual Expert, i.e. a member
//     of the resident set (Section 3.1, Figure 4(b));
//   * expert importance score (Eq. 1): sum over the tokens that chose expert i
//     of |x| * |G(x)_i| * |E_i|;
//   * the count-based score of the "simple scheduling" ablation (Section 4.5);
//   * Virtual-Expert update: important experts in, unimportant out
//     (Section 3.2), every `frequency` inputs (Eq. 2).
// Where the paper is silent the reading taken is stated at the function.
//
// Parity unpinned (fixed only by the stated reading, nothing in the paper or
// in mathematics decides them): the RENORM gate mode, the choice of L2 /
// Frobenius norms in Eq. 1, and the slot-assignment details of the update rule.
//
// Storage dtypes: 0 = fp32, 1 = bf16 bit patterns (uint16), 2 = fp64.
// bf16 values are widened exactly; nothing is ever rounded before the final
// store of a result.  OpenMP is used only across token rows (or experts), each
// row being computed start to finish by one thread, so results do not depend
// on the thread count.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>
#include <limits>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// bf16 bit pattern -> double, exact.
inline double widen(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return (double)f;
}

inline double load(const void* p, int dtype, size_t i) {
    if (dtype == 0) return (double)((const float*)p)[i];
    if (dtype == 2) return ((const double*)p)[i];
    return widen(((const uint16_t*)p)[i]);
}

// Round a double to bf16 (nearest, ties to even), by scaling the
// value exactly so one bf16 quantum is 1.0 and rounding to an integer, so there
// is no double rounding through fp32.
inline uint16_t to_bf16(double v) {
    if (std::isnan(v)) return 0x7FC0;
    uint16_t sign = std::signbit(v) ? 0x8000 : 0;
    double a = std::fabs(v);
    if (std::isinf(a)) return sign | 0x7F80;
    if (a == 0.0) return sign;
    int ex;
    (void)std::frexp(a, &ex);               // a = m * 2^ex, m in [0.5,1)
    int e = ex - 1;                         // a = (2m) * 2^e, 2m in [1,2)
    int qexp = (e < -126) ? -126 : e;       // exponent of the quantum's scale
    // quantum = 2^(qexp-7): bf16 keeps 7 fraction bits
    double scaled = std::ldexp(a, 7 - qexp);   // exact
    double r = std::nearbyint(scaled);         // default mode: ties to even
    double q = std::ldexp(r, qexp - 7);
    if (q >= std::ldexp(1.0, 128)) return sign | 0x7F80;
    float f = (float)q;                        // exact: q is a bf16 value
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return sign | (uint16_t)(u >> 16);
}

inline void store(void* p, int dtype, size_t i, double v) {
    if (dtype == 0) ((float*)p)[i] = (float)v;
    else if (dtype == 2) ((double*)p)[i] = v;
    else ((uint16_t*)p)[i] = to_bf16(v);
}

}  // namespace

extern "C" {

// Router, softmax, original top-1, masked top-1 and token norm.
//
// logit[t][e] = sum_j x[t][j] * Wr[e][j]; p = softmax over ALL E experts;
// e* = argmax_e logit (lowest index on an exact tie), g* = p[e*]
// (Background section: with k = 1 only the expert with the largest G(x)_i runs).
// Masked Gating (Section 3.1, Figure 4(b)): s = argmax over resident experts
// only (expert_to_slot[e] >= 0) of the same logits, slot = expert_to_slot[s].
// Reading: gate = p[s] from the softmax over all E (gate_mode 0, "FULL"), or
// p[s] / sum_{r resident} p[r] (gate_mode 1, "RENORM").  xnorm = L2 norm of x_t
// (the |x| factor of Eq. 1).
//
// Optional outputs (may be null): logits [T,E] in double; ambiguous [T] = 1
// when the top-1/top-2 logit gap, over all experts or over the resident ones,
// is below margin * max(1, max_e |logit|) -- such tokens' indices may
// legitimately differ under fp32 rounding and parity tests skip them.
int oracle_route(const void* x, int x_dtype, int T, int d, const float* Wr, int E,
                 const int32_t* expert_to_slot, int gate_mode,
                 int32_t* orig_expert, float* orig_gate, int32_t* slot, float* gate,
                 float* xnorm, double* logits_out, uint8_t* ambiguous, double margin) {
    if (T < 0 || d <= 0 || E <= 0) return -1;
    int n_res = 0;
    for (int e = 0; e < E; ++e) n_res += expert_to_slot[e] >= 0;
    if (n_res == 0) return -2;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        std::vector<double> logit(E), p(E);
        double sq = 0.0;
        for (int j = 0; j < d; ++j) {
            double v = load(x, x_dtype, (size_t)t * d + j);
            sq += v * v;
        }
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int j = 0; j < d; ++j)
                acc += load(x, x_dtype, (size_t)t * d + j) * (double)Wr[(size_t)e * d + j];
            logit[e] = acc;
        }
        double m = logit[0];
        for (int e = 1; e < E; ++e) m = std::max(m, logit[e]);
        double z = 0.0;
        for (int e = 0; e < E; ++e) { p[e] = std::exp(logit[e] - m); z += p[e]; }
        for (int e = 0; e < E; ++e) p[e] /= z;

        int best = 0;
        for (int e = 1; e < E; ++e) if (logit[e] > logit[best]) best = e;
        int rbest = -1;
        double rsum = 0.0;
        for (int e = 0; e < E; ++e) {
            if (expert_to_slot[e] < 0) continue;
            rsum += p[e];
            if (rbest < 0 || logit[e] > logit[rbest]) rbest = e;
        }
        orig_expert[t] = best;
        orig_gate[t] = (float)p[best];
        slot[t] = expert_to_slot[rbest];
        gate[t] = (float)(gate_mode == 1 ? p[rbest] / rsum : p[rbest]);
        xnorm[t] = (float)std::sqrt(sq);
        if (logits_out)
            for (int e = 0; e < E; ++e) logits_out[(size_t)t * E + e] = logit[e];
        if (ambiguous) {
            double amax = 0.0, second = -std::numeric_limits<double>::infinity(),
                   rsecond = -std::numeric_limits<double>::infinity();
            for (int e = 0; e < E; ++e) {
                amax = std::max(amax, std::fabs(logit[e]));
                if (e != best) second = std::max(second, logit[e]);
                if (e != rbest && expert_to_slot[e] >= 0) rsecond = std::max(rsecond, logit[e]);
            }
            double delta = margin * std::max(1.0, amax);
            bool amb = (E > 1 && logit[best] - second < delta) ||
                       (n_res > 1 && logit[rbest] - rsecond < delta);
            ambiguous[t] = amb ? 1 : 0;
        }
    }
    return 0;
}

// |E_i| of Eq. 1.  Reading: the Frobenius norm of all of the expert's
// parameters, sqrt(|W1_i|_F^2 + |W2_i|_F^2); a per-expert constant of the bank
// (the same magnitude the "Pruning" baseline ranks experts by).
int oracle_expert_norm(const void* W1, const void* W2, int w_dtype, int n_experts, int d, int f,
                       double* out) {
    size_t per = (size_t)d * f;
#pragma omp parallel for schedule(static)
    for (int e = 0; e < n_experts; ++e) {
        double s = 0.0;
        for (size_t i = 0; i < per; ++i) { double v = load(W1, w_dtype, e * per + i); s += v * v; }
        for (size_t i = 0; i < per; ++i) { double v = load(W2, w_dtype, e * per + i); s += v * v; }
        out[e] = std::sqrt(s);
    }
    return 0;
}

// Importance accumulation (Eq. 1) plus the two simpler statistics.
// X_i is the set of tokens whose ORIGINAL (unmasked) choice is expert i:
// under the other reading a non-resident expert could never score and so
// could never be loaded, which contradicts Section 3.2.
//   count[i] += |X_i|                       (Section 4.5 "simple scheduling")
//   gsum[i]  += sum_{t in X_i} g*_t
//   score[i] += expert_norm[i] * sum_{t in X_i} xnorm_t * g*_t   (Eq. 1)
// accumulate = 0 overwrites the three outputs, 1 adds to them.
int oracle_importance(const int32_t* orig_expert, const float* orig_gate, const float* xnorm, int T,
                      const double* expert_norm, int E, int32_t* count, double* gsum, double* score,
                      int accumulate) {
    std::vector<double> g(E, 0.0), raw(E, 0.0);
    std::vector<int32_t> c(E, 0);
    for (int t = 0; t < T; ++t) {
        int e = orig_expert[t];
        if (e < 0 || e >= E) return -1;
        c[e] += 1;
        g[e] += (double)orig_gate[t];
        raw[e] += (double)xnorm[t] * (double)orig_gate[t];
    }
    for (int e = 0; e < E; ++e) {
        double s = expert_norm[e] * raw[e];
        if (accumulate) { count[e] += c[e]; gsum[e] += g[e]; score[e] += s; }
        else { count[e] = c[e]; gsum[e] = g[e]; score[e] = s; }
    }
    return 0;
}

// Stable counting sort of the tokens by slot: segments in slot order 0..K-1,
// ascending token index inside a segment.  perm[pos] = token, inv_perm[token]
// = pos, offsets[k] = number of tokens with slot < k (offsets[K] = T).
// x_perm may be null; otherwise row pos of x_perm is row perm[pos] of x
// (row_bytes bytes each, copied verbatim).
int oracle_permute(const void* x, size_t row_bytes, const int32_t* slot, int T, int K,
                   void* x_perm, int32_t* perm, int32_t* inv_perm, int32_t* offsets) {
    for (int k = 0; k <= K; ++k) offsets[k] = 0;
    for (int t = 0; t < T; ++t) {
        if (slot[t] < 0 || slot[t] >= K) return -1;
        offsets[slot[t] + 1] += 1;
    }
    for (int k = 0; k < K; ++k) offsets[k + 1] += offsets[k];
    std::vector<int32_t> cursor(offsets, offsets + K);
    for (int t = 0; t < T; ++t) {
        int pos = cursor[slot[t]]++;
        perm[pos] = t;
        inv_perm[t] = pos;
    }
    if (x_perm && x)
        for (int pos = 0; pos < T; ++pos)
            std::memcpy((char*)x_perm + (size_t)pos * row_bytes,
                        (const char*)x + (size_t)perm[pos] * row_bytes, row_bytes);
    return 0;
}

// Grouped expert FFN on permuted rows: row r in [offsets[k], offsets[k+1])
// belongs to slot k and gets y[r] = ReLU(x_perm[r] . W1_k) . W2_k, no biases
// (E_i(x) of the Background section; d_model -> d_ff -> ReLU -> d_model).
// The hidden vector is kept in double and never rounded.  rows/n_rows select
// which rows to compute (null = all T); y is [T, d] double and only the
// selected rows are written.
int oracle_expert_ffn(const void* x_perm, int x_dtype, const void* W1, const void* W2, int w_dtype,
                      const int32_t* offsets, int K, int d, int f, int T,
                      const int32_t* rows, int n_rows, double* y) {
    int n = rows ? n_rows : T;
    std::vector<int32_t> slot_of(T);
    if (offsets[0] != 0 || offsets[K] != T) return -1;
    for (int k = 0; k < K; ++k) {
        if (offsets[k] > offsets[k + 1] || offsets[k] < 0 || offsets[k + 1] > T) return -1;
        for (int r = offsets[k]; r < offsets[k + 1]; ++r) slot_of[r] = k;
    }
#pragma omp parallel for schedule(dynamic, 4)
    for (int i = 0; i < n; ++i) {
        int r = rows ? rows[i] : i;
        int k = slot_of[r];
        size_t w1 = (size_t)k * d * f, w2 = (size_t)k * f * d;
        std::vector<double> h(f, 0.0), out(d, 0.0);
        for (int j = 0; j < d; ++j) {
            double xv = load(x_perm, x_dtype, (size_t)r * d + j);
            if (w_dtype == 1) {
                const uint16_t* w = (const uint16_t*)W1 + w1 + (size_t)j * f;
                for (int c = 0; c < f; ++c) h[c] += xv * widen(w[c]);
            } else {
                for (int c = 0; c < f; ++c) h[c] += xv * load(W1, w_dtype, w1 + (size_t)j * f + c);
            }
        }
        for (int c = 0; c < f; ++c) {
            double hv = h[c] > 0.0 ? h[c] : 0.0;      // ReLU
            if (w_dtype == 1) {
                const uint16_t* w = (const uint16_t*)W2 + w2 + (size_t)c * d;
                for (int m = 0; m < d; ++m) out[m] += hv * widen(w[m]);
            } else {
                for (int m = 0; m < d; ++m) out[m] += hv * load(W2, w_dtype, w2 + (size_t)c * d + m);
            }
        }
        for (int m = 0; m < d; ++m) y[(size_t)r * d + m] = out[m];
    }
    return 0;
}

// Gate-weighted combine: out[t] = gate_t * y_perm[inv_perm[t]] (+ residual[t]),
// i.e. y = G(x)_i E_i(x) put back in token order, rounded once to out_dtype.
int oracle_combine(const void* y_perm, int y_dtype, const int32_t* inv_perm, const float* gate,
                   const void* residual, int res_dtype, int T, int d, void* out, int out_dtype) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        size_t src = (size_t)inv_perm[t] * d;
        for (int m = 0; m < d; ++m) {
            double v = (double)gate[t] * load(y_perm, y_dtype, src + m);
            if (residual) v += load(residual, res_dtype, (size_t)t * d + m);
            store(out, out_dtype, (size_t)t * d + m, v);
        }
    }
    return 0;
}

// Virtual-Expert update rule (Section 3.2).  Reading: the new resident set is
// the K experts with the largest score (ties: lower expert id first); experts
// that stay keep their slot; the freed slots, in ascending slot order, receive
// the incoming experts in descending score order.  The maps are updated in
// place; changed_slots/changed_experts (size K) list the (slot, new expert)
// pairs whose weights must be loaded, and the count is returned (< 0 on error).
int oracle_select_resident(const double* score, int E, int K, int32_t* slot_to_expert,
                           int32_t* expert_to_slot, int32_t* changed_slots, int32_t* changed_experts) {
    if (K > E || K <= 0) return -1;
    std::vector<int> order(E);
    for (int e = 0; e < E; ++e) order[e] = e;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return score[a] > score[b]; });
    std::vector<char> keep(E, 0);
    for (int i = 0; i < K; ++i) keep[order[i]] = 1;
    std::vector<int> incoming;                       // descending score order
    for (int i = 0; i < K; ++i) if (expert_to_slot[order[i]] < 0) incoming.push_back(order[i]);
    int n = 0;
    size_t next = 0;
    for (int s = 0; s < K; ++s) {
        int old = slot_to_expert[s];
        if (old >= 0 && keep[old]) continue;
        if (next >= incoming.size()) return -2;
        int e = incoming[next++];
        if (old >= 0) expert_to_slot[old] = -1;
        slot_to_expert[s] = e;
        expert_to_slot[e] = s;
        changed_slots[n] = s;
        changed_experts[n] = e;
        ++n;
    }
    return n;
}

// The rankings the paper's evaluation compares, as inputs to the update rule above:
//   policy 0  SwapMoE's own scheduling: the Eq. 1 importance score
//   policy 1  "simple scheduling" (Section 4.5): the number of tokens dispatched to the expert
//   policy 2  the "Pruning" baseline (Section 4.1): the expert's magnitude |E_i|, fixed
int oracle_policy_scores(int policy, int E, const int32_t* count, const double* score,
                         const double* expert_norm, double* rank) {
    for (int e = 0; e < E; ++e) {
        if (policy == 0) rank[e] = score[e];
        else if (policy == 1) rank[e] = (double)count[e];
        else if (policy == 2) rank[e] = expert_norm[e];
        else return -1;
    }
    return 0;
}

// The "On demand" baseline (Section 4.1): a portion of the experts is resident
// and an expert that is asked for and missing is loaded.  The paper gives no
// replacement rule; reading: least recently used.  One call = one batch.
//   clock      in/out, incremented once per batch
//   last_use   in/out [K]: the batch in which each slot's expert was last some
//              token's own choice (or was loaded)
// Step 1: every token whose own expert is resident stamps that slot with the
// new clock; the others add one request to their expert.  Step 2: repeatedly
// take the most requested missing expert (lowest id among equals) and the slot
// with the oldest stamp that this batch has not used (lowest slot among
// equals), pair them, stamp the slot; stop when either runs out.  The maps are
// NOT changed here (the caller applies the loads); returns the pair count.
int oracle_on_demand(const int32_t* orig_expert, int T, int E, int K, const int32_t* expert_to_slot,
                     int64_t* clock, int64_t* last_use, int32_t* changed_slots, int32_t* changed_experts) {
    *clock += 1;
    std::vector<int> requests(E, 0);
    for (int t = 0; t < T; ++t) {
        int e = orig_expert[t];
        if (e < 0 || e >= E) return -1;
        if (expert_to_slot[e] >= 0) last_use[expert_to_slot[e]] = *clock;
        else requests[e] += 1;
    }
    int n = 0;
    for (;;) {
        int want = -1;
        for (int e = 0; e < E; ++e)
            if (requests[e] > 0 && (want < 0 || requests[e] > requests[want])) want = e;
        int victim = -1;
        for (int s = 0; s < K; ++s)
            if (last_use[s] < *clock && (victim < 0 || last_use[s] < last_use[victim])) victim = s;
        if (want < 0 || victim < 0) break;
        changed_slots[n] = victim;
        changed_experts[n] = want;
        ++n;
        requests[want] = 0;
        last_use[victim] = *clock;
    }
    return n;
}

// Threads the row loops will use (reported next to the oracle's timings).
int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

// Round-to-nearest-even double -> bf16 bit patterns (exposed for the tests).
void oracle_round_bf16(const double* in, size_t n, uint16_t* out) {
    for (size_t i = 0; i < n; ++i) out[i] = to_bf16(in[i]);
}

}  // extern "C"
