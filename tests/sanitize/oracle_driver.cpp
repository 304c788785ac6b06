// Runs every entry point of the CPU oracle on small inputs.  Built together with
// oracle.cpp under AddressSanitizer and UndefinedBehaviorSanitizer by
// tests/test_sanitizers_cpu.py: the run must end with "ok" and no report.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
int oracle_route(const void* x, int x_dtype, int T, int d, const float* Wr, int E, const int32_t* expert_to_slot,
                 int gate_mode, int32_t* orig_expert, float* orig_gate, int32_t* slot, float* gate, float* xnorm,
                 double* logits_out, uint8_t* ambiguous, double margin);
int oracle_expert_norm(const void* W1, const void* W2, int w_dtype, int n_experts, int d, int f, double* out);
int oracle_importance(const int32_t* orig_expert, const float* orig_gate, const float* xnorm, int T,
                      const double* expert_norm, int E, int32_t* count, double* gsum, double* score, int accumulate);
int oracle_permute(const void* x, size_t row_bytes, const int32_t* slot, int T, int K, void* x_perm, int32_t* perm,
                   int32_t* inv_perm, int32_t* offsets);
int oracle_expert_ffn(const void* x_perm, int x_dtype, const void* W1, const void* W2, int w_dtype,
                      const int32_t* offsets, int K, int d, int f, int T, const int32_t* rows, int n_rows, double* y);
int oracle_combine(const void* y_perm, int y_dtype, const int32_t* inv_perm, const float* gate, const void* residual,
                   int res_dtype, int T, int d, void* out, int out_dtype);
int oracle_select_resident(const double* score, int E, int K, int32_t* slot_to_expert, int32_t* expert_to_slot,
                           int32_t* changed_slots, int32_t* changed_experts);
int oracle_policy_scores(int policy, int E, const int32_t* count, const double* score, const double* expert_norm,
                         double* rank);
int oracle_on_demand(const int32_t* orig_expert, int T, int E, int K, const int32_t* expert_to_slot, int64_t* clock,
                     int64_t* last_use, int32_t* changed_slots, int32_t* changed_experts);
void oracle_round_bf16(const double* in, size_t n, uint16_t* out);
}

static float frand() { return (float)rand() / RAND_MAX - 0.5f; }

int main() {
    srand(7);
    const int E = 7, K = 3, d = 12, f = 20;
    for (int T : {0, 1, 37}) {
        for (int dtype : {0, 1}) {                       // fp32, bf16 bit patterns
            std::vector<float> xf(T * d + 1), Wr(E * d);
            for (auto& v : xf) v = frand();
            for (auto& v : Wr) v = 4 * frand();
            std::vector<uint16_t> xb(T * d + 1);
            std::vector<double> tmp(xf.begin(), xf.end());
            oracle_round_bf16(tmp.data(), tmp.size(), xb.data());
            const void* x = dtype ? (const void*)xb.data() : (const void*)xf.data();
            std::vector<int32_t> e2s = {-1, 0, -1, 2, -1, 1, -1}, s2e = {1, 5, 3};
            std::vector<int32_t> oe(T + 1), slot(T + 1), perm(T + 1), inv(T + 1), offsets(K + 1), count(E);
            std::vector<float> og(T + 1), gate(T + 1), xn(T + 1);
            std::vector<double> logits(T * E + 1), en(E), gsum(E), score(E), rank(E);
            std::vector<uint8_t> amb(T + 1);
            for (int mode : {0, 1})
                if (oracle_route(x, dtype, T, d, Wr.data(), E, e2s.data(), mode, oe.data(), og.data(), slot.data(),
                                 gate.data(), xn.data(), logits.data(), amb.data(), 1e-4)) return 1;
            std::vector<float> W1f(E * d * f), W2f(E * f * d);
            for (auto& v : W1f) v = frand();
            for (auto& v : W2f) v = frand();
            std::vector<double> t1(W1f.begin(), W1f.end()), t2(W2f.begin(), W2f.end());
            std::vector<uint16_t> W1b(W1f.size()), W2b(W2f.size());
            oracle_round_bf16(t1.data(), t1.size(), W1b.data());
            oracle_round_bf16(t2.data(), t2.size(), W2b.data());
            const void* W1 = dtype ? (const void*)W1b.data() : (const void*)W1f.data();
            const void* W2 = dtype ? (const void*)W2b.data() : (const void*)W2f.data();
            if (oracle_expert_norm(W1, W2, dtype, E, d, f, en.data())) return 2;
            for (int acc : {0, 1})
                if (oracle_importance(oe.data(), og.data(), xn.data(), T, en.data(), E, count.data(), gsum.data(),
                                      score.data(), acc)) return 3;
            const size_t row_bytes = (size_t)d * (dtype ? 2 : 4);
            std::vector<uint8_t> xp(T * row_bytes + 1);
            if (oracle_permute(x, row_bytes, slot.data(), T, K, xp.data(), perm.data(), inv.data(), offsets.data())) return 4;
            std::vector<double> y(T * d + 1);
            if (oracle_expert_ffn(xp.data(), dtype, W1, W2, dtype, offsets.data(), K, d, f, T, nullptr, 0, y.data())) return 5;
            std::vector<int32_t> rows = {0};
            if (T > 0 && oracle_expert_ffn(xp.data(), dtype, W1, W2, dtype, offsets.data(), K, d, f, T, rows.data(), 1, y.data())) return 6;
            std::vector<uint8_t> out(T * row_bytes + 1);
            if (oracle_combine(y.data(), 2, inv.data(), gate.data(), x, dtype, T, d, out.data(), dtype)) return 7;
            if (oracle_combine(y.data(), 2, inv.data(), gate.data(), nullptr, dtype, T, d, out.data(), dtype)) return 8;
            for (int policy : {0, 1, 2})
                if (oracle_policy_scores(policy, E, count.data(), score.data(), en.data(), rank.data())) return 9;
            std::vector<int32_t> cs(K), ce(K);
            if (oracle_select_resident(rank.data(), E, K, s2e.data(), e2s.data(), cs.data(), ce.data()) < 0) return 10;
            int64_t clock = 0;
            std::vector<int64_t> last(K, 0);
            for (int rep = 0; rep < 3; ++rep)
                if (oracle_on_demand(oe.data(), T, E, K, e2s.data(), &clock, last.data(), cs.data(), ce.data()) < 0) return 11;
        }
    }
    printf("ok\n");
    return 0;
}
