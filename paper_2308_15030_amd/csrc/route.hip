// smoe_route: router product, softmax, original top-1, masked top-1 and |x|.
//
// For every token:  logit = x . Wr^T,  p = softmax(logit) over all E experts,
// e* = argmax logit (SwapMoE, Background: the expert with max G(x)_i), and the
// Masked-Gating choice s = argmax over resident experts only (Section 3.1,
// Figure 4(b)).  |x|_2 is produced on the way because x is already in flight
// (it is the first factor of the importance score, Eq. 1).
//
// One workgroup of 256 threads owns 32 tokens and all E experts.  x and Wr are
// staged through LDS in slices of 64 along d_model; thread (ty, tx) keeps a
// 2-token x (E/16)-expert block of logits in registers.  Every logit is one
// sequential fp32 FMA chain in ascending j, so results do not depend on the
// launch shape.  The logits then go to LDS and 8 lanes per token do the
// softmax / arg-max epilogue with xor-shuffles.

#include "smoe_internal.h"

namespace {

constexpr int TB = 32;        // tokens per workgroup
constexpr int DK = 64;        // slice of d_model staged per iteration
constexpr int LDW = DK + 4;   // padded LDS row (floats): 16-lane b128 reads hit 64 distinct banks
constexpr int THREADS = 256;

template <typename XT> struct Loader;
template <> struct Loader<float> {
    // 8 consecutive elements starting at p (16-byte aligned), valid count n (multiple of 4)
    static __device__ __forceinline__ void load8(const float* p, int n, float* v) {
        float4 a = n >= 4 ? *(const float4*)p : make_float4(0, 0, 0, 0);
        float4 b = n >= 8 ? *(const float4*)(p + 4) : make_float4(0, 0, 0, 0);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
};
template <> struct Loader<uint16_t> {
    static __device__ __forceinline__ void load8(const uint16_t* p, int n, float* v) {
        uint4 a = n >= 8 ? *(const uint4*)p : make_uint4(0, 0, 0, 0);
        uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};

// NEC = number of 64-expert groups (E <= 64*NEC).
template <typename XT, int NEC>
__global__ __launch_bounds__(THREADS) void route_kernel(
    const XT* __restrict__ x, const float* __restrict__ Wr, const int32_t* __restrict__ e2s,
    int T, int d, int E, int gate_mode,
    int32_t* __restrict__ orig_expert, float* __restrict__ orig_gate, int32_t* __restrict__ slot,
    float* __restrict__ gate, float* __restrict__ xnorm) {
    extern __shared__ __align__(16) float smem[];
    constexpr int ER = 64 * NEC;                 // expert rows held in LDS
    float* xs = smem;                            // [TB][LDW]
    float* ws = smem + TB * LDW;                 // [ER][LDW]; reused as logits [TB][ER+1]
    __shared__ int32_t s_e2s[ER];

    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * TB;
    const int tx = tid & 15, ty = tid >> 4;      // compute mapping
    const int st = tid >> 3, sj = (tid & 7) * 8; // staging mapping: token, first column

    for (int e = tid; e < ER; e += THREADS) s_e2s[e] = e < E ? e2s[e] : -1;

    float acc[2][4 * NEC];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4 * NEC; ++b) acc[a][b] = 0.f;
    float sq = 0.f;

    const int tok = t0 + st;
    for (int k0 = 0; k0 < d; k0 += DK) {
        __syncthreads();
        {   // x slice: each thread brings 8 columns of one token
            float v[8];
            // columns past d_model (last slice) and tokens past T read as zero;
            // an fp32 row may end in the middle of a group of 8 (n == 4)
            int n = tok < T ? min(8, max(0, d - (k0 + sj))) : 0;
            const XT* p = n > 0 ? x + (size_t)tok * d + k0 + sj : x;
            Loader<XT>::load8(p, n, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) { sq = fmaf(v[i], v[i], sq); }
            *(float4*)&xs[st * LDW + sj] = make_float4(v[0], v[1], v[2], v[3]);
            *(float4*)&xs[st * LDW + sj + 4] = make_float4(v[4], v[5], v[6], v[7]);
        }
        // router slice: ER rows x 64 columns, float4 per thread per step
#pragma unroll
        for (int i = 0; i < ER * (DK / 4) / THREADS; ++i) {
            int idx = tid + i * THREADS;
            int row = idx >> 4, c4 = (idx & 15) * 4;
            float4 w = make_float4(0, 0, 0, 0);
            if (row < E && k0 + c4 < d) w = *(const float4*)&Wr[(size_t)row * d + k0 + c4];
            *(float4*)&ws[row * LDW + c4] = w;
        }
        __syncthreads();
#pragma unroll 4
        for (int j = 0; j < DK; j += 4) {
            float4 xa = *(const float4*)&xs[(2 * ty) * LDW + j];
            float4 xb = *(const float4*)&xs[(2 * ty + 1) * LDW + j];
#pragma unroll
            for (int b = 0; b < 4 * NEC; ++b) {
                float4 w = *(const float4*)&ws[(tx + 16 * b) * LDW + j];
                acc[0][b] = fmaf(xa.x, w.x, acc[0][b]); acc[0][b] = fmaf(xa.y, w.y, acc[0][b]);
                acc[0][b] = fmaf(xa.z, w.z, acc[0][b]); acc[0][b] = fmaf(xa.w, w.w, acc[0][b]);
                acc[1][b] = fmaf(xb.x, w.x, acc[1][b]); acc[1][b] = fmaf(xb.y, w.y, acc[1][b]);
                acc[1][b] = fmaf(xb.z, w.z, acc[1][b]); acc[1][b] = fmaf(xb.w, w.w, acc[1][b]);
            }
        }
    }
    __syncthreads();
    float* lg = ws;                               // [TB][ER + 1]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4 * NEC; ++b) lg[(2 * ty + a) * (ER + 1) + tx + 16 * b] = acc[a][b];
    __syncthreads();

    // epilogue: lanes 8*st .. 8*st+7 of the workgroup own token st
    const int sub = tid & 7;
    const float* row = lg + st * (ER + 1);
    float best = -INFINITY, rbest = -INFINITY;
    int bi = 0x7fffffff, rbi = 0x7fffffff;
    for (int e = sub; e < E; e += 8) {
        float v = row[e];
        if (v > best) { best = v; bi = e; }
        if (s_e2s[e] >= 0 && v > rbest) { rbest = v; rbi = e; }
    }
#pragma unroll
    for (int m = 1; m < 8; m <<= 1) {
        float ov = __shfl_xor(best, m); int oi = __shfl_xor(bi, m);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
        float rv = __shfl_xor(rbest, m); int ri = __shfl_xor(rbi, m);
        if (rv > rbest || (rv == rbest && ri < rbi)) { rbest = rv; rbi = ri; }
    }
    float z = 0.f, zr = 0.f;
    for (int e = sub; e < E; e += 8) {
        float p = expf(row[e] - best);
        z += p;
        if (s_e2s[e] >= 0) zr += p;
    }
#pragma unroll
    for (int m = 1; m < 8; m <<= 1) {
        z += __shfl_xor(z, m);
        zr += __shfl_xor(zr, m);
        sq += __shfl_xor(sq, m);
    }
    if (sub == 0 && tok < T) {
        float ps = expf(rbest - best);
        orig_expert[tok] = bi;
        orig_gate[tok] = 1.0f / z;
        slot[tok] = rbi < ER ? s_e2s[rbi] : 0;   // rbi is always valid once every slot is set
        gate[tok] = gate_mode == SMOE_GATE_RENORM ? ps / zr : ps / z;
        xnorm[tok] = sqrtf(sq);
    }
}

template <typename XT, int NEC>
int launch(const smoe_layer* L, const void* x, int T, int32_t* oe, float* og, int32_t* sl, float* g,
           float* xn, hipStream_t s) {
    constexpr int ER = 64 * NEC;
    size_t lds_main = (size_t)(TB * LDW + ER * LDW) * 4;
    size_t lds_epi = (size_t)(TB * LDW + TB * (ER + 1)) * 4;
    size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
    auto kern = route_kernel<XT, NEC>;
    if (lds > 48 * 1024) {
        int rc = smoe_check_hip(hipFuncSetAttribute((const void*)kern,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                                "smoe_route: LDS size");
        if (rc) return rc;
    }
    dim3 grid((T + TB - 1) / TB);
    hipLaunchKernelGGL(kern, grid, dim3(THREADS), lds, s, (const XT*)x, L->router_w,
                       L->d_expert_to_slot, T, L->cfg.d_model, L->cfg.E, L->cfg.gate_mode, oe, og, sl, g, xn);
    return smoe_check_hip(hipGetLastError(), "smoe_route launch");
}

template <typename XT>
int dispatch(const smoe_layer* L, const void* x, int T, int32_t* oe, float* og, int32_t* sl, float* g,
             float* xn, hipStream_t s) {
    int nec = (L->cfg.E + 63) / 64;
    switch (nec) {
        case 1: return launch<XT, 1>(L, x, T, oe, og, sl, g, xn, s);
        case 2: return launch<XT, 2>(L, x, T, oe, og, sl, g, xn, s);
        case 3: return launch<XT, 3>(L, x, T, oe, og, sl, g, xn, s);
        case 4: return launch<XT, 4>(L, x, T, oe, og, sl, g, xn, s);
        default: return smoe_fail(SMOE_EINVAL, "smoe_route: E=%d exceeds 256", L->cfg.E);
    }
}

}  // namespace

int smoe_launch_route(const smoe_layer* L, const void* x, int T, int32_t* orig_expert,
                      float* orig_gate, int32_t* slot, float* gate, float* xnorm, hipStream_t s) {
    if (L->cfg.dtype == SMOE_F32)
        return dispatch<float>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, s);
    return dispatch<uint16_t>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, s);
}
