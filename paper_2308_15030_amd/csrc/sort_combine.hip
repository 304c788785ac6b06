// smoe_importance, smoe_permute and smoe_combine: the memory-bound steps
// around the expert FFN.
//
//  * importance (SwapMoE Eq. 1): one workgroup per expert walks all T tokens
//    and keeps those whose original choice is that expert; a fixed-shape LDS
//    tree gives the three sums, so the result is bit-reproducible (no atomics).
//  * permute: stable counting sort by slot in three launches -- per-block
//    histograms, a ranking pass that turns them into exact positions with
//    wavefront ballots (no atomics on positions, hence one unique, stable
//    order), and a row gather spread over the whole chip.
//  * combine: out[t] = gate[t] * y_perm[inv_perm[t]] (+ residual); top-1 means
//    one source row per token, so this is a gather with 16-byte accesses.

#include <mutex>

#include "smoe_internal.h"

namespace {

// ------------------------------------------------------------- importance
// One workgroup per expert walks all T tokens with coalesced, branch-free loads
// and keeps those whose original choice is that expert; per-thread sums in
// token order and a fixed-shape LDS tree give the three totals, so the result
// is bit-reproducible (no atomics, no dependence on scheduling).
constexpr int IMP_THREADS = 256;

// Thread tid's share of expert e's three sums: tokens tid, tid + 256, ... added
// in that order.  The loads of IMP_UNROLL tokens are issued together, the adds
// stay sequential, so the result does not depend on the unrolling.
constexpr int IMP_UNROLL = 8;

__device__ __forceinline__ void importance_share(const int32_t* __restrict__ orig_expert,
                                                 const float* __restrict__ orig_gate,
                                                 const float* __restrict__ xnorm, int T, int e, int tid,
                                                 int& c, float& g, float& r) {
    c = 0; g = 0.f; r = 0.f;
    int t = tid;
    for (; t + (IMP_UNROLL - 1) * IMP_THREADS < T; t += IMP_UNROLL * IMP_THREADS) {
        int ev[IMP_UNROLL];
        float gv[IMP_UNROLL], xv[IMP_UNROLL];
#pragma unroll
        for (int i = 0; i < IMP_UNROLL; ++i) {
            ev[i] = orig_expert[t + i * IMP_THREADS];
            gv[i] = orig_gate[t + i * IMP_THREADS];
            xv[i] = xnorm[t + i * IMP_THREADS];
        }
#pragma unroll
        for (int i = 0; i < IMP_UNROLL; ++i) {
            c += ev[i] == e;
            g += ev[i] == e ? gv[i] : 0.f;
            r += ev[i] == e ? xv[i] * gv[i] : 0.f;
        }
    }
    for (; t < T; t += IMP_THREADS) {
        int e0 = orig_expert[t];
        float g0 = orig_gate[t], x0 = xnorm[t];
        c += e0 == e;
        g += e0 == e ? g0 : 0.f;
        r += e0 == e ? x0 * g0 : 0.f;
    }
}

__global__ __launch_bounds__(IMP_THREADS) void importance_kernel(
    const int32_t* __restrict__ orig_expert, const float* __restrict__ orig_gate,
    const float* __restrict__ xnorm, const float* __restrict__ expert_norm, int T,
    int32_t* __restrict__ count, float* __restrict__ gsum, float* __restrict__ score, int accumulate) {
    __shared__ int32_t s_c[IMP_THREADS];
    __shared__ float s_g[IMP_THREADS], s_r[IMP_THREADS];
    const int e = blockIdx.x, tid = threadIdx.x;
    int c;
    float g, r;
    importance_share(orig_expert, orig_gate, xnorm, T, e, tid, c, g, r);
    s_c[tid] = c; s_g[tid] = g; s_r[tid] = r;
    __syncthreads();
    for (int w = IMP_THREADS / 2; w > 0; w >>= 1) {
        if (tid < w) { s_c[tid] += s_c[tid + w]; s_g[tid] += s_g[tid + w]; s_r[tid] += s_r[tid + w]; }
        __syncthreads();
    }
    if (tid == 0) {
        float sc = expert_norm[e] * s_r[0];
        if (accumulate) { count[e] += s_c[0]; gsum[e] += s_g[0]; score[e] += sc; }
        else { count[e] = s_c[0]; gsum[e] = s_g[0]; score[e] = sc; }
    }
}

// ------------------------------------------------------------- permute
constexpr int SB = SMOE_SORT_BLOCK;          // tokens (= threads) per sort block
constexpr int SB_WAVES = SB / 64;

__global__ __launch_bounds__(SB) void sort_hist_kernel(const int32_t* __restrict__ slot, int T, int K,
                                                       int32_t* __restrict__ hist) {
    extern __shared__ int32_t s_hist[];      // [K]
    for (int k = threadIdx.x; k < K; k += SB) s_hist[k] = 0;
    __syncthreads();
    int t = blockIdx.x * SB + threadIdx.x;
    if (t < T) {
        int k = slot[t];
        if ((unsigned)k < (unsigned)K) atomicAdd(&s_hist[k], 1);   // integer: order cannot matter
    }
    __syncthreads();
    for (int k = threadIdx.x; k < K; k += SB) hist[(size_t)blockIdx.x * K + k] = s_hist[k];
}

// Position of token t = offsets[slot] + (tokens of that slot in earlier blocks)
//                     + (in earlier waves of this block) + (in lower lanes of this wave).
// With a single block (T <= 1024) the histogram pass is skipped (hist == nullptr)
// and the block's own wave counts give the totals.
__global__ __launch_bounds__(SB) void sort_rank_kernel(const int32_t* __restrict__ slot, int T, int K,
                                                       int nblk, const int32_t* __restrict__ hist,
                                                       int32_t* __restrict__ perm,
                                                       int32_t* __restrict__ inv_perm,
                                                       int32_t* __restrict__ offsets) {
    extern __shared__ int32_t sm[];
    int32_t* s_base = sm;                    // [K]  first position of this block's tokens per slot
    int32_t* s_total = sm + K;               // [K]  tokens per slot over all blocks
    int32_t* s_wave = sm + 2 * K;            // [SB_WAVES][K] per-wave counts -> exclusive prefix
    const int tid = threadIdx.x, blk = blockIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    for (int i = tid; i < SB_WAVES * K; i += SB) s_wave[i] = 0;
    __syncthreads();

    const int t = blk * SB + tid;
    int my = t < T ? slot[t] : -1;
    const bool live = (unsigned)my < (unsigned)K;   // out-of-contract slot values are skipped
    if (!live) my = 0;
    // lanes of this wave that hold the same slot: refine the live mask bit by bit
    unsigned long long peers = __ballot(live);
    for (int bit = 0; (1 << bit) < K; ++bit) {
        unsigned long long b = __ballot(live && ((my >> bit) & 1));
        peers &= ((my >> bit) & 1) ? b : ~b;
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    const int rank_in_wave = __popcll(peers & below);
    if (live && rank_in_wave == 0) s_wave[wave * K + my] = __popcll(peers);
    __syncthreads();
    for (int k = tid; k < K; k += SB) {      // exclusive prefix over the waves, per slot
        int run = 0;
        for (int w = 0; w < SB_WAVES; ++w) {
            int c = s_wave[w * K + k];
            s_wave[w * K + k] = run;
            run += c;
        }
        int before = 0, total = run;
        if (hist) {
            total = 0;
            for (int b = 0; b < nblk; ++b) {
                int h = hist[(size_t)b * K + k];
                if (b < blk) before += h;
                total += h;
            }
        }
        s_base[k] = before;
        s_total[k] = total;
    }
    __syncthreads();
    if (tid == 0) {                          // exclusive scan over slots (K <= 256)
        int run = 0;
        for (int k = 0; k < K; ++k) {
            int tot = s_total[k];
            if (blk == 0) offsets[k] = run;
            s_base[k] += run;
            run += tot;
        }
        if (blk == 0) offsets[K] = run;
    }
    __syncthreads();
    if (live) {
        int pos = s_base[my] + s_wave[wave * K + my] + rank_in_wave;
        perm[pos] = t;
        inv_perm[t] = pos;
    }
}

// Fused launch used by smoe_forward: blocks [0, nblk) rank the tokens exactly as
// sort_rank_kernel does, taking the per-32-token slot histograms the router
// wrote (so no histogram launch); blocks [nblk, nblk + E) are the importance
// reduction, one expert each.  The two halves are independent; sharing a launch
// only saves dispatch latency.
__global__ __launch_bounds__(SB) void rank_importance_kernel(
    const int32_t* __restrict__ slot, int T, int K, int nblk, const int32_t* __restrict__ hist32,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm, int32_t* __restrict__ offsets,
    const int32_t* __restrict__ orig_expert, const float* __restrict__ orig_gate,
    const float* __restrict__ xnorm, const float* __restrict__ expert_norm,
    int32_t* __restrict__ count, float* __restrict__ gsum, float* __restrict__ score, int accumulate) {
    extern __shared__ int32_t sm[];
    const int tid = threadIdx.x;
    if ((int)blockIdx.x >= nblk) {
        // ---- importance of expert e: the first IMP_THREADS threads repeat importance_kernel's
        // summation order exactly (thread j takes tokens j, j+256, ...; fixed LDS tree), so the
        // fused and the separate call give the same bits
        const int e = blockIdx.x - nblk;
        int32_t* s_c = sm;
        float* s_g = (float*)(sm + IMP_THREADS);
        float* s_r = (float*)(sm + 2 * IMP_THREADS);
        if (tid < IMP_THREADS) {
            int c;
            float g, r;
            importance_share(orig_expert, orig_gate, xnorm, T, e, tid, c, g, r);
            s_c[tid] = c; s_g[tid] = g; s_r[tid] = r;
        }
        __syncthreads();
        for (int w = IMP_THREADS / 2; w > 0; w >>= 1) {
            if (tid < w) { s_c[tid] += s_c[tid + w]; s_g[tid] += s_g[tid + w]; s_r[tid] += s_r[tid + w]; }
            __syncthreads();
        }
        if (tid == 0) {
            const float sc = expert_norm[e] * s_r[0];
            if (accumulate) { count[e] += s_c[0]; gsum[e] += s_g[0]; score[e] += sc; }
            else { count[e] = s_c[0]; gsum[e] = s_g[0]; score[e] = sc; }
        }
        return;
    }
    // ---- stable rank of the tokens of sort block blk
    int32_t* s_base = sm;                    // [K]
    int32_t* s_total = sm + K;               // [K]
    int32_t* s_wave = sm + 2 * K;            // [SB_WAVES][K]
    const int blk = blockIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < (2 + SB_WAVES) * K; i += SB) sm[i] = 0;
    __syncthreads();
    {   // totals and "before this block" from the router's histograms (integer adds: order-free)
        const int nrb = (T + 31) / 32, first_rb = blk * (SB / 32);
        for (int idx = tid; idx < nrb * K; idx += SB) {
            const int rb = idx / K, k = idx - rb * K;
            const int h = hist32[idx];
            if (h) {
                atomicAdd(&s_total[k], h);
                if (rb < first_rb) atomicAdd(&s_base[k], h);
            }
        }
    }
    const int t = blk * SB + tid;
    int my = t < T ? slot[t] : -1;
    const bool live = (unsigned)my < (unsigned)K;
    if (!live) my = 0;
    unsigned long long peers = __ballot(live);
    for (int bit = 0; (1 << bit) < K; ++bit) {
        unsigned long long b = __ballot(live && ((my >> bit) & 1));
        peers &= ((my >> bit) & 1) ? b : ~b;
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    const int rank_in_wave = __popcll(peers & below);
    if (live && rank_in_wave == 0) s_wave[wave * K + my] = __popcll(peers);
    __syncthreads();
    for (int k = tid; k < K; k += SB) {      // exclusive prefix over the waves, per slot
        int run = 0;
        for (int w = 0; w < SB_WAVES; ++w) {
            int c = s_wave[w * K + k];
            s_wave[w * K + k] = run;
            run += c;
        }
    }
    __syncthreads();
    if (tid == 0) {                          // exclusive scan over slots
        int run = 0;
        for (int k = 0; k < K; ++k) {
            int tot = s_total[k];
            if (blk == 0) offsets[k] = run;
            s_base[k] += run;
            run += tot;
        }
        if (blk == 0) offsets[K] = run;
    }
    __syncthreads();
    if (live) {
        int pos = s_base[my] + s_wave[wave * K + my] + rank_in_wave;
        perm[pos] = t;
        inv_perm[t] = pos;
    }
}

// x_perm[pos, :] = x[perm[pos], :], 16 bytes per thread.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ x,
                                                          const int32_t* __restrict__ perm, int T,
                                                          int chunks_per_row, uint4* __restrict__ x_perm) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)T * chunks_per_row;
    if (idx >= total) return;
    int pos = (int)(idx / chunks_per_row), c = (int)(idx % chunks_per_row);
    int src = min(max(perm[pos], 0), T - 1);         // in range by construction; clamp guards misuse
    x_perm[idx] = x[(size_t)src * chunks_per_row + c];
}

// ------------------------------------------------------------- combine
template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ y_perm,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ gate,
                                                      const uint4* __restrict__ residual, int T,
                                                      int chunks_per_row, uint4* __restrict__ out) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)T * chunks_per_row;
    if (idx >= total) return;
    int t = (int)(idx / chunks_per_row), c = (int)(idx % chunks_per_row);
    const float g = gate[t];
    int src = min(max(inv_perm[t], 0), T - 1);
    uint4 y = y_perm[(size_t)src * chunks_per_row + c];
    uint4 r = residual ? residual[idx] : make_uint4(0, 0, 0, 0);
    uint32_t yw[4] = {y.x, y.y, y.z, y.w}, rw[4] = {r.x, r.y, r.z, r.w}, ow[4];
    if (BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float lo = __uint_as_float(yw[i] << 16), hi = __uint_as_float(yw[i] & 0xFFFF0000u);
            if (residual) {
                lo = fmaf(g, lo, __uint_as_float(rw[i] << 16));
                hi = fmaf(g, hi, __uint_as_float(rw[i] & 0xFFFF0000u));
            } else {
                lo *= g;
                hi *= g;
            }
            ow[i] = (uint32_t)smoe_f32_to_bf16(lo) | ((uint32_t)smoe_f32_to_bf16(hi) << 16);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v = __uint_as_float(yw[i]);
            v = residual ? fmaf(g, v, __uint_as_float(rw[i])) : g * v;
            ow[i] = __float_as_uint(v);
        }
    }
    out[idx] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
}

}  // namespace

int smoe_launch_importance(const smoe_layer* L, const int32_t* orig_expert, const float* orig_gate,
                           const float* xnorm, int T, int32_t* count, float* gsum, float* score,
                           int accumulate, hipStream_t s) {
    hipLaunchKernelGGL(importance_kernel, dim3(L->cfg.E), dim3(IMP_THREADS), 0, s, orig_expert,
                       orig_gate, xnorm, L->expert_norm, T, count, gsum, score, accumulate);
    return smoe_check_hip(hipGetLastError(), "smoe_importance launch");
}

int smoe_launch_permute(const smoe_layer* L, const void* x, const int32_t* slot, int T, void* x_perm,
                        int32_t* perm, int32_t* inv_perm, int32_t* offsets, hipStream_t s) {
    const int K = L->cfg.K;
    const int nblk = T > 0 ? smoe_sort_blocks(T) : 1;       // T = 0 still writes offsets = 0
    if (nblk > 1)
        hipLaunchKernelGGL(sort_hist_kernel, dim3(nblk), dim3(SB), K * sizeof(int32_t), s, slot, T, K,
                           L->d_sort_hist);
    hipLaunchKernelGGL(sort_rank_kernel, dim3(nblk), dim3(SB), (2 + SB_WAVES) * K * sizeof(int32_t), s,
                       slot, T, K, nblk, nblk > 1 ? L->d_sort_hist : nullptr, perm, inv_perm, offsets);
    if (T > 0) {
        int cpr = (int)((size_t)L->cfg.d_model * smoe_elem_size(L->cfg.dtype) / 16);
        size_t total = (size_t)T * cpr;
        hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const uint4*)x, perm, T, cpr, (uint4*)x_perm);
    }
    return smoe_check_hip(hipGetLastError(), "smoe_permute launch");
}

// ---------------------------------------------------------------------------
// smoe_permute for callers that may not allocate and have no workspace to bind:
// the per-block slot histograms, the one piece of device memory the sort needs
// beyond its inputs and outputs, live in a fixed array inside the library
// image instead of the bound workspace.  Every GPU the library runs on holds
// its own copy of the array (64 KiB) from the moment the code object is loaded
// until the process ends, at an address of its own, which is asked of the
// runtime once per device; host code never uses the array's name for anything
// else (the name is a host-side stand-in, not a device address).
constexpr int STATIC_MAX_TOKENS = 65536;                         // 64 sort blocks
constexpr int STATIC_MAX_SLOTS = 256;                            // K <= E <= 256 by the C ABI
constexpr int STATIC_HIST_INTS = (STATIC_MAX_TOKENS / SMOE_SORT_BLOCK) * STATIC_MAX_SLOTS;
static __device__ __align__(256) int32_t scratch[STATIC_HIST_INTS];

constexpr int MAX_DEVICES = 64;
static int32_t* g_scratch_ptr[MAX_DEVICES];                      // device address of `scratch`, per device
static std::mutex g_scratch_mu;

// Address of this device's copy of the array (the current device), or an error.
static int static_scratch(int32_t** out) {
    int dev = -1;
    int rc = smoe_check_hip(hipGetDevice(&dev), "smoe_permute_static: current device");
    if (rc) return rc;
    if (dev < 0 || dev >= MAX_DEVICES)
        return smoe_fail(SMOE_EINVAL, "smoe_permute_static: device index %d outside [0,%d)", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        rc = smoe_check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "smoe_permute_static: scratch address");
        if (rc) return rc;
        if (!p) return smoe_fail(SMOE_EHIP, "smoe_permute_static: the runtime returned no address for the scratch array");
        g_scratch_ptr[dev] = (int32_t*)p;
    }
    *out = g_scratch_ptr[dev];
    return SMOE_OK;
}

int smoe_static_max_tokens() { return STATIC_MAX_TOKENS; }

// Same three launches as smoe_launch_permute; only the histogram buffer differs.  Nothing in
// the array has to start at zero: the histogram launch overwrites every entry the ranking
// launch reads ([blocks of this call][K]), so a smaller call after a larger one is safe.
int smoe_launch_permute_static(const smoe_config& c, const void* x, const int32_t* slot, int T, void* x_perm,
                               int32_t* perm, int32_t* inv_perm, int32_t* offsets, hipStream_t s) {
    const int K = c.K;
    const int nblk = T > 0 ? smoe_sort_blocks(T) : 1;
    int32_t* hist = nullptr;
    if (nblk > 1) {
        int rc = static_scratch(&hist);
        if (rc) return rc;
        hipLaunchKernelGGL(sort_hist_kernel, dim3(nblk), dim3(SB), K * sizeof(int32_t), s, slot, T, K, hist);
    }
    hipLaunchKernelGGL(sort_rank_kernel, dim3(nblk), dim3(SB), (2 + SB_WAVES) * K * sizeof(int32_t), s,
                       slot, T, K, nblk, hist, perm, inv_perm, offsets);
    if (T > 0) {
        int cpr = (int)((size_t)c.d_model * smoe_elem_size(c.dtype) / 16);
        size_t total = (size_t)T * cpr;
        hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const uint4*)x, perm, T, cpr, (uint4*)x_perm);
    }
    return smoe_check_hip(hipGetLastError(), "smoe_permute_static launch");
}

int smoe_launch_rank_importance(const smoe_layer* L, const int32_t* orig_expert, const float* orig_gate,
                                const float* xnorm, const int32_t* slot, int T, int32_t* count, float* gsum,
                                float* score, int accumulate, int32_t* perm, int32_t* inv_perm,
                                int32_t* offsets, hipStream_t s) {
    const int K = L->cfg.K, E = L->cfg.E;
    const int nblk = smoe_sort_blocks(T);
    size_t lds = (size_t)(2 + SB_WAVES) * K * sizeof(int32_t);
    if (lds < 3 * IMP_THREADS * sizeof(int32_t)) lds = 3 * IMP_THREADS * sizeof(int32_t);
    hipLaunchKernelGGL(rank_importance_kernel, dim3(nblk + E), dim3(SB), lds, s, slot, T, K, nblk, L->d_hist32,
                       perm, inv_perm, offsets, orig_expert, orig_gate, xnorm, L->expert_norm, count, gsum,
                       score, accumulate);
    return smoe_check_hip(hipGetLastError(), "smoe_forward: sort/importance launch");
}

int smoe_launch_combine(const smoe_layer* L, const void* y_perm, const int32_t* inv_perm,
                        const float* gate, const void* residual, int T, void* out, hipStream_t s) {
    int cpr = (int)((size_t)L->cfg.d_model * smoe_elem_size(L->cfg.dtype) / 16);
    size_t total = (size_t)T * cpr;
    dim3 grid((unsigned)((total + 255) / 256));
    if (L->cfg.dtype == SMOE_BF16)
        hipLaunchKernelGGL(combine_kernel<true>, grid, dim3(256), 0, s, (const uint4*)y_perm, inv_perm,
                           gate, (const uint4*)residual, T, cpr, (uint4*)out);
    else
        hipLaunchKernelGGL(combine_kernel<false>, grid, dim3(256), 0, s, (const uint4*)y_perm, inv_perm,
                           gate, (const uint4*)residual, T, cpr, (uint4*)out);
    return smoe_check_hip(hipGetLastError(), "smoe_combine launch");
}
