// smoe_expert_ffn, fp32 path: y = ReLU(x W1_k) W2_k per slot segment (the
// expert E_i(x) of SwapMoE's Background section, d_model -> d_ff -> ReLU ->
// d_model, no biases) as two grouped fp32 GEMMs with plain FMA chains.
//
// This path exists for exactness checks at fp32 (tolerance 1e-4), not for
// speed: every output element is one sequential fp32 FMA chain in ascending
// reduction index, independent of the tiling.  A workgroup owns a 32-row x
// 64-column output tile of one slot's segment; row tiles are enumerated per
// slot from the device-side offsets, so no host read-back is needed.

#include "smoe_internal.h"

namespace {

constexpr int BM = 32, BN = 64, BK = 16;

// Finds the slot and row range of row-tile `mt`, counting ceil(len/BM) tiles
// per slot in slot order.  Returns false when mt is past the last tile.
__device__ __forceinline__ bool find_tile(const int32_t* __restrict__ offsets, int nslots, int T, int mt,
                                          int bm, int& slot, int& m0, int& m_end) {
    for (int k = 0; k < nslots; ++k) {
        int a = min(max(offsets[k], 0), T), b = min(max(offsets[k + 1], a), T);   // clamp guards misuse
        int tiles = (b - a + bm - 1) / bm;
        if (mt < tiles) { slot = k; m0 = a + mt * bm; m_end = b; return true; }
        mt -= tiles;
    }
    return false;
}

template <bool RELU>
__global__ __launch_bounds__(256) void grouped_gemm_f32(const float* __restrict__ X,
                                                        const float* __restrict__ W,
                                                        const int32_t* __restrict__ offsets,
                                                        const int32_t* __restrict__ phys, int nslots, int T,
                                                        float* __restrict__ Y, int R, int N) {
    __shared__ float xs[BM][BK + 1];
    __shared__ __align__(16) float ws[BK][BN];
    int slot, m0, m_end;
    if (!find_tile(offsets, nslots, T, blockIdx.x, BM, slot, m0, m_end)) return;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int n0 = blockIdx.y * BN;
    const float* Wk = W + (size_t)phys[slot] * R * N;
    float acc[2][4] = {};
    for (int k0 = 0; k0 < R; k0 += BK) {
        __syncthreads();
        if (tid < BM * BK / 4) {              // 128 threads: one float4 of x each
            int r = tid >> 2, c = (tid & 3) * 4;
            int row = min(m0 + r, m_end - 1);
            float4 v = make_float4(0, 0, 0, 0);
            if (k0 + c < R) v = *(const float4*)&X[(size_t)row * R + k0 + c];
            xs[r][c] = v.x; xs[r][c + 1] = v.y; xs[r][c + 2] = v.z; xs[r][c + 3] = v.w;
        }
        {
            int r = tid >> 4, c = (tid & 15) * 4;
            float4 v = make_float4(0, 0, 0, 0);
            if (k0 + r < R && n0 + c < N) v = *(const float4*)&Wk[(size_t)(k0 + r) * N + n0 + c];
            *(float4*)&ws[r][c] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a0 = xs[2 * ty][kk], a1 = xs[2 * ty + 1][kk];
            float4 w = *(const float4*)&ws[kk][tx * 4];
            acc[0][0] = fmaf(a0, w.x, acc[0][0]); acc[0][1] = fmaf(a0, w.y, acc[0][1]);
            acc[0][2] = fmaf(a0, w.z, acc[0][2]); acc[0][3] = fmaf(a0, w.w, acc[0][3]);
            acc[1][0] = fmaf(a1, w.x, acc[1][0]); acc[1][1] = fmaf(a1, w.y, acc[1][1]);
            acc[1][2] = fmaf(a1, w.z, acc[1][2]); acc[1][3] = fmaf(a1, w.w, acc[1][3]);
        }
    }
    const int c = n0 + tx * 4;
    if (c >= N) return;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        int row = m0 + 2 * ty + a;
        if (row >= m_end) continue;
        float4 v = make_float4(acc[a][0], acc[a][1], acc[a][2], acc[a][3]);
        if (RELU) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
        *(float4*)&Y[(size_t)row * N + c] = v;
    }
}

}  // namespace

int smoe_launch_ffn_f32(const smoe_layer* L, const float* x_perm, const int32_t* offsets, int T,
                        float* y_perm, hipStream_t s) {
    const smoe_config& c = L->cfg;
    const int mtiles = (T + BM - 1) / BM + c.K;            // upper bound; surplus workgroups exit
    float* h = (float*)L->d_hidden;
    smoe_launch_timed(grouped_gemm_f32<true>, dim3(mtiles, (c.d_ff + BN - 1) / BN), dim3(256), s, L->prof_ev[0],
                      L->prof_ev[1], x_perm, (const float*)L->slot_w1, offsets, L->d_phys, c.K, T, h, c.d_model,
                      c.d_ff);
    smoe_launch_timed(grouped_gemm_f32<false>, dim3(mtiles, (c.d_model + BN - 1) / BN), dim3(256), s,
                      L->prof_ev[2], L->prof_ev[3], (const float*)h, (const float*)L->slot_w2, offsets, L->d_phys, c.K, T,
                      y_perm, c.d_ff, c.d_model);
    return smoe_check_hip(hipGetLastError(), "smoe_expert_ffn launch");
}
