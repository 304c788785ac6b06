// smoe_expert_ffn, bf16 path: y = ReLU(x W1_k) W2_k per slot segment (the
// expert E_i(x) of SwapMoE's Background section; d_model -> d_ff -> ReLU ->
// d_model, no biases) as two grouped GEMMs on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation); the hidden activations are
// rounded to bf16 and kept in the workspace between the two.
//
// Shape of one GEMM:  Y[T, N] = act(X[T, R] . B_k[R, N])  for the rows of slot k.
//
// The weights are the MFMA's first operand and the tokens its second, so an
// accumulator lane ends up holding 4 consecutive output features of ONE token
// and stores them as one 8-byte word; and the token operand (8 consecutive
// reduction elements of one row) is contiguous in the row-major activations.
//
// Weights arrive in fragment order (see resident.hip): every wave streams its
// own feature blocks straight from HBM into registers with contiguous 1-KiB
// loads, prefetched one 64-deep reduction slice ahead -- they never touch LDS,
// since no other wave of the workgroup needs them.  The token tile is what the
// waves share; it is staged through a double-buffered, padded LDS tile.
//
// Workgroup = NW waves; tile = (32*BFR tokens) x (NW*AF*32 features); wave w
// owns AF feature blocks and all BFR token blocks: AF*BFR accumulators of 16
// VGPRs.  Token tiles are enumerated per slot from the device-side offsets.

#include <cstdlib>

#include "smoe_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;             // reduction slice per LDS stage
constexpr int KS = BK / 16;        // MFMA steps per slice
constexpr int LDR = BK + 8;        // LDS row pitch in bf16: 144 B, conflict-free b128 reads

__device__ __forceinline__ bool find_tile(const int32_t* __restrict__ offsets, int nslots, int T, int mt,
                                          int bt, int& slot, int& m0, int& m_end) {
    for (int k = 0; k < nslots; ++k) {
        int a = min(max(offsets[k], 0), T), b = min(max(offsets[k + 1], a), T);   // clamp guards misuse
        int tiles = (b - a + bt - 1) / bt;
        if (mt < tiles) { slot = k; m0 = a + mt * bt; m_end = b; return true; }
        mt -= tiles;
    }
    return false;
}

__device__ __forceinline__ bf16x8 as_frag(uint4 v) {
    union { uint4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

template <int AF, int BFR, int NW, bool RELU>
__global__ __launch_bounds__(NW * 64) void grouped_gemm_bf16(
    const uint16_t* __restrict__ X, const uint4* __restrict__ Wp, const int32_t* __restrict__ offsets,
    int nslots, int T, uint16_t* __restrict__ Y, int R, int N) {
    constexpr int BT = 32 * BFR;
    constexpr int THREADS = NW * 64;
    constexpr int CPT = BT * (BK / 8) / THREADS;      // 16-byte chunks of the token tile per thread
    static_assert(BT * (BK / 8) % THREADS == 0, "token tile must split evenly over the threads");
    __shared__ __align__(16) uint16_t xs[2][BT * LDR];

    int slot, m0, m_end;
    if (!find_tile(offsets, nslots, T, blockIdx.x, BT, slot, m0, m_end)) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nfb = N >> 5;                           // 32-feature blocks in B
    const int nrb = R >> 4;                           // 16-deep reduction blocks in B
    const int fb0 = (blockIdx.y * NW + wave) * AF;
    const int nbf = min(BFR, (m_end - m0 + 31) >> 5); // token blocks that hold real rows
    const int nchunks = (R + BK - 1) / BK;

    // per-feature-block base of this lane's 16-byte units (clamped: surplus blocks
    // recompute the last one and are not stored)
    const uint4* wbase[AF];
#pragma unroll
    for (int a = 0; a < AF; ++a) {
        int fb = min(fb0 + a, nfb - 1);
        wbase[a] = Wp + ((size_t)slot * nfb + fb) * nrb * 64 + lane;
    }

    f32x16 acc[AF][BFR];
#pragma unroll
    for (int a = 0; a < AF; ++a)
#pragma unroll
        for (int b = 0; b < BFR; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    uint4 treg[CPT];
    uint4 wcur[KS][AF], wnext[KS][AF];

    auto load_tokens = [&](int chunk) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int idx = tid + i * THREADS;
            int r = idx >> 3, c = idx & 7;
            int row = min(m0 + r, m_end - 1);
            int col = chunk * BK + c * 8;
            treg[i] = col < R ? *(const uint4*)&X[(size_t)row * R + col] : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_tokens = [&](int stage) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int idx = tid + i * THREADS;
            int r = idx >> 3, c = idx & 7;
            *(uint4*)&xs[stage][r * LDR + c * 8] = treg[i];
        }
    };
    auto load_weights = [&](int chunk, uint4 (&w)[KS][AF]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            int rb = min(chunk * KS + ks, nrb - 1);   // past the end: tokens there are zero
#pragma unroll
            for (int a = 0; a < AF; ++a) w[ks][a] = wbase[a][(size_t)rb * 64];
        }
    };

    load_tokens(0);
    load_weights(0, wcur);
    store_tokens(0);
    __syncthreads();

    for (int chunk = 0; chunk < nchunks; ++chunk) {
        const bool more = chunk + 1 < nchunks;
        if (more) {
            load_tokens(chunk + 1);
            load_weights(chunk + 1, wnext);
        }
        const uint16_t* tile = xs[chunk & 1];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int b = 0; b < BFR; ++b) {
                if (b < nbf) {
                    const int r = b * 32 + (lane & 31);
                    bf16x8 xf = as_frag(*(const uint4*)&tile[r * LDR + ks * 16 + (lane >> 5) * 8]);
#pragma unroll
                    for (int a = 0; a < AF; ++a)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(wcur[ks][a]), xf,
                                                                            acc[a][b], 0, 0, 0);
                }
            }
        }
        if (more) store_tokens((chunk + 1) & 1);
        __syncthreads();
        if (more) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int a = 0; a < AF; ++a) wcur[ks][a] = wnext[ks][a];
        }
    }

    // accumulator register i of lane l: feature 8*(i/4) + 4*(l/32) + i%4, token l%32
#pragma unroll
    for (int a = 0; a < AF; ++a) {
        if (fb0 + a >= nfb) continue;
#pragma unroll
        for (int b = 0; b < BFR; ++b) {
            if (b >= nbf) continue;
            const int row = m0 + b * 32 + (lane & 31);
            if (row >= m_end) continue;
            uint16_t* yrow = Y + (size_t)row * N + (fb0 + a) * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float v0 = acc[a][b][4 * g], v1 = acc[a][b][4 * g + 1], v2 = acc[a][b][4 * g + 2],
                      v3 = acc[a][b][4 * g + 3];
                if (RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                uint2 o;
                o.x = (uint32_t)smoe_f32_to_bf16(v0) | ((uint32_t)smoe_f32_to_bf16(v1) << 16);
                o.y = (uint32_t)smoe_f32_to_bf16(v2) | ((uint32_t)smoe_f32_to_bf16(v3) << 16);
                *(uint2*)(yrow + 8 * g) = o;
            }
        }
    }
}

template <int AF, int BFR, int NW, bool RELU>
void launch_gemm(const uint16_t* X, const void* Wp, const int32_t* offsets, int nslots, uint16_t* Y,
                 int R, int N, int T, hipStream_t s) {
    constexpr int BT = 32 * BFR;
    int mtiles = (T + BT - 1) / BT + nslots;               // upper bound; surplus workgroups exit
    int ftiles = ((N >> 5) + NW * AF - 1) / (NW * AF);
    hipLaunchKernelGGL((grouped_gemm_bf16<AF, BFR, NW, RELU>), dim3(mtiles, ftiles), dim3(NW * 64), 0, s, X,
                       (const uint4*)Wp, offsets, nslots, T, Y, R, N);
}

template <bool RELU>
void launch_variant(int v, const uint16_t* X, const void* Wp, const int32_t* offsets, int nslots,
                    uint16_t* Y, int R, int N, int T, hipStream_t s) {
    switch (v) {
        case 0: launch_gemm<2, 8, 4, RELU>(X, Wp, offsets, nslots, Y, R, N, T, s); break;  // 256 tok x 256 feat
        case 1: launch_gemm<2, 4, 4, RELU>(X, Wp, offsets, nslots, Y, R, N, T, s); break;  // 128 x 256
        case 2: launch_gemm<1, 8, 4, RELU>(X, Wp, offsets, nslots, Y, R, N, T, s); break;  // 256 x 128
        case 3: launch_gemm<1, 4, 4, RELU>(X, Wp, offsets, nslots, Y, R, N, T, s); break;  // 128 x 128
        case 4: launch_gemm<2, 2, 4, RELU>(X, Wp, offsets, nslots, Y, R, N, T, s); break;  //  64 x 256
        case 5: launch_gemm<1, 2, 4, RELU>(X, Wp, offsets, nslots, Y, R, N, T, s); break;  //  64 x 128
        default: launch_gemm<1, 1, 4, RELU>(X, Wp, offsets, nslots, Y, R, N, T, s); break; //  32 x 128
    }
}

// Tile shapes for the two GEMMs.  SMOE_FFN_VARIANT="v1,v2" overrides the
// built-in choice (a tuning aid; the indices are those of launch_variant).
void pick_variants(const smoe_config& c, int T, int& v1, int& v2) {
    int per_slot = T / c.K;
    if (per_slot >= 192) { v1 = 0; v2 = 1; }
    else if (per_slot >= 96) { v1 = 1; v2 = 3; }
    else if (per_slot >= 48) { v1 = 4; v2 = 5; }
    else { v1 = 6; v2 = 6; }
    static const char* env = getenv("SMOE_FFN_VARIANT");
    if (env) {
        int a = -1, b = -1;
        if (sscanf(env, "%d,%d", &a, &b) == 2 && a >= 0 && b >= 0) { v1 = a; v2 = b; }
    }
}

}  // namespace

int smoe_launch_ffn_bf16(const smoe_layer* L, const uint16_t* x_perm, const int32_t* offsets, int T,
                         uint16_t* y_perm, hipStream_t s) {
    const smoe_config& c = L->cfg;
    int v1, v2;
    pick_variants(c, T, v1, v2);
    uint16_t* h = (uint16_t*)L->d_hidden;
    if (L->prof_ev[0]) (void)hipEventRecord(L->prof_ev[0], s);
    launch_variant<true>(v1, x_perm, L->slot_w1, offsets, c.K, h, c.d_model, c.d_ff, T, s);
    if (L->prof_ev[1]) (void)hipEventRecord(L->prof_ev[1], s);
    launch_variant<false>(v2, h, L->slot_w2, offsets, c.K, y_perm, c.d_ff, c.d_model, T, s);
    if (L->prof_ev[2]) (void)hipEventRecord(L->prof_ev[2], s);
    return smoe_check_hip(hipGetLastError(), "smoe_expert_ffn launch");
}
