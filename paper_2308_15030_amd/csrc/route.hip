// smoe_route: router product, softmax, original top-1, masked top-1 and |x|.
//
// For every token:  logit = x . Wr^T,  p = softmax(logit) over all E experts,
// e* = argmax logit (SwapMoE, Background: the expert with max G(x)_i), and the
// Masked-Gating choice s = argmax over resident experts only (Section 3.1,
// Figure 4(b)).  |x|_2 is produced on the way because x is already in flight
// (it is the first factor of the importance score, Eq. 1).
//
// fp32 activations (route_kernel; the bf16 kernel has its own description below):
// one workgroup of 256 threads owns 32 tokens and all E experts.  x and Wr are
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
    float* __restrict__ gate, float* __restrict__ xnorm, int32_t* __restrict__ hist32, int K) {
    extern __shared__ __align__(16) float smem[];
    __shared__ int32_t s_slot[TB];
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
        const int sv = rbi < ER ? s_e2s[rbi] : 0;   // rbi is always valid once every slot is set
        slot[tok] = sv;
        s_slot[st] = sv;
        gate[tok] = gate_mode == SMOE_GATE_RENORM ? ps / zr : ps / z;
        xnorm[tok] = sqrtf(sq);
    }
    if (hist32) {                                 // tokens per slot in this block, for the fused sort
        __syncthreads();
        const int n = min(TB, T - t0);
        for (int k = tid; k < K; k += THREADS) {
            int c = 0;
            for (int i = 0; i < n; ++i) c += s_slot[i] == k;
            hist32[(size_t)blockIdx.x * K + k] = c;
        }
    }
}

// ---------------------------------------------------------------------------
// bf16 activations: the router product on the matrix cores at fp32 accuracy.
//
// x is exactly bf16, and an fp32 router weight is exactly the sum of three
// bf16 numbers (8 + 8 + 8 significand bits): w = hi + mid + lo.  Every product
// x * {hi, mid, lo} is exact in fp32, so three bf16 MFMA passes with fp32
// accumulation give the fp32-weight logits up to accumulation rounding -- the
// same error class as an fp32 FMA chain, at matrix-core speed.  The split
// weights are kept in MFMA operand order in the workspace (made on the first
// smoe_route after smoe_bind).
//
// One workgroup = one or two blocks of 32 tokens x all experts.  Its NWR waves
// (8 up to 64 experts, 4 above) split the reduction (d_model) NWR ways, each
// accumulating a partial [experts x tokens] tile; the partials meet in LDS and
// are added in wave order (fixed, so results are reproducible).  In the
// epilogue every thread takes part: lane l of wave w owns token l % 32 and
// every (2 NWR)-th expert, and the per-token arg-max, masked arg-max and softmax
// sums meet through small LDS tables, again in wave order.

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 frag_of(uint4 v) {
    union { uint4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

// Wr [E, d] fp32 -> units [eb][kb][split][lane] of 8 bf16: expert eb*32 + lane%32,
// reduction index kb*16 + (lane/32)*8 + i.  Experts past E are zero.
__global__ __launch_bounds__(256) void split_router_kernel(const float* __restrict__ Wr, int E, int d,
                                                           uint4* __restrict__ out, int neb) {
    int unit = blockIdx.x * 256 + threadIdx.x;             // (eb * nkb + kb) * 64 + lane
    int nkb = d >> 4;
    if (unit >= neb * nkb * 64) return;
    int lane = unit & 63, kb = (unit >> 6) % nkb, eb = (unit >> 6) / nkb;
    int e = eb * 32 + (lane & 31), k0 = kb * 16 + (lane >> 5) * 8;
    uint32_t hi[8], mid[8], lo[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float w = e < E ? Wr[(size_t)e * d + k0 + i] : 0.f;
        uint16_t h = smoe_f32_to_bf16(w);
        float r1 = w - smoe_bf16_to_f32(h);                // exact
        uint16_t m = smoe_f32_to_bf16(r1);
        float r2 = r1 - smoe_bf16_to_f32(m);               // exact
        hi[i] = h; mid[i] = m; lo[i] = smoe_f32_to_bf16(r2);
    }
    uint4* dst = out + ((size_t)(eb * nkb + kb) * 3) * 64 + lane;
    dst[0] = make_uint4(hi[0] | hi[1] << 16, hi[2] | hi[3] << 16, hi[4] | hi[5] << 16, hi[6] | hi[7] << 16);
    dst[64] = make_uint4(mid[0] | mid[1] << 16, mid[2] | mid[3] << 16, mid[4] | mid[5] << 16, mid[6] | mid[7] << 16);
    dst[128] = make_uint4(lo[0] | lo[1] << 16, lo[2] | lo[3] << 16, lo[4] | lo[5] << 16, lo[6] | lo[7] << 16);
}

constexpr int RT = 32;            // tokens per token block (one MFMA operand)

// A batch of at most RT tokens is one workgroup, which then holds every token's
// result and can finish the step's ranking (smoe_permute's index part) and the
// importance sums (Eq. 1) itself: the single-call path saves a launch.
// perm == nullptr: plain router.
struct TailArgs {
    const float* expert_norm;
    int32_t* count;
    float* gsum;
    float* score;
    int accumulate;
    int32_t* perm;
    int32_t* inv_perm;
    int32_t* offsets;
};

// NEB = 32-expert blocks, NWR = waves per workgroup (each takes 1/NWR of d_model),
// TB = 32-token blocks per workgroup: every workgroup streams the whole router once, so
// when the batch has more 32-token blocks than the chip has compute units a workgroup takes
// two blocks and the weights are fetched half as often.
template <int NEB, int NWR, int TB>
__device__ __forceinline__ void route_mfma_body(
    const int block, const uint16_t* __restrict__ x, const uint4* __restrict__ Wsplit, const int32_t* __restrict__ e2s,
    int T, int d, int E, int gate_mode,
    int32_t* __restrict__ orig_expert, float* __restrict__ orig_gate, int32_t* __restrict__ slot,
    float* __restrict__ gate, float* __restrict__ xnorm, int32_t* __restrict__ hist32, int K,
    const TailArgs tail) {
    extern __shared__ __align__(16) float smem[];
    __shared__ int32_t s_slot[RT];
    __shared__ int32_t s_oe[RT];                  // per-token results kept for the single-workgroup tail
    __shared__ float s_og[RT], s_xn[RT];
    constexpr int EP = NEB * 32;
    constexpr int THREADS = NWR * 64;
    // reduction steps whose operands are fetched together, so that one memory
    // round trip feeds several MFMAs: bounded by registers (1 + 3*NEB loads per step)
    constexpr int G = NEB == 1 ? 8 : NEB == 2 ? 6 : NEB <= 5 ? 2 : 1;
    constexpr int CP = RT * TB + 1;               // padded row of the partial-logit tile
    float* part = smem;                           // [NWR waves][EP][CP] partial logits
    float* sqp = smem + NWR * EP * CP;            // [NWR waves][2 halves][TB][RT] partial sums of squares
    __shared__ int32_t s_e2s[EP];

    // wave index as a scalar: loop bounds that guard MFMAs must be wave-uniform for the
    // compiler as well (an MFMA under a lane mask still runs for every lane)
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int tw0 = block * RT * TB;              // first token of the workgroup
    for (int e = tid; e < EP; e += THREADS) s_e2s[e] = e < E ? e2s[e] : -1;

    const int nkb = d >> 4;
    const int per = (nkb + NWR - 1) / NWR;
    const int kb_lo = min(wave * per, nkb), kb_hi = min(kb_lo + per, nkb);
    const uint16_t* xp[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int trow = min(tw0 + tb * RT + (lane & 31), T - 1);
        xp[tb] = x + (size_t)trow * d + (lane >> 5) * 8;
    }
    const uint4* wp = Wsplit + lane;

    f32x16 acc[NEB][TB];
    float sq[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        sq[tb] = 0.f;
#pragma unroll
        for (int b = 0; b < NEB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][tb][i] = 0.f;
    }

    for (int g0 = kb_lo; g0 < kb_hi; g0 += G) {
        uint4 xv[G][TB];
        uint4 w[G][NEB][3];
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const int kb = min(g0 + i, kb_hi - 1);            // past the end: reloaded, not used
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) xv[i][tb] = *(const uint4*)(xp[tb] + kb * 16);
#pragma unroll
            for (int b = 0; b < NEB; ++b)
#pragma unroll
                for (int s3 = 0; s3 < 3; ++s3) w[i][b][s3] = wp[((size_t)(b * nkb + kb) * 3 + s3) * 64];
        }
        __builtin_amdgcn_sched_barrier(0);                    // all of the group's loads are issued first
#pragma unroll
        for (int i = 0; i < G; ++i) {
            bf16x8 xf[TB];
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                // steps past the end of the range contribute a zero token operand
                const uint4 xz = g0 + i < kb_hi ? xv[i][tb] : make_uint4(0, 0, 0, 0);
                uint32_t xw[4] = {xz.x, xz.y, xz.z, xz.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float a = __uint_as_float(xw[q] << 16), c = __uint_as_float(xw[q] & 0xFFFF0000u);
                    sq[tb] = fmaf(a, a, sq[tb]);
                    sq[tb] = fmaf(c, c, sq[tb]);
                }
                xf[tb] = frag_of(xz);
            }
            // smallest terms first, so they are not absorbed by the large partial sums
#pragma unroll
            for (int s3 = 2; s3 >= 0; --s3)
#pragma unroll
                for (int b = 0; b < NEB; ++b)
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
                        acc[b][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_of(w[i][b][s3]), xf[tb], acc[b][tb],
                                                                             0, 0, 0);
        }
    }
    // accumulator register i of lane l: expert 8*(i/4) + 4*(l/32) + i%4 (+32 per block), token l%32
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
#pragma unroll
        for (int b = 0; b < NEB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int e = b * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                part[(wave * EP + e) * CP + tb * RT + (lane & 31)] = acc[b][tb][i];
            }
        sqp[((wave * 2 + (lane >> 5)) * TB + tb) * RT + (lane & 31)] = sq[tb];
    }
    __syncthreads();

    for (int tb = 0; tb < TB; ++tb) {                 // one 32-token block at a time through the epilogue
    const int t0 = tw0 + tb * RT;
    if (TB > 1 && t0 >= T) break;                     // uniform: the batch ended inside this workgroup

    // epilogue: lane l of wave w owns token l%32 and the experts j, j + 2*NWR, ... with
    // j = 2w + l/32, so a wave's LDS reads walk consecutive tokens (no bank conflicts) and
    // every thread takes part; the per-token results meet through small LDS tables.
    constexpr int EG = 2 * NWR;                   // expert groups per token
    constexpr int EPL = EP / EG;                  // experts per lane
    __shared__ float s_best[NWR][RT], s_rbest[NWR][RT], s_z[NWR][RT], s_zr[NWR][RT];
    __shared__ int32_t s_bi[NWR][RT], s_rbi[NWR][RT];
    const int st = lane & 31, half = lane >> 5;
    // Everything below is written with selects, not branches: a compare-and-update under a
    // lane mask costs the wave a jump per candidate.  Experts past E carry -inf, which never
    // wins and adds exp(-inf) = 0 to the sums.
    auto better = [](float ov, int oi, float& bv, int& bidx) {   // the lowest index wins a tie
        const bool take = (ov > bv) | ((ov == bv) & (oi < bidx));   // no short circuit: no jumps
        bv = take ? ov : bv;
        bidx = take ? oi : bidx;
    };
    float v[EPL];
    bool res[EPL];
    float best = -INFINITY, rbest = -INFINITY;
    int bi = 0x7fffffff, rbi = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const int e = wave * 2 + half + EG * i;
        float sum = part[e * CP + tb * RT + st];
#pragma unroll
        for (int w = 1; w < NWR; ++w) sum += part[(w * EP + e) * CP + tb * RT + st];   // fixed order
        res[i] = s_e2s[e] >= 0;                   // -1 past E as well
        v[i] = e < E ? sum : -INFINITY;
        better(v[i], e, best, bi);                // ascending e within the lane
        better(res[i] ? v[i] : -INFINITY, res[i] ? e : 0x7fffffff, rbest, rbi);
    }
    better(__shfl_xor(best, 32), __shfl_xor(bi, 32), best, bi);
    better(__shfl_xor(rbest, 32), __shfl_xor(rbi, 32), rbest, rbi);
    if (half == 0) { s_best[wave][st] = best; s_bi[wave][st] = bi; s_rbest[wave][st] = rbest; s_rbi[wave][st] = rbi; }
    __syncthreads();
    {
        float wb[NWR], wrb[NWR];
        int wi[NWR], wri[NWR];
#pragma unroll
        for (int w = 0; w < NWR; ++w) {           // all the reads first, then the merges in wave order
            wb[w] = s_best[w][st]; wi[w] = s_bi[w][st]; wrb[w] = s_rbest[w][st]; wri[w] = s_rbi[w][st];
        }
        best = wb[0]; bi = wi[0]; rbest = wrb[0]; rbi = wri[0];
#pragma unroll
        for (int w = 1; w < NWR; ++w) {
            better(wb[w], wi[w], best, bi);
            better(wrb[w], wri[w], rbest, rbi);
        }
    }
    float z = 0.f, zr = 0.f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const float p = expf(v[i] - best);
        z += p;
        zr += res[i] ? p : 0.f;
    }
    z += __shfl_xor(z, 32);
    zr += __shfl_xor(zr, 32);
    if (half == 0) { s_z[wave][st] = z; s_zr[wave][st] = zr; }
    __syncthreads();
    if (tid < RT && t0 + tid < T) {               // st == tid: one lane per token finishes
        const int tok = t0 + tid;
        z = s_z[0][st]; zr = s_zr[0][st];
#pragma unroll
        for (int w = 1; w < NWR; ++w) { z += s_z[w][st]; zr += s_zr[w][st]; }
        float ss = 0.f;
#pragma unroll
        for (int q = 0; q < 2 * NWR; ++q) ss += sqp[(q * TB + tb) * RT + st];
        const float ps = expf(rbest - best);
        orig_expert[tok] = bi;
        orig_gate[tok] = 1.0f / z;
        const int sv = rbi < EP ? s_e2s[rbi] : 0;    // rbi is always valid once every slot is set
        slot[tok] = sv;
        s_slot[st] = sv;
        gate[tok] = gate_mode == SMOE_GATE_RENORM ? ps / zr : ps / z;
        const float xn = sqrtf(ss);
        xnorm[tok] = xn;
        s_oe[st] = bi; s_og[st] = 1.0f / z; s_xn[st] = xn;      // for the single-workgroup tail
    }
    if (hist32) {                                 // tokens per slot in this block, for the fused sort
        __syncthreads();
        const int n = min(RT, T - t0);
        for (int k = tid; k < K; k += THREADS) {
            int c = 0;
            for (int i = 0; i < n; ++i) c += s_slot[i] == k;
            hist32[((size_t)block * TB + tb) * K + k] = c;
        }
    }
    if (TB > 1) __syncthreads();                      // the tables are reused by the next block
    }
    if (TB > 1 || !tail.perm) return;
    // ---- single-workgroup tail (T <= RT, one workgroup): ranking and importance
    __shared__ int32_t s_cnt[256], s_off[256];
    for (int k = tid; k < 256; k += THREADS) s_cnt[k] = 0;
    __syncthreads();
    // stable rank by slot (wave 0): position = slot offset + earlier tokens of the same slot,
    // exactly the order of the sorting kernels
    int my = 0, rank_in_slot = 0;
    const bool live = wave == 0 && lane < T;
    if (wave == 0) {
        my = live ? s_slot[lane & 31] : 0;
        unsigned long long peers = __ballot(live);
        for (int bit = 0; (1 << bit) < K; ++bit) {
            const unsigned long long b = __ballot(live && ((my >> bit) & 1));
            peers &= ((my >> bit) & 1) ? b : ~b;
        }
        rank_in_slot = __popcll(peers & ((1ull << lane) - 1ull));
        if (live && rank_in_slot == 0) s_cnt[my] = __popcll(peers);
    }
    __syncthreads();
    if (wave == 0) {                              // exclusive scan of the slot counts, 64 slots at a time
        int before = 0;
        for (int base = 0; base < K; base += 64) {
            const int k = base + lane;
            const int c = k < K ? s_cnt[k] : 0;
            int incl = c;
#pragma unroll
            for (int dd = 1; dd < 64; dd <<= 1) {
                const int o = __shfl_up(incl, dd);
                if (lane >= dd) incl += o;
            }
            if (k < K) { s_off[k] = before + incl - c; tail.offsets[k] = before + incl - c; }
            before += __shfl(incl, 63);
        }
        if (lane == 0) tail.offsets[K] = before;
    }
    __syncthreads();
    if (live) {
        const int pos = s_off[my] + rank_in_slot;
        tail.perm[pos] = lane;
        tail.inv_perm[lane] = pos;
    }
    // importance: thread e sums expert e's tokens (those whose own top-1 it is).  The tokens sit
    // in leaves 0..31 of the separate call's 256-leaf summation tree and its other leaves are
    // zero, so evaluating that tree's last five levels in registers gives the same bits.
    if (tid < E) {
        const int e = tid;
        const float en = tail.expert_norm[e];                 // asked for before the arithmetic
        int c0 = 0;
        float g0 = 0.f, r0 = 0.f;
        if (tail.accumulate) { c0 = tail.count[e]; g0 = tail.gsum[e]; r0 = tail.score[e]; }
        int c = 0;
        float g[RT], r[RT];
#pragma unroll
        for (int t = 0; t < RT; ++t) {                         // same address in every lane: LDS broadcasts
            const bool hit = (t < T) & (s_oe[t] == e);
            c += hit;
            g[t] = hit ? s_og[t] : 0.f;
            r[t] = hit ? s_xn[t] * s_og[t] : 0.f;
        }
#pragma unroll
        for (int w = RT / 2; w > 0; w >>= 1)
#pragma unroll
            for (int i = 0; i < w; ++i) { g[i] += g[i + w]; r[i] += r[i + w]; }
        const float sc = en * r[0];
        tail.count[e] = c0 + c;
        tail.gsum[e] = tail.accumulate ? g0 + g[0] : g[0];
        tail.score[e] = tail.accumulate ? r0 + sc : sc;
    }
}

template <int NEB, int NWR, int TB>
__global__ __launch_bounds__(NWR * 64) void route_mfma_kernel(
    const uint16_t* __restrict__ x, const uint4* __restrict__ Wsplit, const int32_t* __restrict__ e2s,
    int T, int d, int E, int gate_mode,
    int32_t* __restrict__ orig_expert, float* __restrict__ orig_gate, int32_t* __restrict__ slot,
    float* __restrict__ gate, float* __restrict__ xnorm, int32_t* __restrict__ hist32, int K,
    const TailArgs tail) {
    route_mfma_body<NEB, NWR, TB>(blockIdx.x, x, Wsplit, e2s, T, d, E, gate_mode, orig_expert, orig_gate, slot, gate, xnorm,
                                  hist32, K, tail);
}

// ---------------------------------------------------------------------------
// Decode step, first launch (bf16, at most 32 tokens, at most 64 experts): the router and the
// first FFN product side by side.  The router of a 32-token batch is one workgroup that needs
// ~9 us for 340 KB of operands, a softmax epilogue and the ranking tail, while the other 255
// compute units wait for its slot ids only to learn which slots are empty.  Here the first
// workgroup of the launch is that router, and the others compute the first product for EVERY
// slot and EVERY token of the batch at once: workgroup (slot, feature tile) multiplies all T
// tokens, staged once in LDS, by the slot's weight tile and stores the hidden activations
// h[slot][feature / 8][token] for all of them.  An MFMA column depends on its own token only
// and the reduction runs in the same order as in the other FFN kernels, so the columns that
// the second product later picks (the tokens routed to the slot) hold the same bits as on the
// sorted path.  The price is the weight matrices of the slots nobody was routed to (3 of 16 on
// the decode workload, +24 % bytes for this launch); what it buys is the router's whole time.
// 8 waves per workgroup, one 32-feature block per wave; the token operands come from LDS
// (row pitch d_model + 8 elements: conflict-free 16-byte reads), so the vector-memory pipe
// carries nothing but the 1-KiB weight loads, 16 of them in flight per wave.
// STREAM: the weight loads are marked non-temporal (see smoe_weights_outgrow_cache).
template <bool STREAM>
__device__ __forceinline__ void dense_first_all(const uint16_t* __restrict__ x, const uint4* __restrict__ Wp,
                                                int T, uint16_t* __restrict__ h, int R, int N,
                                                const int32_t* __restrict__ phys, int block) {
    extern __shared__ __align__(16) float smem[];
    uint16_t* xs = (uint16_t*)smem;                        // [32][R + 8]
    constexpr int G = 8, NWV = 8;
    const int nfb = N >> 5, nrb = R >> 4, ldx = R + 8;
    const int ftiles = (nfb + NWV - 1) / NWV;
    const int slot = block / ftiles, ftile = block - slot * ftiles;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int fb = ftile * NWV + wave;
    const bool fb_ok = fb < nfb;
    const uint4* wp = Wp + ((size_t)(phys ? phys[slot] : slot) * nfb + min(fb, nfb - 1)) * nrb * 64 + lane;
    uint4 wA[G], wB[G];
    auto fetch_w = [&](uint4 (&w)[G], int g0) {
#pragma unroll
        for (int i = 0; i < G; ++i) {                      // past the end: reloaded, not used
            const uint4* src = wp + (size_t)min(g0 + i, nrb - 1) * 64;
            w[i] = STREAM ? smoe_load_stream(src) : *src;
        }
    };
    fetch_w(wA, 0);                                        // on their way while the tokens are staged
    const int cpr = R >> 3;                                // 16-byte pieces per token row
    for (int idx = tid; idx < 32 * cpr; idx += NWV * 64) {
        const int r = idx / cpr, c = idx - r * cpr;
        uint4 v = make_uint4(0, 0, 0, 0);                  // rows past the batch are zero
        if (r < T) v = *(const uint4*)(x + (size_t)r * R + c * 8);
        *(uint4*)&xs[r * ldx + c * 8] = v;
    }
    __syncthreads();
    const uint16_t* xrow = xs + (lane & 31) * ldx + (lane >> 5) * 8;
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    auto consume = [&](uint4 (&w)[G], int g0) {
#pragma unroll
        for (int i = 0; i < G; ++i) {
            // steps past the end of the reduction multiply by a zero token operand
            const uint4 xv = g0 + i < nrb ? *(const uint4*)(xrow + (size_t)min(g0 + i, nrb - 1) * 16) : make_uint4(0, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_of(w[i]), frag_of(xv), acc, 0, 0, 0);
        }
    };
    for (int g0 = 0; g0 < nrb; g0 += 2 * G) {
        fetch_w(wB, g0 + G);
        __builtin_amdgcn_sched_barrier(0);
        consume(wA, g0);
        __builtin_amdgcn_sched_barrier(0);
        fetch_w(wA, g0 + 2 * G);
        __builtin_amdgcn_sched_barrier(0);
        consume(wB, g0 + G);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (!fb_ok) return;
    // accumulator register i of lane l: feature 8*(i/4) + 4*(l/32) + i%4, token l%32
    uint16_t* ydst = h + (((size_t)slot * (N >> 3) + fb * 4) * 32 + (lane & 31)) * 8 + (lane >> 5) * 4;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const float v0 = fmaxf(acc[4 * g], 0.f), v1 = fmaxf(acc[4 * g + 1], 0.f), v2 = fmaxf(acc[4 * g + 2], 0.f),
                    v3 = fmaxf(acc[4 * g + 3], 0.f);
        uint2 o;
        o.x = (uint32_t)smoe_f32_to_bf16(v0) | ((uint32_t)smoe_f32_to_bf16(v1) << 16);
        o.y = (uint32_t)smoe_f32_to_bf16(v2) | ((uint32_t)smoe_f32_to_bf16(v3) << 16);
        *(uint2*)(ydst + g * 32 * 8) = o;
    }
}

#define SMOE_DECODE_FIRST_PARAMS                                                                            \
    const uint16_t* __restrict__ x, const uint4* __restrict__ Wsplit, const int32_t* __restrict__ e2s,          \
    int T, int d, int E, int gate_mode, int32_t* __restrict__ orig_expert, float* __restrict__ orig_gate,       \
    int32_t* __restrict__ slot, float* __restrict__ gate, float* __restrict__ xnorm, int K, const TailArgs tail, \
    const uint4* __restrict__ W1, uint16_t* __restrict__ h, int d_ff, const int32_t* __restrict__ phys

// Workgroup 0 is the router: it is the launch's critical path, so it is dispatched first.
template <int NEB, bool STREAM>
__device__ __forceinline__ void decode_first_body(SMOE_DECODE_FIRST_PARAMS) {
    if (blockIdx.x == 0)
        route_mfma_body<NEB, 8, 1>(0, x, Wsplit, e2s, T, d, E, gate_mode, orig_expert, orig_gate, slot, gate, xnorm,
                                   nullptr, K, tail);
    else
        dense_first_all<STREAM>(x, W1, T, h, d, d_ff, phys, blockIdx.x - 1);
}

// Two kernels with one body: the second streams its weights past the caches.
template <int NEB>
__global__ __launch_bounds__(512) void decode_first_kernel(SMOE_DECODE_FIRST_PARAMS) {
    decode_first_body<NEB, false>(x, Wsplit, e2s, T, d, E, gate_mode, orig_expert, orig_gate, slot, gate, xnorm, K, tail,
                                  W1, h, d_ff, phys);
}

template <int NEB>
__global__ __launch_bounds__(512) void decode_first_stream_kernel(SMOE_DECODE_FIRST_PARAMS) {
    decode_first_body<NEB, true>(x, Wsplit, e2s, T, d, E, gate_mode, orig_expert, orig_gate, slot, gate, xnorm, K, tail,
                                 W1, h, d_ff, phys);
}

template <int NEB, int TB>
int launch_mfma_tb(const smoe_layer* L, const void* x, int T, int32_t* oe, float* og, int32_t* sl, float* g,
                   float* xn, int32_t* hist32, const TailArgs& tail, hipStream_t s) {
    constexpr int EP = NEB * 32;
    constexpr int NWR = NEB <= 2 ? 8 : 4;
    size_t lds = (size_t)(NWR * EP * (RT * TB + 1) + 2 * NWR * RT * TB) * 4;
    auto kern = route_mfma_kernel<NEB, NWR, TB>;
    if (lds > 48 * 1024) {   // raise the kernel's dynamic-LDS limit once per device, not on every launch
        static int raised_on = -1;
        int dev_now = 0;
        (void)hipGetDevice(&dev_now);
        if (raised_on != dev_now) {
            int rc = smoe_check_hip(hipFuncSetAttribute((const void*)kern,
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                                    "smoe_route: LDS size");
            if (rc) return rc;
            raised_on = dev_now;
        }
    }
    hipLaunchKernelGGL(kern, dim3((T + RT * TB - 1) / (RT * TB)), dim3(NWR * 64), lds, s, (const uint16_t*)x,
                       (const uint4*)L->d_router_split, L->d_expert_to_slot, T, L->cfg.d_model, L->cfg.E,
                       L->cfg.gate_mode, oe, og, sl, g, xn, hist32, L->cfg.K, tail);
    return smoe_check_hip(hipGetLastError(), "smoe_route launch");
}

template <int NEB>
int launch_mfma(const smoe_layer* L, const void* x, int T, int32_t* oe, float* og, int32_t* sl, float* g,
                float* xn, int32_t* hist32, const TailArgs& tail, hipStream_t s) {
    // more 32-token blocks than compute units (256): two blocks per workgroup, while the partial-logit
    // tile of 64 tokens still fits the LDS (up to 128 experts)
    if constexpr (NEB <= 4) {
        if ((T + RT - 1) / RT > 256 && !tail.perm)
            return launch_mfma_tb<NEB, 2>(L, x, T, oe, og, sl, g, xn, hist32, tail, s);
    }
    return launch_mfma_tb<NEB, 1>(L, x, T, oe, og, sl, g, xn, hist32, tail, s);
}

template <typename XT, int NEC>
int launch(const smoe_layer* L, const void* x, int T, int32_t* oe, float* og, int32_t* sl, float* g,
           float* xn, int32_t* hist32, hipStream_t s) {
    constexpr int ER = 64 * NEC;
    size_t lds_main = (size_t)(TB * LDW + ER * LDW) * 4;
    size_t lds_epi = (size_t)(TB * LDW + TB * (ER + 1)) * 4;
    size_t lds = lds_main > lds_epi ? lds_main : lds_epi;
    auto kern = route_kernel<XT, NEC>;
    if (lds > 48 * 1024) {   // raise the kernel's dynamic-LDS limit once per device, not on every launch
        static int raised_on = -1;
        int dev_now = 0;
        (void)hipGetDevice(&dev_now);
        if (raised_on != dev_now) {
            int rc = smoe_check_hip(hipFuncSetAttribute((const void*)kern,
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                                    "smoe_route: LDS size");
            if (rc) return rc;
            raised_on = dev_now;
        }
    }
    dim3 grid((T + TB - 1) / TB);
    hipLaunchKernelGGL(kern, grid, dim3(THREADS), lds, s, (const XT*)x, L->router_w,
                       L->d_expert_to_slot, T, L->cfg.d_model, L->cfg.E, L->cfg.gate_mode, oe, og, sl, g, xn,
                       hist32, L->cfg.K);
    return smoe_check_hip(hipGetLastError(), "smoe_route launch");
}

template <typename XT>
int dispatch(const smoe_layer* L, const void* x, int T, int32_t* oe, float* og, int32_t* sl, float* g,
             float* xn, int32_t* hist32, hipStream_t s) {
    int nec = (L->cfg.E + 63) / 64;
    switch (nec) {
        case 1: return launch<XT, 1>(L, x, T, oe, og, sl, g, xn, hist32, s);
        case 2: return launch<XT, 2>(L, x, T, oe, og, sl, g, xn, hist32, s);
        case 3: return launch<XT, 3>(L, x, T, oe, og, sl, g, xn, hist32, s);
        case 4: return launch<XT, 4>(L, x, T, oe, og, sl, g, xn, hist32, s);
        default: return smoe_fail(SMOE_EINVAL, "smoe_route: E=%d exceeds 256", L->cfg.E);
    }
}

}  // namespace

int smoe_launch_split_router(const smoe_layer* L, hipStream_t s) {
    const int neb = (L->cfg.E + 31) / 32;
    const int units = neb * (L->cfg.d_model >> 4) * 64;
    hipLaunchKernelGGL(split_router_kernel, dim3((units + 255) / 256), dim3(256), 0, s, L->router_w, L->cfg.E,
                       L->cfg.d_model, (uint4*)L->d_router_split, neb);
    return smoe_check_hip(hipGetLastError(), "smoe_route: router split launch");
}

namespace {

int route_bf16(const smoe_layer* L, const void* x, int T, int32_t* orig_expert, float* orig_gate,
               int32_t* slot, float* gate, float* xnorm, int32_t* hist32, const TailArgs& tail, hipStream_t s) {
    switch ((L->cfg.E + 31) / 32) {
        case 1: return launch_mfma<1>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, tail, s);
        case 2: return launch_mfma<2>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, tail, s);
        case 3: return launch_mfma<3>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, tail, s);
        case 4: return launch_mfma<4>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, tail, s);
        case 5: return launch_mfma<5>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, tail, s);
        case 6: return launch_mfma<6>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, tail, s);
        case 7: return launch_mfma<7>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, tail, s);
        case 8: return launch_mfma<8>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, tail, s);
        default: return smoe_fail(SMOE_EINVAL, "smoe_route: E=%d exceeds 256", L->cfg.E);
    }
}

}  // namespace

int smoe_launch_route(const smoe_layer* L, const void* x, int T, int32_t* orig_expert,
                      float* orig_gate, int32_t* slot, float* gate, float* xnorm, int32_t* hist32,
                      hipStream_t s) {
    if (L->cfg.dtype == SMOE_F32)
        return dispatch<float>(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, s);
    return route_bf16(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, hist32, TailArgs{}, s);
}

// bf16 layers, 1 <= T <= 32, E <= 64: router (with the ranking tail) and the first FFN product of
// every slot in one launch.  e0 / e1 (optional) take the launch's start and end.
static size_t decode_first_lds(const smoe_config& c) {
    const int ep = (c.E + 31) / 32 * 32;
    const size_t lds_router = (size_t)(8 * ep * (RT + 1) + 2 * 8 * RT) * 4;      // partial logits of 8 waves + norms
    const size_t lds_tokens = (size_t)RT * (c.d_model + 8) * 2;                  // the batch, staged for the first product
    return lds_router > lds_tokens ? lds_router : lds_tokens;
}

bool smoe_decode_first_applies(const smoe_layer* L, int T) {
    return L->cfg.dtype == SMOE_BF16 && T >= 1 && T <= RT && L->cfg.E <= 64 && decode_first_lds(L->cfg) <= 120 * 1024;
}

int smoe_launch_decode_first(const smoe_layer* L, const void* x, int T, int32_t* orig_expert, float* orig_gate,
                             int32_t* slot, float* gate, float* xnorm, int32_t* count, float* gsum, float* score,
                             int accumulate, int32_t* perm, int32_t* inv_perm, int32_t* offsets, hipStream_t s,
                             hipEvent_t e0, hipEvent_t e1) {
    if (!smoe_decode_first_applies(L, T)) return smoe_fail(SMOE_EINVAL, "smoe_forward: the fused decode launch does not apply");
    const smoe_config& c = L->cfg;
    const TailArgs tail{L->expert_norm, count, gsum, score, accumulate, perm, inv_perm, offsets};
    const int neb = (c.E + 31) / 32;
    const size_t lds = decode_first_lds(c);
    const int ftiles = ((c.d_ff >> 5) + 7) / 8;
    const dim3 grid(c.K * ftiles + 1);
    const int32_t* phys = c.spare_slots > 0 ? L->d_phys : nullptr;
    auto launch = [&](auto kern) -> int {
        // raise the kernel's dynamic-LDS limit once per kernel and device (the four instances share
        // one function type, hence one instance of this lambda: the table is keyed by the pointer)
        static const void* raised_kern[8];
        static int raised_dev[8];
        static int nraised = 0;
        int dev_now = 0;
        (void)hipGetDevice(&dev_now);
        if (lds > 48 * 1024) {
            bool done = false;
            for (int i = 0; i < nraised; ++i) done |= raised_kern[i] == (const void*)kern && raised_dev[i] == dev_now;
            if (!done) {
                int rc = smoe_check_hip(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 120 * 1024),
                                        "smoe_forward: LDS size");
                if (rc) return rc;
                if (nraised < 8) { raised_kern[nraised] = (const void*)kern; raised_dev[nraised] = dev_now; ++nraised; }
            }
        }
        if (e0 && e1)
            hipExtLaunchKernelGGL(kern, grid, dim3(512), lds, s, e0, e1, 0, (const uint16_t*)x, (const uint4*)L->d_router_split,
                                  L->d_expert_to_slot, T, c.d_model, c.E, c.gate_mode, orig_expert, orig_gate, slot, gate, xnorm,
                                  c.K, tail, (const uint4*)L->slot_w1, (uint16_t*)L->d_hidden, c.d_ff, phys);
        else
            hipLaunchKernelGGL(kern, grid, dim3(512), lds, s, (const uint16_t*)x, (const uint4*)L->d_router_split,
                               L->d_expert_to_slot, T, c.d_model, c.E, c.gate_mode, orig_expert, orig_gate, slot, gate, xnorm,
                               c.K, tail, (const uint4*)L->slot_w1, (uint16_t*)L->d_hidden, c.d_ff, phys);
        return smoe_check_hip(hipGetLastError(), "smoe_forward: decode launch");
    };
    if (smoe_weights_outgrow_cache())
        return neb == 1 ? launch(decode_first_stream_kernel<1>) : launch(decode_first_stream_kernel<2>);
    return neb == 1 ? launch(decode_first_kernel<1>) : launch(decode_first_kernel<2>);
}

// bf16 layers, 1 <= T <= 32: the router's single workgroup also ranks the tokens by slot
// and adds the importance sums, so the step needs no second launch.
int smoe_launch_route_rank_small(const smoe_layer* L, const void* x, int T, int32_t* orig_expert,
                                 float* orig_gate, int32_t* slot, float* gate, float* xnorm, int32_t* count,
                                 float* gsum, float* score, int accumulate, int32_t* perm, int32_t* inv_perm,
                                 int32_t* offsets, hipStream_t s) {
    if (L->cfg.dtype != SMOE_BF16 || T < 1 || T > RT)
        return smoe_fail(SMOE_EINVAL, "smoe_forward: the one-launch router needs bf16 and 1..%d tokens", RT);
    const TailArgs tail{L->expert_norm, count, gsum, score, accumulate, perm, inv_perm, offsets};
    return route_bf16(L, x, T, orig_expert, orig_gate, slot, gate, xnorm, nullptr, tail, s);
}
