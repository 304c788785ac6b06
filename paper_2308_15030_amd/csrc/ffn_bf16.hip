// smoe_expert_ffn, bf16 path: y = ReLU(x W1_k) W2_k per slot segment (the
// expert E_i(x) of SwapMoE's Background section; d_model -> d_ff -> ReLU ->
// d_model, no biases) as two grouped GEMMs on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation); the hidden activations are
// rounded to bf16 and kept in the workspace between the two.
//
// Shape of one GEMM:  Y[T, N] = act(X[T, R] . B_k[R, N])  for the rows of slot k.
//
// The weights are the MFMA's first operand and the tokens its second, so an
// accumulator lane ends up holding 4 consecutive output features of ONE token,
// and the token operand is 8 consecutive reduction elements of one row.
//
// Weights arrive in fragment order (see resident.hip): every wave streams its
// own feature blocks straight from HBM into registers with contiguous 1-KiB
// loads, prefetched PD reduction slices ahead in a register ring -- they never
// touch LDS, since no other wave of the workgroup needs them.  The token tile
// is what the waves share; it is staged through a three-stage LDS ring.
//
// The hidden activations h never leave the library, so they are kept in
// fragment order too: rows are re-based per segment to a multiple of 32
// ("padded rows"), and h is stored as 16-byte units [row/32][feature/8][row%32]
// of 8 features.  The first GEMM's accumulator layout then stores straight into
// 512-byte runs, and the second GEMM stages its token tile with a linear copy
// and reads operands from LDS without padding or bank conflicts.
//
// Workgroup = NW waves; tile = (32*MAXB tokens) x (NW*AF*32 features); wave w
// owns AF feature blocks and all token blocks: AF*NBF accumulators of 16 VGPRs.
// Token tiles are enumerated per slot from the device-side offsets; the tiled
// kernel runs as persistent workgroups that each walk a fixed share of the tiles.

#include <algorithm>
#include <cstdio>
#include <string>
#include <type_traits>

#include "smoe_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int KPAD = 8;   // row-major token tile: LDS pitch (BKT+8)*2 B keeps b128 reads conflict-free

constexpr int XCDS = 8;   // MI355X: 8 accelerator dies, each with a private L2

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int o = __shfl_up(v, d);
        if (lane >= d) v += o;
    }
    return v;
}

// ---------------------------------------------------------------------------
// Work enumeration of the tiled kernel.  A work item is (row tile, feature
// tile); the row tiles of all slots form one list in slot order, ceil(len/bt)
// per slot.  Workgroups are dealt to the 8 XCDs round-robin by their linear id,
// so workgroup wg runs on XCD wg % 8.  The items are numbered slot by slot --
// inside a slot with the feature tile fastest (second product: g = mt * ftiles
// + ft) or with the row tile fastest (first product, see the kernel) -- and die
// x owns the x-th eighth of that list: the dies' shares differ by at most one
// item (a split by whole row tiles can leave one die with a fifth more work and
// a whole extra round of tiles) and a share still covers few slots, whose
// token or weight tiles the die's workgroups share through its L2.  The grid
// holds as many workgroups as the chip keeps resident; the j-th workgroup of a
// die takes the die's items j, j + n, j + 2n, ... (n workgroups per die).  Each
// workgroup builds the per-slot tables once, in LDS.
constexpr int MAX_SLOTS = 256;            // K <= E <= 256 by the C ABI

struct ItemMap {
    int first[MAX_SLOTS + 1];             // row tiles before slot k; [nslots] = all row tiles
    int pad[MAX_SLOTS];                   // padded rows (segments re-based to multiples of 32) before slot k
    int a[MAX_SLOTS], b[MAX_SLOTS];       // clamped segment bounds
};

// Called by every thread of the workgroup; ends with a barrier.
__device__ __forceinline__ void build_item_map(ItemMap& m, const int32_t* __restrict__ offsets, int nslots,
                                               int T, int bt) {
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        int tiles_before = 0, pad_before = 0;
        for (int base = 0; base < nslots; base += 64) {
            const int k = base + lane;
            int a = 0, b = 0, tiles = 0, pad = 0;
            if (k < nslots) {
                a = min(max(offsets[k], 0), T);                 // clamps guard misuse
                b = max(min(max(offsets[k + 1], 0), T), a);
                tiles = (b - a + bt - 1) / bt;
                pad = (b - a + 31) & ~31;
            }
            const int tin = wave_incl_scan(tiles, lane), pin = wave_incl_scan(pad, lane);
            if (k < nslots) {
                m.first[k] = tiles_before + tin - tiles;
                m.pad[k] = pad_before + pin - pad;
                m.a[k] = a;
                m.b[k] = b;
            }
            tiles_before += __shfl(tin, 63);
            pad_before += __shfl(pin, 63);
        }
        if (lane == 0) m.first[nslots] = tiles_before;
    }
    __syncthreads();
}

// Row tile mt of the global list: its slot, first row, segment end and padded
// first row.  Every wave works this out for itself; the results are scalars.
__device__ __forceinline__ void row_tile_at(const ItemMap& m, int nslots, int bt, int mt, int& slot, int& m0,
                                            int& m_end, int& pm0) {
    const int lane = threadIdx.x & 63;
    int nle = 0;                                               // slots whose first row tile is <= mt
    for (int base = 0; base < nslots; base += 64) {
        const int k = base + lane;
        nle += __popcll(__ballot(k < nslots && m.first[k] <= mt));
    }
    const int k = __builtin_amdgcn_readfirstlane(nle - 1);     // the last of them holds mt (empty slots repeat the next first)
    const int within = mt - __builtin_amdgcn_readfirstlane(m.first[k]);
    slot = k;
    m0 = __builtin_amdgcn_readfirstlane(m.a[k]) + within * bt;
    m_end = __builtin_amdgcn_readfirstlane(m.b[k]);
    pm0 = __builtin_amdgcn_readfirstlane(m.pad[k]) + within * bt;
}

__device__ __forceinline__ bf16x8 as_frag(uint4 v) {
    union { uint4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

// Optional fusion of the permute and combine steps into the two products
// (perm == nullptr: plain products on x_perm / y_perm).
//   first product:  row r of the sorted order is read from x[perm[r]] (no x_perm);
//   second product: row r is written to out[perm[r]] = gate[perm[r]] * y (+ residual[perm[r]]),
//                   i.e. y = G(x)_i E_i(x) lands in token order (no y_perm).
struct FuseArgs {
    const int32_t* phys;      // virtual slot -> physical weight slot, [nslots]; NULL = identity (no spare slots)
    const int32_t* perm;
    const float* gate;
    const uint16_t* residual;
};

// Fused combine on 4 consecutive outputs of one token.  The product is first
// rounded to bf16 exactly as the unfused path stores y_perm, so both paths give
// the same bits; then out = gate * y (+ residual) in fp32 with one final rounding.
__device__ __forceinline__ void apply_gate_v(float& v0, float& v1, float& v2, float& v3, float g, uint2 r,
                                             bool has_res, bool fused) {
    if (!fused) return;
    v0 = smoe_bf16_to_f32(smoe_f32_to_bf16(v0)); v1 = smoe_bf16_to_f32(smoe_f32_to_bf16(v1));
    v2 = smoe_bf16_to_f32(smoe_f32_to_bf16(v2)); v3 = smoe_bf16_to_f32(smoe_f32_to_bf16(v3));
    if (has_res) {
        v0 = fmaf(g, v0, __uint_as_float(r.x << 16)); v1 = fmaf(g, v1, __uint_as_float(r.x & 0xFFFF0000u));
        v2 = fmaf(g, v2, __uint_as_float(r.y << 16)); v3 = fmaf(g, v3, __uint_as_float(r.y & 0xFFFF0000u));
    } else {
        v0 *= g; v1 *= g; v2 *= g; v3 *= g;
    }
}

__device__ __forceinline__ void apply_gate(float& v0, float& v1, float& v2, float& v3, float g,
                                           const uint16_t* res, bool fused) {
    uint2 r = make_uint2(0, 0);
    if (fused && res) r = *(const uint2*)res;
    apply_gate_v(v0, v1, v2, v3, g, r, res != nullptr, fused);
}

// One workgroup tile with NBF live token blocks.  Everything is compile-time
// shaped: no branch inside the reduction loop.
//   AF    feature blocks per wave          NW    waves per workgroup
//   BKT   reduction slice per LDS stage    PD    weight prefetch distance in slices
//   XFRAG token operand X is in fragment order (else row-major [T, R])
//   YFRAG output Y is written in fragment order (else row-major [T, N])
template <int AF, int NBF, int NW, int BKT, int PD, bool XFRAG, bool YFRAG, bool RELU, bool EARLY>
__device__ __forceinline__ void run_tile(const uint16_t* __restrict__ X, const uint4* __restrict__ Wp,
                                         uint16_t* __restrict__ Y, int R, int N, int slot, int m0,
                                         int m_end, int pm0, int ftile, uint16_t* xs, int stage_elems,
                                         int* orow, float* ogate, const FuseArgs fz) {
    constexpr int THREADS = NW * 64;
    constexpr int KS = BKT / 16;
    constexpr int LDR = BKT + KPAD;
    constexpr int CPR = BKT / 8;                          // 16-byte pieces per token row and slice
    constexpr int PIECES = 32 * NBF * CPR;                // pieces of the token tile per slice
    constexpr int CPT = (PIECES + THREADS - 1) / THREADS;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nfb = N >> 5, nrb = R >> 4;
    const int fb0 = (ftile * NW + wave) * AF;
    const int nchunks = R / BKT;

    const uint4* wbase[AF];
#pragma unroll
    for (int a = 0; a < AF; ++a) {
        int fb = min(fb0 + a, nfb - 1);                   // surplus blocks recompute the last one, unstored
        wbase[a] = Wp + ((size_t)slot * nfb + fb) * nrb * 64 + lane;
    }
    // this thread's pieces of the token tile: global source, its stride per slice, LDS destination
    const uint16_t* tsrc[CPT];
    int tdst[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        int idx = min(tid + i * THREADS, PIECES - 1);     // surplus threads repeat the last piece
        if (XFRAG) {
            int b = idx / (CPR * 32), j = (idx / 32) % CPR, t = idx % 32;
            tsrc[i] = X + (((size_t)((pm0 >> 5) + b) * (R >> 3) + j) * 32 + t) * 8;
            tdst[i] = idx * 8;
        } else {
            int r = idx / CPR, c = idx % CPR;
            int row = min(m0 + r, m_end - 1);
            if (fz.perm) row = fz.perm[row];
            tsrc[i] = X + (size_t)row * R + c * 8;
            tdst[i] = r * LDR + c * 8;
        }
    }
    const size_t tstep = XFRAG ? (size_t)CPR * 32 * 8 : (size_t)BKT;     // elements per slice
    // this lane's operand inside token block 0, reduction step 0; per block / per step strides
    const int xoff = XFRAG ? ((lane >> 5) * 32 + (lane & 31)) * 8 : (lane & 31) * LDR + (lane >> 5) * 8;
    constexpr int XB = XFRAG ? CPR * 32 * 8 : 32 * LDR;   // token block stride in LDS
    constexpr int XK = XFRAG ? 2 * 32 * 8 : 16;           // reduction step stride in LDS

    // Row-major output: where each row of the tile goes (out[perm[row]] in the single-call
    // path, y_perm[row] otherwise; -1 past the segment's end) and its gate are fetched now,
    // a whole reduction before the epilogue needs them.
    if (!YFRAG) {
        for (int r = tid; r < 32 * NBF; r += THREADS) {
            int dst = -1;
            float g = 1.f;
            if (m0 + r < m_end) {
                dst = fz.perm ? fz.perm[m0 + r] : m0 + r;
                if (fz.perm) g = fz.gate[dst];
            }
            orow[r] = dst;
            ogate[r] = g;
        }
    }

    f32x16 acc[AF][NBF];
#pragma unroll
    for (int a = 0; a < AF; ++a)
#pragma unroll
        for (int b = 0; b < NBF; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // Software pipeline over the reduction slices c = 0 .. nchunks-1.
    //   weights: a ring of PD+1 slices in registers, loaded PD slices ahead;
    //   tokens:  TD register sets, loaded TD+1 slices ahead, written to LDS one
    //            slice ahead; LDS holds three stages (slice c in stage c % 3);
    //   operands: the next MFMA step's LDS reads are issued before the current
    //            step's MFMAs, across the slice boundary as well.
    // The one barrier per slice sits in the MIDDLE of the slice's MFMA steps: it
    // publishes stage (c+1)%3, written at the top of slice c, before the first
    // read of it at the bottom of slice c, and it orders the last reads of slice
    // c-1 (all issued before it) ahead of the writes that recycle that stage at
    // the top of slice c+1.  So no wave ever waits at a barrier with an empty
    // matrix pipe behind it.
    // Loads past the last slice are clamped to it (fetched again, never used),
    // so the loop body has no conditional loads.
    // With more than 4 token blocks the operand reads are pipelined in two
    // half-steps of the block range, which halves the operand registers.
    constexpr int TD = ((PD & 1) && AF * NBF < 16) ? 2 : 1;   // the largest tile keeps one set only
    constexpr int NG = NBF > 4 ? 2 : 1;                   // operand groups per reduction step
    constexpr int GB = (NBF + NG - 1) / NG;               // token blocks per group
    constexpr int NSTEP = KS * NG;
    static_assert(KS % 2 == 0, "the operand double buffer assumes an even number of steps per slice");
    uint4 tregA[CPT], tregB[CPT];                       // token register sets 0 and 1
    uint4 wbuf[PD + 1][KS][AF];
    bf16x8 xf[2][GB];
#pragma unroll
    for (int i = 0; i < CPT; ++i) tregA[i] = *(const uint4*)tsrc[i];
#pragma unroll
    for (int p = 0; p < PD; ++p) {
        const int cp = min(p, nchunks - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int a = 0; a < AF; ++a) wbuf[p][ks][a] = wbase[a][(size_t)(cp * KS + ks) * 64];
    }
    if (TD == 2) {
        const int c1 = min(1, nchunks - 1);
#pragma unroll
        for (int i = 0; i < CPT; ++i) tregB[i] = *(const uint4*)(tsrc[i] + (size_t)c1 * tstep);
    }
#pragma unroll
    for (int i = 0; i < CPT; ++i) *(uint4*)&xs[tdst[i]] = tregA[i];
    {   // set 0 is free again: it takes slice TD (the slice after the ones already loaded)
        const int c2 = min(TD, nchunks - 1);
#pragma unroll
        for (int i = 0; i < CPT; ++i) tregA[i] = *(const uint4*)(tsrc[i] + (size_t)c2 * tstep);
    }
    __syncthreads();
    // Row-major output, single-call path: the residual rows come from far away by now (two
    // weight streams have passed through the caches since x was read), so small tiles ask for
    // their pieces here and carry them through the reduction in registers.
    constexpr int OF = NW * AF * 32;                      // features of the workgroup tile
    constexpr int OCPR = OF / 8;                          // 16-byte pieces per output row
    constexpr int ONP = YFRAG ? 1 : 32 * NBF * OCPR / THREADS;   // pieces per thread (2 * NBF * AF)
    constexpr bool EARLY_RES = !YFRAG && EARLY;           // the launcher knows the register budget
    // small tiles store straight from the accumulator layout: this lane's rows and gates, taken
    // from the tables now (the next tile refills the tables while slower waves are still storing)
    constexpr int NDIRECT = (!YFRAG && NBF <= 2 && !EARLY) ? NBF : 1;
    int drow[NDIRECT];
    float dgate[NDIRECT];
    if constexpr (!YFRAG && NBF <= 2 && !EARLY) {
#pragma unroll
        for (int b = 0; b < NBF; ++b) {
            drow[b] = orow[b * 32 + (lane & 31)];
            dgate[b] = ogate[b * 32 + (lane & 31)];
        }
    }
    uint4 res[EARLY_RES ? ONP : 1];
    if (EARLY_RES && fz.perm && fz.residual) {
#pragma unroll
        for (int i = 0; i < ONP; ++i) {
            const int idx = tid + i * THREADS, r = idx / OCPR, c = idx % OCPR;
            const int col = ftile * OF + c * 8, row = col < N ? orow[r] : -1;
            res[i] = make_uint4(0, 0, 0, 0);
            if (row >= 0) res[i] = *(const uint4*)(fz.residual + (size_t)row * N + col);
        }
    }
#pragma unroll
    for (int b = 0; b < GB; ++b) xf[0][b] = as_frag(*(const uint4*)&xs[xoff + b * XB]);

    int st = 0;                                           // LDS stage of the current slice
    // nchunks is a multiple of PD+1 (the launcher picks PD so; PD is 0, 1 or 3),
    // and every ring index below is a compile-time constant.
    auto slice = [&](auto uc, int c0) {
        constexpr int u = decltype(uc)::value;            // position in the ring: compile-time
        const int c = c0 + u;
        const int cw = min(c + PD, nchunks - 1), ct = min(c + TD + 1, nchunks - 1);
        const int st1 = st == 2 ? 0 : st + 1;
        const uint16_t* tile = xs + st * stage_elems + xoff;
        const uint16_t* tile1 = xs + st1 * stage_elems + xoff;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int a = 0; a < AF; ++a)
                wbuf[(u + PD) % (PD + 1)][ks][a] = wbase[a][(size_t)(cw * KS + ks) * 64];
        // the set that holds slice c+1 goes to stage (c+1)%3 and is reloaded with slice c+TD+1
        uint16_t* dst = xs + st1 * stage_elems;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            if constexpr ((u + 1) % TD == 0) *(uint4*)&dst[tdst[i]] = tregA[i];
            else *(uint4*)&dst[tdst[i]] = tregB[i];
        }
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            uint4 v = *(const uint4*)(tsrc[i] + (size_t)ct * tstep);
            if constexpr ((u + 1) % TD == 0) tregA[i] = v; else tregB[i] = v;
        }
        __builtin_amdgcn_sched_barrier(0);                // keep the prefetches ahead of the math
#pragma unroll
        for (int t = 0; t < NSTEP; ++t) {
            const int ks = t / NG, g = t % NG;
            if (t == NSTEP / 2) __syncthreads();          // stage (c+1)%3 is complete from here on
            {   // operands of step t+1: the next group, the next reduction step, or the next slice
                const int t1 = t + 1;
                const int ks1 = (t1 % NSTEP) / NG, g1 = t1 % NG;
                const uint16_t* src = (t1 == NSTEP ? tile1 : tile) + ks1 * XK;
#pragma unroll
                for (int b = 0; b < GB; ++b)
                    if (g1 * GB + b < NBF) xf[t1 & 1][b] = as_frag(*(const uint4*)&src[(g1 * GB + b) * XB]);
            }
            __builtin_amdgcn_sched_barrier(0);            // next step's operands are on their way
#pragma unroll
            for (int b = 0; b < GB; ++b)
#pragma unroll
                for (int a = 0; a < AF; ++a)
                    if (g * GB + b < NBF)
                        acc[a][g * GB + b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            as_frag(wbuf[u][ks][a]), xf[t & 1][b], acc[a][g * GB + b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        st = st1;
    };
    for (int c0 = 0; c0 < nchunks; c0 += PD + 1) {
        slice(std::integral_constant<int, 0>{}, c0);
        if constexpr (PD >= 1) slice(std::integral_constant<int, 1>{}, c0);
        if constexpr (PD >= 3) {
            slice(std::integral_constant<int, 2>{}, c0);
            slice(std::integral_constant<int, 3>{}, c0);
        }
    }
    __syncthreads();                                      // the next tile's first write may hit any stage

    // accumulator register i of lane l: feature 8*(i/4) + 4*(l/32) + i%4, token l%32
    if constexpr (YFRAG) {   // unit [(pm0/32 + b)][(fb0+a)*4 + g][lane%32], 8 bytes at half (lane/32)
#pragma unroll
        for (int a = 0; a < AF; ++a) {
            if (fb0 + a >= nfb) continue;
#pragma unroll
            for (int b = 0; b < NBF; ++b) {
                uint16_t* ydst = Y + (((size_t)((pm0 >> 5) + b) * (N >> 3) + (fb0 + a) * 4) * 32 + (lane & 31)) * 8 +
                                 (lane >> 5) * 4;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float v0 = acc[a][b][4 * g], v1 = acc[a][b][4 * g + 1], v2 = acc[a][b][4 * g + 2],
                          v3 = acc[a][b][4 * g + 3];
                    if (RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                    uint2 o;
                    o.x = (uint32_t)smoe_f32_to_bf16(v0) | ((uint32_t)smoe_f32_to_bf16(v1) << 16);
                    o.y = (uint32_t)smoe_f32_to_bf16(v2) | ((uint32_t)smoe_f32_to_bf16(v3) << 16);
                    *(uint2*)(ydst + g * 32 * 8) = o;
                }
            }
        }
    } else if constexpr (NBF <= 2 && !EARLY) {
        // Row-major output of a small tile of the small-tile kernels, straight from the accumulator layout (a lane holds 4
        // consecutive features of one token): the two extra barriers of the LDS turn below cost
        // more than the scattered 8-byte stores of at most two token blocks.
        const bool fused = fz.perm != nullptr, has_res = fused && fz.residual != nullptr;
#pragma unroll
        for (int a = 0; a < AF; ++a) {
            if (fb0 + a >= nfb) continue;
            const int col = (fb0 + a) * 32 + (lane >> 5) * 4;
            int dst[NBF];
            uint2 rr[NBF][4];
#pragma unroll
            for (int b = 0; b < NBF; ++b) {       // every residual piece of this feature block is asked for first
                dst[b] = drow[b];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    rr[b][g] = make_uint2(0, 0);
                    if (has_res && dst[b] >= 0) rr[b][g] = *(const uint2*)(fz.residual + (size_t)dst[b] * N + col + g * 8);
                }
            }
#pragma unroll
            for (int b = 0; b < NBF; ++b) {
                if (dst[b] < 0) continue;
                const float gmul = dgate[b];
                uint16_t* ydst = Y + (size_t)dst[b] * N + col;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float v0 = acc[a][b][4 * g], v1 = acc[a][b][4 * g + 1], v2 = acc[a][b][4 * g + 2],
                          v3 = acc[a][b][4 * g + 3];
                    apply_gate_v(v0, v1, v2, v3, gmul, rr[b][g], has_res, fused);
                    if (RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                    uint2 o;
                    o.x = (uint32_t)smoe_f32_to_bf16(v0) | ((uint32_t)smoe_f32_to_bf16(v1) << 16);
                    o.y = (uint32_t)smoe_f32_to_bf16(v2) | ((uint32_t)smoe_f32_to_bf16(v3) << 16);
                    *(uint2*)(ydst + g * 8) = o;
                }
            }
        }
    } else {
        // Row-major output.  In the accumulator layout a store instruction would touch 32 rows
        // with 8 bytes each; the tile is turned through LDS instead (the ring is idle now), so
        // that 16 lanes write one row's 256 contiguous bytes.  The product is rounded to bf16
        // on the way in -- the value the plain path stores, and the one the fused path scales
        // by the gate (+ residual) in fp32 before its single final rounding.
        constexpr int F = OF, CPR8 = OCPR, NP = ONP;
        constexpr int LDO = F + 4;                        // LDS row pitch in elements (8-byte aligned rows)
        static_assert(32 * NBF * CPR8 % THREADS == 0, "pieces divide evenly");
#pragma unroll
        for (int a = 0; a < AF; ++a)
#pragma unroll
            for (int b = 0; b < NBF; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float v0 = acc[a][b][4 * g], v1 = acc[a][b][4 * g + 1], v2 = acc[a][b][4 * g + 2],
                          v3 = acc[a][b][4 * g + 3];
                    if (RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                    uint2 o;
                    o.x = (uint32_t)smoe_f32_to_bf16(v0) | ((uint32_t)smoe_f32_to_bf16(v1) << 16);
                    o.y = (uint32_t)smoe_f32_to_bf16(v2) | ((uint32_t)smoe_f32_to_bf16(v3) << 16);
                    *(uint2*)&xs[(b * 32 + (lane & 31)) * LDO + (wave * AF + a) * 32 + g * 8 + (lane >> 5) * 4] = o;
                }
        __syncthreads();
        const bool fused = fz.perm != nullptr, has_res = fused && fz.residual != nullptr;
        const int col0 = ftile * F;
        constexpr int CH = NP < 8 ? NP : 8;               // pieces handled together (bounds the registers)
#pragma unroll
        for (int i0 = 0; i0 < NP; i0 += CH) {
            int prow[CH], pcol[CH];
            uint4 rs[CH];
#pragma unroll
            for (int j = 0; j < CH; ++j) {                // residual pieces not fetched earlier are asked for first
                // the last group is short when NP is not a multiple of CH: a piece past NP would belong
                // to a row below the tile, whose entry of the row table is stale
                if (i0 + j >= NP) { prow[j] = -1; pcol[j] = 0; rs[j] = make_uint4(0, 0, 0, 0); continue; }
                const int idx = tid + (i0 + j) * THREADS, r = idx / CPR8, c = idx % CPR8;
                pcol[j] = col0 + c * 8;
                prow[j] = pcol[j] < N ? orow[r] : -1;
                if constexpr (EARLY_RES) {
                    rs[j] = res[i0 + j];
                } else {
                    rs[j] = make_uint4(0, 0, 0, 0);
                    if (has_res && prow[j] >= 0) rs[j] = *(const uint4*)(fz.residual + (size_t)prow[j] * N + pcol[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                if (prow[j] < 0) continue;
                const int idx = tid + (i0 + j) * THREADS, r = idx / CPR8, c = idx % CPR8;
                const uint2 lo = *(const uint2*)&xs[r * LDO + c * 8], hi = *(const uint2*)&xs[r * LDO + c * 8 + 4];
                uint4 o = make_uint4(lo.x, lo.y, hi.x, hi.y);
                if (fused) {
                    const float g = ogate[r];
                    uint32_t yw[4] = {o.x, o.y, o.z, o.w}, rw[4] = {rs[j].x, rs[j].y, rs[j].z, rs[j].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float y0 = __uint_as_float(yw[q] << 16), y1 = __uint_as_float(yw[q] & 0xFFFF0000u);
                        float o0, o1;
                        if (has_res) {
                            o0 = fmaf(g, y0, __uint_as_float(rw[q] << 16));
                            o1 = fmaf(g, y1, __uint_as_float(rw[q] & 0xFFFF0000u));
                        } else {
                            o0 = g * y0;
                            o1 = g * y1;
                        }
                        yw[q] = (uint32_t)smoe_f32_to_bf16(o0) | ((uint32_t)smoe_f32_to_bf16(o1) << 16);
                    }
                    o = make_uint4(yw[0], yw[1], yw[2], yw[3]);
                }
                *(uint4*)(Y + (size_t)prow[j] * N + pcol[j]) = o;
            }
        }
        __syncthreads();                                  // the next tile's prologue reuses the ring
    }
}

template <int AF, int NBF, int MAXB, int NW, int BKT, int PD, bool XFRAG, bool YFRAG, bool RELU, bool EARLY>
struct TileSwitch {
    static __device__ __forceinline__ void go(int nbf, const uint16_t* X, const uint4* Wp, uint16_t* Y, int R,
                                              int N, int slot, int m0, int m_end, int pm0, int ftile,
                                              uint16_t* xs, int* orow, float* ogate, const FuseArgs fz) {
        constexpr int stage = MAXB * 32 * (BKT + KPAD);
        if (nbf == NBF)
            run_tile<AF, NBF, NW, BKT, PD, XFRAG, YFRAG, RELU, EARLY>(X, Wp, Y, R, N, slot, m0, m_end, pm0, ftile, xs,
                                                               stage, orow, ogate, fz);
        else if constexpr (NBF > 1)
            TileSwitch<AF, NBF - 1, MAXB, NW, BKT, PD, XFRAG, YFRAG, RELU, EARLY>::go(nbf, X, Wp, Y, R, N, slot, m0,
                                                                              m_end, pm0, ftile, xs, orow, ogate, fz);
    }
};

// FIRST = the d_model -> d_ff product: row-major x_perm in, ReLU, fragment-order h out.
// Otherwise the d_ff -> d_model product: fragment-order h in, row-major y_perm out.
// Persistent workgroups (see the enumeration above).
template <int AF, int MAXB, int NW, int BKT, int PD, int OCC, bool FIRST>
__global__ __launch_bounds__(NW * 64, OCC) void grouped_gemm_bf16(
    const uint16_t* __restrict__ X, const uint4* __restrict__ Wp, const int32_t* __restrict__ offsets,
    int nslots, int T, uint16_t* __restrict__ Y, int R, int N, const FuseArgs fz) {
    // the ring of token stages; the second product's epilogue turns its output tile through it
    constexpr int RING = 3 * MAXB * 32 * (BKT + KPAD), OUT_TILE = FIRST ? 0 : MAXB * 32 * (NW * AF * 32 + 4);
    __shared__ __align__(16) uint16_t xs[RING > OUT_TILE ? RING : OUT_TILE];
    __shared__ int s_orow[MAXB * 32];
    __shared__ float s_ogate[MAXB * 32];
    __shared__ ItemMap map;
    constexpr int BT = MAXB * 32;
    const int ftiles = ((N >> 5) + NW * AF - 1) / (NW * AF);
    build_item_map(map, offsets, nslots, T, BT);
    const long long G = (long long)__builtin_amdgcn_readfirstlane(map.first[nslots]) * ftiles;
    const int die = blockIdx.x % XCDS, nwg = gridDim.x / XCDS;   // the grid is a multiple of 8
    const long long lo = G * die / XCDS;
    const int cnt = (int)(G * (die + 1) / XCDS - lo);
    for (int j = blockIdx.x / XCDS; j < cnt; j += nwg) {
        const long long g = lo + j;
        int mt = (int)(g / ftiles), ftile = (int)(g % ftiles);
        int slot, m0, m_end, pm0;
        row_tile_at(map, nslots, BT, mt, slot, m0, m_end, pm0);
        if (FIRST) {
            // First product: inside a slot the items are numbered (feature tile, row tile) with the
            // row tile fastest.  A die's share of a large slot is then a range of feature tiles over
            // ALL the slot's rows, so no weight tile is fetched by two dies (the slot's token rows,
            // a quarter of the bytes, are what two dies may both read), and the workgroups that run
            // together read the same weight tile.  Measured on the Switch-base-64 shape: the L2s
            // request 93 MB per launch instead of 126 MB (the weights and tokens alone are 82 MB).
            // The second product keeps the row-tile-major numbering: its token tile (the hidden
            // activations of 128 rows) is as large as its weight tile, and the other order fetched
            // 15 % more at the Switch-large shape.
            const int first_k = __builtin_amdgcn_readfirstlane(map.first[slot]);
            const int tiles_k = __builtin_amdgcn_readfirstlane(map.first[slot + 1]) - first_k;
            const int local = (int)(g - (long long)first_k * ftiles);
            ftile = local / tiles_k;
            mt = first_k + (local - ftile * tiles_k);
            row_tile_at(map, nslots, BT, mt, slot, m0, m_end, pm0);
        }
        if (fz.phys) slot = __builtin_amdgcn_readfirstlane(fz.phys[slot]);   // from here on: where the weights live
        const int nbf = min(MAXB, (m_end - m0 + 31) >> 5);    // token blocks that hold real rows
        TileSwitch<AF, MAXB, MAXB, NW, BKT, PD, !FIRST, FIRST, FIRST, !FIRST && AF * MAXB <= 4 && OCC <= 2>::go(nbf, X, Wp, Y, R, N, slot, m0, m_end,
                                                                         pm0, ftile, xs, s_orow, s_ogate, fz);
    }
}

// ---------------------------------------------------------------------------
// Small-batch (decode) variant: row tiles of 32 tokens, nothing but weight
// streaming.  With a handful of tokens per slot the FFN is bound by reading
// each active slot's weights once, so the kernel is built around keeping many
// 1-KiB weight loads in flight: no LDS staging and no barrier in the loop --
// the token operand (32 rows) is read straight from L2 -- and the operands of
// G reduction steps are fetched together, two groups in flight per wave.
// A workgroup of NWV waves covers NWV / KSPLIT neighbouring feature blocks;
// the KSPLIT waves that share a feature block split its reduction and meet in
// LDS at the end (added in wave order: reproducible).  Splitting shortens the
// stream each wave has to pull through its own queue of loads, which is what
// bounds a wave's share of the HBM bandwidth.
// Workgroup b serves (slot b / ftiles, feature tile b % ftiles): it knows its
// weights before it knows whether the slot has any tokens, so the first group
// of weight loads is issued ahead of the read of the offsets and the latency of
// the two overlaps; the workgroup of an empty slot then simply leaves.  A slot
// with more than 32 tokens (rare at these batch sizes) is worked off 32 rows
// at a time.
template <int NWV, int KSPLIT, bool FIRST>
__global__ __launch_bounds__(NWV * 64) void small_gemm_bf16(
    const uint16_t* __restrict__ X, const uint4* __restrict__ Wp, const int32_t* __restrict__ offsets,
    int nslots, int T, uint16_t* __restrict__ Y, int R, int N, const FuseArgs fz) {
    constexpr int G = 8;                                   // reduction steps fetched together
    constexpr int FBW = NWV / KSPLIT;                      // feature blocks per workgroup
    constexpr bool XFRAG = !FIRST, YFRAG = FIRST, RELU = FIRST;
    __shared__ __align__(16) float red[KSPLIT > 1 ? (KSPLIT - 1) * FBW * 16 * 64 : 1];
    const int nfb = N >> 5, nrb = R >> 4;
    const int ftiles = (nfb + FBW - 1) / FBW;
    const int slot = blockIdx.x / ftiles, ftile = blockIdx.x % ftiles;
    // the wave index as a scalar: the reduction range below must be wave-uniform in the
    // compiler's eyes too, because an MFMA under a lane mask still runs for every lane
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int fbi = wave / KSPLIT, part = wave % KSPLIT;   // feature block in the workgroup, share of the reduction
    const int fb = ftile * FBW + fbi;
    const bool fb_ok = fb < nfb;
    const int per = (nrb + KSPLIT - 1) / KSPLIT;
    const int kb_lo = min(part * per, nrb), kb_hi = min(kb_lo + per, nrb);
    const uint4* wp = Wp + ((size_t)(fz.phys ? fz.phys[slot] : slot) * nfb + min(fb, nfb - 1)) * nrb * 64 + lane;

    uint4 wA[G], xA[G], wB[G], xB[G];
    auto fetch_w = [&](uint4 (&w)[G], int g0) {
#pragma unroll
        for (int i = 0; i < G; ++i) w[i] = wp[(size_t)max(min(g0 + i, kb_hi - 1), 0) * 64];   // past the end: reloaded, not used
    };
    fetch_w(wA, kb_lo);                                    // on its way before anything else is known

    // this slot's rows and the padded rows before it (segments re-based to multiples of 32)
    int seg_a = 0, seg_b = 0, pad_before = 0;
    for (int base = 0; base < nslots; base += 64) {
        const int k = base + lane;
        int a = 0, b = 0;
        if (k < nslots) {
            a = min(max(offsets[k], 0), T);                 // clamps guard misuse
            b = max(min(max(offsets[k + 1], 0), T), a);
        }
        const int pad = (b - a + 31) & ~31;
        const int pin = wave_incl_scan(pad, lane);
        if (slot >= base && slot < base + 64) {
            seg_a = __shfl(a, slot - base);
            seg_b = __shfl(b, slot - base);
            pad_before += __shfl(pin - pad, slot - base);
            break;
        }
        pad_before += __shfl(pin, 63);
    }
    seg_a = __builtin_amdgcn_readfirstlane(seg_a);
    seg_b = __builtin_amdgcn_readfirstlane(seg_b);
    pad_before = __builtin_amdgcn_readfirstlane(pad_before);
    if (seg_b <= seg_a) return;                            // nothing routed to this slot

    for (int m0 = seg_a; m0 < seg_b; m0 += 32) {
        const int m_end = seg_b, pm0 = pad_before + (m0 - seg_a);
        const uint4* xp;                                   // this lane's token operand at reduction step 0
        size_t xstep;                                      // in uint4 units per reduction step
        if (XFRAG) {
            xp = (const uint4*)X + ((size_t)(pm0 >> 5) * (R >> 3) + (lane >> 5)) * 32 + (lane & 31);
            xstep = 2 * 32;
        } else {
            int row = min(m0 + (lane & 31), m_end - 1);
            if (fz.perm) row = fz.perm[row];
            xp = (const uint4*)(X + (size_t)row * R + (lane >> 5) * 8);
            xstep = 2;
        }
        auto fetch_x = [&](uint4 (&xv)[G], int g0) {
#pragma unroll
            for (int i = 0; i < G; ++i) xv[i] = xp[(size_t)max(min(g0 + i, kb_hi - 1), 0) * xstep];
        };
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        auto consume = [&](uint4 (&w)[G], uint4 (&xv)[G], int g0) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                // steps past the end of the range multiply by a zero token operand
                const uint4 xz = g0 + i < kb_hi ? xv[i] : make_uint4(0, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(w[i]), as_frag(xz), acc, 0, 0, 0);
            }
        };
        // two groups of G reduction steps are always in flight: while one group's
        // MFMAs run, the next group's operands are already on their way
        if (m0 != seg_a) fetch_w(wA, kb_lo);               // (the first row tile's were issued at the top)
        fetch_x(xA, kb_lo);
        for (int g0 = kb_lo; g0 < kb_hi; g0 += 2 * G) {
            fetch_w(wB, g0 + G);
            fetch_x(xB, g0 + G);
            __builtin_amdgcn_sched_barrier(0);
            consume(wA, xA, g0);
            __builtin_amdgcn_sched_barrier(0);
            fetch_w(wA, g0 + 2 * G);
            fetch_x(xA, g0 + 2 * G);
            __builtin_amdgcn_sched_barrier(0);
            consume(wB, xB, g0 + G);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (KSPLIT > 1) {
            if (m0 != seg_a) __syncthreads();              // the previous row tile's sums have been read
            if (part > 0) {
#pragma unroll
                for (int i = 0; i < 16; ++i) red[(((part - 1) * FBW + fbi) * 16 + i) * 64 + lane] = acc[i];
            }
            __syncthreads();
            if (part == 0) {
#pragma unroll
                for (int w2 = 0; w2 < KSPLIT - 1; ++w2)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] += red[((w2 * FBW + fbi) * 16 + i) * 64 + lane];
            }
        }
        if (part > 0 || !fb_ok) continue;
        // accumulator register i of lane l: feature 8*(i/4) + 4*(l/32) + i%4, token l%32
        uint16_t* ydst;
        const uint16_t* rsrc = nullptr;
        float gmul = 1.f;
        if (YFRAG) {
            ydst = Y + (((size_t)(pm0 >> 5) * (N >> 3) + fb * 4) * 32 + (lane & 31)) * 8 + (lane >> 5) * 4;
        } else {
            int row = m0 + (lane & 31);
            if (row >= m_end) continue;
            if (fz.perm) {
                row = fz.perm[row];
                gmul = fz.gate[row];
                if (fz.residual) rsrc = fz.residual + (size_t)row * N + fb * 32 + (lane >> 5) * 4;
            }
            ydst = Y + (size_t)row * N + fb * 32 + (lane >> 5) * 4;
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float v0 = acc[4 * g], v1 = acc[4 * g + 1], v2 = acc[4 * g + 2], v3 = acc[4 * g + 3];
            if (!YFRAG) apply_gate(v0, v1, v2, v3, gmul, rsrc ? rsrc + g * 8 : nullptr, fz.perm != nullptr);
            if (RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
            uint2 o;
            o.x = (uint32_t)smoe_f32_to_bf16(v0) | ((uint32_t)smoe_f32_to_bf16(v1) << 16);
            o.y = (uint32_t)smoe_f32_to_bf16(v2) | ((uint32_t)smoe_f32_to_bf16(v3) << 16);
            *(uint2*)(ydst + (YFRAG ? g * 32 * 8 : g * 8)) = o;
        }
    }
}

// ---------------------------------------------------------------------------
// One 32-token tile for the whole batch (T <= 32, the single-call path only).
// With at most 32 tokens every slot's segment fits one MFMA token block, so
// the sort is not needed to form the tiles: workgroup (slot, feature tile)
// multiplies ALL T tokens, in token order, by the slot's weights and keeps the
// columns of the tokens that were routed to the slot (an MFMA column depends on
// its own token only, and the reduction order per element is that of
// small_gemm_bf16, so the results are the same bits).  Nothing the workgroup
// loads depends on another load: weights, token operands and the slot ids all
// go out at once, instead of the chain offsets -> permutation -> rows.  A slot
// nobody was routed to leaves after one group of weight loads.
// The hidden activations are kept per slot: h[slot][feature/8][token] units of
// 8 features (fragment order with the token index as the row).
// STREAM: the weight loads are marked non-temporal (see smoe_weights_outgrow_cache).
template <int NWV, int KSPLIT, bool FIRST, bool STREAM>
__device__ __forceinline__ void dense_gemm_body(
    const uint16_t* __restrict__ X, const uint4* __restrict__ Wp, const int32_t* __restrict__ slot_of,
    int T, uint16_t* __restrict__ Y, int R, int N, const int32_t* __restrict__ phys,
    const float* __restrict__ gate, const uint16_t* __restrict__ residual) {
    constexpr int G = 8;                                   // reduction steps fetched together
    constexpr int FBW = NWV / KSPLIT;                      // feature blocks per workgroup
    __shared__ __align__(16) float red[KSPLIT > 1 ? (KSPLIT - 1) * FBW * 16 * 64 : 1];
    const int nfb = N >> 5, nrb = R >> 4;
    const int ftiles = (nfb + FBW - 1) / FBW;
    const int slot = blockIdx.x / ftiles, ftile = blockIdx.x % ftiles;
    // wave index as a scalar: MFMA loop bounds must be wave-uniform for the compiler too
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int fbi = wave / KSPLIT, part = wave % KSPLIT;
    const int fb = ftile * FBW + fbi;
    const bool fb_ok = fb < nfb;
    const int per = (nrb + KSPLIT - 1) / KSPLIT;
    const int kb_lo = min(part * per, nrb), kb_hi = min(kb_lo + per, nrb);
    const int tok = lane & 31;
    const uint4* wp = Wp + ((size_t)(phys ? phys[slot] : slot) * nfb + min(fb, nfb - 1)) * nrb * 64 + lane;
    uint4 wA[G], xA[G], wB[G], xB[G];
    auto fetch_w = [&](uint4 (&w)[G], int g0) {
#pragma unroll
        for (int i = 0; i < G; ++i) {                      // past the end: reloaded, not used
            const uint4* src = wp + (size_t)max(min(g0 + i, kb_hi - 1), 0) * 64;
            w[i] = STREAM ? smoe_load_stream(src) : *src;
        }
    };
    fetch_w(wA, kb_lo);                                    // on its way before anything else is known
    const bool mine = tok < T && slot_of[min(tok, T - 1)] == slot;
    const unsigned long long who = __ballot(mine);
    if (who == 0) return;                                  // nothing routed to this slot (uniform over the workgroup)
    // columns of other slots' tokens repeat the first routed token's operand: lanes that ask for
    // the same address share one request, which keeps the token operand's traffic negligible
    const int src_tok = mine ? tok : ((__ffsll((long long)who) - 1) & 31);
    const uint4* xp;
    size_t xstep;
    if (FIRST) {                                           // row-major x, token order
        xp = (const uint4*)(X + (size_t)src_tok * R + (lane >> 5) * 8);
        xstep = 2;
    } else {                                               // h[slot] in fragment order
        xp = (const uint4*)X + ((size_t)slot * (R >> 3) + (lane >> 5)) * 32 + src_tok;
        xstep = 2 * 32;
    }
    auto fetch_x = [&](uint4 (&xv)[G], int g0) {
#pragma unroll
        for (int i = 0; i < G; ++i) xv[i] = xp[(size_t)max(min(g0 + i, kb_hi - 1), 0) * xstep];
    };
    auto fetch = [&](uint4 (&w)[G], uint4 (&xv)[G], int g0) {
        fetch_w(w, g0);
        fetch_x(xv, g0);
    };
    fetch_x(xA, kb_lo);
    float gmul = 1.f;
    uint2 rres[4] = {};
    if (!FIRST && mine && part == 0 && fb_ok) {            // asked for now, used after the loop
        gmul = gate[tok];
        if (residual) {
            const uint16_t* rp = residual + (size_t)tok * N + fb * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int g = 0; g < 4; ++g) rres[g] = *(const uint2*)(rp + g * 8);
        }
    }
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    auto consume = [&](uint4 (&w)[G], uint4 (&xv)[G], int g0) {
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const uint4 xz = g0 + i < kb_hi ? xv[i] : make_uint4(0, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(w[i]), as_frag(xz), acc, 0, 0, 0);
        }
    };
    for (int g0 = kb_lo; g0 < kb_hi; g0 += 2 * G) {
        fetch(wB, xB, g0 + G);
        __builtin_amdgcn_sched_barrier(0);
        consume(wA, xA, g0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(wA, xA, g0 + 2 * G);
        __builtin_amdgcn_sched_barrier(0);
        consume(wB, xB, g0 + G);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (KSPLIT > 1) {
        if (part > 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) red[(((part - 1) * FBW + fbi) * 16 + i) * 64 + lane] = acc[i];
        }
        __syncthreads();
        if (part > 0) return;
#pragma unroll
        for (int w2 = 0; w2 < KSPLIT - 1; ++w2)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] += red[((w2 * FBW + fbi) * 16 + i) * 64 + lane];
    }
    if (!fb_ok || !mine) return;
    // accumulator register i of lane l: feature 8*(i/4) + 4*(l/32) + i%4, token l%32
    uint16_t* ydst = FIRST ? Y + (((size_t)slot * (N >> 3) + fb * 4) * 32 + tok) * 8 + (lane >> 5) * 4
                           : Y + (size_t)tok * N + fb * 32 + (lane >> 5) * 4;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        float v0 = acc[4 * g], v1 = acc[4 * g + 1], v2 = acc[4 * g + 2], v3 = acc[4 * g + 3];
        if (!FIRST) apply_gate_v(v0, v1, v2, v3, gmul, rres[g], residual != nullptr, true);
        if (FIRST) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
        uint2 o;
        o.x = (uint32_t)smoe_f32_to_bf16(v0) | ((uint32_t)smoe_f32_to_bf16(v1) << 16);
        o.y = (uint32_t)smoe_f32_to_bf16(v2) | ((uint32_t)smoe_f32_to_bf16(v3) << 16);
        *(uint2*)(ydst + (FIRST ? g * 32 * 8 : g * 8)) = o;
    }
}

// Two kernels with one body: the second streams its weights past the caches.
#define SMOE_DENSE_GEMM_PARAMS                                                                              \
    const uint16_t* __restrict__ X, const uint4* __restrict__ Wp, const int32_t* __restrict__ slot_of, int T,  \
    uint16_t* __restrict__ Y, int R, int N, const int32_t* __restrict__ phys, const float* __restrict__ gate,  \
    const uint16_t* __restrict__ residual

template <int NWV, int KSPLIT, bool FIRST>
__global__ __launch_bounds__(NWV * 64) void dense_gemm_bf16(SMOE_DENSE_GEMM_PARAMS) {
    dense_gemm_body<NWV, KSPLIT, FIRST, false>(X, Wp, slot_of, T, Y, R, N, phys, gate, residual);
}

template <int NWV, int KSPLIT, bool FIRST>
__global__ __launch_bounds__(NWV * 64) void dense_gemm_stream_bf16(SMOE_DENSE_GEMM_PARAMS) {
    dense_gemm_body<NWV, KSPLIT, FIRST, true>(X, Wp, slot_of, T, Y, R, N, phys, gate, residual);
}

template <int NWV, int KSPLIT, bool FIRST>
void launch_small(const uint16_t* X, const void* Wp, const int32_t* offsets, int nslots, uint16_t* Y, int R,
                  int N, int T, const FuseArgs& fz, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    constexpr int FBW = NWV / KSPLIT;
    (void)T;
    int nfb = N >> 5;
    int ftiles = (nfb + FBW - 1) / FBW;
    dim3 grid(nslots * ftiles);                            // one workgroup per (slot, feature tile)
    smoe_launch_timed(small_gemm_bf16<NWV, KSPLIT, FIRST>, grid, dim3(NWV * 64), s, e0, e1, X, (const uint4*)Wp,
                      offsets, nslots, T, Y, R, N, fz);
}

// Compute units per die, asked of the runtime once.
int cus_per_die() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, cus = 0;
        (void)hipGetDevice(&dev);
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < XCDS)
            cus = 256;
        n = cus / XCDS;
    }
    return n;
}

template <int AF, int MAXB, int NW, int BKT, int PD, int OCC, bool FIRST>
void launch_gemm(const uint16_t* X, const void* Wp, const int32_t* offsets, int nslots, uint16_t* Y,
                 int R, int N, int T, const FuseArgs& fz, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    constexpr int BT = 32 * MAXB;
    const int mtiles = (T + BT - 1) / BT + nslots;         // upper bound on the row tiles of all slots
    const int ftiles = ((N >> 5) + NW * AF - 1) / (NW * AF);
    const long long items = (long long)mtiles * ftiles;
    // as many workgroups as the chip holds at once (OCC waves per SIMD), or fewer if the items run out
    const int resident = cus_per_die() * std::max(1, OCC * 4 / NW);
    const int per_die = (int)std::min<long long>((items + XCDS - 1) / XCDS, resident);
    dim3 grid(XCDS * std::max(per_die, 1));
    if ((R / BKT) % (PD + 1) == 0)
        smoe_launch_timed(grouped_gemm_bf16<AF, MAXB, NW, BKT, PD, OCC, FIRST>, grid, dim3(NW * 64), s, e0, e1, X,
                          (const uint4*)Wp, offsets, nslots, T, Y, R, N, fz);
    else   // slice count not a multiple of the ring length: same tile without weight prefetch
        smoe_launch_timed(grouped_gemm_bf16<AF, MAXB, NW, BKT, 0, OCC, FIRST>, grid, dim3(NW * 64), s, e0, e1, X,
                          (const uint4*)Wp, offsets, nslots, T, Y, R, N, fz);
}

// The tile shapes launch_variant knows (every one of them is chosen somewhere by pick_variants,
// except the 256 x 256 tile as the second product: 139 KB of LDS for the output turn and 85
// spilled registers make it slow, and it is there for the override only).
constexpr bool is_variant(int v) {
    return v == 1 || v == 3 || v == 4 || v == 5 || v == 6 || v == 8 || v == 10;
}

template <bool FIRST>
void launch_variant(int v, const uint16_t* X, const void* Wp, const int32_t* offsets, int nslots,
                    uint16_t* Y, int R, int N, int T, const FuseArgs& fz, hipStream_t s, hipEvent_t e0,
                    hipEvent_t e1) {
    if (R % 64 != 0 && v != 5 && v != 6) {   // d_model / d_ff are multiples of 32 by contract: 32-deep slices always fit
        launch_gemm<1, 4, 4, 32, 1, 2, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1);
        return;
    }
    switch (v) {             //            AF MAXB NW BKT PD OCC     tokens x features per workgroup
        case 1: launch_gemm<1, 4, 4, 64, 1, 2, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1); break;  // 128 x 128
        case 3: launch_gemm<1, 2, 4, 64, 1, 4, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1); break;  //  64 x 128
        case 4: launch_gemm<1, 1, 4, 64, 3, 4, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1); break;  //  32 x 128
        case 8: launch_gemm<1, 4, 8, 64, 1, 2, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1); break;  // 128 x 256, 8 waves
        case 10: launch_gemm<1, 8, 8, 64, 1, 2, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1); break;  // 256 x 256, 8 waves
        case 5: launch_small<4, 1, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1); break;   // 32 x 128, streaming
        case 6: launch_small<4, 4, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1); break;   // 32 x 32, reduction split 4 ways
        default: launch_small<4, 4, FIRST>(X, Wp, offsets, nslots, Y, R, N, T, fz, s, e0, e1); break;
    }
}

// Tile shapes for the two GEMMs.  A pair fixed at smoe_create (SMOE_FFN_VARIANT="v1,v2", a
// tuning aid; the indices are those of launch_variant) overrides the built-in choice.
void pick_variants(const smoe_layer* L, int T, int& v1, int& v2) {
    // Thresholds measured on the Switch-base-64 shape (K = 16, 768 x 3072) over T = 48 .. 8192.
    // What decides in the middle range is whether the first product's tiles fit the chip in one
    // round (256-row tiles at 120-183 tokens per slot: one tile per slot and feature tile).
    int per_slot = T / L->cfg.K;
    if (per_slot >= 384) { v1 = 10; v2 = 1; }
    else if (per_slot >= 184) { v1 = 8; v2 = 1; }
    else if (per_slot >= 120) { v1 = 10; v2 = 3; }
    else if (per_slot >= 60) { v1 = 8; v2 = 3; }
    else if (per_slot >= 28) { v1 = 3; v2 = 4; }
    else if (per_slot >= 6) { v1 = 4; v2 = 6; }
    else { v1 = 5; v2 = 6; }             // decode: a few tokens per slot, weight streaming
    if (is_variant(L->ffn_variant[0]) && is_variant(L->ffn_variant[1])) {
        v1 = L->ffn_variant[0];
        v2 = L->ffn_variant[1];
    }
}

}  // namespace

// Names of the two kernel instances the FFN of a T-token batch runs, as a profiler prints them
// (the benchmark uses this to check that a stored counter summary still describes the kernels
// it has just timed).
int smoe_describe_ffn_bf16(const smoe_layer* L, int T, int fused, char* out, size_t n) {
    int v[2];
    pick_variants(L, T, v[0], v[1]);
    std::string text;
    for (int i = 0; i < 2; ++i) {
        const bool first = i == 0;
        const int R = first ? L->cfg.d_model : L->cfg.d_ff;
        const char* shape = nullptr;                       // AF, MAXB, NW, BKT, PD, OCC of launch_variant
        std::string name;
        const std::string st = smoe_weights_outgrow_cache() ? "_stream" : "";
        if (fused && T <= 32 && v[0] == 5 && v[1] == 6 && smoe_decode_first_applies(L, T))
            name = first ? "decode_first" + st + (L->cfg.E <= 32 ? "_kernel<1>" : "_kernel<2>") : "dense_gemm" + st + "_bf16<4, 4, false>";
        else if (fused && T <= 32 && v[0] == 5 && v[1] == 6)
            name = "dense_gemm" + st + (first ? "_bf16<6, 1, true>" : "_bf16<4, 4, false>");
        else if (v[i] == 5) name = std::string("small_gemm_bf16<4, 1, ") + (first ? "true>" : "false>");
        else if (v[i] == 6) name = std::string("small_gemm_bf16<4, 4, ") + (first ? "true>" : "false>");
        else if (R % 64 != 0) shape = "1, 4, 4, 32, ";
        else if (v[i] == 1) shape = "1, 4, 4, 64, ";
        else if (v[i] == 3) shape = "1, 2, 4, 64, ";
        else if (v[i] == 4) shape = "1, 1, 4, 64, ";
        else if (v[i] == 8) shape = "1, 4, 8, 64, ";
        else if (v[i] == 10) shape = "1, 8, 8, 64, ";
        if (shape) {
            const int bkt = R % 64 != 0 ? 32 : 64, pd = (R % 64 == 0 && v[i] == 4) ? 3 : 1;
            const int occ = (R % 64 == 0 && (v[i] == 3 || v[i] == 4)) ? 4 : 2;
            const int pd_used = (R / bkt) % (pd + 1) == 0 ? pd : 0;
            name = std::string("grouped_gemm_bf16<") + shape + std::to_string(pd_used) + ", " + std::to_string(occ) + ", " +
                   (first ? "true>" : "false>");
        }
        text += (i ? " | " : "") + name;
    }
    if (!out || n == 0) return SMOE_EINVAL;
    snprintf(out, n, "%s", text.c_str());
    return SMOE_OK;
}

int smoe_launch_ffn_bf16(const smoe_layer* L, const uint16_t* x_perm, const int32_t* offsets, int T,
                         uint16_t* y_perm, hipStream_t s) {
    const smoe_config& c = L->cfg;
    int v1, v2;
    pick_variants(L, T, v1, v2);
    uint16_t* h = (uint16_t*)L->d_hidden;
    const int32_t* phys = L->cfg.spare_slots > 0 ? L->d_phys : nullptr;   // identity without spare slots
    const FuseArgs none{phys, nullptr, nullptr, nullptr};
    launch_variant<true>(v1, x_perm, L->slot_w1, offsets, c.K, h, c.d_model, c.d_ff, T, none, s, L->prof_ev[0], L->prof_ev[1]);
    launch_variant<false>(v2, h, L->slot_w2, offsets, c.K, y_perm, c.d_ff, c.d_model, T, none, s, L->prof_ev[2], L->prof_ev[3]);
    return smoe_check_hip(hipGetLastError(), "smoe_expert_ffn launch");
}

bool smoe_ffn_dense_path(const smoe_layer* L, int T) {
    int v1, v2;
    pick_variants(L, T, v1, v2);
    return T <= 32 && v1 == 5 && v2 == 6;
}

// Second product of a decode-sized batch whose first product was computed for every slot (the
// fused decode launch): reads h[slot][feature / 8][token], keeps the routed tokens' columns.
int smoe_launch_ffn_bf16_dense_second(const smoe_layer* L, const int32_t* slot_of, const float* gate,
                                      const uint16_t* residual, int T, uint16_t* out, hipStream_t s) {
    const smoe_config& c = L->cfg;
    const int32_t* phys = c.spare_slots > 0 ? L->d_phys : nullptr;
    if (smoe_weights_outgrow_cache())
        smoe_launch_timed(dense_gemm_stream_bf16<4, 4, false>, dim3(c.K * (c.d_model >> 5)), dim3(256), s, L->prof_ev[2],
                          L->prof_ev[3], (const uint16_t*)L->d_hidden, (const uint4*)L->slot_w2, slot_of, T, out, c.d_ff,
                          c.d_model, phys, gate, residual);
    else
        smoe_launch_timed(dense_gemm_bf16<4, 4, false>, dim3(c.K * (c.d_model >> 5)), dim3(256), s, L->prof_ev[2],
                          L->prof_ev[3], (const uint16_t*)L->d_hidden, (const uint4*)L->slot_w2, slot_of, T, out, c.d_ff,
                          c.d_model, phys, gate, residual);
    return smoe_check_hip(hipGetLastError(), "smoe_forward: FFN launch");
}

// Fused form used by smoe_forward: the first product gathers its rows from x
// through perm, the second scatters gate * y (+ residual) to out in token order.
int smoe_launch_ffn_bf16_fused(const smoe_layer* L, const uint16_t* x, const int32_t* slot_of,
                               const int32_t* perm, const int32_t* offsets, const float* gate,
                               const uint16_t* residual, int T, uint16_t* out, hipStream_t s) {
    const smoe_config& c = L->cfg;
    int v1, v2;
    pick_variants(L, T, v1, v2);
    uint16_t* h = (uint16_t*)L->d_hidden;
    const int32_t* phys = L->cfg.spare_slots > 0 ? L->d_phys : nullptr;   // identity without spare slots
    if (T <= 32 && v1 == 5 && v2 == 6) {      // the whole batch is one token block: no sorted tiles needed
        const int nfb1 = c.d_ff >> 5, nfb2 = c.d_model >> 5;
        if (smoe_weights_outgrow_cache()) {
            smoe_launch_timed(dense_gemm_stream_bf16<6, 1, true>, dim3(c.K * ((nfb1 + 5) / 6)), dim3(384), s, L->prof_ev[0],
                              L->prof_ev[1], x, (const uint4*)L->slot_w1, slot_of, T, h, c.d_model, c.d_ff,
                              phys, (const float*)nullptr, (const uint16_t*)nullptr);
            smoe_launch_timed(dense_gemm_stream_bf16<4, 4, false>, dim3(c.K * nfb2), dim3(256), s, L->prof_ev[2],
                              L->prof_ev[3], (const uint16_t*)h, (const uint4*)L->slot_w2, slot_of, T, out, c.d_ff,
                              c.d_model, phys, gate, residual);
        } else {
            smoe_launch_timed(dense_gemm_bf16<6, 1, true>, dim3(c.K * ((nfb1 + 5) / 6)), dim3(384), s, L->prof_ev[0],
                              L->prof_ev[1], x, (const uint4*)L->slot_w1, slot_of, T, h, c.d_model, c.d_ff,
                              phys, (const float*)nullptr, (const uint16_t*)nullptr);
            smoe_launch_timed(dense_gemm_bf16<4, 4, false>, dim3(c.K * nfb2), dim3(256), s, L->prof_ev[2],
                              L->prof_ev[3], (const uint16_t*)h, (const uint4*)L->slot_w2, slot_of, T, out, c.d_ff,
                              c.d_model, phys, gate, residual);
        }
        return smoe_check_hip(hipGetLastError(), "smoe_forward: FFN launch");
    }
    const FuseArgs gather{phys, perm, nullptr, nullptr}, scatter{phys, perm, gate, residual};
    launch_variant<true>(v1, x, L->slot_w1, offsets, c.K, h, c.d_model, c.d_ff, T, gather, s, L->prof_ev[0], L->prof_ev[1]);
    launch_variant<false>(v2, h, L->slot_w2, offsets, c.K, out, c.d_ff, c.d_model, T, scatter, s, L->prof_ev[2], L->prof_ev[3]);
    return smoe_check_hip(hipGetLastError(), "smoe_forward: FFN launch");
}
