// smoe_set_resident's device side: the Virtual-Expert update of SwapMoE
// (Section 3.2) -- one expert's weights enter a slot and the slot<->expert maps
// change in stream order -- plus the per-expert magnitude |E_i| of Eq. 1.
//
// bf16 slots are kept in MFMA fragment order so the FFN streams them with
// contiguous 16-byte loads per lane and no LDS transpose.  For a weight matrix
// B [R, N] (R = reduction length, N = output features; W1: R = d_model,
// N = d_ff; W2: R = d_ff, N = d_model), element (r, n) lives at
//     ((n/32 * R/16 + r/16) * 64 + lane) * 8 + r%8,   lane = n%32 + 32*((r%16)/8)
// i.e. one 1-KiB block per (32 features x 16 reduction steps): exactly one
// operand of the 32x32x16 bf16 MFMA, lane-major, and all blocks of one feature
// group contiguous along the reduction.  fp32 slots keep the bank layout.

#include "smoe_internal.h"

namespace {

__global__ void clear_maps_kernel(int32_t* e2s, int E, int32_t* s2e, int32_t* phys, int K) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < E) e2s[i] = -1;
    if (i < K) { s2e[i] = -1; phys[i] = i; }
}

__global__ void set_map_kernel(int32_t* e2s, int32_t* s2e, int32_t* phys, int slot, int expert, int old_expert,
                               int p) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        if (old_expert >= 0) e2s[old_expert] = -1;
        e2s[expert] = slot;
        s2e[slot] = expert;
        phys[slot] = p;
    }
}

// One workgroup re-lays a tile of 16 reduction rows x 128 feature columns (4 blocks of the
// packed order).  The source rows are read with 16-byte pieces, 256 contiguous bytes per
// row, and turned through LDS; each thread then gathers one packed unit (8 consecutive
// reduction rows of one feature column) and the workgroup writes four full 1-KiB blocks.
constexpr int PACK_COLS = 128;
constexpr int PACK_LD = PACK_COLS + 8;       // LDS row pitch in elements (16-byte aligned rows)

__device__ __forceinline__ void pack_tile(const uint16_t* __restrict__ src, int R, int N,
                                          uint4* __restrict__ dst, int tile, uint16_t* lds) {
    const int ctiles = (N + PACK_COLS - 1) / PACK_COLS;
    const int rb = tile / ctiles, ct = tile - rb * ctiles;       // 16-row block, 128-column tile
    const int n0 = ct * PACK_COLS, r0 = rb * 16, tid = threadIdx.x;
    {   // thread t brings 8 columns of row t / 16
        const int row = tid >> 4, col = n0 + (tid & 15) * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (col < N) v = *(const uint4*)(src + (size_t)(r0 + row) * N + col);   // N is a multiple of 32: whole pieces
        *(uint4*)&lds[row * PACK_LD + (tid & 15) * 8] = v;
    }
    __syncthreads();
    const int nbl = tid >> 6, lane = tid & 63;                    // feature block inside the tile, lane of the unit
    const int nb = ct * (PACK_COLS / 32) + nbl;
    if (nb * 32 < N) {
        const int c = nbl * 32 + (lane & 31), rr = (lane >> 5) * 8;
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = (uint32_t)lds[(rr + 2 * i) * PACK_LD + c] | ((uint32_t)lds[(rr + 2 * i + 1) * PACK_LD + c] << 16);
        dst[((size_t)nb * (R / 16) + rb) * 64 + lane] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Loads one expert into a physical slot in a single launch: blocks [0, nblk1) re-lay
// W1 [d_model, d_ff], the rest W2 [d_ff, d_model]; with map_slot >= 0 the first thread
// also switches the maps.  The maps are read only by later launches of the stream, which
// start after this whole launch (weights included) has completed.
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint16_t* __restrict__ w1, const uint16_t* __restrict__ w2,
                                                        int d_model, int d_ff, uint4* __restrict__ dst1,
                                                        uint4* __restrict__ dst2, int nblk1, int32_t* e2s,
                                                        int32_t* s2e, int32_t* phys, int map_slot, int expert,
                                                        int old_expert, int p) {
    __shared__ __align__(16) uint16_t lds[16 * PACK_LD];
    if ((int)blockIdx.x < nblk1) pack_tile(w1, d_model, d_ff, dst1, blockIdx.x, lds);
    else pack_tile(w2, d_ff, d_model, dst2, blockIdx.x - nblk1, lds);
    if (map_slot >= 0 && blockIdx.x == 0 && threadIdx.x == 0) {
        if (old_expert >= 0) e2s[old_expert] = -1;
        e2s[expert] = map_slot;
        s2e[map_slot] = expert;
        phys[map_slot] = p;
    }
}

// The update rule (Section 3.2; important experts in, unimportant out) on the device, one
// workgroup: the K highest scores form the new resident set (ties: lower expert id), experts that
// stay keep their slots, the freed slots in ascending order receive the newcomers in descending
// score.  Switches the device maps and leaves the loads in plan: [0] their number, [1 .. K] the
// slots, [1 + K .. 2K] the experts.  E, K <= 256; every slot holds an expert (the host checks).
__global__ __launch_bounds__(256) void plan_update_kernel(const float* __restrict__ score, int E, int K, int32_t* e2s,
                                                          int32_t* s2e, int32_t* __restrict__ plan) {
    __shared__ float s_score[256];
    __shared__ int32_t s_e2s[256], s_s2e[256], s_rank[256], s_newc[256];
    __shared__ unsigned char s_wanted[256], s_isnew[256], s_free[256];
    const int tid = threadIdx.x;
    s_score[tid] = tid < E ? score[tid] : 0.f;
    s_e2s[tid] = tid < E ? e2s[tid] : 0;
    s_s2e[tid] = tid < K ? s2e[tid] : -1;
    s_newc[tid] = -1;
    __syncthreads();
    int rank = 0;                                          // experts that come before this one
    if (tid < E) {
        const float me = s_score[tid];
        for (int j = 0; j < E; ++j) {
            const float o = s_score[j];
            rank += (o > me) | ((o == me) & (j < tid));
        }
    }
    const bool wanted = tid < E && rank < K;
    const bool isnew = wanted && s_e2s[tid] < 0;
    s_rank[tid] = rank;
    s_wanted[tid] = wanted;
    s_isnew[tid] = isnew;
    __syncthreads();
    if (isnew) {                                           // newcomers in descending score
        int ord = 0;
        for (int j = 0; j < E; ++j) ord += s_isnew[j] && s_rank[j] < rank;
        if (ord < 256) s_newc[ord] = tid;
    }
    bool fr = false;                                       // slots whose expert leaves
    if (tid < K) {
        const int cur = s_s2e[tid];
        fr = !(cur >= 0 && s_wanted[cur]);
    }
    s_free[tid] = fr;
    __syncthreads();
    if (fr) {
        int ord = 0;
        for (int k = 0; k < tid; ++k) ord += s_free[k];
        const int expert = ord < K ? s_newc[ord] : -1, old = s_s2e[tid];
        if (expert >= 0) {                                 // (always, with consistent maps and finite scores)
            plan[1 + ord] = tid;
            plan[1 + K + ord] = expert;
            if (old >= 0) e2s[old] = -1;
            e2s[expert] = tid;
            s2e[tid] = expert;
        }
    }
    const int nf = __syncthreads_count(fr), nn = __syncthreads_count(isnew);
    if (tid == 0) plan[0] = nf < nn ? nf : nn;             // pairs = the shorter of the two lists
}

// The planned loads from a bank [E][d_model][d_ff] / [E][d_ff][d_model] in GPU-readable memory:
// workgroup b re-lays tile b of every planned expert in turn (the plan is short; most updates
// change a few slots).
__global__ __launch_bounds__(256) void pack_planned_kernel(const uint16_t* __restrict__ bank1, const uint16_t* __restrict__ bank2,
                                                           int d_model, int d_ff, uint4* __restrict__ slot1,
                                                           uint4* __restrict__ slot2, int nblk1, const int32_t* __restrict__ plan,
                                                           int K, const int32_t* __restrict__ phys) {
    __shared__ __align__(16) uint16_t lds[16 * PACK_LD];
    const int n = plan[0];
    const size_t per = (size_t)d_model * d_ff;             // elements per matrix
    for (int j = 0; j < n; ++j) {
        const int slot = plan[1 + j], expert = plan[1 + K + j];
        const size_t dst = (size_t)phys[slot] * (per / 8);   // 16-byte units
        if ((int)blockIdx.x < nblk1) pack_tile(bank1 + (size_t)expert * per, d_model, d_ff, slot1 + dst, blockIdx.x, lds);
        else pack_tile(bank2 + (size_t)expert * per, d_ff, d_model, slot2 + dst, blockIdx.x - nblk1, lds);
        __syncthreads();                                   // the tile buffer is reused by the next expert
    }
}

__global__ __launch_bounds__(256) void copy16_kernel(const uint4* __restrict__ src, size_t n16,
                                                     uint4* __restrict__ dst) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

// |E_i|^2 partial sums: grid (chunks, experts); a fixed tree per block and a
// fixed-order final pass keep the result reproducible.
constexpr int NORM_CHUNKS = 64;

template <bool BF16>
__global__ __launch_bounds__(256) void sumsq_kernel(const uint4* __restrict__ w1, const uint4* __restrict__ w2,
                                                    size_t n16_per_expert, float* __restrict__ partial) {
    __shared__ float red[256];
    const int e = blockIdx.y, chunk = blockIdx.x, tid = threadIdx.x;
    float acc = 0.f;
    for (int m = 0; m < 2; ++m) {
        const uint4* w = (m == 0 ? w1 : w2) + (size_t)e * n16_per_expert;
        for (size_t i = (size_t)chunk * 256 + tid; i < n16_per_expert; i += (size_t)NORM_CHUNKS * 256) {
            uint4 v = w[i];
            uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (BF16) {
                    float lo = __uint_as_float(u[j] << 16), hi = __uint_as_float(u[j] & 0xFFFF0000u);
                    acc = fmaf(lo, lo, acc);
                    acc = fmaf(hi, hi, acc);
                } else {
                    float f = __uint_as_float(u[j]);
                    acc = fmaf(f, f, acc);
                }
            }
        }
    }
    red[tid] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) partial[(size_t)e * NORM_CHUNKS + chunk] = red[0];
}

__global__ void norm_finish_kernel(const float* __restrict__ partial, int n, float* __restrict__ out) {
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    float s = 0.f;
    for (int c = 0; c < NORM_CHUNKS; ++c) s += partial[(size_t)e * NORM_CHUNKS + c];
    out[e] = sqrtf(s);
}

}  // namespace

int smoe_launch_clear_maps(const smoe_layer* L, hipStream_t s) {
    int n = L->cfg.E > L->cfg.K ? L->cfg.E : L->cfg.K;
    hipLaunchKernelGGL(clear_maps_kernel, dim3((n + 255) / 256), dim3(256), 0, s, L->d_expert_to_slot,
                       L->cfg.E, L->d_slot_to_expert, L->d_phys, L->cfg.K);
    return smoe_check_hip(hipGetLastError(), "smoe_set_resident: map reset");
}

// map_slot >= 0: the launch that loads the weights also switches the maps (bf16 layers; fp32
// layers take the separate map launch).  Returns 1 in *map_done when it did.
int smoe_launch_pack_slot(const smoe_layer* L, int slot, const void* w1_src, const void* w2_src, hipStream_t s,
                          int map_slot, int expert, int old_expert, int* map_done) {
    const smoe_config& c = L->cfg;
    const size_t per = (size_t)c.d_model * c.d_ff;               // elements per matrix
    if (map_done) *map_done = 0;
    if (c.dtype == SMOE_BF16) {
        const int nblk1 = (c.d_model / 16) * ((c.d_ff + PACK_COLS - 1) / PACK_COLS);
        const int nblk2 = (c.d_ff / 16) * ((c.d_model + PACK_COLS - 1) / PACK_COLS);
        uint4* d1 = (uint4*)((uint16_t*)L->slot_w1 + (size_t)slot * per);
        uint4* d2 = (uint4*)((uint16_t*)L->slot_w2 + (size_t)slot * per);
        hipLaunchKernelGGL(pack_bf16_kernel, dim3(nblk1 + nblk2), dim3(256), 0, s, (const uint16_t*)w1_src,
                           (const uint16_t*)w2_src, c.d_model, c.d_ff, d1, d2, nblk1, L->d_expert_to_slot,
                           L->d_slot_to_expert, L->d_phys, map_slot, expert, old_expert, slot);
        if (map_done && map_slot >= 0) *map_done = 1;
    } else {
        size_t n16 = per * 4 / 16;
        dim3 grid((unsigned)((n16 + 255) / 256));
        hipLaunchKernelGGL(copy16_kernel, grid, dim3(256), 0, s, (const uint4*)w1_src, n16,
                           (uint4*)((float*)L->slot_w1 + (size_t)slot * per));
        hipLaunchKernelGGL(copy16_kernel, grid, dim3(256), 0, s, (const uint4*)w2_src, n16,
                           (uint4*)((float*)L->slot_w2 + (size_t)slot * per));
    }
    return smoe_check_hip(hipGetLastError(), "expert load launch");
}

int smoe_launch_set_map(const smoe_layer* L, int slot, int expert, int old_expert, int phys, hipStream_t s) {
    hipLaunchKernelGGL(set_map_kernel, dim3(1), dim3(64), 0, s, L->d_expert_to_slot, L->d_slot_to_expert,
                       L->d_phys, slot, expert, old_expert, phys);
    return smoe_check_hip(hipGetLastError(), "map update launch");
}

int smoe_launch_expert_norm(const smoe_layer* L, const void* w1, const void* w2, int n, float* out,
                            hipStream_t s) {
    if (!L->bound) return smoe_fail(SMOE_ESTATE, "smoe_expert_norm: call smoe_bind first");
    const smoe_config& c = L->cfg;
    float* partial = L->d_norm_partial;                       // [n <= E][NORM_CHUNKS]
    size_t n16 = (size_t)c.d_model * c.d_ff * smoe_elem_size(c.dtype) / 16;
    dim3 grid(NORM_CHUNKS, n);
    if (c.dtype == SMOE_BF16)
        hipLaunchKernelGGL(sumsq_kernel<true>, grid, dim3(256), 0, s, (const uint4*)w1, (const uint4*)w2, n16, partial);
    else
        hipLaunchKernelGGL(sumsq_kernel<false>, grid, dim3(256), 0, s, (const uint4*)w1, (const uint4*)w2, n16, partial);
    hipLaunchKernelGGL(norm_finish_kernel, dim3((n + 63) / 64), dim3(64), 0, s, partial, n, out);
    return smoe_check_hip(hipGetLastError(), "smoe_expert_norm launch");
}

// ---------------------------------------------------------------------------
// Calibration for the roofline of the weight-streaming kernels: a plain read of the first K
// slots of one of the two slot arrays, nothing else.  Every workgroup reads one contiguous
// chunk with eight 16-byte loads in flight per thread; the sums go nowhere (the store below
// never executes) and only keep the loads alive.
namespace {
__global__ __launch_bounds__(512) void stream_read_kernel(const uint4* __restrict__ buf, size_t n16,
                                                          float* __restrict__ sink) {
    const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per_wg, hi = lo + per_wg < n16 ? lo + per_wg : n16;
    uint32_t a = 0, b = 0;
    for (size_t i = lo + threadIdx.x; i < hi; i += 512 * 8) {
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            size_t k = i + (size_t)j * 512;
            if (k >= hi) k = hi - 1;                       // past the chunk: its last piece again
            v[j] = buf[k];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) { a ^= v[j].x ^ v[j].z; b += v[j].y + v[j].w; }
    }
    if (a == 0x9E3779B9u && b == 0x7F4A7C15u) sink[0] = 1.f;   // keeps the loads; practically never true
}
}  // namespace

int smoe_launch_stream_read(const smoe_layer* L, int which, hipStream_t s) {
    const smoe_config& c = L->cfg;
    const size_t n16 = (size_t)c.K * c.d_model * c.d_ff * smoe_elem_size(c.dtype) / 16;
    const void* buf = which == 0 ? L->slot_w1 : L->slot_w2;
    int dev = 0, cus = 256;
    (void)hipGetDevice(&dev);
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    hipLaunchKernelGGL(stream_read_kernel, dim3(cus), dim3(512), 0, s, (const uint4*)buf, n16, L->d_norm_partial);
    return smoe_check_hip(hipGetLastError(), "smoe_profile_stream_read launch");
}

int smoe_launch_update_on_device(const smoe_layer* L, const float* score, const void* bank_w1, const void* bank_w2,
                                 hipStream_t s) {
    const smoe_config& c = L->cfg;
    hipLaunchKernelGGL(plan_update_kernel, dim3(1), dim3(256), 0, s, score, c.E, c.K, L->d_expert_to_slot,
                       L->d_slot_to_expert, L->d_plan);
    const int nblk1 = (c.d_model / 16) * ((c.d_ff + PACK_COLS - 1) / PACK_COLS);
    const int nblk2 = (c.d_ff / 16) * ((c.d_model + PACK_COLS - 1) / PACK_COLS);
    hipLaunchKernelGGL(pack_planned_kernel, dim3(nblk1 + nblk2), dim3(256), 0, s, (const uint16_t*)bank_w1,
                       (const uint16_t*)bank_w2, c.d_model, c.d_ff, (uint4*)L->slot_w1, (uint4*)L->slot_w2, nblk1,
                       L->d_plan, c.K, L->d_phys);
    return smoe_check_hip(hipGetLastError(), "smoe_update_on_device launch");
}
