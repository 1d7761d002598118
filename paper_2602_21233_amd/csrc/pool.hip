// Block mean pooling of Q and K (pattern computation, step 1; Sec. 4.1.1 of the
// AngelSlim report: the dynamic regime first locates the sparse regions).
//
// Pure HBM stream: every bf16 element of Q and K is read exactly once with
// 16-byte loads, one workgroup per (head, block).  A row of head_dim elements is
// covered by head_dim/8 adjacent lanes, so each wave instruction reads whole
// contiguous rows.  Partial sums are fp32; the 16 (or 32) row groups of a
// workgroup are combined through LDS in a fixed order, so results are
// deterministic.
#include "common.hpp"

namespace spa {
namespace {

template <int D, int BS>
__global__ __launch_bounds__(256) void pool_kernel(const uint16_t* __restrict__ q, Strides qs,
                                                   int n_q_rows /* B*Hq or 0 */, int Hq,
                                                   const uint16_t* __restrict__ k, Strides ks, int Hkv,
                                                   float* __restrict__ qp, float* __restrict__ kp, int NBq, int Sq,
                                                   int NBk, int Skv, int k_tiled,
                                                   const int32_t* __restrict__ seq_lens) {
    constexpr int TPR = D / 8;          // lanes per token row
    constexpr int RPP = 256 / TPR;      // token rows per pass
    constexpr int PASSES = BS / RPP;
    __shared__ float part[RPP][D];

    const int blk = blockIdx.x;
    int hy = blockIdx.y;
    const uint16_t* src;
    float* dst;
    int S;                                   // tokens of this tensor (K may carry a prefix)
    if (hy < n_q_rows) {
        int b = hy / Hq, h = hy % Hq;
        Sq = entry_len(seq_lens, b, Sq);     // ragged batch: this entry's own length
        if (blk * BS >= Sq) return;          // the grid spans the key blocks of the longest entry
        src = q + b * qs.b + h * qs.h + (int64_t)blk * BS * qs.t;
        dst = qp + ((int64_t)hy * NBq + blk) * D;
        S = Sq;
        k = nullptr;
    } else {
        hy -= n_q_rows;
        int b = hy / Hkv, h = hy % Hkv;
        Skv = Skv - Sq + entry_len(seq_lens, b, Sq);
        if (blk * BS >= Skv) return;
        src = k + b * ks.b + h * ks.h + (int64_t)blk * BS * ks.t;
        dst = kp + ((int64_t)hy * NBk + blk) * D;
        S = Skv;
        qs = ks;
        // k_tiled: pooled K goes out in the operand layout of the score kernel instead of row
        // major fp32: per KV head, tiles of 32 key blocks (32 * D * 4 bytes); every value is
        // already split into its bf16 head and bf16 tail (x = hi + lo), and inside a tile the 8
        // dims 16s + 8h .. +7 of block r sit at bf16 offset (((2s + h) * 2 + part) * 32 + r) * 8,
        // part 0 = hi, 1 = lo, so a wavefront of that kernel reads whole 1-KB pieces that are its
        // MFMA operands as they are.  Heads are ceil(NBk / 32) tiles apart.
        if (k_tiled) dst = kp + ((int64_t)hy * ((NBk + 31) >> 5) + (blk >> 5)) * (32 * D);
    }
    const int tid = threadIdx.x;
    const int row0 = tid / TPR, chunk = tid % TPR;

    // the last block of a sequence may be partial: tokens past the end are not read
    const int n_valid = S - blk * BS < BS ? S - blk * BS : BS;
    uint4 raw[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        raw[p] = make_uint4(0u, 0u, 0u, 0u);
        if (p * RPP + row0 < n_valid)
            raw[p] = stream_load16(src + (int64_t)(p * RPP + row0) * qs.t + chunk * 8);
    }
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        acc[0] += bf16_lo(raw[p].x); acc[1] += bf16_hi(raw[p].x);
        acc[2] += bf16_lo(raw[p].y); acc[3] += bf16_hi(raw[p].y);
        acc[4] += bf16_lo(raw[p].z); acc[5] += bf16_hi(raw[p].z);
        acc[6] += bf16_lo(raw[p].w); acc[7] += bf16_hi(raw[p].w);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[row0][chunk * 8 + e] = acc[e];
    __syncthreads();
    if (tid < D) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < RPP; ++r) s += part[r][tid];
        const float mean = n_valid == BS ? s * (1.0f / (float)BS) : s / (float)n_valid;
        if (k != nullptr && k_tiled) {
            const __bf16 hi = (__bf16)mean;                       // round to nearest even, twice
            const __bf16 lo = (__bf16)(mean - (float)hi);
            __bf16* t = reinterpret_cast<__bf16*>(dst);
            const int at = (((tid >> 3) * 2) * 32 + (blk & 31)) * 8 + (tid & 7);
            t[at] = hi;
            t[at + 32 * 8] = lo;
        } else {
            dst[tid] = mean;
        }
    }
}

template <int D, int BS>
hipError_t launch(const Dims& d, const void* q, Strides qs, const void* k, Strides ks, float* qp,
                  float* kp, bool k_tiled, hipStream_t st) {
    int nq = q ? d.B * d.Hq : 0, nk = k ? d.B * d.Hkv : 0;
    if (nq + nk == 0) return hipSuccess;
    dim3 grid(nk ? d.NBk : d.NB, nq + nk);
    hipLaunchKernelGGL((pool_kernel<D, BS>), grid, dim3(256), 0, st, (const uint16_t*)q, qs, nq, d.Hq,
                       (const uint16_t*)k, ks, d.Hkv, qp, kp, d.NB, d.S, d.NBk, d.Skv, k_tiled ? 1 : 0, d.seq_lens);
    return hipGetLastError();
}

// ln of the mean L2 norm of a key block's value vectors (the value-magnitude term of the
// output-aware ranking score, Sec. 4.1.2 Fig. "Stem" (c)).  Same access pattern as pool_kernel:
// D/8 adjacent lanes cover one token, combine their partial sums of squares with lane-xor
// exchanges, and the token norms of the 16 (or 32) row groups are added through LDS in a fixed
// order.  A block of all-zero values gives -inf.
template <int D, int BS>
__global__ __launch_bounds__(256) void vnorm_kernel(const uint16_t* __restrict__ v, Strides vs, int Hkv, int NB,
                                                    int S, float* __restrict__ lvn,
                                                    const int32_t* __restrict__ seq_lens, int Sq) {
    constexpr int TPR = D / 8;
    constexpr int RPP = 256 / TPR;
    constexpr int PASSES = BS / RPP;
    __shared__ float part[RPP];
    const int blk = blockIdx.x, hy = blockIdx.y;
    const int b = hy / Hkv, h = hy % Hkv;
    const uint16_t* src = v + b * vs.b + h * vs.h + (int64_t)blk * BS * vs.t;
    const int tid = threadIdx.x;
    const int row0 = tid / TPR, chunk = tid % TPR;
    S = S - Sq + entry_len(seq_lens, b, Sq);                        // ragged batch: key tokens of this entry
    if (blk * BS >= S) return;
    const int n_valid = S - blk * BS < BS ? S - blk * BS : BS;      // partial last block
    uint4 raw[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        raw[p] = make_uint4(0u, 0u, 0u, 0u);                          // a missing token adds a norm of 0
        if (p * RPP + row0 < n_valid)
            raw[p] = stream_load16(src + (int64_t)(p * RPP + row0) * vs.t + chunk * 8);
    }
    float acc = 0.f;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const uint32_t w[4] = {raw[p].x, raw[p].y, raw[p].z, raw[p].w};
        float sq = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float lo = bf16_lo(w[e]), hi = bf16_hi(w[e]);
            sq = fmaf(lo, lo, sq);
            sq = fmaf(hi, hi, sq);
        }
#pragma unroll
        for (int off = 1; off < TPR; off <<= 1) sq += __shfl_xor(sq, off);
        acc += sqrtf(sq);
    }
    if (chunk == 0) part[row0] = acc;
    __syncthreads();
    if (tid == 0) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < RPP; ++r) s += part[r];
        lvn[(int64_t)hy * NB + blk] = logf(n_valid == BS ? s * (1.0f / (float)BS) : s / (float)n_valid);
    }
}

// group-shared selection: the pooled queries of the G heads of a KV group are averaged
__global__ __launch_bounds__(256) void group_mean_kernel(const float4* __restrict__ qp, float4* __restrict__ qg, int G,
                                                         int64_t n4 /* float4 per head */, int64_t total4) {
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (x >= total4) return;
    const int64_t head = x / n4, within = x % n4;      // head = b * Hkv + kv head
    const float4* src = qp + head * G * n4 + within;
    float4 acc = src[0];
    for (int g = 1; g < G; ++g) {
        const float4 t = src[g * n4];
        acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
    }
    const float inv = 1.0f / (float)G;
    qg[x] = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

template <int D, int BS>
hipError_t launch_vn(const Dims& d, const void* v, Strides vs, float* lvn, hipStream_t st) {
    dim3 grid(d.NBk, d.B * d.Hkv);
    hipLaunchKernelGGL((vnorm_kernel<D, BS>), grid, dim3(256), 0, st, (const uint16_t*)v, vs, d.Hkv, d.NBk, d.Skv, lvn, d.seq_lens, d.S);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_group_mean(const Dims& d, const float* qp, float* qg, hipStream_t st) {
    const int64_t n4 = (int64_t)d.NB * d.D / 4, total4 = n4 * d.B * d.Hkv;
    hipLaunchKernelGGL(group_mean_kernel, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, st,
                       (const float4*)qp, (float4*)qg, d.G, n4, total4);
    return hipGetLastError();
}

hipError_t launch_vnorm(const Dims& d, const void* v, Strides vs, float* lvn, hipStream_t st) {
    if (d.D == 128 && d.Bs == 128) return launch_vn<128, 128>(d, v, vs, lvn, st);
    if (d.D == 128 && d.Bs == 64) return launch_vn<128, 64>(d, v, vs, lvn, st);
    if (d.D == 64 && d.Bs == 128) return launch_vn<64, 128>(d, v, vs, lvn, st);
    if (d.D == 64 && d.Bs == 64) return launch_vn<64, 64>(d, v, vs, lvn, st);
    return hipErrorInvalidValue;
}

hipError_t launch_pool(const Dims& d, const void* q, Strides qs, const void* k, Strides ks,
                       float* qp, float* kp, bool k_tiled, hipStream_t st) {
    if (d.D == 128 && d.Bs == 128) return launch<128, 128>(d, q, qs, k, ks, qp, kp, k_tiled, st);
    if (d.D == 128 && d.Bs == 64) return launch<128, 64>(d, q, qs, k, ks, qp, kp, k_tiled, st);
    if (d.D == 64 && d.Bs == 128) return launch<64, 128>(d, q, qs, k, ks, qp, kp, k_tiled, st);
    if (d.D == 64 && d.Bs == 64) return launch<64, 64>(d, q, qs, k, ks, qp, kp, k_tiled, st);
    return hipErrorInvalidValue;
}

}  // namespace spa
