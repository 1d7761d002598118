// Pooled scores, per-row top-k and merge with the static A-shape pattern
// (pattern computation, steps 2-4; Sec. 4.1.1 dynamic sparsity, uniform top-k
// budget of Sec. 4.1.2 Fig. "Stem" (a), static A-shape of Sec. 4.1.1).
//
// One 64-lane wavefront owns one row (b, h, i).  Lane l scores key blocks
// j = l, l+64, ... and turns each fp32 score into an order-preserving uint32 key
// kept in the wave's LDS slice.  The k-th largest key is found exactly by a
// bitwise descent (ballot + popcount per step), ties at the threshold are
// resolved by block index with a running prefix count, and because the final
// pass walks j in ascending order the emitted list is already sorted, with the
// static blocks simply forced on.
#include "common.hpp"

namespace spa {
namespace {

// Total order used for ranking: larger score first, -0 == +0, NaN below
// everything (including -inf).  The +1 keeps 0 free to mean "not a candidate".
__device__ __forceinline__ uint32_t rank_key(float s) {
    uint32_t u = __float_as_uint(s);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 1u;           // NaN
    if (u == 0x80000000u) u = 0u;                             // -0 -> +0
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return u + 1u;                                            // max finite/inf key is 0xff800000, no wrap
}

__device__ __forceinline__ int lanes_below(uint64_t mask, int lane) {
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// keys[0 .. 64*ceil((i+1)/64)): rank_key of candidates, 0 for static blocks and padding.
// Runs on one full wave; all control flow is wave-uniform.
__device__ void select_row(const uint32_t* keys, int i, int ns, int nl, int k, int T,
                           int32_t* __restrict__ idx_row, int32_t* __restrict__ cnt_out) {
    const int lane = threadIdx.x & 63;
    const int n = i + 1;
    const int chunks = (n + 63) >> 6;
    const int lo = i - nl + 1;                                // first local-window block (may be < 0)
    int n_sink = ns < n ? ns : n;
    int n_local = nl < n ? nl : n;
    int first_local = lo > 0 ? lo : 0;
    int overlap = n_sink - first_local; if (overlap < 0) overlap = 0;
    const int n_static = n_sink + n_local - overlap;
    const int n_cand = n - n_static;
    const int kk = k < n_cand ? k : n_cand;

    uint32_t thr = 0xffffffffu;   // select key > thr ... nothing, by default
    int need_eq = 0;              // plus the first need_eq candidates with key == thr
    if (kk > 0) {
        if (kk == n_cand) {
            thr = 0u;             // every candidate has key >= 1
        } else {
            uint32_t p = 0u;
            int c_at_p = n_cand;
            for (int bit = 31; bit >= 0; --bit) {
                uint32_t trial = p | (1u << bit);
                int c = 0;
                for (int m = 0; m < chunks; ++m)
                    c += __popcll(__ballot(keys[(m << 6) + lane] >= trial));
                if (c >= kk) { p = trial; c_at_p = c; if (c == kk) break; }
            }
            // p = k-th largest candidate key (or a bound that isolates exactly kk keys)
            if (c_at_p == kk) {
                thr = p - 1u;     // key >= p  <=>  key > p-1 ; p >= 1
            } else {
                int gt = 0;
                for (int m = 0; m < chunks; ++m)
                    gt += __popcll(__ballot(keys[(m << 6) + lane] > p));
                thr = p;
                need_eq = kk - gt;
            }
        }
    }
    int eq_seen = 0, out_pos = 0;
    for (int m = 0; m < chunks; ++m) {
        int j = (m << 6) + lane;
        uint32_t key = keys[j];
        bool in_row = j < n;
        bool is_static = in_row && (j < ns || j >= lo);
        bool is_eq = need_eq > 0 && key == thr && key != 0u;
        uint64_t eq_mask = __ballot(is_eq);
        bool take = is_static || (key != 0u && key > thr) ||
                    (is_eq && eq_seen + lanes_below(eq_mask, lane) < need_eq);
        uint64_t take_mask = __ballot(take);
        if (take) idx_row[out_pos + lanes_below(take_mask, lane)] = j;
        eq_seen += __popcll(eq_mask);
        out_pos += __popcll(take_mask);
    }
    for (int t = out_pos + lane; t < T; t += 64) idx_row[t] = -1;
    if (lane == 0) *cnt_out = out_pos;
}

constexpr int kWaves = 4;

// scores come from memory: [rows_total, NB, NB]
__global__ __launch_bounds__(kWaves * 64) void topk_from_scores_kernel(
    const float* __restrict__ scores, int64_t n_rows, int NB, int ns, int nl, int k, int T,
    int32_t* __restrict__ idx, int32_t* __restrict__ cnt) {
    extern __shared__ uint32_t lds_keys[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kWaves + wave;
    if (row >= n_rows) return;                               // whole wave leaves together
    const int i = (int)(row % NB);
    const int padded = ((NB + 63) >> 6) << 6;
    uint32_t* keys = lds_keys + wave * padded;
    const float* srow = scores + row * NB;
    const int lo = i - nl + 1;
    const int chunks = (i + 64) >> 6;
    for (int m = 0; m < chunks; ++m) {
        int j = (m << 6) + lane;
        uint32_t key = 0u;
        if (j <= i && !(j < ns || j >= lo)) key = rank_key(srow[j]);
        keys[j] = key;
    }
    // each wave reads back only its own slice; LDS ops of one wave are ordered
    select_row(keys, i, ns, nl, k, T, idx + row * T, cnt + row);
}

// scores computed here: lane j does the full dot product <qp[row], kp[j]>.
template <int D>
__global__ __launch_bounds__(kWaves * 64) void score_topk_kernel(
    const float* __restrict__ qp, const float* __restrict__ kp, int64_t n_rows, int Hq, int G, int NB,
    int ns, int nl, int k, int T, float scale, int32_t* __restrict__ idx, int32_t* __restrict__ cnt,
    float* __restrict__ scores_out) {
    extern __shared__ uint32_t lds_keys[];
    __shared__ float qrow[kWaves][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kWaves + wave;
    if (row >= n_rows) return;
    const int i = (int)(row % NB);
    const int64_t bh = row / NB;                            // b*Hq + h
    const int64_t b = bh / Hq;
    const int h = (int)(bh % Hq);
    const int Hkv = Hq / G;
    const float* kbase = kp + ((b * Hkv + h / G) * NB) * D;
    const int padded = ((NB + 63) >> 6) << 6;
    uint32_t* keys = lds_keys + wave * padded;
    for (int d = lane; d < D; d += 64) qrow[wave][d] = qp[row * D + d];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();             // qrow is read across lanes of this wave only
    const int lo = i - nl + 1;
    const int chunks = (i + 64) >> 6;
    for (int m = 0; m < chunks; ++m) {
        int j = (m << 6) + lane;
        uint32_t key = 0u;
        if (j <= i) {
            const float4* kr = reinterpret_cast<const float4*>(kbase + (int64_t)j * D);
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 8
            for (int d4 = 0; d4 < D / 4; ++d4) {
                float4 kv = kr[d4];
                float4 qv = *reinterpret_cast<const float4*>(&qrow[wave][d4 * 4]);
                a0 = fmaf(qv.x, kv.x, a0); a1 = fmaf(qv.y, kv.y, a1);
                a2 = fmaf(qv.z, kv.z, a2); a3 = fmaf(qv.w, kv.w, a3);
            }
            float s = scale * ((a0 + a1) + (a2 + a3));
            if (scores_out) scores_out[row * NB + j] = s;
            if (!(j < ns || j >= lo)) key = rank_key(s);
        }
        keys[j] = key;
    }
    if (scores_out)
        for (int j = i + 1 + lane; j < NB; j += 64) scores_out[row * NB + j] = -INFINITY;
    select_row(keys, i, ns, nl, k, T, idx + row * T, cnt + row);
}

// Dynamic LDS above the default cap has to be requested per kernel.
hipError_t allow_lds(const void* kernel, size_t bytes) {
    if (bytes <= 32768) return hipSuccess;
    return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

size_t keys_lds_bytes(int NB) { return (size_t)kWaves * (((NB + 63) >> 6) << 6) * sizeof(uint32_t); }

}  // namespace

hipError_t launch_topk_from_scores(const Dims& d, const float* scores, int32_t* idx, int32_t* cnt,
                                   hipStream_t st) {
    int64_t n_rows = (int64_t)d.B * d.Hq * d.NB;
    unsigned grid = (unsigned)((n_rows + kWaves - 1) / kWaves);
    hipError_t e = allow_lds((const void*)topk_from_scores_kernel, keys_lds_bytes(d.NB));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(topk_from_scores_kernel, dim3(grid), dim3(kWaves * 64), keys_lds_bytes(d.NB), st,
                       scores, n_rows, d.NB, d.ns, d.nl, d.k, d.T, idx, cnt);
    return hipGetLastError();
}

hipError_t launch_score_topk(const Dims& d, const float* qp, const float* kp, int32_t* idx,
                             int32_t* cnt, float* scores_or_null, hipStream_t st) {
    int64_t n_rows = (int64_t)d.B * d.Hq * d.NB;
    unsigned grid = (unsigned)((n_rows + kWaves - 1) / kWaves);
    size_t lds = keys_lds_bytes(d.NB);
    hipError_t e = allow_lds(d.D == 128 ? (const void*)score_topk_kernel<128> : (const void*)score_topk_kernel<64>, lds);
    if (e != hipSuccess) return e;
    if (d.D == 128)
        hipLaunchKernelGGL((score_topk_kernel<128>), dim3(grid), dim3(kWaves * 64), lds, st, qp, kp, n_rows,
                           d.Hq, d.G, d.NB, d.ns, d.nl, d.k, d.T, d.scale, idx, cnt, scores_or_null);
    else if (d.D == 64)
        hipLaunchKernelGGL((score_topk_kernel<64>), dim3(grid), dim3(kWaves * 64), lds, st, qp, kp, n_rows,
                           d.Hq, d.G, d.NB, d.ns, d.nl, d.k, d.T, d.scale, idx, cnt, scores_or_null);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace spa
