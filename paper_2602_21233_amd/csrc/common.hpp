// Shared declarations of the sparse-prefill HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sparse_prefill.h"

namespace spa {

constexpr int kMaxBlocks = 4096;  // NB limit: one score row must fit a wave's LDS slice

// Derived sizes every launcher needs.
struct Dims {
    int B, Hq, Hkv, G, S, D, Bs, NB, T;   // S, NB: query tokens / query blocks of the call
    int Skv, NBk, off;                    // key tokens, key blocks, block position of query block 0
    int ns, nl, k;
    int shared;                   // 1: block lists are per KV head (group-shared selection)
    int stride, n_dense, reach;   // strided static columns, dense bottom strip, reach of the strided columns (0 = off)
    float scale;
    int gamma_q16;                // cumulative-mass budget in 16-bit fixed point, -1 = none
    const int32_t* seq_lens;      // device array [B] of per-entry token counts (ragged batch), or nullptr
};

inline Dims dims_of(const spa_params& p) {
    Dims d;
    d.B = p.batch; d.Hq = p.n_q_heads; d.Hkv = p.n_kv_heads; d.G = p.n_q_heads / p.n_kv_heads;
    d.S = p.seq_len; d.D = p.head_dim; d.Bs = p.block_size; d.NB = (p.seq_len + p.block_size - 1) / p.block_size;   // the last block may be partial
    d.ns = p.n_sink_blocks; d.nl = p.n_local_blocks; d.k = p.top_k_blocks;
    d.off = p.kv_prefix_len / p.block_size; d.Skv = p.kv_prefix_len + p.seq_len; d.NBk = d.off + d.NB;
    d.shared = p.lists_per_kv_head != 0;
    d.stride = p.stride_blocks; d.n_dense = p.n_dense_q_blocks; d.reach = p.stride_reach_blocks;
    int64_t far = d.NBk - 1;
    if (d.reach > 0 && d.reach - 1 < far) far = d.reach - 1;
    int64_t t = (int64_t)d.ns + d.nl + d.k + (d.stride > 0 ? far / d.stride : 0);
    d.T = (int)((t < d.NBk && d.n_dense <= 0) ? t : d.NBk);
    d.scale = p.softmax_scale;
    d.gamma_q16 = -1;
    d.seq_lens = p.seq_lens;
    return d;
}

// Ragged batch: tokens of batch entry b (the tensors keep their padded length S)
__device__ __forceinline__ int entry_len(const int32_t* __restrict__ seq_lens, int b, int S) {
    if (seq_lens == nullptr) return S;
    const int v = seq_lens[b];
    return v < 0 ? 0 : (v > S ? S : v);
}

// 16 bytes that will not be read again soon: a non-temporal load keeps them from displacing
// other data in the caches (measured: 232 -> 220 us for the pooling pass at 131072 tokens)
__device__ __forceinline__ uint4 stream_load16(const uint16_t* p) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(t[0], t[1], t[2], t[3]);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

struct Strides { int64_t b, h, t; };
inline Strides strides_of(const int64_t s[3]) { return Strides{s[0], s[1], s[2]}; }

// Launchers (one per kernel file).  Each returns a hipError_t from the launch.
// k_tiled: write the pooled K in the score kernel's operand layout (tiles of 32 key blocks,
// heads ceil(NBk / 32) tiles apart) instead of row major [.., NBk, D].
hipError_t launch_pool(const Dims& d, const void* q, Strides qs, const void* k, Strides ks,
                       float* qp, float* kp, bool k_tiled, hipStream_t st);
// qg[b, kv head, :] = mean over the G query heads of the group of qp[b, head, :]  (n = NB * D values per head)
hipError_t launch_group_mean(const Dims& d, const float* qp, float* qg, hipStream_t st);
// lvn [B*Hkv, NB] fp32: ln of the mean value-vector norm of every key block.
hipError_t launch_vnorm(const Dims& d, const void* v, Strides vs, float* lvn, hipStream_t st);
// k_rows: optional device array of NB per-query-block budgets (clamped to [0, d.k] in the kernel).
// lvn: optional; added to the score of key block j (output-aware ranking).
// kp is in the tiled layout launch_pool writes with k_tiled.
// head_pattern: optional device array [Hq][3] = (n_sink, n_local, top_k) per query head.
// q: if not nullptr, the kernel pools the query blocks from Q itself (layout qs) and qp is not read.
hipError_t launch_score_topk(const Dims& d, const float* qp, const float* kp, const int32_t* k_rows,
                             const int32_t* head_pattern, const float* lvn, int32_t* idx, int32_t* cnt,
                             float* scores_or_null, const void* q, Strides qs, hipStream_t st);
hipError_t launch_topk_from_scores(const Dims& d, const float* scores, const int32_t* k_rows,
                                   const int32_t* head_pattern, int32_t* idx, int32_t* cnt, hipStream_t st);
// vt is scratch for V transposed per block, B*Hkv*NBk*Bs*D bf16.
// counts, into *n_bad (device), the list rows that break the attention kernel's layout rules
hipError_t launch_check_lists(const Dims& d, const int32_t* idx, const int32_t* cnt, int32_t* n_bad, hipStream_t st);
hipError_t launch_attn(const Dims& d, const void* q, Strides qs, const void* k, Strides ks,
                       const void* v, Strides vs, const int32_t* idx, const int32_t* cnt,
                       void* out, Strides os, float* lse, void* vt, hipStream_t st);
// The two halves of launch_attn: V -> V^T for the key blocks first .. first + n - 1 into an allocation of
// vt_bph blocks per head ([B, Hkv, vt_bph, D, Bs] bf16), and the attention on such a V^T.
hipError_t launch_transpose_v(const Dims& d, const void* v, Strides vs, void* vt, int64_t vt_bph, int first, int n,
                              hipStream_t st);
hipError_t launch_attn_vt(const Dims& d, const void* q, Strides qs, const void* k, Strides ks, const void* vt,
                          int64_t vt_bph, const int32_t* idx, const int32_t* cnt, void* out, Strides os, float* lse,
                          hipStream_t st);

}  // namespace spa
