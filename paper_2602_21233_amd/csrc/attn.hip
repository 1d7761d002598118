// Block-sparse causal attention over selected key blocks (the "sparse attention
// kernel" stage of Sec. 4.1.1 of the AngelSlim report), for gfx950.
//
// One workgroup owns one (batch, query head, query block); each of its
// BS/32 wavefronts owns 32 query rows.  For every selected key block the K and V
// tiles are staged in LDS and the wave computes the TRANSPOSED logits tile
//   S^T[key, query] = K . Q^T      (v_mfma_f32_32x32x16_bf16, A = K from LDS,
//                                   B = Q^T held in registers for the whole kernel)
// so that one lane holds 64 of the 128 logits of a single query: the online
// softmax needs one cross-lane exchange (lane ^ 32) per statistic, the rescale
// factor is a per-lane scalar, and exp(S^T) is already in the B-operand layout
// of the second product
//   O^T[d, query] += V^T . P^T     (A = V^T read from the row-major V tile with
//                                   the LDS transpose load ds_read_b64_tr_b16).
// The list of key blocks is ascending and ends with the diagonal block, so only
// the last iteration applies the causal mask.
#include "common.hpp"

namespace spa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

__device__ __forceinline__ bf16x8 lds_read_tr_pair(const uint16_t* p0, const uint16_t* p1) {
    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p0);
    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p1);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int BS, int D>
__global__ __launch_bounds__(BS * 2) void attn_kernel(
    const uint16_t* __restrict__ q, Strides qs, const uint16_t* __restrict__ k, Strides ks,
    const uint16_t* __restrict__ v, Strides vs, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cnt, uint16_t* __restrict__ out, Strides os, float* __restrict__ lse,
    int Hq, int G, int NB, int T, int S, float scale, int shared, int Skv, const int32_t* __restrict__ seq_lens) {
    constexpr int NT = BS * 2;        // threads
    constexpr int KC = BS / 32;       // 32-key chunks of a key tile
    constexpr int DS = D / 16;        // 16-wide slices of head_dim (QK^T reduction)
    constexpr int DC = D / 32;        // 32-wide chunks of head_dim (rows of O^T)
    constexpr int LDK = D + 8;        // K row pitch: +16 B  -> conflict-free 16-byte column reads
    constexpr int LDV = D + 32;       // V row pitch: +64 B  -> conflict-free transpose reads
    constexpr int CPT = D / 16;       // 16-byte chunks per thread per tile
    __shared__ __attribute__((aligned(16))) uint16_t sK[BS * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t sV[BS * LDV];

    // Workgroup -> (b, kv head, query block, head in group).  Consecutive
    // workgroup ids go round-robin over the 8 XCDs, so give each XCD one
    // contiguous slice of the logical order: the G heads of a group and
    // neighbouring query blocks, which share most of their key blocks, then
    // meet in the same L2.
    const int nwg = gridDim.x;
    int wg = blockIdx.x;
    if ((nwg & 7) == 0) wg = (wg & 7) * (nwg >> 3) + (wg >> 3);
    const int g = wg % G;
    int rest = wg / G;
    const int i = rest % NB;
    rest /= NB;
    const int Hkv = Hq / G;
    const int kvh = rest % Hkv;
    const int b = rest / Hkv;
    const int h = kvh * G + g;
    // ragged batch: this entry's own length; query blocks past it leave (the whole workgroup, before any barrier)
    const int Sb = entry_len(seq_lens, b, S);
    if (i * BS >= Sb) return;
    const int Skvb = Skv - S + Sb;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int t16 = lane & 15, dsub = (lane >> 4) & 1;

    const uint16_t* qb = q + b * qs.b + h * qs.h + (int64_t)i * BS * qs.t;
    const uint16_t* kb = k + b * ks.b + kvh * ks.h;
    const uint16_t* vb = v + b * vs.b + kvh * vs.h;
    // block lists are per query head, or per KV head when the group shares its selection
    const int64_t row_id = shared ? ((int64_t)b * Hkv + kvh) * NB + i : ((int64_t)b * Hq + h) * NB + i;
    const int32_t* sel = idx + row_id * T;
    const int n_sel = cnt[row_id];

    // Q^T fragments (B operand): lane holds query row 32*wave + l32, dims 16s + 8*half .. +7.
    bf16x8 qf[DS];
    {
        // rows past the end of a partial last block read the last token (never stored)
        int qr = 32 * wave + l32;
        if (i * BS + qr > Sb - 1) qr = Sb - 1 - i * BS;
        const uint16_t* qrow = qb + (int64_t)qr * qs.t + 8 * half;
#pragma unroll
        for (int s = 0; s < DS; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qrow + 16 * s);
    }

    f32x16 oacc[DC];
#pragma unroll
    for (int dc = 0; dc < DC; ++dc)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dc][r] = 0.f;
    float m_run = -INFINITY;   // running max of the raw (unscaled) logits of this lane's query
    float l_run = 0.f;         // this lane's half of the running sum of exponentials
    const float c = scale * 1.44269504088896340736f;

    // tile staging: thread -> CPT 16-byte chunks of the K tile and of the V tile
    uint4 kreg[CPT], vreg[CPT];
    auto fetch = [&](int blk) {
        const uint16_t* kt = kb + (int64_t)blk * BS * ks.t;
        const uint16_t* vt = vb + (int64_t)blk * BS * vs.t;
        const int last_row = Skvb - 1 - blk * BS;       // >= BS - 1 except in a partial last block
#pragma unroll
        for (int p = 0; p < CPT; ++p) {
            int cidx = p * NT + tid;
            int row = cidx / (D / 8), col = (cidx % (D / 8)) * 8;
            if (row > last_row) row = last_row;         // keys past the end: re-read the last token, always masked
            kreg[p] = *reinterpret_cast<const uint4*>(kt + (int64_t)row * ks.t + col);
            vreg[p] = *reinterpret_cast<const uint4*>(vt + (int64_t)row * vs.t + col);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int p = 0; p < CPT; ++p) {
            int cidx = p * NT + tid;
            int row = cidx / (D / 8), col = (cidx % (D / 8)) * 8;
            *reinterpret_cast<uint4*>(&sK[row * LDK + col]) = kreg[p];
            *reinterpret_cast<uint4*>(&sV[row * LDV + col]) = vreg[p];
        }
    };

    fetch(sel[0]);
    for (int e = 0; e < n_sel; ++e) {
        __syncthreads();                 // every wave is done reading the previous tile
        stage();
        __syncthreads();
        if (e + 1 < n_sel) fetch(sel[e + 1]);

        // ---- S^T = K Q^T --------------------------------------------------
        f32x16 sacc[KC];
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kc][r] = 0.f;
            const uint16_t* krow = &sK[(32 * kc + l32) * LDK + 8 * half];
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                bf16x8 a = *reinterpret_cast<const bf16x8*>(krow + 16 * s);
                sacc[kc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], sacc[kc], 0, 0, 0);
            }
        }
        // ---- causal mask on the diagonal block (always the last entry) -----
        if (e == n_sel - 1) {
            const int qpos = 32 * wave + l32;
#pragma unroll
            for (int kc = 0; kc < KC; ++kc)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int kpos = 32 * kc + 8 * (r >> 2) + 4 * half + (r & 3);
                    if (kpos > qpos) sacc[kc][r] = -INFINITY;
                }
        }
        // ---- online softmax ------------------------------------------------
        float mx = sacc[0][0];
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kc][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);            // finite: the diagonal key is always visible
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        const float mc = m_new * c;
        float psum = 0.f;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float pv = __builtin_amdgcn_exp2f(fmaf(sacc[kc][r], c, -mc));
                sacc[kc][r] = pv;
                psum += pv;
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int dc = 0; dc < DC; ++dc)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dc][r] *= alpha;

        // ---- O^T += V^T P^T -------------------------------------------------
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                f32x8 pf;
#pragma unroll
                for (int x = 0; x < 8; ++x) pf[x] = sacc[kc][8 * u + x];
                bf16x8 pb = __builtin_convertvector(pf, bf16x8);
                // keys of this 16-key slice held by this lane: base0 + 0..3 and base0 + 8 + 0..3
                const int key0 = 32 * kc + 16 * u + 4 * half + (t16 >> 2);
                const uint16_t* v0 = &sV[key0 * LDV + 16 * dsub + 4 * (t16 & 3)];
                const uint16_t* v1 = v0 + 8 * LDV;
#pragma unroll
                for (int dc = 0; dc < DC; ++dc) {
                    bf16x8 a = lds_read_tr_pair(v0 + 32 * dc, v1 + 32 * dc);
                    oacc[dc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, oacc[dc], 0, 0, 0);
                }
            }
    }

    // ---- epilogue: normalise, write O (bf16) and LSE ---------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.0f / l_tot;
    const int qpos = 32 * wave + l32;
    if (i * BS + qpos >= Sb) return;                     // token past the end of a partial last block
    uint16_t* orow = out + b * os.b + h * os.h + ((int64_t)i * BS + qpos) * os.t;
#pragma unroll
    for (int dc = 0; dc < DC; ++dc)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            typedef __attribute__((ext_vector_type(4))) float f32x4;
            f32x4 o4;
#pragma unroll
            for (int x = 0; x < 4; ++x) o4[x] = oacc[dc][4 * rq + x] * inv;
            bf16x4 ob = __builtin_convertvector(o4, bf16x4);
            *reinterpret_cast<bf16x4*>(orow + 32 * dc + 8 * rq + 4 * half) = ob;
        }
    if (lse != nullptr && half == 0)
        lse[((int64_t)b * Hq + h) * S + (int64_t)i * BS + qpos] = m_run * scale + __logf(l_tot);
}

template <int BS, int D>
hipError_t launch(const Dims& d, const void* q, Strides qs, const void* k, Strides ks, const void* v,
                  Strides vs, const int32_t* idx, const int32_t* cnt, void* out, Strides os, float* lse,
                  hipStream_t st) {
    int64_t nwg = (int64_t)d.B * d.Hq * d.NB;
    hipLaunchKernelGGL((attn_kernel<BS, D>), dim3((unsigned)nwg), dim3(BS * 2), 0, st,
                       (const uint16_t*)q, qs, (const uint16_t*)k, ks, (const uint16_t*)v, vs, idx, cnt,
                       (uint16_t*)out, os, lse, d.Hq, d.G, d.NB, d.T, d.S, d.scale, d.shared, d.Skv, d.seq_lens);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn(const Dims& d, const void* q, Strides qs, const void* k, Strides ks,
                       const void* v, Strides vs, const int32_t* idx, const int32_t* cnt, void* out,
                       Strides os, float* lse, hipStream_t st) {
    if (d.Bs == 128 && d.D == 128) return launch<128, 128>(d, q, qs, k, ks, v, vs, idx, cnt, out, os, lse, st);
    if (d.Bs == 64 && d.D == 128) return launch<64, 128>(d, q, qs, k, ks, v, vs, idx, cnt, out, os, lse, st);
    if (d.Bs == 128 && d.D == 64) return launch<128, 64>(d, q, qs, k, ks, v, vs, idx, cnt, out, os, lse, st);
    if (d.Bs == 64 && d.D == 64) return launch<64, 64>(d, q, qs, k, ks, v, vs, idx, cnt, out, os, lse, st);
    return hipErrorInvalidValue;
}

}  // namespace spa
