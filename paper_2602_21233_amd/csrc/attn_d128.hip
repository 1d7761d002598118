// Block-sparse causal attention, head_dim 128 fast path for gfx950 (the "sparse
// attention kernel" stage of Sec. 4.1.1 of the AngelSlim report).
//
// Same transposed formulation as attn.hip (S^T = K Q^T, O^T += V^T P^T, one
// workgroup per (batch, head, query block), one wavefront per 32 query rows),
// restructured around what the LDS can deliver:
//   * V is transposed once per call into a workspace ([.., block, d, token]) by
//     transpose_v_kernel, so both MFMA A operands (K rows, V^T rows) are plain
//     16-byte LDS reads; the LDS transpose read is ~4x slower per byte.
//   * key blocks are consumed as 64-key sub-tiles, staged by direct
//     global->LDS loads (global_load_lds_dwordx4, no VGPR round trip) into a
//     double buffer: the loads of sub-tile n+1 fly during the math of sub-tile n
//     and there is one barrier per sub-tile.  64 KB of LDS per workgroup leaves
//     room for two workgroups per CU, so one's softmax overlaps the other's MFMA.
//   * direct loads land lane-contiguous, so bank conflicts are avoided by an
//     XOR swizzle applied on the global side (which 16-byte chunk a lane
//     fetches) instead of row padding.
//   * K rows are assigned to MFMA rows with bits 2 and 3 of the row index
//     swapped; the logits a lane ends up holding are then 8 consecutive keys per
//     16-key slice, which is exactly the B-operand order of the second product.
//   * the running maximum is only raised when a row's new maximum exceeds it by
//     more than 2^8 in the exp2 domain, so the O^T rescale is rare; the final
//     normalisation makes the result independent of this.
#include <type_traits>

#include "common.hpp"

namespace spa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

constexpr int D = 128;
constexpr int KT = 64;                 // keys per staged sub-tile
constexpr int TILE = KT * D;           // elements of one K (or V^T) sub-tile: 16 KB

__device__ __forceinline__ int swz_k(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }   // 256-B rows
__device__ __forceinline__ int swz_v(int row) { return (row >> 1) & 7; }                        // 128-B rows
// value held by lane ^ 32, via v_permlane32_swap (no LDS round trip)
__device__ __forceinline__ float other_half(float x) {
    typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
    u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    // r[0]: lanes 32..63 now hold lanes 0..31's value; r[1]: lanes 0..31 hold lanes 32..63's value
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ int swap_bits23(int x) { return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1); }

// ---------------------------------------------------------------------------
// V [B,Hkv,S,D] (strided) -> Vt [B,Hkv,NB,D,BS] contiguous.
template <int BS>
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint16_t* __restrict__ v, Strides vs, int Hkv,
                                                          int NB, uint16_t* __restrict__ vt) {
    constexpr int PITCH = D + 2;
    __shared__ uint16_t tile[BS * PITCH];
    const int blk = blockIdx.x, bh = blockIdx.y;
    const int b = bh / Hkv, h = bh % Hkv;
    const uint16_t* src = v + b * vs.b + h * vs.h + (int64_t)blk * BS * vs.t;
    const int tid = threadIdx.x;
#pragma unroll
    for (int p = 0; p < BS * D / 8 / 256; ++p) {
        int c = p * 256 + tid;
        int row = c / (D / 8), col = (c % (D / 8)) * 8;
        uint4 x = *reinterpret_cast<const uint4*>(src + (int64_t)row * vs.t + col);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[row * PITCH + col]);   // PITCH even: 4-byte aligned
        dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
    }
    __syncthreads();
    uint16_t* dstb = vt + (((int64_t)bh * NB + blk) * D) * BS;
    constexpr int CPR = BS / 8;         // 16-byte chunks per output row
#pragma unroll
    for (int p = 0; p < BS * D / 8 / 256; ++p) {
        int c = p * 256 + tid;
        int d = c / CPR, t0 = (c % CPR) * 8;
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[e] = (uint32_t)tile[(t0 + 2 * e) * PITCH + d] | ((uint32_t)tile[(t0 + 2 * e + 1) * PITCH + d] << 16);
        *reinterpret_cast<uint4*>(dstb + (int64_t)d * BS + t0) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// ---------------------------------------------------------------------------
template <int BS>
__global__ __launch_bounds__(BS * 2, BS / 64) void attn_d128_kernel(
    const uint16_t* __restrict__ q, Strides qs, const uint16_t* __restrict__ k, Strides ks,
    const uint16_t* __restrict__ vt, const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt,
    uint16_t* __restrict__ out, Strides os, float* __restrict__ lse, int Hq, int G, int NB, int T, int S,
    float scale) {
    constexpr int NW = BS / 32;         // wavefronts
    constexpr int NSUB = BS / KT;       // sub-tiles per key block
    constexpr int LPW = 16 / NW;        // 1-KB load instructions per wave per operand per sub-tile
    __shared__ __attribute__((aligned(1024))) uint16_t smem[2][2][TILE];   // [buffer][K | V^T]

    // Workgroup -> (b, kv head, query block, head in group).  Workgroup ids go round robin over
    // the 8 XCDs.  In time, the whole chip works through one KV head after the other, so that the
    // K and V^T of the current head (tens of MB) stay in the memory-side cache; in space, each XCD
    // takes a contiguous range of that head's query blocks with all G heads of the group, which
    // share most of their key blocks in that XCD's L2.
    const int per_head = NB * G;
    int wg = blockIdx.x;
    const int head_slot = wg / per_head;                  // b * Hkv + kv head
    int local = wg % per_head;
    if ((per_head & 7) == 0) local = (local & 7) * (per_head >> 3) + (local >> 3);
    const int g = local % G;
    const int i = local / G;
    const int Hkv = Hq / G;
    const int kvh = head_slot % Hkv;
    const int b = head_slot / Hkv;
    const int h = kvh * G + g;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;

    const uint16_t* qb = q + b * qs.b + h * qs.h + (int64_t)i * BS * qs.t;
    const uint16_t* kb = k + b * ks.b + kvh * ks.h;
    const uint16_t* vtb = vt + ((int64_t)(b * Hkv + kvh) * NB) * D * BS;
    const int64_t row_id = ((int64_t)b * Hq + h) * NB + i;
    const int32_t* sel = idx + row_id * T;
    const int n_sel = cnt[row_id];
    const int n_st = n_sel * NSUB;

    // Direct global->LDS loads: instruction `inst` of a sub-tile fills 1 KB of LDS in lane order
    // (4 K rows of 256 B, or 8 V^T rows of 128 B); the lane picks the global 16-byte chunk whose
    // swizzled position it is writing.  Per-lane byte offsets are fixed for the whole kernel; the
    // tile base is wave-uniform, so each load is base (SGPRs) + 32-bit lane offset.
    uint32_t k_offb[LPW], v_offb[LPW];
#pragma unroll
    for (int x = 0; x < LPW; ++x) {
        const int inst = wave * LPW + x;
        const int krow = 4 * inst + (lane >> 4);
        const int vrow = 8 * inst + (lane >> 3);
        k_offb[x] = 2u * ((uint32_t)krow * (uint32_t)ks.t + (uint32_t)(((lane & 15) ^ swz_k(krow)) << 3));
        v_offb[x] = 2u * (uint32_t)(vrow * BS + (((lane & 7) ^ swz_v(vrow)) << 3));
    }
    // K and V^T sub-tiles are staged separately: K runs one sub-tile ahead of V^T because the
    // logits of sub-tile n+1 are computed while the softmax of sub-tile n is in progress.
    auto issue_k = [&](int st, int blk) {
        const char* kt = reinterpret_cast<const char*>(kb + ((int64_t)blk * BS + (st % NSUB) * KT) * ks.t);
#pragma unroll
        for (int x = 0; x < LPW; ++x)
            __builtin_amdgcn_global_load_lds((gbl_void*)(kt + k_offb[x]),
                                             (lds_void*)&smem[st & 1][0][(wave * LPW + x) * 512], 16, 0, 0);
    };
    auto issue_v = [&](int st, int blk) {
        const char* vtt = reinterpret_cast<const char*>(vtb + (int64_t)blk * D * BS + (st % NSUB) * KT);
#pragma unroll
        for (int x = 0; x < LPW; ++x)
            __builtin_amdgcn_global_load_lds((gbl_void*)(vtt + v_offb[x]),
                                             (lds_void*)&smem[st & 1][1][(wave * LPW + x) * 512], 16, 0, 0);
    };
    auto blk_of = [&](int st) {        // key block of sub-tile st (clamped: never read past the list)
        const int e = st / NSUB;
        return sel[e < n_sel ? e : n_sel - 1];
    };

    issue_k(0, sel[0]);
    issue_v(0, sel[0]);
    if (n_st > 1) issue_k(1, blk_of(1));

    // Q^T fragments (B operand): query row 32*wave + l32, dims 16s + 8*half .. +7
    bf16x8 qf[8];
    {
        const uint16_t* qrow = qb + (int64_t)(32 * wave + l32) * qs.t + 8 * half;
#pragma unroll
        for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qrow + 16 * s);
    }
    // LDS read offsets (elements within a tile)
    int k_rd[2], k_sw[2];
#pragma unroll
    for (int kc = 0; kc < 2; ++kc) {
        const int row = swap_bits23(32 * kc + l32);
        k_rd[kc] = row * D;
        k_sw[kc] = swz_k(row);
    }
    int v_rd[4], v_sw[4];
#pragma unroll
    for (int dc = 0; dc < 4; ++dc) {
        const int row = 32 * dc + l32;
        v_rd[dc] = row * KT;
        v_sw[dc] = swz_v(row);
    }
    f32x16 oacc[4];
#pragma unroll
    for (int dc = 0; dc < 4; ++dc)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dc][r] = 0.f;
    float m_run = -INFINITY;     // reference maximum (raw logits) used for the exponentials
    float l_run = 0.f;           // this lane's half of the running denominator
    const float c = scale * 1.44269504088896340736f;
    const int q_in_blk = 32 * wave + l32;

    // One K fragment (A operand of S^T = K Q^T): 8 dims of the lane's key row.
    auto k_frag = [&](const uint16_t* sK, int kc, int s) {
        return *reinterpret_cast<const bf16x8*>(sK + k_rd[kc] + (((2 * s + half) ^ k_sw[kc]) << 3));
    };

    // The pipeline step.  Works on 32-key chunks: while the VALU turns the logits of the current
    // chunk (s_cur) into probabilities and the MFMA pipe accumulates them into O^T, the same MFMA
    // pipe also produces the logits of a later chunk (s_nxt, the same chunk position of the next
    // sub-tile), so MFMA and VALU work always come from independent dependency chains.
    //   KCN / KCC: chunk index (0/1) inside its 64-key sub-tile of the produced / current chunk.
    auto step = [&](auto kcn_tag, auto kcc_tag, f32x16& s_cur, f32x16& s_nxt, const uint16_t* sKn,
                    const uint16_t* sV, bool diag, int sub) {
        constexpr int KCN = decltype(kcn_tag)::value, KCC = decltype(kcc_tag)::value;
        // causal mask on the diagonal block: register r of a chunk holds key
        // 32*chunk + 16*(r>>3) + 8*half + (r&7) of the sub-tile
        if (diag && KT * sub + 32 * KCC + 31 > 32 * wave) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int kpos = KT * sub + 32 * KCC + 16 * (r >> 3) + 8 * half + (r & 7);
                if (kpos > q_in_blk) s_cur[r] = -INFINITY;
            }
        }
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int sidx = 0; sidx < 4; ++sidx)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(sKn, KCN, sidx), qf[sidx], acc, 0, 0, 0);
        float mx = fmaxf(s_cur[0], s_cur[1]);
#pragma unroll
        for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s_cur[r]);
        mx = fmaxf(mx, other_half(mx));
        // Raise the reference maximum only when some row outgrew it by more than 2^8 (exp2
        // domain); wave-uniform; always true on the first chunk.  A fully masked chunk
        // (mx = -inf) never triggers it and contributes exact zeros.
        if (__any((mx - m_run) * c > 8.0f)) {
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dc = 0; dc < 4; ++dc)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[dc][r] *= alpha;
        }
#pragma unroll
        for (int sidx = 4; sidx < 8; ++sidx)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(sKn, KCN, sidx), qf[sidx], acc, 0, 0, 0);
        s_nxt = acc;
        const float mc = m_run * c;
        float psum = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            f32x8 pf;
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                pf[x] = __builtin_amdgcn_exp2f(fmaf(s_cur[8 * u + x], c, -mc));
                psum += pf[x];
            }
            const bf16x8 pb = __builtin_convertvector(pf, bf16x8);
            const int chunk = 2 * (2 * KCC + u) + half;          // 8 keys = one 16-byte chunk of a V^T row
#pragma unroll
            for (int dc = 0; dc < 4; ++dc) {
                bf16x8 a = *reinterpret_cast<const bf16x8*>(sV + v_rd[dc] + ((chunk ^ v_sw[dc]) << 3));
                oacc[dc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, oacc[dc], 0, 0, 0);
            }
        }
        l_run += psum;
    };

    // ---- prologue: logits of the two chunks of sub-tile 0 ------------------------------
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)
    __syncthreads();
    f32x16 s0, s1, s2;                             // logits: two chunks waiting/current + one being produced
#pragma unroll
    for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
#pragma unroll
    for (int sidx = 0; sidx < 8; ++sidx) {
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(smem[0][0], 0, sidx), qf[sidx], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(smem[0][0], 1, sidx), qf[sidx], s1, 0, 0, 0);
    }
    int blk1 = blk_of(1), blk2 = blk_of(2);        // key blocks of sub-tiles n+1 and n+2
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    // One 64-key sub-tile n: its two chunks are current (a = chunk 0, b = chunk 1, both computed
    // during sub-tile n-1); the logits of sub-tile n+1 are produced into c and then a.  Only K(n+1)
    // and V^T(n) are read, so each operand needs just two LDS buffers.
    auto sub_tile = [&](int n, f32x16& a, f32x16& b, f32x16& cnext) {
        // K(n+1) and V(n) have been requested; make them visible and retire the previous
        // sub-tile's readers of the buffers refilled below.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (n + 2 < n_st) issue_k(n + 2, blk2);
        if (n + 1 < n_st) issue_v(n + 1, blk1);
        blk1 = blk2;
        blk2 = blk_of(n + 3);
        const uint16_t* sKn = smem[(n + 1) & 1][0];   // on the last sub-tile: idle buffer, result dropped
        const uint16_t* sV = smem[n & 1][1];
        const bool diag = n >= n_st - NSUB;           // the diagonal block is always the last of the list
        const int sub = n % NSUB;
        step(I0{}, I0{}, a, cnext, sKn, sV, diag, sub);
        step(I1{}, I1{}, b, a, sKn, sV, diag, sub);
    };
    for (int n = 0;;) {                               // register roles rotate with period 3
        sub_tile(n, s0, s1, s2);
        if (++n == n_st) break;
        sub_tile(n, s2, s0, s1);
        if (++n == n_st) break;
        sub_tile(n, s1, s2, s0);
        if (++n == n_st) break;
    }

    // ---- epilogue ----------------------------------------------------------------
    const float l_tot = l_run + other_half(l_run);
    const float inv = 1.0f / l_tot;
    uint16_t* orow = out + b * os.b + h * os.h + ((int64_t)i * BS + q_in_blk) * os.t;
#pragma unroll
    for (int dc = 0; dc < 4; ++dc)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            f32x4 o4;
#pragma unroll
            for (int x = 0; x < 4; ++x) o4[x] = oacc[dc][4 * rq + x] * inv;
            *reinterpret_cast<bf16x4*>(orow + 32 * dc + 8 * rq + 4 * half) = __builtin_convertvector(o4, bf16x4);
        }
    if (lse != nullptr && half == 0)
        lse[((int64_t)b * Hq + h) * S + (int64_t)i * BS + q_in_blk] = m_run * scale + __logf(l_tot);
}

template <int BS>
hipError_t launch(const Dims& d, const void* q, Strides qs, const void* k, Strides ks, const void* v,
                  Strides vs, const int32_t* idx, const int32_t* cnt, void* out, Strides os, float* lse,
                  void* vt, hipStream_t st) {
    hipLaunchKernelGGL((transpose_v_kernel<BS>), dim3(d.NB, d.B * d.Hkv), dim3(256), 0, st,
                       (const uint16_t*)v, vs, d.Hkv, d.NB, (uint16_t*)vt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int64_t nwg = (int64_t)d.B * d.Hq * d.NB;
    hipLaunchKernelGGL((attn_d128_kernel<BS>), dim3((unsigned)nwg), dim3(BS * 2), 0, st, (const uint16_t*)q, qs,
                       (const uint16_t*)k, ks, (const uint16_t*)vt, idx, cnt, (uint16_t*)out, os, lse, d.Hq,
                       d.G, d.NB, d.T, d.S, d.scale);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_d128(const Dims& d, const void* q, Strides qs, const void* k, Strides ks,
                            const void* v, Strides vs, const int32_t* idx, const int32_t* cnt, void* out,
                            Strides os, float* lse, void* vt, hipStream_t st) {
    if (d.D != 128 || vt == nullptr) return hipErrorInvalidValue;
    if (d.Bs == 128) return launch<128>(d, q, qs, k, ks, v, vs, idx, cnt, out, os, lse, vt, st);
    if (d.Bs == 64) return launch<64>(d, q, qs, k, ks, v, vs, idx, cnt, out, os, lse, vt, st);
    return hipErrorInvalidValue;
}

}  // namespace spa
