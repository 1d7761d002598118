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
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
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
// 16 bytes per lane straight from global memory into LDS (global_load_lds_dwordx4): the wave's 64
// lanes fill 1 KB starting at LDS byte address lds_addr, lane l from sbase + voff(l).  Written as
// inline assembly on purpose: the compiler models the builtin form as an access whose completion
// order is unknown, and from then on turns every wait for an LDS read into a wait for all of
// them, which defeats the read-ahead in the pipeline step.  The kernel waits for these loads
// itself (s_waitcnt vmcnt(0) before the barrier that publishes a sub-tile).
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16(uint32_t lds_addr, uint32_t voff, const void* sbase) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(size_t)(lds_void*)p; }
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
// Instruction order inside a pipeline step is written out by hand: every group between two
// fences holds one MFMA, the LDS read of an operand needed three MFMAs later and a handful of
// softmax VALU instructions, and the scheduler may not move anything across a fence.  Left to
// itself the compiler (register pressure is high) sinks each LDS read to just before the MFMA
// that uses it and clusters the VALU work, so the wave stalls on the LDS latency once per MFMA.
#define SPA_FENCE() __builtin_amdgcn_sched_barrier(0)

template <int BS>
__global__ __launch_bounds__(BS * 2, BS / 64) void attn_d128_kernel(
    const uint16_t* __restrict__ q, Strides qs, const uint16_t* __restrict__ k, Strides ks,
    const uint16_t* __restrict__ vt, const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt,
    uint16_t* __restrict__ out, Strides os, float* __restrict__ lse, int Hq, int G, int NB, int T, int S,
    float scale) {
    constexpr int NW = BS / 32;         // wavefronts
    constexpr int NSUB = BS / KT;       // sub-tiles per key block
    constexpr int LPW = 16 / NW;        // 1-KB load instructions per wave per operand per sub-tile
    constexpr int TILE_B = TILE * 2;    // bytes of a sub-tile
    // K sub-tile n lives in buffer n % 3, V^T sub-tile n in buffer n % 2.  Three K buffers make the
    // buffer index follow the period-3 rotation of the logit registers below, so every K read is a
    // per-lane base register plus an immediate offset.
    __shared__ __attribute__((aligned(1024))) uint16_t smemK[3][TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t smemV[2][TILE];

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
    auto issue_k = [&](int st, int blk, int buf) {
        const char* kt = reinterpret_cast<const char*>(kb + ((int64_t)blk * BS + (st % NSUB) * KT) * ks.t);
#pragma unroll
        for (int x = 0; x < LPW; ++x) lds_dma16(lds_address(&smemK[buf][(wave * LPW + x) * 512]), k_offb[x], kt);
    };
    auto issue_v = [&](int st, int blk) {
        const char* vtt = reinterpret_cast<const char*>(vtb + (int64_t)blk * D * BS + (st % NSUB) * KT);
#pragma unroll
        for (int x = 0; x < LPW; ++x) lds_dma16(lds_address(&smemV[st & 1][(wave * LPW + x) * 512]), v_offb[x], vtt);
    };
    auto blk_of = [&](int st) {        // key block of sub-tile st (clamped: never read past the list)
        const int e = st / NSUB;
        return sel[e < n_sel ? e : n_sel - 1];
    };

    issue_k(0, sel[0], 0);
    issue_v(0, sel[0]);
    if (n_st > 1) issue_k(1, blk_of(1), 1);

    // Q^T fragments (B operand): query row 32*wave + l32, dims 16s + 8*half .. +7
    bf16x8 qf[8];
    {
        const uint16_t* qrow = qb + (int64_t)(32 * wave + l32) * qs.t + 8 * half;
#pragma unroll
        for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qrow + 16 * s);
    }
    // Per-lane LDS byte offsets.  K (A operand of S^T = K Q^T): the lane's key row of chunk 0 and
    // its 8-dim slice s; chunk 1 and the buffer add constants.  The row assignment swaps bits 2
    // and 3, see the file header.  V^T (A operand of O^T += V^T P^T): d row l32 (+32 per d tile, a
    // constant) and the 8-key slice x of the sub-tile.
    int kofs[8], vofs[4];
    {
        const int row = swap_bits23(l32);
#pragma unroll
        for (int s = 0; s < 8; ++s) kofs[s] = 2 * (row * D + (((2 * s + half) ^ swz_k(row)) << 3));
#pragma unroll
        for (int x = 0; x < 4; ++x) vofs[x] = 2 * (l32 * KT + (((2 * x + half) ^ swz_v(l32)) << 3));
    }
    const char* const ldsK = reinterpret_cast<const char*>(&smemK[0][0]);
    const char* const ldsV = reinterpret_cast<const char*>(&smemV[0][0]);

    f32x16 oacc[4];
#pragma unroll
    for (int dc = 0; dc < 4; ++dc)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dc][r] = 0.f;
    float m_run = -INFINITY;     // reference maximum (raw logits) used for the exponentials
    float l_run = 0.f;           // this lane's half of the running denominator
    const float c = scale * 1.44269504088896340736f;
    const int q_in_blk = 32 * wave + l32;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    // The pipeline step.  Works on 32-key chunks: while the VALU turns the logits of the current
    // chunk (s_cur) into probabilities and the MFMA pipe accumulates them into O^T, the same MFMA
    // pipe also produces the logits of a later chunk (s_nxt, the same chunk position of the next
    // sub-tile), so MFMA and VALU work always come from independent dependency chains.
    //   KB: K buffer the produced chunk is read from; KC: chunk index (0/1) of both the produced
    //   and the current chunk inside their 64-key sub-tiles; vb: byte offset of the V^T buffer.
    //   f0..f3: rotating operand registers; on entry f0..f2 hold K slices 0..2 of the produced
    //   chunk, on exit (KC == 0) those of the next chunk of the same sub-tile.
    auto step = [&](auto kb_tag, auto kc_tag, f32x16& s_cur, f32x16& s_nxt, int vb, bool diag, int sub,
                    bf16x8& f0, bf16x8& f1, bf16x8& f2, bf16x8& f3) {
        constexpr int KB = decltype(kb_tag)::value, KC = decltype(kc_tag)::value;
        constexpr int KOFF = KB * TILE_B + KC * 32 * D * 2;
        auto ldk = [&](int s) { return *reinterpret_cast<const bf16x8*>(ldsK + KOFF + kofs[s]); };
        const char* const v0 = ldsV + vb + vofs[2 * KC];
        const char* const v1 = ldsV + vb + vofs[2 * KC + 1];
        auto ldv = [&](const char* base, int dc) { return *reinterpret_cast<const bf16x8*>(base + dc * 32 * KT * 2); };
        // causal mask on the diagonal block: register r of a chunk holds key
        // 32*chunk + 16*(r>>3) + 8*half + (r&7) of the sub-tile
        if (diag && KT * sub + 32 * KC + 31 > 32 * wave) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int kpos = KT * sub + 32 * KC + 16 * (r >> 3) + 8 * half + (r & 7);
                if (kpos > q_in_blk) s_cur[r] = -INFINITY;
            }
        }
        f32x16 zero;
#pragma unroll
        for (int r = 0; r < 16; ++r) zero[r] = 0.f;
        SPA_FENCE();
        // ---- logits of the look-ahead chunk, row maximum of the current chunk ---------------
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0, qf[0], zero, 0, 0, 0);
        f3 = ldk(3);
        float mx = fmaxf(s_cur[0], s_cur[1]);
        mx = fmaxf(fmaxf(mx, s_cur[2]), s_cur[3]);
        mx = fmaxf(fmaxf(mx, s_cur[4]), s_cur[5]);
        mx = fmaxf(fmaxf(mx, s_cur[6]), s_cur[7]);
        SPA_FENCE();
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1, qf[1], s_nxt, 0, 0, 0);
        f0 = ldk(4);
        mx = fmaxf(fmaxf(mx, s_cur[8]), s_cur[9]);
        mx = fmaxf(fmaxf(mx, s_cur[10]), s_cur[11]);
        mx = fmaxf(fmaxf(mx, s_cur[12]), s_cur[13]);
        mx = fmaxf(fmaxf(mx, s_cur[14]), s_cur[15]);
        SPA_FENCE();
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2, qf[2], s_nxt, 0, 0, 0);
        f1 = ldk(5);
        // Raise the reference maximum only when some row outgrew it by more than 2^8 (exp2
        // domain).  The test uses each lane's own half of the keys; the halves are combined only
        // when it fires.  Always true on the first chunk; a fully masked half (mx = -inf) never
        // triggers it and contributes exact zeros.
        const bool grow = (mx - m_run) * c > 8.0f;
        SPA_FENCE();
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f3, qf[3], s_nxt, 0, 0, 0);
        f2 = ldk(6);
        if (__any(grow)) {
            mx = fmaxf(mx, other_half(mx));
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dc = 0; dc < 4; ++dc)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[dc][r] *= alpha;
        }
        SPA_FENCE();
        // ---- probabilities of the first 16 keys --------------------------------------------
        const float mc = m_run * c;
        f32x8 e0, e1;
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0, qf[4], s_nxt, 0, 0, 0);
        f3 = ldk(7);
#pragma unroll
        for (int x = 0; x < 8; ++x) e0[x] = fmaf(s_cur[x], c, -mc);
        SPA_FENCE();
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1, qf[5], s_nxt, 0, 0, 0);
        f0 = ldv(v0, 0);
#pragma unroll
        for (int x = 0; x < 4; ++x) e0[x] = __builtin_amdgcn_exp2f(e0[x]);
        SPA_FENCE();
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2, qf[6], s_nxt, 0, 0, 0);
        f1 = ldv(v0, 1);
#pragma unroll
        for (int x = 4; x < 8; ++x) e0[x] = __builtin_amdgcn_exp2f(e0[x]);
        SPA_FENCE();
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f3, qf[7], s_nxt, 0, 0, 0);
        f2 = ldv(v0, 2);
        const bf16x8 p0 = __builtin_convertvector(e0, bf16x8);
        // the denominator sums the bf16-rounded weights, exactly what the second product uses
#pragma unroll
        for (int x = 0; x < 4; ++x)
            l_run = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{p0[2 * x], p0[2 * x + 1]}, ones, l_run, false);
        SPA_FENCE();
        // ---- O^T += V^T P^T, probabilities of the second 16 keys ---------------------------
        oacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0, p0, oacc[0], 0, 0, 0);
        f3 = ldv(v0, 3);
#pragma unroll
        for (int x = 0; x < 8; ++x) e1[x] = fmaf(s_cur[8 + x], c, -mc);
        SPA_FENCE();
        oacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1, p0, oacc[1], 0, 0, 0);
        f0 = ldv(v1, 0);
#pragma unroll
        for (int x = 0; x < 4; ++x) e1[x] = __builtin_amdgcn_exp2f(e1[x]);
        SPA_FENCE();
        oacc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2, p0, oacc[2], 0, 0, 0);
        f1 = ldv(v1, 1);
#pragma unroll
        for (int x = 4; x < 8; ++x) e1[x] = __builtin_amdgcn_exp2f(e1[x]);
        SPA_FENCE();
        oacc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f3, p0, oacc[3], 0, 0, 0);
        f2 = ldv(v1, 2);
        const bf16x8 p1 = __builtin_convertvector(e1, bf16x8);
#pragma unroll
        for (int x = 0; x < 4; ++x)
            l_run = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{p1[2 * x], p1[2 * x + 1]}, ones, l_run, false);
        SPA_FENCE();
        oacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0, p1, oacc[0], 0, 0, 0);
        f3 = ldv(v1, 3);
        SPA_FENCE();
        oacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1, p1, oacc[1], 0, 0, 0);
        if constexpr (KC == 0) f0 = *reinterpret_cast<const bf16x8*>(ldsK + KOFF + 32 * D * 2 + kofs[0]);
        SPA_FENCE();
        oacc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2, p1, oacc[2], 0, 0, 0);
        if constexpr (KC == 0) f1 = *reinterpret_cast<const bf16x8*>(ldsK + KOFF + 32 * D * 2 + kofs[1]);
        SPA_FENCE();
        oacc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f3, p1, oacc[3], 0, 0, 0);
        if constexpr (KC == 0) f2 = *reinterpret_cast<const bf16x8*>(ldsK + KOFF + 32 * D * 2 + kofs[2]);
        SPA_FENCE();
    };

    // ---- prologue: logits of the two chunks of sub-tile 0 ------------------------------
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)
    __syncthreads();
    f32x16 s0, s1, s2;                             // logits: two chunks waiting/current + one being produced
#pragma unroll
    for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
#pragma unroll
    for (int sidx = 0; sidx < 8; ++sidx) {
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(ldsK + kofs[sidx]), qf[sidx], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(ldsK + 32 * D * 2 + kofs[sidx]), qf[sidx], s1, 0, 0, 0);
    }
    int blk1 = blk_of(1), blk2 = blk_of(2);        // key blocks of sub-tiles n+1 and n+2
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    // One 64-key sub-tile n (R = n % 3): its two chunks are current (a = chunk 0, b = chunk 1, both
    // computed during sub-tile n-1); the logits of sub-tile n+1 are produced into cnext and then a.
    // Only K(n+1) and V^T(n) are read; K(n+2) goes to the buffer that K(n-1) left two barriers ago.
    auto sub_tile = [&](auto r_tag, int n, f32x16& a, f32x16& b, f32x16& cnext) {
        constexpr int R = decltype(r_tag)::value;
        using KRD = std::integral_constant<int, (R + 1) % 3>;
        // K(n+1) and V(n) have been requested; make them visible and retire the previous
        // sub-tile's readers of the V buffer refilled below.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        bf16x8 f0 = *reinterpret_cast<const bf16x8*>(ldsK + KRD::value * TILE_B + kofs[0]);
        bf16x8 f1 = *reinterpret_cast<const bf16x8*>(ldsK + KRD::value * TILE_B + kofs[1]);
        bf16x8 f2 = *reinterpret_cast<const bf16x8*>(ldsK + KRD::value * TILE_B + kofs[2]);
        bf16x8 f3;
        if (n + 2 < n_st) issue_k(n + 2, blk2, (R + 2) % 3);
        if (n + 1 < n_st) issue_v(n + 1, blk1);
        blk1 = blk2;
        blk2 = blk_of(n + 3);
        const int vb = (n & 1) * TILE_B;
        const bool diag = n >= n_st - NSUB;           // the diagonal block is always the last of the list
        const int sub = n % NSUB;
        // on the last sub-tile the look-ahead reads a stale K buffer and its result is dropped
        step(KRD{}, I0{}, a, cnext, vb, diag, sub, f0, f1, f2, f3);
        step(KRD{}, I1{}, b, a, vb, diag, sub, f0, f1, f2, f3);
    };
    using R0 = std::integral_constant<int, 0>;
    using R1 = std::integral_constant<int, 1>;
    using R2 = std::integral_constant<int, 2>;
    for (int n = 0;;) {                               // register roles rotate with period 3
        sub_tile(R0{}, n, s0, s1, s2);
        if (++n == n_st) break;
        sub_tile(R1{}, n, s2, s0, s1);
        if (++n == n_st) break;
        sub_tile(R2{}, n, s1, s2, s0);
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
