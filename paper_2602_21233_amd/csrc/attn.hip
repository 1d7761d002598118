// Block-sparse causal attention for gfx950 (the "sparse attention kernel" stage of
// Sec. 4.1.1 of the AngelSlim report), head_dim 128 or 64, blocks of 128 or 64 tokens.
//
// Transposed formulation: S^T = K Q^T, O^T += V^T P^T with v_mfma_f32_32x32x16_bf16, one
// workgroup per (batch, head, query block) (two heads of a KV group per workgroup when the group
// shares its block list), one wavefront per 32 query rows.  A lane then
// owns the logits of one query: the rescale factor is a per-lane scalar and exp(S^T) is
// already the B operand of the second product.  Built around what the LDS can deliver:
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
//   * no running maximum: weights are 2^(x*c - m*c) against a reference m that is only moved
//     when a query's running denominator passes 2^40 (one compare per step); the final
//     normalisation makes the result independent of m, and floating point keeps the relative
//     precision of weights and sums at any magnitude in between.
//   * a step (32 keys) overlaps three chains: logits of chunk n+2 (MFMA), weights of chunk
//     n+1 (VALU), O^T += V^T P^T of chunk n (MFMA); its instruction order is fixed by hand.
// Blocks of 64 tokens with one head per workgroup run attn_chunked_kernel: the same step, staged in
// 32-key chunks through half the LDS, so that two wavefronts share a SIMD.
#include <type_traits>

#include "common.hpp"

namespace spa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

constexpr int KT = 64;                 // keys per staged sub-tile

__device__ __forceinline__ int swz_v(int row) { return (row >> 1) & 7; }                        // 128-B rows
// K rows are 2 * head_dim bytes: 256 B (16 chunks of 16 B) or 128 B (8 chunks, same rule as V^T rows)
template <int HD>
__device__ __forceinline__ int swz_k(int row) {
    if constexpr (HD == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    else return (row >> 1) & 7;
}
// value held by lane ^ 32, via v_permlane32_swap (no LDS round trip)
__device__ __forceinline__ float other_half(float x) {
    typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
    u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    // r[0]: lanes 32..63 now hold lanes 0..31's value; r[1]: lanes 0..31 hold lanes 32..63's value
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
// 16 bytes per lane straight from global memory into LDS (global_load_lds_dwordx4): the wave's 64
// lanes fill 1 KB starting at LDS byte address lds_addr + IMM, lane l from sbase + voff(l).  Written as
// inline assembly on purpose: the compiler models the builtin form as an access whose completion
// order is unknown, and from then on turns every wait for an LDS read into a wait for all of
// them, which defeats the read-ahead in the pipeline step.  The kernel waits for these loads
// itself (s_waitcnt vmcnt(0) before the barrier that publishes a sub-tile).
#pragma clang diagnostic ignored "-Winline-asm"
template <int IMM>
__device__ __forceinline__ void lds_dma16(uint32_t lds_addr, uint32_t voff, const void* sbase) {
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase), "i"(IMM)
                 : "memory", "m0", "scc");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(size_t)(lds_void*)p; }
__device__ __forceinline__ int swap_bits23(int x) { return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1); }

// ---------------------------------------------------------------------------
// V [B,Hkv,S,D] (strided) -> Vt [B,Hkv,vt_bph,D,BS] contiguous, blocks first .. first + gridDim.x - 1.
// vt_bph: blocks per head in the V^T allocation (>= the key blocks of the call); first: first block to do
template <int BS, int D>
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint16_t* __restrict__ v, Strides vs, int Hkv,
                                                          int64_t vt_bph, int S, uint16_t* __restrict__ vt,
                                                          const int32_t* __restrict__ seq_lens, int Sq, int first) {
    constexpr int PITCH = D + 2;
    __shared__ uint16_t tile[BS * PITCH];
    const int blk = first + blockIdx.x, bh = blockIdx.y;
    const int b = bh / Hkv, h = bh % Hkv;
    const uint16_t* src = v + b * vs.b + h * vs.h + (int64_t)blk * BS * vs.t;
    const int tid = threadIdx.x;
    const int Sb = S - Sq + entry_len(seq_lens, b, Sq);    // ragged batch: key tokens of this entry
    if (blk * BS >= Sb) return;                            // block past its end: never read by the attention kernel
    const int n_valid = Sb - blk * BS < BS ? Sb - blk * BS : BS;
#pragma unroll
    for (int p = 0; p < BS * D / 8 / 256; ++p) {
        int c = p * 256 + tid;
        int row = c / (D / 8), col = (c % (D / 8)) * 8;
        uint4 x = make_uint4(0u, 0u, 0u, 0u);           // tokens past the end of a partial last block: zeros
        if (row < n_valid) {                            // V itself is not read again: non-temporal load
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (int64_t)row * vs.t + col));
            x = make_uint4(t[0], t[1], t[2], t[3]);
        }
        uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[row * PITCH + col]);   // PITCH even: 4-byte aligned
        dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
    }
    __syncthreads();
    uint16_t* dstb = vt + (((int64_t)bh * vt_bph + blk) * D) * BS;
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
// fences holds one MFMA, the LDS read of an operand needed three MFMAs later and a few softmax
// VALU instructions, and the scheduler may not move anything across a fence.  Left to itself the
// compiler (register pressure is high) sinks each LDS read to just before the MFMA that uses it
// and clusters the VALU work, so the wave stalls on the LDS latency once per MFMA.
#define SPA_FENCE() __builtin_amdgcn_sched_barrier(0)

// How the query blocks of a head are dealt to the 8 XCDs (workgroup ids go round robin over the
// XCDs and are dispatched in id order, so the XCDs advance through their sequences in step: what
// has to be equal is the work of the rows that sit at the same position of the 8 sequences).
//   - the n_dense rows of a Tri-shape strip (each visits up to NB blocks) are dealt one by one;
//   - the other rows are dealt in runs of `run` consecutive rows, last row first.  Neighbouring
//     rows share their local-window blocks in the XCD's L2, which favours runs; rows whose length
//     varies with the position (budget schedule, strided columns, the short first rows) favour a
//     fine deal.  run = 8 for the plain A-shape, 1 for the extended patterns.
// seq_len = workgroups per (head, XCD) in the grid; surplus workgroups exit at once.
struct RowDeal {
    int n_dense, run, seq_len;
};

// nh: query heads served by one workgroup (their workgroups per row position number G / nh)
RowDeal deal_rows(const Dims& d, int nh) {
    RowDeal r;
    r.n_dense = d.n_dense < d.NB ? d.n_dense : d.NB;
    r.run = (d.stride > 0 || d.n_dense > 0) ? 1 : 8;
    const int runs = (d.NB - r.n_dense + r.run - 1) / r.run;
    r.seq_len = (((r.n_dense + 7) >> 3) + ((runs + 7) >> 3) * r.run) * (d.G / nh);
    return r;
}

template <int N>
using IC = std::integral_constant<int, N>;
// f(IC<0>{}), ..., f(IC<N-1>{})
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(IC<N - 1>{});
    }
}

// ---------------------------------------------------------------------------
// What the two attention kernels below share: the row a workgroup serves, its block list, the
// softmax arithmetic of a wavefront, the instruction groups of a pipeline step, the final store.
// They differ in how the K and V^T tiles are staged.

// Workgroup -> (b, kv head, query block, head in group).  In time, the whole chip works
// through one KV head after the other, so that the K and V^T of the current head (tens of MB)
// stay in the memory-side cache; in space, see RowDeal.  All G heads of a group follow each
// other, they share most of their key blocks.
struct RowOfWorkgroup {
    int i, b, kvh;      // query block, batch entry, KV head
    int first_head;     // first of the workgroup's NH query heads within the group
    int Sb, Skv;        // this entry's own query and key tokens (ragged batch)
};
// false: nothing to do (a surplus workgroup, or a query block past the entry's end); the whole
// workgroup then leaves, before any barrier
template <int BS, int NH>
__device__ __forceinline__ bool row_of_workgroup(const RowDeal& deal, int Hq, int G, int NB, int S, int Skv_max,
                                                 const int32_t* __restrict__ seq_lens, RowOfWorkgroup& r) {
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int head_slot = slot / deal.seq_len;            // b * Hkv + kv head
    const int within = slot % deal.seq_len;
    const int GH = G / NH;                                // workgroups per row position
    const int pos = within / GH;                          // position in this XCD's row sequence
    const int n_single = (deal.n_dense + 7) >> 3;
    if (pos < n_single) {
        const int hidx = pos * 8 + xcd;
        if (hidx >= deal.n_dense) return false;
        r.i = NB - 1 - hidx;
    } else {
        const int rr = pos - n_single;
        const int ridx = ((rr / deal.run) * 8 + xcd) * deal.run + rr % deal.run;
        if (ridx >= NB - deal.n_dense) return false;
        r.i = NB - deal.n_dense - 1 - ridx;
    }
    const int Hkv = Hq / G;
    r.kvh = head_slot % Hkv;
    r.b = head_slot / Hkv;
    r.first_head = (within % GH) * NH;
    r.Sb = entry_len(seq_lens, r.b, S);
    if (r.i * BS >= r.Sb) return false;
    r.Skv = Skv_max - S + r.Sb;
    return true;
}

// A row's block list.  Lists are the caller's: a count outside [1, T] or a block outside the entry's
// own key blocks [0, ceil(Skv / BS)) is clamped so that a malformed list can never make the kernel
// read outside the tensors (the row's output is then unspecified).  The bound is the entry's, not
// the padded NBk: in a ragged batch a block past the entry's last token would make the
// partial-block path of the tile loads compute a negative last row.  Skv >= 1.  Scalar work, once
// per list entry.
struct BlockList {
    const int32_t* sel;
    int n_sel, blk_last;
    __device__ __forceinline__ BlockList(const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt, int64_t row_id,
                                         int T, int Skv, int BS, int NBk)
        : sel(idx + row_id * T) {
        const int n = cnt[row_id];
        n_sel = n < 1 ? 1 : (n > T ? T : n);
        blk_last = (Skv - 1) / BS < NBk - 1 ? (Skv - 1) / BS : NBk - 1;
    }
    __device__ __forceinline__ int at(int e) const {
        const int blk = sel[e];
        return blk < 0 ? 0 : (blk > blk_last ? blk_last : blk);
    }
    // entry e, or the last one when e is past the end (look-ahead never reads past the list)
    __device__ __forceinline__ int at_or_last(int e) const { return at(e < n_sel ? e : n_sel - 1); }
};

// Q^T fragments (B operand of S^T = K Q^T): query row 32*wq + l32 of the block, dims 16s + 8*half .. +7.
// Rows past the end of a partial last block read the last token (their results are never stored).
template <int BS, int D>
__device__ __forceinline__ void load_q_fragments(const uint16_t* qb, int64_t q_stride_t, int i, int Sb, int wq, int l32,
                                                 int half, bf16x8 (&qf)[D / 16]) {
    int qr = 32 * wq + l32;
    if (i * BS + qr > Sb - 1) qr = Sb - 1 - i * BS;
    const uint16_t* qrow = qb + (int64_t)qr * q_stride_t + 8 * half;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qrow + 16 * s);
}

// causal mask inside the diagonal block: register r of the 32-key chunk that starts at key
// `first_key` of the block holds key first_key + 16*(r>>3) + 8*half + (r&7)
__device__ __forceinline__ void mask_diagonal_chunk(f32x16& s, int first_key, int wq, int half, int q_in_blk) {
    if (first_key + 31 > 32 * wq) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kpos = first_key + 16 * (r >> 3) + 8 * half + (r & 7);
            if (kpos > q_in_blk) s[r] = -INFINITY;
        }
    }
}

// Running softmax of a wavefront: a lane pair (lane, lane ^ 32) owns one query.
// Weights are w = 2^(x*c - mcb) with mcb = m_run*c, m_run a reference logit (raw).  The reference
// need not be the running maximum: a common factor 2^-mcb cancels between numerator and
// denominator, and bf16 weights and fp32 sums keep their relative precision at any magnitude.
// All it has to do is keep the numbers inside the fp32 range, so it is only moved when the
// running denominator (which bounds every weight so far) passes kRescaleAt.
constexpr float kRescaleAt = 1.099511627776e12f;      // 2^40
template <int DT>
struct RunningSoftmax {
    f32x16 oacc[DT];             // O^T tiles, unnormalised
    float m_run, mcb;
    float l_run;                 // this lane's half of the running denominator (sum of bf16 weights)
    float c;                     // softmax scale * log2 e

    __device__ __forceinline__ explicit RunningSoftmax(float scale)
        : m_run(-INFINITY), mcb(0.f), l_run(0.f), c(scale * 1.44269504088896340736f) {
#pragma unroll
        for (int dc = 0; dc < DT; ++dc)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dc][r] = 0.f;
    }
    __device__ __forceinline__ void weights(const f32x16& s, bf16x8& p0, bf16x8& p1, float& lsum) const {
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        f32x8 e0, e1;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            e0[x] = __builtin_amdgcn_exp2f(fmaf(s[x], c, -mcb));
            e1[x] = __builtin_amdgcn_exp2f(fmaf(s[8 + x], c, -mcb));
        }
        p0 = __builtin_convertvector(e0, bf16x8);
        p1 = __builtin_convertvector(e1, bf16x8);
        lsum = 0.f;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            lsum = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{p0[2 * x], p0[2 * x + 1]}, ones, lsum, false);
            lsum = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{p1[2 * x], p1[2 * x + 1]}, ones, lsum, false);
        }
    }
    // Slow path: move the reference so that the chunk `s` has weights <= 1 and the denominator so
    // far is about 1 or less, rescale what has been accumulated and recompute the chunk's weights.
    // Always taken on the first chunk, almost never after; wave-uniform.
    __device__ __forceinline__ void raise_reference(const f32x16& s, bf16x8& p0, bf16x8& p1, float& lsum) {
        float mx = fmaxf(s[0], s[1]);
#pragma unroll
        for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s[r]);
        mx = fmaxf(mx, other_half(mx));
        const float lq = l_run + other_half(l_run);          // this query's denominator so far
        const float lift = lq > 1.0f ? __log2f(lq) / c : 0.0f;
        const float m_new = fmaxf(m_run + lift, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        m_run = m_new;
        mcb = m_new * c;
        l_run *= alpha;
#pragma unroll
        for (int dc = 0; dc < DT; ++dc)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dc][r] *= alpha;
        weights(s, p0, p1, lsum);
    }
    // End of a step whose weights pn (of the logits s_cur) brought the denominator to l_new.  The
    // weights are positive, so the running denominator bounds every one of them: while it stays
    // below kRescaleAt no weight, and no sum of weights times values, can leave the fp32 range.
    // Beyond it (or inf / NaN) the chunk has outgrown the reference by far.
    __device__ __forceinline__ void settle(float l_new, const f32x16& s_cur, bf16x8& pn0, bf16x8& pn1) {
        if (__any(!(l_new < kRescaleAt))) {
            float lsum;
            raise_reference(s_cur, pn0, pn1, lsum);
            l_new = l_run + lsum;
        }
        l_run = l_new;
    }
    // normalise and store the wavefront's 32 query rows (orow: this lane's row), LSE by the lower half;
    // valid = false: a token past the end of a partial last block, nothing is stored
    template <int D>
    __device__ __forceinline__ void store(bool valid, uint16_t* orow, float* lse_or_null, int half) const {
        const float l_tot = l_run + other_half(l_run);
        const float inv = 1.0f / l_tot;
        if (!valid) return;
#pragma unroll
        for (int dc = 0; dc < DT; ++dc)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                f32x4 o4;
#pragma unroll
                for (int x = 0; x < 4; ++x) o4[x] = oacc[dc][4 * rq + x] * inv;
                *reinterpret_cast<bf16x4*>(orow + 32 * dc + 8 * rq + 4 * half) = __builtin_convertvector(o4, bf16x4);
            }
        if (lse_or_null != nullptr && half == 0) *lse_or_null = mcb * (0.69314718055994530942f) + __logf(l_tot);
    }
};

// Instruction group g of a pipeline step (a step = one 32-key chunk = NG = D / 8 groups, one MFMA each).
// The MFMA: even groups add slice g / 2 of the logits of chunk n + 2 (A operand `a` = 32 K rows x 16
// dims), odd groups add V^T (32 d rows x 16 keys) times the weights pc of chunk n into O^T.
template <int g, int D>
__device__ __forceinline__ void group_mfma(const bf16x8& a, const bf16x8 (&qf)[D / 16], f32x16& s_nxt,
                                           f32x16 (&oacc)[D / 32], const bf16x8& pc0, const bf16x8& pc1) {
    constexpr int NG = D / 8, DT = D / 32;
    if constexpr (g % 2 == 0) {
        if constexpr (g == 0) {
            f32x16 zero;
#pragma unroll
            for (int r = 0; r < 16; ++r) zero[r] = 0.f;
            s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[g / 2], zero, 0, 0, 0);
        } else {
            s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[g / 2], s_nxt, 0, 0, 0);
        }
    } else {
        constexpr int dc = (g / 2) % DT;
        if constexpr (g < NG / 2) oacc[dc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pc0, oacc[dc], 0, 0, 0);
        else oacc[dc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pc1, oacc[dc], 0, 0, 0);
    }
}
// The group's share of the softmax arithmetic of chunk n + 1: its 16 logits s_cur form two halves of
// 8 (keys 0-15 / 16-31), each turned into weights pn over NG / 2 consecutive groups: scaled
// differences (8 fma), powers of two (8 exp2), conversion to bf16, denominator.
template <int g, int D>
__device__ __forceinline__ void group_weights(const f32x16& s_cur, float c, float mcb, f32x8& e, bf16x8& pn0, bf16x8& pn1,
                                              float& l_new) {
    constexpr int NG = D / 8;
    constexpr int HG = NG / 2;               // groups per half of the chunk's 16 logits
    constexpr int hb = (g / HG) * 8;         // which half
    constexpr int gg = g % HG;
    constexpr bool first_half = g < HG;
    auto scale_sub = [&](int x0, int n) {
#pragma unroll
        for (int x = x0; x < x0 + n; ++x) e[x] = fmaf(s_cur[hb + x], c, -mcb);
    };
    auto exps = [&](int x0, int n) {
#pragma unroll
        for (int x = x0; x < x0 + n; ++x) e[x] = __builtin_amdgcn_exp2f(e[x]);
    };
    auto convert = [&]() {
        if constexpr (first_half) pn0 = __builtin_convertvector(e, bf16x8);
        else pn1 = __builtin_convertvector(e, bf16x8);
    };
    auto sum_and_test = [&]() {
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        const bf16x8 pw = first_half ? pn0 : pn1;
#pragma unroll
        for (int x = 0; x < 4; ++x)
            l_new = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{pw[2 * x], pw[2 * x + 1]}, ones, l_new, false);
        if constexpr (g == NG - 1) asm volatile("" : "+v"(l_new));   // keep the sums inside their groups
    };
    if constexpr (HG == 8) {                 // head_dim 128: 8 groups per half
        if constexpr (gg < 2) scale_sub(4 * gg, 4);
        else if constexpr (gg < 6) exps(2 * (gg - 2), 2);
        else if constexpr (gg == 6) convert();
        else sum_and_test();
    } else {                                 // head_dim 64: 4 groups per half
        static_assert(HG == 4 || HG == 8, "head_dim 64 or 128");
        if constexpr (gg == 0) scale_sub(0, 8);
        else if constexpr (gg == 1) exps(0, 4);
        else if constexpr (gg == 2) exps(4, 4);
        else { convert(); sum_and_test(); }
    }
}

// NH: query heads of one KV group served by one workgroup (BS / 32 wavefronts each).  NH = 2 is for
// lists shared by the group (one list per KV head): the heads then walk the same key blocks, and
// two of them take every K and V^T sub-tile from one staged copy, which halves the tile traffic
// (L2 -> LDS) per FLOP; with blocks of 64 tokens it also puts two wavefronts on every SIMD.
template <int BS, int D, int NH>
__global__ __launch_bounds__(BS * 2 * NH, NH == 1 ? BS / 64 : (BS == 64 ? 2 : 1)) void attn_kernel(
    const uint16_t* __restrict__ q, Strides qs, const uint16_t* __restrict__ k, Strides ks,
    const uint16_t* __restrict__ vt, const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt,
    uint16_t* __restrict__ out, Strides os, float* __restrict__ lse, int Hq, int G, int NB, int T, int S,
    float scale, RowDeal deal, int shared, int NBk, int Skv_max, const int32_t* __restrict__ seq_lens, int64_t vt_bph) {
    constexpr int NWH = BS / 32;        // wavefronts per head
    constexpr int NW = NWH * NH;        // wavefronts
    constexpr int NSUB = BS / KT;       // sub-tiles per key block
    constexpr int DS = D / 16;          // 16-dim slices of a key row = MFMAs of one logits tile
    constexpr int DT = D / 32;          // 32-row tiles of O^T = MFMAs per 16 keys of the second product
    constexpr int NG = 2 * DS;          // MFMAs (= instruction groups) of a pipeline step
    constexpr int TILE = KT * D;        // elements of one K (or V^T) sub-tile: 16 KB / 8 KB
    constexpr int CPR = D / 8;          // 16-byte chunks of a K row
    constexpr int RPI = 64 / CPR;       // K rows filled by one 1-KB load instruction
    constexpr int LPW = TILE / 512 / NW;  // 1-KB load instructions per wave per operand per sub-tile
    constexpr int TILE_B = TILE * 2;    // bytes of a sub-tile
    constexpr int CHUNK_B = 32 * D * 2; // bytes of a 32-key chunk of a K sub-tile
    constexpr int DTILE_B = 32 * KT * 2;  // bytes of 32 d rows of a V^T sub-tile
    __shared__ __attribute__((aligned(1024))) uint16_t smemK[2][TILE];   // K sub-tile t in buffer t % 2
    __shared__ __attribute__((aligned(1024))) uint16_t smemV[2][TILE];   // V^T likewise

    RowOfWorkgroup row;
    if (!row_of_workgroup<BS, NH>(deal, Hq, G, NB, S, Skv_max, seq_lens, row)) return;
    const int i = row.i, b = row.b, kvh = row.kvh, Sb = row.Sb, Skv = row.Skv;
    const int Hkv = Hq / G;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int wq = wave % NWH;                            // which 32 queries of the block
    const int h = kvh * G + row.first_head + wave / NWH;  // this wavefront's query head

    const uint16_t* qb = q + b * qs.b + h * qs.h + (int64_t)i * BS * qs.t;
    const uint16_t* kb = k + b * ks.b + kvh * ks.h;
    const uint16_t* vtb = vt + ((int64_t)(b * Hkv + kvh) * vt_bph) * D * BS;   // K, V, V^T may carry a prefix
    // block lists are per query head, or per KV head when the group shares its selection
    const int64_t row_id = shared ? ((int64_t)b * Hkv + kvh) * NB + i : ((int64_t)b * Hq + h) * NB + i;
    const BlockList list(idx, cnt, row_id, T, Skv, BS, NBk);
    const int n_sel = list.n_sel;
    const int n_st = n_sel * NSUB;

    // Direct global->LDS loads: instruction `inst` of a sub-tile fills 1 KB of LDS in lane order
    // (4 K rows of 256 B or 8 of 128 B, 8 V^T rows of 128 B); the lane picks the global 16-byte chunk whose
    // swizzled position it is writing.  Per-lane byte offsets are fixed for the whole kernel; the
    // tile base is wave-uniform, so each load is base (SGPRs) + 32-bit lane offset.
    uint32_t k_offb[LPW], v_offb[LPW];
#pragma unroll
    for (int x = 0; x < LPW; ++x) {
        const int inst = wave * LPW + x;
        const int krow = RPI * inst + lane / CPR;
        const int vrow = 8 * inst + (lane >> 3);
        k_offb[x] = 2u * ((uint32_t)krow * (uint32_t)ks.t + (uint32_t)(((lane % CPR) ^ swz_k<D>(krow)) << 3));
        v_offb[x] = 2u * (uint32_t)(vrow * BS + (((lane & 7) ^ swz_v(vrow)) << 3));
    }
    // K and V^T sub-tiles are staged separately: K runs one sub-tile ahead of V^T because the
    // logits are produced two 32-key chunks before the second product consumes them.
    const uint32_t k_dst = lds_address(&smemK[0][0]) + wave * LPW * 1024;   // this wave's 1-KB slots
    const uint32_t v_dst = lds_address(&smemV[0][0]) + wave * LPW * 1024;
    auto issue_k = [&](auto buf_tag, int st, int blk) {
        constexpr int BUF = decltype(buf_tag)::value;
        const int sub = st % NSUB;
        if ((blk + 1) * BS <= Skv) {
            const char* kt = reinterpret_cast<const char*>(kb + ((int64_t)blk * BS + sub * KT) * ks.t);
            static_for<LPW>([&](auto x_tag) {
                constexpr int X = decltype(x_tag)::value;
                lds_dma16<BUF * TILE_B + X * 1024>(k_dst, k_offb[X], kt);
            });
        } else {
            // partial last block (only ever the diagonal block of the last query block): key rows past
            // the end re-read the last token; they are masked for every query that exists
            const char* kt = reinterpret_cast<const char*>(kb + (int64_t)blk * BS * ks.t);
            const int last_row = Skv - 1 - blk * BS;
            static_for<LPW>([&](auto x_tag) {
                constexpr int X = decltype(x_tag)::value;
                const int krow = RPI * (wave * LPW + X) + lane / CPR;
                int row = sub * KT + krow;
                if (row > last_row) row = last_row;
                const uint32_t off = 2u * ((uint32_t)row * (uint32_t)ks.t + (uint32_t)(((lane % CPR) ^ swz_k<D>(krow)) << 3));
                lds_dma16<BUF * TILE_B + X * 1024>(k_dst, off, kt);
            });
        }
    };
    auto issue_v = [&](auto buf_tag, int st, int blk) {
        constexpr int BUF = decltype(buf_tag)::value;
        const char* vtt = reinterpret_cast<const char*>(vtb + (int64_t)blk * D * BS + (st % NSUB) * KT);
        static_for<LPW>([&](auto x_tag) {
            constexpr int X = decltype(x_tag)::value;
            lds_dma16<BUF * TILE_B + X * 1024>(v_dst, v_offb[X], vtt);
        });
    };
    auto blk_of = [&](int st) { return list.at_or_last(st / NSUB); };   // key block of sub-tile st

    issue_k(IC<0>{}, 0, list.at(0));
    issue_v(IC<0>{}, 0, list.at(0));
    if (n_st > 1) issue_k(IC<1>{}, 1, blk_of(1));

    bf16x8 qf[DS];
    load_q_fragments<BS, D>(qb, qs.t, i, Sb, wq, l32, half, qf);
    // Per-lane LDS byte offsets.  K (A operand of S^T = K Q^T): the lane's key row of chunk 0 and
    // its 8-dim slice s; chunk 1 and the buffer add constants.  The row assignment swaps bits 2
    // and 3, see the file header.  V^T (A operand of O^T += V^T P^T): d row l32 (+32 per d tile, a
    // constant) and the 8-key slice x of the sub-tile.
    int kofs[DS], vofs[4];
    {
        const int row = swap_bits23(l32);
#pragma unroll
        for (int s = 0; s < DS; ++s) kofs[s] = 2 * (row * D + (((2 * s + half) ^ swz_k<D>(row)) << 3));
#pragma unroll
        for (int x = 0; x < 4; ++x) vofs[x] = 2 * (l32 * KT + (((2 * x + half) ^ swz_v(l32)) << 3));
    }
    const char* const ldsK = reinterpret_cast<const char*>(&smemK[0][0]);
    const char* const ldsV = reinterpret_cast<const char*>(&smemV[0][0]);
    auto lds16 = [](const char* p) { return *reinterpret_cast<const bf16x8*>(p); };

    RunningSoftmax<DT> sm(scale);
    const int q_in_blk = 32 * wq + l32;
    auto mask_diag = [&](f32x16& s, int sub, int kc) { mask_diagonal_chunk(s, KT * sub + 32 * kc, wq, half, q_in_blk); };

    // The pipeline step n (chunk n = 32 keys) runs three independent chains side by side:
    //   MFMA   s_nxt = logits of chunk n+2 (same chunk position KC of the next sub-tile, K buffer KB)
    //   VALU   pn    = weights of chunk n+1 from its logits s_cur (produced by step n-1)
    //   MFMA   O^T  += V^T(chunk n, V buffer VB) pc^T, pc = weights of chunk n (made by step n-1)
    // f[0..3]: rotating MFMA A operands, read from LDS three MFMAs ahead of their use.  The NG
    // operands of a step in MFMA order are K slice 0, V^T (keys 0-15, d tile 0), K slice 1,
    // V^T (0-15, 1), ..., K slice DS-1, V^T (16-31, DT-1) (head_dim 128: 16 of them, 64: 8).  On
    // entry f[0..2] hold operands 0..2; a KC = 0 step leaves the first three operands of the KC = 1
    // step behind.
    auto step = [&](auto kb_tag, auto vb_tag, auto kc_tag, const f32x16& s_cur, f32x16& s_nxt, const bf16x8& pc0,
                    const bf16x8& pc1, bf16x8& pn0, bf16x8& pn1, bf16x8 (&f)[4]) {
        constexpr int KB = decltype(kb_tag)::value, VB = decltype(vb_tag)::value, KC = decltype(kc_tag)::value;
        const char* const vbase = ldsV + VB * TILE_B;
        auto operand = [&](auto j_tag) {            // operand j of this step (j < NG) or of the next one
            constexpr int J = decltype(j_tag)::value;
            constexpr int j = J % NG;
            constexpr int kc = KC + J / NG;         // only used with J >= NG when KC == 0
            const char* const kb2 = ldsK + KB * TILE_B + kc * CHUNK_B;
            if constexpr (j % 2 == 0) return lds16(kb2 + kofs[j / 2]);
            else return lds16(vbase + vofs[2 * kc + (j / 2) / DT] + ((j / 2) % DT) * DTILE_B);
        };
        f32x8 e;
        float l_new = sm.l_run;
        // Group g holds MFMA g of the step, the LDS read of operand g + 3 and a share of the softmax
        // arithmetic of the chunk's logits.
        auto group = [&](auto g_tag) {
            constexpr int g = decltype(g_tag)::value;
            group_mfma<g, D>(f[g % 4], qf, s_nxt, sm.oacc, pc0, pc1);
            if constexpr (g + 3 < NG || KC == 0) f[(g + 3) % 4] = operand(IC<g + 3>{});
            group_weights<g, D>(s_cur, sm.c, sm.mcb, e, pn0, pn1, l_new);
            SPA_FENCE();
        };
        SPA_FENCE();
        static_for<NG>([&](auto g_tag) { group(g_tag); });
        sm.settle(l_new, s_cur, pn0, pn1);
    };

    // ---- prologue: logits of the two chunks of sub-tile 0, weights of chunk 0 -----------
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)
    __syncthreads();
    f32x16 sA, sB;                                 // logits of even / odd chunks
#pragma unroll
    for (int r = 0; r < 16; ++r) { sA[r] = 0.f; sB[r] = 0.f; }
#pragma unroll
    for (int sidx = 0; sidx < DS; ++sidx) {
        sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds16(ldsK + kofs[sidx]), qf[sidx], sA, 0, 0, 0);
        sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds16(ldsK + CHUNK_B + kofs[sidx]), qf[sidx], sB, 0, 0, 0);
    }
    bf16x8 pA0, pA1, pB0, pB1;                     // weights of even / odd chunks
    {
        if (n_st <= NSUB) mask_diag(sA, 0, 0);     // the only block is the diagonal one
        float lsum;
        sm.raise_reference(sA, pA0, pA1, lsum);
        sm.l_run = lsum;
    }
    int blk1 = blk_of(1), blk2 = blk_of(2);        // key blocks of sub-tiles t+1 and t+2

    // One 64-key sub-tile t = steps 2t and 2t+1.  Reads K(t+1) (look-ahead logits) and V^T(t).
    auto sub_tile = [&](auto par_tag, auto plain_tag, int t) {
        constexpr int PAR = decltype(par_tag)::value;      // t % 2
        constexpr bool PLAIN = decltype(plain_tag)::value != 0;   // far from the end: all loads exist, no masks
        using KB = IC<1 - PAR>;
        using VB = IC<PAR>;
        // K(t+1) and V(t) have been requested; make them visible and retire the previous
        // sub-tile's readers of the buffers refilled below.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        bf16x8 f[4];
        f[0] = lds16(ldsK + KB::value * TILE_B + kofs[0]);
        f[1] = lds16(ldsV + VB::value * TILE_B + vofs[0]);
        f[2] = lds16(ldsK + KB::value * TILE_B + kofs[1]);
        if (PLAIN || t + 2 < n_st) issue_k(IC<PAR>{}, t + 2, blk2);
        if (PLAIN || t + 1 < n_st) issue_v(IC<1 - PAR>{}, t + 1, blk1);
        blk1 = blk2;
        blk2 = blk_of(t + 3);
        // logits about to be turned into weights: chunk 1 of this sub-tile, then chunk 0 of the next
        if constexpr (!PLAIN)
            if (t >= n_st - NSUB) mask_diag(sB, t % NSUB, 1);      // the diagonal block is the last of the list
        step(KB{}, VB{}, IC<0>{}, sB, sA, pA0, pA1, pB0, pB1, f);
        if constexpr (PLAIN) {
        } else if (t + 1 >= n_st) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sA[r] = -INFINITY;        // past the end: look-ahead of a stale buffer
        } else if (t + 1 >= n_st - NSUB) {
            mask_diag(sA, (t + 1) % NSUB, 0);
        }
        step(KB{}, VB{}, IC<1>{}, sA, sB, pB0, pB1, pA0, pA1, f);
    };
    // sub-tiles whose two softmaxed chunks lie before the diagonal block and whose loads all exist
    // run without the mask and end-of-list tests; the last NSUB + 2 (rounded to even) keep them
    int t = 0;
    const int t_plain = (n_st - NSUB - 2) & ~1;
    for (; t < t_plain; t += 2) {
        sub_tile(IC<0>{}, IC<1>{}, t);
        sub_tile(IC<1>{}, IC<1>{}, t + 1);
    }
    for (;;) {
        sub_tile(IC<0>{}, IC<0>{}, t);
        if (++t == n_st) break;
        sub_tile(IC<1>{}, IC<0>{}, t);
        if (++t == n_st) break;
    }

    // ---- epilogue ----------------------------------------------------------------
    sm.template store<D>(i * BS + q_in_blk < Sb, out + b * os.b + h * os.h + ((int64_t)i * BS + q_in_blk) * os.t,
                         lse != nullptr ? lse + ((int64_t)b * Hq + h) * S + (int64_t)i * BS + q_in_blk : nullptr, half);
}

// ---------------------------------------------------------------------------
// Variant for blocks of 64 tokens.  A 64-key tile serves only 64 queries there, so a workgroup is two
// wavefronts and the 64 KB of tile buffers of the kernel above leave one wavefront per SIMD, with
// nothing to fill the time its tiles take to arrive.  This one stages K and V^T in 32-key chunks, two
// stages per operand (32 KB with head_dim 128): four workgroups per CU, two wavefronts per SIMD, one
// barrier per step (= chunk); the loads of a chunk are requested one step before it is read.  Same
// arithmetic in the same order: the two kernels give the same bits.
__device__ __forceinline__ int swz_c(int row) { return (row >> 2) & 3; }     // V^T stage rows are 64 B

template <int BS, int D, int NH>
__global__ __launch_bounds__(BS * 2 * NH, 2) void attn_chunked_kernel(
    const uint16_t* __restrict__ q, Strides qs, const uint16_t* __restrict__ k, Strides ks,
    const uint16_t* __restrict__ vt, const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt,
    uint16_t* __restrict__ out, Strides os, float* __restrict__ lse, int Hq, int G, int NB, int T, int S,
    float scale, RowDeal deal, int shared, int NBk, int Skv_max, const int32_t* __restrict__ seq_lens, int64_t vt_bph) {
    constexpr int NWH = BS / 32;        // wavefronts per head
    constexpr int NW = NWH * NH;        // wavefronts
    constexpr int CPB = BS / 32;        // 32-key chunks per key block
    constexpr int DS = D / 16;          // MFMAs of one logits tile
    constexpr int DT = D / 32;          // 32-row tiles of O^T
    constexpr int NG = 2 * DS;          // MFMAs (= instruction groups) of a step
    constexpr int STG = 32 * D;         // elements of a stage: one 32-key chunk of K or of V^T (8 KB / 4 KB)
    constexpr int STG_B = STG * 2;
    constexpr int CPR = D / 8;          // 16-byte pieces of a K row
    constexpr int RPI = 64 / CPR;       // K rows filled by one 1-KB load instruction
    constexpr int LPW = STG / 512 / NW; // 1-KB load instructions per wave per operand per chunk
    constexpr int DTILE_B = 32 * 32 * 2;  // bytes of 32 d rows of a V^T stage
    static_assert(LPW >= 1 && CPB >= 2, "blocks of 64 tokens");
    __shared__ __attribute__((aligned(1024))) uint16_t smemK[2][STG];   // K chunk n in stage n % 2
    __shared__ __attribute__((aligned(1024))) uint16_t smemV[2][STG];   // V^T chunk n likewise

    RowOfWorkgroup row;
    if (!row_of_workgroup<BS, NH>(deal, Hq, G, NB, S, Skv_max, seq_lens, row)) return;
    const int i = row.i, b = row.b, kvh = row.kvh, Sb = row.Sb, Skv = row.Skv;
    const int Hkv = Hq / G;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int wq = wave % NWH;
    const int h = kvh * G + row.first_head + wave / NWH;

    const uint16_t* qb = q + b * qs.b + h * qs.h + (int64_t)i * BS * qs.t;
    const uint16_t* kb = k + b * ks.b + kvh * ks.h;
    const uint16_t* vtb = vt + ((int64_t)(b * Hkv + kvh) * vt_bph) * D * BS;
    const int64_t row_id = shared ? ((int64_t)b * Hkv + kvh) * NB + i : ((int64_t)b * Hq + h) * NB + i;
    const BlockList list(idx, cnt, row_id, T, Skv, BS, NBk);
    const int n_ch = list.n_sel * CPB;                    // chunks (= steps) of the row
    auto blk_of = [&](int n) { return list.at_or_last(n / CPB); };      // key block of chunk n

    // direct global->LDS loads, 1 KB per instruction in lane order: 4 K rows of 256 B (8 of 128 B), or
    // 16 rows of 64 B of a V^T chunk; the XOR swizzle is applied on the global side
    uint32_t k_offb[LPW], v_offb[LPW];
#pragma unroll
    for (int x = 0; x < LPW; ++x) {
        const int inst = wave * LPW + x;
        const int krow = RPI * inst + lane / CPR;
        const int vrow = 16 * inst + (lane >> 2);
        k_offb[x] = 2u * ((uint32_t)krow * (uint32_t)ks.t + (uint32_t)(((lane % CPR) ^ swz_k<D>(krow)) << 3));
        v_offb[x] = 2u * (uint32_t)(vrow * BS + (((lane & 3) ^ swz_c(vrow)) << 3));
    }
    const uint32_t k_dst = lds_address(&smemK[0][0]) + wave * LPW * 1024;
    const uint32_t v_dst = lds_address(&smemV[0][0]) + wave * LPW * 1024;
    auto issue_k = [&](auto stg_tag, int n, int blk) {
        constexpr int ST = decltype(stg_tag)::value;
        const int cib = n % CPB;                          // chunk in block
        if ((blk + 1) * BS <= Skv) {
            const char* kt = reinterpret_cast<const char*>(kb + ((int64_t)blk * BS + cib * 32) * ks.t);
            static_for<LPW>([&](auto x_tag) {
                constexpr int X = decltype(x_tag)::value;
                lds_dma16<ST * STG_B + X * 1024>(k_dst, k_offb[X], kt);
            });
        } else {
            // partial last block: key rows past the end re-read the last token (masked for every query that exists)
            const char* kt = reinterpret_cast<const char*>(kb + (int64_t)blk * BS * ks.t);
            const int last_row = Skv - 1 - blk * BS;
            static_for<LPW>([&](auto x_tag) {
                constexpr int X = decltype(x_tag)::value;
                const int krow = RPI * (wave * LPW + X) + lane / CPR;
                int row = cib * 32 + krow;
                if (row > last_row) row = last_row;
                const uint32_t off = 2u * ((uint32_t)row * (uint32_t)ks.t + (uint32_t)(((lane % CPR) ^ swz_k<D>(krow)) << 3));
                lds_dma16<ST * STG_B + X * 1024>(k_dst, off, kt);
            });
        }
    };
    auto issue_v = [&](auto stg_tag, int n, int blk) {
        constexpr int ST = decltype(stg_tag)::value;
        const char* vtt = reinterpret_cast<const char*>(vtb + (int64_t)blk * D * BS + (n % CPB) * 32);
        static_for<LPW>([&](auto x_tag) {
            constexpr int X = decltype(x_tag)::value;
            lds_dma16<ST * STG_B + X * 1024>(v_dst, v_offb[X], vtt);
        });
    };

    issue_k(IC<0>{}, 0, blk_of(0));
    issue_k(IC<1>{}, 1, blk_of(1));
    issue_v(IC<0>{}, 0, blk_of(0));

    bf16x8 qf[DS];
    load_q_fragments<BS, D>(qb, qs.t, i, Sb, wq, l32, half, qf);
    // per-lane LDS byte offsets of the A operands inside a stage: K row (bits 2 and 3 swapped) and 8-dim
    // slice s; V^T d row l32 (+32 per d tile) and 8-key slice x
    int kofs[DS], vofs[2];
    {
        const int row = swap_bits23(l32);
#pragma unroll
        for (int s = 0; s < DS; ++s) kofs[s] = 2 * (row * D + (((2 * s + half) ^ swz_k<D>(row)) << 3));
#pragma unroll
        for (int x = 0; x < 2; ++x) vofs[x] = 2 * (l32 * 32 + (((2 * x + half) ^ swz_c(l32)) << 3));
    }
    const char* const ldsK = reinterpret_cast<const char*>(&smemK[0][0]);
    const char* const ldsV = reinterpret_cast<const char*>(&smemV[0][0]);
    auto lds16 = [](const char* p) { return *reinterpret_cast<const bf16x8*>(p); };

    RunningSoftmax<DT> sm(scale);
    const int q_in_blk = 32 * wq + l32;
    auto mask_diag = [&](f32x16& s, int cib) { mask_diagonal_chunk(s, 32 * cib, wq, half, q_in_blk); };

    int blk_v = blk_of(1), blk_k = blk_of(3);             // key blocks of the next V^T and K chunk to request

    // Step n, P = n % 2: logits of chunk n + 2 (K stage P), weights of chunk n + 1, O^T += V^T(chunk n,
    // stage P) pc^T; the instruction groups of the kernel above.  K chunk n + 2 and V^T chunk n were
    // requested by step n - 1; after the barrier the stages read by step n - 1 take K chunk n + 3 and
    // V^T chunk n + 1.
    auto step = [&](auto p_tag, auto plain_tag, int n, const f32x16& s_cur, f32x16& s_nxt, const bf16x8& pc0,
                    const bf16x8& pc1, bf16x8& pn0, bf16x8& pn1) {
        constexpr int P = decltype(p_tag)::value;
        constexpr bool PLAIN = decltype(plain_tag)::value != 0;
        auto operand = [&](auto j_tag) {
            constexpr int j = decltype(j_tag)::value;
            if constexpr (j % 2 == 0) return lds16(ldsK + P * STG_B + kofs[j / 2]);
            else return lds16(ldsV + P * STG_B + vofs[(j / 2) / DT] + ((j / 2) % DT) * DTILE_B);
        };
        __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wave's loads have landed
        __syncthreads();
        bf16x8 f[4];
        f[0] = operand(IC<0>{});
        f[1] = operand(IC<1>{});
        f[2] = operand(IC<2>{});
        if (PLAIN || n + 1 < n_ch) issue_v(IC<1 - P>{}, n + 1, blk_v);
        if (PLAIN || n + 3 < n_ch) issue_k(IC<1 - P>{}, n + 3, blk_k);
        blk_v = blk_of(n + 2);
        blk_k = blk_of(n + 4);
        f32x8 e;
        float l_new = sm.l_run;
        auto group = [&](auto g_tag) {
            constexpr int g = decltype(g_tag)::value;
            group_mfma<g, D>(f[g % 4], qf, s_nxt, sm.oacc, pc0, pc1);
            if constexpr (g + 3 < NG) f[(g + 3) % 4] = operand(IC<g + 3>{});
            group_weights<g, D>(s_cur, sm.c, sm.mcb, e, pn0, pn1, l_new);
            SPA_FENCE();
        };
        SPA_FENCE();
        static_for<NG>([&](auto g_tag) { group(g_tag); });
        sm.settle(l_new, s_cur, pn0, pn1);
        if constexpr (!PLAIN) {                      // the logits just produced: chunk n + 2
            if (n + 2 >= n_ch) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s_nxt[r] = -INFINITY;           // past the end: a stale stage
            } else if (n + 2 >= n_ch - CPB) {
                mask_diag(s_nxt, (n + 2) % CPB);                             // the diagonal block ends the list
            }
        }
    };

    // ---- prologue: logits of chunks 0 and 1, weights of chunk 0, then K chunk 2 -----------
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)
    __syncthreads();
    f32x16 sA, sB;                                 // logits of even / odd chunks
#pragma unroll
    for (int r = 0; r < 16; ++r) { sA[r] = 0.f; sB[r] = 0.f; }
#pragma unroll
    for (int sidx = 0; sidx < DS; ++sidx) {
        sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds16(ldsK + kofs[sidx]), qf[sidx], sA, 0, 0, 0);
        sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds16(ldsK + STG_B + kofs[sidx]), qf[sidx], sB, 0, 0, 0);
    }
    if (n_ch <= CPB) {                             // the only block is the diagonal one
        mask_diag(sA, 0);
        mask_diag(sB, 1);
    }
    bf16x8 pA0, pA1, pB0, pB1;                     // weights of even / odd chunks
    {
        float lsum;
        sm.raise_reference(sA, pA0, pA1, lsum);
        sm.l_run = lsum;
    }
    __syncthreads();                               // K chunks 0 and 1 have been read by every wave
    if (n_ch > 2) issue_k(IC<0>{}, 2, blk_of(2));

    // steps far from the end of the list run without the mask and end-of-list tests
    int n = 0;
    const int n_plain = n_ch > CPB + 2 ? (n_ch - CPB - 2) & ~1 : 0;      // n + 3 < n_ch and n + 2 < n_ch - CPB
    for (; n < n_plain; n += 2) {
        step(IC<0>{}, IC<1>{}, n, sB, sA, pA0, pA1, pB0, pB1);
        step(IC<1>{}, IC<1>{}, n + 1, sA, sB, pB0, pB1, pA0, pA1);
    }
    for (;;) {
        step(IC<0>{}, IC<0>{}, n, sB, sA, pA0, pA1, pB0, pB1);
        if (++n == n_ch) break;
        step(IC<1>{}, IC<0>{}, n, sA, sB, pB0, pB1, pA0, pA1);
        if (++n == n_ch) break;
    }

    // ---- epilogue ----------------------------------------------------------------
    sm.template store<D>(i * BS + q_in_blk < Sb, out + b * os.b + h * os.h + ((int64_t)i * BS + q_in_blk) * os.t,
                         lse != nullptr ? lse + ((int64_t)b * Hq + h) * S + (int64_t)i * BS + q_in_blk : nullptr, half);
}

// One wavefront per list row: counts the rows that break the rules the attention kernel relies on
// (1 <= cnt <= T, entries strictly ascending, first >= 0, last == the row's diagonal block).
__global__ __launch_bounds__(256) void check_lists_kernel(const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ cnt, int Hl, int NB, int T,
                                                          int off, int Bs, int S, const int32_t* __restrict__ seq_lens,
                                                          int64_t n_rows, int32_t* __restrict__ n_bad) {
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int lane = threadIdx.x & 63;
    const int i = (int)(row % NB);
    const int b = (int)(row / ((int64_t)NB * Hl));
    const int Sb = entry_len(seq_lens, b, S);
    if ((int64_t)i * Bs >= Sb) return;                     // past the entry's end: never read
    const int c = cnt[row];
    const int32_t* e = idx + row * T;
    bool bad = c < 1 || c > T;
    if (!bad) {
        for (int j = lane; j < c; j += 64) {
            const int v = e[j];
            if (j == 0 ? v < 0 : v <= e[j - 1]) bad = true;
            if (j == c - 1 && v != off + i) bad = true;
        }
    }
    if (__any(bad) && lane == 0) atomicAdd(n_bad, 1);
}

__global__ void zero_i32_kernel(int32_t* p) { *p = 0; }

template <int BS, int D, int NH>
hipError_t launch_nh(const Dims& d, const void* q, Strides qs, const void* k, Strides ks,
                     const int32_t* idx, const int32_t* cnt, void* out, Strides os, float* lse, const void* vt, int64_t vt_bph,
                     hipStream_t st) {
    const RowDeal deal = deal_rows(d, NH);
    const int64_t nwg = 8ll * deal.seq_len * d.B * d.Hkv;
    if (nwg > 0x7fffffffll) return hipErrorInvalidValue;
    // blocks of 64 tokens, one head per workgroup: the chunked kernel (two wavefronts per SIMD instead of one);
    // with two heads per workgroup the sub-tile kernel already has them and is the faster one
    if constexpr (BS == 64 && NH == 1)
        hipLaunchKernelGGL((attn_chunked_kernel<BS, D, NH>), dim3((unsigned)nwg), dim3(BS * 2 * NH), 0, st, (const uint16_t*)q,
                           qs, (const uint16_t*)k, ks, (const uint16_t*)vt, idx, cnt, (uint16_t*)out, os, lse, d.Hq, d.G,
                           d.NB, d.T, d.S, d.scale, deal, d.shared, d.NBk, d.Skv, d.seq_lens, vt_bph);
    else
        hipLaunchKernelGGL((attn_kernel<BS, D, NH>), dim3((unsigned)nwg), dim3(BS * 2 * NH), 0, st, (const uint16_t*)q, qs,
                           (const uint16_t*)k, ks, (const uint16_t*)vt, idx, cnt, (uint16_t*)out, os, lse, d.Hq,
                           d.G, d.NB, d.T, d.S, d.scale, deal, d.shared, d.NBk, d.Skv, d.seq_lens, vt_bph);
    return hipGetLastError();
}

template <int BS, int D>
hipError_t launch_tv(const Dims& d, const void* v, Strides vs, void* vt, int64_t vt_bph, int first, int n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL((transpose_v_kernel<BS, D>), dim3(n, d.B * d.Hkv), dim3(256), 0, st,
                       (const uint16_t*)v, vs, d.Hkv, vt_bph, d.Skv, (uint16_t*)vt, d.seq_lens, d.S, first);
    return hipGetLastError();
}

template <int BS, int D>
hipError_t launch(const Dims& d, const void* q, Strides qs, const void* k, Strides ks,
                  const int32_t* idx, const int32_t* cnt, void* out, Strides os, float* lse,
                  const void* vt, int64_t vt_bph, hipStream_t st) {
    // lists shared by the heads of a group: two heads per workgroup take every tile from one staged copy
    if (d.shared && d.G % 2 == 0) return launch_nh<BS, D, 2>(d, q, qs, k, ks, idx, cnt, out, os, lse, vt, vt_bph, st);
    return launch_nh<BS, D, 1>(d, q, qs, k, ks, idx, cnt, out, os, lse, vt, vt_bph, st);
}

}  // namespace

hipError_t launch_check_lists(const Dims& d, const int32_t* idx, const int32_t* cnt, int32_t* n_bad, hipStream_t st) {
    const int Hl = d.shared ? d.Hkv : d.Hq;
    const int64_t n_rows = (int64_t)d.B * Hl * d.NB;
    const int64_t nwg = (n_rows + 3) / 4;
    if (nwg > 0x7fffffffll) return hipErrorInvalidValue;
    hipLaunchKernelGGL(zero_i32_kernel, dim3(1), dim3(1), 0, st, n_bad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(check_lists_kernel, dim3((unsigned)nwg), dim3(256), 0, st, idx, cnt, Hl, d.NB, d.T, d.off, d.Bs,
                       d.S, d.seq_lens, n_rows, n_bad);
    return hipGetLastError();
}

hipError_t launch_transpose_v(const Dims& d, const void* v, Strides vs, void* vt, int64_t vt_bph, int first, int n,
                              hipStream_t st) {
    if (vt == nullptr || vt_bph < d.NBk || first < 0 || n < 0 || first + n > d.NBk) return hipErrorInvalidValue;
    if (d.D == 128 && d.Bs == 128) return launch_tv<128, 128>(d, v, vs, vt, vt_bph, first, n, st);
    if (d.D == 128 && d.Bs == 64) return launch_tv<64, 128>(d, v, vs, vt, vt_bph, first, n, st);
    if (d.D == 64 && d.Bs == 128) return launch_tv<128, 64>(d, v, vs, vt, vt_bph, first, n, st);
    if (d.D == 64 && d.Bs == 64) return launch_tv<64, 64>(d, v, vs, vt, vt_bph, first, n, st);
    return hipErrorInvalidValue;
}

hipError_t launch_attn_vt(const Dims& d, const void* q, Strides qs, const void* k, Strides ks, const void* vt,
                          int64_t vt_bph, const int32_t* idx, const int32_t* cnt, void* out, Strides os, float* lse,
                          hipStream_t st) {
    if (vt == nullptr || vt_bph < d.NBk) return hipErrorInvalidValue;
    if (d.D == 128 && d.Bs == 128) return launch<128, 128>(d, q, qs, k, ks, idx, cnt, out, os, lse, vt, vt_bph, st);
    if (d.D == 128 && d.Bs == 64) return launch<64, 128>(d, q, qs, k, ks, idx, cnt, out, os, lse, vt, vt_bph, st);
    if (d.D == 64 && d.Bs == 128) return launch<128, 64>(d, q, qs, k, ks, idx, cnt, out, os, lse, vt, vt_bph, st);
    if (d.D == 64 && d.Bs == 64) return launch<64, 64>(d, q, qs, k, ks, idx, cnt, out, os, lse, vt, vt_bph, st);
    return hipErrorInvalidValue;
}

hipError_t launch_attn(const Dims& d, const void* q, Strides qs, const void* k, Strides ks,
                       const void* v, Strides vs, const int32_t* idx, const int32_t* cnt, void* out,
                       Strides os, float* lse, void* vt, hipStream_t st) {
    hipError_t e = launch_transpose_v(d, v, vs, vt, d.NBk, 0, d.NBk, st);
    if (e != hipSuccess) return e;
    return launch_attn_vt(d, q, qs, k, ks, vt, d.NBk, idx, cnt, out, os, lse, st);
}

}  // namespace spa
