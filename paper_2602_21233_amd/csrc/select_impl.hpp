// Pooled scores, per-row top-k and merge with the static pattern
// (pattern computation, steps 2-4; Sec. 4.1.1 dynamic sparsity, uniform top-k
// budget of Sec. 4.1.2 Fig. "Stem" (a) or the per-query-block budget schedule of
// Token Position-Decay, Fig. "Stem" (b); optional value-magnitude term of the
// Output-Aware Metric, Fig. "Stem" (c); static patterns of Sec. 4.1.1: A-shape,
// Strided, Dilated, Tri-shape; optional per-head settings, a KV prefix, ragged
// batches and a cumulative-mass budget).
//
// score_topk_mfma_kernel: one workgroup (512 threads; two per CU) owns R consecutive
// query blocks of one query head.
//   Phase 0 - query pooling (step 1 for Q, in the kernel).  The workgroup streams its R
//   query blocks from Q and pools them itself, so that the Q stream of the select stage
//   (four fifths of its bytes) runs while other workgroups score and select; the split
//   pooled queries go straight to LDS.  (Group-shared lists read pooled queries from
//   memory instead.)
//   Phase 1 - scores on the matrix cores.  The fp32 pooled vectors are split
//   into a bf16 head and a bf16 tail (x = hi + lo, |x - hi - lo| <= 2^-18 |x|)
//   and each 32x32 tile of Qp Kp^T is accumulated in fp32 from three
//   v_mfma_f32_32x32x16_bf16 products (hi.hi + hi.lo + lo.hi); the dropped
//   lo.lo term is below 2^-17 of a product.  The wavefronts take the key-block
//   tiles round robin, reading Kp straight from L2 in operand layout.  The scores
//   of the R rows stay in LDS; the NB x NB matrix never exists in memory unless
//   the caller asks for it.
//   Phase 2 - exact selection.  A wavefront owns a row: lane l holds the keys of
//   blocks l, l+64, ... in registers as order-preserving uint32 and finds the k-th
//   largest in two steps: a bound from the lanes (the smallest of the 64 lanes' largest
//   keys is reached by at least 64 keys), below which keys drop out, then radix
//   selection among the rest, 8 bits per pass (the wavefront histograms the current
//   digit into 256 LDS counters, a prefix sum over the lanes finds the bin of the wanted
//   rank; a pass that takes its whole bin ends early).  Ties at the threshold are
//   resolved by block index with a running prefix count, and static U top-k is written
//   in ascending order from the keys in registers.  With a cumulative-mass budget a
//   weighted variant of the same search first finds how many blocks the row may take.
// topk_from_scores_kernel applies the same rule to caller-supplied scores (one
// wavefront per row, keys in LDS).
//
// This file is the implementation, included by three translation units so that the many kernel
// instantiations compile in parallel: select.hip (top-k on caller scores and the dispatcher) and
// select_d128.hip / select_d64.hip (score/top-k kernels for one head_dim each, SPA_SELECT_D set).
#pragma once
#include <mutex>
#include <type_traits>
#include <vector>

#include "common.hpp"

namespace spa {
namespace {

template <int N>
using IC_sel = std::integral_constant<int, N>;
// f(IC_sel<0>{}), ..., f(IC_sel<N-1>{})
template <int N, typename F>
__device__ __forceinline__ void static_for_sel(F&& f) {
    if constexpr (N > 0) {
        static_for_sel<N - 1>(f);
        f(IC_sel<N - 1>{});
    }
}

// Total order used for ranking: larger score first, -0 == +0, NaN below
// everything (including -inf).  The +1 keeps 0 free to mean "not a candidate".
__device__ __forceinline__ uint32_t rank_key(float s) {
    uint32_t u = __float_as_uint(s);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 1u;           // NaN
    if (u == 0x80000000u) u = 0u;                             // -0 -> +0
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return u + 1u;                                            // max finite/inf key is 0xff800000, no wrap
}

// number of set bits of `mask` that belong to lanes below the calling lane
__device__ __forceinline__ int lanes_below(uint64_t mask, int /*lane*/) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The static pattern.  Plain A-shape: sink blocks + local window.  EXT adds the strided columns
// ((i - j) % stride == 0, within a reach for the Dilated pattern) and the dense bottom strip of the Tri-shape (rows i >= NB - n_dense).
struct Pattern {
    int ns, nl, stride, n_dense, NB, reach;   // reach: strided blocks count while i - j < reach
    float inv_stride;
};
inline Pattern pattern_of(const Dims& d) {
    return Pattern{d.ns, d.nl, d.stride, d.n_dense, d.NBk, d.reach > 0 ? d.reach : d.NBk,
                   d.stride > 0 ? 1.0f / (float)d.stride : 0.f};
}
inline bool extended(const Dims& d) { return d.stride > 0 || d.n_dense > 0; }

// is key block j (0 <= j <= i) static for the query block at block position i (pt.NB = key blocks)?
template <bool EXT>
__device__ __forceinline__ bool static_block(const Pattern& pt, int i, int j) {
    bool s = j < pt.ns || j >= i - pt.nl + 1;
    if constexpr (EXT) {
        if (pt.stride > 0) {
            // i - j < 4096: the nearest integer to (i - j) / stride is exact for multiples
            const int dist = i - j;
            const int quot = (int)__builtin_rintf((float)dist * pt.inv_stride);
            s = s || (quot * pt.stride == dist && dist < pt.reach);
        }
        s = s || (i >= pt.NB - pt.n_dense);
    }
    return s;
}

// keys[0 .. 64*ceil((i+1)/64)): rank_key of candidates, 0 for static blocks and padding.
// Runs on one full wave; all control flow is wave-uniform.
template <bool EXT>
__device__ void select_row(const uint32_t* keys, int i, const Pattern& pt, int k, int T,
                           int32_t* __restrict__ idx_row, int32_t* __restrict__ cnt_out) {
    const int lane = threadIdx.x & 63;
    const int n = i + 1;
    const int chunks = (n + 63) >> 6;
    int n_cand = 0;                                           // candidates are the nonzero keys
    for (int m = 0; m < chunks; ++m) n_cand += __popcll(__ballot(keys[(m << 6) + lane] != 0u));
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
        bool is_static = j < n && static_block<EXT>(pt, i, j);
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

// scores come from memory: [rows_total = heads * NB, NBk]
// budget of query block i: the uniform k, or the schedule's entry clamped to [0, k]
__device__ __forceinline__ int row_budget(const int32_t* __restrict__ k_rows, int i, int k) {
    if (k_rows == nullptr) return k;
    const int v = k_rows[i];
    return v < 0 ? 0 : (v > k ? k : v);
}

// Per-head configuration: head h replaces (n_sink, n_local, top_k) by its own triple, clamped to
// [0, ns], [1, nl], [0, k] of the call (which are then the maxima that fix the row capacity).
__device__ __forceinline__ void head_config(const int32_t* __restrict__ head_pattern, int h, Pattern& pt, int& k) {
    if (head_pattern == nullptr) return;
    const int32_t* hp = head_pattern + 3 * h;
    const int a = hp[0], b = hp[1], c = hp[2];
    pt.ns = a < 0 ? 0 : (a > pt.ns ? pt.ns : a);
    pt.nl = b < 1 ? 1 : (b > pt.nl ? pt.nl : b);
    k = c < 0 ? 0 : (c > k ? k : c);
}

// cumulative-mass budget of a row, defined further down
template <bool EXT, typename ScoreFn>
__device__ int mass_budget_row(ScoreFn score, int i, const Pattern& pt, uint32_t gamma_q16, uint32_t* hist, int lane);

template <bool EXT>
__global__ __launch_bounds__(kWaves * 64) void topk_from_scores_kernel(
    const float* __restrict__ scores, int64_t n_rows, int NB /* query blocks */, int NBk, int off, Pattern pt, int k,
    const int32_t* __restrict__ k_rows, const int32_t* __restrict__ head_pattern, int Hq, int T,
    int32_t* __restrict__ idx, int32_t* __restrict__ cnt, int gamma_q16 /* -1: no mass budget */,
    const int32_t* __restrict__ seq_lens, int S, int Bs) {
    extern __shared__ uint32_t lds_keys[];       // [kWaves][padded NBk] keys, then 256 counters per wave (mass budget)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kWaves + wave;
    if (row >= n_rows) return;                               // whole wave leaves together
    const int iq = (int)(row % NB);
    const int i = iq + off;                                  // block position in the sequence
    const int NB_b = (entry_len(seq_lens, (int)(row / NB / Hq), S) + Bs - 1) / Bs;   // ragged batch
    if (iq >= NB_b) {                                        // a row past its entry's end: empty list
        for (int t = lane; t < T; t += 64) idx[row * T + t] = -1;
        if (lane == 0) cnt[row] = 0;
        return;
    }
    pt.NB = off + NB_b;
    head_config(head_pattern, (int)((row / NB) % Hq), pt, k);
    const int padded = ((NBk + 63) >> 6) << 6;
    uint32_t* keys = lds_keys + wave * padded;
    const float* srow = scores + row * NBk;
    const int chunks = (i + 64) >> 6;
    for (int m = 0; m < chunks; ++m) {
        int j = (m << 6) + lane;
        uint32_t key = 0u;
        if (j <= i && !static_block<EXT>(pt, i, j)) key = rank_key(srow[j]);
        keys[j] = key;
    }
    // each wave reads back only its own slice; LDS ops of one wave are ordered
    int k_i = row_budget(k_rows, iq, k);
    if (gamma_q16 >= 0) {
        uint32_t* hist = lds_keys + kWaves * padded + 256 * wave;
        const int k_m = mass_budget_row<EXT>([&](int j) { return srow[j]; }, i, pt, (uint32_t)gamma_q16, hist, lane);
        k_i = k_m < k_i ? k_m : k_i;
    }
    select_row<EXT>(keys, i, pt, k_i, T, idx + row * T, cnt + row);
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// x = hi + lo with both parts bf16 (round to nearest even twice)
__device__ __forceinline__ void split_bf16(const float4 a, const float4 b, bf16x8& hi, bf16x8& lo) {
    f32x8 x = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    hi = __builtin_convertvector(x, bf16x8);
    f32x8 back = __builtin_convertvector(hi, f32x8);
    lo = __builtin_convertvector(x - back, bf16x8);
}

// sum of v over the 64 lanes (DPP row reductions + row broadcasts), returned wave-uniform
__device__ __forceinline__ int wave_sum(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);   // row_half_mirror
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);   // row_mirror: every lane = its row's sum
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, true);   // row_bcast15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, true);   // row_bcast31 into rows 2 and 3
    return __builtin_amdgcn_readlane(v, 63);
}


// inclusive prefix sum of v over the 64 lanes (Hillis-Steele inside the rows of 16 with DPP row
// shifts, then the row totals are carried over with the row broadcasts)
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1, lanes shifted out read 0
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, true);   // row_bcast15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, true);   // row_bcast31 into rows 2 and 3
    return v;
}

// maximum / minimum of v over the 64 lanes, returned wave-uniform (same lane walk as wave_sum;
// lanes of rows that a step leaves out combine with the neutral element)
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    auto mx = [](uint32_t a, int b) { return a > (uint32_t)b ? a : (uint32_t)b; };
    v = mx(v, __builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true));
    v = mx(v, __builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true));
    v = mx(v, __builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true));
    v = mx(v, __builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true));
    v = mx(v, __builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, true));
    v = mx(v, __builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, true));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) { return ~wave_max_u32(~v); }

// Exact k-th largest key of a row, in two steps.
// 1. A bound from the lanes: with t = ceil(kk / 64), every lane's t-th largest key is matched or
//    beaten by t keys of that lane, so at least 64 t >= kk keys reach L = the smallest of the 64
//    lanes' t-th largest keys: the k-th largest is >= L, keys below L can neither be selected nor
//    tie with the threshold and drop out.  With 16 keys per lane and kk = 64 that leaves about a
//    tenth of the row.  (t <= 2 here; a lane without t candidates gives L = 0: no bound.)
// 2. Most-significant-digit radix selection among the keys in [L, H] (H = the row maximum), up
//    to 8 bits per pass, starting at the highest bit in which L and H differ (the bits above are
//    common to all of them): the wavefront histograms the current digit of the keys that still match
//    the decided prefix into its own 256 LDS counters (LDS atomics), lane l then owns the four bins
//    255-4l .. 252-4l, a prefix sum over the lanes finds the bin that holds the wanted rank, and
//    that bin's digit extends the prefix.  A pass that takes its whole bin ends the search.
// key[m] belongs to block 64*m + lane and is 0 for static blocks, blocks beyond i and unused chunks
// (0 is never counted); NC <= MAXC: only key[0 .. NC) can be nonzero for this row.  Returns
// thr / need_eq: take key > thr, plus the first need_eq keys equal to thr in block order.
// hist: this wavefront's 256 counters.
template <int MAXC, int NC>
__device__ __forceinline__ void find_threshold_hist(const uint32_t (&key)[MAXC], int kk, int n_cand, uint32_t* hist,
                                                    int lane, uint32_t& thr, int& need_eq) {
    thr = 0xffffffffu;
    need_eq = 0;
    if (kk <= 0) return;
    if (kk == n_cand) { thr = 0u; return; }
    uint32_t m1 = 0u, m2 = 0u;           // largest and second largest key of the lane
#pragma unroll
    for (int m = 0; m < NC; ++m) {
        const uint32_t v = key[m];
        const uint32_t lo = v < m1 ? v : m1;
        m2 = m2 > lo ? m2 : lo;
        m1 = m1 > v ? m1 : v;
    }
    const uint32_t H = wave_max_u32(m1);
    uint32_t L = kk <= 64 ? wave_min_u32(m1) : (kk <= 128 ? wave_min_u32(m2) : 0u);
    if (L == 0u) L = 1u;                 // no bound: every candidate (keys are >= 1) takes part
    if (L == H) {                        // all keys that matter are equal
        thr = H;
        need_eq = kk;
        return;
    }
    const int hb = 31 - __builtin_clz(L ^ H);                 // highest bit in which the keys in [L, H] can differ
    uint32_t prefix = hb == 31 ? 0u : (H >> (hb + 1)) << (hb + 1);   // decided bits, the rest zero
    int want = kk;                       // rank wanted among the keys that match the prefix (1 = largest)
    int top = hb + 1;                    // bits [top, 32) are decided
#pragma nounroll
    while (top > 0) {
        const int shift = top > 8 ? top - 8 : 0;              // this pass decides bits [shift, top)
        const uint32_t dmask = (1u << (top - shift)) - 1u;
        *reinterpret_cast<uint4*>(hist + 4 * lane) = make_uint4(0u, 0u, 0u, 0u);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
        for (int m = 0; m < NC; ++m) {
            const uint32_t kv = key[m];
            // kv >= L, and its decided bits match (two shifts: top may be 32)
            if (kv >= L && (((kv ^ prefix) >> (top - 1)) >> 1) == 0u) atomicAdd(&hist[(kv >> shift) & dmask], 1u);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint4 h = *reinterpret_cast<const uint4*>(hist + 252 - 4 * lane);   // .w = bin 255-4l ... .x = bin 252-4l
        const int own = (int)(h.x + h.y + h.z + h.w);
        const int incl = wave_inclusive_scan(own);
        const int Ln = __ffsll((unsigned long long)__ballot(incl >= want)) - 1;  // lane whose bins hold the wanted rank
        const int before = __builtin_amdgcn_readlane(incl - own, Ln);                // keys in higher bins
        const int b3 = __builtin_amdgcn_readlane((int)h.w, Ln), b2 = __builtin_amdgcn_readlane((int)h.z, Ln);
        const int b1 = __builtin_amdgcn_readlane((int)h.y, Ln), b0 = __builtin_amdgcn_readlane((int)h.x, Ln);
        const int rem = want - before;                                               // 1 .. own(Ln)
        int digit, above, in_bin;
        if (rem <= b3) { digit = 255 - 4 * Ln; above = 0; in_bin = b3; }
        else if (rem <= b3 + b2) { digit = 254 - 4 * Ln; above = b3; in_bin = b2; }
        else if (rem <= b3 + b2 + b1) { digit = 253 - 4 * Ln; above = b3 + b2; in_bin = b1; }
        else { digit = 252 - 4 * Ln; above = b3 + b2 + b1; in_bin = b0; }
        want = rem - above;                                                          // rank inside the chosen bin
        prefix |= (uint32_t)digit << shift;
        if (want == in_bin) {          // the whole bin is taken: every key that reaches both the bin's
            const uint32_t edge = prefix > L ? prefix : L;    // lower edge and L, none below
            thr = edge - 1u;           // edge >= L >= 1
            return;
        }
        top = shift;
    }
    thr = prefix;                      // the k-th largest key itself; `want` of its copies are taken
    need_eq = want;
}

// ---- cumulative-mass budget (the rule of the FlexPrefill family, named among the dynamic algorithms
// in Sec. 4.1.1 / "Other Sparse Attention Strategies" of Sec. 4.1.2; no formula in the paper) ----------
// A row takes, in ranking order, the fewest candidates for which the selected blocks (static ones
// included) hold the fraction gamma of the row's block-level softmax mass.  The mass is defined in
// integers so that the number of blocks does not depend on the order of a floating-point sum:
//   W_j = mass_weight(x_j, m) in [0, 2^19], m = the row's largest score that is not NaN,
//   target = ceil(Gamma * sum_j W_j / 65536), Gamma = gamma in 16-bit fixed point.
// mass_weight ~ 2^19 exp(x - m): every step is one IEEE fp32 operation, written with the
// never-contracted intrinsics, so that a CPU gets the same bits from the same sequence.
__device__ __forceinline__ uint32_t mass_weight(float x, float m) {
    if (x != x || m != m) return 0u;
    if (x == m) return 1u << 19;                          // also m = +inf
    if (__builtin_isinf(x) || __builtin_isinf(m)) return 0u;
    const float t = __fmul_rn(__fsub_rn(x, m), 1.44269504088896340736f);
    if (!(t >= -40.0f)) return 0u;
    const float n = __builtin_rintf(t);                   // ties to even
    const float f = __fsub_rn(t, n);
    float p = 1.5403530393381609954e-4f;                  // Taylor coefficients of e^(f ln 2), degree 6 .. 0
    p = __fmaf_rn(p, f, 1.3333558146428443423e-3f);
    p = __fmaf_rn(p, f, 9.6181291076284771619e-3f);
    p = __fmaf_rn(p, f, 5.5504108664821579953e-2f);
    p = __fmaf_rn(p, f, 2.4022650695910071233e-1f);
    p = __fmaf_rn(p, f, 6.9314718055994530942e-1f);
    p = __fmaf_rn(p, f, 1.0f);
    const float w = ldexpf(p, (int)n);
    return (uint32_t)__fadd_rn(__fmul_rn(w, 524288.0f), 0.5f);
}

// the score a rank key came from (keys >= 2; -0 has become +0)
__device__ __forceinline__ float score_of_key(uint32_t key) {
    uint32_t u = key - 1u;
    u = (u & 0x80000000u) ? (u ^ 0x80000000u) : ~u;
    return __uint_as_float(u);
}

// Number of candidates the mass budget lets the query block at block position i take (before the
// count budgets cap it).  One full wavefront; score(j) returns the ranking score of key block j <= i.
// hist: 256 LDS counters of this wavefront.  gamma_q16 = Gamma.
template <bool EXT, typename ScoreFn>
__device__ int mass_budget_row(ScoreFn score, int i, const Pattern& pt, uint32_t gamma_q16, uint32_t* hist, int lane) {
    const int chunks = (i + 64) >> 6;
    float mloc = -INFINITY;
    for (int c = 0; c < chunks; ++c) {
        const int j = (c << 6) + lane;
        const float x = j <= i ? score(j) : -INFINITY;
        if (x == x && x > mloc) mloc = x;
    }
    // wave maximum of floats through the order-preserving keys (mloc is never NaN)
    const uint32_t mk = wave_max_u32(rank_key(mloc));
    const float m = mk >= 2u ? score_of_key(mk) : -INFINITY;
    int z_l = 0, ms_l = 0;                                 // lane sums; a row's total is < 2^31
    for (int c = 0; c < chunks; ++c) {
        const int j = (c << 6) + lane;
        if (j <= i) {
            const int w = (int)mass_weight(score(j), m);
            z_l += w;
            if (static_block<EXT>(pt, i, j)) ms_l += w;
        }
    }
    const uint32_t Z = (uint32_t)wave_sum(z_l), Ms = (uint32_t)wave_sum(ms_l);
    const uint32_t target = (uint32_t)(((uint64_t)gamma_q16 * Z + 65535ull) >> 16);
    if (Ms >= target) return 0;
    uint32_t need = target - Ms;                           // mass still wanted from the candidates, >= 1
    // weighted radix selection: the key at which the mass of the better-ranked candidates reaches `need`
    uint32_t prefix = 0u;
#pragma nounroll
    for (int shift = 24; shift >= 0; shift -= 8) {
        *reinterpret_cast<uint4*>(hist + 4 * lane) = make_uint4(0u, 0u, 0u, 0u);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        for (int c = 0; c < chunks; ++c) {
            const int j = (c << 6) + lane;
            if (j <= i && !static_block<EXT>(pt, i, j)) {
                const float x = score(j);
                const uint32_t kv = rank_key(x);
                if ((((kv ^ prefix) >> shift) >> 8) == 0u) {
                    const uint32_t w = mass_weight(x, m);
                    if (w != 0u) atomicAdd(&hist[(kv >> shift) & 255u], w);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint4 h = *reinterpret_cast<const uint4*>(hist + 252 - 4 * lane);   // .w = bin 255-4l ... .x = bin 252-4l
        const int own = (int)(h.x + h.y + h.z + h.w);
        const int incl = wave_inclusive_scan(own);
        const int Ln = __ffsll((unsigned long long)__ballot((uint32_t)incl >= need)) - 1;   // exists: candidates' mass >= need
        const uint32_t before = (uint32_t)__builtin_amdgcn_readlane(incl - own, Ln);
        const uint32_t b3 = (uint32_t)__builtin_amdgcn_readlane((int)h.w, Ln), b2 = (uint32_t)__builtin_amdgcn_readlane((int)h.z, Ln);
        const uint32_t b1 = (uint32_t)__builtin_amdgcn_readlane((int)h.y, Ln);
        const uint32_t rem = need - before;
        uint32_t digit, above;
        if (rem <= b3) { digit = 255 - 4 * Ln; above = 0; }
        else if (rem <= b3 + b2) { digit = 254 - 4 * Ln; above = b3; }
        else if (rem <= b3 + b2 + b1) { digit = 253 - 4 * Ln; above = b3 + b2; }
        else { digit = 252 - 4 * Ln; above = b3 + b2 + b1; }
        need = rem - above;                                // mass wanted from the chosen bin, >= 1
        prefix |= digit << shift;
    }
    // prefix = the key tau of the last block taken; all of the better keys, plus as many copies of tau
    // (equal keys have equal weights) as it takes to cover what is left
    int n_above = 0;
    for (int c = 0; c < chunks; ++c) {
        const int j = (c << 6) + lane;
        const bool gt = j <= i && !static_block<EXT>(pt, i, j) && rank_key(score(j)) > prefix;
        n_above += __popcll(__ballot(gt));
    }
    const uint32_t w_tau = mass_weight(score_of_key(prefix), m);
    return n_above + (int)((need + w_tau - 1u) / w_tau);
}

// The same budget for a row whose keys already sit in registers (the select kernel): the weights are
// computed once per block, the weighted radix passes run over registers.  key[m] / is_static_bits
// as in the select kernel (block 64 m + lane; 0 = not a candidate); score(j) returns the ranking
// score of block j; chunks = chunks of 64 blocks the row reaches.  Integer arithmetic: the result is
// the one mass_budget_row gives, whatever the order of the sums.
template <int MAXC, typename ScoreFn>
__device__ __forceinline__ int mass_budget_regs(const uint32_t (&key)[MAXC], uint64_t is_static_bits, ScoreFn score, int i,
                                                int chunks, uint32_t gamma_q16, uint32_t* hist, int lane) {
    float x[MAXC];
    float mloc = -INFINITY;
#pragma unroll
    for (int m = 0; m < MAXC; ++m) {
        x[m] = -INFINITY;
        if (m < chunks) {
            const int j = (m << 6) + lane;
            x[m] = j <= i ? score(j) : __builtin_nanf("");   // NaN: weighs nothing, never the maximum
            if (x[m] == x[m] && x[m] > mloc) mloc = x[m];
        }
    }
    const uint32_t mk = wave_max_u32(rank_key(mloc));
    const float mx = mk >= 2u ? score_of_key(mk) : -INFINITY;
    uint32_t w[MAXC];
    int z_l = 0, ms_l = 0;
#pragma unroll
    for (int m = 0; m < MAXC; ++m) {
        w[m] = 0u;
        if (m < chunks) {
            w[m] = mass_weight(x[m], mx);
            z_l += (int)w[m];
            if ((is_static_bits >> m) & 1ull) ms_l += (int)w[m];
        }
    }
    const uint32_t Z = (uint32_t)wave_sum(z_l), Ms = (uint32_t)wave_sum(ms_l);
    const uint32_t target = (uint32_t)(((uint64_t)gamma_q16 * Z + 65535ull) >> 16);
    if (Ms >= target) return 0;
    uint32_t need = target - Ms;
    uint32_t prefix = 0u;
#pragma nounroll
    for (int shift = 24; shift >= 0; shift -= 8) {
        *reinterpret_cast<uint4*>(hist + 4 * lane) = make_uint4(0u, 0u, 0u, 0u);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
        for (int m = 0; m < MAXC; ++m) {
            const uint32_t kv = key[m];
            if (m < chunks && kv != 0u && w[m] != 0u && (((kv ^ prefix) >> shift) >> 8) == 0u)
                atomicAdd(&hist[(kv >> shift) & 255u], w[m]);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint4 h = *reinterpret_cast<const uint4*>(hist + 252 - 4 * lane);   // .w = bin 255-4l ... .x = bin 252-4l
        const int own = (int)(h.x + h.y + h.z + h.w);
        const int incl = wave_inclusive_scan(own);
        const int Ln = __ffsll((unsigned long long)__ballot((uint32_t)incl >= need)) - 1;
        const uint32_t before = (uint32_t)__builtin_amdgcn_readlane(incl - own, Ln);
        const uint32_t b3 = (uint32_t)__builtin_amdgcn_readlane((int)h.w, Ln), b2 = (uint32_t)__builtin_amdgcn_readlane((int)h.z, Ln);
        const uint32_t b1 = (uint32_t)__builtin_amdgcn_readlane((int)h.y, Ln);
        const uint32_t rem = need - before;
        uint32_t digit, above;
        if (rem <= b3) { digit = 255 - 4 * Ln; above = 0; }
        else if (rem <= b3 + b2) { digit = 254 - 4 * Ln; above = b3; }
        else if (rem <= b3 + b2 + b1) { digit = 253 - 4 * Ln; above = b3 + b2; }
        else { digit = 252 - 4 * Ln; above = b3 + b2 + b1; }
        need = rem - above;
        prefix |= digit << shift;
    }
    int n_above_l = 0;
#pragma unroll
    for (int m = 0; m < MAXC; ++m) n_above_l += (m < chunks && key[m] > prefix) ? 1 : 0;
    const int n_above = wave_sum(n_above_l);
    const uint32_t w_tau = mass_weight(score_of_key(prefix), mx);
    return n_above + (int)((need + w_tau - 1u) / w_tau);
}

// Everything the score + top-k step of one workgroup needs besides its rows.
struct ScoreArgs {
    const float* qp;              // pooled Q [B*Hq, NB, D] fp32
    const float* kp;              // pooled K, tiled in operand layout by the pooling kernel
    int Hq, G, NB /* query blocks */, NBk, off /* block position of query block 0 */;
    Pattern pt;
    int k;
    const int32_t* k_rows;
    const int32_t* head_pattern;
    const float* lvn;
    int T;
    float scale;
    int32_t* idx;
    int32_t* cnt;
    float* scores_out;
    uint32_t gamma_q16;           // cumulative-mass budget in 16-bit fixed point (MASS kernels only)
    const int32_t* seq_lens;      // ragged batch: tokens per batch entry, or nullptr
    int S, Bs;                    // padded query tokens, block size (to turn seq_lens into block counts)
    const uint16_t* q;            // QPOOL kernels: the queries themselves (pooled in the kernel), layout qs
    Strides qs;
};

// Phase 0 of the score kernels: the split pooled queries (MFMA A operands) of the query blocks
// i0 .. i0 + R - 1 of head bh go to LDS behind the SW words of score space at S, in the space of the
// phase-2 counters, instead of being held in 8 * D / 16 registers per lane: the kernels stay within
// 128 registers.  Needs R * D * 4 bytes <= the counters' NWV KB.
// QPOOL: the workgroup pools its R query blocks from Q itself (the block mean pooling of step 1,
// same arithmetic in the same order as pool_kernel) instead of reading pooled queries.  Streaming
// 16 blocks (512 KB) per workgroup with two blocks per 256 threads in flight keeps the HBM busy
// while the other workgroup of the CU scores and selects: the Q stream, four fifths of the bytes
// of the select stage, hides the rest of the stage.  Ends with a barrier.
template <int D, int R, int SW, int NWV, bool QPOOL>
__device__ __forceinline__ void stage_queries(const ScoreArgs& a, const int bh, const int i0, float* S) {
    constexpr int DS = D / 16;
    const int NB = a.NB;
    const int b = bh / a.Hq, h = bh % a.Hq;
    const float* qbase = a.qp + (int64_t)bh * NB * D;
    // LDS copy of the split queries: the 8 dims 16s + 8 * half .. +7 of row r, part p (0 = hi, 1 = lo)
    // at bf16 offset ((((s * 2 + p) * R + r) * 2 + half) * 8
    __bf16* const qlds = reinterpret_cast<__bf16*>(S + SW);
    static_assert(R * D * 4 <= NWV * 256 * 4, "staged queries must fit the counters' space");
    if constexpr (QPOOL) {
        constexpr int TPR = D / 8, RPP = 256 / TPR;      // lanes per token row, token rows per pass
        constexpr int NGRP = NWV / 4;                    // groups of 256 threads, one block at a time each
        constexpr int ROWS = (R + NGRP - 1) / NGRP;      // query blocks per group
        constexpr int DEPTH = 2;                         // blocks in flight per group
        // the partial sums live in the score rows' space, or (short rows) behind the counters
        constexpr bool PART_IN_S = 2 * NGRP * RPP * D <= SW;
        const int t = threadIdx.x, grp = t >> 8, t256 = t & 255;
        const int prow = t256 / TPR, chunk = t256 % TPR;
        const int Bs = a.Bs, passes = Bs / RPP;          // at most 8
        const int Sq_b = entry_len(a.seq_lens, b, a.S);
        typedef float (*Part)[D];
        Part const part = reinterpret_cast<Part>(PART_IN_S ? S : S + SW + NWV * 256) + grp * 2 * RPP;   // two buffers of RPP rows per group
        const uint16_t* const qhead = a.q + b * a.qs.b + h * a.qs.h;
        const int64_t tstride = a.qs.t;
        // tokens of this group's rr-th block that exist (0: block past the call, the entry or the tile)
        auto valid_tokens = [&](int rr) {
            const int r = grp + rr * NGRP, iq = i0 + r;
            if (r >= R || iq >= NB) return 0;
            const int n = Sq_b - iq * Bs;
            return n < 0 ? 0 : (n > Bs ? Bs : n);
        };
        // One instantiation per number of passes (block size / token rows per pass) and per kind of
        // tile.  FULL: every block of the tile exists and is whole, so all loads are unconditional: the
        // compiler can then wait for exactly the block it is about to reduce while the next two stay in
        // flight (with a conditional load anywhere in the loop it waits for all of them, and a
        // workgroup streams at a third of the rate).  Otherwise (last tile of a sequence) rows are
        // predicated; that path is rare and not tuned.
        auto pool_rows = [&](auto passes_tag, auto full_tag) {
            constexpr int PASSES = decltype(passes_tag)::value;
            constexpr bool FULL = decltype(full_tag)::value != 0;
            uint4 raw[DEPTH][PASSES];
            // per-lane byte offsets inside a block (fixed for the kernel; token stride <= 2^22 elements,
            // so they fit 32 bits) on top of a wave-uniform block base
            uint32_t voff[PASSES];
#pragma unroll
            for (int p2 = 0; p2 < PASSES; ++p2) voff[p2] = 2u * ((uint32_t)(p2 * RPP + prow) * (uint32_t)tstride + (uint32_t)chunk * 8u);
            const int grp_u = __builtin_amdgcn_readfirstlane(grp);
            auto load = [&](auto slot_tag, int rr) {
                constexpr int SLOT = decltype(slot_tag)::value;
                const char* const base = reinterpret_cast<const char*>(qhead + (int64_t)(i0 + grp_u + rr * NGRP) * Bs * tstride);
                const int nv = FULL ? Bs : valid_tokens(rr);
#pragma unroll
                for (int p2 = 0; p2 < PASSES; ++p2) {
                    if constexpr (FULL) {
                        raw[SLOT][p2] = stream_load16(reinterpret_cast<const uint16_t*>(base + voff[p2]));
                    } else {
                        raw[SLOT][p2] = make_uint4(0u, 0u, 0u, 0u);
                        if (p2 * RPP + prow < nv) raw[SLOT][p2] = stream_load16(reinterpret_cast<const uint16_t*>(base + voff[p2]));
                    }
                }
            };
            static_for_sel<(DEPTH < ROWS ? DEPTH : ROWS)>([&](auto rr_tag) { load(rr_tag, decltype(rr_tag)::value); });
            static_for_sel<ROWS>([&](auto rr_tag) {
                constexpr int RR = decltype(rr_tag)::value;
                constexpr int SLOT = RR % DEPTH;
                float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int p2 = 0; p2 < PASSES; ++p2) {
                    acc[0] += bf16_lo(raw[SLOT][p2].x); acc[1] += bf16_hi(raw[SLOT][p2].x);
                    acc[2] += bf16_lo(raw[SLOT][p2].y); acc[3] += bf16_hi(raw[SLOT][p2].y);
                    acc[4] += bf16_lo(raw[SLOT][p2].z); acc[5] += bf16_hi(raw[SLOT][p2].z);
                    acc[6] += bf16_lo(raw[SLOT][p2].w); acc[7] += bf16_hi(raw[SLOT][p2].w);
                }
                Part const buf = part + (RR & 1) * RPP;
#pragma unroll
                for (int e = 0; e < 8; ++e) buf[prow][chunk * 8 + e] = acc[e];
                if constexpr (RR + DEPTH < ROWS) load(IC_sel<SLOT>{}, RR + DEPTH);
                __syncthreads();
                const int r = grp + RR * NGRP;
                if (t256 < D && r < R) {
                    float sum = 0.f;
#pragma unroll
                    for (int rr2 = 0; rr2 < RPP; ++rr2) sum += buf[rr2][t256];
                    const int nv = FULL ? Bs : valid_tokens(RR);
                    const float mean = nv == Bs ? sum * (1.0f / (float)Bs) : (nv > 0 ? sum / (float)nv : 0.f);
                    const __bf16 hi = (__bf16)mean;                   // round to nearest even, twice
                    const __bf16 lo = (__bf16)(mean - (float)hi);
                    const int at = ((((t256 >> 4) * 2 + 0) * R + r) * 2 + ((t256 >> 3) & 1)) * 8 + (t256 & 7);
                    qlds[at] = hi;
                    qlds[at + R * 2 * 8] = lo;
                }
            });
        };
        // whole tile inside the call, the entry and (rows per group) the tile: every block is full
        const bool full = R % NGRP == 0 && (int64_t)(i0 + R) * Bs <= (int64_t)Sq_b;
        constexpr int P128 = 128 / RPP, P64 = 64 / RPP;  // passes for blocks of 128 / 64 tokens
        if (passes == P128) {
            if (full) pool_rows(IC_sel<P128>{}, IC_sel<1>{}); else pool_rows(IC_sel<P128>{}, IC_sel<0>{});
        } else {
            if (full) pool_rows(IC_sel<P64>{}, IC_sel<1>{}); else pool_rows(IC_sel<P64>{}, IC_sel<0>{});
        }
        __syncthreads();
    } else {
        const int t = threadIdx.x;
        if (t < R * DS * 2) {
            const int r = t % R, s2 = (t / R) >> 1, hf = (t / R) & 1;
            int row = i0 + r;
            if (row > NB - 1) row = NB - 1;               // rows past the end are computed but never used
            const float* src = qbase + (int64_t)row * D + 16 * s2 + 8 * hf;
            bf16x8 hi, lo;
            split_bf16(*reinterpret_cast<const float4*>(src), *reinterpret_cast<const float4*>(src + 4), hi, lo);
            *reinterpret_cast<bf16x8*>(qlds + (((s2 * 2 + 0) * R + r) * 2 + hf) * 8) = hi;
            *reinterpret_cast<bf16x8*>(qlds + (((s2 * 2 + 1) * R + r) * 2 + hf) * 8) = lo;
        }
        __syncthreads();
    }
}

// Scores, top-k and merged lists of the query blocks i0 .. i0 + R - 1 of head bh = b * Hq + h, by a
// 512-thread workgroup.  S: R * (MAXC * 64 + 8) floats of LDS for the scores, then 256 counters per
// wavefront.  Ends without a barrier; the caller must not reuse S before one.
// The split pooled queries are staged in LDS by stage_queries (QPOOL: pooled from Q in the kernel).
template <int D, int R, int MAXC, bool EXT, bool MASS, int NWV, bool QPOOL>
__device__ __forceinline__ void score_topk_rows(const ScoreArgs& a, const int bh, const int i0, float* S) {
    constexpr int LD = MAXC * 64 + 8;          // +8 words: the two lane halves of a store hit different banks
    constexpr int DS = D / 16;
    const float* __restrict__ kp = a.kp;
    const int Hq = a.Hq, G = a.G, NB = a.NB, NBk = a.NBk, off = a.off, T = a.T;
    Pattern pt = a.pt;
    int k = a.k;
    const int32_t* __restrict__ k_rows = a.k_rows;
    const int32_t* __restrict__ head_pattern = a.head_pattern;
    const float* __restrict__ lvn = a.lvn;
    const float scale = a.scale;
    int32_t* __restrict__ idx = a.idx;
    int32_t* __restrict__ cnt = a.cnt;
    float* __restrict__ scores_out = a.scores_out;

    const int b = bh / Hq, h = bh % Hq;
    const int Hkv = Hq / G;
    const float* kbase = kp + (int64_t)(b * Hkv + h / G) * ((NBk + 31) >> 5) * (32 * D);   // tiled, see fetch_tile
    const float* lvbase = lvn != nullptr ? lvn + (int64_t)(b * Hkv + h / G) * NBk : nullptr;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int i_last = (i0 + R - 1 < NB - 1) ? i0 + R - 1 : NB - 1;
    const int n_jt = ((i_last + off) >> 5) + 1;           // 32-wide key-block tiles with some causal j

    // ---- phase 0 / phase 1 ------------------------------------------------------------
    // LDS copy of the split queries: the 8 dims 16s + 8 * half .. +7 of row r, part p (0 = hi, 1 = lo)
    // at bf16 offset ((((s * 2 + p) * R + r) * 2 + half) * 8
    stage_queries<D, R, R * LD, NWV, QPOOL>(a, bh, i0, S);
    const __bf16* const qlds = reinterpret_cast<const __bf16*>(S + R * LD);
    // The pooled K arrives tiled in operand layout and already split into bf16 head and tail:
    // tile jt of 32 key blocks is 32 * D * 4 bytes, and the 8 dims 16s + 8 * half .. +7 of block
    // l32 sit at bf16 offset (((2s + half) * 2 + part) * 32 + l32) * 8 (part 0 = hi, 1 = lo), so
    // every load instruction of a wavefront covers 1-KB pieces (row-major rows would cost 32 cache
    // lines per instruction) and what it loads is the MFMA operand.  One register buffer serves
    // as a whole-tile pipeline: as soon as the three products of a 16-dim slice have been issued,
    // the same registers are refilled with that slice of the wave's next tile, so every load has a
    // full tile of MFMA work to arrive.  Blocks past NBk in the last tile hold whatever the
    // workspace held: their columns are never ranked or written out.
    bf16x8 kraw[2 * DS];                                  // [2s] = hi, [2s + 1] = lo of slice s
    auto tile_ptr = [&](int jt) {
        return reinterpret_cast<const __bf16*>(kbase + (int64_t)jt * (32 * D)) + (half * 64 + l32) * 8;
    };
    if (wave < n_jt) {
        const __bf16* src = tile_ptr(wave);
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            kraw[2 * s] = *reinterpret_cast<const bf16x8*>(src + s * 1024);
            kraw[2 * s + 1] = *reinterpret_cast<const bf16x8*>(src + s * 1024 + 256);
        }
    }
    for (int jt = wave; jt < n_jt; jt += NWV) {
        const int j = 32 * jt + l32;
        // output-aware ranking: the key block's ln(value magnitude) joins its score
        const float lv = lvbase != nullptr ? lvbase[j < NBk ? j : NBk - 1] : 0.f;
        // the last tile refills from itself: in bounds, never used
        const __bf16* next = tile_ptr(jt + NWV < n_jt ? jt + NWV : jt);
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            const bf16x8 k_hi = kraw[2 * s], k_lo = kraw[2 * s + 1];
            const bf16x8 qh = *reinterpret_cast<const bf16x8*>(qlds + (((s * 2 + 0) * R + l32 % R) * 2 + half) * 8);
            const bf16x8 ql = *reinterpret_cast<const bf16x8*>(qlds + (((s * 2 + 1) * R + l32 % R) * 2 + half) * 8);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ql, k_hi, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qh, k_lo, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qh, k_hi, acc, 0, 0, 0);
            kraw[2 * s] = *reinterpret_cast<const bf16x8*>(next + s * 1024);
            kraw[2 * s + 1] = *reinterpret_cast<const bf16x8*>(next + s * 1024 + 256);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int mrow = 8 * (r >> 2) + 4 * half + (r & 3);     // row of the 32x32 result held in acc[r]
            if (mrow < R) {
                const float sc = lvbase != nullptr ? scale * acc[r] + lv : scale * acc[r];
                S[mrow * LD + j] = sc;
                const int i = i0 + mrow;
                if (scores_out != nullptr && i < NB && j < NBk)
                    scores_out[((int64_t)bh * NB + i) * NBk + j] = j <= i + off ? sc : -INFINITY;
            }
        }
    }
    if (scores_out != nullptr) {                          // key blocks past the last computed tile
        const int j_first = 32 * n_jt;
        for (int r = 0; r < R && i0 + r < NB; ++r)
            for (int j = j_first + (int)threadIdx.x; j < NBk; j += NWV * 64)
                scores_out[((int64_t)bh * NB + i0 + r) * NBk + j] = -INFINITY;
    }
    __syncthreads();

    // ---- phase 2 ---------------------------------------------------------------------
    head_config(head_pattern, h, pt, k);
    // ragged batch: this entry's own block count; its rows beyond get empty lists, and the dense
    // strip of the Tri-shape means the entry's own last rows
    const int NB_b = (entry_len(a.seq_lens, b, a.S) + a.Bs - 1) / a.Bs;
    pt.NB = off + NB_b;
#pragma nounroll
    for (int r = wave; r < R; r += NWV) {
        const int iq = i0 + r;                            // query block of the call
        if (iq >= NB) break;                              // wave-uniform
        if (iq >= NB_b) {
            const int64_t row = (int64_t)bh * NB + iq;
            for (int t = lane; t < T; t += 64) idx[row * T + t] = -1;
            if (lane == 0) cnt[row] = 0;
            continue;
        }
        const int i = iq + off;                           // its block position in the sequence
        const int n = i + 1;
        const float* srow = S + r * LD;
        // keys and static flags of the row's blocks stay in registers until the lists are written;
        // rows are causal: a row early in the sequence fills only its first chunks of 64 blocks
        const int chunks = (n + 63) >> 6;                 // wave-uniform
        uint32_t key[MAXC];
        uint64_t is_static_bits = 0ull;                   // bit m: block 64 m + lane is static
#pragma unroll
        for (int m = 0; m < MAXC; ++m) {
            key[m] = 0u;
            if (m < chunks) {
                const int j = (m << 6) + lane;            // < MAXC*64 <= LD: always inside the row
                const bool st = j <= i && static_block<EXT>(pt, i, j);
                const uint32_t kv = rank_key(srow[j]);    // columns past the computed tiles hold junk: masked next
                key[m] = (j <= i && !st) ? kv : 0u;
                is_static_bits |= st ? (1ull << m) : 0ull;
            }
        }
        int n_cand;
        if constexpr (EXT) {                              // count the candidates: no closed form worth having
            int ncl = 0;
#pragma unroll
            for (int m = 0; m < MAXC; ++m) ncl += key[m] != 0u ? 1 : 0;
            n_cand = wave_sum(ncl);
        } else {
            const int lo = i - pt.nl + 1;
            int n_sink = pt.ns < n ? pt.ns : n;
            int n_local = pt.nl < n ? pt.nl : n;
            int first_local = lo > 0 ? lo : 0;
            int overlap = n_sink - first_local; if (overlap < 0) overlap = 0;
            n_cand = n - (n_sink + n_local - overlap);
        }
        int k_i = row_budget(k_rows, iq, k);
        uint32_t* hist = reinterpret_cast<uint32_t*>(S + R * LD) + 256 * wave;
        if constexpr (MASS) {                             // the mass budget on top of the count budgets
            int k_m;                                      // rows of up to 2048 blocks: weights kept in registers
            if constexpr (MAXC <= 32)
                k_m = mass_budget_regs<MAXC>(key, is_static_bits, [&](int j) { return srow[j]; }, i, chunks, a.gamma_q16, hist, lane);
            else
                k_m = mass_budget_row<EXT>([&](int j) { return srow[j]; }, i, pt, a.gamma_q16, hist, lane);
            k_i = k_m < k_i ? k_m : k_i;
        }
        const int kk = k_i < n_cand ? k_i : n_cand;
        uint32_t thr;
        int need_eq;
        const int nc4 = 4 * chunks;
        if (nc4 <= MAXC) find_threshold_hist<MAXC, (MAXC + 3) / 4>(key, kk, n_cand, hist, lane, thr, need_eq);
        else if (nc4 <= 2 * MAXC) find_threshold_hist<MAXC, (MAXC + 1) / 2>(key, kk, n_cand, hist, lane, thr, need_eq);
        else if (nc4 <= 3 * MAXC) find_threshold_hist<MAXC, (3 * MAXC + 3) / 4>(key, kk, n_cand, hist, lane, thr, need_eq);
        else find_threshold_hist<MAXC, MAXC>(key, kk, n_cand, hist, lane, thr, need_eq);

        // emit static U top-k in ascending block order
        const int64_t row = (int64_t)bh * NB + iq;
        int32_t* idx_row = idx + row * T;
        int eq_seen = 0, out_pos = 0;
#pragma unroll
        for (int m = 0; m < MAXC; ++m) {
            if (m < chunks) {
                const uint32_t kv = key[m];
                const bool is_eq = need_eq > 0 && kv == thr && kv != 0u;
                const uint64_t eq_mask = __ballot(is_eq);
                const bool take = ((is_static_bits >> m) & 1ull) != 0ull || (kv != 0u && kv > thr) ||
                                  (is_eq && eq_seen + lanes_below(eq_mask, lane) < need_eq);
                const uint64_t take_mask = __ballot(take);
                if (take) idx_row[out_pos + lanes_below(take_mask, lane)] = (m << 6) + lane;
                eq_seen += __popcll(eq_mask);
                out_pos += __popcll(take_mask);
            }
        }
        for (int t = out_pos + lane; t < T; t += 64) idx_row[t] = -1;
        if (lane == 0) cnt[row] = out_pos;
    }
}

// Column-chunked variant for rows of 1025 .. 2048 key blocks: R = 16 query blocks per workgroup, as
// for 1024-block rows, so that every pooled-K tile a workgroup reads from L2 serves 16 rows (8-row
// workgroups re-read the pooled K twice as often: 5.2 GB against the 2.7 GB Q stream at 262144
// tokens, and use a quarter of every MFMA), while the scores in LDS stay those of one chunk of
// CW = 1024 key blocks: 66 KB, two workgroups per CU.  A wavefront owns two rows; the scores of the
// first chunk wait in registers (16 per lane and row) while the second chunk is scored, then each
// row is selected exactly as in the plain kernel, from 32 scores per lane.  (No cumulative-mass
// variant: that budget keeps the 8-row kernel.)
template <int D, int R, int MAXCH, bool EXT, int NWV, bool QPOOL>
__device__ __forceinline__ void score_topk_rows_chunked(const ScoreArgs& a, const int bh, const int i0, float* S) {
    constexpr int CC = 16;                     // 64-block register chunks per column chunk
    constexpr int CW = CC * 64;                // key blocks per column chunk
    constexpr int LD = CW + 8;
    constexpr int DS = D / 16;
    constexpr int RPW = R / NWV;               // rows per wavefront
    constexpr int MAXC = MAXCH * CC;
    static_assert(R % NWV == 0 && MAXCH == 2, "two column chunks");
    const float* __restrict__ kp = a.kp;
    const int Hq = a.Hq, G = a.G, NB = a.NB, NBk = a.NBk, off = a.off, T = a.T;
    Pattern pt = a.pt;
    int k = a.k;
    const float scale = a.scale;
    int32_t* __restrict__ idx = a.idx;
    int32_t* __restrict__ cnt = a.cnt;
    float* __restrict__ scores_out = a.scores_out;

    const int b = bh / Hq, h = bh % Hq;
    const int Hkv = Hq / G;
    const float* kbase = kp + (int64_t)(b * Hkv + h / G) * ((NBk + 31) >> 5) * (32 * D);
    const float* lvbase = a.lvn != nullptr ? a.lvn + (int64_t)(b * Hkv + h / G) * NBk : nullptr;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int i_last = (i0 + R - 1 < NB - 1) ? i0 + R - 1 : NB - 1;
    const int n_jt = ((i_last + off) >> 5) + 1;           // 32-wide key-block tiles with some causal j
    const int n_ch = (i_last + off) / CW + 1;             // column chunks with some causal j (workgroup-uniform)

    stage_queries<D, R, R * LD, NWV, QPOOL>(a, bh, i0, S);
    const __bf16* const qlds = reinterpret_cast<const __bf16*>(S + R * LD);

    head_config(a.head_pattern, h, pt, k);
    const int NB_b = (entry_len(a.seq_lens, b, a.S) + a.Bs - 1) / a.Bs;      // ragged batch
    pt.NB = off + NB_b;

    auto tile_ptr = [&](int jt) {
        return reinterpret_cast<const __bf16*>(kbase + (int64_t)jt * (32 * D)) + (half * 64 + l32) * 8;
    };
    // Scores of column chunk c into S (phase 1 of the plain kernel, restricted to the chunk's tiles).
    // NBUF = DS: the whole-tile register pipeline of the plain kernel (a slice's registers are refilled
    // with the same slice of the wave's next tile as soon as its three products are issued).
    // NBUF = DS / 2, for the second chunk, when 32 registers per lane hold the first chunk's scores: a
    // rolling buffer of half a tile; slot s % NBUF holds slice s and is refilled with slice s + NBUF,
    // of this tile or the next, so a load still has half a tile of MFMA work to arrive.
    auto score_chunk = [&](int c, auto nbuf_tag) {
        constexpr int NBUF = decltype(nbuf_tag)::value;
        bf16x8 kraw[2 * NBUF];                            // [2b] = hi, [2b + 1] = lo of the slice in slot b
        const int jt_end = n_jt < (c + 1) * (CW / 32) ? n_jt : (c + 1) * (CW / 32);
        const int jt_first = c * (CW / 32) + wave;
        if (jt_first < jt_end) {
            const __bf16* src = tile_ptr(jt_first);
#pragma unroll
            for (int s = 0; s < NBUF; ++s) {
                kraw[2 * s] = *reinterpret_cast<const bf16x8*>(src + s * 1024);
                kraw[2 * s + 1] = *reinterpret_cast<const bf16x8*>(src + s * 1024 + 256);
            }
        }
        for (int jt = jt_first; jt < jt_end; jt += NWV) {
            const int j = 32 * jt + l32;
            const float lv = lvbase != nullptr ? lvbase[j < NBk ? j : NBk - 1] : 0.f;
            const __bf16* cur = tile_ptr(jt);
            const __bf16* next = tile_ptr(jt + NWV < jt_end ? jt + NWV : jt);      // the last tile refills from itself: in bounds, never used
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                const int slot = s % NBUF;
                const bf16x8 k_hi = kraw[2 * slot], k_lo = kraw[2 * slot + 1];
                const bf16x8 qh = *reinterpret_cast<const bf16x8*>(qlds + (((s * 2 + 0) * R + l32 % R) * 2 + half) * 8);
                const bf16x8 ql = *reinterpret_cast<const bf16x8*>(qlds + (((s * 2 + 1) * R + l32 % R) * 2 + half) * 8);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ql, k_hi, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qh, k_lo, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qh, k_hi, acc, 0, 0, 0);
                const int s_fill = (s + NBUF) % DS;                               // the slice this slot holds next
                const __bf16* from = s + NBUF < DS ? cur : next;
                kraw[2 * slot] = *reinterpret_cast<const bf16x8*>(from + s_fill * 1024);
                kraw[2 * slot + 1] = *reinterpret_cast<const bf16x8*>(from + s_fill * 1024 + 256);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int mrow = 8 * (r >> 2) + 4 * half + (r & 3);
                if (mrow < R) {
                    const float sc = lvbase != nullptr ? scale * acc[r] + lv : scale * acc[r];
                    S[mrow * LD + j - c * CW] = sc;
                    const int i = i0 + mrow;
                    if (scores_out != nullptr && i < NB && j < NBk)
                        scores_out[((int64_t)bh * NB + i) * NBk + j] = j <= i + off ? sc : -INFINITY;
                }
            }
        }
    };
    // scores of the blocks c * CW + 64 m + lane of row r from the chunk's scores in S (columns past the
    // computed tiles hold junk; they lie beyond the causal limit and are never candidates)
    auto load_scores = [&](int r, float* x) {
        const float* srow = S + r * LD;
#pragma unroll
        for (int m = 0; m < CC; ++m) x[m] = srow[(m << 6) + lane];
    };

    float x0[RPW][CC];                                    // first-chunk scores of this wavefront's rows
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
        for (int m = 0; m < CC; ++m) x0[rr][m] = -INFINITY;
    score_chunk(0, IC_sel<DS>{});
    __syncthreads();
    if (n_ch > 1) {                                       // workgroup-uniform
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) {
            const int iq = i0 + wave + rr * NWV;
            if (iq < NB && iq < NB_b) load_scores(wave + rr * NWV, x0[rr]);
        }
        __syncthreads();                                  // every row's first-chunk scores are in registers
        score_chunk(1, IC_sel<DS / 2>{});
        __syncthreads();
    }
    if (scores_out != nullptr) {                          // key blocks past the last computed tile
        const int j_first = 32 * n_jt;
        for (int r = 0; r < R && i0 + r < NB; ++r)
            for (int j = j_first + (int)threadIdx.x; j < NBk; j += NWV * 64)
                scores_out[((int64_t)bh * NB + i0 + r) * NBk + j] = -INFINITY;
    }

    // ---- selection, row by row, as in the plain kernel; the staged queries are not needed any more,
    // their space holds the counters of the search ----
    uint32_t* const hist = reinterpret_cast<uint32_t*>(S + R * LD) + 256 * wave;
    static_for_sel<RPW>([&](auto rr_tag) {
        constexpr int rr = decltype(rr_tag)::value;
        const int r = wave + rr * NWV;
        const int iq = i0 + r;
        if (iq >= NB) return;                             // wave-uniform
        const int64_t row = (int64_t)bh * NB + iq;
        int32_t* idx_row = idx + row * T;
        if (iq >= NB_b) {                                 // past the entry's end: empty list
            for (int t = lane; t < T; t += 64) idx_row[t] = -1;
            if (lane == 0) cnt[row] = 0;
            return;
        }
        const int i = iq + off;
        const int n = i + 1;
        const int chunks = (n + 63) >> 6;
        float x[MAXC];
        if (n_ch > 1) {
#pragma unroll
            for (int m = 0; m < CC; ++m) x[m] = x0[rr][m];
            load_scores(r, x + CC);
        } else {
            load_scores(r, x);
#pragma unroll
            for (int m = CC; m < MAXC; ++m) x[m] = -INFINITY;
        }
        const int k_i = row_budget(a.k_rows, iq, k);
        {
            uint32_t key[MAXC];
            uint64_t is_static_bits = 0ull;
            int ncl = 0;
#pragma unroll
            for (int m = 0; m < MAXC; ++m) {
                key[m] = 0u;
                if (m < chunks) {
                    const int j = (m << 6) + lane;
                    const bool st = j <= i && static_block<EXT>(pt, i, j);
                    key[m] = (j <= i && !st) ? rank_key(x[m]) : 0u;
                    is_static_bits |= st ? (1ull << m) : 0ull;
                    if constexpr (EXT) ncl += key[m] != 0u ? 1 : 0;
                }
            }
            int n_cand;
            if constexpr (EXT) {
                n_cand = wave_sum(ncl);
            } else {                                      // sinks 0 .. ns-1, window i-nl+1 .. i, the rest are candidates
                const int n_sink = pt.ns < n ? pt.ns : n;
                const int first_local = i - pt.nl + 1 > n_sink ? i - pt.nl + 1 : n_sink;
                n_cand = first_local - n_sink;
            }
            const int kk = k_i < n_cand ? k_i : n_cand;
            uint32_t thr;
            int need_eq;
            const int nc4 = 4 * chunks;
            if (nc4 <= MAXC) find_threshold_hist<MAXC, (MAXC + 3) / 4>(key, kk, n_cand, hist, lane, thr, need_eq);
            else if (nc4 <= 2 * MAXC) find_threshold_hist<MAXC, (MAXC + 1) / 2>(key, kk, n_cand, hist, lane, thr, need_eq);
            else if (nc4 <= 3 * MAXC) find_threshold_hist<MAXC, (3 * MAXC + 3) / 4>(key, kk, n_cand, hist, lane, thr, need_eq);
            else find_threshold_hist<MAXC, MAXC>(key, kk, n_cand, hist, lane, thr, need_eq);
            int eq_seen = 0, out_pos = 0;
#pragma unroll
            for (int m = 0; m < MAXC; ++m) {
                if (m < chunks) {
                    const uint32_t kv = key[m];
                    const bool is_eq = need_eq > 0 && kv == thr && kv != 0u;
                    const uint64_t eq_mask = __ballot(is_eq);
                    const bool take = ((is_static_bits >> m) & 1ull) != 0ull || (kv != 0u && kv > thr) ||
                                      (is_eq && eq_seen + lanes_below(eq_mask, lane) < need_eq);
                    const uint64_t take_mask = __ballot(take);
                    if (take) idx_row[out_pos + lanes_below(take_mask, lane)] = (m << 6) + lane;
                    eq_seen += __popcll(eq_mask);
                    out_pos += __popcll(take_mask);
                }
            }
            for (int t = out_pos + lane; t < T; t += 64) idx_row[t] = -1;
            if (lane == 0) cnt[row] = out_pos;
        }
    });
}

template <int D, int R, int MAXCH, bool EXT, int NWV, bool QPOOL>
__global__ __launch_bounds__(NWV * 64, 4) void score_topk_chunked_kernel(ScoreArgs a, int n_tiles) {
    extern __shared__ __attribute__((aligned(128))) float S[];   // [R][1024 + 8] scores of one column chunk, then the staged queries
    const int nwg = gridDim.x;
    int wg = blockIdx.x;
    if ((nwg & 7) == 0) wg = (wg & 7) * (nwg >> 3) + (wg >> 3);   // each XCD a contiguous slice, as in the plain kernel
    const int tile = n_tiles - 1 - wg % n_tiles;          // long rows first
    score_topk_rows_chunked<D, R, MAXCH, EXT, NWV, QPOOL>(a, wg / n_tiles, tile * R, S);
}

// Two workgroups per CU (4 wavefronts per SIMD): at most 128 registers, which is why the query
// operands are staged in LDS.
template <int D, int R, int MAXC, bool EXT, bool MASS, int NWV, bool QPOOL>
__global__ __launch_bounds__(NWV * 64, 4) void score_topk_mfma_kernel(ScoreArgs a, int n_tiles) {
    extern __shared__ __attribute__((aligned(128))) float S[];   // [R][LD] scores of this workgroup's rows, then 256 counters per wave
    // Workgroup ids go round robin over the 8 XCDs; give each XCD a contiguous slice of the
    // (b, head, row tile) order so that one L2 serves few KV heads and their Kp stays resident.
    const int nwg = gridDim.x;
    int wg = blockIdx.x;
    if ((nwg & 7) == 0) wg = (wg & 7) * (nwg >> 3) + (wg >> 3);
    const int tile = n_tiles - 1 - wg % n_tiles;          // long rows first
    score_topk_rows<D, R, MAXC, EXT, MASS, NWV, QPOOL>(a, wg / n_tiles, tile * R, S);
}

// Dynamic LDS above the default cap has to be requested per kernel and device.  That is done on the
// first launch of a (kernel, device) pair and remembered: later launches, also those recorded into a
// stream capture, make no runtime call besides the launch itself.
hipError_t allow_lds(const void* kernel, size_t bytes) {
    if (bytes <= 32768) return hipSuccess;
    struct Granted { const void* kernel; int device; size_t bytes; };
    static std::mutex mu;
    static std::vector<Granted> granted;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    for (Granted& g : granted)
        if (g.kernel == kernel && g.device == dev) {
            if (g.bytes >= bytes) return hipSuccess;
            e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e == hipSuccess) g.bytes = bytes;
            return e;
        }
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) granted.push_back(Granted{kernel, dev, bytes});
    return e;
}

ScoreArgs score_args(const Dims& d, const float* qp, const float* kp, const int32_t* k_rows, const int32_t* head_pattern,
                     const float* lvn, int32_t* idx, int32_t* cnt, float* scores_or_null, const void* q, Strides qs) {
    return ScoreArgs{qp, kp, d.Hq, d.G, d.NB, d.NBk, d.off, pattern_of(d), d.k, k_rows, head_pattern, lvn, d.T, d.scale,
                     idx, cnt, scores_or_null, d.gamma_q16 >= 0 ? (uint32_t)d.gamma_q16 : 0u, d.seq_lens, d.S, d.Bs, (const uint16_t*)q, qs};
}

size_t keys_lds_bytes(int NB) { return (size_t)kWaves * (((NB + 63) >> 6) << 6) * sizeof(uint32_t); }

}  // namespace

#define SPA_SCORE_TOPK_ARGS const Dims& d, const float* qp, const float* kp, const int32_t* k_rows, const int32_t* head_pattern, \
    const float* lvn, int32_t* idx, int32_t* cnt, float* scores_or_null, const void* q, Strides qs, hipStream_t st

#ifdef SPA_SELECT_D
namespace {
// one call of the score / top-k kernel
struct ScoreCall {
    const Dims& d;
    ScoreArgs a;
    hipStream_t st;
};

template <int D, int R, int MAXC, bool EXT, bool MASS, bool QPOOL, int NWV = (R * (MAXC * 64 + 8) * 4 > 80 * 1024 ? 16 : 8)>
hipError_t launch_mfma_e(const ScoreCall& c) {
    constexpr size_t part_words = 2 * (NWV / 4) * (256 / (D / 8)) * D;    // partial sums of the in-kernel pooling
    constexpr size_t lds = ((size_t)R * (MAXC * 64 + 8) + NWV * 256 +
                            (QPOOL && part_words > (size_t)R * (MAXC * 64 + 8) ? part_words : 0)) * sizeof(float);
    hipError_t e = allow_lds((const void*)score_topk_mfma_kernel<D, R, MAXC, EXT, MASS, NWV, QPOOL>, lds);
    if (e != hipSuccess) return e;
    const int n_tiles = (c.d.NB + R - 1) / R;
    dim3 grid((unsigned)(n_tiles * c.d.B * c.d.Hq));
    hipLaunchKernelGGL((score_topk_mfma_kernel<D, R, MAXC, EXT, MASS, NWV, QPOOL>), grid, dim3(NWV * 64), lds, c.st, c.a, n_tiles);
    return hipGetLastError();
}

template <int D, int R, int MAXC, bool EXT, bool MASS>
hipError_t launch_mfma_q(const ScoreCall& c) {
    if (c.a.q != nullptr) return launch_mfma_e<D, R, MAXC, EXT, MASS, true>(c);
    return launch_mfma_e<D, R, MAXC, EXT, MASS, false>(c);
}

template <int D, int MAXCH, bool EXT, bool QPOOL>
hipError_t launch_chunked_e(const ScoreCall& c) {
    constexpr int R = 16, NWV = 8;
    constexpr size_t lds = ((size_t)R * (1024 + 8) + NWV * 256) * sizeof(float);
    static_assert(2 * (NWV / 4) * (256 / (D / 8)) * D <= R * (1024 + 8), "the pooling partial sums fit the score space");
    hipError_t e = allow_lds((const void*)score_topk_chunked_kernel<D, R, MAXCH, EXT, NWV, QPOOL>, lds);
    if (e != hipSuccess) return e;
    const int n_tiles = (c.d.NB + R - 1) / R;
    dim3 grid((unsigned)(n_tiles * c.d.B * c.d.Hq));
    hipLaunchKernelGGL((score_topk_chunked_kernel<D, R, MAXCH, EXT, NWV, QPOOL>), grid, dim3(NWV * 64), lds, c.st, c.a, n_tiles);
    return hipGetLastError();
}

template <int D, int MAXCH>
hipError_t launch_chunked(const ScoreCall& c) {
    const bool qpool = c.a.q != nullptr;
    if (extended(c.d)) return qpool ? launch_chunked_e<D, MAXCH, true, true>(c) : launch_chunked_e<D, MAXCH, true, false>(c);
    return qpool ? launch_chunked_e<D, MAXCH, false, true>(c) : launch_chunked_e<D, MAXCH, false, false>(c);
}

template <int D, int R, int MAXC>
hipError_t launch_mfma(const ScoreCall& c) {
    const bool mass = c.d.gamma_q16 >= 0;
    if (extended(c.d)) return mass ? launch_mfma_q<D, R, MAXC, true, true>(c) : launch_mfma_q<D, R, MAXC, true, false>(c);
    return mass ? launch_mfma_q<D, R, MAXC, false, true>(c) : launch_mfma_q<D, R, MAXC, false, false>(c);
}

template <int D>
hipError_t launch_mfma_d(const ScoreCall& c) {
    // rows per workgroup shrink as rows get longer: up to 1024 blocks R * (NB padded) fp32 scores stay
    // within 66 KB of LDS, so that two 8-wave workgroups share a CU (measured at 131072 tokens:
    // 125 -> 106 us against 32 rows with one 8-wave workgroup per CU)
    const int NBk = c.d.NBk;
    // up to 512 blocks: 8 rows per workgroup give the chip more rounds of workgroups, so that one round's
    // streaming overlaps another's scoring (0.065 -> 0.062 ms at 32768 tokens, 0.135 -> 0.124 ms at 65536);
    // from 513 blocks 16 rows stay: 8 there re-read the pooled K twice as often (0.20 against 0.19 ms at 768
    // blocks, 0.29 against 0.26 ms at 1024)
    if (NBk <= 256) return launch_mfma<D, 8, 4>(c);
    if (NBk <= 512) return launch_mfma<D, 8, 8>(c);
    if (NBk <= 1024) return launch_mfma<D, 16, 16>(c);
    // 1025 .. 2048 blocks: 16 rows per workgroup with the columns scored in two chunks of 1024, still two
    // workgroups per CU (0.84 -> 0.78 ms at 262144 tokens against 8 rows scored in one pass, which is what a
    // mass budget still takes there)
    const bool chunked = c.d.gamma_q16 < 0;
    if (NBk <= 2048) return chunked ? launch_chunked<D, 2>(c) : launch_mfma<D, 8, 32>(c);
    return launch_mfma<D, 4, 64>(c);
}

}  // namespace

#define SPA_CAT2(a, b) a##b
#define SPA_CAT(a, b) SPA_CAT2(a, b)
hipError_t SPA_CAT(launch_score_topk_d, SPA_SELECT_D)(SPA_SCORE_TOPK_ARGS) {
    const ScoreCall c{d, score_args(d, qp, kp, k_rows, head_pattern, lvn, idx, cnt, scores_or_null, q, qs), st};
    return launch_mfma_d<SPA_SELECT_D>(c);
}

#else
hipError_t launch_score_topk_d128(SPA_SCORE_TOPK_ARGS);
hipError_t launch_score_topk_d64(SPA_SCORE_TOPK_ARGS);

hipError_t launch_topk_from_scores(const Dims& d, const float* scores, const int32_t* k_rows,
                                   const int32_t* head_pattern, int32_t* idx, int32_t* cnt, hipStream_t st) {
    int64_t n_rows = (int64_t)d.B * d.Hq * d.NB;
    unsigned grid = (unsigned)((n_rows + kWaves - 1) / kWaves);
    const void* fn = extended(d) ? (const void*)topk_from_scores_kernel<true> : (const void*)topk_from_scores_kernel<false>;
    const size_t lds = keys_lds_bytes(d.NBk) + (d.gamma_q16 >= 0 ? kWaves * 256 * sizeof(uint32_t) : 0);
    hipError_t e = allow_lds(fn, lds);
    if (e != hipSuccess) return e;
    if (extended(d))
        hipLaunchKernelGGL(topk_from_scores_kernel<true>, dim3(grid), dim3(kWaves * 64), lds, st,
                           scores, n_rows, d.NB, d.NBk, d.off, pattern_of(d), d.k, k_rows, head_pattern, d.Hq, d.T, idx, cnt, d.gamma_q16, d.seq_lens, d.S, d.Bs);
    else
        hipLaunchKernelGGL(topk_from_scores_kernel<false>, dim3(grid), dim3(kWaves * 64), lds, st,
                           scores, n_rows, d.NB, d.NBk, d.off, pattern_of(d), d.k, k_rows, head_pattern, d.Hq, d.T, idx, cnt, d.gamma_q16, d.seq_lens, d.S, d.Bs);
    return hipGetLastError();
}

hipError_t launch_score_topk(SPA_SCORE_TOPK_ARGS) {
    if (d.D == 128) return launch_score_topk_d128(d, qp, kp, k_rows, head_pattern, lvn, idx, cnt, scores_or_null, q, qs, st);
    if (d.D == 64) return launch_score_topk_d64(d, qp, kp, k_rows, head_pattern, lvn, idx, cnt, scores_or_null, q, qs, st);
    return hipErrorInvalidValue;
}
#endif

}  // namespace spa
