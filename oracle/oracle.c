/*
 * CPU oracle for block-sparse prefill attention.  TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call this file.  It shares no code with the HIP library and is deliberately
 * plain: straight loops, fp64 accumulation, no blocking, no fusion.
 *
 * What it computes follows the two-stage scheme of the paper's sparse
 * attention framework (Sec. 4.1.1, "A Versatile Library of Sparse Attention
 * Patterns": dynamic sparsity first does a pattern computation that locates
 * the sparse regions, then runs sparse attention on them), with
 *   - the static part of the mask = the "A-shape" pattern (attention sinks +
 *     a causal local window; Introduction and Sec. 4.1.1),
 *   - the dynamic part = the uniform top-k budget per query position that
 *     Sec. 4.1.2 describes as the common baseline (Fig. "Stem" (a)),
 *   - the union of both (the "hybrid of static patterns and dynamic token
 *     selection" of the abstract),
 *   - optionally the position-dependent budget of Stem's Token Position-Decay
 *     (Sec. 4.1.2, Fig. "Stem" (b)) in place of the uniform one; the schedule
 *     itself is an input, the paper prints none,
 *   - optionally the value-aware ranking score of Stem's Output-Aware Metric
 *     (Sec. 4.1.2, Fig. "Stem" (c)); reading stated at oracle_vnorm.
 * The paper gives no formula for any step.  The concrete readings taken here:
 * block granularity, arithmetic-mean pooling, raw pooled logit as the ranking
 * score, top-k drawn from the causal candidates that are not already static,
 * ties to the lowest block index, NaN ranked below every number, -0 == +0.
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py to
 * textbook special cases (dense causal attention via a library routine, brute
 * force masked softmax, closed forms, a full sort).  Against the paper itself
 * the whole pipeline is "parity unpinned": the paper prints no value for it.
 *
 * Layouts: all tensors contiguous.  Q [B,Hq,S,D], K/V [B,Hkv,S,D] as bf16 bit
 * patterns (uint16).  NB = ceil(S/Bs): the last block may be partial (it then
 * holds S - (NB-1)*Bs tokens; block means are taken over the tokens that exist,
 * and tokens past S neither attend nor are attended to).  T = min(NB, ns+nl+k).
 * KV prefix (chunked prefill): the queries may be the last Sq tokens of a
 * sequence of Skv = P + Sq tokens whose keys and values are all present, P a
 * multiple of Bs.  Query block i then sits at block position i + off, off = P/Bs,
 * of NBk = off + NBq key blocks; everything below is written for that case and
 * off = 0 is the plain one.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_f64(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Step 1 (pattern computation, pooling): xp[n,i,d] = mean over the Bs tokens
 * of block i of x[n,i*Bs+t,d].  fp64 sum, one rounding to fp32 on export.
 * x: [n_heads_total, S, D] bf16; xp: [n_heads_total, NB, D] fp32. */
int oracle_pool(const uint16_t *x, int64_t n_heads_total, int64_t S, int64_t D,
                int64_t Bs, float *xp) {
    if (Bs <= 0 || S <= 0) return -1;
    int64_t NB = (S + Bs - 1) / Bs;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < n_heads_total; ++n)
        for (int64_t i = 0; i < NB; ++i)
            for (int64_t d = 0; d < D; ++d) {
                int64_t len = S - i * Bs < Bs ? S - i * Bs : Bs;   /* tokens of block i */
                double acc = 0.0;
                for (int64_t t = 0; t < len; ++t)
                    acc += bf16_to_f64(x[(n * S + i * Bs + t) * D + d]);
                xp[(n * NB + i) * D + d] = (float)(acc / (double)len);
            }
    return 0;
}

/* Step 2 (pattern computation, scoring): sp[b,h,i,j] = scale * <qp[b,h,i,:],
 * kp[b,h/G,j,:]> for j <= i + off, from the fp32 pooled values, fp64 accumulate,
 * one rounding to fp32.  Entries with j > i + off are set to -inf.
 * qp [B,Hq,NBq,D], kp [B,Hkv,NBk,D], sp [B,Hq,NBq,NBk], off = NBk - NBq. */
int oracle_scores(const float *qp, const float *kp, int64_t B, int64_t Hq,
                  int64_t Hkv, int64_t NBq, int64_t NBk, int64_t D, float scale, float *sp) {
    if (Hkv <= 0 || Hq % Hkv || NBk < NBq) return -1;
    int64_t G = Hq / Hkv, off = NBk - NBq;
#pragma omp parallel for collapse(3) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < Hq; ++h)
            for (int64_t i = 0; i < NBq; ++i) {
                const float *qrow = qp + ((b * Hq + h) * NBq + i) * D;
                float *srow = sp + ((b * Hq + h) * NBq + i) * NBk;
                for (int64_t j = 0; j < NBk; ++j) {
                    if (j > i + off) { srow[j] = -INFINITY; continue; }
                    const float *krow = kp + ((b * Hkv + h / G) * NBk + j) * D;
                    double acc = 0.0;
                    for (int64_t d = 0; d < D; ++d)
                        acc += (double)qrow[d] * (double)krow[d];
                    srow[j] = (float)((double)scale * acc);
                }
            }
    return 0;
}

/* Output-aware ranking score (Stem's Output-Aware Metric, Sec. 4.1.2, Fig.
 * "Stem" (c): the selection metric combines the attention score with the
 * magnitude of the value vectors, so a block whose values are weak is less
 * likely to be kept).  The paper prints no formula.  Reading taken here: a key
 * block's contribution to the output is its attention weight times the size
 * of its values, which in the logit domain is a sum:
 *   vn[n,j]  = (1/Bs) sum_t || V[n, j*Bs+t, :] ||_2        (fp64, rounded to fp32)
 *   sp'[b,h,i,j] = sp[b,h,i,j] + ln vn[b,h/G,j]             (j <= i)
 * from the fp32 score and fp32 vn, added in fp64, rounded once to fp32.  A
 * block of all-zero values gets -inf.  oracle_vnorm computes vn,
 * oracle_scores_oam applies the second line in place. */
int oracle_vnorm(const uint16_t *v, int64_t n_heads_total, int64_t S, int64_t D,
                 int64_t Bs, float *vn) {
    if (Bs <= 0 || S <= 0) return -1;
    int64_t NB = (S + Bs - 1) / Bs;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < n_heads_total; ++n)
        for (int64_t j = 0; j < NB; ++j) {
            int64_t len = S - j * Bs < Bs ? S - j * Bs : Bs;
            double acc = 0.0;
            for (int64_t t = 0; t < len; ++t) {
                double sq = 0.0;
                for (int64_t d = 0; d < D; ++d) {
                    double x = bf16_to_f64(v[(n * S + j * Bs + t) * D + d]);
                    sq += x * x;
                }
                acc += sqrt(sq);
            }
            vn[n * NB + j] = (float)(acc / (double)len);
        }
    return 0;
}

int oracle_scores_oam(float *sp, const float *vn, int64_t B, int64_t Hq, int64_t Hkv,
                      int64_t NBq, int64_t NBk) {
    if (Hkv <= 0 || Hq % Hkv || NBk < NBq) return -1;
    int64_t G = Hq / Hkv, off = NBk - NBq;
#pragma omp parallel for collapse(3) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < Hq; ++h)
            for (int64_t i = 0; i < NBq; ++i) {
                float *srow = sp + ((b * Hq + h) * NBq + i) * NBk;
                const float *vrow = vn + (b * Hkv + h / G) * NBk;
                for (int64_t j = 0; j <= i + off; ++j)
                    srow[j] = (float)((double)srow[j] + log((double)vrow[j]));
            }
    return 0;
}

/* Ranking order of two candidates: larger score first; equal scores (and
 * -0 vs +0) by lower block index; NaN after every number. */
static int ranks_before(float sa, int64_t ja, float sb, int64_t jb) {
    int na = isnan(sa), nb = isnan(sb);
    if (na != nb) return nb;
    if (!na && sa != sb) return sa > sb;
    return ja < jb;
}

/* Steps 3+4 (top-k and merge with the static pattern) for every query block:
 *   Static_i = {j < ns, j <= i} U {max(0,i-nl+1) .. i}   (A-shape; more below)
 *   C_i      = {0..i} \ Static_i
 *   TopK_i   = the min(k_i,|C_i|) best-ranked members of C_i
 *   Sel_i    = Static_i U TopK_i, written ascending, padded with -1.
 * Budget k_i: the uniform budget k for every query block (the baseline of
 * Sec. 4.1.2, Fig. "Stem" (a)) when k_row is NULL; otherwise the position
 * dependent budget of Token Position-Decay (Sec. 4.1.2, Fig. "Stem" (b)):
 * k_i = k_row[i] clamped to [0, k], one value per query block, shared by all
 * heads.  The paper prints no decay schedule, so the schedule is an input.
 * Further static patterns of the library (Sec. 4.1.1 names A-shape, Tri-shape,
 * Dilated and Strided; none is given a formula, readings at block level):
 *   stride > 0  (Strided): also static are the blocks j with (i - j) % stride == 0,
 *                          every stride-th block back from the diagonal;
 *   reach > 0   (Dilated): ... but only those closer than reach blocks, i - j < reach:
 *                          a local window of reach/stride blocks with gaps (dilation = stride);
 *   n_dense > 0 (Tri-shape): the last n_dense query blocks attend to every
 *                          causal block (A-shape plus a dense bottom strip).
 * Per-head configuration (Sec. 4.1.1, "Decoupling Sparse Kernels from Model
 * Architectures": the settings are metadata applied to specific heads): with
 * head_pattern != NULL query head h = n % Hq uses its own triple
 *   (ns_h, nl_h, k_h) = head_pattern[3h .. 3h+2] clamped to [0,ns], [1,nl], [0,k];
 * ns, nl, k are then the stated maxima (they fix T); a budget schedule is
 * capped per head: k_{i,h} = min(k_row[i] clamped to [0,k], k_h).
 * sp: [n_rows_total = B*Hq, NB, NB] fp32; idx: [B*Hq, NB, T]; cnt: [B*Hq, NB];
 * T = oracle_row_capacity(...): min(NB, ns+nl+k+floor((NB-1)/stride)), or NB with
 * a dense strip; with a schedule k is its stated maximum. */
int64_t oracle_row_capacity(int64_t NB, int64_t ns, int64_t nl, int64_t k, int64_t stride,
                            int64_t n_dense, int64_t reach) {
    if (n_dense > 0) return NB;
    int64_t far = NB - 1;                       /* largest distance i - j of a strided block */
    if (reach > 0 && reach - 1 < far) far = reach - 1;
    int64_t T = ns + nl + k + (stride > 0 ? far / stride : 0);
    return T < NB ? T : NB;
}

static int64_t clamp64(int64_t x, int64_t lo, int64_t hi) { return x < lo ? lo : (x > hi ? hi : x); }

/* Cumulative-mass budget (the rule of the FlexPrefill family, which Sec. 4.1.1 lists among the
 * dynamic algorithms of the framework and Sec. 4.1.2 under "Other Sparse Attention Strategies";
 * the paper gives no formula).  Reading: a query block keeps, in ranking order, the fewest
 * candidates for which the selected blocks (static ones included) hold at least the fraction
 * gamma of the row's block-level softmax mass, and never more than its count budget.
 *
 * A floating-point sum would decide an integer here (how many blocks), so the mass is DEFINED in
 * integer arithmetic, which any implementation can reproduce bit for bit whatever its order of
 * summation.  For the causal blocks j <= i of a row with ranking scores x_j (fp32):
 *   m   = max_j x_j over the scores that are not NaN
 *   W_j = mass_weight(x_j, m), an integer in [0, 2^19] ~ 2^19 exp(x_j - m), see below
 *   Z   = sum_j W_j;  Gamma = floor(gamma * 65536 + 0.5) (gamma clamped to [0, 1])
 *   target = ceil(Gamma * Z / 65536)
 * and the row takes candidates in ranking order until mass(static) + mass(taken) >= target.
 *
 * mass_weight: every step is a single IEEE fp32 operation (no contraction), so the result does
 * not depend on the machine: t = (x - m) * log2(e); n = nearest integer to t (ties to even);
 * f = t - n in [-1/2, 1/2]; 2^f by the degree-6 Taylor polynomial of e^(f ln 2) in Horner form
 * with fused multiply-adds (truncation error < 1.3e-7); w = that times 2^n; W = floor(w * 2^19 + 1/2).
 * NaN and -inf scores, and anything more than 2^-40 below the maximum, weigh 0. */
static uint32_t mass_weight(float x, float m) {
    if (isnan(x) || isnan(m)) return 0u;
    if (x == m) return 1u << 19;                 /* also covers m = +inf */
    if (isinf(x) || isinf(m)) return 0u;         /* x = -inf, or finite x under m = +inf */
    const float t = (x - m) * 1.44269504088896340736f;
    if (!(t >= -40.0f)) return 0u;
    const float n = rintf(t);
    const float f = t - n;
    float p = 1.5403530393381609954e-4f;
    p = fmaf(p, f, 1.3333558146428443423e-3f);
    p = fmaf(p, f, 9.6181291076284771619e-3f);
    p = fmaf(p, f, 5.5504108664821579953e-2f);
    p = fmaf(p, f, 2.4022650695910071233e-1f);
    p = fmaf(p, f, 6.9314718055994530942e-1f);
    p = fmaf(p, f, 1.0f);
    const float w = ldexpf(p, (int)n);
    return (uint32_t)(w * 524288.0f + 0.5f);
}

/* The weights alone, for the tests: W [n_rows_total, NBq, NBk] uint32 (0 beyond the causal limit). */
int oracle_mass_weights(const float *sp, int64_t n_heads_total, int64_t NBq, int64_t NBk, uint32_t *W) {
    if (NBk < NBq) return -1;
    const int64_t off = NBk - NBq;
    for (int64_t r = 0; r < n_heads_total * NBq; ++r) {
        const int64_t i = r % NBq + off;
        const float *srow = sp + r * NBk;
        float m = -INFINITY;
        for (int64_t j = 0; j <= i; ++j)
            if (!isnan(srow[j]) && srow[j] > m) m = srow[j];
        for (int64_t j = 0; j < NBk; ++j) W[r * NBk + j] = j <= i ? mass_weight(srow[j], m) : 0u;
    }
    return 0;
}

int oracle_topk_mass(const float *sp, int64_t n_heads_total, int64_t NBq, int64_t NBk, int64_t ns_max,
                     int64_t nl_max, int64_t k_max, const int32_t *k_row, int64_t stride,
                     int64_t n_dense, int64_t reach, const int32_t *head_pattern, int64_t Hq,
                     double gamma, int32_t *idx, int32_t *cnt);

int oracle_topk(const float *sp, int64_t n_heads_total, int64_t NBq, int64_t NBk, int64_t ns_max,
                int64_t nl_max, int64_t k_max, const int32_t *k_row, int64_t stride,
                int64_t n_dense, int64_t reach, const int32_t *head_pattern, int64_t Hq,
                int32_t *idx, int32_t *cnt) {
    return oracle_topk_mass(sp, n_heads_total, NBq, NBk, ns_max, nl_max, k_max, k_row, stride, n_dense, reach,
                            head_pattern, Hq, -1.0, idx, cnt);
}

/* gamma < 0: count budgets only (oracle_topk); gamma in [0, 1]: the cumulative-mass budget on top. */
int oracle_topk_mass(const float *sp, int64_t n_heads_total, int64_t NBq, int64_t NBk, int64_t ns_max,
                     int64_t nl_max, int64_t k_max, const int32_t *k_row, int64_t stride,
                     int64_t n_dense, int64_t reach, const int32_t *head_pattern, int64_t Hq,
                     double gamma, int32_t *idx, int32_t *cnt) {
    if (ns_max < 0 || nl_max < 1 || k_max < 0 || stride < 0 || n_dense < 0 || reach < 0) return -1;
    if (gamma > 1.0) gamma = 1.0;
    const int use_mass = gamma >= 0.0;
    const uint64_t Gamma = use_mass ? (uint64_t)floor(gamma * 65536.0 + 0.5) : 0;
    if (head_pattern && Hq < 1) return -1;
    if (NBk < NBq) return -1;
    const int64_t ns0 = ns_max, nl0 = nl_max, k0 = k_max, off = NBk - NBq;
    int64_t T = oracle_row_capacity(NBk, ns0, nl0, k0, stride, n_dense, reach);
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int64_t n = 0; n < n_heads_total; ++n)
        for (int64_t iq = 0; iq < NBq; ++iq) {
            const int64_t i = iq + off;           /* block position of query block iq in the sequence */
            const float *srow = sp + (n * NBq + iq) * NBk;
            int32_t *orow = idx + (n * NBq + iq) * T;
            int64_t ns = ns0, nl = nl0, k = k0;
            if (head_pattern) {
                const int32_t *hp = head_pattern + 3 * (n % Hq);
                ns = clamp64(hp[0], 0, ns0);
                nl = clamp64(hp[1], 1, nl0);
                k = clamp64(hp[2], 0, k0);
            }
            /* state[j]: 0 = candidate, 1 = selected */
            unsigned char *sel = (unsigned char *)calloc((size_t)NBk, 1);
            if (!sel) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            for (int64_t j = 0; j <= i; ++j) {
                int is_sink = j < ns;
                int is_local = j >= i - nl + 1;
                int is_strided = stride > 0 && (i - j) % stride == 0 && (reach == 0 || i - j < reach);
                int is_dense_row = i >= NBk - n_dense;
                sel[j] = (unsigned char)(is_sink || is_local || is_strided || is_dense_row);
            }
            int64_t k_i = k;
            if (k_row) {                          /* one entry per query block of this call */
                k_i = clamp64(k_row[iq], 0, k0);
                if (k_i > k) k_i = k;
            }
            uint64_t have = 0, target = 0;        /* mass selected so far, mass wanted */
            float m = -INFINITY;
            if (use_mass) {
                uint64_t Z = 0;
                for (int64_t j = 0; j <= i; ++j)
                    if (!isnan(srow[j]) && srow[j] > m) m = srow[j];
                for (int64_t j = 0; j <= i; ++j) {
                    const uint64_t w = mass_weight(srow[j], m);
                    Z += w;
                    if (sel[j]) have += w;
                }
                target = (Gamma * Z + 65535) >> 16;
            }
            for (int64_t pick = 0; pick < k_i; ++pick) {
                if (use_mass && have >= target) break;   /* the mass budget is met */
                int64_t best = -1;
                for (int64_t j = 0; j <= i; ++j) {
                    if (sel[j]) continue;
                    if (best < 0 || ranks_before(srow[j], j, srow[best], best)) best = j;
                }
                if (best < 0) break; /* candidates exhausted */
                sel[best] = 1;
                if (use_mass) have += mass_weight(srow[best], m);
            }
            int64_t c = 0;
            for (int64_t j = 0; j <= i; ++j)
                if (sel[j]) orow[c++] = (int32_t)j;
            cnt[n * NBq + iq] = (int32_t)c;
            for (; c < T; ++c) orow[c] = -1;
            free(sel);
        }
    return fail ? -2 : 0;
}

/* Step 5 (sparse attention on the located regions).  For query token t in
 * block i (sequence position P + t with a KV prefix of P tokens):
 * keys = { s : s/Bs in Sel_i, s <= P + t }, logits x_s = scale * q_t.k_s,
 * m = max x_s, p_s = exp(x_s - m), out_t = sum p_s v_s / sum p_s,
 * lse_t = m + log sum p_s.  Everything in fp64; results rounded once to fp32.
 *
 * rows: optional [n_rows,3] list of (b,h,i) query blocks to compute; NULL means
 * all of them in (b,h,i) order, so out is then laid out [B,Hq,S,D].
 * out: [n_rows, Bs, D] fp32; lse: [n_rows, Bs] fp32 (may be NULL). */
int oracle_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                int64_t B, int64_t Hq, int64_t Hkv, int64_t S, int64_t Skv, int64_t D,
                int64_t Bs, int64_t T, float scale, const int32_t *idx,
                const int32_t *cnt, const int32_t *rows, int64_t n_rows,
                float *out, float *lse) {
    if (Hkv <= 0 || Hq % Hkv || Bs <= 0 || S <= 0 || Skv < S || (Skv - S) % Bs) return -1;
    /* S query tokens = the last S of Skv; P = Skv - S tokens of KV prefix */
    int64_t G = Hq / Hkv, NB = (S + Bs - 1) / Bs, P = Skv - S;
    if (!rows) n_rows = B * Hq * NB;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int64_t r = 0; r < n_rows; ++r)
        for (int64_t tq = 0; tq < Bs; ++tq) {
            int64_t b, h, i;
            if (rows) { b = rows[3 * r]; h = rows[3 * r + 1]; i = rows[3 * r + 2]; }
            else { b = r / (Hq * NB); h = (r / NB) % Hq; i = r % NB; }
            int64_t t = i * Bs + tq;
            /* with rows == NULL the output is [B,Hq,S,D]; with a list it is [n_rows,Bs,D] */
            int64_t orow_idx = rows ? r * Bs + tq : (b * Hq + h) * S + t;
            if (t >= S) {                      /* token past the end of a partial last block */
                if (rows) {
                    for (int64_t d = 0; d < D; ++d) out[orow_idx * D + d] = 0.0f;
                    if (lse) lse[orow_idx] = 0.0f;
                }
                continue;
            }
            const uint16_t *qt = q + ((b * Hq + h) * S + t) * D;
            const uint16_t *kh = k + ((b * Hkv + h / G) * Skv) * D;
            const uint16_t *vh = v + ((b * Hkv + h / G) * Skv) * D;
            const int32_t *sel = idx + ((b * Hq + h) * NB + i) * T;
            int64_t c = cnt[(b * Hq + h) * NB + i];
            double *x = (double *)malloc(sizeof(double) * (size_t)(c * Bs + 1));
            int64_t *key = (int64_t *)malloc(sizeof(int64_t) * (size_t)(c * Bs + 1));
            double *acc = (double *)calloc((size_t)D, sizeof(double));
            if (!x || !key || !acc) {
#pragma omp atomic write
                fail = 1;
                free(x); free(key); free(acc);
                continue;
            }
            int64_t n = 0;
            for (int64_t e = 0; e < c; ++e)
                for (int64_t u = 0; u < Bs; ++u) {
                    int64_t s = (int64_t)sel[e] * Bs + u;
                    if (s > P + t) continue; /* causal; P + t < Skv, so keys past the end never pass */
                    double dot = 0.0;
                    for (int64_t d = 0; d < D; ++d)
                        dot += bf16_to_f64(qt[d]) * bf16_to_f64(kh[s * D + d]);
                    x[n] = (double)scale * dot;
                    key[n] = s;
                    ++n;
                }
            double m = -INFINITY;
            for (int64_t e = 0; e < n; ++e) if (x[e] > m) m = x[e];
            double l = 0.0;
            for (int64_t e = 0; e < n; ++e) {
                double p = exp(x[e] - m);
                l += p;
                for (int64_t d = 0; d < D; ++d)
                    acc[d] += p * bf16_to_f64(vh[key[e] * D + d]);
            }
            float *orow = out + orow_idx * D;
            for (int64_t d = 0; d < D; ++d) orow[d] = (float)(acc[d] / l);
            if (lse) lse[orow_idx] = (float)(m + log(l));
            free(x); free(key); free(acc);
        }
    return fail ? -2 : 0;
}

int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
