/*
 * sparse_prefill.h — C ABI of the MI355X (gfx950) block-sparse prefill
 * attention library.
 *
 * The library implements the hot path of the training-free sparse attention
 * framework of the AngelSlim technical report (arXiv 2602.21233, Sec. 4.1):
 * long-context prefill attention ("KV Cache Generation stage", Sec. 4.1) over
 * a block mask that unites
 *   - a static pattern: the "A-shape" of Sec. 4.1.1 (attention-sink blocks plus
 *     a causal local window), and
 *   - a dynamic pattern: per query block, the top-k key blocks under a uniform
 *     budget (the baseline scheme of Sec. 4.1.2 / Fig. "Stem" (a)), ranked by
 *     the scaled dot product of block-mean-pooled queries and keys,
 * followed by online-softmax attention that visits only the selected blocks.
 * The two stages are the paper's "pattern computation" and "sparse attention
 * kernel" (Sec. 4.1.1, dynamic sparsity).
 *
 * Conventions (all entry points)
 *   - `p` is a HOST pointer.  Every other pointer is a DEVICE pointer into
 *     memory the CALLER owns; the library never allocates, frees or
 *     synchronises.  All work is enqueued on `hip_stream` (a hipStream_t passed
 *     as void*, NULL = the default stream) and completes asynchronously.
 *   - Q is [batch, n_q_heads, seq_len, head_dim], K and V are
 *     [batch, n_kv_heads, kv_prefix_len + seq_len, head_dim], OUT has Q's shape; bf16.  The
 *     strides (in elements) of the batch, head and token axes come from
 *     `*_stride`; the head_dim axis is contiguous.  Base pointers must be
 *     16-byte aligned and every stride a multiple of 8 elements.
 *     Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - NB = ceil(seq_len / block_size) query blocks and key blocks; seq_len need not be a
 *     multiple of block_size: the last block is then partial, block means are taken over
 *     the tokens that exist and nothing is read or written past seq_len.  Row capacity
 *     T = min(NB, n_sink_blocks + n_local_blocks + top_k_blocks
 *                 + (stride_blocks > 0 ? min(NB - 1, reach - 1) / stride_blocks : 0)),
 *     reach = stride_reach_blocks or NB when that is 0,
 *     or NB when n_dense_q_blocks > 0 (spa_row_capacity returns it).  With a KV prefix
 *     (kv_prefix_len > 0) the key blocks number NBk = kv_prefix_len / block_size + NB and
 *     NBk takes the place of NB in T; block_idx keeps NB rows.
 *   - block_idx is [batch, n_q_heads, NB, T] int32, contiguous: for query
 *     block i the selected key blocks in ascending order, then -1 padding.
 *     block_cnt is [batch, n_q_heads, NB] int32: the number of valid entries:
 *     the row's static blocks plus min(top_k, causal blocks that are not static)
 *     (for the plain A-shape that is min(i + 1, n_sink + n_local + top_k); with a
 *     budget schedule: top_k of that row); the last valid entry is always i (the
 *     diagonal block).
 *   - Return value: SPA_OK (0) or a negative SPA_ERR_* code.  Arguments are
 *     validated on the host before anything is enqueued, so a failed call has
 *     no effect on the device.  Results are deterministic run to run.
 */
#ifndef SPARSE_PREFILL_H
#define SPARSE_PREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SPA_OK = 0,
    SPA_ERR_NULLPTR = -1,             /* a required pointer is NULL                         */
    SPA_ERR_BAD_SHAPE = -2,           /* unsupported sizes, see spa_params                  */
    SPA_ERR_BAD_PATTERN = -3,         /* n_sink < 0, n_local < 1, a negative top_k, stride, reach or
                                         n_dense, lists_per_kv_head not 0 or 1               */
    SPA_ERR_BAD_STRIDE = -4,          /* stride not a multiple of 8 / pointer not 16-B aligned */
    SPA_ERR_WORKSPACE_TOO_SMALL = -5, /* ws_bytes < spa_workspace_bytes()                   */
    SPA_ERR_LAUNCH = -6,              /* the HIP runtime rejected a launch                  */
    SPA_ERR_STATIC_SCRATCH_TOO_SMALL = -7 /* sparse_prefill_select_static: the call needs more than
                                         SPA_STATIC_SCRATCH_BYTES of scratch                 */
};

typedef struct spa_params {
    int32_t batch;          /* >= 1                                                   */
    int32_t n_q_heads;      /* >= 1, multiple of n_kv_heads                           */
    int32_t n_kv_heads;     /* >= 1                                                   */
    int32_t seq_len;        /* >= 1 query tokens; at most 4096 key blocks (see kv_prefix_len) */
    int32_t head_dim;       /* 64 or 128                                              */
    int32_t block_size;     /* 64 or 128 tokens                                       */
    int32_t n_sink_blocks;  /* >= 0: key blocks 0 .. n_sink-1 are always selected     */
    int32_t n_local_blocks; /* >= 1: key blocks i-n_local+1 .. i (the diagonal counts)*/
    int32_t top_k_blocks;   /* >= 0: budget drawn from the causal blocks that are not
                               already static; fewer if fewer exist                   */
    float softmax_scale;    /* 0 selects 1/sqrt(head_dim)                             */
    int64_t q_stride[3];    /* elements: batch, head, token                           */
    int64_t k_stride[3];
    int64_t v_stride[3];
    int64_t o_stride[3];
    /* Further static patterns of the library (Sec. 4.1.1 names A-shape, Tri-shape, Dilated and
     * Strided; readings at block level).  All three 0 for the plain A-shape.                 */
    int32_t stride_blocks;    /* >= 0.  s > 0 (Strided): key blocks j with (i - j) % s == 0 are
                                 static too, every s-th block back from the diagonal          */
    int32_t n_dense_q_blocks; /* >= 0.  n > 0 (Tri-shape): the last n query blocks attend to
                                 every causal block                                           */
    int32_t stride_reach_blocks; /* >= 0.  r > 0 (Dilated): the strided blocks count only while
                                 i - j < r, i.e. a local window of r / s blocks with dilation s;
                                 0 = the whole sequence.  Ignored when stride_blocks == 0     */
    int32_t kv_prefix_len;    /* >= 0, multiple of block_size.  P > 0 (chunked prefill): K and V hold
                                 P + seq_len tokens and the seq_len queries are the last of them.
                                 Query block i then has block position i + P / block_size among
                                 NBk = P / block_size + NB key blocks: the causal limit, the static
                                 pattern, the row capacity (with NBk in place of NB) and the key
                                 axis of the score output refer to those positions; block_idx and
                                 block_cnt keep one row per query block of the call, and a budget
                                 schedule one entry per query block of the call.  NBk <= 4096     */
    int32_t lists_per_kv_head; /* 0 or 1.  1 (group-shared selection): one list per KV head, shared
                                 by the n_q_heads / n_kv_heads query heads of its group; the group
                                 is ranked by the mean of its heads' pooled scores.  block_idx,
                                 block_cnt and the optional scores then have n_kv_heads in their
                                 head axis (also for sparse_prefill_attn and, per KV head, for
                                 spa_select_opts.head_pattern).  The heads of a group then walk the
                                 same key blocks at the same time, which the L2 turns into reuse */
    const int32_t *seq_lens;   /* NULL, or a DEVICE array of `batch` int32 (ragged batch): entry b has
                                 seq_lens[b] query tokens (clamped to [0, seq_len]) and kv_prefix_len +
                                 seq_lens[b] key tokens; the tensors keep their padded shapes and
                                 strides, seq_len stays the padded length that fixes NB and T.  Entry b
                                 is processed exactly as a batch-1 call of its own length would be
                                 (its last block may be partial; a Tri-shape strip means the entry's
                                 own last query blocks).  Rows of block_idx / block_cnt past an entry's
                                 last block get count 0 and -1 entries; tokens past an entry's length
                                 are not read, and their out / lse / pooled / score entries are not
                                 written                                                          */
} spa_params;

/* Human-readable text for a return code.  Never NULL. */
const char *spa_strerror(int code);

/* Row capacity T of block_idx for these parameters.  Host only. */
int spa_row_capacity(const spa_params *p, int32_t *row_capacity);

/* Bytes of device scratch that the select, attn and fused calls (all variants)
 * need in `ws` (pooled Q and K; the block lists of a fused call whose caller
 * does not ask for them; the value norms of the output-aware calls; a per-block
 * transposed copy of V).  One size serves every call.
 * Host only. */
int spa_workspace_bytes(const spa_params *p, size_t *bytes);

/* Pattern computation, step 1 (Sec. 4.1.1): block mean pooling.
 *   q_pooled[b,h,i,:] = mean over the block's tokens of Q[b,h,i*Bs+t,:]   (fp32)
 *   k_pooled likewise.  q_pooled is [batch, n_q_heads, NB, head_dim] and
 *   k_pooled [batch, n_kv_heads, NBk, head_dim] (NBk = NB without a KV prefix),
 *   contiguous fp32; a partial last block is averaged over the tokens it has.
 * Either of (q, q_pooled) or (k, k_pooled) may be NULL as a pair to skip it. */
int sparse_prefill_pool(const spa_params *p, const void *q, const void *k,
                        float *q_pooled, float *k_pooled, void *hip_stream);

/* Pattern computation, all steps (Sec. 4.1.1 dynamic sparsity; budget rule of
 * Sec. 4.1.2 Fig. "Stem" (a); static A-shape of Sec. 4.1.1): pool Q and K,
 * score every causal (query block, key block) pair with
 *   score[b,h,i,j] = scale * <q_pooled[b,h,i,:], k_pooled[b,h/G,j,:]>   (fp32),
 * take per row the top_k_blocks best non-static causal blocks (ties: lowest
 * block index; NaN ranks below every number; -0 equals +0) and unite them with
 * the static blocks.  Writes block_idx / block_cnt.
 * pooled_scores_or_null: if not NULL, [batch, n_q_heads, NB, NBk] fp32 receives
 * the scores (entries beyond the causal limit, j > i + NBk - NB, are written as
 * -inf; NBk = NB without a KV prefix).
 * ws: spa_workspace_bytes() bytes of scratch, 256-byte aligned. */
int sparse_prefill_select(const spa_params *p, const void *q, const void *k,
                          int32_t *block_idx, int32_t *block_cnt,
                          float *pooled_scores_or_null, void *ws, size_t ws_bytes,
                          void *hip_stream);

/* sparse_prefill_select for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * computation, same outputs and same checks as sparse_prefill_select, bit for bit, but the scratch
 * of the stage (the pooled K in the score kernel's layout; with lists_per_kv_head also the pooled
 * queries and their group means) lives in a static device array inside the library instead of
 * `ws`: SPA_STATIC_SCRATCH_BYTES per GPU the library is used on, held until the process ends.  The
 * call allocates and frees nothing and enqueues only kernels on hip_stream.
 *   - Limit: 256-byte-aligned regions of
 *       batch * n_kv_heads * 32 * ceil(NBk / 32) * head_dim * 4 bytes,
 *     plus, with lists_per_kv_head, batch * (n_q_heads + n_kv_heads) * NB * head_dim * 4 bytes,
 *     must fit SPA_STATIC_SCRATCH_BYTES (8 MiB: e.g. 8 KV heads x 2048 key blocks x head_dim 128,
 *     the 262144-token workload); beyond it the call returns SPA_ERR_STATIC_SCRATCH_TOO_SMALL and
 *     enqueues nothing.
 *   - Every call on a GPU shares that GPU's one array: calls that overlap in time on the same GPU
 *     (different streams, or threads) race on it and give unspecified lists; serialise them.  The
 *     array keeps the previous call's contents; nothing in it has to start at zero (the stage reads
 *     only what it has written in the same call, stale parts feed columns that are never ranked).
 *   - The array's address is looked up once per device, on the first call made with that device
 *     current (a runtime query, no allocation); make that first call outside stream capture. */
#define SPA_STATIC_SCRATCH_BYTES (8u << 20)
int sparse_prefill_select_static(const spa_params *p, const void *q, const void *k,
                                 int32_t *block_idx, int32_t *block_cnt,
                                 float *pooled_scores_or_null, void *hip_stream);

/* The top-k + static-merge step alone, on caller-supplied scores
 * [batch, n_q_heads, NB, NBk] fp32 (entries beyond the causal limit are ignored).  Given the
 * same scores this produces the same lists as sparse_prefill_select, bit for
 * bit.  Uses of p: shape, pattern. */
int sparse_prefill_topk_from_scores(const spa_params *p, const float *pooled_scores,
                                    int32_t *block_idx, int32_t *block_cnt,
                                    void *hip_stream);

/* Sparse attention kernel (Sec. 4.1.1): for query token t of block i,
 *   out[t] = softmax over { s <= t : block(s) in block_idx[b,h,i,:cnt] } of
 *            scale * q_t . k_s, applied to v_s     (s, t counted from the start of K/V),
 * bf16 MFMA with fp32 accumulation and fp32 online softmax; out is bf16.
 * lse_or_null: if not NULL, [batch, n_q_heads, seq_len] fp32 receives the
 * natural-log sum of exponentials of the scaled logits of each row.
 * block_idx / block_cnt must satisfy the layout rules at the top of this file
 * (ascending, unique, 0 <= entry <= i, last valid entry == i, 1 <= cnt <= T);
 * lists produced by the select calls always do.  They are not validated: a count outside
 * [1, T] or a block outside [0, NBk) is clamped, so a malformed list cannot make the kernel read
 * outside the tensors, but the output of such a row is unspecified
 * (sparse_prefill_check_lists counts the rows that break the rules).
 * Of p this call uses the shape, strides and scale; the pattern fields fix T and
 * serve as a hint of how uneven the rows are (a dense strip or strided columns
 * make the library deal the query blocks to the chip's partitions one by one).
 * ws: spa_workspace_bytes() bytes of scratch, 256-byte aligned; its contents
 * need not survive between calls. */
int sparse_prefill_attn(const spa_params *p, const void *q, const void *k, const void *v,
                        const int32_t *block_idx, const int32_t *block_cnt,
                        void *out, float *lse_or_null, void *ws, size_t ws_bytes,
                        void *hip_stream);

/* The attention kernel reads V transposed per key block (both of its matrix-core operands are then
 * plain 16-byte reads of the staged tile): sparse_prefill_attn makes that copy in `ws` on every
 * call.  A caller that keeps the copy itself, e.g. beside V in its KV cache, so that a chunked
 * prefill (Sec. 4.1: the KV cache generation stage; kv_prefix_len > 0) does not transpose the
 * whole prefix again for every chunk, uses these two calls instead; sparse_prefill_attn is exactly
 * transpose_v of all key blocks into `ws` followed by attn_vt.
 *   vt: [batch, n_kv_heads, vt_blocks_per_head, head_dim, block_size] bf16, contiguous, 16-byte
 *       aligned; vt_blocks_per_head >= NBk (the key blocks of this call; room to grow).  Block j of
 *       (b, kv head) holds V[b, kv head, j*Bs + t, d] at [d, t]; tokens past the end of a partial
 *       last block are zeros.
 * sparse_prefill_transpose_v fills the blocks first_block .. first_block + n_blocks - 1 (0 <=
 *   first_block, first_block + n_blocks <= NBk, else SPA_ERR_BAD_SHAPE; n_blocks = 0 is a no-op)
 *   from V in the layout of p->v_stride; a block that was partial when it was last written has to
 *   be written again once it has more tokens.  Uses of p: shape, kv_prefix_len, seq_lens, v_stride.
 * sparse_prefill_attn_vt is sparse_prefill_attn with that vt in place of v and no workspace. */
int sparse_prefill_transpose_v(const spa_params *p, const void *v, void *vt,
                               int64_t vt_blocks_per_head, int32_t first_block, int32_t n_blocks,
                               void *hip_stream);

int sparse_prefill_attn_vt(const spa_params *p, const void *q, const void *k, const void *vt,
                           int64_t vt_blocks_per_head, const int32_t *block_idx,
                           const int32_t *block_cnt, void *out, float *lse_or_null,
                           void *hip_stream);

/* Check of caller-made lists against the rules sparse_prefill_attn relies on (Sec. 4.1.1: the
 * attention kernel consumes the block-level indices as they are).  For every list row of a query
 * block that exists (ragged batches: inside its entry's length) it tests 1 <= cnt <= T, entries
 * strictly ascending, first >= 0 and last == the row's diagonal block
 * (kv_prefix_len / block_size + i), and stores the number of rows that fail in *n_bad_rows, a
 * DEVICE int32 the call overwrites (0 = every row is well formed).  Lists are [batch, n_q_heads,
 * NB, T], or [batch, n_kv_heads, NB, T] with lists_per_kv_head.  Uses of p: shape, pattern (T),
 * kv_prefix_len, lists_per_kv_head, seq_lens.  Asynchronous like every other call. */
int sparse_prefill_check_lists(const spa_params *p, const int32_t *block_idx,
                               const int32_t *block_cnt, int32_t *n_bad_rows, void *hip_stream);

/* select followed by attn on one stream.  block_idx_or_null / block_cnt_or_null:
 * pass both to receive the lists, or both NULL to keep them in the workspace. */
int sparse_prefill_fused(const spa_params *p, const void *q, const void *k, const void *v,
                         void *out, float *lse_or_null,
                         int32_t *block_idx_or_null, int32_t *block_cnt_or_null,
                         void *ws, size_t ws_bytes, void *hip_stream);

/* ---- Position-dependent budget: Token Position-Decay (Sec. 4.1.2, Fig. "Stem" (b)) ------------
 * The three calls below are the select, top-k and fused calls above with the uniform budget
 * replaced by a schedule: query block i draws k_i = min(max(top_k_per_block[i], 0),
 * p->top_k_blocks) blocks from its non-static causal candidates, so
 * block_cnt[b,h,i] = min(i + 1, n_sink + n_local + k_i).  The paper describes a budget that is
 * highest for the first positions and decays along the sequence but prints no formula, so the
 * schedule is an input: top_k_per_block is a DEVICE array of NB int32, one value per query block,
 * shared by all heads and batch entries.  p->top_k_blocks states its maximum and fixes the row
 * capacity T (and with it the layout of block_idx) exactly as in the uniform calls; larger
 * entries are clamped to it, negative ones to 0.  Ranking, ties, the static pattern, the output
 * layout, workspace and error behaviour are those of the uniform calls; a NULL schedule returns
 * SPA_ERR_NULLPTR. */
int sparse_prefill_select_tpd(const spa_params *p, const void *q, const void *k,
                              const int32_t *top_k_per_block, int32_t *block_idx,
                              int32_t *block_cnt, float *pooled_scores_or_null, void *ws,
                              size_t ws_bytes, void *hip_stream);

int sparse_prefill_topk_from_scores_tpd(const spa_params *p, const float *pooled_scores,
                                        const int32_t *top_k_per_block, int32_t *block_idx,
                                        int32_t *block_cnt, void *hip_stream);

int sparse_prefill_fused_tpd(const spa_params *p, const void *q, const void *k, const void *v,
                             const int32_t *top_k_per_block, void *out, float *lse_or_null,
                             int32_t *block_idx_or_null, int32_t *block_cnt_or_null, void *ws,
                             size_t ws_bytes, void *hip_stream);

/* ---- Output-aware ranking: Stem's Output-Aware Metric (Sec. 4.1.2, Fig. "Stem" (c)) --------------
 * The paper ranks key blocks by a metric that combines the attention score with the magnitude of
 * the value vectors and prints no formula.  Reading implemented here: a block's contribution to
 * the output is its attention weight times the size of its values, a sum in the logit domain:
 *   vn[b,hk,j]      = mean over the block's tokens t of || V[b,hk,j*Bs+t,:] ||_2      (fp32)
 *   rank[b,h,i,j]   = score[b,h,i,j] + ln vn[b,h/G,j]                                 (fp32)
 * with score as in sparse_prefill_select; a block of all-zero values ranks as -inf.  Only the
 * ranking changes: budget, ties, static pattern, list layout and the attention itself do not.
 *
 * sparse_prefill_value_norms: log_value_norms [batch, n_kv_heads, NB] fp32 <- ln vn.
 * sparse_prefill_select_stem: select with rank in place of score.  top_k_per_block_or_null: NULL
 *   for the uniform budget, else the Token Position-Decay schedule of the _tpd calls (both ideas
 *   together are the paper's Stem).  ranking_scores_or_null receives rank (j > i: -inf).
 * sparse_prefill_fused_stem: select_stem followed by attn.
 * V is read once more than in the plain calls (+ batch*n_kv_heads*seq_len*head_dim*2 bytes). */
int sparse_prefill_value_norms(const spa_params *p, const void *v, float *log_value_norms,
                               void *hip_stream);

int sparse_prefill_select_stem(const spa_params *p, const void *q, const void *k, const void *v,
                               const int32_t *top_k_per_block_or_null, int32_t *block_idx,
                               int32_t *block_cnt, float *ranking_scores_or_null, void *ws,
                               size_t ws_bytes, void *hip_stream);

int sparse_prefill_fused_stem(const spa_params *p, const void *q, const void *k, const void *v,
                              const int32_t *top_k_per_block_or_null, void *out,
                              float *lse_or_null, int32_t *block_idx_or_null,
                              int32_t *block_cnt_or_null, void *ws, size_t ws_bytes,
                              void *hip_stream);

/* ---- General form: every selection option in one place ---------------------------------------
 * The paper's framework applies its sparsity settings as metadata to specific layers or heads
 * (Sec. 4.1.1, "Decoupling Sparse Kernels from Model Architectures").  spa_select_opts carries
 * the per-call metadata; the struct is read on the HOST, its pointers are DEVICE pointers, any of
 * them may be NULL, and a NULL opts means the plain call.
 *   top_k_per_block  [NB] int32: Token Position-Decay schedule, as in the _tpd calls.
 *   v                V in the layout of p->v_stride: switches the ranking to the output-aware
 *                    score of the _stem calls (for the fused call only "non-NULL" matters, the
 *                    values read are those of its own v argument).
 *   head_pattern     [n_q_heads][3] int32 = (n_sink, n_local, top_k) of each query head, clamped
 *                    in the kernels to [0, p->n_sink_blocks], [1, p->n_local_blocks],
 *                    [0, p->top_k_blocks]: the spa_params values are then the maxima and fix the row
 *                    capacity.  With a schedule, head h draws min(schedule[i], top_k of h) blocks.
 *   mass_gamma       cumulative-mass budget, the rule of the FlexPrefill family that Sec. 4.1.1 lists
 *                    among the framework's dynamic algorithms (no formula in the paper).  0 = off.
 *                    gamma in (0, 1] (larger values count as 1): query block i takes, in ranking
 *                    order, the fewest candidates for which the selected blocks (static ones
 *                    included) hold at least the fraction gamma of the row's block-level softmax mass,
 *                    and never more than its count budget (top_k_blocks, schedule, per-head top_k),
 *                    which keeps fixing the row capacity.  So that the number of blocks does not
 *                    hinge on the order of a floating-point sum, the mass is defined in integers:
 *                    with x_j the ranking scores of the causal blocks j <= i and m their maximum,
 *                    W_j = floor(2^19 w_j + 1/2), w_j = 2^((x_j - m) log2 e) evaluated in fp32 as
 *                    2^n p(f), n the integer nearest to the exponent, f the rest, p the degree-6
 *                    Taylor polynomial of e^(f ln 2) in Horner form (NaN, -inf and exponents below
 *                    -40 weigh 0); target = ceil(Gamma sum_j W_j / 65536), Gamma = floor(65536 gamma
 *                    + 1/2); candidates are taken until mass(static) + mass(taken) >= target.
 *                    A negative or NaN gamma returns SPA_ERR_BAD_PATTERN.
 * The _tpd and _stem calls above are these calls with the corresponding fields set. */
typedef struct spa_select_opts {
    const int32_t *top_k_per_block;
    const void *v;
    const int32_t *head_pattern;
    float mass_gamma;
} spa_select_opts;

int sparse_prefill_select_ex(const spa_params *p, const void *q, const void *k,
                             const spa_select_opts *opts, int32_t *block_idx, int32_t *block_cnt,
                             float *ranking_scores_or_null, void *ws, size_t ws_bytes,
                             void *hip_stream);

int sparse_prefill_topk_from_scores_ex(const spa_params *p, const float *scores,
                                       const spa_select_opts *opts, int32_t *block_idx,
                                       int32_t *block_cnt, void *hip_stream);

int sparse_prefill_fused_ex(const spa_params *p, const void *q, const void *k, const void *v,
                            const spa_select_opts *opts, void *out, float *lse_or_null,
                            int32_t *block_idx_or_null, int32_t *block_cnt_or_null, void *ws,
                            size_t ws_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SPARSE_PREFILL_H */
