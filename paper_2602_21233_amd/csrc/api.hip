// C-ABI entry points: host-side validation, workspace carving, launches.
// Nothing here allocates, frees or synchronises; see include/sparse_prefill.h.
#include <math.h>

#include <mutex>

#include "common.hpp"

using namespace spa;

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

int check_shape(const spa_params* p) {
    if (!p) return SPA_ERR_NULLPTR;
    if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->seq_len < 1) return SPA_ERR_BAD_SHAPE;
    if (p->n_q_heads % p->n_kv_heads) return SPA_ERR_BAD_SHAPE;
    if (p->head_dim != 64 && p->head_dim != 128) return SPA_ERR_BAD_SHAPE;
    if (p->block_size != 64 && p->block_size != 128) return SPA_ERR_BAD_SHAPE;
    if (p->kv_prefix_len < 0 || p->kv_prefix_len % p->block_size) return SPA_ERR_BAD_SHAPE;
    if (((int64_t)p->kv_prefix_len + p->seq_len + p->block_size - 1) / p->block_size > kMaxBlocks) return SPA_ERR_BAD_SHAPE;
    if ((int64_t)p->batch * p->n_q_heads * ((p->seq_len + p->block_size - 1) / p->block_size) > 0x7fffffffLL) return SPA_ERR_BAD_SHAPE;
    if (p->n_sink_blocks < 0 || p->n_local_blocks < 1 || p->top_k_blocks < 0) return SPA_ERR_BAD_PATTERN;
    if (p->lists_per_kv_head != 0 && p->lists_per_kv_head != 1) return SPA_ERR_BAD_PATTERN;
    if (p->stride_blocks < 0 || p->n_dense_q_blocks < 0 || p->stride_reach_blocks < 0) return SPA_ERR_BAD_PATTERN;
    if (!(p->softmax_scale >= 0.0f) || isinf(p->softmax_scale)) return SPA_ERR_BAD_SHAPE;
    return SPA_OK;
}

int check_tensor(const void* ptr, const int64_t s[3], int head_dim) {
    if (!ptr) return SPA_ERR_NULLPTR;
    if (((uintptr_t)ptr) & 15u) return SPA_ERR_BAD_STRIDE;
    for (int a = 0; a < 3; ++a)
        if (s[a] < 0 || (s[a] & 7)) return SPA_ERR_BAD_STRIDE;
    if (s[2] < head_dim || s[2] > (1 << 22)) return SPA_ERR_BAD_STRIDE;   // 32-bit byte offsets inside a block
    return SPA_OK;
}

Dims resolved(const spa_params* p) {
    Dims d = dims_of(*p);
    if (d.scale == 0.0f) d.scale = 1.0f / sqrtf((float)d.D);
    return d;
}

struct Workspace {
    size_t qp_off, kp_off, qg_off, idx_off, cnt_off, lvn_off, vt_off, total;
};

Workspace carve(const Dims& d) {
    Workspace w;
    size_t off = 0;
    w.qp_off = off; off = align_up(off + (size_t)d.B * d.Hq * d.NB * d.D * sizeof(float));
    w.kp_off = off; off = align_up(off + (size_t)d.B * d.Hkv * ((d.NBk + 31) / 32 * 32) * d.D * sizeof(float));   // whole tiles of 32 blocks
    w.qg_off = off; if (d.shared) off = align_up(off + (size_t)d.B * d.Hkv * d.NB * d.D * sizeof(float));
    w.idx_off = off; off = align_up(off + (size_t)d.B * d.Hq * d.NB * d.T * sizeof(int32_t));
    w.cnt_off = off; off = align_up(off + (size_t)d.B * d.Hq * d.NB * sizeof(int32_t));
    w.lvn_off = off; off = align_up(off + (size_t)d.B * d.Hkv * d.NBk * sizeof(float));
    w.vt_off = off;
    off = align_up(off + (size_t)d.B * d.Hkv * d.NBk * d.Bs * d.D * sizeof(uint16_t));
    w.total = off;
    return w;
}

int launch_code(hipError_t e) { return e == hipSuccess ? SPA_OK : SPA_ERR_LAUNCH; }

// mass_gamma: 0 = no cumulative-mass budget; (0, 1] (larger: 1) = the budget; negative or NaN: error
int set_mass_budget(Dims& d, float mass_gamma) {
    if (!(mass_gamma >= 0.0f)) return SPA_ERR_BAD_PATTERN;
    if (mass_gamma == 0.0f) return SPA_OK;
    const double g = mass_gamma > 1.0f ? 1.0 : (double)mass_gamma;
    d.gamma_q16 = (int)floor(g * 65536.0 + 0.5);
    return SPA_OK;
}

}  // namespace

namespace {
// The scratch regions of the select stage: pooled Q and the group means (group-shared lists only),
// pooled K in the score kernel's operand layout, ln of the value magnitudes (output-aware score only).
struct SelectScratch {
    float *qp, *kp, *qg, *lvn;
};

// Shape, pointer and budget checks of a select call; on success d holds the resolved sizes.
int check_select(const spa_params* p, const void* q, const void* k, const void* v_or_null, float mass_gamma,
                 const int32_t* block_idx, const int32_t* block_cnt, Dims& d) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!block_idx || !block_cnt) return SPA_ERR_NULLPTR;
    if ((rc = check_tensor(q, p->q_stride, p->head_dim))) return rc;
    if ((rc = check_tensor(k, p->k_stride, p->head_dim))) return rc;
    if (v_or_null && (rc = check_tensor(v_or_null, p->v_stride, p->head_dim))) return rc;
    d = resolved(p);
    return set_mass_budget(d, mass_gamma);
}

int select_launches(Dims d, const spa_params* p, const void* q, const void* k, const void* v_or_null, const int32_t* k_rows,
                    const int32_t* head_pattern, int32_t* block_idx, int32_t* block_cnt, float* pooled_scores_or_null,
                    const SelectScratch& sc, hipStream_t st);

// v_or_null: values for the output-aware ranking score, or nullptr for the plain pooled score
int select_impl(const spa_params* p, const void* q, const void* k, const void* v_or_null, const int32_t* k_rows,
                const int32_t* head_pattern, float mass_gamma, int32_t* block_idx, int32_t* block_cnt, float* pooled_scores_or_null, void* ws, size_t ws_bytes,
                void* hip_stream) {
    Dims d;
    int rc = check_select(p, q, k, v_or_null, mass_gamma, block_idx, block_cnt, d);
    if (rc) return rc;
    if (!ws) return SPA_ERR_NULLPTR;
    if (((uintptr_t)ws) & (kAlign - 1)) return SPA_ERR_BAD_STRIDE;
    Workspace w = carve(d);
    if (ws_bytes < w.total) return SPA_ERR_WORKSPACE_TOO_SMALL;
    const SelectScratch sc{(float*)((char*)ws + w.qp_off), (float*)((char*)ws + w.kp_off), (float*)((char*)ws + w.qg_off),
                           (float*)((char*)ws + w.lvn_off)};
    return select_launches(d, p, q, k, v_or_null, k_rows, head_pattern, block_idx, block_cnt, pooled_scores_or_null, sc,
                           (hipStream_t)hip_stream);
}

int select_launches(Dims d, const spa_params* p, const void* q, const void* k, const void* v_or_null, const int32_t* k_rows,
                    const int32_t* head_pattern, int32_t* block_idx, int32_t* block_cnt, float* pooled_scores_or_null,
                    const SelectScratch& sc, hipStream_t st) {
    float* qp = sc.qp;
    float* kp = sc.kp;
    // Group-shared lists rank the mean of the group's pooled queries, which needs them in memory; all other
    // calls pool K only and let the score kernel pool its own query blocks from Q (the Q stream then hides
    // the scoring and selection)
    const bool q_in_kernel = !d.shared;
    hipError_t e = launch_pool(d, q_in_kernel ? nullptr : q, strides_of(p->q_stride), k, strides_of(p->k_stride), qp, kp, true, st);
    if (e != hipSuccess) return SPA_ERR_LAUNCH;
    float* lvn = nullptr;
    if (v_or_null) {
        lvn = sc.lvn;
        if (launch_vnorm(d, v_or_null, strides_of(p->v_stride), lvn, st) != hipSuccess) return SPA_ERR_LAUNCH;
    }
    if (d.shared) {
        // one list per KV head: rank the group by its mean pooled query, then select as if the
        // KV heads were the query heads
        float* qg = sc.qg;
        if (launch_group_mean(d, qp, qg, st) != hipSuccess) return SPA_ERR_LAUNCH;
        d.Hq = d.Hkv;
        d.G = 1;
        qp = qg;
    }
    return launch_code(launch_score_topk(d, qp, kp, k_rows, head_pattern, lvn, block_idx, block_cnt, pooled_scores_or_null,
                                         q_in_kernel ? q : nullptr, strides_of(p->q_stride), st));
}

int topk_impl(const spa_params* p, const float* pooled_scores, const int32_t* k_rows,
              const int32_t* head_pattern, float mass_gamma, int32_t* block_idx,
              int32_t* block_cnt, void* hip_stream) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!pooled_scores || !block_idx || !block_cnt) return SPA_ERR_NULLPTR;
    Dims d = resolved(p);
    if ((rc = set_mass_budget(d, mass_gamma))) return rc;
    if (d.shared) { d.Hq = d.Hkv; d.G = 1; }
    return launch_code(launch_topk_from_scores(d, pooled_scores, k_rows, head_pattern, block_idx, block_cnt,
                                               (hipStream_t)hip_stream));
}

int fused_impl(const spa_params* p, const void* q, const void* k, const void* v, const int32_t* k_rows,
               const int32_t* head_pattern, float mass_gamma, bool output_aware, void* out, float* lse_or_null, int32_t* block_idx_or_null,
               int32_t* block_cnt_or_null, void* ws, size_t ws_bytes, void* hip_stream) {
    int rc = check_shape(p);
    if (rc) return rc;
    if ((block_idx_or_null == nullptr) != (block_cnt_or_null == nullptr)) return SPA_ERR_NULLPTR;
    if (!ws) return SPA_ERR_NULLPTR;
    if ((rc = check_tensor(v, p->v_stride, p->head_dim))) return rc;
    if ((rc = check_tensor(out, p->o_stride, p->head_dim))) return rc;
    if (((uintptr_t)ws) & (kAlign - 1)) return SPA_ERR_BAD_STRIDE;
    Dims d = resolved(p);
    Workspace w = carve(d);
    if (ws_bytes < w.total) return SPA_ERR_WORKSPACE_TOO_SMALL;
    int32_t* idx = block_idx_or_null ? block_idx_or_null : (int32_t*)((char*)ws + w.idx_off);
    int32_t* cnt = block_cnt_or_null ? block_cnt_or_null : (int32_t*)((char*)ws + w.cnt_off);
    rc = select_impl(p, q, k, output_aware ? v : nullptr, k_rows, head_pattern, mass_gamma, idx, cnt, nullptr, ws, ws_bytes, hip_stream);
    if (rc) return rc;
    return sparse_prefill_attn(p, q, k, v, idx, cnt, out, lse_or_null, ws, ws_bytes, hip_stream);
}
}  // namespace


// ---- scratch that the library owns: for callers that cannot allocate ---------------------------
// One array per GPU, in the device image of this library, held until the process ends.  In host
// code the array's name is only a stand-in for the symbol, not a device address: its address on a
// given device comes from hipGetSymbolAddress, asked once per device with that device current
// and remembered; everything below uses that pointer, never the name.
constexpr size_t kStaticScratchBytes = SPA_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
std::mutex scratch_mu;
void* scratch_ptr[kMaxDevices];             // per device; nullptr = not asked yet

// address of this device's copy of the array, or nullptr with *err set
void* static_scratch(hipError_t* err) {
    int dev = 0;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || ptr == nullptr) {
            if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
            return nullptr;
        }
        scratch_ptr[dev] = ptr;
    }
    return scratch_ptr[dev];
}

// bytes of scratch a plain select call needs: pooled K in tiles of 32 key blocks, plus, with
// group-shared lists, the pooled queries and their group means
struct StaticCarve {
    size_t kp_off, qp_off, qg_off, total;
};
StaticCarve carve_static(const Dims& d) {
    StaticCarve c;
    size_t off = 0;
    c.kp_off = off; off = align_up(off + (size_t)d.B * d.Hkv * ((d.NBk + 31) / 32 * 32) * d.D * sizeof(float));
    c.qp_off = off; if (d.shared) off = align_up(off + (size_t)d.B * d.Hq * d.NB * d.D * sizeof(float));
    c.qg_off = off; if (d.shared) off = align_up(off + (size_t)d.B * d.Hkv * d.NB * d.D * sizeof(float));
    c.total = off;
    return c;
}
}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char* spa_strerror(int code) {
    switch (code) {
        case SPA_OK: return "ok";
        case SPA_ERR_NULLPTR: return "a required pointer is NULL";
        case SPA_ERR_BAD_SHAPE: return "unsupported shape (head_dim and block_size must be 64 or 128, at most 4096 key blocks, kv_prefix_len a non-negative multiple of block_size, n_q_heads a multiple of n_kv_heads)";
        case SPA_ERR_BAD_PATTERN: return "bad static pattern or budget (need n_sink >= 0, n_local >= 1, top_k >= 0, stride >= 0, n_dense >= 0)";
        case SPA_ERR_BAD_STRIDE: return "strides must be non-negative multiples of 8 elements, token stride >= head_dim, pointers 16-byte aligned";
        case SPA_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than spa_workspace_bytes()";
        case SPA_ERR_LAUNCH: return "the HIP runtime rejected a kernel launch";
        case SPA_ERR_STATIC_SCRATCH_TOO_SMALL: return "the call needs more scratch than the library's static device array holds (SPA_STATIC_SCRATCH_BYTES); use the call that takes a workspace";
        default: return "unknown error code";
    }
}

int spa_row_capacity(const spa_params* p, int32_t* row_capacity) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!row_capacity) return SPA_ERR_NULLPTR;
    *row_capacity = dims_of(*p).T;
    return SPA_OK;
}

int spa_workspace_bytes(const spa_params* p, size_t* bytes) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!bytes) return SPA_ERR_NULLPTR;
    *bytes = carve(dims_of(*p)).total;
    return SPA_OK;
}

int sparse_prefill_pool(const spa_params* p, const void* q, const void* k, float* q_pooled,
                        float* k_pooled, void* hip_stream) {
    int rc = check_shape(p);
    if (rc) return rc;
    if ((q == nullptr) != (q_pooled == nullptr) || (k == nullptr) != (k_pooled == nullptr)) return SPA_ERR_NULLPTR;
    if (!q && !k) return SPA_ERR_NULLPTR;
    if (q && (rc = check_tensor(q, p->q_stride, p->head_dim))) return rc;
    if (k && (rc = check_tensor(k, p->k_stride, p->head_dim))) return rc;
    Dims d = resolved(p);
    return launch_code(launch_pool(d, q, strides_of(p->q_stride), k, strides_of(p->k_stride), q_pooled,
                                   k_pooled, false, (hipStream_t)hip_stream));
}


int sparse_prefill_select(const spa_params* p, const void* q, const void* k, int32_t* block_idx,
                          int32_t* block_cnt, float* pooled_scores_or_null, void* ws, size_t ws_bytes,
                          void* hip_stream) {
    return select_impl(p, q, k, nullptr, nullptr, nullptr, 0.0f, block_idx, block_cnt, pooled_scores_or_null, ws, ws_bytes,
                       hip_stream);
}

int sparse_prefill_select_static(const spa_params* p, const void* q, const void* k, int32_t* block_idx,
                                 int32_t* block_cnt, float* pooled_scores_or_null, void* hip_stream) {
    Dims d;
    int rc = check_select(p, q, k, nullptr, 0.0f, block_idx, block_cnt, d);
    if (rc) return rc;
    const StaticCarve c = carve_static(d);
    if (c.total > kStaticScratchBytes) return SPA_ERR_STATIC_SCRATCH_TOO_SMALL;
    hipError_t e;
    char* base = (char*)static_scratch(&e);
    if (base == nullptr) return SPA_ERR_LAUNCH;
    const SelectScratch sc{(float*)(base + c.qp_off), (float*)(base + c.kp_off), (float*)(base + c.qg_off), nullptr};
    return select_launches(d, p, q, k, nullptr, nullptr, nullptr, block_idx, block_cnt, pooled_scores_or_null, sc,
                           (hipStream_t)hip_stream);
}

int sparse_prefill_select_tpd(const spa_params* p, const void* q, const void* k, const int32_t* top_k_per_block,
                              int32_t* block_idx, int32_t* block_cnt, float* pooled_scores_or_null, void* ws,
                              size_t ws_bytes, void* hip_stream) {
    if (!top_k_per_block) return SPA_ERR_NULLPTR;
    return select_impl(p, q, k, nullptr, top_k_per_block, nullptr, 0.0f, block_idx, block_cnt, pooled_scores_or_null, ws,
                       ws_bytes, hip_stream);
}

int sparse_prefill_topk_from_scores(const spa_params* p, const float* pooled_scores, int32_t* block_idx,
                                    int32_t* block_cnt, void* hip_stream) {
    return topk_impl(p, pooled_scores, nullptr, nullptr, 0.0f, block_idx, block_cnt, hip_stream);
}

int sparse_prefill_topk_from_scores_tpd(const spa_params* p, const float* pooled_scores,
                                        const int32_t* top_k_per_block, int32_t* block_idx, int32_t* block_cnt,
                                        void* hip_stream) {
    if (!top_k_per_block) return SPA_ERR_NULLPTR;
    return topk_impl(p, pooled_scores, top_k_per_block, nullptr, 0.0f, block_idx, block_cnt, hip_stream);
}

int sparse_prefill_attn(const spa_params* p, const void* q, const void* k, const void* v,
                        const int32_t* block_idx, const int32_t* block_cnt, void* out,
                        float* lse_or_null, void* ws, size_t ws_bytes, void* hip_stream) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!block_idx || !block_cnt || !ws) return SPA_ERR_NULLPTR;
    if ((rc = check_tensor(q, p->q_stride, p->head_dim))) return rc;
    if ((rc = check_tensor(k, p->k_stride, p->head_dim))) return rc;
    if ((rc = check_tensor(v, p->v_stride, p->head_dim))) return rc;
    if ((rc = check_tensor(out, p->o_stride, p->head_dim))) return rc;
    if (((uintptr_t)ws) & (kAlign - 1)) return SPA_ERR_BAD_STRIDE;
    Dims d = resolved(p);
    Workspace w = carve(d);
    if (ws_bytes < w.total) return SPA_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;
    return launch_code(launch_attn(d, q, strides_of(p->q_stride), k, strides_of(p->k_stride), v,
                                   strides_of(p->v_stride), block_idx, block_cnt, out,
                                   strides_of(p->o_stride), lse_or_null, (char*)ws + w.vt_off, st));
}

int sparse_prefill_transpose_v(const spa_params* p, const void* v, void* vt, int64_t vt_blocks_per_head,
                               int32_t first_block, int32_t n_blocks, void* hip_stream) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!vt) return SPA_ERR_NULLPTR;
    if ((rc = check_tensor(v, p->v_stride, p->head_dim))) return rc;
    if (((uintptr_t)vt) & 15u) return SPA_ERR_BAD_STRIDE;
    const Dims d = resolved(p);
    if (vt_blocks_per_head < d.NBk || first_block < 0 || n_blocks < 0 || (int64_t)first_block + n_blocks > d.NBk)
        return SPA_ERR_BAD_SHAPE;
    return launch_code(launch_transpose_v(d, v, strides_of(p->v_stride), vt, vt_blocks_per_head, first_block, n_blocks,
                                          (hipStream_t)hip_stream));
}

int sparse_prefill_attn_vt(const spa_params* p, const void* q, const void* k, const void* vt, int64_t vt_blocks_per_head,
                           const int32_t* block_idx, const int32_t* block_cnt, void* out, float* lse_or_null,
                           void* hip_stream) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!block_idx || !block_cnt || !vt) return SPA_ERR_NULLPTR;
    if ((rc = check_tensor(q, p->q_stride, p->head_dim))) return rc;
    if ((rc = check_tensor(k, p->k_stride, p->head_dim))) return rc;
    if ((rc = check_tensor(out, p->o_stride, p->head_dim))) return rc;
    if (((uintptr_t)vt) & 15u) return SPA_ERR_BAD_STRIDE;
    const Dims d = resolved(p);
    if (vt_blocks_per_head < d.NBk) return SPA_ERR_BAD_SHAPE;
    return launch_code(launch_attn_vt(d, q, strides_of(p->q_stride), k, strides_of(p->k_stride), vt, vt_blocks_per_head,
                                      block_idx, block_cnt, out, strides_of(p->o_stride), lse_or_null,
                                      (hipStream_t)hip_stream));
}

int sparse_prefill_check_lists(const spa_params* p, const int32_t* block_idx, const int32_t* block_cnt,
                               int32_t* n_bad_rows, void* hip_stream) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!block_idx || !block_cnt || !n_bad_rows) return SPA_ERR_NULLPTR;
    const Dims d = resolved(p);
    return launch_code(launch_check_lists(d, block_idx, block_cnt, n_bad_rows, (hipStream_t)hip_stream));
}

int sparse_prefill_fused(const spa_params* p, const void* q, const void* k, const void* v, void* out,
                         float* lse_or_null, int32_t* block_idx_or_null, int32_t* block_cnt_or_null,
                         void* ws, size_t ws_bytes, void* hip_stream) {
    return fused_impl(p, q, k, v, nullptr, nullptr, 0.0f, false, out, lse_or_null, block_idx_or_null, block_cnt_or_null, ws,
                      ws_bytes, hip_stream);
}

int sparse_prefill_fused_tpd(const spa_params* p, const void* q, const void* k, const void* v,
                             const int32_t* top_k_per_block, void* out, float* lse_or_null,
                             int32_t* block_idx_or_null, int32_t* block_cnt_or_null, void* ws, size_t ws_bytes,
                             void* hip_stream) {
    if (!top_k_per_block) return SPA_ERR_NULLPTR;
    return fused_impl(p, q, k, v, top_k_per_block, nullptr, 0.0f, false, out, lse_or_null, block_idx_or_null, block_cnt_or_null,
                      ws, ws_bytes, hip_stream);
}

int sparse_prefill_value_norms(const spa_params* p, const void* v, float* log_value_norms, void* hip_stream) {
    int rc = check_shape(p);
    if (rc) return rc;
    if (!log_value_norms) return SPA_ERR_NULLPTR;
    if ((rc = check_tensor(v, p->v_stride, p->head_dim))) return rc;
    Dims d = resolved(p);
    return launch_code(launch_vnorm(d, v, strides_of(p->v_stride), log_value_norms, (hipStream_t)hip_stream));
}

int sparse_prefill_select_stem(const spa_params* p, const void* q, const void* k, const void* v,
                               const int32_t* top_k_per_block_or_null, int32_t* block_idx, int32_t* block_cnt,
                               float* ranking_scores_or_null, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!v) return SPA_ERR_NULLPTR;
    return select_impl(p, q, k, v, top_k_per_block_or_null, nullptr, 0.0f, block_idx, block_cnt, ranking_scores_or_null, ws,
                       ws_bytes, hip_stream);
}

int sparse_prefill_fused_stem(const spa_params* p, const void* q, const void* k, const void* v,
                              const int32_t* top_k_per_block_or_null, void* out, float* lse_or_null,
                              int32_t* block_idx_or_null, int32_t* block_cnt_or_null, void* ws, size_t ws_bytes,
                              void* hip_stream) {
    return fused_impl(p, q, k, v, top_k_per_block_or_null, nullptr, 0.0f, true, out, lse_or_null, block_idx_or_null,
                      block_cnt_or_null, ws, ws_bytes, hip_stream);
}

int sparse_prefill_select_ex(const spa_params* p, const void* q, const void* k, const spa_select_opts* opts,
                             int32_t* block_idx, int32_t* block_cnt, float* ranking_scores_or_null, void* ws,
                             size_t ws_bytes, void* hip_stream) {
    const spa_select_opts none = {nullptr, nullptr, nullptr, 0.0f};
    const spa_select_opts* o = opts ? opts : &none;
    return select_impl(p, q, k, o->v, o->top_k_per_block, o->head_pattern, o->mass_gamma, block_idx, block_cnt,
                       ranking_scores_or_null, ws, ws_bytes, hip_stream);
}

int sparse_prefill_topk_from_scores_ex(const spa_params* p, const float* scores, const spa_select_opts* opts,
                                       int32_t* block_idx, int32_t* block_cnt, void* hip_stream) {
    const spa_select_opts none = {nullptr, nullptr, nullptr, 0.0f};
    const spa_select_opts* o = opts ? opts : &none;
    return topk_impl(p, scores, o->top_k_per_block, o->head_pattern, o->mass_gamma, block_idx, block_cnt, hip_stream);
}

int sparse_prefill_fused_ex(const spa_params* p, const void* q, const void* k, const void* v,
                            const spa_select_opts* opts, void* out, float* lse_or_null, int32_t* block_idx_or_null,
                            int32_t* block_cnt_or_null, void* ws, size_t ws_bytes, void* hip_stream) {
    const spa_select_opts none = {nullptr, nullptr, nullptr, 0.0f};
    const spa_select_opts* o = opts ? opts : &none;
    return fused_impl(p, q, k, v, o->top_k_per_block, o->head_pattern, o->mass_gamma, o->v != nullptr, out, lse_or_null,
                      block_idx_or_null, block_cnt_or_null, ws, ws_bytes, hip_stream);
}

}  // extern "C"
#pragma GCC visibility pop
