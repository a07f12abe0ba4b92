// Host side of libstem_hip: argument checks, shape bookkeeping, the Token Position-Decay schedule
// helper (Eq. 3) and the dispatch of the four kernels.  No allocation, no synchronisation.
#include <cmath>
#include <cstring>

#include "stem_common.h"

namespace stem {

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int make_problem(const stem_shape* s, Problem* out) {
    if (!s || !out || !s->host_cu_seqlens) return STEM_ERR_INVALID_ARG;
    if (s->num_q_heads <= 0 || s->num_kv_heads <= 0 || s->num_q_heads % s->num_kv_heads)
        return STEM_ERR_INVALID_ARG;
    if (s->batch < 1 || s->batch > STEM_MAX_BATCH) return STEM_ERR_INVALID_ARG;
    if (s->head_dim <= 0 || s->block_size <= 0) return STEM_ERR_INVALID_ARG;
    if (s->head_dim != 64 && s->head_dim != 128 && s->head_dim != 256) return STEM_ERR_UNSUPPORTED;
    if (s->block_size != 64 && s->block_size != 128) return STEM_ERR_UNSUPPORTED;
    if (s->q_stride_head < s->head_dim || s->kv_stride_head < s->head_dim) return STEM_ERR_INVALID_ARG;
    if (s->q_stride_token < s->head_dim || s->kv_stride_token < s->head_dim) return STEM_ERR_INVALID_ARG;
    if ((s->q_stride_head | s->q_stride_token | s->kv_stride_head | s->kv_stride_token) & 7)
        return STEM_ERR_INVALID_ARG;
    Problem p;
    std::memset(&p, 0, sizeof(p));
    p.Hq = s->num_q_heads;
    p.Hkv = s->num_kv_heads;
    p.G = p.Hq / p.Hkv;
    p.B = s->block_size;
    p.d = s->head_dim;
    p.batch = s->batch;
    p.q_st = s->q_stride_token;
    p.q_sh = s->q_stride_head;
    p.kv_st = s->kv_stride_token;
    p.kv_sh = s->kv_stride_head;
    if (s->host_cu_seqlens[0] != 0) return STEM_ERR_INVALID_ARG;
    if ((s->host_chunk_start == nullptr) != (s->host_chunk_end == nullptr)) return STEM_ERR_INVALID_ARG;
    p.seq.batch = p.batch;
    int64_t rows = 0, key_rows = 0, q_tokens = 0;
    int32_t nbmax = 0;
    for (int i = 0; i < p.batch; ++i) {
        int64_t lo = s->host_cu_seqlens[i], hi = s->host_cu_seqlens[i + 1];
        if (hi < lo) return STEM_ERR_INVALID_ARG;
        const int64_t len = hi - lo;
        const int64_t nb = (len + p.B - 1) / p.B;
        if (nb > STEM_MAX_BLOCKS) return STEM_ERR_UNSUPPORTED;
        // the chunk of this call: block-aligned start; the end is block-aligned or the sequence's end
        int64_t cs = 0, ce = len;
        if (s->host_chunk_start) {
            cs = s->host_chunk_start[i];
            ce = s->host_chunk_end[i];
            if (cs < 0 || ce < cs || ce > len) return STEM_ERR_INVALID_ARG;
            if (ce > cs && (cs % p.B || (ce % p.B && ce != len))) return STEM_ERR_INVALID_ARG;
        }
        const int64_t first = cs / p.B, seen = (ce + p.B - 1) / p.B;   // blocks before / up to the chunk's end
        p.seq.tok_start[i] = (int32_t)lo;
        p.seq.row_start[i] = (int32_t)rows;
        p.seq.q_tok_start[i] = (int32_t)q_tokens;
        p.seq.key_row_start[i] = (int32_t)key_rows;
        p.seq.first_block[i] = (int32_t)first;
        p.seq.kv_end[i] = (int32_t)(lo + ce);
        rows += ce > cs ? seen - first : 0;
        q_tokens += ce - cs;
        key_rows += nb;
        if (ce > cs && seen > nbmax) nbmax = (int32_t)seen;
    }
    if (rows > (int64_t)1 << 24 || key_rows > (int64_t)1 << 24) return STEM_ERR_UNSUPPORTED;
    for (int i = p.batch; i <= STEM_MAX_BATCH; ++i) {
        p.seq.tok_start[i] = s->host_cu_seqlens[p.batch];
        p.seq.row_start[i] = (int32_t)rows;
        p.seq.q_tok_start[i] = (int32_t)q_tokens;
        p.seq.key_row_start[i] = (int32_t)key_rows;
        if (i < STEM_MAX_BATCH) {
            p.seq.first_block[i] = 0;
            p.seq.kv_end[i] = s->host_cu_seqlens[p.batch];
        }
    }
    p.T = (int32_t)q_tokens;
    p.R = (int32_t)rows;
    p.Rk = (int32_t)key_rows;
    p.NBmax = nbmax;
    *out = p;
    return STEM_OK;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

int check_ad_stride(const Problem& p, int ad_stride) {
    if (ad_stride < 1 || p.B % ad_stride) return STEM_ERR_INVALID_ARG;
    if (ad_stride > 16) return STEM_ERR_UNSUPPORTED;   // divisors of 64 / 128 up to 16 are 1, 2, 4, 8, 16
    return STEM_OK;
}

WorkspaceLayout workspace_layout(const Problem& p, int ad_stride) {
    WorkspaceLayout w;
    // the key parts come first and depend on the sequences only, not on the chunk: a caller that
    // keeps the workspace between the chunks of a prompt finds the earlier chunks' keys in place
    w.k_bar = 0;
    w.m_v = align256(w.k_bar + sizeof(float) * (size_t)p.Hkv * p.Rk * ad_stride * p.d);
    w.q_bar = align256(w.m_v + sizeof(float) * (size_t)p.Hkv * p.Rk);
    w.total = align256(w.q_bar + sizeof(float) * (size_t)p.Hq * p.R * ad_stride * p.d);
    if (w.total == 0) w.total = 256;
    return w;
}

}  // namespace stem

using namespace stem;

extern "C" {

int stem_version(void) { return 300; }

const char* stem_strerror(int status) {
    switch (status) {
        case STEM_OK: return "ok";
        case STEM_ERR_INVALID_ARG: return "invalid argument";
        case STEM_ERR_UNSUPPORTED: return "unsupported shape or option";
        case STEM_ERR_WORKSPACE: return "workspace too small";
        case STEM_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int stem_rows(const stem_shape* shape, int32_t* host_total_rows, int32_t* host_max_blocks) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if (host_total_rows) *host_total_rows = p.R;
    if (host_max_blocks) *host_max_blocks = p.NBmax;
    return STEM_OK;
}

int stem_workspace_bytes(const stem_shape* shape, int32_t ad_stride, size_t* host_bytes) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if ((st = check_ad_stride(p, ad_stride)) != STEM_OK) return st;
    if (!host_bytes) return STEM_ERR_INVALID_ARG;
    *host_bytes = workspace_layout(p, ad_stride).total;
    return STEM_OK;
}

int stem_workspace_layout(const stem_shape* shape, int32_t ad_stride, size_t* host_q_bar_offset,
                          size_t* host_k_bar_offset, size_t* host_m_v_offset) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if ((st = check_ad_stride(p, ad_stride)) != STEM_OK) return st;
    WorkspaceLayout w = workspace_layout(p, ad_stride);
    if (host_q_bar_offset) *host_q_bar_offset = w.q_bar;
    if (host_k_bar_offset) *host_k_bar_offset = w.k_bar;
    if (host_m_v_offset) *host_m_v_offset = w.m_v;
    return STEM_OK;
}

int stem_budget_schedule(const stem_shape* shape, const double* host_k_start_blocks, double mu,
                         int32_t k_min, int32_t n_sink, int32_t n_local, int32_t* host_budget,
                         int32_t* host_kmax) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if (!host_k_start_blocks || !host_budget) return STEM_ERR_INVALID_ARG;
    if (!(mu > 0.0) || mu > 1.0 || k_min < 0 || n_sink < 0 || n_local < 0) return STEM_ERR_INVALID_ARG;
    for (int s = 0; s < p.batch; ++s)
        if (!(host_k_start_blocks[s] >= 0.0) || host_k_start_blocks[s] > 1e9) return STEM_ERR_INVALID_ARG;
    int32_t kmax = 0;
    for (int s = 0; s < p.batch; ++s) {
        // n of Eq. 3 is the whole sequence; the call's rows are blocks first .. first + rows - 1 of it
        const int32_t n = p.seq.key_row_start[s + 1] - p.seq.key_row_start[s];
        const int32_t first = p.seq.first_block[s], rows = p.seq.row_start[s + 1] - p.seq.row_start[s];
        const double ks = host_k_start_blocks[s];
        // per-row decrement of Eq. 3; volatile keeps the compiler from contracting the
        // multiply-subtract below into one fused operation
        volatile double step = n > 0 ? (ks * (1.0 - mu)) / (double)n : 0.0;
        for (int32_t i = first; i < first + rows; ++i) {
            volatile double dec = step * (double)(i + 1);
            int64_t k = (int64_t)std::floor(ks - dec + 1e-9);
            const int32_t head = n_sink < i + 1 ? n_sink : i + 1;             // blocks 0..head-1
            const int32_t tail_lo = i - n_local + 1 > head ? i - n_local + 1 : head;
            const int64_t forced = head + (i + 1 - tail_lo);
            if (k < k_min) k = k_min;
            if (k < forced) k = forced;
            if (k > i + 1) k = i + 1;
            host_budget[p.seq.row_start[s] + (i - first)] = (int32_t)k;
            if (k > kmax) kmax = (int32_t)k;
        }
    }
    if (host_kmax) *host_kmax = kmax;
    return STEM_OK;
}

static int check_qkv(const void* q, const void* k, const void* v) {
    if (!q || !k || !v) return STEM_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v)) return STEM_ERR_INVALID_ARG;
    return STEM_OK;
}

int stem_pool(const stem_shape* shape, const void* q, const void* k, const void* v, int32_t ad_stride,
              void* workspace, size_t workspace_bytes, void* hip_stream) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if ((st = check_ad_stride(p, ad_stride)) != STEM_OK) return st;
    if ((st = check_qkv(q, k, v)) != STEM_OK) return st;
    if (!workspace || !aligned16(workspace)) return STEM_ERR_INVALID_ARG;
    WorkspaceLayout w = workspace_layout(p, ad_stride);
    if (workspace_bytes < w.total) return STEM_ERR_WORKSPACE;
    if (p.R == 0) return STEM_OK;
    char* ws = static_cast<char*>(workspace);
    return launch_pool(p, ad_stride, q, k, v, reinterpret_cast<float*>(ws + w.q_bar),
                       reinterpret_cast<float*>(ws + w.k_bar), reinterpret_cast<float*>(ws + w.m_v),
                       static_cast<hipStream_t>(hip_stream));
}

int stem_block_scores(const stem_shape* shape, const void* workspace, size_t workspace_bytes,
                      int32_t ad_stride, float beta, float route_scale, int32_t fill_non_causal,
                      float* scores, void* hip_stream) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if (fill_non_causal != 0 && fill_non_causal != 1) return STEM_ERR_INVALID_ARG;
    if ((st = check_ad_stride(p, ad_stride)) != STEM_OK) return st;
    if (!workspace || !aligned16(workspace) || !scores || !aligned16(scores)) return STEM_ERR_INVALID_ARG;
    if (!std::isfinite(beta) || !std::isfinite(route_scale)) return STEM_ERR_INVALID_ARG;
    WorkspaceLayout w = workspace_layout(p, ad_stride);
    if (workspace_bytes < w.total) return STEM_ERR_WORKSPACE;
    if (p.R == 0) return STEM_OK;
    const char* ws = static_cast<const char*>(workspace);
    return launch_block_scores(p, ad_stride, reinterpret_cast<const float*>(ws + w.q_bar),
                               reinterpret_cast<const float*>(ws + w.k_bar),
                               reinterpret_cast<const float*>(ws + w.m_v), beta, route_scale,
                               fill_non_causal != 0, scores, static_cast<hipStream_t>(hip_stream));
}

int stem_estimate(const stem_shape* shape, const void* q, const void* k, const void* v, float beta,
                  float route_scale, int32_t ad_stride, int32_t fill_non_causal, float* scores,
                  void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!scores || !aligned16(scores)) return STEM_ERR_INVALID_ARG;
    if (fill_non_causal != 0 && fill_non_causal != 1) return STEM_ERR_INVALID_ARG;
    if (!std::isfinite(beta) || !std::isfinite(route_scale)) return STEM_ERR_INVALID_ARG;
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if ((st = check_ad_stride(p, ad_stride)) != STEM_OK) return st;
    st = stem_pool(shape, q, k, v, ad_stride, workspace, workspace_bytes, hip_stream);
    if (st != STEM_OK) return st;
    return stem_block_scores(shape, workspace, workspace_bytes, ad_stride, beta, route_scale,
                             fill_non_causal, scores, hip_stream);
}

int stem_estimate_select(const stem_shape* shape, const void* q, const void* k, const void* v,
                         float beta, float route_scale, int32_t ad_stride, const int32_t* budget,
                         int32_t n_sink, int32_t n_local, int32_t* counts, int32_t* indices,
                         int32_t kmax, float* debug_scores, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    if (!std::isfinite(beta) || !std::isfinite(route_scale)) return STEM_ERR_INVALID_ARG;
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if ((st = check_ad_stride(p, ad_stride)) != STEM_OK) return st;
    if (!budget || !counts || !indices) return STEM_ERR_INVALID_ARG;
    if (debug_scores && !aligned16(debug_scores)) return STEM_ERR_INVALID_ARG;
    // the diagonal block is always kept (Algorithm 1 step 3c), so the local window holds at least it
    if (n_sink < 0 || n_local < 1 || kmax < 1) return STEM_ERR_INVALID_ARG;
    if ((int64_t)kmax < (int64_t)n_sink + n_local && kmax < p.NBmax) return STEM_ERR_INVALID_ARG;
    st = stem_pool(shape, q, k, v, ad_stride, workspace, workspace_bytes, hip_stream);
    if (st != STEM_OK || p.R == 0) return st;
    WorkspaceLayout w = workspace_layout(p, ad_stride);
    const char* ws = static_cast<const char*>(workspace);
    return launch_score_select(p, ad_stride, reinterpret_cast<const float*>(ws + w.q_bar),
                               reinterpret_cast<const float*>(ws + w.k_bar),
                               reinterpret_cast<const float*>(ws + w.m_v), beta, route_scale, budget, n_sink,
                               n_local, counts, indices, kmax, debug_scores,
                               static_cast<hipStream_t>(hip_stream));
}

int stem_group_scores(const stem_shape* shape, const float* scores, int32_t reduce,
                      float* group_scores, void* hip_stream) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if (!scores || !group_scores) return STEM_ERR_INVALID_ARG;
    if (reduce != STEM_GROUP_MAX && reduce != STEM_GROUP_MEAN) return STEM_ERR_INVALID_ARG;
    if (p.R == 0) return STEM_OK;
    return launch_group_scores(p, scores, reduce, group_scores, static_cast<hipStream_t>(hip_stream));
}

int stem_select(const stem_shape* shape, const float* scores, const int32_t* budget, int32_t n_sink,
                int32_t n_local, int32_t lists_per_kv_head, int32_t* counts, int32_t* indices,
                int32_t kmax, void* hip_stream) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if (lists_per_kv_head != 0 && lists_per_kv_head != 1) return STEM_ERR_INVALID_ARG;
    if (!scores || !budget || !counts || !indices) return STEM_ERR_INVALID_ARG;
    // the diagonal block is always kept (Algorithm 1 step 3c), so the local window holds at least it
    if (n_sink < 0 || n_local < 1 || kmax < 1) return STEM_ERR_INVALID_ARG;
    if ((int64_t)kmax < (int64_t)n_sink + n_local && kmax < p.NBmax) return STEM_ERR_INVALID_ARG;
    if (p.R == 0) return STEM_OK;
    return launch_select(p, lists_per_kv_head ? p.Hkv : p.Hq, scores, budget, n_sink, n_local, counts,
                         indices, kmax, static_cast<hipStream_t>(hip_stream));
}

int stem_sparse_attn(const stem_shape* shape, const void* q, const void* k, const void* v,
                     const int32_t* counts, const int32_t* indices, int32_t kmax,
                     int32_t lists_per_kv_head, float softmax_scale, void* out, float* lse,
                     void* hip_stream) {
    Problem p;
    int st = make_problem(shape, &p);
    if (st != STEM_OK) return st;
    if (lists_per_kv_head != 0 && lists_per_kv_head != 1) return STEM_ERR_INVALID_ARG;
    if ((st = check_qkv(q, k, v)) != STEM_OK) return st;
    if (!counts || !indices || !out || !aligned16(out) || kmax < 1) return STEM_ERR_INVALID_ARG;
    if (!std::isfinite(softmax_scale) || !(softmax_scale > 0.f)) return STEM_ERR_INVALID_ARG;
    // the kernel addresses one sequence of one KV head through a 32-bit byte offset, with offsets
    // from 2^31 on reserved for requests that must fetch nothing
    for (int s = 0; s < p.batch; ++s) {
        const int64_t rows = p.seq.tok_start[s + 1] - p.seq.tok_start[s];
        if (rows > 0 && (rows - 1) * p.kv_st * 2 + p.d * 2 > 0x7fffffffll) return STEM_ERR_UNSUPPORTED;
    }
    if (p.R == 0) return STEM_OK;
    return launch_sparse_attn(p, q, k, v, counts, indices, kmax, lists_per_kv_head != 0, softmax_scale,
                              out, lse, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
