// Internal declarations shared by the host API and the gfx950 kernels of libstem_hip.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stem.h"

namespace stem {

// Packed-sequence table, passed to kernels by value (no device-side cu_seqlens read, no sync).
// A call covers, of every sequence, the query blocks of one chunk [chunk_start, chunk_end) (the
// whole sequence unless the shape says otherwise) and the keys before chunk_end.
struct SeqTable {
    int32_t batch;
    int32_t tok_start[STEM_MAX_BATCH + 1];      // cu_seqlens: token rows of K and V
    int32_t row_start[STEM_MAX_BATCH + 1];      // prefix sums of the call's query-block rows
    int32_t q_tok_start[STEM_MAX_BATCH + 1];    // prefix sums of the call's query tokens (rows of Q, O, lse)
    int32_t key_row_start[STEM_MAX_BATCH + 1];  // prefix sums of all blocks per sequence (rows of k_bar, m_v)
    int32_t first_block[STEM_MAX_BATCH];        // index in its sequence of the first query block of the call
    int32_t kv_end[STEM_MAX_BATCH];             // token row of K/V one past the last key of the call
};

// Everything the host derives from a stem_shape.
struct Problem {
    int32_t Hq, Hkv, G, B, batch;
    int32_t d;        // head size: 64, 128 or 256
    int32_t T;        // query tokens of the call (rows of Q, O, lse)
    int32_t R;        // query-block rows of the call
    int32_t Rk;       // blocks of all sequences (rows of k_bar, m_v)
    int32_t NBmax;    // most key blocks any row of the call can see
    int64_t q_st, q_sh, kv_st, kv_sh;
    SeqTable seq;
};

int make_problem(const stem_shape* shape, Problem* out);

struct WorkspaceLayout {
    size_t q_bar, k_bar, m_v, total;
};
WorkspaceLayout workspace_layout(const Problem& p, int ad_stride);
// STEM_OK if S is a supported anti-diagonal stride for this block size.
int check_ad_stride(const Problem& p, int ad_stride);

// Kernel launchers (one per translation unit); each returns a STEM_* status.
int launch_pool(const Problem& p, int ad_stride, const void* q, const void* k, const void* v,
                float* q_bar, float* k_bar, float* m_v, hipStream_t stream);
int launch_block_scores(const Problem& p, int ad_stride, const float* q_bar, const float* k_bar,
                        const float* m_v, float beta, float route_scale, bool fill_non_causal,
                        float* scores, hipStream_t stream);
int launch_group_scores(const Problem& p, const float* scores, int reduce, float* group_scores,
                        hipStream_t stream);
// heads = number of lists per row: Hq, or Hkv for group-shared lists
int launch_select(const Problem& p, int heads, const float* scores, const int32_t* budget,
                  int32_t n_sink, int32_t n_local, int32_t* counts, int32_t* indices, int32_t kmax,
                  hipStream_t stream);
int launch_score_select(const Problem& p, int ad_stride, const float* q_bar, const float* k_bar,
                        const float* m_v, float beta, float route_scale, const int32_t* budget,
                        int32_t n_sink, int32_t n_local, int32_t* counts, int32_t* indices,
                        int32_t kmax, float* debug_scores, hipStream_t stream);
int launch_sparse_attn(const Problem& p, const void* q, const void* k, const void* v,
                       const int32_t* counts, const int32_t* indices, int32_t kmax,
                       bool lists_per_kv_head, float softmax_scale, void* out, float* lse,
                       hipStream_t stream);

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? STEM_OK : STEM_ERR_HIP;
}

#if defined(__HIPCC__)
// Sequence of a global query-block row: the last s with row_start[s] <= r.  Wave-uniform.
__device__ __forceinline__ int seq_of_row(const SeqTable& t, int r) {
    int s = 0;
    for (int x = 1; x < t.batch; ++x) s = (r >= t.row_start[x]) ? x : s;
    return s;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
#endif

}  // namespace stem
