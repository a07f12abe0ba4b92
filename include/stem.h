/*
 * stem.h - C ABI of the MI355X (gfx950) implementation of Stem's block-sparse prefill attention.
 *
 * The three stages of the method (Overall Algorithm section, Algorithm 1):
 *   1. stem_estimate     block-wise pooling of Q, K and of the value magnitude, then the coarse
 *                        Output-Aware Metric of every causal (query block, key block) pair
 *                        (Algorithm 1 step 1 and step 3a, Eq. 7);
 *   2. stem_select       Token Position-Decay top-k(i) of each metric row with the initial and
 *                        local windows always kept (Eq. 3, Algorithm 1 steps 3b-3c, Implementation
 *                        Details);
 *   3. stem_sparse_attn  exact softmax attention over the selected key blocks only
 *                        (Algorithm 1 step 3d).
 *
 * Conventions shared by every entry point
 *   - Every function returns an int status: STEM_OK (0) or a negative STEM_ERR_* code.  Arguments
 *     are checked on the host before anything is enqueued; on an error nothing was launched.
 *   - Pointers are DEVICE pointers unless their name starts with host_.  The caller owns every
 *     buffer (inputs, outputs, workspace).  The library allocates nothing, keeps no state, does not
 *     synchronise, and enqueues all work on the caller's stream (`hip_stream` is a hipStream_t; NULL
 *     is the default stream).  Buffers must stay alive until that work has finished.
 *   - Q is [T, Hq, d], K and V are [T, Hkv, d], bf16, packed over `batch` sequences whose token
 *     ranges are host_cu_seqlens[s] .. host_cu_seqlens[s+1].  The last dimension is contiguous;
 *     token and head strides are given in elements and must be multiples of 8, and base pointers
 *     must be 16-byte aligned.  Query head h reads KV head h / (Hq / Hkv).
 *   - A sequence of len tokens has ceil(len / B) blocks; the last block may be partial.  Query-block
 *     rows of all sequences are numbered consecutively: R = sum of blocks ("rows"), NBmax = the
 *     longest sequence in blocks.  Key-block indices are 0-based and local to the row's sequence;
 *     row i of a sequence may use key blocks 0..i.
 *   - Chunked pre-filling (a long prompt processed piece by piece against its growing KV cache):
 *     with host_chunk_start / host_chunk_end set, a call covers of sequence s only the queries at
 *     positions chunk_start[s] .. chunk_end[s] - 1 (relative to the sequence's first token) and the
 *     keys before chunk_end[s].  Then Q, O and lse hold the chunks' tokens only, packed in sequence
 *     order (T = sum of chunk lengths), while K and V keep the layout given by host_cu_seqlens
 *     (rows at or after chunk_end[s] are not read).  R counts the chunks' query blocks, NBmax the
 *     most key blocks a row of the call can see, and rows keep their block index i inside the
 *     sequence for the schedule, the causal limit and the windows, so the chunks of a prompt give
 *     the rows of the one-piece call.  chunk_start must be a multiple of B, chunk_end a multiple
 *     of B or the sequence's length; an empty chunk (start == end) contributes nothing.
 *   - Q, K and V are expected to hold finite values.  An inf or NaN in them is not detected: it
 *     spreads as IEEE arithmetic spreads it (a non-finite key or value makes the output rows that
 *     attend to it non-finite, a non-finite pooled score is ranked by its bit pattern), and
 *     affects nothing else; no entry point reads or writes out of bounds or hangs because of it.
 *   - Supported: head_dim 64, 128 or 256; block_size 64 or 128; 1 <= batch <= STEM_MAX_BATCH; Hq a
 *     multiple of Hkv; at most STEM_MAX_BLOCKS blocks per sequence.
 */
#ifndef STEM_H
#define STEM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STEM_OK                 0
#define STEM_ERR_INVALID_ARG   (-1)  /* null pointer, bad size, misaligned pointer or stride       */
#define STEM_ERR_UNSUPPORTED   (-2)  /* a valid request this build has no kernel for               */
#define STEM_ERR_WORKSPACE     (-3)  /* workspace_bytes smaller than stem_workspace_bytes reports  */
#define STEM_ERR_HIP           (-4)  /* the HIP runtime refused a launch                           */

#define STEM_MAX_BATCH   64
#define STEM_MAX_BLOCKS  4096        /* key blocks per sequence (512K tokens at B = 128)           */

typedef struct stem_shape {
    int32_t num_q_heads;             /* Hq                                                          */
    int32_t num_kv_heads;            /* Hkv, divides Hq                                             */
    int32_t head_dim;                /* d = 64, 128 or 256                                          */
    int32_t block_size;              /* B = 64 or 128 (the paper fixes 128)                         */
    int32_t batch;                   /* number of packed sequences                                  */
    const int32_t* host_cu_seqlens;  /* HOST [batch+1], cu[0] = 0, non-decreasing; read during call */
    int64_t q_stride_token;          /* elements between consecutive tokens of Q (and of O)         */
    int64_t q_stride_head;           /* elements between consecutive heads of Q (and of O)          */
    int64_t kv_stride_token;         /* same for K and V (they share strides)                       */
    int64_t kv_stride_head;
    const int32_t* host_chunk_start; /* HOST [batch] or NULL: first query position of the call      */
    const int32_t* host_chunk_end;   /* HOST [batch] or NULL (both or neither): one past the last   */
} stem_shape;

/* Library version: major * 10000 + minor * 100 + patch. */
int stem_version(void);

/* Static, NUL-terminated description of a status code. */
const char* stem_strerror(int status);

/* R (query-block rows of the call) and NBmax (most key blocks a row can see: the blocks of the
 * longest sequence, or up to the latest chunk end) of a shape. */
int stem_rows(const stem_shape* shape, int32_t* host_total_rows, int32_t* host_max_blocks);

/*
 * ad_stride S, taken by the stage-1 entry points: the stride of the anti-diagonal sample that the
 * pooled routing term stands for (Algorithm 1 steps 1 and 3a).  A block keeps S partial means,
 * one per residue class of the in-block token position modulo S, and the routing term of a block
 * pair is
 *     route = (1 / S) * sum over a < S of <q_bar[.., a, :], k_bar[.., S - 1 - a, :]>,
 * the mean over the S anti-diagonal classes of the class's mean logit <Q_r, K_c> (r in class a, c in
 * class S - 1 - a).  On full blocks that is the mean of <Q_r, K_c> over all positions with
 * (r + c) mod S = S - 1; on a partial last block each class is normalised by its own number of
 * valid tokens (pooling comes first, the product second, as in Algorithm 1) and a class without
 * valid tokens contributes 0.
 * S = 1 is block-mean pooling (one vector per block, the 2 N^2 d / B^2 metric cost of the
 * Complexity Analysis); larger S samples the block's logits more finely at S times the cost.
 * Supported: S in {1, 2, 4, 8, 16}; other divisors of B return STEM_ERR_UNSUPPORTED, values that
 * do not divide B or are < 1 STEM_ERR_INVALID_ARG.
 */

/* Bytes of device workspace stem_estimate / stem_pool need for this shape and ad_stride S.
 * Layout (fp32), Rk = blocks of all sequences (whole sequences, whatever the chunk):
 *   k_bar [Hkv, Rk, S, d] | m_v [Hkv, Rk] | q_bar [Hq, R, S, d]   (each part 256-byte aligned).
 * The key parts come first and do not depend on the chunk: a caller that keeps one workspace
 * (sized for the largest chunk) across the chunks of a prompt keeps the pooled keys of earlier
 * chunks, and stem_pool only pools the blocks of the current chunk. */
int stem_workspace_bytes(const stem_shape* shape, int32_t ad_stride, size_t* host_bytes);

/* Byte offsets of the three workspace parts (for callers that want to look at them). */
int stem_workspace_layout(const stem_shape* shape, int32_t ad_stride, size_t* host_q_bar_offset,
                          size_t* host_k_bar_offset, size_t* host_m_v_offset);

/*
 * Token Position-Decay schedule, Eq. 3 in block units, on the host.
 * For the 0-based row i of a sequence with n blocks and start budget ks = host_k_start_blocks[s]:
 *     k(i)     = floor( ks - (ks * (1 - mu) / n) * (i + 1) + 1e-9 )
 *     k_eff(i) = min( i + 1, max( k(i), k_min, |forced(i)| ) )
 * where forced(i) = first n_sink blocks united with the last n_local causal blocks (diagonal
 * included).  n counts the whole sequence also when the call covers a chunk of it (whose rows
 * keep their index i).  mu = 1 gives the uniform top-k control.  Writes host_budget[R] and, if not NULL,
 * the largest entry to *host_kmax.  Requires 0 < mu <= 1, ks >= 0, k_min, n_sink, n_local >= 0.
 * (n_local = 0 is accepted here as plain arithmetic - rows may then get a budget of 0 - but the
 * selection entry points require n_local >= 1 and raise such rows to their forced blocks.)
 */
int stem_budget_schedule(const stem_shape* shape, const double* host_k_start_blocks, double mu,
                         int32_t k_min, int32_t n_sink, int32_t n_local,
                         int32_t* host_budget, int32_t* host_kmax);

/*
 * Algorithm 1 step 1: pooled block representations into the workspace (layout above), for the
 * blocks of the call's chunks (all blocks without chunks).  With kr = the block's row among all
 * blocks of all sequences:
 *   q_bar[h, r, a, :] = mean of Q[t, h, :] over the valid tokens t of row r's block whose in-block
 *                       position is congruent to a modulo S (zeros if there is none)     (fp32)
 *   k_bar[g, kr, a, :] = the same for K
 *   m_v[g, kr]        = max over the block's valid tokens of ln ||V[t, g, :]||_2  (-inf if all zero)
 */
int stem_pool(const stem_shape* shape, const void* q, const void* k, const void* v,
              int32_t ad_stride, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Algorithm 1 step 3a, Eq. 7, from a workspace pooled with the same ad_stride:
 *   scores[h, r, j] = route_scale * route(h, r, j) + beta * max(0, m_v[g, row0(r) + j])
 * for 0 <= j <= i(r), with route as defined above from q_bar[h, r] and k_bar[g, row0(r) + j].
 * scores is fp32 [Hq, R, NBmax].
 * route_scale = 1 is Eq. 7 as printed; 1/sqrt(d) gives the scaling of Eq. 6.
 * fill_non_causal = 1: every entry i(r) < j < NBmax is written as -inf (the whole rectangle is
 * defined).  fill_non_causal = 0: the kernel works in tiles of 64 rows x 64 key blocks and does not
 * touch the tiles that hold no causal pair; inside the other tiles j > i(r) still reads -inf, beyond
 * them the buffer keeps whatever it held.  stem_select never reads an entry with j > i(r), so the
 * lists are the same either way; at 128K this halves what stage 1 writes (134 -> 67 MB).
 */
int stem_block_scores(const stem_shape* shape, const void* workspace, size_t workspace_bytes,
                      int32_t ad_stride, float beta, float route_scale, int32_t fill_non_causal,
                      float* scores, void* hip_stream);

/* Stage 1 = stem_pool followed by stem_block_scores with the same ad_stride. */
int stem_estimate(const stem_shape* shape, const void* q, const void* k, const void* v,
                  float beta, float route_scale, int32_t ad_stride, int32_t fill_non_causal,
                  float* scores, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * stem_estimate (with fill_non_causal = 1) for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and
 * same scores as stem_estimate, but the pooled block representations live in an array inside the library's code
 * object (STEM_STATIC_WORKSPACE_BYTES per GPU, held from module load until the process ends) instead
 * of a caller-provided workspace.  The call allocates nothing and frees nothing.
 *   - STEM_ERR_WORKSPACE if stem_workspace_bytes(shape, ad_stride) exceeds STEM_STATIC_WORKSPACE_BYTES
 *     (32 MiB: the 128K-token layer with 32/8 heads of size 128 needs 21 MB at ad_stride 1);
 *     STEM_ERR_UNSUPPORTED for chunked shapes (a chunk's scores need the pooled keys of earlier
 *     calls, which a shared array cannot promise); STEM_ERR_HIP if the array's address cannot be found.
 *   - The first call on a device looks the array's device address up (once per device, kept
 *     afterwards); make that first call outside graph capture.
 *   - All calls on one GPU share that GPU's array, which keeps the last call's pooled vectors.
 *     Nothing in it has to start at zero (every call writes all it reads), but two calls that
 *     overlap in time on one GPU, on different streams or from different threads, race on it.
 */
#define STEM_STATIC_WORKSPACE_BYTES (32u << 20)
int stem_estimate_static(const stem_shape* shape, const void* q, const void* k, const void* v,
                         float beta, float route_scale, int32_t ad_stride, float* scores,
                         void* hip_stream);

/*
 * Group-shared selection for grouped-query attention (an extension: the paper derives the method
 * per head).  Reduces the metric over the G = Hq / Hkv query heads of each KV head:
 *   group_scores[g, r, j] = max (STEM_GROUP_MAX) or mean (STEM_GROUP_MEAN) over h in g*G .. g*G+G-1
 *                           of scores[h, r, j]                 (-inf stays -inf; entries that
 *                           stem_block_scores left unwritten stay unspecified, and unread)
 * scores is fp32 [Hq, R, NBmax], group_scores fp32 [Hkv, R, NBmax].  Selecting from group_scores
 * with lists_per_kv_head = 1 gives one list per (KV head, row), which stem_sparse_attn then uses
 * for all G heads of the group: G times fewer lists, and the heads of a group read the same K/V
 * blocks at the same time.
 */
#define STEM_GROUP_MAX   0
#define STEM_GROUP_MEAN  1
int stem_group_scores(const stem_shape* shape, const float* scores, int32_t reduce,
                      float* group_scores, void* hip_stream);

/*
 * Stage 2, Algorithm 1 step 3c with forced windows.  For every head h and row r (local index i):
 *   k = min(i + 1, max(budget[r], |forced(i)|));
 *   list = forced(i) united with the k - |forced(i)| best-scoring other causal blocks, equal
 *          scores going to the lower block index; written ascending.
 * budget is device int32 [R] (from stem_budget_schedule, copied by the caller).
 * counts is device int32 [Hq, R]; indices is device int32 [Hq, R, kmax], padded with -1.
 * With lists_per_kv_head = 1 "head" means KV head: scores is [Hkv, R, NBmax] (from
 * stem_group_scores), counts [Hkv, R], indices [Hkv, R, kmax]; 0 is the paper's per-head selection.
 * kmax is the row pitch of indices.  It must be at least n_sink + n_local (or at least NBmax), so the
 * forced blocks always fit; a row whose budget exceeds kmax is cut to kmax blocks (k = min(k, kmax)).
 * n_sink >= 0 and n_local >= 1: the method always keeps the diagonal block, so every list holds
 * block i and no row comes out empty, whatever the budget array says (STEM_ERR_INVALID_ARG otherwise).
 */
int stem_select(const stem_shape* shape, const float* scores, const int32_t* budget,
                int32_t n_sink, int32_t n_local, int32_t lists_per_kv_head, int32_t* counts,
                int32_t* indices, int32_t kmax, void* hip_stream);

/*
 * Stages 1 and 2 in one call that never writes the score tensor: stem_pool, then one kernel that
 * computes the metric of a band of rows into on-chip memory and selects from there.  Same results
 * as stem_estimate followed by stem_select with lists_per_kv_head = 0, up to the rounding order of
 * the fp32 score sums (near-ties may resolve differently).  debug_scores, if not NULL, is a device
 * fp32 [Hq, R, NBmax] buffer that receives the scores the selection saw (for checking; it defeats
 * the purpose otherwise).  Arguments as for the two calls it replaces.
 */
int stem_estimate_select(const stem_shape* shape, const void* q, const void* k, const void* v,
                         float beta, float route_scale, int32_t ad_stride, const int32_t* budget,
                         int32_t n_sink, int32_t n_local, int32_t* counts, int32_t* indices,
                         int32_t kmax, float* debug_scores, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/*
 * Stage 3, Algorithm 1 step 3d: for every head h, row r and valid query token t of the row's block
 *   out[t, h, :] = sum_u softmax_u( softmax_scale * <Q[t,h], K[u,g]> ) V[u,g]
 * over the tokens u <= t of the key blocks indices[h, r, 0 .. counts[h,r]) (of indices[h / G, r, ..]
 * with counts [Hkv, R] and indices [Hkv, R, kmax] if lists_per_kv_head = 1).  bf16 inputs, bf16 MFMA
 * products with fp32 accumulation, fp32 softmax, bf16 output with Q's strides.  softmax_scale > 0.
 * lse (device fp32 [Hq, T], may be NULL) receives log sum_u exp(softmax_scale * <Q,K>) per query,
 * accurate to 4e-3 absolute: the softmax runs in fp32, but the row sum is taken over the
 * probabilities as the second matrix product uses them, rounded to bf16 (each within 2^-8 of its
 * fp32 value), which makes every output row an exact convex combination of value rows; a caller
 * that merges partial results through lse inherits that bound.  A query with no visible key gets
 * lse = -inf.
 * Any list is accepted, not only stem_select's, provided each row's list is ascending, causal
 * (entries <= i) and holds the diagonal block i.  Lists are not validated: entries outside 0..i
 * contribute nothing (they cost the time of a block, never an out-of-bounds access); a row with
 * no usable entry yields zeros and lse = -inf.  STEM_ERR_UNSUPPORTED if one sequence of one KV
 * head spans 2 GiB or more, i.e. (tokens - 1) * kv_stride_token * 2 + 256 bytes > 2^31 - 1.
 */
int stem_sparse_attn(const stem_shape* shape, const void* q, const void* k, const void* v,
                     const int32_t* counts, const int32_t* indices, int32_t kmax,
                     int32_t lists_per_kv_head, float softmax_scale, void* out, float* lse,
                     void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* STEM_H */
