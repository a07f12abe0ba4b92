// Stage 1b (Algorithm 1 step 3a, Eq. 7): coarse Output-Aware Metric of every causal block pair,
//   scores[h, r, j] = route_scale * route(h, r, j) + beta * max(0, m_v[g, row0 + j]),
//   route = (1 / S) * sum over residue classes a < S of <q_bar[h, r, a], k_bar[g, row0 + j, S - 1 - a]>
// (S = 1: the plain product of the two block means).
//
// A small fp32 contraction over S * d per head and sequence, lower-triangular in (i, j).  It is
// kept in full fp32 arithmetic (no bf16 matrix cores) because stage 2 ranks these numbers and must
// reproduce the ranking of an fp64 evaluation except for genuine near-ties: the products run on
// the fp32 matrix instruction v_mfma_f32_32x32x2_f32.  64 x 64 output tiles, one 32 x 32 quadrant
// per wave.  The operands go through LDS row-major exactly as they lie in memory (16-byte stores
// of coalesced 16-byte loads); a lane then reads four consecutive depth positions of its row with
// one 16-byte read and feeds them to four products.  Which depth position a product step pairs is
// free as long as both operands agree, so step (u, x) takes position 8u + x from the lower half
// of the wave and 8u + 4 + x from the upper half.  The loads of the next slice are in flight
// during the products of the current one.  Tiles above the diagonal are only filled with -inf, or
// left alone if the caller does not want the rectangle completed (the selection never reads them).
#include "stem_common.h"

namespace stem {

constexpr int kTile = 64;
constexpr int kChunk = 32;                             // slice of d staged per step
constexpr int kScoreThreads = 256;

struct TileTable {
    int32_t tile_start[STEM_MAX_BATCH + 1];            // prefix sums of ceil(n_s / kTile)
};

__global__ __launch_bounds__(kScoreThreads) void block_scores_kernel(
    const float* __restrict__ q_bar, const float* __restrict__ k_bar, const float* __restrict__ m_v,
    float* __restrict__ scores, SeqTable seq, TileTable tiles, int R, int Rk, int NBmax, int G, int S,
    int d_log2, float beta, float route_scale, bool fill_non_causal) {
    // sequence and local row tile of this workgroup
    int s = 0;
    for (int x = 1; x < seq.batch; ++x) s = ((int)blockIdx.x >= tiles.tile_start[x]) ? x : s;
    const int row0 = seq.row_start[s];
    const int n_rows = seq.row_start[s + 1] - row0;    // query-block rows of this sequence in the call
    const int first = seq.first_block[s];              // block index of the first of them
    const int n = first + n_rows;                      // key blocks the call can see
    const int krow0 = seq.key_row_start[s];
    const int i0 = ((int)blockIdx.x - tiles.tile_start[s]) * kTile;   // first row of the tile, call-local
    const int j0 = blockIdx.y * kTile;
    const int h = blockIdx.z;
    const int g = h / G;
    const int tid = threadIdx.x;
    const int ti = tid >> 4, tj = tid & 15;            // 4 rows x 4 columns per thread

    float* out = scores + ((int64_t)h * R + row0) * NBmax;
    const float neg_inf = -__builtin_huge_valf();

    if (j0 > first + i0 + kTile - 1) {                 // entirely above the diagonal
        if (!fill_non_causal) return;
        const bool vec = (NBmax & 3) == 0;             // rows 16-byte aligned (the base is)
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int i = i0 + x * 16 + ti;            // a wave stores four rows of 256 contiguous bytes
            if (i >= n_rows) continue;
            const int j = j0 + tj * 4;
            if (vec && j + 3 < NBmax) {
                *reinterpret_cast<float4*>(out + (int64_t)i * NBmax + j) = make_float4(neg_inf, neg_inf, neg_inf, neg_inf);
            } else {
#pragma unroll
                for (int y = 0; y < 4; ++y)
                    if (j + y < NBmax) out[(int64_t)i * NBmax + j + y] = neg_inf;
            }
        }
        return;
    }

    // [row][k] with rows 144 bytes apart: the 16-byte reads of 16 consecutive rows fall on 16
    // different groups of four banks
    // two buffers per operand: one barrier per slice
    __shared__ __attribute__((aligned(16))) float a_s[2][kTile][kChunk + 4];
    __shared__ __attribute__((aligned(16))) float b_s[2][kTile][kChunk + 4];

    typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
    f32x16_t acc;
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[x] = 0.f;
    const int lane = tid & 63, wv = tid >> 6;
    const int col = lane & 31, hi = lane >> 5;
    const int wi = (wv >> 1) * 32, wj = (wv & 1) * 32; // this wave's quadrant of the tile

    const int d = 1 << d_log2;
    const int depth = S * d;                           // floats per pooled block
    const float* a_src = q_bar + ((int64_t)h * R + row0) * depth;
    const float* b_src = k_bar + ((int64_t)g * Rk + krow0) * depth;

    // 64 rows x 32 floats per operand and slice = 512 float4: two per thread and operand.  The
    // slices are fetched two groups (of two slices) ahead of their use, so at d = 128, S = 1 the
    // whole contraction is in flight before the first product and the memory latency is paid once
    // per tile, not once per slice; a group's registers are refilled as soon as it is staged.
    float4 av[2][2][2], bv[2][2][2];                   // [group parity][slice of the group][part]
    auto fetch = [&](int kc, float4 (&a)[2], float4 (&b)[2]) {
        // a slice lies inside one residue class a of the query block; its partner is class S-1-a
        const int kb = (S - 1 - (kc >> d_log2)) * d + (kc & (d - 1));
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + kScoreThreads * u;
            const int row = idx >> 3, c4 = (idx & 7) * 4;
            a[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            b[u] = a[u];
            if (i0 + row < n_rows) a[u] = *reinterpret_cast<const float4*>(a_src + (int64_t)(i0 + row) * depth + kc + c4);
            if (j0 + row < n) b[u] = *reinterpret_cast<const float4*>(b_src + (int64_t)(j0 + row) * depth + kb + c4);
        }
    };
    auto stage = [&](int buf, const float4 (&a)[2], const float4 (&b)[2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + kScoreThreads * u;
            const int row = idx >> 3, c4 = (idx & 7) * 4;
            *reinterpret_cast<float4*>(&a_s[buf][row][c4]) = a[u];
            *reinterpret_cast<float4*>(&b_s[buf][row][c4]) = b[u];
        }
    };
    auto products = [&](int buf) {
#pragma unroll
        for (int u = 0; u < kChunk / 8; ++u) {
            const float4 a = *reinterpret_cast<const float4*>(&a_s[buf][wi + col][u * 8 + hi * 4]);
            const float4 b = *reinterpret_cast<const float4*>(&b_s[buf][wj + col][u * 8 + hi * 4]);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
        }
    };
    // depth is a multiple of 64 (head sizes 64, 128, 256 times S): groups of two slices
    const int groups = depth / (2 * kChunk);
    auto fetch_group = [&](int g, int par) {
        fetch(g * 2 * kChunk, av[par][0], bv[par][0]);
        fetch(g * 2 * kChunk + kChunk, av[par][1], bv[par][1]);
    };
    fetch_group(0, 0);
    if (groups > 1) fetch_group(1, 1);
    stage(0, av[0][0], bv[0][0]);
    __syncthreads();
    // one group: slice 0 sits in LDS buffer 0; every barrier separates the last read of a buffer from
    // its next write (the buffer staged during a slice's products was last read before the previous barrier)
    auto one_group = [&](int g, int par) {
        stage(1, av[par][1], bv[par][1]);              // the group's second slice
        products(0);
        __syncthreads();
        const bool more = g + 1 < groups;
        if (more) stage(0, av[par ^ 1][0], bv[par ^ 1][0]);   // the next group's first slice
        if (g + 2 < groups) fetch_group(g + 2, par);   // this group's registers are free again
        products(1);
        __syncthreads();
    };
    for (int g = 0; g < groups; g += 2) {
        one_group(g, 0);
        if (g + 1 < groups) one_group(g + 1, 1);
    }

    // accumulator v of a lane: column wj + col, row wi + 8*(v/4) + 4*hi + v%4
    const int j = j0 + wj + col;
    const float mag = (j < n) ? beta * fmaxf(0.f, m_v[(int64_t)g * Rk + krow0 + j]) : 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = i0 + wi + 8 * (v >> 2) + 4 * hi + (v & 3);
        if (i >= n_rows || j >= NBmax) continue;
        out[(int64_t)i * NBmax + j] = (j <= first + i) ? fmaf(route_scale / (float)S, acc[v], mag) : neg_inf;
    }
}

int launch_block_scores(const Problem& p, int ad_stride, const float* q_bar, const float* k_bar,
                        const float* m_v, float beta, float route_scale, bool fill_non_causal,
                        float* scores, hipStream_t stream) {
    TileTable tiles;
    int total = 0;
    for (int s = 0; s <= STEM_MAX_BATCH; ++s) {
        tiles.tile_start[s] = total;
        if (s < p.batch) total += (p.seq.row_start[s + 1] - p.seq.row_start[s] + kTile - 1) / kTile;
    }
    if (total == 0) return STEM_OK;
    if (p.Hq > 65535) return STEM_ERR_UNSUPPORTED;
    dim3 grid(total, (p.NBmax + kTile - 1) / kTile, p.Hq), block(kScoreThreads);
    hipLaunchKernelGGL(block_scores_kernel, grid, block, 0, stream, q_bar, k_bar, m_v, scores, p.seq,
                       tiles, p.R, p.Rk, p.NBmax, p.G, ad_stride, __builtin_ctz(p.d), beta, route_scale,
                       fill_non_causal);
    return check_launch();
}

__global__ __launch_bounds__(256) void group_scores_scalar_kernel(const float* __restrict__ scores,
                                                                  float* __restrict__ group_scores,
                                                                  int64_t per_head, int G, int take_mean,
                                                                  int64_t total) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int64_t g = idx / per_head, off = idx - g * per_head;
    const float* src = scores + g * G * per_head + off;
    float acc = src[0];
    for (int x = 1; x < G; ++x) {
        const float y = src[(int64_t)x * per_head];
        acc = take_mean ? acc + y : fmaxf(acc, y);
    }
    group_scores[idx] = take_mean ? acc / (float)G : acc;
}

// Group-shared selection for grouped-query attention: the metric of a KV head is the maximum or
// the mean of the metric of its G query heads.  One thread per four consecutive key blocks; the G
// values are combined in head order (deterministic fp32).
__global__ __launch_bounds__(256) void group_scores_kernel(const float* __restrict__ scores,
                                                           float* __restrict__ group_scores,
                                                           int64_t per_head, int G, int take_mean,
                                                           int64_t total) {
    const int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;   // per_head % 4 == 0
    if (idx >= total) return;
    const int64_t g = idx / per_head, off = idx - g * per_head;
    const float* src = scores + g * G * per_head + off;
    float4 acc = *reinterpret_cast<const float4*>(src);
    for (int x = 1; x < G; ++x) {
        const float4 y = *reinterpret_cast<const float4*>(src + (int64_t)x * per_head);
        acc.x = take_mean ? acc.x + y.x : fmaxf(acc.x, y.x);
        acc.y = take_mean ? acc.y + y.y : fmaxf(acc.y, y.y);
        acc.z = take_mean ? acc.z + y.z : fmaxf(acc.z, y.z);
        acc.w = take_mean ? acc.w + y.w : fmaxf(acc.w, y.w);
    }
    if (take_mean) {
        const float inv = (float)G;
        acc.x /= inv; acc.y /= inv; acc.z /= inv; acc.w /= inv;
    }
    *reinterpret_cast<float4*>(group_scores + idx) = acc;
}

int launch_group_scores(const Problem& p, const float* scores, int reduce, float* group_scores,
                        hipStream_t stream) {
    const int64_t per_head = (int64_t)p.R * p.NBmax;
    const int64_t total = per_head * p.Hkv;
    if (total == 0) return STEM_OK;
    // four elements per thread when they cannot straddle two heads and the rows are 16-byte
    // aligned, else one
    if (per_head % 4 || (reinterpret_cast<uintptr_t>(scores) | reinterpret_cast<uintptr_t>(group_scores)) & 15) {
        const int64_t blocks = (total + 255) / 256;
        if (blocks > 0x7fffffff) return STEM_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(group_scores_scalar_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, scores,
                           group_scores, per_head, p.G, reduce == STEM_GROUP_MEAN, total);
        return check_launch();
    }
    const int64_t blocks = (total / 4 + 255) / 256;
    if (blocks > 0x7fffffff) return STEM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(group_scores_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, scores, group_scores,
                       per_head, p.G, reduce == STEM_GROUP_MEAN, total);
    return check_launch();
}

}  // namespace stem
