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
// of the wave and 8u + 4 + x from the upper half.
//
// A tile is only 64 products per wave, less than the latency of fetching its operands, so the
// workgroups are persistent: as many as fit the chip at once, each walking every P-th tile of the
// list of causal tiles.  The operand slices of all its tiles form one stream that is fetched two
// groups (of two 32-deep slices) ahead of the products, across tile boundaries, so the memory
// latency is paid once per workgroup, not once per tile.  Tiles above the diagonal are never
// computed; a second kernel fills them with -inf if the caller wants the rectangle completed (the
// selection never reads them).
#include <type_traits>

#include "stem_common.h"

namespace stem {

constexpr int kTile = 64;
constexpr int kChunk = 32;                             // slice of d staged per step
constexpr int kScoreThreads = 256;
constexpr int kScoreWorkgroupsPerCU = 4;               // what the LDS buffers allow

struct TileTable {
    int32_t tile_start[STEM_MAX_BATCH + 1];            // prefix sums of ceil(n_s / kTile): row tiles
    int32_t causal_start[STEM_MAX_BATCH + 1];          // prefix sums of the causal tiles of one head
};

// causal tiles of row tile `it` of a sequence whose call starts at block `first`: column tiles 0 ..
// (first + 64 it + 63) / 64, as far as the score tensor has columns
__host__ __device__ inline int causal_tiles_of_row_tile(int it, int first, int NBmax) {
    const int last = (first + it * kTile + kTile - 1) / kTile;
    const int cols = (NBmax + kTile - 1) / kTile;
    return (last < cols - 1 ? last : cols - 1) + 1;
}

struct ScoreTile {                                     // what one tile's work needs; wave-uniform
    const float* a_src;                                // q_bar rows of the sequence, this head
    const float* b_src;                                // k_bar rows of the sequence, this KV head
    const float* m_v;                                  // m_v of the sequence, this KV head
    float* out;                                        // scores rows of the sequence, this head
    int i0, j0, n_rows, n, first;
};

__global__ __launch_bounds__(kScoreThreads) void block_scores_kernel(
    const float* __restrict__ q_bar, const float* __restrict__ k_bar, const float* __restrict__ m_v,
    float* __restrict__ scores, SeqTable seq, TileTable tiles, int tiles_per_head, int total_tiles, int R,
    int Rk, int NBmax, int G, int S, int d_log2, float beta, float route_scale) {
    const int tid = threadIdx.x;
    const int d = 1 << d_log2;
    const int depth = S * d;                           // floats per pooled block
    const float neg_inf = -__builtin_huge_valf();

    // tile f of the list: head-major, then sequence, row tile, column tile
    auto decode = [&](int f) {
        const int h = f / tiles_per_head;
        int x = f - h * tiles_per_head;
        int s = 0;
        for (int y = 1; y < seq.batch; ++y) s = (x >= tiles.causal_start[y]) ? y : s;
        x -= tiles.causal_start[s];
        const int row0 = seq.row_start[s];
        const int first = seq.first_block[s];          // block index of the sequence's first row in the call
        int it = 0;
        for (int c = causal_tiles_of_row_tile(0, first, NBmax); x >= c; c = causal_tiles_of_row_tile(it, first, NBmax)) {
            x -= c;
            ++it;
        }
        const int g = h / G;
        ScoreTile t;
        t.n_rows = seq.row_start[s + 1] - row0;        // query-block rows of this sequence in the call
        t.first = first;
        t.n = first + t.n_rows;                        // key blocks the call can see
        t.i0 = it * kTile;
        t.j0 = x * kTile;
        t.a_src = q_bar + ((int64_t)h * R + row0) * depth;
        t.b_src = k_bar + ((int64_t)g * Rk + seq.key_row_start[s]) * depth;
        t.m_v = m_v + (int64_t)g * Rk + seq.key_row_start[s];
        t.out = scores + ((int64_t)h * R + row0) * NBmax;
        return t;
    };

    // [row][k] with rows 144 bytes apart: the 16-byte reads of 16 consecutive rows fall on 16
    // different groups of four banks
    // two buffers per operand: one barrier per slice
    __shared__ __attribute__((aligned(16))) float a_s[2][kTile][kChunk + 4];
    __shared__ __attribute__((aligned(16))) float b_s[2][kTile][kChunk + 4];

    typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
    f32x16_t acc;
    const int lane = tid & 63, wv = tid >> 6;
    const int col = lane & 31, hi = lane >> 5;
    const int wi = (wv >> 1) * 32, wj = (wv & 1) * 32; // this wave's quadrant of the tile

    // 64 rows x 32 floats per operand and slice = 512 float4: two per thread and operand
    float4 av[2][2][2], bv[2][2][2];                   // [group parity][slice of the group][part]
    auto fetch = [&](const ScoreTile& t, int kc, float4 (&a)[2], float4 (&b)[2]) {
        // a slice lies inside one residue class a of the query block; its partner is class S-1-a
        const int kb = (S - 1 - (kc >> d_log2)) * d + (kc & (d - 1));
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + kScoreThreads * u;
            const int row = idx >> 3, c4 = (idx & 7) * 4;
            a[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            b[u] = a[u];
            if (t.i0 + row < t.n_rows) a[u] = *reinterpret_cast<const float4*>(t.a_src + (int64_t)(t.i0 + row) * depth + kc + c4);
            if (t.j0 + row < t.n) b[u] = *reinterpret_cast<const float4*>(t.b_src + (int64_t)(t.j0 + row) * depth + kb + c4);
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

    // this workgroup's tiles: blockIdx.x, blockIdx.x + P, ...; depth is a multiple of 64 (head
    // sizes 64, 128, 256 times S), so a tile is `groups` groups of two slices
    const int P = gridDim.x;
    const int my_tiles = (total_tiles - (int)blockIdx.x + P - 1) / P;
    const int groups = depth / (2 * kChunk);
    const int n_groups = my_tiles * groups;            // the workgroup's whole stream

    // the fetching side runs two groups ahead of the products and has its own place in the list
    int f_tile = 0, f_group = 0;
    ScoreTile ft = decode(blockIdx.x);
    auto fetch_next = [&](auto par_tag) {          // the register set is a compile-time choice
        constexpr int par = decltype(par_tag)::value;
        fetch(ft, f_group * 2 * kChunk, av[par][0], bv[par][0]);
        fetch(ft, f_group * 2 * kChunk + kChunk, av[par][1], bv[par][1]);
        if (++f_group == groups) {
            f_group = 0;
            if (++f_tile < my_tiles) ft = decode(blockIdx.x + f_tile * P);
        }
    };
    using Even = std::integral_constant<int, 0>;
    using Odd = std::integral_constant<int, 1>;
    fetch_next(Even{});
    if (n_groups > 1) fetch_next(Odd{});
    stage(0, av[0][0], bv[0][0]);
    __syncthreads();

    ScoreTile ct = decode(blockIdx.x);
    int c_tile = 0, c_group = 0;
    float mag = 0.f;
    auto one_group = [&](int gi, auto par_tag) {
        constexpr int par = decltype(par_tag)::value;
        if (c_group == 0) {
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[x] = 0.f;
            // the value-magnitude term of this lane's column, asked for now, used after the tile's last product
            const int j = ct.j0 + wj + col;
            mag = (j < ct.n) ? ct.m_v[j] : 0.f;
        }
        // Slice 0 of the group sits in LDS buffer 0.  Every barrier separates the last read of a buffer
        // from its next write (the buffer staged during a slice's products was last read before the
        // previous barrier); a group's registers are refilled as soon as both its slices are staged.
        stage(1, av[par][1], bv[par][1]);              // the group's second slice
        products(0);
        __syncthreads();
        if (gi + 1 < n_groups) stage(0, av[par ^ 1][0], bv[par ^ 1][0]);   // the next group's first slice
        if (gi + 2 < n_groups) fetch_next(par_tag);
        products(1);
        __syncthreads();
        if (++c_group == groups) {
            // accumulator v of a lane: column wj + col, row wi + 8*(v/4) + 4*hi + v%4
            const int j = ct.j0 + wj + col;
            const float m = beta * fmaxf(0.f, mag);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = ct.i0 + wi + 8 * (v >> 2) + 4 * hi + (v & 3);
                if (i >= ct.n_rows || j >= NBmax) continue;
                ct.out[(int64_t)i * NBmax + j] = (j <= ct.first + i) ? fmaf(route_scale / (float)S, acc[v], m) : neg_inf;
            }
            c_group = 0;
            if (++c_tile < my_tiles) ct = decode(blockIdx.x + c_tile * P);
        }
    };
    for (int gi = 0; gi < n_groups; gi += 2) {
        one_group(gi, Even{});
        if (gi + 1 < n_groups) one_group(gi + 1, Odd{});
    }
}

// The tiles entirely above the diagonal, for callers that want the whole rectangle defined.
__global__ __launch_bounds__(kScoreThreads) void fill_non_causal_kernel(float* __restrict__ scores, SeqTable seq,
                                                                        TileTable tiles, int R, int NBmax) {
    int s = 0;
    for (int x = 1; x < seq.batch; ++x) s = ((int)blockIdx.x >= tiles.tile_start[x]) ? x : s;
    const int row0 = seq.row_start[s];
    const int n_rows = seq.row_start[s + 1] - row0;
    const int first = seq.first_block[s];
    const int i0 = ((int)blockIdx.x - tiles.tile_start[s]) * kTile;   // first row of the tile, call-local
    const int j0 = blockIdx.y * kTile;
    if (j0 <= first + i0 + kTile - 1) return;          // a causal tile: the score kernel writes all of it
    const int h = blockIdx.z;
    const int tid = threadIdx.x;
    const int ti = tid >> 4, tj = tid & 15;            // 4 rows x 4 columns per thread
    float* out = scores + ((int64_t)h * R + row0) * NBmax;
    const float neg_inf = -__builtin_huge_valf();
    const bool vec = (NBmax & 3) == 0;                 // rows 16-byte aligned (the base is)
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int i = i0 + x * 16 + ti;                // a wave stores four rows of 256 contiguous bytes
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
}

int launch_block_scores(const Problem& p, int ad_stride, const float* q_bar, const float* k_bar,
                        const float* m_v, float beta, float route_scale, bool fill_non_causal,
                        float* scores, hipStream_t stream) {
    TileTable tiles;
    int row_tiles = 0, causal = 0;
    for (int s = 0; s <= STEM_MAX_BATCH; ++s) {
        tiles.tile_start[s] = row_tiles;
        tiles.causal_start[s] = causal;
        if (s < p.batch) {
            const int nt = (p.seq.row_start[s + 1] - p.seq.row_start[s] + kTile - 1) / kTile;
            row_tiles += nt;
            for (int it = 0; it < nt; ++it) causal += causal_tiles_of_row_tile(it, p.seq.first_block[s], p.NBmax);
        }
    }
    if (row_tiles == 0) return STEM_OK;
    if (p.Hq > 65535 || (int64_t)causal * p.Hq > 0x7fffffff) return STEM_ERR_UNSUPPORTED;
    int device = 0, cus = 0;
    if (hipGetDevice(&device) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0)
        return STEM_ERR_HIP;
    const int total = causal * p.Hq;
    const int workgroups = total < cus * kScoreWorkgroupsPerCU ? total : cus * kScoreWorkgroupsPerCU;
    hipLaunchKernelGGL(block_scores_kernel, dim3(workgroups), dim3(kScoreThreads), 0, stream, q_bar, k_bar, m_v,
                       scores, p.seq, tiles, causal, total, p.R, p.Rk, p.NBmax, p.G, ad_stride,
                       __builtin_ctz(p.d), beta, route_scale);
    if (fill_non_causal) {
        dim3 grid(row_tiles, (p.NBmax + kTile - 1) / kTile, p.Hq);
        hipLaunchKernelGGL(fill_non_causal_kernel, grid, dim3(kScoreThreads), 0, stream, scores, p.seq, tiles,
                           p.R, p.NBmax);
    }
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
