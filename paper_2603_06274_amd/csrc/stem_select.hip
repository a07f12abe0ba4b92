// Stage 2 (Algorithm 1 step 3c; forced windows of Implementation Details): per-row top-k(i).
//
// One 64-lane wavefront owns one (head, row).  The row's candidate scores are held in registers as
// order-preserving 32-bit keys, lane-strided (element e of lane l is key block fs + 64 e + l).  The
// k-th largest key is found exactly by a bitwise search (at most 32 steps; it stops as soon as a
// prefix separates exactly the wanted number of keys) whose counts come from wave ballots
// (scalar popcounts, no atomics, no LDS), and the list is then emitted in ascending block order by
// ballot prefix compaction: forced blocks, every key above the threshold, and the lowest-indexed
// keys equal to it until the budget is met.  The result is therefore deterministic and ties go to
// the lower block index.
#include <type_traits>

#include "stem_common.h"

namespace stem {

constexpr int kSelectThreads = 256;

__device__ __forceinline__ uint32_t ordered_key(float x) {
    uint32_t u = __float_as_uint(x + 0.0f);            // -0 -> +0 so equal floats give equal keys
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int lanes_below(uint64_t mask, int lane) {
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// The selection of one row by one wavefront.  load(j) returns the score of key block j of the row
// (any memory); i is the row's block index in its sequence.
template <int ITEMS, typename Load>
__device__ __forceinline__ void select_row(Load load, int i, int row_budget, int n_sink, int n_local,
                                           int kmax, int lane, int32_t* __restrict__ out,
                                           int32_t* __restrict__ count_out) {
    const int fs = min(n_sink, i + 1);                 // forced head: blocks [0, fs)
    const int fe = max(fs, i - n_local + 1);           // forced tail: blocks [fe, i]
    const int nfree = fe - fs;
    const int forced = i + 1 - nfree;
    int k = max(row_budget, forced);
    k = min(k, min(i + 1, kmax));
    const int need = max(0, k - forced);               // free blocks to pick, <= nfree

    // Groups of 64 candidates beyond the row's free range hold nothing.  The loops over the items
    // run to a compile-time bound N picked per row from a few sizes (a wave-uniform choice), so a
    // short row costs about what it holds and no loop carries a test per item.
    const int items = (nfree + 63) >> 6;
    const bool take_all = (need >= nfree);
    int base = fs;
    for (int j = lane; j < fs; j += 64) out[j] = j;    // forced head
    auto run = [&](auto bound) {
        constexpr int N = decltype(bound)::value;
        uint32_t key[N];
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const int j = fs + e * 64 + lane;
            key[e] = (j < fe) ? ordered_key(load(j)) : 0u; // 0 sorts below every real key
        }
        uint32_t tau = 0;
        int n_eq = 0;                                  // keys equal to tau that are still needed
        if (need > 0 && need < nfree) {
            bool exact = false;                        // exactly `need` keys are >= tau
            for (int bit = 31; bit >= 0 && !exact; --bit) {
                const uint32_t cand = tau | (1u << bit);
                int cnt = 0;
#pragma unroll
                for (int e = 0; e < N; ++e) cnt += __popcll(__ballot(key[e] >= cand));
                if (cnt >= need) tau = cand;
                exact = cnt == need;
            }
            if (exact) {
                // the keys >= tau are the answer whatever the remaining bits of the k-th largest
                // key are: express it as "above tau - 1, none equal" (tau >= 1: a bit was just set)
                tau -= 1;
            } else {
                int above = 0;
#pragma unroll
                for (int e = 0; e < N; ++e) above += __popcll(__ballot(key[e] > tau));
                n_eq = need - above;
            }
        }
        // chosen free blocks, ascending
        if (need > 0) {
            int eq_seen = 0;
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const int j = fs + e * 64 + lane;
                const bool valid = j < fe;
                const bool eq = valid && !take_all && key[e] == tau;
                const uint64_t eq_mask = __ballot(eq);
                const bool take = valid && (take_all || key[e] > tau ||
                                            (eq && eq_seen + lanes_below(eq_mask, lane) < n_eq));
                const uint64_t take_mask = __ballot(take);
                if (take) out[base + lanes_below(take_mask, lane)] = j;
                base += __popcll(take_mask);
                eq_seen += __popcll(eq_mask);
            }
        }
    };
    // bounds: an eighth, a quarter, a half, three quarters of ITEMS, and ITEMS
    constexpr int kN1 = ITEMS / 8 > 0 ? ITEMS / 8 : 1, kN2 = ITEMS / 4 > 0 ? ITEMS / 4 : 1, kN4 = ITEMS / 2,
                  kN6 = (3 * ITEMS) / 4;
    if (items <= kN1) run(std::integral_constant<int, kN1>{});
    else if (items <= kN2) run(std::integral_constant<int, kN2>{});
    else if (items <= kN4) run(std::integral_constant<int, kN4>{});
    else if (items <= kN6) run(std::integral_constant<int, kN6>{});
    else run(std::integral_constant<int, ITEMS>{});
    const int tail = min(i + 1 - fe, k - base);        // forced tail always fits: k >= forced
    for (int x = lane; x < tail; x += 64) out[base + x] = fe + x;
    for (int x = k + lane; x < kmax; x += 64) out[x] = -1;
    if (lane == 0) *count_out = k;
}

template <int ITEMS>
__global__ __launch_bounds__(kSelectThreads) void select_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ budget,
    int32_t* __restrict__ counts, int32_t* __restrict__ indices, SeqTable seq, int Hq, int R,
    int NBmax, int n_sink, int n_local, int kmax) {
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * (kSelectThreads / 64) + (threadIdx.x >> 6);
    if (item >= (int64_t)Hq * R) return;               // wave-uniform; the kernel has no barriers
    const int h = (int)(item / R);
    const int r = (int)(item - (int64_t)h * R);
    const int s = seq_of_row(seq, r);
    const int i = seq.first_block[s] + (r - seq.row_start[s]);   // block index in the sequence
    const float* row = scores + ((int64_t)h * R + r) * NBmax;
    select_row<ITEMS>([&](int j) { return row[j]; }, i, budget[r], n_sink, n_local, kmax, lane,
                      indices + ((int64_t)h * R + r) * kmax, counts + (int64_t)h * R + r);
}

int launch_select(const Problem& p, int heads, const float* scores, const int32_t* budget,
                  int32_t n_sink, int32_t n_local, int32_t* counts, int32_t* indices, int32_t kmax,
                  hipStream_t stream) {
    const int64_t items = (int64_t)heads * p.R;
    const int64_t blocks = (items + kSelectThreads / 64 - 1) / (kSelectThreads / 64);
    if (blocks > 0x7fffffff) return STEM_ERR_UNSUPPORTED;
    dim3 grid((unsigned)blocks), block(kSelectThreads);
#define STEM_SELECT_LAUNCH(N)                                                                      \
    hipLaunchKernelGGL(select_kernel<N>, grid, block, 0, stream, scores, budget, counts, indices,  \
                       p.seq, heads, p.R, p.NBmax, n_sink, n_local, kmax)
    if (p.NBmax <= 64 * 4) STEM_SELECT_LAUNCH(4);
    else if (p.NBmax <= 64 * 16) STEM_SELECT_LAUNCH(16);
    else if (p.NBmax <= 64 * 64) STEM_SELECT_LAUNCH(64);
    else return STEM_ERR_UNSUPPORTED;
#undef STEM_SELECT_LAUNCH
    return check_launch();
}

// ------------------------------------------------------------------------------------------------
// Fused metric + selection: the scores of a band of query-block rows are computed into LDS and
// selected from there, so the [Hq, R, NBmax] score tensor never exists in HBM.
//
// One workgroup owns (head h, band of ROWS consecutive rows of one sequence).  Phase 1 fills
// sc[row][key block] for the key blocks the band can see; phase 2: every wave runs select_row on
// its rows with the scores read from LDS.  ROWS = 16 serves up to 1024 key blocks per row, ROWS = 4
// up to 4096 (64 KiB of fp32 scores either way).
//
// Phase 1, ROWS = 16: the fp32 matrix instruction v_mfma_f32_16x16x4_f32 on tiles of 16 key blocks
// x the band's 16 rows, operands loaded straight from the pooled workspace into registers (it is
// L2-resident and every value is used once per tile, so LDS staging would only add traffic).  The
// order in which the products walk the depth is free as long as both operands agree: lane
// (r = lane % 16, c = lane / 16) holds, of its key block or row r, the floats 16u + 4c .. + 3 of
// every 64-byte group u, so a 16-byte load serves four product steps and the four lanes of a row
// read 64 contiguous bytes.  The workgroup has 8 waves; wave w owns the tiles w, w + 8, ...; their
// accumulators (at most 8 tiles x 4 registers) stay in registers across the whole depth, which is
// walked 64 floats at a time; the next tile's keys are in flight during the products of the
// current one.  With 128 registers per lane two such workgroups (16 waves) share a CU.
// Phase 1, ROWS = 4: v_mfma_f32_4x4x1_16B_f32 on 256-key chunks staged through LDS 8 floats of the
// contraction at a time; every wave takes 64 keys against the band's four rows.
// ------------------------------------------------------------------------------------------------
struct BandTable {
    int32_t band_start[STEM_MAX_BATCH + 1];            // prefix sums of ceil(rows of the call / ROWS)
};

constexpr int kScorePad = 4;                           // floats between rows of sc: 16-byte writes of 16 rows spread over all banks

template <int ROWS>
__global__ __launch_bounds__(ROWS == 16 ? 512 : 256, 2) void score_select_kernel(
    const float* __restrict__ q_bar, const float* __restrict__ k_bar, const float* __restrict__ m_v,
    const int32_t* __restrict__ budget, int32_t* __restrict__ counts, int32_t* __restrict__ indices,
    float* __restrict__ debug_scores, SeqTable seq, BandTable bands, int R, int Rk, int NBmax, int G,
    int S, int d_log2, float beta, float route_scale, int n_sink, int n_local, int kmax) {
    constexpr int NBcap = ROWS == 16 ? 1024 : 4096;    // key blocks per row held in LDS
    constexpr int WAVES = ROWS == 16 ? 8 : 4;
    constexpr int RPW = ROWS / WAVES;                  // rows per wave in phase 2
    constexpr int ITEMS = NBcap / 64;
    __shared__ __attribute__((aligned(16))) float sc[ROWS][NBcap + kScorePad];

    // bands are handed out last first: within a sequence the later bands see more keys and take longer
    const int band = bands.band_start[seq.batch] - 1 - (int)blockIdx.x;
    int s = 0;
    for (int x = 1; x < seq.batch; ++x) s = (band >= bands.band_start[x]) ? x : s;
    const int row0 = seq.row_start[s];
    const int n_rows = seq.row_start[s + 1] - row0;    // rows of this sequence in the call
    const int first = seq.first_block[s];
    const int krow0 = seq.key_row_start[s];
    const int ic0 = (band - bands.band_start[s]) * ROWS;   // first row of the band, call-local
    const int band_rows = min(ROWS, n_rows - ic0);
    const int n_keys = first + ic0 + band_rows;        // key blocks the band's last row can see
    const int h = blockIdx.y, g = h / G;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int d = 1 << d_log2;
    const int depth = S * d;
    const float neg_inf = -__builtin_huge_valf();

    const float* a_src = q_bar + ((int64_t)h * R + row0 + ic0) * depth;
    const float* b_src = k_bar + ((int64_t)g * Rk + krow0) * depth;
    const float* mag_src = m_v + (int64_t)g * Rk + krow0;
    float* dbg = debug_scores != nullptr ? debug_scores + ((int64_t)h * R + row0 + ic0) * NBmax : nullptr;
    int done;                                          // key blocks per row that phase 1 gives a value

    if constexpr (ROWS == 16) {
        typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
        constexpr int TPW = NBcap / 16 / WAVES;        // tiles per wave
        const int r = lane & 15, c = lane >> 4;
        const int n_tiles = (n_keys + 15) >> 4;
        done = n_tiles * 16;
        f32x4_t acc[TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        // The contraction runs over S * d / 64 segments of 64 floats, each inside one residue class
        // a of the query block; its partner among the keys is the same columns of class S-1-a.
        const int segs_per_class = d >> 6;
        for (int seg = 0; seg < S * segs_per_class; ++seg) {
            const int a = seg / segs_per_class, col0 = (seg - a * segs_per_class) * 64 + 4 * c;
            float4 qv[4];
            const float* q_row = a_src + (int64_t)r * depth + a * d + col0;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                qv[u] = (r < band_rows) ? *reinterpret_cast<const float4*>(q_row + 16 * u) : make_float4(0.f, 0.f, 0.f, 0.f);
            const float* k_cls = b_src + (S - 1 - a) * d + col0;
            float4 kv[4], kn[4];
            auto load_keys = [&](float4* dst, int tile) {
                const int j = tile * 16 + r;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    dst[u] = (j < n_keys) ? *reinterpret_cast<const float4*>(k_cls + (int64_t)j * depth + 16 * u)
                                          : make_float4(0.f, 0.f, 0.f, 0.f);
            };
            if (w < n_tiles) load_keys(kv, w);
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const int tile = WAVES * t + w;
                if (tile >= n_tiles) break;            // wave-uniform
                if (tile + WAVES < n_tiles) load_keys(kn, tile + WAVES);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(kv[u].x, qv[u].x, acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(kv[u].y, qv[u].y, acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(kv[u].z, qv[u].z, acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(kv[u].w, qv[u].w, acc[t], 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) kv[u] = kn[u];
            }
        }
        // accumulator x of a lane: band row r, key block 16 tile + 4c + x
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int tile = WAVES * t + w;
            if (tile >= n_tiles) break;
            const int j0 = tile * 16 + 4 * c;
            float val[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int j = j0 + x;
                val[x] = neg_inf;
                if (r < band_rows && j <= first + ic0 + r)   // implies j < n_keys
                    val[x] = fmaf(route_scale / (float)S, acc[t][x], beta * fmaxf(0.f, mag_src[j]));
            }
            if (r >= band_rows) continue;
            *reinterpret_cast<float4*>(&sc[r][j0]) = make_float4(val[0], val[1], val[2], val[3]);
            if (dbg != nullptr) {
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    if (j0 + x < NBmax) dbg[(int64_t)r * NBmax + j0 + x] = val[x];
            }
        }
    } else {
        // 4-row bands: v_mfma_f32_4x4x1_16B_f32, sixteen independent 4 x 4 outer products per
        // instruction: block l / 4 of the wave pairs the band's row l % 4 (A operand) with key
        // block 4 (l / 4) + l % 4 = l of the wave's 64 (B operand), and lane l ends up with the four
        // rows' scores of its key block.  Keys are staged through LDS 256 at a time (64 per wave),
        // 8 floats of the contraction per step, row-major with 48-byte rows, so a lane's 16-byte
        // reads of its own key row are conflict-free; the next step's global loads are in flight
        // during the products.  The staging is kept this small so that, next to the 64 KiB of
        // scores, two workgroups fit a CU: the selection phase of one then runs beside the score
        // phase of the other.
        typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
        constexpr int kKeys = 64 * WAVES, kSlice = 8, kPad = kSlice + 4;
        __shared__ __attribute__((aligned(16))) float ks[kKeys][kPad];   // [key][contraction]
        __shared__ __attribute__((aligned(16))) float qs[ROWS][kPad];    // [row][contraction]
        const int slices = depth / kSlice;             // per key chunk
        const int chunks = (n_keys + kKeys - 1) / kKeys;
        const int steps = chunks * slices;
        done = chunks * kKeys;
        constexpr int kPerThread = kKeys * (kSlice / 4) / (64 * WAVES);   // float4 per thread and step
        float4 bv[kPerThread], av;
        auto fetch = [&](int step) {
            const int j0 = (step / slices) * kKeys, kc = (step % slices) * kSlice;
            // a slice lies inside one residue class a of the query block; its partner is class S-1-a
            const int kb = (S - 1 - (kc >> d_log2)) * d + (kc & (d - 1));
#pragma unroll
            for (int u = 0; u < kPerThread; ++u) {
                const int idx = tid + 64 * WAVES * u;
                const int row = idx / (kSlice / 4), c4 = (idx % (kSlice / 4)) * 4;
                bv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (j0 + row < n_keys) bv[u] = *reinterpret_cast<const float4*>(b_src + (int64_t)(j0 + row) * depth + kb + c4);
            }
            av = make_float4(0.f, 0.f, 0.f, 0.f);
            if (tid < ROWS * (kSlice / 4) && tid / (kSlice / 4) < band_rows)
                av = *reinterpret_cast<const float4*>(a_src + (int64_t)(tid / (kSlice / 4)) * depth + kc + (tid % (kSlice / 4)) * 4);
        };
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
        if (steps > 0) fetch(0);
        for (int step = 0; step < steps; ++step) {
#pragma unroll
            for (int u = 0; u < kPerThread; ++u) {
                const int idx = tid + 64 * WAVES * u;
                *reinterpret_cast<float4*>(&ks[idx / (kSlice / 4)][(idx % (kSlice / 4)) * 4]) = bv[u];
            }
            if (tid < ROWS * (kSlice / 4))
                *reinterpret_cast<float4*>(&qs[tid / (kSlice / 4)][(tid % (kSlice / 4)) * 4]) = av;
            __syncthreads();
            if (step + 1 < steps) fetch(step + 1);
#pragma unroll
            for (int u = 0; u < kSlice / 4; ++u) {
                const float4 kf = *reinterpret_cast<const float4*>(&ks[w * 64 + lane][4 * u]);
                const float4 qf = *reinterpret_cast<const float4*>(&qs[lane & 3][4 * u]);
                acc = __builtin_amdgcn_mfma_f32_4x4x1f32(qf.x, kf.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_4x4x1f32(qf.y, kf.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_4x4x1f32(qf.z, kf.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_4x4x1f32(qf.w, kf.w, acc, 0, 0, 0);
            }
            __syncthreads();
            if (step % slices == slices - 1) {         // the chunk's contraction is complete
                const int j = (step / slices) * kKeys + w * 64 + lane;
                const float mag = (j < n_keys) ? beta * fmaxf(0.f, mag_src[j]) : 0.f;
#pragma unroll
                for (int row = 0; row < ROWS; ++row) {
                    const float val = (j <= first + ic0 + row) ? fmaf(route_scale / (float)S, acc[row], mag) : neg_inf;
                    if (row >= band_rows || j >= NBcap) continue;
                    sc[row][j] = val;
                    if (dbg != nullptr && j < NBmax) dbg[(int64_t)row * NBmax + j] = val;
                }
                acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
            }
        }
    }
    // the rest of a debug row is -inf, as in the unfused score tensor
    if (dbg != nullptr) {
        for (int x = 0; x < RPW; ++x) {
            const int row = w * RPW + x;
            if (row >= band_rows) continue;
            for (int j = done + lane; j < NBmax; j += 64) dbg[(int64_t)row * NBmax + j] = neg_inf;
        }
    }
    __syncthreads();

    // ---- phase 2: selection from LDS, one row at a time per wave ----
    for (int x = 0; x < RPW; ++x) {
        const int row = w * RPW + x;
        if (row >= band_rows) break;                   // wave-uniform
        const int r = row0 + ic0 + row;
        const float* scr = sc[row];
        select_row<ITEMS>([&](int j) { return scr[j]; }, first + ic0 + row, budget[r], n_sink, n_local, kmax,
                          lane, indices + ((int64_t)h * R + r) * kmax, counts + (int64_t)h * R + r);
    }
}

int launch_score_select(const Problem& p, int ad_stride, const float* q_bar, const float* k_bar,
                        const float* m_v, float beta, float route_scale, const int32_t* budget,
                        int32_t n_sink, int32_t n_local, int32_t* counts, int32_t* indices,
                        int32_t kmax, float* debug_scores, hipStream_t stream) {
    if (p.NBmax > 4096) return STEM_ERR_UNSUPPORTED;
    const int rows_per_band = p.NBmax <= 1024 ? 16 : 4;
    BandTable bands;
    int total = 0;
    for (int s = 0; s <= STEM_MAX_BATCH; ++s) {
        bands.band_start[s] = total;
        if (s < p.batch) total += (p.seq.row_start[s + 1] - p.seq.row_start[s] + rows_per_band - 1) / rows_per_band;
    }
    if (total == 0) return STEM_OK;
    if (p.Hq > 65535) return STEM_ERR_UNSUPPORTED;
    dim3 grid(total, p.Hq), block(rows_per_band == 16 ? 512 : 256);
    if (rows_per_band == 16)
        hipLaunchKernelGGL(score_select_kernel<16>, grid, block, 0, stream, q_bar, k_bar, m_v, budget, counts,
                           indices, debug_scores, p.seq, bands, p.R, p.Rk, p.NBmax, p.G, ad_stride,
                           __builtin_ctz(p.d), beta, route_scale, n_sink, n_local, kmax);
    else
        hipLaunchKernelGGL(score_select_kernel<4>, grid, block, 0, stream, q_bar, k_bar, m_v, budget, counts,
                           indices, debug_scores, p.seq, bands, p.R, p.Rk, p.NBmax, p.G, ad_stride,
                           __builtin_ctz(p.d), beta, route_scale, n_sink, n_local, kmax);
    return check_launch();
}

}  // namespace stem
