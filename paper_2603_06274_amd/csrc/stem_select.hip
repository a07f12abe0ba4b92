// Stage 2 (Algorithm 1 step 3c; forced windows of Implementation Details): per-row top-k(i).
//
// One 64-lane wavefront owns one (head, row).  The row's candidate scores are held in registers as
// order-preserving 32-bit keys, lane-strided (element e of lane l is key block fs + 64 e + l).  The
// k-th largest key is found exactly by a 32-step bitwise search whose counts come from wave ballots
// (scalar popcounts, no atomics, no LDS), and the list is then emitted in ascending block order by
// ballot prefix compaction: forced blocks, every key above the threshold, and the lowest-indexed
// keys equal to it until the budget is met.  The result is therefore deterministic and ties go to
// the lower block index.
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

    const int fs = min(n_sink, i + 1);                 // forced head: blocks [0, fs)
    const int fe = max(fs, i - n_local + 1);           // forced tail: blocks [fe, i]
    const int nfree = fe - fs;
    const int forced = i + 1 - nfree;
    int k = max(budget[r], forced);
    k = min(k, min(i + 1, kmax));
    const int need = max(0, k - forced);               // free blocks to pick, <= nfree

    const float* row = scores + ((int64_t)h * R + r) * NBmax;
    int32_t* out = indices + ((int64_t)h * R + r) * kmax;

    uint32_t key[ITEMS];
#pragma unroll
    for (int e = 0; e < ITEMS; ++e) {
        const int j = fs + e * 64 + lane;
        key[e] = (j < fe) ? ordered_key(row[j]) : 0u;  // 0 sorts below every real key
    }

    uint32_t tau = 0;
    int n_eq = 0;                                      // keys equal to tau that are still needed
    if (need > 0 && need < nfree) {
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t cand = tau | (1u << bit);
            int cnt = 0;
#pragma unroll
            for (int e = 0; e < ITEMS; ++e) cnt += __popcll(__ballot(key[e] >= cand));
            if (cnt >= need) tau = cand;
        }
        int above = 0;
#pragma unroll
        for (int e = 0; e < ITEMS; ++e) above += __popcll(__ballot(key[e] > tau));
        n_eq = need - above;
    }
    const bool take_all = (need >= nfree);

    // emit ascending: forced head, chosen free blocks, forced tail
    for (int j = lane; j < fs; j += 64) out[j] = j;
    int base = fs;
    if (need > 0) {
        int eq_seen = 0;
#pragma unroll
        for (int e = 0; e < ITEMS; ++e) {
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
    const int tail = min(i + 1 - fe, k - base);        // forced tail always fits: k >= forced
    for (int x = lane; x < tail; x += 64) out[base + x] = fe + x;
    for (int x = k + lane; x < kmax; x += 64) out[x] = -1;
    if (lane == 0) counts[(int64_t)h * R + r] = k;
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

}  // namespace stem
