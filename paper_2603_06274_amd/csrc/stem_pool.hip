// Stage 1a (Algorithm 1 step 1): block-wise pooling of Q and K and max-pooled value magnitude.
//
// Pure HBM stream: every bf16 element of Q, K and V is read exactly once, in 16-byte lane loads
// that cover one head row (2 d bytes) per d / 8 lanes.  One workgroup owns one block row of one
// tensor and HW adjacent heads of it (two where the head size allows; with the usual
// [token][head][d] layout a token's lanes then read 512 contiguous bytes, which the memory system
// serves measurably better than 256): 2 d HW threads = 16 token lanes x HW heads x d / 8 column
// chunks (512 threads at d = 128); every thread issues all of its loads (B/16 tokens) before it
// touches the first value, so a workgroup keeps the whole B x 2 d HW bytes in flight.  Column sums
// are reduced across the 16 token lanes through LDS in a fixed order (deterministic fp32).
//
// With an anti-diagonal stride S > 1 (S divides 16) a block keeps S partial means, one per residue
// class of the in-block token position modulo S.  A thread's tokens tl, tl + 16, ... all fall in
// class tl mod S, so the only change is that the LDS reduction adds the 16 / S token lanes of each
// class separately.
#include "stem_common.h"

namespace stem {

// 16-byte load marked non-temporal: the stream is read once here, and a read that does not claim
// cache lines runs measurably closer to the HBM rate (7.0 against 6.3 TB/s for a bare read).
__device__ __forceinline__ uint4 load_streaming(const uint16_t* p) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t x = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(x.x, x.y, x.z, x.w);
}

template <int B, int D, int HW>
__global__ __launch_bounds__(2 * D * HW) void pool_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    float* __restrict__ q_bar, float* __restrict__ k_bar, float* __restrict__ m_v, SeqTable seq,
    int Hq, int Hkv, int R, int Rk, int S, int64_t q_st, int64_t q_sh, int64_t kv_st, int64_t kv_sh) {
    constexpr int kTok = B / 16;                       // tokens per thread
    constexpr int kThreads = 2 * D * HW;
    constexpr int kChunks = D / 8;                     // 16-byte chunks per row: 8, 16 or 32
    // HW adjacent heads per workgroup: with the usual [token][head][d] layout the lanes of a token
    // then read HW * 2 d contiguous bytes
    const int slots = (Hq + 2 * Hkv) / HW;
    const int r = blockIdx.x / slots;
    const int slot = (blockIdx.x - r * slots) * HW;    // first of the workgroup's HW heads, counted over Q, K, V
    const int s = seq_of_row(seq, r);
    const int ic = r - seq.row_start[s];               // row inside the call's chunk of the sequence
    const int i = seq.first_block[s] + ic;             // block index in the sequence
    const int kv_tok0 = seq.tok_start[s] + i * B;      // first token row of the block in K and V
    const int q_tok0 = seq.q_tok_start[s] + ic * B;    // and in Q, which holds the chunk's tokens only
    const int n_valid = min(B, seq.kv_end[s] - kv_tok0);
    const int key_row = seq.key_row_start[s] + i;      // row of k_bar and m_v

    const uint16_t* src;
    int64_t st;
    int kind, head, tok0;                              // 0: Q, 1: K, 2: V
    if (slot < Hq) {
        kind = 0; head = slot; src = q + (int64_t)head * q_sh; st = q_st; tok0 = q_tok0;
    } else if (slot < Hq + Hkv) {
        kind = 1; head = slot - Hq; src = k + (int64_t)head * kv_sh; st = kv_st; tok0 = kv_tok0;
    } else {
        kind = 2; head = slot - Hq - Hkv; src = v + (int64_t)head * kv_sh; st = kv_st; tok0 = kv_tok0;
    }

    const int tid = threadIdx.x;
    const int c = tid % kChunks;                       // 16-byte chunk of the row
    const int hp = (tid / kChunks) % HW;               // which of the workgroup's heads
    const int tl = tid / (kChunks * HW);               // token lane 0..15
    head += hp;
    src += (int64_t)hp * (kind == 0 ? q_sh : kv_sh);

    uint4 raw[kTok];
#pragma unroll
    for (int u = 0; u < kTok; ++u) {
        const int t = tl + 16 * u;
        raw[u] = make_uint4(0u, 0u, 0u, 0u);
        if (t < n_valid) raw[u] = load_streaming(src + (int64_t)(tok0 + t) * st + c * 8);
    }

    __shared__ float part[16][HW * D + 4];             // [token lane][head, column]
    __shared__ float vmax[kThreads / 64][HW];

    if (kind != 2) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < kTok; ++u) {
            acc[0] += bf16_lo(raw[u].x); acc[1] += bf16_hi(raw[u].x);
            acc[2] += bf16_lo(raw[u].y); acc[3] += bf16_hi(raw[u].y);
            acc[4] += bf16_lo(raw[u].z); acc[5] += bf16_hi(raw[u].z);
            acc[6] += bf16_lo(raw[u].w); acc[7] += bf16_hi(raw[u].w);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) part[tl][hp * D + c * 8 + e] = acc[e];
        __syncthreads();
        const int head0 = head - hp;
        for (int o = tid; o < HW * S * D; o += kThreads) {
            const int ho = o / (S * D), oo = o % (S * D);     // head of the workgroup, offset in its output
            const int a = oo / D, col = oo % D;               // residue class, column
            float* dst = kind == 0 ? q_bar + ((int64_t)(head0 + ho) * R + r) * S * D
                                   : k_bar + ((int64_t)(head0 + ho) * Rk + key_row) * S * D;
            float sum = 0.f;
            for (int x = a; x < 16; x += S) sum += part[x][ho * D + col];
            const int members = (n_valid - a + S - 1) / S;    // valid tokens of the class (n_valid > a)
            dst[oo] = n_valid > a ? sum / (float)members : 0.f;
        }
    } else {
        // squared L2 norm of each token row: 8 columns per lane, then across the row's chunk lanes
        float best = 0.f;
#pragma unroll
        for (int u = 0; u < kTok; ++u) {
            float x0 = bf16_lo(raw[u].x), x1 = bf16_hi(raw[u].x), x2 = bf16_lo(raw[u].y),
                  x3 = bf16_hi(raw[u].y), x4 = bf16_lo(raw[u].z), x5 = bf16_hi(raw[u].z),
                  x6 = bf16_lo(raw[u].w), x7 = bf16_hi(raw[u].w);
            float ss = ((x0 * x0 + x1 * x1) + (x2 * x2 + x3 * x3)) +
                       ((x4 * x4 + x5 * x5) + (x6 * x6 + x7 * x7));
#pragma unroll
            for (int x = 1; x < kChunks; x *= 2) ss += __shfl_xor(ss, x);
            best = fmaxf(best, ss);                    // padded tokens contribute 0
        }
        // across the wave's other token lanes of the same head (the lane bits above chunk and head)
#pragma unroll
        for (int x = kChunks * HW; x < 64; x *= 2) best = fmaxf(best, __shfl_xor(best, x));
        if ((tid & 63) < kChunks * HW && c == 0) vmax[tid >> 6][hp] = best;
        __syncthreads();
        if (tid < HW) {
            float m = vmax[0][tid];
#pragma unroll
            for (int x = 1; x < kThreads / 64; ++x) m = fmaxf(m, vmax[x][tid]);
            // max_t ln ||v_t|| = 0.5 ln max_t ||v_t||^2 ; ln 0 = -inf
            m_v[(int64_t)(head - hp + tid) * Rk + key_row] = 0.5f * logf(m);
        }
    }
}

int launch_pool(const Problem& p, int ad_stride, const void* q, const void* k, const void* v,
                float* q_bar, float* k_bar, float* m_v, hipStream_t stream) {
    if (ad_stride < 1 || 16 % ad_stride) return STEM_ERR_UNSUPPORTED;
    // two adjacent heads per workgroup where that keeps the workgroup within 512 threads and no
    // pair straddles two of the tensors (four heads, or 1024 threads, measured no better)
    const int hw = (p.d <= 128 && p.Hq % 2 == 0 && p.Hkv % 2 == 0) ? 2 : 1;
    const int64_t blocks = (int64_t)p.R * ((p.Hq + 2 * p.Hkv) / hw);
    if (blocks > 0x7fffffff) return STEM_ERR_UNSUPPORTED;
    dim3 grid((unsigned)blocks), block(2 * p.d * hw);
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint16_t* kk = static_cast<const uint16_t*>(k);
    const uint16_t* vv = static_cast<const uint16_t*>(v);
#define STEM_POOL_LAUNCH(BB, DD, HH)                                                                \
    hipLaunchKernelGGL((pool_kernel<BB, DD, HH>), grid, block, 0, stream, qq, kk, vv, q_bar, k_bar, \
                       m_v, p.seq, p.Hq, p.Hkv, p.R, p.Rk, ad_stride, p.q_st, p.q_sh, p.kv_st, p.kv_sh)
#define STEM_POOL_LAUNCH_D(BB, DD)                     \
    do {                                               \
        if (hw == 2) STEM_POOL_LAUNCH(BB, DD, 2);      \
        else STEM_POOL_LAUNCH(BB, DD, 1);              \
    } while (0)
    if (p.B == 128 && p.d == 128) STEM_POOL_LAUNCH_D(128, 128);
    else if (p.B == 64 && p.d == 128) STEM_POOL_LAUNCH_D(64, 128);
    else if (p.B == 128 && p.d == 64) STEM_POOL_LAUNCH_D(128, 64);
    else if (p.B == 64 && p.d == 64) STEM_POOL_LAUNCH_D(64, 64);
    else if (p.B == 128 && p.d == 256) STEM_POOL_LAUNCH(128, 256, 1);
    else if (p.B == 64 && p.d == 256) STEM_POOL_LAUNCH(64, 256, 1);
    else return STEM_ERR_UNSUPPORTED;
#undef STEM_POOL_LAUNCH_D
#undef STEM_POOL_LAUNCH
    return check_launch();
}

}  // namespace stem
