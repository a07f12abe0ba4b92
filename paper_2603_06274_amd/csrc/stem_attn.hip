// Stage 3 (Algorithm 1 step 3d): block-sparse causal flash attention over the selected key blocks.
//
// One workgroup owns one (query head, query block): B query rows, 32 per wavefront.  For every
// listed key block the workgroup stages K (row-major, 16-byte chunks XOR-swizzled by row) and V
// (transposed to [d][key]) in LDS, and each wave runs
//     S^T = K Q^T      v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = the wave's Q rows (regs)
//     online softmax   in the exp2 domain, fp32, one query column per lane
//     O^T += V^T P^T   A = V^T rows from LDS, B = P^T taken straight from the S^T accumulators
// Computing the transposed products puts one query in one lane, so the softmax row reductions are
// in-lane plus a single exchange with lane^32, and the S^T accumulator registers are already in
// the B-operand layout of the second product: the key rows of each 32-row S^T tile are fed in an
// order (bits 2 and 3 of the row index swapped) that makes each lane's eight accumulator values of
// a 16-key step eight consecutive keys.
#include "stem_common.h"

namespace stem {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 x) { return __builtin_bit_cast(bf16x8_t, x); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ int swap_bits_2_3(int x) {
    return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1);
}

template <int B>
struct AttnSmem {
    static constexpr int kKRow = kHeadDim * 2;         // bytes per K row
    static constexpr int kVtRow = B * 2 + 16;          // bytes per V^T row (padded)
    static constexpr int kKBytes = B * kKRow;
    static constexpr int kVtBytes = kHeadDim * kVtRow;
};

template <int B>
__global__ __launch_bounds__(B * 2) void sparse_attn_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ counts, const int32_t* __restrict__ indices,
    uint16_t* __restrict__ out, float* __restrict__ lse, SeqTable seq, int Hq, int R, int G, int T,
    int kmax, int64_t q_st, int64_t q_sh, int64_t kv_st, int64_t kv_sh, float scale,
    int items_per_xcd) {
    constexpr int NT = B * 2;                          // threads
    constexpr int KT = B / 32;                         // 32-key tiles per block
    using S = AttnSmem<B>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* k_lds = smem;
    unsigned char* vt_lds = smem + S::kKBytes;

    // ---- which (head, row): consecutive workgroup ids go to different XCDs, so give every XCD a
    // contiguous range of the (kv head, row descending, head in group) order ----
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int64_t item = (int64_t)xcd * items_per_xcd + slot;
    if (slot >= items_per_xcd || item >= (int64_t)Hq * R) return;
    const int g = (int)(item / ((int64_t)R * G));
    const int rem = (int)(item - (int64_t)g * R * G);
    const int r = R - 1 - rem / G;
    const int h = g * G + rem % G;

    const int s = seq_of_row(seq, r);
    const int i = r - seq.row_start[s];
    const int seq_lo = seq.tok_start[s], seq_hi = seq.tok_start[s + 1];
    const int tok_q0 = seq_lo + i * B;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int col = lane & 31, hi = lane >> 5;
    const int qrow = w * 32 + col;                     // query row inside the block
    const int tok_q = tok_q0 + qrow;
    const bool q_valid = tok_q < seq_hi;

    // ---- Q rows of this wave as B operands: 8 k-steps of 16 along d ----
    bf16x8_t q_reg[8];
    {
        const uint16_t* src = q + (int64_t)tok_q * q_st + (int64_t)h * q_sh + hi * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 x = make_uint4(0u, 0u, 0u, 0u);
            if (q_valid) x = *reinterpret_cast<const uint4*>(src + ks * 16);
            q_reg[ks] = as_bf16x8(x);
        }
    }

    f32x16_t o_acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int x = 0; x < 16; ++x) o_acc[dt][x] = 0.f;
    float m_run = -__builtin_huge_valf();              // running max of raw scores
    float l_run = 0.f;                                 // this lane's share of the softmax sum
    const float sl2 = scale * 1.4426950408889634f;

    const int cnt = min(counts[(int64_t)h * R + r], kmax);
    const int32_t* list = indices + ((int64_t)h * R + r) * kmax;
    const uint16_t* k_head = k + (int64_t)g * kv_sh;
    const uint16_t* v_head = v + (int64_t)g * kv_sh;

    for (int it = 0; it < cnt; ++it) {
        const int j = list[it];
        if (j < 0 || j > i) continue;                  // uniform over the workgroup
        const int tok_k0 = seq_lo + j * B;
        const bool diag = (j == i);

        __syncthreads();                               // everyone is done with the previous block
        // ---- stage K: B rows x 16 chunks of 16 B, chunk position XORed with (row & 15) ----
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = tid + NT * u;
            const int row = idx >> 4, c = idx & 15;
            uint4 x = make_uint4(0u, 0u, 0u, 0u);
            if (tok_k0 + row < seq_hi)
                x = *reinterpret_cast<const uint4*>(k_head + (int64_t)(tok_k0 + row) * kv_st + c * 8);
            *reinterpret_cast<uint4*>(k_lds + row * S::kKRow + ((c ^ (row & 15)) << 4)) = x;
        }
        // ---- stage V transposed: a unit is 4 keys x 8 columns -> eight 8-byte writes ----
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + NT * u;
            const int m_lo = idx & 15, c_lo = (idx >> 4) & 3, rest = idx >> 6;
            const int c = (rest & 3) * 4 + c_lo, m = (rest >> 2) * 16 + m_lo;
            uint4 x[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int row = 4 * m + qd;
                x[qd] = make_uint4(0u, 0u, 0u, 0u);
                if (tok_k0 + row < seq_hi)
                    x[qd] = *reinterpret_cast<const uint4*>(v_head + (int64_t)(tok_k0 + row) * kv_st + c * 8);
            }
            const uint32_t w0[4] = {x[0].x, x[0].y, x[0].z, x[0].w};
            const uint32_t w1[4] = {x[1].x, x[1].y, x[1].z, x[1].w};
            const uint32_t w2[4] = {x[2].x, x[2].y, x[2].z, x[2].w};
            const uint32_t w3[4] = {x[3].x, x[3].y, x[3].z, x[3].w};
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                uint2 even, odd;                       // columns 2*e2 and 2*e2+1, keys 4m..4m+3
                even.x = (w0[e2] & 0xffffu) | (w1[e2] << 16);
                even.y = (w2[e2] & 0xffffu) | (w3[e2] << 16);
                odd.x = (w0[e2] >> 16) | (w1[e2] & 0xffff0000u);
                odd.y = (w2[e2] >> 16) | (w3[e2] & 0xffff0000u);
                const int d0 = c * 8 + 2 * e2;
                *reinterpret_cast<uint2*>(vt_lds + d0 * S::kVtRow + m * 8) = even;
                *reinterpret_cast<uint2*>(vt_lds + (d0 + 1) * S::kVtRow + m * 8) = odd;
            }
        }
        __syncthreads();

        // ---- S^T = K Q^T : KT tiles of 32 keys x 32 queries ----
        f32x16_t s_acc[KT];
#pragma unroll
        for (int t = 0; t < KT; ++t) {
#pragma unroll
            for (int x = 0; x < 16; ++x) s_acc[t][x] = 0.f;
            const int row = t * 32 + swap_bits_2_3(col);
            const unsigned char* base = k_lds + row * S::kKRow;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const int c = ks * 2 + hi;
                const uint4 a = *reinterpret_cast<const uint4*>(base + ((c ^ (row & 15)) << 4));
                s_acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), q_reg[ks], s_acc[t], 0, 0, 0);
            }
        }

        // ---- causal mask inside the diagonal block: accumulator x of tile t is key
        //      t*32 + 16*(x/8) + 8*hi + x%8 of the block ----
        if (diag) {
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int key = t * 32 + 16 * (x >> 3) + 8 * hi + (x & 7);
                    if (key > qrow) s_acc[t][x] = -__builtin_huge_valf();
                }
        }

        // ---- online softmax ----
        float mx = s_acc[0][0];
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int x = 0; x < 16; ++x) mx = fmaxf(mx, s_acc[t][x]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -__builtin_huge_valf()) ? 0.f : m_new;
        const float corr = __builtin_amdgcn_exp2f((m_run - m_use) * sl2);
        const float off = m_use * sl2;
        float psum = 0.f;
        uint32_t p_pk[KT][8];                          // bf16 pairs: [tile][16-key step * 4 + pair]
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int x = 0; x < 16; x += 2) {
                const float p0 = __builtin_amdgcn_exp2f(s_acc[t][x] * sl2 - off);
                const float p1 = __builtin_amdgcn_exp2f(s_acc[t][x + 1] * sl2 - off);
                psum += p0 + p1;
                p_pk[t][x >> 1] = pack_bf16(p0, p1);
            }
        l_run = l_run * corr + psum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int x = 0; x < 16; ++x) o_acc[dt][x] *= corr;

        // ---- O^T += V^T P^T ----
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint4 pb = make_uint4(p_pk[t][u * 4], p_pk[t][u * 4 + 1], p_pk[t][u * 4 + 2],
                                            p_pk[t][u * 4 + 3]);
                const int key0 = t * 32 + 16 * u + 8 * hi;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    const uint4 a = *reinterpret_cast<const uint4*>(vt_lds + (dt * 32 + col) * S::kVtRow + key0 * 2);
                    o_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(pb), o_acc[dt], 0, 0, 0);
                }
            }
    }

    // ---- normalise and store: accumulator x of d tile dt is column dt*32 + 8*(x/4) + 4*hi + x%4 ----
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (q_valid) {
        uint16_t* dst = out + (int64_t)tok_q * q_st + (int64_t)h * q_sh + hi * 4;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int x4 = 0; x4 < 4; ++x4) {
                uint2 pk;
                pk.x = pack_bf16(o_acc[dt][x4 * 4 + 0] * inv, o_acc[dt][x4 * 4 + 1] * inv);
                pk.y = pack_bf16(o_acc[dt][x4 * 4 + 2] * inv, o_acc[dt][x4 * 4 + 3] * inv);
                *reinterpret_cast<uint2*>(dst + dt * 32 + x4 * 8) = pk;
            }
        if (lse != nullptr && hi == 0)
            lse[(int64_t)h * T + tok_q] = l_tot > 0.f ? m_run * scale + __logf(l_tot) : -__builtin_huge_valf();
    }
}

int launch_sparse_attn(const Problem& p, const void* q, const void* k, const void* v,
                       const int32_t* counts, const int32_t* indices, int32_t kmax,
                       float softmax_scale, void* out, float* lse, hipStream_t stream) {
    const int64_t items = (int64_t)p.Hq * p.R;
    const int64_t per_xcd = (items + 7) / 8;
    if (per_xcd * 8 > 0x7fffffff) return STEM_ERR_UNSUPPORTED;
    dim3 grid((unsigned)(per_xcd * 8));
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint16_t* kk = static_cast<const uint16_t*>(k);
    const uint16_t* vv = static_cast<const uint16_t*>(v);
    uint16_t* oo = static_cast<uint16_t*>(out);
#define STEM_ATTN_LAUNCH(BS)                                                                        \
    do {                                                                                            \
        constexpr int smem = AttnSmem<BS>::kKBytes + AttnSmem<BS>::kVtBytes;                        \
        static bool configured = false;                                                             \
        if (!configured) {                                                                          \
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(sparse_attn_kernel<BS>),          \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess) \
                return STEM_ERR_HIP;                                                                \
            configured = true;                                                                      \
        }                                                                                           \
        hipLaunchKernelGGL(sparse_attn_kernel<BS>, grid, dim3(BS * 2), smem, stream, qq, kk, vv,    \
                           counts, indices, oo, lse, p.seq, p.Hq, p.R, p.G, p.T, kmax, p.q_st,      \
                           p.q_sh, p.kv_st, p.kv_sh, softmax_scale, (int)per_xcd);                  \
    } while (0)
    if (p.B == 128) STEM_ATTN_LAUNCH(128);
    else STEM_ATTN_LAUNCH(64);
#undef STEM_ATTN_LAUNCH
    return check_launch();
}

}  // namespace stem
