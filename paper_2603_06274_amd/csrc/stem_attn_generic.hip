// Stage 3 (Algorithm 1 step 3d) for the head sizes other than 128: block-sparse causal flash
// attention over the selected key blocks, head size D = 64 or 256.
//
// The same mathematics and the same transposed matrix products as the kernel for D = 128
// (S^T = K Q^T, online softmax with one query per lane, O^T += V^T P^T, bf16 inputs, fp32
// accumulation, key rows of each 32-row S^T tile fed with bits 2 and 3 of the row index swapped so
// that a lane's accumulators of a 16-key step are eight consecutive keys), in a plain schedule: per
// listed block the workgroup copies the K and V blocks into LDS through registers, synchronises,
// and every wave then runs its two products and a textbook running-maximum softmax.  Nothing is
// overlapped inside a workgroup; the workgroups sharing a CU overlap each other.
//
// LDS rows are padded instead of swizzled: K rows by 16 bytes (the 16 rows one quarter-wave reads
// 16 bytes of fall on different banks), V rows by 32 bytes (the 4 rows x 32 bytes a quarter-wave
// touches in a transposing read do the same).
#include "stem_common.h"

namespace stem {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 x) { return __builtin_bit_cast(bf16x8_t, x); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ int swap_bits_2_3(int x) {
    return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1);
}

template <int B, int D>
__global__ __launch_bounds__(B * 2) void sparse_attn_generic_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ counts, const int32_t* __restrict__ indices,
    uint16_t* __restrict__ out, float* __restrict__ lse, SeqTable seq, int Hq, int R, int G, int T,
    int kmax, bool shared_lists, int64_t q_st, int64_t q_sh, int64_t kv_st, int64_t kv_sh, float scale) {
    constexpr int KT = B / 32;                         // 32-key tiles per block
    constexpr int KS = D / 16;                         // 16-wide steps of S^T along d
    constexpr int DT = D / 32;                         // 32-row tiles of O^T along d
    constexpr int NT = B * 2;                          // threads: 32 query rows per wave
    constexpr int kChunks = D / 8;                     // 16-byte chunks per row
    constexpr int kKRow = D * 2 + 16, kVRow = D * 2 + 32;   // padded LDS rows (bytes)
    __shared__ __attribute__((aligned(16))) unsigned char k_lds[B * kKRow];
    __shared__ __attribute__((aligned(16))) unsigned char v_lds[B * kVRow];

    // (KV head, row descending, head in group): the long rows first, a group's heads side by side
    const int64_t item = blockIdx.x;
    const int g = (int)(item / ((int64_t)R * G));
    const int rem = (int)(item - (int64_t)g * R * G);
    const int r = R - 1 - rem / G;
    const int h = g * G + rem % G;

    const int s = seq_of_row(seq, r);
    const int ic = r - seq.row_start[s];               // row inside the call's chunk of the sequence
    const int i = seq.first_block[s] + ic;             // block index in the sequence
    const int seq_lo = seq.tok_start[s], seq_hi = seq.kv_end[s];   // key token rows the call may read
    const int tok_q0 = seq.q_tok_start[s] + ic * B;    // Q, O and lse hold the chunk's tokens only
    const int q_hi = seq.q_tok_start[s + 1];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int col = lane & 31, hi = lane >> 5;
    const int qrow = w * 32 + col;                     // query row inside the block
    const int tok_q = tok_q0 + qrow;
    const bool q_valid = tok_q < q_hi;

    const int lh = shared_lists ? g : h;               // whose list: the KV head's or the query head's
    const int cnt = min(counts[(int64_t)lh * R + r], kmax);
    const int32_t* list = indices + ((int64_t)lh * R + r) * kmax;
    const uint16_t* k_head = k + (int64_t)g * kv_sh;
    const uint16_t* v_head = v + (int64_t)g * kv_sh;

    // Q rows of this wave as B operands: lane (col, hi) holds columns 16 ks + 8 hi .. + 7 of query col
    bf16x8_t q_reg[KS];
    {
        const uint16_t* src = q + (int64_t)tok_q * q_st + (int64_t)h * q_sh + hi * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint4 x = make_uint4(0u, 0u, 0u, 0u);
            if (q_valid) x = *reinterpret_cast<const uint4*>(src + ks * 16);
            q_reg[ks] = as_bf16x8(x);
        }
    }

    f32x16_t o_acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int x = 0; x < 16; ++x) o_acc[dt][x] = 0.f;
    const float neg_inf = -__builtin_huge_valf();
    float m_run = neg_inf;                             // running maximum (raw score units)
    float l_run = 0.f;                                 // this lane's share of the softmax sum
    const float sl2 = scale * 1.4426950408889634f;

    // per-lane LDS offsets: K row swap(col) of a tile, 16-byte chunk hi of a step; transposing V
    // read: row 8 hi + (lane % 16) / 4 (and + 4) of a 16-key step, 8 bytes at column
    // 16 ((lane >> 4) & 1) + 4 (lane & 3) of a 32-column tile
    const uint32_t k_base = swap_bits_2_3(col) * kKRow + hi * 16;
    const uint32_t v_base = (hi * 8 + ((lane & 15) >> 2)) * kVRow + (((lane >> 4) & 1) << 5) + ((lane & 3) << 3);

    for (int e = 0; e < cnt; ++e) {
        const int j = list[e];
        if (j < 0 || j > i) continue;                  // not a visible block: contributes nothing (uniform)
        __syncthreads();                               // the previous block's operand reads are done
        // ---- K and V blocks into LDS; rows past the end of the sequence are zeros ----
        {
            const int tok0 = seq_lo + j * B;
            constexpr int kPerThread = B * kChunks / NT;   // 16-byte chunks per thread and tensor
#pragma unroll
            for (int u0 = 0; u0 < kPerThread; u0 += 4) {
                uint4 kx[4], vx[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int idx = tid + NT * (u0 + u);
                    const int row = idx / kChunks, ch = idx % kChunks;
                    kx[u] = make_uint4(0u, 0u, 0u, 0u);
                    vx[u] = kx[u];
                    if (tok0 + row < seq_hi) {
                        const int64_t off = (int64_t)(tok0 + row) * kv_st + ch * 8;
                        kx[u] = *reinterpret_cast<const uint4*>(k_head + off);
                        vx[u] = *reinterpret_cast<const uint4*>(v_head + off);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int idx = tid + NT * (u0 + u);
                    const int row = idx / kChunks, ch = idx % kChunks;
                    *reinterpret_cast<uint4*>(k_lds + row * kKRow + ch * 16) = kx[u];
                    *reinterpret_cast<uint4*>(v_lds + row * kVRow + ch * 16) = vx[u];
                }
            }
        }
        __syncthreads();

        // ---- S^T = K Q^T: accumulator x of tile t is key 32 t + 16 (x / 8) + 8 hi + x % 8 ----
        f32x16_t s_acc[KT];
#pragma unroll
        for (int t = 0; t < KT; ++t) {
#pragma unroll
            for (int x = 0; x < 16; ++x) s_acc[t][x] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const uint4 a = *reinterpret_cast<const uint4*>(k_lds + k_base + t * 32 * kKRow + ks * 32);
                s_acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), q_reg[ks], s_acc[t], 0, 0, 0);
            }
        }
        // causal mask inside the diagonal block (which also hides the zero rows of a partial block)
        if (j == i) {
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int key = t * 32 + 16 * (x >> 3) + 8 * hi + (x & 7);
                    if (key > qrow) s_acc[t][x] = neg_inf;
                }
        }

        // ---- online softmax, exp2 domain; the two lanes of a query (lane, lane ^ 32) agree on the maximum ----
        float m_blk = neg_inf;
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int x = 0; x < 16; ++x) m_blk = fmaxf(m_blk, s_acc[t][x]);
        m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32));
        const float m_new = fmaxf(m_run, m_blk);
        const float m_use = m_new == neg_inf ? 0.f : m_new;    // nothing visible yet: every p is 0
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * sl2);   // m_run = -inf gives 0
        const float off = m_use * sl2;
        uint32_t p_pk[KT][8];                          // bf16 pairs: [tile][16-key step * 4 + pair]
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int x = 0; x < 16; x += 2) {
                const float p0 = __builtin_amdgcn_exp2f(s_acc[t][x] * sl2 - off);
                const float p1 = __builtin_amdgcn_exp2f(s_acc[t][x + 1] * sl2 - off);
                const uint32_t pk = pack_bf16(p0, p1);
                p_pk[t][x >> 1] = pk;
                sum += bf16_lo(pk) + bf16_hi(pk);      // the sum of the rounded values that O^T uses
            }
        l_run = l_run * alpha + sum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int x = 0; x < 16; ++x) o_acc[dt][x] *= alpha;

        // ---- O^T += V^T P^T: per 16-key step, V^T rows through the transposing read ----
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint4 pb = make_uint4(p_pk[t][u * 4], p_pk[t][u * 4 + 1], p_pk[t][u * 4 + 2], p_pk[t][u * 4 + 3]);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const unsigned char* p0 = v_lds + v_base + (t * 32 + u * 16) * kVRow + dt * 64;
                    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p0);
                    const s16x4_t up = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p0 + 4 * kVRow));
                    const uint2 lo2 = __builtin_bit_cast(uint2, lo), up2 = __builtin_bit_cast(uint2, up);
                    const uint4 a = make_uint4(lo2.x, lo2.y, up2.x, up2.y);
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
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int x4 = 0; x4 < 4; ++x4) {
                const uint2 pk = make_uint2(pack_bf16(o_acc[dt][x4 * 4 + 0] * inv, o_acc[dt][x4 * 4 + 1] * inv),
                                            pack_bf16(o_acc[dt][x4 * 4 + 2] * inv, o_acc[dt][x4 * 4 + 3] * inv));
                *reinterpret_cast<uint2*>(dst + dt * 32 + x4 * 8) = pk;
            }
        if (lse != nullptr && hi == 0)
            lse[(int64_t)h * T + tok_q] = l_tot > 0.f ? m_run * scale + __logf(l_tot) : neg_inf;
    }
}

}  // namespace

int launch_sparse_attn_generic(const Problem& p, const void* q, const void* k, const void* v,
                               const int32_t* counts, const int32_t* indices, int32_t kmax,
                               bool lists_per_kv_head, float softmax_scale, void* out, float* lse,
                               hipStream_t stream) {
    const int64_t items = (int64_t)p.Hq * p.R;
    if (items == 0) return STEM_OK;
    if (items > 0x7fffffff) return STEM_ERR_UNSUPPORTED;
    dim3 grid((unsigned)items), block(p.B * 2);
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint16_t* kk = static_cast<const uint16_t*>(k);
    const uint16_t* vv = static_cast<const uint16_t*>(v);
    uint16_t* oo = static_cast<uint16_t*>(out);
#define STEM_ATTN_LAUNCH(BB, DD)                                                                          \
    hipLaunchKernelGGL((sparse_attn_generic_kernel<BB, DD>), grid, block, 0, stream, qq, kk, vv, counts,  \
                       indices, oo, lse, p.seq, p.Hq, p.R, p.G, p.T, kmax, lists_per_kv_head, p.q_st,     \
                       p.q_sh, p.kv_st, p.kv_sh, softmax_scale)
    if (p.B == 128 && p.d == 64) STEM_ATTN_LAUNCH(128, 64);
    else if (p.B == 64 && p.d == 64) STEM_ATTN_LAUNCH(64, 64);
    else if (p.B == 128 && p.d == 256) STEM_ATTN_LAUNCH(128, 256);
    else if (p.B == 64 && p.d == 256) STEM_ATTN_LAUNCH(64, 256);
    else return STEM_ERR_UNSUPPORTED;
#undef STEM_ATTN_LAUNCH
    return check_launch();
}

}  // namespace stem
