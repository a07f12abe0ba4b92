// Stage 3 (Algorithm 1 step 3d) for the head sizes other than 128: block-sparse causal flash
// attention over the selected key blocks, head size D = 64 or 256.
//
// The same mathematics and the same transposed matrix products as the kernel for D = 128
// (S^T = K Q^T, online softmax with one query per lane, O^T += V^T P^T, bf16 inputs, fp32
// accumulation, key rows of each 32-row S^T tile fed with bits 2 and 3 of the row index swapped so
// that a lane's accumulators of a 16-key step are eight consecutive keys), in a plainer schedule:
// a textbook running-maximum softmax between the two products, no operand ring, no interleaving of
// vector and matrix work by hand.  What it shares with the tuned kernel is the data movement: K and
// V blocks go from global memory straight into LDS (buffer_load ... lds, 1 KiB per wave and
// instruction, no staging registers), one buffer each, refilled in split phases behind two barriers
// per block: V(j) is requested before S^T and awaited after the softmax, K(next) is requested before
// O^T and awaited at the top of the next iteration.  At D = 256 the kernel needs 128 KiB of LDS and
// about 450 registers, so a CU holds one workgroup and this overlap inside it is all there is.
//
// LDS rows are unpadded (the direct loads write 1 KiB contiguously) and swizzled on the global
// side, each lane fetching the 16-byte chunk that belongs at its LDS position.  K: chunk index XOR
// row & 15 (D = 256) or (row >> 1) & 7 (D = 64, where two 128-byte rows share the 64 banks), so the
// 16 rows a quarter-wave reads one chunk of fall on 16 different bank groups.  V: 64-byte group
// index XOR row & 3 (D = 256) or (row >> 1) & 1 (D = 64), which does the same for the 4 rows x
// 32 bytes a quarter-wave touches in a transposing read.  Loads go through a buffer resource that
// ends with the sequence's last row: rows past it are never read and arrive as zeros.
#include "stem_common.h"

namespace stem {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((address_space(3))) void lds_void_t;

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
    constexpr int NW = B / 32;                         // waves
    constexpr int kRow = D * 2;                        // bytes per LDS row
    constexpr int kSliceRows = 1024 / kRow;            // rows one wave-wide 1 KiB request covers
    constexpr int NSL = D / 16;                        // requests per wave, tensor and block
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds[B * kRow];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds[B * kRow];
    auto k_swz = [](int row) { return D == 64 ? (row >> 1) & 7 : row & 15; };           // on the chunk index
    auto v_swz = [](int row) { return (D == 64 ? (row >> 1) & 1 : row & 3) << 2; };     // on the chunk index

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

    // per-lane LDS addressing: K row swap(col) of a tile (tiles are 32 rows, so the swizzle term of
    // the row does not depend on the tile), 16-byte chunk 2 ks + hi of step ks; transposing V read:
    // row 8 hi + (lane % 16) / 4 (and + 4: same swizzle term) of a 16-key step, 8 bytes at column
    // 16 ((lane >> 4) & 1) + 4 (lane & 3) of a 32-column tile, i.e. 64-byte group dt
    const int k_row = swap_bits_2_3(col);
    const uint32_t k_row_off = k_row * kRow;
    const int k_x = k_swz(k_row);
    const int v_row = hi * 8 + ((lane & 15) >> 2);
    const uint32_t v_row_off = v_row * kRow + (((lane >> 4) & 1) << 5) + ((lane & 3) << 3);
    const int v_x = v_swz(v_row) >> 2;                 // on the 64-byte group index

    // block requests: slice u of wave w is the 1 KiB at LDS offset (u NW + w) KiB; lane l writes its
    // bytes 16 l .. 16 l + 15, i.e. chunk pc of row lrow(u), and fetches the chunk swizzled there
    const int64_t row_bytes = kv_st * 2;
    const int seq_rows = seq_hi - seq_lo;
    const int64_t seq_bytes = seq_rows > 0 ? (int64_t)(seq_rows - 1) * row_bytes + kRow : 0;   // < 2^31 (host check)
    const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(k_head + (int64_t)seq_lo * kv_st), 0, (int)seq_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(v_head + (int64_t)seq_lo * kv_st), 0, (int)seq_bytes, 0x00020000);
    const int pc = (lane * 16 % kRow) >> 4, slice_row = lane * 16 / kRow;
    auto request = [&](const __amdgpu_buffer_rsrc_t& rsrc, unsigned char* lds, int j, bool is_k) {
        const uint32_t block_off = (uint32_t)j * (uint32_t)(B * row_bytes);
#pragma unroll
        for (int u = 0; u < NSL; ++u) {
            const int lrow = (u * NW + w) * kSliceRows + slice_row;
            const int chunk = pc ^ (is_k ? k_swz(lrow) : v_swz(lrow));
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_t*)(lds + (u * NW + w) * 1024), 16,
                                                     block_off + (uint32_t)(lrow * row_bytes) + chunk * 16, 0, 0, 0);
        }
    };
    // the visible entries of the list, in order (anything outside 0..i contributes nothing)
    auto next_visible = [&](int e) {
        while (e < cnt) {
            const int j = list[e];
            if (j >= 0 && j <= i) break;
            ++e;
        }
        return e;
    };
    int e = next_visible(0);
    if (e < cnt) request(k_rsrc, k_lds, list[e], true);

    while (e < cnt) {
        const int j = list[e];
        const int e_next = next_visible(e + 1);
        __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wave's requests have landed
        __syncthreads();                               // K(j) is in LDS; V buffer is free
        request(v_rsrc, v_lds, j, false);

        // ---- S^T = K Q^T: accumulator x of tile t is key 32 t + 16 (x / 8) + 8 hi + x % 8 ----
        f32x16_t s_acc[KT];
#pragma unroll
        for (int t = 0; t < KT; ++t) {
#pragma unroll
            for (int x = 0; x < 16; ++x) s_acc[t][x] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const uint4 a = *reinterpret_cast<const uint4*>(k_lds + k_row_off + t * 32 * kRow + (((2 * ks + hi) ^ k_x) << 4));
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

        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();                               // V(j) is in LDS; every wave is done with K(j)
        if (e_next < cnt) request(k_rsrc, k_lds, list[e_next], true);

        // ---- O^T += V^T P^T: per 16-key step, V^T rows through the transposing read ----
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint4 pb = make_uint4(p_pk[t][u * 4], p_pk[t][u * 4 + 1], p_pk[t][u * 4 + 2], p_pk[t][u * 4 + 3]);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const unsigned char* p0 = v_lds + v_row_off + (t * 32 + u * 16) * kRow + ((dt ^ v_x) << 6);
                    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p0);
                    const s16x4_t up = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p0 + 4 * kRow));
                    const uint2 lo2 = __builtin_bit_cast(uint2, lo), up2 = __builtin_bit_cast(uint2, up);
                    const uint4 a = make_uint4(lo2.x, lo2.y, up2.x, up2.y);
                    o_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(pb), o_acc[dt], 0, 0, 0);
                }
            }
        e = e_next;
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
    // the block requests address one sequence of one KV head through a 32-bit byte offset
    for (int s = 0; s < p.batch; ++s) {
        const int64_t rows = p.seq.tok_start[s + 1] - p.seq.tok_start[s];
        if (rows > 0 && (rows - 1) * p.kv_st * 2 + p.d * 2 > 0x7fffffffll) return STEM_ERR_UNSUPPORTED;
    }
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
