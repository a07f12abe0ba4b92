// Stage 3 (Algorithm 1 step 3d): block-sparse causal flash attention over the selected key blocks.
//
// One workgroup owns one (query head, query block): B query rows, 32 per wavefront.  Per listed key
// block each wave runs
//     S^T = K Q^T      v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = the wave's Q rows (regs)
//     online softmax   exp2 domain, fp32, one query column per lane
//     O^T += V^T P^T   A = V^T rows read from row-major V in LDS with ds_read_b64_tr_b16,
//                      B = P^T taken straight from the S^T accumulators
// Computing the transposed products puts one query in one lane, so the softmax row reductions are
// in-lane plus a single exchange with lane^32, and the S^T accumulator registers are already in
// the B-operand layout of the second product: the key rows of each 32-row S^T tile are fed in an
// order (bits 2 and 3 of the row index swapped) that makes each lane's eight accumulator values of
// a 16-key step eight consecutive keys.
//
// K and V blocks go from global memory straight into LDS (global_load_lds_dwordx4, no staging
// registers), one buffer each, refilled in split phases: the next K block is requested as soon as
// every wave has finished S^T and lands while softmax and O^T run; the V block is requested at
// the top of the iteration and lands while S^T and softmax run.  Two workgroups share a CU, so one
// workgroup's matrix work overlaps the other's softmax and waits.
//
// LDS layouts (256-byte rows): K has its 16-byte chunks XORed with (row & 15), so the 32 rows a
// b128 operand read touches spread over all banks; V has its 64-byte groups XORed with (row & 3),
// which does the same for the 4-row x 64-byte footprint of a transposing read.  The swizzle is
// applied on the global side (each lane fetches the chunk that belongs at its LDS position).
#include "stem_common.h"

namespace stem {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 x) { return __builtin_bit_cast(bf16x8_t, x); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ int swap_bits_2_3(int x) {
    return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1);
}

// Workgroup barrier without the memory fence of __syncthreads (which would wait for every
// outstanding global->LDS load); the waits are placed by hand.
#define STEM_BARRIER()                              \
    do {                                            \
        asm volatile("" ::: "memory");              \
        __builtin_amdgcn_s_barrier();               \
        asm volatile("" ::: "memory");              \
    } while (0)
// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt[3:0], expcnt[6:4]=7, lgkmcnt[11:8]=15); the
// builtin, unlike inline asm, is seen by the compiler's own wait-count bookkeeping.
#define STEM_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | (N))

// Nothing is scheduled across this point: keeps the next group of LDS operand reads ahead of the
// matrix instructions that consume the current group.
#define STEM_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

constexpr int kRowBytes = kHeadDim * 2;               // one K or V row in LDS

// One 1 KiB slice (4 rows) of a B x 128 bf16 block, global -> LDS.  A block is 8 slices per wave:
// wave w issues slices u*NW + w, u = 0..7, so that the row's swizzle term does not depend on u (for
// B = 64 it depends on the parity of u only).  Requests are issued one or two at a time between
// groups of matrix instructions, never as a burst: the texture-address unit takes a wave's 1 KiB
// request at 64 B/clk, and a wave that finds its queue full cannot issue anything else.
//
// The loads use buffer addressing: a per-block resource whose base is the block's first row in
// this KV head and whose size ends with the sequence's last row, so rows past the end of a
// partial last block (and past the end of the tensor) are never read and arrive in LDS as zeros
// (their keys are masked by causality, their values get weight 0).  The per-lane byte offset is
// computed once per kernel; a slice costs one vector add.
struct BlockRequest {
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t lane_off[2];           // per-lane byte offset for even / odd u
    uint32_t slice_step;            // bytes between the rows of slices u and u+1 of one wave

    __device__ __forceinline__ void issue(int u, unsigned char* __restrict__ slice0) const {
        // slice0 = LDS address of this wave's slice for u = 0; slice u lies u*NW KiB further on
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_t*)(slice0 + u * (int)(slice_lds_step)), 16,
                                                 lane_off[u & 1] + u * slice_step, 0, 0, 0);
    }
    int slice_lds_step;
};

__device__ __forceinline__ BlockRequest make_request(const unsigned char* block_base, int rows_left,
                                                     int64_t row_bytes, uint32_t off_even, uint32_t off_odd,
                                                     int waves) {
    BlockRequest rq;
    // bytes from the block's first row to the end of the last existing row of this head
    int64_t limit = (int64_t)(rows_left - 1) * row_bytes + kHeadDim * 2;
    if (limit > 0xffffffffll) limit = 0xffffffffll;
    // raw buffer (stride 0): num_records in bytes, loads beyond it return zero; 0x00020000 is the
    // gfx9-family descriptor word for untyped 32-bit data
    rq.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(block_base), 0, (int)(uint32_t)limit, 0x00020000);
    rq.lane_off[0] = off_even;
    rq.lane_off[1] = off_odd;
    rq.slice_step = (uint32_t)(waves * 4 * row_bytes);
    rq.slice_lds_step = waves * 1024;
    return rq;
}

// The body takes the two LDS buffers as __restrict__ parameters: once inlined, every access carries
// alias-scope information, which lets the compiler's wait-count insertion tell a read of one buffer
// from an in-flight global->LDS load into the other (otherwise it waits for all of them).
template <int B>
__device__ __forceinline__ void sparse_attn_body(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ counts, const int32_t* __restrict__ indices,
    uint16_t* __restrict__ out, float* __restrict__ lse, const SeqTable& seq, int Hq, int R, int G,
    int T, int kmax, int64_t q_st, int64_t q_sh, int64_t kv_st, int64_t kv_sh, float scale,
    int items_per_xcd, unsigned char* __restrict__ k_lds, unsigned char* __restrict__ v_lds) {
    constexpr int KT = B / 32;                         // 32-key tiles per block

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

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hi = lane >> 5;
    const int qrow = w * 32 + col;                     // query row inside the block
    const int tok_q = tok_q0 + qrow;
    const bool q_valid = tok_q < seq_hi;

    const int cnt = min(counts[(int64_t)h * R + r], kmax);
    const int32_t* list = indices + ((int64_t)h * R + r) * kmax;
    const uint16_t* k_head = k + (int64_t)g * kv_sh;
    const uint16_t* v_head = v + (int64_t)g * kv_sh;

    // per-lane byte offsets of the block requests (see request_block)
    const int64_t row_bytes = kv_st * 2;
    const int lrow = w * 4 + (lane >> 4), pc = lane & 15;
    const uint32_t lane_row_off = (uint32_t)(lrow * row_bytes);
    const uint32_t k_off_even = lane_row_off + ((pc ^ (lrow & 15)) << 4);
    const uint32_t k_off_odd = (B == 128) ? k_off_even : lane_row_off + ((pc ^ ((lrow + 8) & 15)) << 4);
    const uint32_t v_off = lane_row_off + ((pc ^ ((lrow & 3) << 2)) << 4);
    auto k_request = [&](int j) {
        const int tok0 = seq_lo + j * B;
        return make_request(reinterpret_cast<const unsigned char*>(k_head + (int64_t)tok0 * kv_st), seq_hi - tok0,
                            row_bytes, k_off_even, k_off_odd, B / 32);
    };
    auto v_request = [&](int j) {
        const int tok0 = seq_lo + j * B;
        return make_request(reinterpret_cast<const unsigned char*>(v_head + (int64_t)tok0 * kv_st), seq_hi - tok0,
                            row_bytes, v_off, v_off, B / 32);
    };
    unsigned char* k_slice0 = k_lds + w * 1024;        // this wave's first request slice
    unsigned char* v_slice0 = v_lds + w * 1024;

    // List entries outside 0..i break the precondition; they are processed as fully masked
    // blocks (clamped for addressing), which costs time but keeps the control flow flat.
    auto usable = [&](int j) { return j >= 0 && j <= i; };
    auto clamped = [&](int j) { return min(max(j, 0), i); };
    int j_cur = cnt > 0 ? list[0] : 0;
    if (cnt > 0) {
        const auto rq = k_request(clamped(j_cur));
#pragma unroll
        for (int u = 0; u < 8; ++u) rq.issue(u, k_slice0);
    }

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
    const float neg_inf = -__builtin_huge_valf();
    float m_ref = neg_inf;                             // softmax reference (raw score units)
    float l_run = 0.f;                                 // this lane's share of the softmax sum
    const float sl2 = scale * 1.4426950408889634f;

    // per-lane LDS addresses that do not change between blocks
    const int k_row = swap_bits_2_3(col);              // + t*32 ; (row & 15) == (k_row & 15)
    const unsigned char* k_rd = k_lds + k_row * kRowBytes;
    const int k_swz = k_row & 15;
    // transposing V read: lane l fetches row key0 + 8*hi + (l%16)/4 (+4), 8 bytes at column
    // dt*32 + 16*((l>>4)&1) + 4*(l&3); the 64-byte group index dt is XORed with (row & 3)
    const int v_row = hi * 8 + ((lane & 15) >> 2);
    const int v_swz = v_row & 3;                       // key0 and the +4 keep (row & 3)
    const unsigned char* v_rd = v_lds + v_row * kRowBytes + (((lane >> 4) & 1) << 5) + ((lane & 3) << 3);

    auto load_k_group = [&](int grp, uint4* dst) {     // operands of matrix instructions 4*grp .. 4*grp+3 of S^T
        const int t = grp >> 1, part = grp & 1;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int c = (part * 4 + x) * 2 + hi;
            dst[x] = *reinterpret_cast<const uint4*>(k_rd + t * 32 * kRowBytes + ((c ^ k_swz) << 4));
        }
    };
    auto load_v_step = [&](int step, uint4* dst) {     // step = 16 keys; 4 d tiles x 8 keys
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const unsigned char* p0 = v_rd + step * 16 * kRowBytes + ((dt ^ v_swz) << 6);
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p0);
            const s16x4_t up = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p0 + 4 * kRowBytes));
            const uint2 lo2 = __builtin_bit_cast(uint2, lo), up2 = __builtin_bit_cast(uint2, up);
            dst[dt] = make_uint4(lo2.x, lo2.y, up2.x, up2.y);
        }
    };

    // The block's keys are handled as two halves (tiles [0, HT) and [HT, KT)) so that, inside one
    // wave's instruction stream, the softmax of one half is issued between the matrix instructions
    // of the other: vector and matrix instructions of the SAME wave overlap well, those of two
    // waves sharing a SIMD do not.
    constexpr int HT = KT / 2;                         // tiles per half
    constexpr int HG = HT * 2;                         // groups of 4 matrix instructions per half and product
    f32x16_t s_acc[KT];
    uint32_t p_pk[KT][8];                              // bf16 pairs: [tile][16-key step * 4 + pair]
    float ps[2][4];                                    // row-sum partials of the two halves

    // softmax of one accumulator pair (tile t, elements x, x+1): exp2 domain, reference m_ref,
    // packed to bf16, summed from the rounded values with one v_dot2c_f32_bf16
    auto softmax_pair = [&](int half, int t, int x, float off) {
        const float p0 = __builtin_amdgcn_exp2f(s_acc[t][x] * sl2 - off);
        const float p1 = __builtin_amdgcn_exp2f(s_acc[t][x + 1] * sl2 - off);
        const uint32_t pk = pack_bf16(p0, p1);
        p_pk[t][x >> 1] = pk;
        ps[half][(x >> 1) & 3] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pk),
                                                                 __builtin_bit_cast(bf16x2_t, 0x3f803f80u),
                                                                 ps[half][(x >> 1) & 3], false);
    };
    auto half_sum = [&](int half) { return (ps[half][0] + ps[half][1]) + (ps[half][2] + ps[half][3]); };
    // Slow path of the softmax for one half: take the true maximum, move the reference up to it
    // (rescaling O and l), and recompute the half's probabilities.
    auto fix_half = [&](int half) {
        float mx4[4] = {neg_inf, neg_inf, neg_inf, neg_inf};
#pragma unroll
        for (int t = half * HT; t < (half + 1) * HT; ++t)
#pragma unroll
            for (int x = 0; x < 16; ++x) mx4[x & 3] = fmaxf(mx4[x & 3], s_acc[t][x]);
        float mx = fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3]));
        {
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
            mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));   // both lanes of the query
        }
        if (mx > m_ref) {
            const float corr = (m_ref == neg_inf) ? 0.f : __builtin_amdgcn_exp2f((m_ref - mx) * sl2);
            m_ref = mx;
            l_run *= corr;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int x = 0; x < 16; ++x) o_acc[dt][x] *= corr;
        }
        if (m_ref == neg_inf) m_ref = 0.f;             // nothing visible yet: any finite reference
        const float off = m_ref * sl2;
#pragma unroll
        for (int e = 0; e < 4; ++e) ps[half][e] = 0.f;
#pragma unroll
        for (int t = half * HT; t < (half + 1) * HT; ++t)
#pragma unroll
            for (int x = 0; x < 16; x += 2) softmax_pair(half, t, x, off);
    };
    // a sum that is not a modest finite number (a probability above 2^16, inf, NaN) means the
    // reference is too low for this half
    auto overflowed = [&](float sum) { return __builtin_amdgcn_ballot_w64(!(sum <= 65536.0f)) != 0; };
    auto mask_half = [&](int half, int limit) {
#pragma unroll
        for (int t = half * HT; t < (half + 1) * HT; ++t)
#pragma unroll
            for (int x = 0; x < 16; ++x)
                if (t * 32 + 16 * (x >> 3) + (x & 7) > limit) s_acc[t][x] = neg_inf;
    };

    bool first_block = true;
    for (int it = 0; it < cnt; ++it) {
        const int j = clamped(j_cur);
        const bool has_next = it + 1 < cnt;
        const int j_nxt = has_next ? list[it + 1] : 0;  // scalar load, consumed after S^T
        // accumulator x of tile t is key t*32 + 16*(x/8) + 8*hi + x%8 of the block: on the diagonal
        // block keys above the query are masked; an unusable entry is masked entirely
        const bool masked = (j == i) || !usable(j_cur);
        const int mask_limit = usable(j_cur) ? qrow - 8 * hi + (i - j) : -1;

        STEM_WAIT_VMCNT(0);
        STEM_BARRIER();                                // K(j) is in LDS; V buffer is free
        const auto v_rq = v_request(j);

        // ---- S^T, first half, with the V requests in between ----
        uint4 ka[2][4];
        load_k_group(0, ka[0]);
        STEM_SCHED_FENCE();
#pragma unroll
        for (int grp = 0; grp < HG; ++grp) {
            load_k_group(grp + 1, ka[(grp + 1) & 1]);
#pragma unroll
            for (int x = 0; x < 8 / HG; ++x) v_rq.issue(grp * (8 / HG) + x, v_slice0);
            STEM_SCHED_FENCE();
            const int t = grp >> 1, part = grp & 1;
            if (part == 0) {
#pragma unroll
                for (int x = 0; x < 16; ++x) s_acc[t][x] = 0.f;
            }
#pragma unroll
            for (int x = 0; x < 4; ++x)
                s_acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka[grp & 1][x]), q_reg[part * 4 + x],
                                                                  s_acc[t], 0, 0, 0);
            STEM_SCHED_FENCE();
        }
        if (masked) mask_half(0, mask_limit);

        // ---- S^T, second half, one matrix instruction per step, with the first half's softmax
        //      (one accumulator pair per step) issued in its shadow ----
        {
            const float off = m_ref * sl2;             // -inf on the first block: redone below
#pragma unroll
            for (int e = 0; e < 4; ++e) ps[0][e] = 0.f;
#pragma unroll
            for (int grp = HG; grp < 2 * HG; ++grp) {
                if (grp + 1 < 2 * HG) load_k_group(grp + 1, ka[(grp + 1) & 1]);
                STEM_SCHED_FENCE();
                const int t = grp >> 1, part = grp & 1;
                if (part == 0) {
#pragma unroll
                    for (int x = 0; x < 16; ++x) s_acc[t][x] = 0.f;
                }
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    s_acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka[grp & 1][x]), q_reg[part * 4 + x],
                                                                      s_acc[t], 0, 0, 0);
                    const int n = (grp - HG) * 4 + x;  // softmax step: pair n of the first half
                    softmax_pair(0, n >> 3, (n & 7) * 2, off);
                    STEM_SCHED_FENCE();
                }
            }
        }
        STEM_BARRIER();                                // every wave is done with K(j)
        const auto k_rq = k_request(clamped(j_nxt));   // issued inside the first part of O^T (if has_next)
        if (masked) mask_half(1, mask_limit);
        if (first_block || overflowed(half_sum(0))) fix_half(0);
        first_block = false;
        l_run += half_sum(0);

        STEM_WAIT_VMCNT(0);
        STEM_BARRIER();                                // V(j) is in LDS

        // ---- O^T, first half of the keys, with the second half's softmax in its shadow and the
        //      next block's K requests in between ----
        uint4 va[2][4];
        load_v_step(0, va[0]);
        STEM_SCHED_FENCE();
        {
            const float off = m_ref * sl2;
#pragma unroll
            for (int e = 0; e < 4; ++e) ps[1][e] = 0.f;
#pragma unroll
            for (int g2 = 0; g2 < HG; ++g2) {
                load_v_step(g2 + 1, va[(g2 + 1) & 1]);
                if (has_next) {
#pragma unroll
                    for (int x = 0; x < 8 / HG; ++x) k_rq.issue(g2 * (8 / HG) + x, k_slice0);
                }
                STEM_SCHED_FENCE();
                const int t = g2 >> 1, u = g2 & 1;
                const uint4 pb = make_uint4(p_pk[t][u * 4], p_pk[t][u * 4 + 1], p_pk[t][u * 4 + 2], p_pk[t][u * 4 + 3]);
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    o_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[g2 & 1][dt]), as_bf16x8(pb),
                                                                       o_acc[dt], 0, 0, 0);
                    const int n = g2 * 4 + dt;         // softmax step: pair n of the second half
                    softmax_pair(1, HT + (n >> 3), (n & 7) * 2, off);
                    STEM_SCHED_FENCE();
                }
            }
        }
        if (overflowed(half_sum(1))) fix_half(1);
        l_run += half_sum(1);

        // ---- O^T, second half of the keys ----
#pragma unroll
        for (int g2 = HG; g2 < 2 * HG; ++g2) {
            if (g2 + 1 < 2 * HG) load_v_step(g2 + 1, va[(g2 + 1) & 1]);
            STEM_SCHED_FENCE();
            const int t = g2 >> 1, u = g2 & 1;
            const uint4 pb = make_uint4(p_pk[t][u * 4], p_pk[t][u * 4 + 1], p_pk[t][u * 4 + 2], p_pk[t][u * 4 + 3]);
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
                o_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[g2 & 1][dt]), as_bf16x8(pb),
                                                                   o_acc[dt], 0, 0, 0);
            STEM_SCHED_FENCE();
        }
        j_cur = j_nxt;
    }

    // ---- normalise and store: accumulator x of d tile dt is column dt*32 + 8*(x/4) + 4*hi + x%4 ----
    float l_tot;
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
        l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
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
            lse[(int64_t)h * T + tok_q] = l_tot > 0.f ? m_ref * scale + __logf(l_tot) : neg_inf;
    }
}

template <int B>
__global__ __launch_bounds__(B * 2, 2) void sparse_attn_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ counts, const int32_t* __restrict__ indices,
    uint16_t* __restrict__ out, float* __restrict__ lse, SeqTable seq, int Hq, int R, int G, int T,
    int kmax, int64_t q_st, int64_t q_sh, int64_t kv_st, int64_t kv_sh, float scale,
    int items_per_xcd) {
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds[B * kRowBytes];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds[B * kRowBytes];
    sparse_attn_body<B>(q, k, v, counts, indices, out, lse, seq, Hq, R, G, T, kmax, q_st, q_sh, kv_st,
                        kv_sh, scale, items_per_xcd, k_lds, v_lds);
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
    if (p.B == 128)
        hipLaunchKernelGGL(sparse_attn_kernel<128>, grid, dim3(256), 0, stream, qq, kk, vv, counts,
                           indices, oo, lse, p.seq, p.Hq, p.R, p.G, p.T, kmax, p.q_st, p.q_sh,
                           p.kv_st, p.kv_sh, softmax_scale, (int)per_xcd);
    else
        hipLaunchKernelGGL(sparse_attn_kernel<64>, grid, dim3(128), 0, stream, qq, kk, vv, counts,
                           indices, oo, lse, p.seq, p.Hq, p.R, p.G, p.T, kmax, p.q_st, p.q_sh,
                           p.kv_st, p.kv_sh, softmax_scale, (int)per_xcd);
    return check_launch();
}

}  // namespace stem
