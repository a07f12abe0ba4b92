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
// K and V blocks go from global memory straight into LDS (buffer_load ... lds, no staging
// registers), one buffer each, refilled in split phases behind two barriers per block: the V block
// is requested during the first half of S^T and must have landed when S^T ends; the next K block
// is requested during O^T and must have landed when the next iteration starts.  Two workgroups
// share a CU, so one workgroup's matrix work fills the other's waits (at head size 256 the two
// 64 KiB buffers and about 490 registers leave room for one).
//
// Inside a wave the instruction stream is kept dense around the matrix instructions: LDS operands
// are read six matrix instructions ahead into a ring of registers, the softmax of a block is
// spread pair by pair over the wave's own matrix instructions (the eight pairs of a 32-key tile
// under the matrix instructions that follow the tile), and the softmax runs without a running
// maximum: a per-query reference is set
// on the first block and moved only when a window of probabilities overflows (slow path).
// The vector unit's issue slots are what the kernel runs short of (every vector instruction taken
// out of the loop shows in the run time), so whatever can go elsewhere does: the row sums of the
// probabilities are taken by the matrix pipe (a 4x4x4 product with a matrix of ones), the
// per-request address arithmetic by the scalar unit (the scalar offset operand of the loads).
//
// The kernel is a template over the block size B (64, 128) and the head size D (64, 128, 256).
//
// LDS layouts (rows of 2 D bytes, unpadded: the direct loads write 1 KiB contiguously): K has its
// 16-byte chunks XORed with (row & 15), so the 16 rows a quarter-wave reads one chunk of spread
// over all banks; V has its 64-byte groups XORed with (row & 3), which does the same for the
// 4-row x 32-byte footprint of a transposing read.  At D = 64 two 128-byte rows share the 64
// banks, so the terms are ((row >> 1) & 7) and ((row >> 1) & 1) there.  The swizzle is applied on
// the global side (each lane fetches the chunk that belongs at its LDS position).
#include <type_traits>

#include "stem_common.h"

namespace stem {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
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
// the same with only lgkmcnt set (vmcnt is split over bits [3:0] and [15:14])
#define STEM_WAIT_LGKMCNT_CASE(N) case N: __builtin_amdgcn_s_waitcnt(0xC07F | ((N) << 8)); break;
__device__ __forceinline__ void wait_lgkmcnt(int n) {   // n is a constant after unrolling: the switch folds away
    switch (n) {
        STEM_WAIT_LGKMCNT_CASE(0) STEM_WAIT_LGKMCNT_CASE(1) STEM_WAIT_LGKMCNT_CASE(2) STEM_WAIT_LGKMCNT_CASE(3)
        STEM_WAIT_LGKMCNT_CASE(4) STEM_WAIT_LGKMCNT_CASE(5) STEM_WAIT_LGKMCNT_CASE(6) STEM_WAIT_LGKMCNT_CASE(7)
        STEM_WAIT_LGKMCNT_CASE(8) STEM_WAIT_LGKMCNT_CASE(9) STEM_WAIT_LGKMCNT_CASE(10) STEM_WAIT_LGKMCNT_CASE(11)
        STEM_WAIT_LGKMCNT_CASE(12) STEM_WAIT_LGKMCNT_CASE(13) STEM_WAIT_LGKMCNT_CASE(14)
        default: break;
    }
}

// Nothing is scheduled across this point: keeps the next group of LDS operand reads ahead of the
// matrix instructions that consume the current group.
#define STEM_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Matrix instructions with the register file chosen by hand (head size 256).  A wave that may use
// more than 256 registers has them in two halves: vector registers, which every instruction can
// use, and accumulator registers, which only matrix instructions (and copies) can.  Left to itself
// the compiler then puts the results of ALL matrix instructions of a function into accumulator
// registers, also the S^T scores that the softmax has to read with vector instructions, and copies
// them back and forth (about 400 copies per block at d = 256).  Written as inline assembly the
// placement is ours: S^T results in vector registers, the O^T accumulators and the Q operands in
// accumulator registers, no copy in the loop.  The price: the compiler no longer knows these are
// matrix instructions, so the wait states it would insert are placed by hand where the instruction
// order does not already guarantee them (kManualHazards sites below): 12 issue slots between a
// 32x32x16 product and a vector access to its result, 5 after a 4x4x4 one, 2 between a vector
// write and a matrix instruction that reads it.  The build checks the finished assembly for these
// distances (wait_states.py), since register allocation may add copies the source does not show.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t as_u32x4(uint4 x) { return u32x4_t{x.x, x.y, x.z, x.w}; }
__device__ __forceinline__ void mfma_scores_first(f32x16_t& d, uint4 a, const u32x4_t& b) {
    // (early clobber: the result registers must not be the ones an operand is still read from)
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(as_u32x4(a)), "a"(b));
}
__device__ __forceinline__ void mfma_scores(f32x16_t& d, uint4 a, const u32x4_t& b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(as_u32x4(a)), "a"(b));
}
__device__ __forceinline__ void mfma_output(f32x16_t& d, uint4 a, uint4 b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(as_u32x4(a)), "v"(as_u32x4(b)));
}
// the first product into an O^T tile: nothing to add to, so no zero has to be written beforehand
__device__ __forceinline__ void mfma_output_first(f32x16_t& d, uint4 a, uint4 b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=a"(d) : "v"(as_u32x4(a)), "v"(as_u32x4(b)));
}
// Pins a Q operand to accumulator registers where it is loaded.  (Given only the "a" constraint at
// its uses, the compiler copies it there right before each use, and a matrix instruction may read
// a register a vector instruction has written only two issue slots later.)
__device__ __forceinline__ void pin_to_acc(u32x4_t& x) { asm volatile("" : "+a"(x)); }
// the row-sum product; its B operand has just been written by a vector instruction (2 wait states)
__device__ __forceinline__ void mfma_row_sum(f32x4_t& d, uint2 ones, uint2 four) {
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    asm volatile("s_nop 1\n\tv_mfma_f32_4x4x4_16b_bf16 %0, %1, %2, %0"
                 : "+v"(d)
                 : "v"(u32x2_t{ones.x, ones.y}), "v"(u32x2_t{four.x, four.y}));
}
// Idle issue slots (4 cycles each): what separates a matrix instruction's write from a dependent
// vector access when nothing else does.  Each form names the registers it protects as operands it
// "modifies": only that data dependence keeps the compiler from moving the dependent instructions
// to the other side of the wait.
template <int N, typename R>
__device__ __forceinline__ void wait_states_v(R& r) {  // r: a result in vector registers
    asm volatile("s_nop %1" : "+v"(r) : "n"(N - 1));
}
template <int N>
__device__ __forceinline__ void wait_states_acc(f32x16_t (&o)[8]) {   // o: the O^T accumulators
    asm volatile("s_nop %8"
                 : "+a"(o[0]), "+a"(o[1]), "+a"(o[2]), "+a"(o[3]), "+a"(o[4]), "+a"(o[5]), "+a"(o[6]), "+a"(o[7])
                 : "n"(N - 1));
}

// One 1 KiB slice (1024 / 2D rows) of a B x D bf16 block, global -> LDS.  A block is D / 16 slices
// per wave: wave w issues slices u*NW + w, so that the row's swizzle term depends on u with a short
// period only (1, 2 or 4).  Requests are issued one at a time between matrix
// instructions, never as a burst: the texture-address unit takes a wave's 1 KiB request at
// 64 B/clk, and a wave that finds its queue full cannot issue anything else.
//
// The loads use buffer addressing with one resource per tensor and workgroup: its base is the
// sequence's first row in this KV head and its size ends with the sequence's last row, so rows
// past the end of a partial last block (and past the end of the tensor) are never read and arrive
// in LDS as zeros (their keys are masked by causality, their values get weight 0).  A block is a
// byte offset added to the per-lane offset (one vector add per block); the slice's offset, which
// is the same for all lanes, travels in the load's scalar offset operand, which the range check
// of a raw buffer takes into account (offset >= num_records - scalar offset reads as zero).
template <int NV>
struct BlockRequest {
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t lane_off[NV];          // block offset + per-lane byte offset, for u % NV (the swizzle term of a
                                    // slice's rows repeats with period NV = 1, 2 or 4 in u)

    __device__ __forceinline__ void issue(int u, unsigned char* __restrict__ slice0, uint32_t slice_step,
                                          int slice_lds_step) const {
        // slice0 = LDS address of this wave's slice for u = 0; slice u lies u*NW KiB further on
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_t*)(slice0 + u * slice_lds_step), 16,
                                                 lane_off[u % NV], u * slice_step, 0, 0);
    }
};

// raw buffer (stride 0): num_records in bytes, loads beyond it return zero; 0x00020000 is the
// gfx9-family descriptor word for untyped 32-bit data
__device__ __forceinline__ __amdgpu_buffer_rsrc_t sequence_resource(const uint16_t* first_row, int rows,
                                                                    int64_t row_bytes, int head_bytes) {
    const int64_t bytes = rows > 0 ? (int64_t)(rows - 1) * row_bytes + head_bytes : 0;   // < 2^31 (host check)
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(first_row), 0, (int)bytes, 0x00020000);
}

// When the softmax pairs of a block are issued and where its reference may be checked, for KT
// 32-key tiles per block and KS = D / 16 matrix instructions per S^T tile.  Slot s = 0 .. 2*NS-1
// counts the wave's matrix instructions of one block (S^T first, then O^T).  Pair q = 8*t + x/2 may
// be issued once tile t of S^T is complete (slot KS*t + KS - 1) and must be done before O^T reaches
// its 16 keys (slot NS + DT*(2t + (q%8)/4), DT = KS / 2 instructions per 16-key step).  At a check
// slot every pair issued so far must be either consumed by O^T already or part of the window being
// checked (the pairs issued since the previous check), so that moving the reference there leaves
// no stale probability behind.  valid() states exactly that and is asserted at compile time.
template <int KT, int KS>
struct SoftmaxSchedule {
    static constexpr int NS = KT * KS;                 // matrix instructions per product and block
    static constexpr int DT = KS / 2;                  // matrix instructions per 16-key step of O^T
    static constexpr int NP = KT * 8;                  // accumulator pairs per block and lane
    static constexpr int kChecks = 2;
    static constexpr int kMaxPerSlot = KS < 8 ? 2 : 1;
    // The reference is checked when O^T starts (tiles 0 .. KT-2 issued, nothing consumed) and when
    // O^T reaches the last tile (its pairs issued, all others consumed).
    static constexpr int check_slot(int c) { return c == 0 ? NS : NS + KS * (KT - 1); }
    // slot after whose matrix instruction pair q is issued: the eight pairs of tile t are spread over
    // the KS slots that follow the tile's completion.  At d = 256, where the matrix instructions are
    // placed by hand, a tile's first pair keeps kLead + 1 matrix instructions (and the operand wait of
    // every second one) between itself and the instruction that completed the tile: the 12 issue
    // slots after which that instruction's result may be read by a vector instruction.
    static constexpr int kLead = KS == 16 ? 7 : 0;
    static constexpr int issue_slot(int q) { return (q / 8 + 1) * KS + kLead + ((q % 8) * (KS - kLead)) / 8; }
    // slot of the O^T instruction that first consumes pair q
    static constexpr int use_slot(int q) { return NS + DT * (2 * (q / 8) + (q % 8) / 4); }
    // pairs issued once slot `slot` is issued
    static constexpr int pairs_by(int slot) {
        int n = 0;
        for (int q = 0; q < NP; ++q) n += issue_slot(q) <= slot ? 1 : 0;
        return n;
    }
    static constexpr bool valid() {
        for (int s = 0; s < 2 * NS; ++s) {
            const int before = s == 0 ? 0 : pairs_by(s - 1), now = pairs_by(s);
            if (now < before || now > before + kMaxPerSlot) return false;
            for (int q = before; q < now; ++q) {
                if (s <= KS * (q / 8) + KS - 1) return false;                // its S^T tile is complete
                if (s >= use_slot(q)) return false;                          // O^T has not reached it
            }
        }
        int lo = 0;
        for (int c = 0; c < kChecks; ++c) {
            const int slot = check_slot(c);
            if (slot < NS || slot % DT) return false;
            if (pairs_by(slot - 1) % 2) return false;        // the row sums are taken two pairs at a time
            if (lo > 4 * ((slot - NS) / DT)) return false;   // pairs below the window are consumed (4 per step)
            for (int q = lo; q < pairs_by(slot - 1); ++q)
                if (use_slot(q) < slot) return false;        // pairs of the window are not consumed yet
            lo = pairs_by(slot - 1);
        }
        return lo == NP && pairs_by(2 * NS - 1) == NP;
    }
    // pairs_by as a table (entry slot + 1; entry 0 stands for "before slot 0"), so that the unrolled
    // kernel indexes registers with literal constants
    struct Table {
        int v[2 * NS + 1];
    };
    static constexpr Table make_table() {
        Table t{};
        for (int s = 0; s < 2 * NS; ++s) t.v[s + 1] = pairs_by(s);
        return t;
    }
    static constexpr Table kTable = make_table();
};
static_assert(SoftmaxSchedule<4, 8>::valid() && SoftmaxSchedule<2, 8>::valid(), "softmax schedule, d = 128");
static_assert(SoftmaxSchedule<4, 16>::valid() && SoftmaxSchedule<2, 16>::valid(), "softmax schedule, d = 256");
static_assert(SoftmaxSchedule<4, 4>::valid() && SoftmaxSchedule<2, 4>::valid(), "softmax schedule, d = 64");

// The body takes the two LDS buffers as __restrict__ parameters: once inlined, every access carries
// alias-scope information, which lets the compiler's wait-count insertion tell a read of one buffer
// from an in-flight global->LDS load into the other (otherwise it waits for all of them).
template <int B, int D>
__device__ __forceinline__ void sparse_attn_body(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ counts, const int32_t* __restrict__ indices,
    uint16_t* __restrict__ out, float* __restrict__ lse, const SeqTable& seq, int Hq, int R, int G,
    int T, int kmax, bool shared_lists, int64_t q_st, int64_t q_sh, int64_t kv_st, int64_t kv_sh,
    float scale, int items_per_xcd, int xcds_per_kv_head, unsigned char* __restrict__ k_lds,
    unsigned char* __restrict__ v_lds) {
    constexpr int KT = B / 32;                         // 32-key tiles per block
    constexpr int KS = D / 16;                         // 16-wide steps of S^T along d; also requests per wave, tensor and block
    constexpr int DT = D / 32;                         // 32-row tiles of O^T along d
    constexpr int NW = B / 32;                         // waves
    constexpr int kRowBytes = D * 2;                   // one K or V row in LDS
    constexpr int kSliceRows = 1024 / kRowBytes;       // rows one wave-wide 1 KiB request covers
    // head size 256 needs more than 256 registers per lane: matrix instructions by hand (see above)
    constexpr bool kManualHazards = D == 256;
    // LDS swizzles, as XORs on the 16-byte chunk index of a row: K spreads the 16 rows a quarter-wave
    // reads one chunk of over all banks, V the 4 rows x 32 bytes of a transposing read (at d = 64 two
    // 128-byte rows share the 64 banks, so the row's bit 0 does the spreading by itself)
    auto k_swz = [](int row) { return D == 64 ? (row >> 1) & 7 : row & 15; };
    auto v_swz = [](int row) { return (D == 64 ? (row >> 1) & 1 : row & 3) << 2; };

    // ---- which (head, row): consecutive workgroup ids go to different XCDs (each with its own
    // L2), so an XCD should see few KV heads, and all XCDs equal work.  With xcds_per_kv_head = m > 0
    // (Hkv divides 8) XCD x serves KV head x / m and every m-th row of it, rows descending (long
    // rows first), the G heads of a group side by side; otherwise every XCD takes a contiguous
    // range of the (KV head, row descending, head in group) order ----
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    int g, r, h;
    if (xcds_per_kv_head > 0) {
        const int rank = (slot / G) * xcds_per_kv_head + xcd % xcds_per_kv_head;
        if (slot >= items_per_xcd || rank >= R) return;
        g = xcd / xcds_per_kv_head;
        r = R - 1 - rank;
        h = g * G + slot % G;
    } else {
        const int64_t item = (int64_t)xcd * items_per_xcd + slot;
        if (slot >= items_per_xcd || item >= (int64_t)Hq * R) return;
        g = (int)(item / ((int64_t)R * G));
        const int rem = (int)(item - (int64_t)g * R * G);
        r = R - 1 - rem / G;
        h = g * G + rem % G;
    }

    const int s = seq_of_row(seq, r);
    const int ic = r - seq.row_start[s];               // row inside the call's chunk of the sequence
    const int i = seq.first_block[s] + ic;             // block index in the sequence
    const int seq_lo = seq.tok_start[s], seq_hi = seq.kv_end[s];   // key token rows the call may read
    const int tok_q0 = seq.q_tok_start[s] + ic * B;    // Q, O and lse hold the chunk's tokens only
    const int q_hi = seq.q_tok_start[s + 1];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hi = lane >> 5;
    const int qrow = w * 32 + col;                     // query row inside the block
    const int tok_q = tok_q0 + qrow;
    const bool q_valid = tok_q < q_hi;

    const int lh = shared_lists ? g : h;               // whose list: the KV head's or the query head's
    const int cnt = min(counts[(int64_t)lh * R + r], kmax);
    const int32_t* list = indices + ((int64_t)lh * R + r) * kmax;
    const uint16_t* k_head = k + (int64_t)g * kv_sh;
    const uint16_t* v_head = v + (int64_t)g * kv_sh;

    // per-lane byte offsets of the block requests (BlockRequest): slice u of wave w is the 1 KiB at
    // LDS offset (u NW + w) KiB; lane l writes chunk pc of row (u NW + w) kSliceRows + slice_row there
    // and fetches the chunk that belongs at that position, i.e. the swizzle is applied to the global
    // column.  Only the low bits of the row enter the swizzle, so it repeats in u with a short period.
    const int64_t row_bytes = kv_st * 2;
    const int slice_row = (lane * 16) / kRowBytes, pc = ((lane * 16) % kRowBytes) >> 4;
    const int lrow = w * kSliceRows + slice_row;       // row of slice u = 0
    const uint32_t lane_row_off = (uint32_t)(lrow * row_bytes);
    constexpr int kKVariants = D == 256 ? (B == 128 ? 2 : 4) : (D == 128 && B == 64) ? 2 : 1;
    static_assert(D == 64 ? (NW * kSliceRows) % 16 == 0 : (kKVariants * NW * kSliceRows) % 16 == 0,
                  "the K swizzle term of slice u repeats with period kKVariants");
    static_assert((NW * kSliceRows) % 4 == 0, "the V swizzle term does not depend on the slice");
    uint32_t k_off[kKVariants];
#pragma unroll
    for (int x = 0; x < kKVariants; ++x) k_off[x] = lane_row_off + ((pc ^ k_swz(lrow + x * NW * kSliceRows)) << 4);
    const uint32_t v_off = lane_row_off + ((pc ^ v_swz(lrow)) << 4);   // NW kSliceRows is a multiple of 4
    const auto k_rsrc = sequence_resource(k_head + (int64_t)seq_lo * kv_st, seq_hi - seq_lo, row_bytes, kRowBytes);
    const auto v_rsrc = sequence_resource(v_head + (int64_t)seq_lo * kv_st, seq_hi - seq_lo, row_bytes, kRowBytes);
    const uint32_t block_bytes = (uint32_t)(B * row_bytes);
    const uint32_t slice_step = (uint32_t)(NW * kSliceRows * row_bytes);   // rows of slices u and u+1 of one wave
    constexpr int slice_lds_step = NW * 1024;
    // !real: an offset beyond any sequence, so that nothing is fetched (zeros land in LDS)
    auto k_request = [&](int j, bool real) {
        const uint32_t off = real ? j * block_bytes : 0x80000000u;
        BlockRequest<kKVariants> rq{k_rsrc, {}};
#pragma unroll
        for (int x = 0; x < kKVariants; ++x) rq.lane_off[x] = k_off[x] + off;
        return rq;
    };
    auto v_request = [&](int j) {
        const uint32_t off = j * block_bytes;
        return BlockRequest<1>{v_rsrc, {v_off + off}};
    };
    unsigned char* k_slice0 = k_lds + w * 1024;        // this wave's first request slice
    unsigned char* v_slice0 = v_lds + w * 1024;

    // List entries outside 0..i break the precondition; they are processed as fully masked
    // blocks (clamped for addressing), which costs time but keeps the control flow flat.
    auto usable = [&](int j) { return j >= 0 && j <= i; };
    auto clamped = [&](int j) { return min(max(j, 0), i); };
    // The list lives in a vector register, 64 entries at a time (lane e holds entry e of the
    // chunk), and entries are taken out with v_readlane: no scalar load sits in the loop, so the
    // in-order LDS operand reads are the only users of their counter there.
    auto list_chunk = [&](int first) { return first + lane < cnt ? list[first + lane] : 0; };
    int list_reg = list_chunk(0);
    int j_cur = __builtin_amdgcn_readlane(list_reg, 0);
    if (cnt > 0) {
        const auto rq = k_request(clamped(j_cur), true);
#pragma unroll
        for (int u = 0; u < KS; ++u) rq.issue(u, k_slice0, slice_step, slice_lds_step);
    }

    // ---- Q rows of this wave as B operands: KS k-steps of 16 along d ----
    bf16x8_t q_reg[KS];
    u32x4_t q_acc[kManualHazards ? KS : 1];            // the same, for the hand-placed form
    {
        const uint16_t* src = q + (int64_t)tok_q * q_st + (int64_t)h * q_sh + hi * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint4 x = make_uint4(0u, 0u, 0u, 0u);
            if (q_valid) x = *reinterpret_cast<const uint4*>(src + ks * 16);
            q_reg[ks] = as_bf16x8(x);
            if constexpr (kManualHazards) {
                q_acc[ks] = as_u32x4(x);
                pin_to_acc(q_acc[ks]);
            }
        }
    }

    f32x16_t o_acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int x = 0; x < 16; ++x) o_acc[dt][x] = 0.f;
    const float neg_inf = -__builtin_huge_valf();
    float m_ref = neg_inf;                             // softmax reference (raw score units)
    float l_run = 0.f;                                 // this lane's share of the softmax sum
    const float sl2 = scale * 1.4426950408889634f;

    // per-lane LDS offsets that do not change between blocks.  Both swizzles are XORs of address
    // bits that are zero in the unswizzled per-lane offset, so the offset of operand n is one
    // v_xor of a per-lane base with a constant, plus an immediate.
    const int k_row = swap_bits_2_3(col);              // + t*32, which leaves the swizzle term alone
    const uint32_t k_base0 = k_row * kRowBytes + ((k_swz(k_row) ^ hi) << 4);
    // transposing V read: lane l fetches row key0 + 8*hi + (l%16)/4 (+4), 8 bytes at column
    // dt*32 + 16*((l>>4)&1) + 4*(l&3); the 64-byte group index dt is XORed with (row & 3)
    const int v_row = hi * 8 + ((lane & 15) >> 2);     // key0 and the +4 leave the swizzle term alone
    const uint32_t v_base0 = v_row * kRowBytes + (v_swz(v_row) << 4) + (((lane >> 4) & 1) << 5) + ((lane & 3) << 3);
    const uint32_t k_base = k_base0, v_base = v_base0;

    // Operand n of S^T (matrix instruction n: key tile n/KS, 16-wide step n%KS along d; the lane's
    // 16-byte chunk is 2*(n%KS) + hi) and of O^T (matrix instruction n: 16-key step n/DT, d tile n%DT).
    auto load_k = [&](int n) {
        const int t = n / KS, ks = n % KS;
        return *reinterpret_cast<const uint4*>(k_lds + (k_base ^ (ks << 5)) + t * 32 * kRowBytes);
    };
    auto load_v = [&](int n) {
        const int step = n / DT, dt = n % DT;
        const unsigned char* p0 = v_lds + (v_base ^ (dt << 6)) + step * 16 * kRowBytes;
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p0);
        const s16x4_t up = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p0 + 4 * kRowBytes));
        const uint2 lo2 = __builtin_bit_cast(uint2, lo), up2 = __builtin_bit_cast(uint2, up);
        return make_uint4(lo2.x, lo2.y, up2.x, up2.y);
    };
    // Operands travel through a ring of kSlots registers, read kAhead matrix instructions before
    // their use: the loaded LDS latency is several matrix instructions long.  They are consumed
    // two at a time behind one wait (every instruction, waits included, takes an issue slot of
    // the wave).  An O^T operand is two reads, and at most 15 reads can be counted in flight.
    constexpr int kSlots = 8, kAhead = 6;

    // The softmax of a block is 8*KT accumulator pairs per lane.  Vector and matrix instructions
    // of the SAME wave overlap well, those of two waves sharing a SIMD do not, so the pairs are
    // spread over the wave's own matrix instructions (SoftmaxSchedule).
    using Sched = SoftmaxSchedule<KT, KS>;
    constexpr int NS = Sched::NS;
    auto pairs_by = [](int slot) { return Sched::kTable.v[slot + 1]; };
    constexpr int kCheckSlot[2] = {Sched::check_slot(0), Sched::check_slot(1)};

    f32x16_t s_acc[KT];
    uint32_t p_pk[KT][8];                              // bf16 pairs: [tile][16-key step * 4 + pair]
    f32x4_t l_win = {0.f, 0.f, 0.f, 0.f};              // row sum of the current window (four equal copies)
    float off = 0.f;                                   // reference in exp2 units; changes on the slow path only

    // softmax of pair q (tile q/8, accumulators 2*(q%8) and +1): exp2 domain, reference m_ref,
    // packed to bf16.  The row sum is taken from the rounded values, two pairs at a time, by the
    // matrix pipe: in v_mfma_f32_4x4x4_16B_bf16 lane l supplies column l % 4 of block l / 4 of B (four
    // values along the contraction) and receives that column of the 4 x 4 result, so with A = ones
    // every lane gets the sum of its own four values, in each of its four result registers.
    auto softmax_pair = [&](int q) {
        const int t = q >> 3, x = (q & 7) * 2;
        // hand-placed form: a matrix result may be read 12 issue slots after its instruction; the
        // schedule keeps that many instructions in between (kLead), two more for margin
        if constexpr (kManualHazards) {
            static_assert(!kManualHazards || Sched::kLead + 1 + (Sched::kLead + 1) / 2 >= 12, "S^T -> softmax distance");
            if ((q & 7) == 0) wait_states_v<2>(s_acc[t]);
        }
        const float p0 = __builtin_amdgcn_exp2f(s_acc[t][x] * sl2 - off);
        const float p1 = __builtin_amdgcn_exp2f(s_acc[t][x + 1] * sl2 - off);
        uint32_t pk = pack_bf16(p0, p1);
        // An opaque use of the result at this point of the instruction stream: without it the
        // compiler gathers the softmax next to the consumer of the results instead of leaving
        // each pair next to "its" matrix instruction.
        asm volatile("" : "+v"(pk));
        p_pk[t][q & 7] = pk;
        if (q & 1) {                                   // windows hold an even number of pairs
            const uint2 four = make_uint2(p_pk[t][(q & 7) - 1], pk);
            const uint2 ones = make_uint2(0x3f803f80u, 0x3f803f80u);
            if constexpr (kManualHazards)
                mfma_row_sum(l_win, ones, four);
            else
                l_win = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(s16x4_t, ones),
                                                               __builtin_bit_cast(s16x4_t, four), l_win, 0, 0, 0);
        }
    };
    auto softmax_slot = [&](int slot) {                // one pair per slot at most (two at d = 64)
#pragma unroll
        for (int q = pairs_by(slot - 1); q < pairs_by(slot); ++q) softmax_pair(q);
    };
    auto window_sum = [&]() {
        if constexpr (kManualHazards) wait_states_v<6>(l_win);   // after the window's last row-sum product
        return l_win[0];
    };
    auto clear_sum = [&]() { l_win = f32x4_t{0.f, 0.f, 0.f, 0.f}; };
    // exp2-domain offset of the reference; a query that has seen nothing yet (m_ref = -inf) uses 0,
    // which keeps its masked scores at exp2(-inf) = 0
    auto reference_offset = [&]() { return m_ref == neg_inf ? 0.f : m_ref * sl2; };
    // Slow path for the window of pairs [q_lo, q_hi): take their true maximum, move the reference
    // up to it (rescaling O and l), and recompute the window's probabilities.
    auto fix_window = [&](int q_lo, int q_hi) {
        float mx4[4] = {neg_inf, neg_inf, neg_inf, neg_inf};
#pragma unroll
        for (int q = q_lo; q < q_hi; ++q) {
            mx4[q & 3] = fmaxf(mx4[q & 3], fmaxf(s_acc[q >> 3][(q & 7) * 2], s_acc[q >> 3][(q & 7) * 2 + 1]));
        }
        float mx = fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3]));
        {
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
            mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));   // both lanes of the query
        }
        if (mx > m_ref) {
            const float corr = (m_ref == neg_inf) ? 0.f : __builtin_amdgcn_exp2f((m_ref - mx) * sl2);
            m_ref = mx;
            l_run *= corr;
            if constexpr (kManualHazards) wait_states_acc<16>(o_acc);   // the last O^T instruction has written
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int x = 0; x < 16; ++x) o_acc[dt][x] *= corr;
            if constexpr (kManualHazards) wait_states_acc<4>(o_acc);    // before the next one reads them
        }
        off = reference_offset();
        clear_sum();
#pragma unroll
        for (int q = q_lo; q < q_hi; ++q) softmax_pair(q);
    };
    // The first window of a row, pairs [0, q_hi): O and l are still zero, so there is nothing to
    // rescale; a query that sees none of the window's keys keeps m_ref = -inf (offset 0, zero
    // probabilities) and gets its reference from a later window's slow path.
    auto first_window = [&](int q_hi) {
        float mx4[4] = {neg_inf, neg_inf, neg_inf, neg_inf};
#pragma unroll
        for (int q = 0; q < q_hi; ++q) {
            mx4[q & 3] = fmaxf(mx4[q & 3], fmaxf(s_acc[q >> 3][(q & 7) * 2], s_acc[q >> 3][(q & 7) * 2 + 1]));
        }
        float mx = fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3]));
        {
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
            mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));   // both lanes of the query
        }
        m_ref = mx;
        off = reference_offset();
        clear_sum();
#pragma unroll
        for (int q = 0; q < q_hi; ++q) softmax_pair(q);
        l_run += window_sum();
        clear_sum();
    };
    // A window needs the slow path if a query has no reference yet (nothing visible to it so far:
    // every query on the first block) or if its sum is not a modest finite number (a probability
    // above 2^16, inf, NaN: the reference is too low for this window).
    auto needs_fix = [&](float sum) {
        return __builtin_amdgcn_ballot_w64(m_ref == neg_inf || !(sum <= 65536.0f)) != 0;
    };
    auto check_window = [&](int c) {                   // at slot boundary kCheckSlot[c]
        const int q_lo = c == 0 ? 0 : pairs_by(kCheckSlot[c - 1] - 1), q_hi = pairs_by(kCheckSlot[c] - 1);
        if (needs_fix(window_sum())) fix_window(q_lo, q_hi);
        l_run += window_sum();
        clear_sum();
    };
    // accumulator x of tile t is key t*32 + 16*(x/8) + 8*hi + x%8 of the block
    auto mask_tile = [&](int t, int limit) {
        if constexpr (kManualHazards) wait_states_v<16>(s_acc[t]);   // the tile's last matrix instruction has written
#pragma unroll
        for (int x = 0; x < 16; ++x)
            if (t * 32 + 16 * (x >> 3) + (x & 7) > limit) s_acc[t][x] = neg_inf;
    };

    constexpr int kStepsPerRequestV = (NS / 2) / KS;   // V's KS requests go under the first half of S^T,
    constexpr int kStepsPerRequestK = NS / KS;         // the next K's under all of O^T
    const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // One listed block.  The first block of a row is a version of its own (first_tag = true): no
    // query has a reference yet, so the probabilities of the first window cannot be formed under
    // the S^T products; they are formed once, at the first check point, from the window's maximum.
    auto one_block = [&](int it, auto first_tag) {
        constexpr bool kFirst = decltype(first_tag)::value;
        const int j = clamped(j_cur);
        const bool has_next = it + 1 < cnt;
        if (((it + 1) & 63) == 0) list_reg = list_chunk(it + 1);
        // on the diagonal block keys above the query are masked; an unusable entry is masked entirely
        const bool masked = (j == i) || !usable(j_cur);
        const int mask_limit = usable(j_cur) ? qrow - 8 * hi + (i - j) : -1;

        STEM_WAIT_VMCNT(0);
        STEM_BARRIER();                                // K(j) is in LDS; V buffer is free

        // ---- S^T = K Q^T, with the V requests in between during the first half ----
        uint4 ka[kSlots];
#pragma unroll
        for (int n = 0; n < kAhead; ++n) ka[n] = load_k(n);
        const auto v_rq = v_request(j);
        const int j_nxt = __builtin_amdgcn_readlane(list_reg, (it + 1) & 63);   // 0 past the end
        clear_sum();
        STEM_SCHED_FENCE();
#pragma unroll
        for (int t = 0; t < KT; ++t) {
#pragma unroll
            for (int n = t * KS; n < t * KS + KS; ++n) {
                if ((n & 1) == 0) {
                    if (n + kAhead < NS) ka[(n + kAhead) % kSlots] = load_k(n + kAhead);
                    if (n + kAhead + 1 < NS) ka[(n + kAhead + 1) % kSlots] = load_k(n + kAhead + 1);
                    wait_lgkmcnt((n + kAhead + 2 < NS ? kAhead + 2 : NS - n) - 2);
                }
                if (n < NS / 2 && n % kStepsPerRequestV == 0)
                    v_rq.issue(n / kStepsPerRequestV, v_slice0, slice_step, slice_lds_step);
                if constexpr (kManualHazards) {
                    if ((n % KS) == 0) mfma_scores_first(s_acc[t], ka[n % kSlots], q_acc[n % KS]);
                    else mfma_scores(s_acc[t], ka[n % kSlots], q_acc[n % KS]);
                } else {
                    s_acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka[n % kSlots]), q_reg[n % KS],
                                                                      (n % KS) == 0 ? zero16 : s_acc[t], 0, 0, 0);
                }
                if constexpr (!kFirst) softmax_slot(n);
                STEM_SCHED_FENCE();
            }
            if (masked) mask_tile(t, mask_limit);
        }

        STEM_WAIT_VMCNT(0);
        STEM_BARRIER();                                // every wave is done with K(j); V(j) is in LDS

        // ---- O^T += V^T P^T.  The next block's K requests are spread over the whole product;
        //      after the last block they are empty (a zero-sized resource: nothing is fetched) ----
        uint4 va[kSlots];
#pragma unroll
        for (int n = 0; n < kAhead; ++n) va[n] = load_v(n);
        const auto k_rq = k_request(clamped(j_nxt), has_next);
        STEM_SCHED_FENCE();
        auto pv_range = [&](int n_lo, int n_hi) {      // even bounds
#pragma unroll
            for (int n = n_lo; n < n_hi; ++n) {
                if ((n & 1) == 0) {
                    if (n + kAhead < NS) va[(n + kAhead) % kSlots] = load_v(n + kAhead);
                    wait_lgkmcnt(2 * ((n + kAhead + 1 < NS ? kAhead + 1 : NS - n) - 2));
                } else {
                    if (n + kAhead < NS) va[(n + kAhead) % kSlots] = load_v(n + kAhead);
                }
                if (n % kStepsPerRequestK == 1) k_rq.issue(n / kStepsPerRequestK, k_slice0, slice_step, slice_lds_step);
                const int g2 = n / DT, t = g2 >> 1, u = g2 & 1, dt = n % DT;
                const uint4 pb = make_uint4(p_pk[t][u * 4], p_pk[t][u * 4 + 1], p_pk[t][u * 4 + 2], p_pk[t][u * 4 + 3]);
                if constexpr (kManualHazards) {
                    if (kFirst && n < DT) mfma_output_first(o_acc[dt], va[n % kSlots], pb);
                    else mfma_output(o_acc[dt], va[n % kSlots], pb);
                } else
                    o_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[n % kSlots]), as_bf16x8(pb),
                                                                       o_acc[dt], 0, 0, 0);
                softmax_slot(NS + n);
                STEM_SCHED_FENCE();
            }
        };
        if constexpr (kFirst) first_window(pairs_by(kCheckSlot[0] - 1));
        else check_window(0);
        pv_range(0, kCheckSlot[1] - NS);
        check_window(1);
        pv_range(kCheckSlot[1] - NS, NS);
        j_cur = j_nxt;
    };
    if (cnt > 0) one_block(0, std::true_type{});
    for (int it = 1; it < cnt; ++it) one_block(it, std::false_type{});
    STEM_WAIT_VMCNT(0);                                // no request may outlive the workgroup's LDS
    if constexpr (kManualHazards) wait_states_acc<16>(o_acc);   // the last O^T instructions have written

    // ---- normalise and store: accumulator x of d tile dt is column dt*32 + 8*(x/4) + 4*hi + x%4 ----
    float l_tot;
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
        l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    // A lane holds four columns of every group of eight (the other four sit in lane ^ 32).  Two
    // groups at a time, one half-wave swap per packed register gives each lane eight consecutive
    // columns, i.e. 16-byte stores.  (The swap runs in every lane, valid query or not.)
    uint4 packed[DT][2];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int xa = m * 8, xb = m * 8 + 4;      // accumulators of groups 2m and 2m+1
            const uint32_t a0 = pack_bf16(o_acc[dt][xa + 0] * inv, o_acc[dt][xa + 1] * inv);
            const uint32_t a1 = pack_bf16(o_acc[dt][xa + 2] * inv, o_acc[dt][xa + 3] * inv);
            const uint32_t b0 = pack_bf16(o_acc[dt][xb + 0] * inv, o_acc[dt][xb + 1] * inv);
            const uint32_t b1 = pack_bf16(o_acc[dt][xb + 2] * inv, o_acc[dt][xb + 3] * inv);
            const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
            const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
            packed[dt][m] = make_uint4(s0[0], s1[0], s0[1], s1[1]);
        }
    if (q_valid) {
        uint16_t* dst = out + (int64_t)tok_q * q_st + (int64_t)h * q_sh + hi * 8;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int m = 0; m < 2; ++m) *reinterpret_cast<uint4*>(dst + dt * 32 + m * 16) = packed[dt][m];
        if (lse != nullptr && hi == 0)
            lse[(int64_t)h * T + tok_q] = l_tot > 0.f ? m_ref * scale + __logf(l_tot) : neg_inf;
    }
}

template <int B, int D>
__global__ __launch_bounds__(B * 2, D == 256 ? 1 : 2) void sparse_attn_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ counts, const int32_t* __restrict__ indices,
    uint16_t* __restrict__ out, float* __restrict__ lse, SeqTable seq, int Hq, int R, int G, int T,
    int kmax, bool shared_lists, int64_t q_st, int64_t q_sh, int64_t kv_st, int64_t kv_sh, float scale,
    int items_per_xcd, int xcds_per_kv_head) {
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds[B * D * 2];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds[B * D * 2];
    sparse_attn_body<B, D>(q, k, v, counts, indices, out, lse, seq, Hq, R, G, T, kmax, shared_lists, q_st, q_sh,
                           kv_st, kv_sh, scale, items_per_xcd, xcds_per_kv_head, k_lds, v_lds);
}

int launch_sparse_attn(const Problem& p, const void* q, const void* k, const void* v,
                       const int32_t* counts, const int32_t* indices, int32_t kmax,
                       bool lists_per_kv_head, float softmax_scale, void* out, float* lse,
                       hipStream_t stream) {
    // (the host entry point has checked that one sequence of one KV head spans less than 2 GiB: the
    // block requests use a 32-bit byte offset, with offsets from 2^31 on reserved for "fetch nothing")
    const int64_t items = (int64_t)p.Hq * p.R;
    const int xcds_per_kv_head = (p.Hkv <= 8 && 8 % p.Hkv == 0) ? 8 / p.Hkv : 0;
    const int64_t per_xcd = xcds_per_kv_head > 0
                                ? (int64_t)((p.R + xcds_per_kv_head - 1) / xcds_per_kv_head) * p.G
                                : (items + 7) / 8;
    if (per_xcd * 8 > 0x7fffffff) return STEM_ERR_UNSUPPORTED;
    dim3 grid((unsigned)(per_xcd * 8)), block(p.B * 2);
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint16_t* kk = static_cast<const uint16_t*>(k);
    const uint16_t* vv = static_cast<const uint16_t*>(v);
    uint16_t* oo = static_cast<uint16_t*>(out);
#define STEM_ATTN_LAUNCH(BB, DD)                                                                          \
    hipLaunchKernelGGL((sparse_attn_kernel<BB, DD>), grid, block, 0, stream, qq, kk, vv, counts, indices, \
                       oo, lse, p.seq, p.Hq, p.R, p.G, p.T, kmax, lists_per_kv_head, p.q_st, p.q_sh,      \
                       p.kv_st, p.kv_sh, softmax_scale, (int)per_xcd, xcds_per_kv_head)
    if (p.B == 128 && p.d == 128) STEM_ATTN_LAUNCH(128, 128);
    else if (p.B == 64 && p.d == 128) STEM_ATTN_LAUNCH(64, 128);
    else if (p.B == 128 && p.d == 64) STEM_ATTN_LAUNCH(128, 64);
    else if (p.B == 64 && p.d == 64) STEM_ATTN_LAUNCH(64, 64);
    else if (p.B == 128 && p.d == 256) STEM_ATTN_LAUNCH(128, 256);
    else if (p.B == 64 && p.d == 256) STEM_ATTN_LAUNCH(64, 256);
    else return STEM_ERR_UNSUPPORTED;
#undef STEM_ATTN_LAUNCH
    return check_launch();
}

}  // namespace stem
