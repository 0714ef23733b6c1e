// Pruning-stage scoring for chunked prefill (Alg. 2 / Alg. 3 with b_q = 16, 32 or 64 queries per
// block): the kernel template and its launcher, shared by the bf16 and the E4M3 translation units.
#pragma once

#include "prune_args.h"
#include <type_traits>

namespace ihip {

// ---------------------------------------------------------------------------
// Chunked-prefill kernel (b_q = 16*MT queries per block).  The score of a key
// is max_t q_t . k over the block's queries: a [b_q x 128] x [128 x 16] matrix
// product per 16 candidate keys, done on the matrix cores
// (v_mfma_f32_16x16x32_bf16; queries are the rows, candidates the columns, so
// the max over queries is an in-lane max over the accumulator plus two
// cross-lane steps).  One wave per query head, G waves per workgroup; a wave
// walks the searches of NT*16 chunks at a time, one candidate row per chunk
// and level.  Workgroups are ordered so that all query blocks and KV heads
// sweep the same chunk range together: the K rows they share stay in L2.
// Operand layout: lane l holds 8 consecutive dims (kq = l/16) of row/column
// l%16; accumulator lane l holds column l%16, rows 4*(l/16)..+3.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kPrefillMaxIters = 4;     // chunk groups (of 32 chunks) per workgroup, at most

//
// ROPE: relative-style dynamic RoPE (Sec. 4 "Dynamic RoPE for OOL generalization"; ApplyRopeQ /
// ApplyRopeK after Alg. 3).  Every query of the block sits at n_stream+1, a left-branch key at 0,
// a right-branch key (and the representative in the chunk score) at 1.  With a table of true
// rotations the key rotations fold into the queries: two rotated copies of the query operands,
// q_L = R(n_stream+1) q and q_R = R(n_stream) q (rounded to bf16 for the matrix cores), and every
// candidate row is scored against both, because a key that wins as the right branch is the left
// branch of the next iteration.  Twice the matrix work and twice the query registers.
//
// Precision of the rotated operands: a rotated vector is kept as two bf16 operands, its rounded
// value and the rounded rest (rotate_bf16x8_split), and the products of the rests with the other
// side's rounded values are added on the matrix cores as well, so that a score agrees with the
// product of the fp32 rotations to about 2^-16 relative and a selection is decided as an fp32
// evaluation decides it.  Relative style: both rotated query sets have a rest (the keys are not
// rotated: exact), twice the matrix work again.  Chunk-indexed style: queries and keys have one
// (q_hi.k_hi + q_lo.k_hi + q_hi.k_lo; the rests' own product is below fp32 rounding), three times the
// plain kernel's matrix work; the rests of a key tile live in a second LDS tile.
//
// ROPE == 2: chunk-indexed style.  Every key of chunk j (index in the stage's chunk list) sits at
// j, query t of the block at min(its own position, n_chunk - 1 + n_stream).  The queries differ in
// position, so nothing folds: the query operands are rotated once (each row to its own position)
// and every candidate row is rotated to its chunk's index after it has landed in LDS, each lane
// turning in place the 16 bytes it fetched itself (tile row 4r + kq is candidate column 4(r%4) + kq
// of tile r/4, whose chunk and therefore table row are the same at every level of a search: the 8
// table pieces of a lane are fetched once per chunk group).  Same carried-score search and matrix
// work as the plain kernel, plus 8 rotations and LDS round trips per level.
__device__ inline void rotate_operand_split(const bf16x8 x, const float *cos4, const float *sin4, bf16x8 &hi,
                                            bf16x8 &lo)
{
    uint4 h, l;
    rotate_bf16x8_split(__builtin_bit_cast(uint4, x), *reinterpret_cast<const float4 *>(cos4),
                        *reinterpret_cast<const float4 *>(sin4), h, l);
    hi = __builtin_bit_cast(bf16x8, h);
    lo = __builtin_bit_cast(bf16x8, l);
}

// PAGED: K is a page pool read through the sequence's row of the block table: the lane that owns a
// candidate looks its page up and forms the row's element offset (64-bit) before the offsets are
// handed to the loading lanes, so a level costs one more dependent (cache-resident) load.
//
// KV8: K rows are 128 bytes of E4M3.  There is no 8-byte direct-to-LDS load, so a lane fetches its 8
// bytes of a row into registers, repacks them as bf16 (exact) and stores the 16 bytes where the
// direct load would have put them (chunk-indexed RoPE: rotated on the way, which saves the round
// trip through LDS); everything after that is the bf16 kernel.  The chunk score is multiplied by the
// tensor's scale at the end.  K strides count 2-byte units.
//
// QS = 2: two waves per query head, each with half of the block's queries (relative-style RoPE with
// 64-query blocks, whose four rotated operand sets of 64 queries leave room for one wave per SIMD
// only; two waves of 32 queries fit a SIMD together).  The two walk the same searches on their own
// copies of the candidate rows and exchange their maxima over the queries through LDS after every
// scoring step, so that both take the same decisions.  The exchange is a handshake of the two
// waves, not a workgroup barrier: a barrier per search level puts all waves of the workgroup in
// step -- all wait for rows at once, then all multiply at once -- and the second wave per SIMD buys
// nothing (3.86 ms on the first stage of cfg4 against 3.81 ms with one wave per SIMD).  Each wave
// writes its maxima, then a turn counter (LDS keeps a wave's requests in order), and reads the
// other's maxima once the other's counter has reached the same turn.  Both write before they wait
// and both are resident (one workgroup), so the wait ends; it is bounded all the same.
template <int MT, int NT, int G, bool WIDE, int ROPE, bool PAGED, int PARTS = 1, bool KV8 = false, int QS = 1>
__global__ __launch_bounds__(64 * G * QS, QS == 2 ? 2 : (ROPE && MT == 4) ? 1 : (ROPE || (KV8 && PARTS > 1)) ? 2 : (PARTS == 1) ? 4 : 3) void prune_prefill_kernel(const PruneArgs a, const int iters,
                                                                            const RopeView rope)
{
    static_assert(NT == 2, "the shared first phase assumes two 16-chunk tiles per wave");
    static_assert(!PAGED || WIDE, "paged pools are addressed with 64-bit offsets");
    static_assert(QS == 1 || (QS == 2 && MT % 2 == 0), "one or two waves per head");
    constexpr int NWV = G * QS;                      // waves of the workgroup
    constexpr int MTW = MT / QS;                     // 16-query tiles of a wave
    constexpr int kTile = NT * 16 * kD;              // one tile: 32 rows of 256 bytes, no padding
    constexpr bool kShare = NWV >= 2;                // two tiles are needed for the shared phase
    __shared__ float sh_sigma[2][G][NT * 16];       // two buffers: a chunk group writes while the last one is still read
    __shared__ float sh_best[kPrefillMaxIters][NT * 16];      // chunk scores over the head parts done so far
    // QS == 2: a wave's maxima over its queries, for the other wave of its head (two buffers: a wave
    // may write its next values while the other still reads the last ones)
    __shared__ float sh_pair[QS == 2 ? 2 : 1][QS == 2 ? NWV : 1][2 * NT][16];
    __shared__ uint32_t sh_pair_turn[QS == 2 ? NWV : 1];      // exchanges a wave has written so far
    constexpr int kLo = ROPE == 2 ? NWV * kTile : 0;  // ROPE == 2: from a tile to the tile of its rests
    __shared__ __attribute__((aligned(16))) uint16_t sh_rows[(ROPE == 2 ? 2 * NWV : NWV) * kTile];
    // Workgroups are dealt to the 8 XCDs round-robin by linear id; let the KV head be the fastest
    // index, so that (with 8 KV heads) one XCD's L2 only ever holds one head's K rows and all
    // query blocks that share those rows run on that XCD at about the same time.
    const int p = ((blockIdx.x / a.ge.Hkv / a.ge.Mq) * a.ge.Hkv + blockIdx.x % a.ge.Hkv) * a.ge.Mq +
                  (blockIdx.x / a.ge.Hkv) % a.ge.Mq;
    const Problem pr = problem_of(a.ge, p);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int hh = wv / QS, qs = wv % QS;             // the wave's query head of the group, and its share of the queries
    const int qrow0 = qs * MTW * 16;                  // first query row of the block that is this wave's
    if (QS == 2 && lane == 0) sh_pair_turn[wv] = 0;   // a workgroup barrier follows before the first exchange
    const int n = lane & 15, kq = lane >> 4;
    // G is the number of heads (waves) a pass works on; a group of G*PARTS heads (8, where 8 waves
    // of this many registers would leave room for one workgroup per CU only) is done in PARTS
    // passes, one after the other, by the same waves
    constexpr int parts = PARTS;
    int h = pr.g * (G * PARTS) + hh;
    using off_t = typename std::conditional<WIDE, int64_t, uint32_t>::type;   // element offset of a row
    const off_t k_st = (off_t)a.k_st;

    // Rows travel from global memory straight into LDS (global_load_lds, 16 bytes per lane: 16
    // lanes fetch one whole 256-byte row, 4 rows per instruction, landing at base + lane*16) and
    // are re-read from there in the MFMA operand layout (lane = (row or column n, 8 dims of group
    // kq)).  Reading them from global memory in that layout costs four times as many L1 accesses
    // per row and makes the L1 tag rate the bound; staging through registers costs 32 VGPRs and 8
    // LDS stores per phase.  The LDS destination of a lane is fixed, so the bank swizzle is applied
    // on the source side: 16-byte slot c of tile row R holds dims 8*(c ^ (R%16)).., which makes the
    // 16 rows of an operand read hit 16 different bank groups.
    // load4(base, stride, dst, row, swz): lanes 16*kq..+15 fetch row `row` (their own copy of it)
    // to the tile row dst + kq; dst is the LDS byte address of a four-row group, wave-uniform.
    // "No candidate" is row 0 (always readable; the lane that owns the candidate substitutes it) and
    // the caller ignores the score, which keeps the loads free of branches: with exec-masked loads
    // every shuffle result has to be waited for on its own.  The instruction is written as
    // assembly so that the destinations can be computed once, outside the search loops.
    // Narrow offsets: the base is wave-uniform (scalar registers) and the lane's byte offset one
    // 24-bit multiply and an add, the load's scalar-base form.
    // `row` is never negative here: the lane that owns a candidate passes row 0 for "no candidate".
    auto load4 = [&](const uint16_t *base, off_t stride, uint32_t dst, int row, int swz) {
        const off_t r = (off_t)row;
        if constexpr (WIDE) {
            const uint16_t *src = base + r * stride + ((n ^ swz) << 3);
            uint32_t m0_saved;           // M0 is put back: the compiler is not told that it changes
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\t"
                         "s_mov_b32 m0, %0"
                         : "=&s"(m0_saved)
                         : "s"(dst), "v"(src)
                         : "memory");
        } else {
            const uint32_t byte_off = __umul24((uint32_t)r, (uint32_t)stride * 2u) + (uint32_t)((n ^ swz) << 4);
            const uint64_t b64 = (uint64_t)(uintptr_t)base;
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b64);
            const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b64 >> 32));
            const uint64_t sbase = ((uint64_t)hi << 32) | lo;
            uint32_t m0_saved;
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\t"
                         "s_mov_b32 m0, %0"
                         : "=&s"(m0_saved)
                         : "s"(dst), "v"(byte_off), "s"(sbase)
                         : "memory");
        }
    };
    // the same with the row's element offset already formed (paged K)
    auto load4_at = [&](const uint16_t *base, int64_t at, uint32_t dst, int swz) {
        const uint16_t *src = base + at + ((n ^ swz) << 3);
        uint32_t m0_saved;
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\t"
                     "s_mov_b32 m0, %0"
                     : "=&s"(m0_saved)
                     : "s"(dst), "v"(src)
                     : "memory");
    };
    // E4M3 keys: this lane's 8 bytes of row `row` (or of the row at element offset `at`), and their
    // place in a four-row group of a tile
    auto fetch8 = [&](const uint16_t *base, off_t stride, int row, int swz) {
        const off_t r = (off_t)max(row, 0);
        const off_t at = WIDE ? r * stride : (off_t)__umul24((uint32_t)r, (uint32_t)stride);
        return *reinterpret_cast<const uint2 *>(base + at + ((n ^ swz) << 2));
    };
    auto fetch8_at = [&](const uint16_t *base, int64_t at, int swz) {
        return *reinterpret_cast<const uint2 *>(base + at + ((n ^ swz) << 2));
    };
    auto put16 = [&](uint16_t *four_rows, const uint4 piece) {
        *reinterpret_cast<uint4 *>(four_rows + kq * kD + n * 8) = piece;
    };
    auto lds_addr = [&](const uint16_t *ptr) {
        return (uint32_t)__builtin_amdgcn_readfirstlane(
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)ptr);
    };
    auto operand = [&](const uint16_t *tile, int row16, int ks) {
        return *reinterpret_cast<const bf16x8 *>(&tile[(row16 + n) * kD + (((ks << 2) + kq) ^ n) * 8]);
    };

    // A operands: the block's queries, [MT tiles of 16 rows] x [4 steps of 32 dims], staged
    // through this wave's own tile, 32 rows at a time
    uint16_t *tile = &sh_rows[wv * kTile];
    uint32_t dst_own[NT * 4];                        // this wave's tile, four rows at a time
#pragma unroll
    for (int r = 0; r < NT * 4; ++r) dst_own[r] = lds_addr(tile + r * 4 * kD);
    bf16x8 qa[MTW][4];                               // relative RoPE: q_L
    bf16x8 qaR[ROPE == 1 ? MTW : 1][4];              // relative RoPE: q_R
    bf16x8 qaLo[ROPE ? MTW : 1][4];                  // RoPE: what rounding the rotated queries to bf16 dropped
    bf16x8 qaRLo[ROPE == 1 ? MTW : 1][4];
    int q_cap = 0;                                   // chunk-indexed RoPE: the largest query position
    if constexpr (ROPE == 2) {
        __shared__ int sh_n_chunk;
        q_cap = stage_n_chunk(a, pr, p, 64 * NWV, &sh_n_chunk) - 1 + a.ge.n_stream;
    }
    auto stage_queries = [&]() {
        const uint16_t *qb = a.q + pr.b * a.q_sb + (int64_t)h * a.q_sh + (int64_t)(pr.m * a.ge.b_q) * a.q_st;
#pragma unroll
        for (int m0 = 0; m0 < MTW; m0 += 2) {
            constexpr int kRows = MTW >= 2 ? 32 : 16;
#pragma unroll
            for (int r = 0; r < kRows / 4; ++r)
                load4(qb, (off_t)a.q_st, dst_own[r], qrow0 + m0 * 16 + r * 4 + kq, (r & 3) * 4 + kq);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int mt = m0; mt < m0 + 2 && mt < MTW; ++mt)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    qa[mt][ks] = operand(tile, (mt - m0) * 16, ks);
                    if constexpr (ROPE == 2) {
                        const int qpos = min(pr.E - a.ge.b_q + qrow0 + mt * 16 + n, q_cap);
                        const int64_t at = (int64_t)qpos * (kD / 2) + ((ks << 2) + kq) * 4;
                        rotate_operand_split(qa[mt][ks], rope.cos + at, rope.sin + at, qa[mt][ks], qaLo[mt][ks]);
                    }
                    if constexpr (ROPE == 1) {
                        const int pair = ((ks << 2) + kq) * 4;       // first of this operand's 4 dim pairs
                        const int64_t posR = (int64_t)a.ge.n_stream * (kD / 2) + pair, posL = posR + kD / 2;
                        rotate_operand_split(qa[mt][ks], rope.cos + posR, rope.sin + posR, qaR[mt][ks], qaRLo[mt][ks]);
                        rotate_operand_split(qa[mt][ks], rope.cos + posL, rope.sin + posL, qa[mt][ks], qaLo[mt][ks]);
                    }
                }
            // the reads must have left LDS before the next loads land in the same tile
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    };
    if constexpr (PARTS == 1) {
        stage_queries();
        if (kShare) __syncthreads();                 // other waves' tiles are written below
    }
    const uint16_t *kb = PAGED ? a.k + pr.g * a.k_sh : a.k + pr.b * a.k_sb + pr.g * a.k_sh;
    const int32_t *table = PAGED ? a.paged.block_table + (int64_t)pr.b * a.paged.table_stride : nullptr;
    const int page_mask = PAGED ? (1 << a.paged.page_log2) - 1 : 0;
    // paged K: element offset of row `pos` from kb (a row of -1 stands for row 0, as in load4)
    auto paged_at = [&](int pos) {
        const int r = max(pos, 0);
        return (int64_t)table[r >> a.paged.page_log2] * a.k_sb + (int64_t)(r & page_mask) * a.k_st;
    };

    // scores of the 32 rows of a tile (column n of 16-row tile t): max over the block's queries
    // (ROPE: sig against q_L, sigR against q_R)
    auto mfma_scores = [&](const uint16_t *src, float (&sig)[NT], float (&sigR)[NT]) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            bf16x8 kr[4], krLo[ROPE == 2 ? 4 : 1];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                kr[ks] = operand(src, t * 16, ks);
                if constexpr (ROPE == 2) krLo[ks] = operand(src + kLo, t * 16, ks);
            }
            float best = -INFINITY, bestR = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) {
                f32x4 c = {0.f, 0.f, 0.f, 0.f};
                if constexpr (ROPE != 0) {           // the small terms first
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qaLo[mt][ks], kr[ks], c, 0, 0, 0);
                }
                if constexpr (ROPE == 2) {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[mt][ks], krLo[ks], c, 0, 0, 0);
                }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[mt][ks], kr[ks], c, 0, 0, 0);
                best = fmaxf(best, fmaxf(fmaxf(c[0], c[1]), fmaxf(c[2], c[3])));
                if constexpr (ROPE == 1) {
                    f32x4 cr = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        cr = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qaRLo[mt][ks], kr[ks], cr, 0, 0, 0);
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        cr = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qaR[mt][ks], kr[ks], cr, 0, 0, 0);
                    bestR = fmaxf(bestR, fmaxf(fmaxf(cr[0], cr[1]), fmaxf(cr[2], cr[3])));
                }
            }
            sig[t] = max_over_rows(best);
            if constexpr (ROPE == 1) {
                sigR[t] = max_over_rows(bestR);
            }
        }
    };
    // QS == 2: the maxima of mfma_scores over all the block's queries, from the two waves of a head
    uint32_t pair_turn = 0;
    auto pair_max = [&](float (&sig)[NT], float (&sigR)[NT]) {
        if constexpr (QS == 2) {
            float (*mine)[16] = sh_pair[pair_turn & 1][wv];
            const float (*theirs)[16] = sh_pair[pair_turn & 1][wv ^ 1];
            if (kq == 0) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    mine[t][n] = sig[t];
                    if constexpr (ROPE == 1) mine[NT + t][n] = sigR[t];
                }
            }
            ++pair_turn;
            if (lane == 0) __hip_atomic_store(&sh_pair_turn[wv], pair_turn, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            int budget = 1 << 18;             // a wait is a few dozen turns of this loop; the bound is ~10 ms
            while ((int32_t)(__hip_atomic_load(&sh_pair_turn[wv ^ 1], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) -
                             pair_turn) < 0 && --budget > 0)
                __builtin_amdgcn_s_sleep(1);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                sig[t] = fmaxf(sig[t], theirs[t][n]);
                if constexpr (ROPE == 1) sigR[t] = fmaxf(sigR[t], theirs[NT + t][n]);
            }
        }
    };
    // chunk-indexed RoPE: table pieces of this lane's 8 rows of a tile (set per chunk group below) and
    // the in-place rotation of the 16 bytes this lane fetched with load instruction r of a tile
    float4 tb_cos[ROPE == 2 ? NT * 4 : 1], tb_sin[ROPE == 2 ? NT * 4 : 1];
    auto rotate_piece = [&](uint16_t *four_rows, const float4 c, const float4 sn) {
        uint4 *piece = reinterpret_cast<uint4 *>(four_rows + kq * kD + n * 8);
        uint4 hi, lo;
        rotate_bf16x8_split(*piece, c, sn, hi, lo);
        *piece = hi;
        *reinterpret_cast<uint4 *>(four_rows + kLo + kq * kD + n * 8) = lo;
    };
    auto rotate_own = [&](uint16_t *four_rows, int r) {      // r: compile-time after unrolling
        rotate_piece(four_rows, tb_cos[ROPE == 2 ? r : 0], tb_sin[ROPE == 2 ? r : 0]);
    };
    // table piece of this lane for load instruction r of the chunk group at jt
    auto table_at = [&](int jt, int r) {
        const int j = min(jt + (r >> 2) * 16 + (r & 3) * 4 + kq, a.max_chunks - 1);
        return (int64_t)j * (kD / 2) + ((n ^ ((r & 3) * 4 + kq)) << 2);
    };
    // score of candidate rows pos[t] of this wave's own searches.  The scores of columns whose
    // search has ended are ignored by the caller.
    auto score = [&](const int (&pos)[NT], const bool (&ok)[NT], float (&sig)[NT], float (&sigR)[NT]) {
        if constexpr (KV8) {
            uint2 raw[NT * 4];
            if constexpr (PAGED) {
                int64_t at[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) at[t] = paged_at(ok[t] ? pos[t] : -1);
#pragma unroll
                for (int r = 0; r < NT * 4; ++r)
                    raw[r] = fetch8_at(kb, __shfl(at[r >> 2], (r & 3) * 4 + kq, 64), (r & 3) * 4 + kq);
            } else {
#pragma unroll
                for (int r = 0; r < NT * 4; ++r)
                    raw[r] = fetch8(kb, k_st, __shfl(ok[r >> 2] ? pos[r >> 2] : -1, (r & 3) * 4 + kq, 64),
                                    (r & 3) * 4 + kq);
            }
#pragma unroll
            for (int r = 0; r < NT * 4; ++r) {
                uint4 piece;
                if constexpr (ROPE == 2) {
                    uint4 rest;
                    rotate_fp8x8_split(raw[r], tb_cos[r], tb_sin[r], piece, rest);
                    put16(tile + kLo + r * 4 * kD, rest);
                } else {
                    piece = fp8x8_to_bf16x8(raw[r]);
                }
                put16(tile + r * 4 * kD, piece);
            }
            // the wave reads back what its other lanes stored: LDS serves a wave's requests in order
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            mfma_scores(tile, sig, sigR);
            pair_max(sig, sigR);
            return;
        }
        if constexpr (PAGED) {
            int64_t at[NT], cand_at[NT * 4];
#pragma unroll
            for (int t = 0; t < NT; ++t) at[t] = paged_at(ok[t] ? pos[t] : -1);
#pragma unroll
            for (int r = 0; r < NT * 4; ++r) cand_at[r] = __shfl(at[r >> 2], (r & 3) * 4 + kq, 64);
#pragma unroll
            for (int r = 0; r < NT * 4; ++r) load4_at(kb, cand_at[r], dst_own[r], (r & 3) * 4 + kq);
        } else {
            int cand[NT * 4];
#pragma unroll
            for (int r = 0; r < NT * 4; ++r)     // lanes 0..15 hold column = lane
                cand[r] = __shfl(ok[r >> 2] ? pos[r >> 2] : 0, (r & 3) * 4 + kq, 64);
#pragma unroll
            for (int r = 0; r < NT * 4; ++r)     // tile row r*4 + kq = candidate (t = r/4, column (r%4)*4 + kq)
                load4(kb, k_st, dst_own[r], cand[r], (r & 3) * 4 + kq);
        }
        // the loads count on vmcnt; the wave reads its own tile, so no barrier is needed
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if constexpr (ROPE == 2) {
#pragma unroll
            for (int r = 0; r < NT * 4; ++r) rotate_own(tile + r * 4 * kD, r);
        }
        mfma_scores(tile, sig, sigR);
        pair_max(sig, sigR);
    };

    // destinations of this wave's share of the loads of the shared first phase
    uint32_t dst_shared[kShare ? 16 / NWV : 1];
#pragma unroll
    for (int i = 0; i < (kShare ? 16 / NWV : 1); ++i) dst_shared[i] = lds_addr(&sh_rows[(wv * (16 / NWV) + i) % (NWV * 8) * 4 * kD]);
    for (int part = 0; part < parts; ++part) {
    if constexpr (PARTS > 1) {
        h = pr.g * (G * PARTS) + part * G + hh;
        stage_queries();
        if (kShare) __syncthreads();                 // other waves' tiles are written below
    }
    for (int it = 0; it < iters; ++it) {
        const int jt = (blockIdx.y * iters + it) * NT * 16;
        int start[NT], len[NT], off[NT], pos[NT];
        bool valid[NT], ok[NT];
        float sigma[NT], s[NT];                      // chunk score so far; scores of the candidates
        float sL[NT], sR[NT];                        // ROPE: the current left key against q_L; candidates against q_R
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int j = jt + t * 16 + n;
            start[t] = j < a.max_chunks
                           ? slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, j)
                           : -1;
            valid[t] = start[t] >= 0;
            len[t] = valid[t] ? min(a.chunk, pr.hi - start[t]) : 0;
            off[t] = 0;
            pos[t] = start[t];
        }
        if constexpr (ROPE == 2) {
#pragma unroll
            for (int r = 0; r < NT * 4; ++r) {
                const int64_t at = table_at(jt, r);
                tb_cos[r] = *reinterpret_cast<const float4 *>(rope.cos + at);
                tb_sin[r] = *reinterpret_cast<const float4 *>(rope.sin + at);
            }
        }
        int half = a.chunk >> 1;
        if (kShare) {
            // The first key of a chunk and of its right half are the same rows for every head of
            // the group: the waves fetch them together, once (tile 0: first keys, tile 1: first
            // keys of the right halves; 16 four-row loads dealt evenly to the G waves), and each
            // wave scores both tiles against its own queries.
            constexpr int kPerWave = 16 / NWV;
            int cand[kPerWave];
            int64_t cand_at[PAGED ? kPerWave : 1];
#pragma unroll
            for (int i = 0; i < kPerWave; ++i) {
                const int ld = wv * kPerWave + i;                    // wave-uniform
                const int set = ld >> 3, r = ld & 7;
                const int st_ = (r >> 2) ? start[1] : start[0], ln_ = (r >> 2) ? len[1] : len[0];
                const int c = set == 0 ? st_ : (half >= 1 && half < ln_ ? st_ + half : -1);
                if constexpr (PAGED) cand_at[i] = __shfl(paged_at(c), (r & 3) * 4 + kq, 64);
                else cand[i] = __shfl(max(c, 0), (r & 3) * 4 + kq, 64);
            }
            if constexpr (KV8) {
                uint2 raw[kPerWave];
#pragma unroll
                for (int i = 0; i < kPerWave; ++i) {
                    const int r = (wv * kPerWave + i) & 7;
                    if constexpr (PAGED) raw[i] = fetch8_at(kb, cand_at[i], (r & 3) * 4 + kq);
                    else raw[i] = fetch8(kb, k_st, cand[i], (r & 3) * 4 + kq);
                }
#pragma unroll
                for (int i = 0; i < kPerWave; ++i) {
                    const int ld = wv * kPerWave + i;
                    uint4 piece;
                    if constexpr (ROPE == 2) {
                        const int64_t at = table_at(jt, ld & 7);
                        uint4 rest;
                        rotate_fp8x8_split(raw[i], *reinterpret_cast<const float4 *>(rope.cos + at),
                                           *reinterpret_cast<const float4 *>(rope.sin + at), piece, rest);
                        put16(&sh_rows[kLo + ld * 4 * kD], rest);
                    } else {
                        piece = fp8x8_to_bf16x8(raw[i]);
                    }
                    put16(&sh_rows[ld * 4 * kD], piece);
                }
            } else {
#pragma unroll
            for (int i = 0; i < kPerWave; ++i) {
                const int r = (wv * kPerWave + i) & 7;
                if constexpr (PAGED) load4_at(kb, cand_at[i], dst_shared[i], (r & 3) * 4 + kq);
                else load4(kb, k_st, dst_shared[i], cand[i], (r & 3) * 4 + kq);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            if constexpr (ROPE == 2 && !KV8) {
#pragma unroll
                for (int i = 0; i < kPerWave; ++i) {
                    // which of the 16 loads this is depends on the wave: the piece is fetched again
                    // rather than picked from the register array with a run-time index
                    const int ld = wv * kPerWave + i;
                    const int64_t at = table_at(jt, ld & 7);
                    rotate_piece(&sh_rows[ld * 4 * kD], *reinterpret_cast<const float4 *>(rope.cos + at),
                                 *reinterpret_cast<const float4 *>(rope.sin + at));
                }
            }
            __syncthreads();
            float l0r[NT];
            mfma_scores(&sh_rows[0], sigma, l0r);
            pair_max(sigma, l0r);
            mfma_scores(&sh_rows[kTile], s, sR);
            pair_max(s, sR);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const bool has_right = half >= 1 && half < len[t];
                if constexpr (ROPE == 1) {
                    const bool right = has_right && sR[t] > sigma[t];        // strict: tie keeps left
                    off[t] = right ? half : 0;
                    sL[t] = right ? s[t] : sigma[t];
                    sigma[t] = right ? sR[t] : l0r[t];
                } else if (has_right && s[t] > sigma[t]) { off[t] = half; sigma[t] = s[t]; }
            }
            half >>= 1;
            __syncthreads();                         // tiles 0 and 1 go back to their waves
        } else {
            score(pos, valid, sigma, sR);
            if constexpr (ROPE == 1) {
#pragma unroll
                for (int t = 0; t < NT; ++t) { sL[t] = sigma[t]; sigma[t] = sR[t]; }
            }
        }
        for (; half >= 1; half >>= 1) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                ok[t] = off[t] + half < len[t];
                pos[t] = start[t] + off[t] + half;
            }
            score(pos, ok, s, sR);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if constexpr (ROPE == 1) {
                    if (ok[t] && sR[t] > sL[t]) { off[t] += half; sL[t] = s[t]; sigma[t] = sR[t]; }
                } else if (ok[t] && s[t] > sigma[t]) { off[t] += half; sigma[t] = s[t]; }   // strict: tie keeps left
            }
        }
        // chunk score = max over the group's heads (waves)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int j = jt + t * 16 + n;
            if (kq == 0) sh_sigma[it & 1][hh][t * 16 + n] = sigma[t];
            if (a.out_rep != nullptr && kq == 0 && qs == 0 && j < a.max_chunks) {
                const int64_t row = ((int64_t)(pr.b * a.ge.Hq + h) * a.ge.Mq + pr.m);
                a.out_rep[row * a.max_chunks + j] = valid[t] ? start[t] + off[t] : -1;
            }
        }
        __syncthreads();
        if (threadIdx.x < NT * 16) {
            const int j = jt + threadIdx.x;
            if (j < a.max_chunks) {
                float best = sh_sigma[it & 1][0][threadIdx.x];
                for (int g2 = 1; g2 < G; ++g2) best = fmaxf(best, sh_sigma[it & 1][g2][threadIdx.x]);
                if (part > 0) best = fmaxf(best, sh_best[it][threadIdx.x]);
                if (part + 1 < parts) {
                    sh_best[it][threadIdx.x] = best;
                } else {
                    // validity is the same for every head; recompute it for this slot
                    const bool v = slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, j) >= 0;
                    a.out_scores[(int64_t)p * a.max_chunks + j] = v ? (KV8 ? best * a.k_scale : best) : -INFINITY;
                }
            }
        }
        // no barrier here: every wave has left its searches (the barrier above), the next chunk group
        // writes the other sh_sigma buffer, and sh_best is per chunk group
    }
    }
}

template <int MT, bool WIDE, int ROPE, bool PAGED, bool KV8 = false>
static void launch_prefill_w(const PruneArgs &a, int P, const RopeView &rope, hipStream_t st)
{
    constexpr int NT = 2;
    // several chunk groups per workgroup amortise the staging of the queries, as long as the
    // launch still has a few thousand workgroups
    int iters = kPrefillMaxIters;
    while (iters > 1 && (int64_t)P * ((a.max_chunks + NT * 16 * iters - 1) / (NT * 16 * iters)) < 2048) iters >>= 1;
    const int per_wg = NT * 16 * iters;
    dim3 grid(P, (a.max_chunks + per_wg - 1) / per_wg);
    KernelTimer timer(stage_name(kNamePrunePrefill, a.parent_starts == nullptr, a.chunk), st);
    // relative-style RoPE on 64-query blocks: two waves per head, 32 queries each
    constexpr int QS = (ROPE == 1 && MT == 4) ? 2 : 1;
    switch (a.ge.G) {
    case 1: hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 1, WIDE, ROPE, PAGED, 1, KV8, QS>), grid, dim3(64 * QS), 0, st, a, iters, rope); break;
    case 2: hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 2, WIDE, ROPE, PAGED, 1, KV8, QS>), grid, dim3(128 * QS), 0, st, a, iters, rope); break;
    case 4: hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 4, WIDE, ROPE, PAGED, 1, KV8, QS>), grid, dim3(256 * QS), 0, st, a, iters, rope); break;
    default:
        // 8 heads with 64-query blocks: 8 waves of ~160 registers fit a CU once only, two passes of 4
        // waves fit three times; with RoPE the query operands alone take more registers than 8 waves
        // leave each other
        if constexpr (MT == 4)
            hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 4, WIDE, ROPE, PAGED, 2, KV8, QS>), grid, dim3(256 * QS), 0, st, a, iters, rope);
        else
            hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 8, WIDE, ROPE, PAGED, 1, KV8>), grid, dim3(512), 0, st, a, iters, rope);
        break;
    }
}

}  // namespace ihip
