// Pruning-stage scoring: representative search (Alg. 3) + chunk score (Alg. 2).
//
// Decode kernel (b_q == 1).  HBM-latency/bandwidth bound gather: each chunk
// needs 1 + log2(l_c) dependent 256-byte row reads per query head.  Mapping:
// 16 lanes share one K row (16 B per lane -> one fully coalesced 256 B read),
// so a wave works on 4 chunk slots at a time and a 16-lane group walks the
// searches of all G query heads of its KV head together (the first two rows
// of a chunk are common to the heads, the rest are G independent loads in
// flight).  U slots per group are interleaved to put more loads in flight.
#include "prune_args.h"
#include <type_traits>

namespace ihip {

// KV8: K rows are 128 bytes of E4M3 (8 bytes per lane); the dot products run on the decoded values
// and the chunk score is multiplied by the tensor's scale.
template <int G, int U, int SRC, bool KV8>
__global__ __launch_bounds__(256) void prune_decode_kernel(const PruneArgs a)
{
    using piece_t = typename std::conditional<KV8, uint2, uint4>::type;     // a lane's share of a row
    const int p = blockIdx.y;
    const Problem pr = problem_of(a.ge, p);
    const int l16 = threadIdx.x & 15;
    const int grp = threadIdx.x >> 4;
    const int j0 = (blockIdx.x * 16 + grp) * U;
    if (j0 >= a.max_chunks) return;

    // this lane's 8 dims of the G query vectors
    float qf[G][8];
    {
        const uint16_t *qb = a.q + pr.b * a.q_sb + (int64_t)(pr.g * G) * a.q_sh +
                             (int64_t)(pr.m * a.ge.b_q) * a.q_st;
#pragma unroll
        for (int h = 0; h < G; ++h) unpack8(load_row16(qb, h * a.q_sh, l16), qf[h]);
    }
    const typename KeySource<SRC>::type src = KeySource<SRC>::make(a, pr);
    const bool leader = l16 == 0;
    const piece_t zero = {};

    int start[U], len[U];
    bool valid[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int j = j0 + u;
        start[u] = j < a.max_chunks
                       ? slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, j)
                       : -1;
        valid[u] = start[u] >= 0;
        len[u] = valid[u] ? min(a.chunk, pr.hi - start[u]) : 0;
    }

    // Paged K: the page ids of a chunk's first 16 pages are fetched once, one per lane of the row
    // group (one coalesced read of the block table), and handed round by a shuffle, so that the
    // search below has no table lookup in front of every row read.
    int page_first[U], page_ids[U];
    if (SRC == 2) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            page_first[u] = max(start[u], 0) >> a.paged.page_log2;
            const int e = page_first[u] + l16;
            page_ids[u] = valid[u] && e < a.paged.table_stride
                              ? a.paged.block_table[(int64_t)pr.b * a.paged.table_stride + e] : 0;
        }
    }
    // page id of row `pos` of chunk u (paged K; every lane of the row group takes part in the shuffle)
    auto page_of = [&](int pos, int u) {
        if constexpr (SRC == 2) {
            const int idx = (pos >> a.paged.page_log2) - page_first[u];
            int page = __shfl(page_ids[u], idx & 15, 16);
            if (idx >= 16) page = src.table[pos >> a.paged.page_log2];      // chunk wider than 16 pages
            return page;
        } else {
            return 0;
        }
    };
    // row `pos` (in page `page`, if K is paged): this lane's share of it
    auto load_row = [&](int pos, int page) {
        if constexpr (SRC == 2)
            return *reinterpret_cast<const piece_t *>(src.row_in_page(page, pos) + l16 * (KV8 ? 4 : 8));
        else
            return *reinterpret_cast<const piece_t *>(src.row(pos, leader) + l16 * (KV8 ? 4 : 8));
    };

    int off[U][G];
    float sigma[U][G];

    // first key of the chunk, and the first key of its right half: common to all heads
    {
        piece_t r0[U], r1[U];
        const int mid = a.chunk >> 1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            r0[u] = zero;
            r1[u] = zero;
            const int pg0 = page_of(max(start[u], 0), u), pg1 = page_of(max(start[u], 0) + mid, u);
            if (valid[u]) r0[u] = load_row(start[u], pg0);
            if (mid >= 1 && mid < len[u]) r1[u] = load_row(start[u] + mid, pg1);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float s0 = row16_sum(dot8(r0[u], qf[h]));
                const float s1 = row16_sum(dot8(r1[u], qf[h]));
                const bool right = (mid >= 1 && mid < len[u]) && s1 > s0;   // strict: tie keeps left
                off[u][h] = right ? mid : 0;
                sigma[u][h] = right ? s1 : s0;
            }
        }
    }

    // remaining halvings: G*U independent row reads per step
    for (int half = a.chunk >> 2; half >= 1; half >>= 1) {
        piece_t r[U][G];
        bool ok[U][G];
        int page[U][G];      // all shuffles first, then all loads: one wait instead of one per row
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int h = 0; h < G; ++h) page[u][h] = page_of(max(start[u], 0) + off[u][h] + half, u);
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const int mid = off[u][h] + half;
                ok[u][h] = mid < len[u];
                r[u][h] = zero;
                if (ok[u][h]) r[u][h] = load_row(start[u] + mid, page[u][h]);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float s = row16_sum(dot8(r[u][h], qf[h]));
                if (ok[u][h] && s > sigma[u][h]) {
                    off[u][h] += half;
                    sigma[u][h] = s;
                }
            }
        }
    }

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int j = j0 + u;
        if (j >= a.max_chunks) break;
        float best = sigma[u][0];
#pragma unroll
        for (int h = 1; h < G; ++h) best = fmaxf(best, sigma[u][h]);
        if (KV8) best *= a.k_scale;
        if (l16 == 0) a.out_scores[(int64_t)p * a.max_chunks + j] = valid[u] ? best : -INFINITY;
        if (a.out_rep != nullptr && l16 < G) {
            int o = off[u][0];
#pragma unroll
            for (int h = 1; h < G; ++h) o = (l16 == h) ? off[u][h] : o;
            const int64_t row = ((int64_t)(pr.b * a.ge.Hq + pr.g * G + l16) * a.ge.Mq + pr.m);
            a.out_rep[row * a.max_chunks + j] = valid[u] ? start[u] + o : -1;
        }
    }
}

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
// ROPE == 2: chunk-indexed style.  Every key of chunk j (index in the stage's chunk list) sits at
// j, query t of the block at min(its own position, n_chunk - 1 + n_stream).  The queries differ in
// position, so nothing folds: the query operands are rotated once (each row to its own position)
// and every candidate row is rotated to its chunk's index after it has landed in LDS, each lane
// turning in place the 16 bytes it fetched itself (tile row 4r + kq is candidate column 4(r%4) + kq
// of tile r/4, whose chunk and therefore table row are the same at every level of a search: the 8
// table pieces of a lane are fetched once per chunk group).  Same carried-score search and matrix
// work as the plain kernel, plus 8 rotations and LDS round trips per level.
__device__ inline bf16x8 rotate_operand(const bf16x8 x, const float *cos4, const float *sin4)
{
    return __builtin_bit_cast(bf16x8, rotate_bf16x8(__builtin_bit_cast(uint4, x), cos4, sin4));
}

// PAGED: K is a page pool read through the sequence's row of the block table: the lane that owns a
// candidate looks its page up and forms the row's element offset (64-bit) before the offsets are
// handed to the loading lanes, so a level costs one more dependent (cache-resident) load.
template <int MT, int NT, int G, bool WIDE, int ROPE, bool PAGED, int PARTS = 1>
__global__ __launch_bounds__(64 * G, ROPE ? 2 : 3) void prune_prefill_kernel(const PruneArgs a, const int iters,
                                                                            const RopeView rope)
{
    static_assert(NT == 2, "the shared first phase assumes two 16-chunk tiles per wave");
    static_assert(!PAGED || WIDE, "paged pools are addressed with 64-bit offsets");
    constexpr int kTile = NT * 16 * kD;              // one tile: 32 rows of 256 bytes, no padding
    constexpr bool kShare = G >= 2;                  // two tiles are needed for the shared phase
    __shared__ float sh_sigma[G][NT * 16];
    __shared__ float sh_best[kPrefillMaxIters][NT * 16];      // chunk scores over the head parts done so far
    __shared__ __attribute__((aligned(16))) uint16_t sh_rows[G * kTile];
    // Workgroups are dealt to the 8 XCDs round-robin by linear id; let the KV head be the fastest
    // index, so that (with 8 KV heads) one XCD's L2 only ever holds one head's K rows and all
    // query blocks that share those rows run on that XCD at about the same time.
    const int p = ((blockIdx.x / a.ge.Hkv / a.ge.Mq) * a.ge.Hkv + blockIdx.x % a.ge.Hkv) * a.ge.Mq +
                  (blockIdx.x / a.ge.Hkv) % a.ge.Mq;
    const Problem pr = problem_of(a.ge, p);
    const int lane = threadIdx.x & 63, hh = threadIdx.x >> 6;      // wave = query head of the group
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
    // to the tile row dst + kq; dst is the LDS byte address of a four-row group, wave-uniform.  A
    // row of -1 stands for "no candidate": row 0 is fetched instead (always readable) and the
    // caller ignores the score, which keeps the loads free of branches: with exec-masked loads
    // every shuffle result has to be waited for on its own.  The instruction is written as
    // assembly so that the destinations can be computed once, outside the search loops.
    auto load4 = [&](const uint16_t *base, off_t stride, uint32_t dst, int row, int swz) {
        const off_t r = (off_t)max(row, 0);
        const off_t at = WIDE ? r * stride : (off_t)__umul24((uint32_t)r, (uint32_t)stride);
        const uint16_t *src = base + at + ((n ^ swz) << 3);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory");
    };
    // the same with the row's element offset already formed (paged K)
    auto load4_at = [&](const uint16_t *base, int64_t at, uint32_t dst, int swz) {
        const uint16_t *src = base + at + ((n ^ swz) << 3);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory");
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
    uint16_t *tile = &sh_rows[hh * kTile];
    uint32_t dst_own[NT * 4];                        // this wave's tile, four rows at a time
#pragma unroll
    for (int r = 0; r < NT * 4; ++r) dst_own[r] = lds_addr(tile + r * 4 * kD);
    bf16x8 qa[MT][4];                                // relative RoPE: q_L
    bf16x8 qaR[ROPE == 1 ? MT : 1][4];               // relative RoPE: q_R
    int q_cap = 0;                                   // chunk-indexed RoPE: the largest query position
    if constexpr (ROPE == 2) {
        __shared__ int sh_n_chunk;
        q_cap = stage_n_chunk(a, pr, p, 64 * G, &sh_n_chunk) - 1 + a.ge.n_stream;
    }
    auto stage_queries = [&]() {
        const uint16_t *qb = a.q + pr.b * a.q_sb + (int64_t)h * a.q_sh + (int64_t)(pr.m * a.ge.b_q) * a.q_st;
#pragma unroll
        for (int m0 = 0; m0 < MT; m0 += 2) {
            constexpr int kRows = MT >= 2 ? 32 : 16;
#pragma unroll
            for (int r = 0; r < kRows / 4; ++r)
                load4(qb, (off_t)a.q_st, dst_own[r], m0 * 16 + r * 4 + kq, (r & 3) * 4 + kq);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int mt = m0; mt < m0 + 2 && mt < MT; ++mt)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    qa[mt][ks] = operand(tile, (mt - m0) * 16, ks);
                    if constexpr (ROPE == 2) {
                        const int qpos = min(pr.E - a.ge.b_q + mt * 16 + n, q_cap);
                        const int64_t at = (int64_t)qpos * (kD / 2) + ((ks << 2) + kq) * 4;
                        qa[mt][ks] = rotate_operand(qa[mt][ks], rope.cos + at, rope.sin + at);
                    }
                    if constexpr (ROPE == 1) {
                        const int pair = ((ks << 2) + kq) * 4;       // first of this operand's 4 dim pairs
                        const int64_t posR = (int64_t)a.ge.n_stream * (kD / 2) + pair, posL = posR + kD / 2;
                        qaR[mt][ks] = rotate_operand(qa[mt][ks], rope.cos + posR, rope.sin + posR);
                        qa[mt][ks] = rotate_operand(qa[mt][ks], rope.cos + posL, rope.sin + posL);
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
        bf16x8 kr[NT][4];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) kr[t][ks] = operand(src, t * 16, ks);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float best = -INFINITY, bestR = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[mt][ks], kr[t][ks], c, 0, 0, 0);
                best = fmaxf(best, fmaxf(fmaxf(c[0], c[1]), fmaxf(c[2], c[3])));
                if constexpr (ROPE == 1) {
                    f32x4 cr = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        cr = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qaR[mt][ks], kr[t][ks], cr, 0, 0, 0);
                    bestR = fmaxf(bestR, fmaxf(fmaxf(cr[0], cr[1]), fmaxf(cr[2], cr[3])));
                }
            }
            best = fmaxf(best, __shfl_xor(best, 16, 64));
            best = fmaxf(best, __shfl_xor(best, 32, 64));
            sig[t] = best;
            if constexpr (ROPE == 1) {
                bestR = fmaxf(bestR, __shfl_xor(bestR, 16, 64));
                bestR = fmaxf(bestR, __shfl_xor(bestR, 32, 64));
                sigR[t] = bestR;
            }
        }
    };
    // chunk-indexed RoPE: table pieces of this lane's 8 rows of a tile (set per chunk group below) and
    // the in-place rotation of the 16 bytes this lane fetched with load instruction r of a tile
    float4 tb_cos[ROPE == 2 ? NT * 4 : 1], tb_sin[ROPE == 2 ? NT * 4 : 1];
    auto rotate_piece = [&](uint16_t *four_rows, const float4 c, const float4 sn) {
        uint4 *piece = reinterpret_cast<uint4 *>(four_rows + kq * kD + n * 8);
        *piece = rotate_bf16x8(*piece, c, sn);
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
                cand[r] = __shfl(ok[r >> 2] ? pos[r >> 2] : -1, (r & 3) * 4 + kq, 64);
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
    };

    // destinations of this wave's share of the loads of the shared first phase
    uint32_t dst_shared[kShare ? 16 / G : 1];
#pragma unroll
    for (int i = 0; i < (kShare ? 16 / G : 1); ++i) dst_shared[i] = lds_addr(&sh_rows[(hh * (16 / G) + i) % (G * 8) * 4 * kD]);
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
            constexpr int kPerWave = 16 / G;
            int cand[kPerWave];
            int64_t cand_at[PAGED ? kPerWave : 1];
#pragma unroll
            for (int i = 0; i < kPerWave; ++i) {
                const int ld = hh * kPerWave + i;                    // wave-uniform
                const int set = ld >> 3, r = ld & 7;
                const int st_ = (r >> 2) ? start[1] : start[0], ln_ = (r >> 2) ? len[1] : len[0];
                const int c = set == 0 ? st_ : (half >= 1 && half < ln_ ? st_ + half : -1);
                if constexpr (PAGED) cand_at[i] = __shfl(paged_at(c), (r & 3) * 4 + kq, 64);
                else cand[i] = __shfl(c, (r & 3) * 4 + kq, 64);
            }
#pragma unroll
            for (int i = 0; i < kPerWave; ++i) {
                const int r = (hh * kPerWave + i) & 7;
                if constexpr (PAGED) load4_at(kb, cand_at[i], dst_shared[i], (r & 3) * 4 + kq);
                else load4(kb, k_st, dst_shared[i], cand[i], (r & 3) * 4 + kq);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if constexpr (ROPE == 2) {
#pragma unroll
                for (int i = 0; i < kPerWave; ++i) {
                    // which of the 16 loads this is depends on the wave: the piece is fetched again
                    // rather than picked from the register array with a run-time index
                    const int ld = hh * kPerWave + i;
                    const int64_t at = table_at(jt, ld & 7);
                    rotate_piece(&sh_rows[ld * 4 * kD], *reinterpret_cast<const float4 *>(rope.cos + at),
                                 *reinterpret_cast<const float4 *>(rope.sin + at));
                }
            }
            __syncthreads();
            float l0r[NT];
            mfma_scores(&sh_rows[0], sigma, l0r);
            mfma_scores(&sh_rows[kTile], s, sR);
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
            if (kq == 0) sh_sigma[hh][t * 16 + n] = sigma[t];
            if (a.out_rep != nullptr && kq == 0 && j < a.max_chunks) {
                const int64_t row = ((int64_t)(pr.b * a.ge.Hq + h) * a.ge.Mq + pr.m);
                a.out_rep[row * a.max_chunks + j] = valid[t] ? start[t] + off[t] : -1;
            }
        }
        __syncthreads();
        if (threadIdx.x < NT * 16) {
            const int j = jt + threadIdx.x;
            if (j < a.max_chunks) {
                float best = sh_sigma[0][threadIdx.x];
                for (int g2 = 1; g2 < G; ++g2) best = fmaxf(best, sh_sigma[g2][threadIdx.x]);
                if (part > 0) best = fmaxf(best, sh_best[it][threadIdx.x]);
                if (part + 1 < parts) {
                    sh_best[it][threadIdx.x] = best;
                } else {
                    // validity is the same for every head; recompute it for this slot
                    const bool v = slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, j) >= 0;
                    a.out_scores[(int64_t)p * a.max_chunks + j] = v ? best : -INFINITY;
                }
            }
        }
        __syncthreads();
    }
    }
}

template <int MT, bool WIDE, int ROPE, bool PAGED>
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
    switch (a.ge.G) {
    case 1: hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 1, WIDE, ROPE, PAGED>), grid, dim3(64), 0, st, a, iters, rope); break;
    case 2: hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 2, WIDE, ROPE, PAGED>), grid, dim3(128), 0, st, a, iters, rope); break;
    case 4: hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 4, WIDE, ROPE, PAGED>), grid, dim3(256), 0, st, a, iters, rope); break;
    default:
        // 8 heads with 64-query blocks and no RoPE: 8 waves of ~160 registers fit a CU once only;
        // two passes of 4 waves fit three times
        if constexpr (MT == 4 && ROPE == 0)
            hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 4, WIDE, ROPE, PAGED, 2>), grid, dim3(256), 0, st, a, iters, rope);
        else
            hipLaunchKernelGGL((prune_prefill_kernel<MT, NT, 8, WIDE, ROPE, PAGED>), grid, dim3(512), 0, st, a, iters, rope);
        break;
    }
}

// 32-bit element offsets (one VGPR per address, full-rate 24-bit multiply) when every row of a
// (batch, head) slab of Q and K lies within 2^31 elements of its base and positions and strides are
// below 2^24; 64-bit offsets otherwise.
template <int MT>
static void launch_prefill(const PruneArgs &a, int P, int64_t max_seq_len, const RopeView *rope, int style,
                           hipStream_t st)
{
    const int64_t lim = (int64_t)1 << 31;
    const int64_t lim24 = (int64_t)1 << 24;         // narrow offsets are formed by a 24-bit multiply
    const bool wide = max_seq_len * a.k_st + kD >= lim || (int64_t)a.ge.b_q * a.q_st + kD >= lim ||
                      a.k_st < 0 || a.q_st < 0 || max_seq_len >= lim24 || a.k_st >= lim24 || a.q_st >= lim24;
    const RopeView none{nullptr, nullptr, 0};
    if (a.paged.block_table) {
        if (rope && style == 2) launch_prefill_w<MT, true, 2, true>(a, P, *rope, st);
        else if (rope) launch_prefill_w<MT, true, 1, true>(a, P, *rope, st);
        else launch_prefill_w<MT, true, 0, true>(a, P, none, st);
    } else if (rope && style == 2) {
        if (wide) launch_prefill_w<MT, true, 2, false>(a, P, *rope, st);
        else launch_prefill_w<MT, false, 2, false>(a, P, *rope, st);
    } else if (rope) {
        if (wide) launch_prefill_w<MT, true, 1, false>(a, P, *rope, st);
        else launch_prefill_w<MT, false, 1, false>(a, P, *rope, st);
    } else {
        if (wide) launch_prefill_w<MT, true, 0, false>(a, P, none, st);
        else launch_prefill_w<MT, false, 0, false>(a, P, none, st);
    }
}

// U chunks per 16-lane group.  What counts is the number of row loads in flight per SIMD, waves x
// 4 groups x U x G, and how finely the work is cut: U = 1 (64 registers, 8 waves per SIMD) is best
// for every later stage, for small problems, for E4M3 rows and for pages; U = 3 (127 registers, 4
// waves, half as many loads again in flight) wins on the large first stage over contiguous bf16 rows
// (cfg3: 278 us against 283 us with U = 1 and 294 us with U = 2, whose 97 registers miss the fifth
// wave by one).
template <int G, int U>
static void launch_decode_u(const PruneArgs &a, int P, bool fp8, hipStream_t st)
{
    dim3 grid((a.max_chunks + 16 * U - 1) / (16 * U), P);
    KernelTimer timer(stage_name(kNamePruneDecode, a.parent_starts == nullptr, a.chunk), st);
    if constexpr (U == 1) {
        if (fp8 && a.bank.page_table != nullptr)
            hipLaunchKernelGGL((prune_decode_kernel<G, U, 1, true>), grid, dim3(256), 0, st, a);
        else if (fp8 && a.paged.block_table != nullptr)
            hipLaunchKernelGGL((prune_decode_kernel<G, U, 2, true>), grid, dim3(256), 0, st, a);
        else if (fp8)
            hipLaunchKernelGGL((prune_decode_kernel<G, U, 0, true>), grid, dim3(256), 0, st, a);
        else if (a.paged.block_table != nullptr)
            hipLaunchKernelGGL((prune_decode_kernel<G, U, 2, false>), grid, dim3(256), 0, st, a);
        else if (a.bank.page_table != nullptr)
            hipLaunchKernelGGL((prune_decode_kernel<G, U, 1, false>), grid, dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL((prune_decode_kernel<G, U, 0, false>), grid, dim3(256), 0, st, a);
    } else {
        hipLaunchKernelGGL((prune_decode_kernel<G, U, 0, false>), grid, dim3(256), 0, st, a);
    }
}

template <int G>
static void launch_decode(const PruneArgs &a, int P, bool fp8, hipStream_t st)
{
    const bool plain = !fp8 && a.paged.block_table == nullptr && a.bank.page_table == nullptr;
    if (plain && a.parent_starts == nullptr && a.chunk >= 128 && (int64_t)P * a.max_chunks >= 65536)
        launch_decode_u<G, 3>(a, P, fp8, st);
    else
        launch_decode_u<G, 1>(a, P, fp8, st);
}

int32_t launch_prune_stage_rope(const PruneArgs &a, const RopeView &rope, int style, int P, bool fp8, hipStream_t st);

int32_t launch_prune_stage(const ihip_shape &s, const ihip_tensor &q, const ihip_tensor &k,
                           const int32_t *parent_starts, int n_parent, int parent_chunk, int chunk,
                           int max_chunks, float *out_scores, int32_t *out_rep, const BankView *bank,
                           const ihip_rope *rope, hipStream_t st, const KvFormat *fmt)
{
    PruneArgs a;
    const bool fp8 = fmt && fmt->fp8;
    a.k_scale = fp8 ? fmt->k_scale : 1.0f;
    a.paged = (fmt && fmt->paged.block_table) ? fmt->paged : PagedView{nullptr, 0, 0};
    if (a.paged.block_table && bank)
        return fail(IHIP_ERR_UNSUPPORTED, "prune_stage: paged K and the host tier exclude each other");
    a.bank = bank ? *bank : BankView{};
    a.ge = make_geometry(s);
    a.q = (const uint16_t *)q.ptr; a.q_sb = q.stride_b; a.q_sh = q.stride_h; a.q_st = q.stride_t;
    a.k = (const uint16_t *)k.ptr; a.k_sb = k.stride_b; a.k_sh = k.stride_h; a.k_st = k.stride_t;
    if (fp8) { a.k_sb /= 2; a.k_sh /= 2; a.k_st /= 2; }      // byte strides (even) in 2-byte units
    a.parent_starts = parent_starts;
    a.n_parent = n_parent;
    a.ratio_log2 = parent_starts ? __builtin_ctz(parent_chunk / chunk) : 0;
    a.chunk = chunk;
    a.max_chunks = max_chunks;
    a.out_scores = out_scores;
    a.out_rep = out_rep;
    const int P = s.B * s.Hkv * (s.Tq / s.b_q);
    if (max_chunks == 0 || P == 0) return IHIP_OK;
    if (bank && s.b_q != 1) return fail(IHIP_ERR_UNSUPPORTED, "prune_stage: the host tier serves decode only");
    if (fp8 && s.b_q != 1)
        return fail(IHIP_ERR_UNSUPPORTED, "prune_stage: FP8 keys are built for decode only");
    if (bank && (bank->row_units == kD) == fp8)
        return fail(IHIP_ERR_INVALID_ARG, "prune_stage: the host tier holds %s rows", fp8 ? "bf16" : "E4M3");
    RopeView rope_view{nullptr, nullptr, 0};
    int rope_style = 0;
    if (rope && rope->prune_style != IHIP_ROPE_NONE) {
        const int style = rope->prune_style;
        if (style != IHIP_ROPE_RELATIVE && style != IHIP_ROPE_CHUNK_INDEXED)
            return fail(IHIP_ERR_INVALID_ARG, "prune_stage: rope prune_style = %d", style);
        if (!rope->cos || !rope->sin) return fail(IHIP_ERR_INVALID_ARG, "prune_stage: rope tables are NULL");
        // largest table row the kernel may read: n_stream + 1, or the query's position (chunk-indexed)
        const int64_t need = style == IHIP_ROPE_RELATIVE ? (int64_t)s.n_stream + 2 : (int64_t)max_chunks + s.n_stream;
        if (rope->n_pos < need)
            return fail(IHIP_ERR_INVALID_ARG, "prune_stage: rope table has %d positions, %lld needed", rope->n_pos,
                        (long long)need);
        rope_view = RopeView{rope->cos, rope->sin, rope->n_pos};
        rope_style = style;
        if (s.b_q == 1) return launch_prune_stage_rope(a, rope_view, style, P, fp8, st);
    }
    const RopeView *rv = rope_view.cos ? &rope_view : nullptr;
    if (s.b_q == 1) {
        switch (a.ge.G) {
        case 1: launch_decode<1>(a, P, fp8, st); break;
        case 2: launch_decode<2>(a, P, fp8, st); break;
        case 4: launch_decode<4>(a, P, fp8, st); break;
        case 8: launch_decode<8>(a, P, fp8, st); break;
        default: return fail(IHIP_ERR_UNSUPPORTED, "Hq/Hkv = %d not in {1,2,4,8}", a.ge.G);
        }
        return check_launch("prune_stage (decode)");
    }
    switch (s.b_q) {
    case 16: launch_prefill<1>(a, P, s.max_seq_len, rv, rope_style, st); break;
    case 32: launch_prefill<2>(a, P, s.max_seq_len, rv, rope_style, st); break;
    case 64: launch_prefill<4>(a, P, s.max_seq_len, rv, rope_style, st); break;
    default: return fail(IHIP_ERR_UNSUPPORTED, "prune_stage: b_q = %d not in {1, 16, 32, 64}", s.b_q);
    }
    return check_launch("prune_stage (prefill)");
}

}  // namespace ihip
