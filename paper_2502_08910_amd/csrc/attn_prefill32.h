// Block-sparse chunked-prefill attention on v_mfma_f32_32x32x16_bf16.
//
// One workgroup per problem (sequence, KV head, query block); one wave per
// (query head of the group, 32 queries of the block), i.e. G * b_q/32 waves
// (8 for Llama-shaped GQA with b_q = 64).  The gathered K/V tile (32 key
// slots) is staged in LDS once and shared by all waves.
//
// "Transposed" scheme:  S^T = K Q^T,  O^T = V^T P^T.
// Layouts: A/B lane l holds 8 consecutive k (group half = l/32) of row/column
// n = l%32; C lane l holds column n, element r = row 8*(r/4) + 4*half + r%4.
// A lane's 16 S^T values are keys {8*(r/4) + 4*half + r%4}; taken 8 at a time
// (r < 8: keys 0..15, r >= 8: keys 16..31) they are, rounded to bf16, the B
// operand of the second product without any data movement: element i of k-step
// kk stands for key 16*kk + 8*(i/4) + 4*half + i%4, and the A operand (V^T) is
// read to match.
//
// On this chip vector and matrix instructions of the waves of a SIMD mostly
// take turns rather than overlap, so the design goal is few vector
// instructions per tile besides the softmax itself:
//  * K and V rows go from global memory straight into LDS (global_load_lds,
//    16 bytes per lane: 16 lanes fetch one 256-byte row, 4 rows per
//    instruction, landing at base + lane*16): no staging registers, no LDS
//    stores, and 16 load instructions per tile for the whole workgroup.
//  * V stays row-major ([key][dim]) in LDS and is transposed by the read
//    (ds_read_b64_tr_b16): within 16 lanes, lane i supplies the address of 4
//    elements and lane L receives element L%4 of the addresses of lanes
//    L/4 + 4j, j = 0..3.  With lane i pointing at key (i/4), dims 4*(i%4)..+3,
//    lane L gets dim L of four keys.
//  * The LDS destination of a direct load is fixed, so bank swizzles are
//    applied on the source side: 16-byte chunk c of a K row sits in slot
//    c ^ (key%16) (conflict-free 16-byte column reads), of a V row in slot
//    c ^ 4*(key%4) (the four keys of a transposing read hit different banks).
//  * The position of every key slot is computed once into LDS, so the steady
//    state has no dependent global loads.  Empty slots fetch row 0 (finite
//    data) and are masked in the scores.
// Three LDS stages: the rows of tile t+2 are requested at the start of period
// t and must have landed at the barrier that ends it.  K(u) is read in period
// u-1 (and before the loop for u = 0), V(u) in period u, so the stage of tile
// t-1 is free when period t begins and takes tile t+2.  The loop is unrolled
// by the three stages.  (A fourth stage, with requests a period earlier, made
// no difference in time -- the other waves of the CU cover a period -- and its
// 16 KB decide how many workgroups of four waves share a CU: with 5,280 key
// slots two instead of one, 484 against 604 us on the shape measured.)
//
// ROPE (streaming-style dynamic RoPE, Sec. 4 "Dynamic RoPE for OOL
// generalization"): the queries are rotated once, to the id of their last key.
// A K tile is rotated in place in LDS, each thread one 16-byte piece, in the
// period between its landing and its first read, which takes a fourth stage:
// tile t+3 is requested at the start of period t and must have landed at its
// end, K(t+2) is rotated during it (with table pieces fetched a period
// earlier) and read in period t+1.  Rotated operands are rounded to bf16.
//
// KV8 (K and V rows are 128 bytes of E4M3): the direct loads bring the raw rows (16 bytes per
// lane: 8 lanes a row, 8 rows an instruction, 8 instructions a tile) into a ring of three raw
// stages; the tile is widened to bf16 (exact) into one of three bf16 stages, every thread 8 bytes
// of K and 8 of V, in the period the RoPE variant uses for its rotation (and rotated on the way
// with ROPE), in the swizzled layout the reads below expect.  The raw ring puts requests a period
// further ahead than ROPE does: tile t+4 is requested at the start of period t, tile t+3 must have
// landed at its end, tile t+2 is widened during it, K(t+1) and V(t) are read.  The K scale is folded into the softmax scale on the host,
// the V scale into the final normalisation.
#pragma once

#include "attn_prefill_args.h"
#include <type_traits>

namespace ihip {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr float kPfMaxSum = 1024.0f;                // row sum of a tile above which the softmax reference moves

// NQ = b_q / 32 query tiles, G query heads per workgroup: NQ*G waves.  A group of more heads than
// that (8 heads with two query tiles would be 16 waves, whose registers spill) is spread over
// G_total/G workgroups placed 8 apart in launch order, i.e. on the same XCD, so that the second
// reads the K and V rows from that XCD's L2.
// WIDE: 64-bit row offsets; otherwise every
// row of a (sequence, KV head) slab of K and V lies within 2^31 elements of its base and positions
// and strides are below 2^24, so an offset is one full-rate 24-bit multiply.
// PAGED: K and V are page pools read through the sequence's row of the block table; the page id of
// every slot is looked up once, next to its position, and kept in LDS as well.
template <int NQ, int G, bool WIDE, bool ROPE, bool PAGED, bool KV8 = false>
__global__ __launch_bounds__(64 * NQ * G, NQ * G < 8 || ((ROPE || KV8) && NQ * G == 8) ? 2 : NQ * G == 8 ? 3 : 4) void attn_prefill32_kernel(const AttnPrefillArgs a)
{
    static_assert(!PAGED || WIDE, "paged pools are addressed with 64-bit offsets");
    static_assert(!KV8 || WIDE, "E4M3 rows are addressed with 64-bit offsets");
    constexpr int kPfStages = KV8 ? kPfStagesFp8 : ROPE ? kPfStagesRope : kPfStagesPlain;
    constexpr bool kTouch = ROPE || KV8;             // a tile is worked on in LDS between landing and first read
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *raw0 = smem + kPfStages * kPfStageEl;                          // KV8: the raw stages
    int *sPos = reinterpret_cast<int *>(raw0 + (KV8 ? kPfRawStages * kPfTileEl : 0));   // one int per key slot
    // the most slots this geometry can have
    const int slots_cap = (a.ge.n_sink + a.n_blocks * a.block + a.ge.n_stream + kPfTile - 1) / kPfTile * kPfTile;
    int *sPage = sPos + slots_cap;                                           // PAGED: one page id per key slot
    // one flag per tile, behind the per-slot arrays
    uint8_t *sMasked = reinterpret_cast<uint8_t *>(sPos + (PAGED ? 2 : 1) * slots_cap);

    int p = blockIdx.x, head_part = 0;
    if (a.ge.G != G) {                               // blocks of 8 problems x (G_total/G) parts
        const int parts = a.ge.G / G;
        const int r = blockIdx.x % (8 * parts);
        p = blockIdx.x / (8 * parts) * 8 + (r & 7);
        head_part = r >> 3;
        if (p >= a.ge.B * a.ge.Hkv * a.ge.Mq) return;
    }
    const Problem pr = problem_of(a.ge, p);
    constexpr int NW = NQ * G;
    constexpr int nthreads = 64 * NW;
    constexpr int b_q = 32 * NQ;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int hh = wave % G, qt = wave / G;          // this wave's head and query tile
    const int n = lane & 31, half = lane >> 5;
    const int h = pr.g * a.ge.G + head_part * G + hh;
    const int q0 = pr.m * b_q + qt * 32;             // first query row of this wave
    const int qpos0 = pr.E - b_q;                    // absolute position of the block's first query
    const int qpos = qpos0 + qt * 32 + n;            // ... of this lane's query

    const int n_sink_eff = min(a.ge.n_sink, pr.E);
    const int w0 = max(pr.hi, a.ge.n_sink);
    const int total = n_sink_eff + (a.n_blocks << a.block_log2) + max(0, pr.E - w0);
    const int n_tiles = (total + kPfTile - 1) / kPfTile;     // host guarantees n_tiles*32 <= kPf32MaxSlots

    // a tile needs masking if it has an empty slot or a key at or after the block's first query
    for (int slot = tid; slot < n_tiles * kPfTile; slot += nthreads) {
        const int pos = slot < total ? pf_slot_to_pos(a, pr, p, slot, n_sink_eff, w0) : -1;
        sPos[slot] = pos;
        if constexpr (PAGED)        // an empty slot fetches row 0 of the sequence
            sPage[slot] = a.paged.block_table[(int64_t)pr.b * a.paged.table_stride + (max(pos, 0) >> a.paged.page_log2)];
        const unsigned long long m = __ballot(pos < 0 || pos >= qpos0);      // a tile is half a wave
        if ((lane & 31) == 0) sMasked[slot >> 5] = (uint32_t)(m >> (lane & 32)) != 0u;
    }

    StreamIds ids{n_sink_eff, a.n_blocks << a.block_log2, 0, w0};
    if constexpr (ROPE) {
        __shared__ int sh_tokens;
        ids.block_tokens = pf_block_tokens(a, pr, p, nthreads, &sh_tokens);
    }

    bf16x8 qb[8];
    {
        const uint16_t *qp = a.q + pr.b * a.q_sb + (int64_t)h * a.q_sh + (int64_t)(q0 + n) * a.q_st + half * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            qb[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
            if constexpr (ROPE) {       // dims 16*ks + 8*half .. +7 = pairs 8*ks + 4*half .. +3
                const int64_t at = (int64_t)ids.query(a.ge.n_sink, qpos) * (kD / 2) + ks * 8 + half * 4;
                qb[ks] = __builtin_bit_cast(
                    bf16x8, rotate_bf16x8(__builtin_bit_cast(uint4, qb[ks]), a.rope_cos + at, a.rope_sin + at));
            }
        }
    }
    const uint16_t *kb = PAGED ? a.k + pr.g * a.k_sh : a.k + pr.b * a.k_sb + pr.g * a.k_sh;
    const uint16_t *vb = PAGED ? a.v + pr.g * a.v_sh : a.v + pr.b * a.v_sb + pr.g * a.v_sh;
    const int page_mask = PAGED ? (1 << a.paged.page_log2) - 1 : 0;

    f32x16 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m_run = kNegBigPf, l_run = 0.f;

    // Loads of a tile: 8 four-row instructions for K and 8 for V (KV8: 4 eight-row instructions
    // each), dealt to the NW waves.
    constexpr int kLoadsPerTile = KV8 ? 8 : 16;
    constexpr int kLoadsPerWave = kLoadsPerTile / NW;
    static_assert(kLoadsPerWave * NW == kLoadsPerTile, "wave count must divide the loads of a tile");
    // The loads are written as assembly: a compiler-visible LDS-bound load makes the compiler
    // drain the vector-memory counter before the next LDS read it cannot tell apart from the
    // destination, which would undo the prefetch distance.  landed() below is the only wait.
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    // the stage of a tile (tile % kPfStages) is a compile-time constant in the unrolled loop below,
    // so LDS addresses are per-lane constants plus immediates
    auto stage_of = [&](int st) { return smem + (st % kPfStages) * kPfStageEl; };
    auto raw_of = [&](int st) { return raw0 + (st % kPfRawStages) * kPfTileEl; };
    // key positions of this lane's rows in the loads of a tile (read a period ahead of the request)
    struct Rows { int pos[kLoadsPerWave]; int page[PAGED ? kLoadsPerWave : 1]; };
    auto rows_of = [&](int tile) {
        Rows r;
#pragma unroll
        for (int i = 0; i < kLoadsPerWave; ++i) {
            const int j = wave_s + i * NW;
            const int key = KV8 ? 8 * (j & 3) + (lane >> 3) : 4 * (j & 7) + (lane >> 4);
            r.pos[i] = tile < n_tiles ? sPos[tile * kPfTile + key] : 0;
            if constexpr (PAGED) r.page[i] = tile < n_tiles ? sPage[tile * kPfTile + key] : 0;
        }
        return r;
    };
    auto request = [&](int tile, int st, const Rows &rows) {
        if (tile >= n_tiles) return;
        if constexpr (KV8) {
            // instruction j of the tile: j < 4 fetches K rows 8j..8j+7, j >= 4 V rows 8(j-4)..; lane l
            // brings bytes 16*(l%8)..+15 of row l/8, to raw row-major order
            uint16_t *stage = raw_of(st);
#pragma unroll
            for (int i = 0; i < kLoadsPerWave; ++i) {
                const int j = wave_s + i * NW;
                const bool is_v = j >= 4;
                const int pos = max(rows.pos[i], 0);
                const uint16_t *src;
                if (PAGED)
                    src = is_v ? vb + (int64_t)rows.page[PAGED ? i : 0] * a.v_sb + (int64_t)(pos & page_mask) * a.v_st
                               : kb + (int64_t)rows.page[PAGED ? i : 0] * a.k_sb + (int64_t)(pos & page_mask) * a.k_st;
                else
                    src = is_v ? vb + (int64_t)pos * a.v_st : kb + (int64_t)pos * a.k_st;
                src += (lane & 7) * 8;
                const uint32_t dst = __builtin_amdgcn_readfirstlane(
                    (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)(stage + j * 512));
                uint32_t m0_saved;       // M0 is put back: the compiler is not told that it changes
                asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\t"
                             "s_mov_b32 m0, %0"
                             : "=&s"(m0_saved)
                             : "s"(dst), "v"(src)
                             : "memory");
            }
            return;
        }
        uint16_t *stage = stage_of(st);
#pragma unroll
        for (int i = 0; i < kLoadsPerWave; ++i) {
            // instruction j of the tile: j < 8 fetches K rows 4j..4j+3, j >= 8 V rows 4(j-8)..
            const bool is_v = NW <= 8 ? i * NW >= 8 : wave_s >= 8;
            const int j = wave_s + i * NW;
            const int key = 4 * (j & 7) + (lane >> 4);
            const int pos = max(rows.pos[i], 0);
            const int slot = lane & 15;
            const int chunk = is_v ? slot ^ ((key & 3) << 2) : slot ^ (key & 15);
            const uint16_t *src;
            if (PAGED)
                src = (is_v ? vb + (int64_t)rows.page[PAGED ? i : 0] * a.v_sb + (int64_t)(pos & page_mask) * a.v_st
                            : kb + (int64_t)rows.page[PAGED ? i : 0] * a.k_sb + (int64_t)(pos & page_mask) * a.k_st) + chunk * 8;
            else if (WIDE) src = (is_v ? vb + (int64_t)pos * a.v_st : kb + (int64_t)pos * a.k_st) + chunk * 8;
            else src = (is_v ? vb : kb) + (__umul24((uint32_t)pos, (uint32_t)(is_v ? a.v_st : a.k_st)) + (uint32_t)(chunk * 8));
            const uint32_t dst = __builtin_amdgcn_readfirstlane(
                (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)(stage + j * 4 * kD));
            uint32_t m0_saved;           // M0 is put back: the compiler is not told that it changes
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\t"
                         "s_mov_b32 m0, %0"
                         : "=&s"(m0_saved)
                         : "s"(dst), "v"(src)
                         : "memory");
        }
    };

    // ROPE: the K part of a stage is 32 rows x 16 pieces of 16 bytes, dealt to the threads; slot s
    // of row r holds dims 8*(s ^ r%16)..  table_of fetches the table pieces of a tile's keys,
    // rotate_k turns the tile in place.
    // KV8: item (row r, piece c) is the row's dims 8c..8c+7, not yet swizzled.
    constexpr int kPieces = kTouch ? (kPfTile * 16 + nthreads - 1) / nthreads : 1;
    struct Table { float4 c[ROPE ? kPieces : 1], s[ROPE ? kPieces : 1]; };
    auto table_of = [&](int tile) {
        Table tb{};
        if constexpr (ROPE) {
#pragma unroll
            for (int i = 0; i < kPieces; ++i) {
                const int item = tid + i * nthreads, r = (item >> 4) & (kPfTile - 1), sl = item & 15;
                const int slot = tile * kPfTile + r;
                const int id = tile < n_tiles && slot < total ? ids.key(slot) : 0;
                const int64_t at = (int64_t)id * (kD / 2) + ((KV8 ? sl : sl ^ (r & 15)) << 2);
                tb.c[i] = *reinterpret_cast<const float4 *>(a.rope_cos + at);
                tb.s[i] = *reinterpret_cast<const float4 *>(a.rope_sin + at);
            }
        }
        return tb;
    };
    auto rotate_k = [&](int tile, int st, const Table &tb) {
        if (tile >= n_tiles) return;
        uint16_t *stage = stage_of(st);
        if constexpr (KV8) {
            const uint16_t *raw = raw_of(st);
#pragma unroll
            for (int i = 0; i < kPieces; ++i) {
                const int item = tid + i * nthreads;
                if (kPfTile * 16 % nthreads != 0 && item >= kPfTile * 16) break;
                const int r = item >> 4, c = item & 15;
                const uint2 rk = *reinterpret_cast<const uint2 *>(raw + item * 4);
                uint4 wk;
                if constexpr (ROPE) wk = rotate_fp8x8(rk, tb.c[ROPE ? i : 0], tb.s[ROPE ? i : 0]);
                else wk = fp8x8_to_bf16x8(rk);
                const uint4 wv = fp8x8_to_bf16x8(*reinterpret_cast<const uint2 *>(raw + kPfTileEl / 2 + item * 4));
                *reinterpret_cast<uint4 *>(stage + r * kD + ((c ^ (r & 15)) << 3)) = wk;
                *reinterpret_cast<uint4 *>(stage + kPfTileEl + r * kD + ((c ^ ((r & 3) << 2)) << 3)) = wv;
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int item = tid + i * nthreads;
            if (kPfTile * 16 % nthreads != 0 && item >= kPfTile * 16) break;
            uint4 *piece = reinterpret_cast<uint4 *>(stage + (item >> 4) * kD + (item & 15) * 8);
            *piece = rotate_bf16x8(*piece, tb.c[i], tb.s[i]);
        }
    };

    // first product of a tile: S^T = K Q^T for this wave's 32 queries
    auto scores = [&](int st) -> f32x16 {
        const uint16_t *cK = stage_of(st) + n * kD;
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(&cK[((ks * 2 + half) ^ (n & 15)) * 8]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[ks], s, 0, 0, 0);
        }
        return s;
    };
    // softmax update of a tile's scores: P (bf16) for the second product, running sum, rescale
    auto softmax = [&](int tile, bool masked, f32x16 &s, bf16x8 (&pb)[2]) {
        if (masked) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kp = sPos[tile * kPfTile + 8 * (r >> 2) + 4 * half + (r & 3)];
                if (kp < 0 || kp > qpos) s[r] = -INFINITY;
            }
        }
        // Reference point m_run of the exponentials, in scaled (log2) units.  It only has to bound
        // the scores from above loosely, so the common path takes the exponentials against the
        // current one without looking for the tile maximum, and checks the row sums: a sum above
        // kPfMaxSum (or an overflow) in any lane sends the whole wave to the exact path, which
        // moves the reference to the maximum and rescales the accumulators (64 multiplies per
        // lane).  p <= kPfMaxSum stays far inside the fp32 and bf16 ranges and out = o / l is
        // unchanged.  The two lanes of a query (key halves) always share one reference.
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float pw = __builtin_amdgcn_exp2f(fmaf(s[r], a.scale_log2e, -m_run));   // exp2(-inf) = 0
            ps += pw;
            pb[r >> 3][r & 7] = (__bf16)pw;
        }
        if (__any(!(ps <= kPfMaxSum))) {
            float mx = s[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float mn = fmaxf(m_run, mx * a.scale_log2e);
            const float corr = __builtin_amdgcn_exp2f(m_run - mn);
            m_run = mn;
            ps = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pw = __builtin_amdgcn_exp2f(fmaf(s[r], a.scale_log2e, -mn));
                ps += pw;
                pb[r >> 3][r & 7] = (__bf16)pw;
            }
            l_run *= corr;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) o[dt] *= corr;
        }
        l_run += ps;                                              // partial over this lane's keys
    };
    // second product of a tile: O^T += V^T P^T.  Address of this lane in a transposing read:
    // key 4*half + i/4 (+16*kk, +8 for the upper four keys), dims 32*dt + 16*(n/16) + 4*(i%4)..+3,
    // i = lane%16; the lane then receives dim 32*dt + n of keys 16*kk (+8) + 4*half + 0..3.
    int voff[4];
    {
        const int i = lane & 15, key = 4 * half + (i >> 2);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const int chunk = dt * 4 + ((n >> 4) << 1) + ((i & 3) >> 1);
            voff[dt] = kPfTileEl + key * kD + ((chunk ^ ((key & 3) << 2)) << 3) + ((i & 1) << 2);
        }
    }
    auto v_operand = [&](const uint16_t *cV, int dt, int kk) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(cV + voff[dt] + (16 * kk) * kD));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(cV + voff[dt] + (16 * kk + 8) * kD));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto accumulate = [&](int st, const bf16x8 (&pb)[2]) {
        const uint16_t *cV = stage_of(st);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(cV, dt, kk), pb[kk], o[dt], 0, 0, 0);
    };
    // Tile t+D is requested at the start of period t (D = kPfStages-1); tile t+2 (ROPE: t+3) must
    // have landed at the barrier that ends it, so one newer request may still be on its way then
    // (near the end of the key list fewer are: everything is waited for).
    constexpr int D = KV8 ? 4 : kPfStages - 1;
    constexpr int kInFlight = kTouch ? D - 3 : D - 2;
    auto landed = [&](bool all) {
        if (all || kInFlight == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kInFlight * kLoadsPerWave) : "memory");
    };

    __syncthreads();                        // sPos complete
    constexpr int kPrologue = KV8 ? kPfRawStages : D;       // the raw ring holds three tiles
#pragma unroll
    for (int t = 0; t < kPrologue; ++t) request(t, t, rows_of(t));
    Rows rows = rows_of(D);
    landed(true);                           // tiles 0 and 1 (and the rest of the prologue's requests)
    __syncthreads();
    Table table{};                          // ROPE: table pieces of the tile that the next period rotates
    if constexpr (kTouch) {
        rotate_k(0, 0, table_of(0));
        rotate_k(1, 1, table_of(1));
        table = table_of(2);
        __syncthreads();
        if constexpr (KV8) request(3, 3, rows_of(3));       // into the raw stage tile 0 has left
    }
    f32x16 s_nxt = scores(0);
    bf16x8 pb[2];
    softmax(0, sMasked[0] != 0, s_nxt, pb);
    int masked_nxt = n_tiles > 1 ? sMasked[1] : 0;      // read a period ahead, like the row positions
    // one tile period; ST = tile % kPfStages
    auto period = [&](auto st_c, int tile) {
        constexpr int ST = decltype(st_c)::value;
        // the table loads come before the request: the wait the compiler puts before their use then
        // lets exactly the newer request stay in flight
        Table table_nxt{};
        if constexpr (ROPE) table_nxt = table_of(tile + 3);
        request(tile + D, ST + D, rows);
        if (tile + 1 < n_tiles) s_nxt = scores(ST + 1);
        accumulate(ST, pb);
        if (tile + 1 < n_tiles) softmax(tile + 1, masked_nxt != 0, s_nxt, pb);
        masked_nxt = tile + 2 < n_tiles ? sMasked[tile + 2] : 0;
        rows = rows_of(tile + D + 1);
        if constexpr (kTouch) {
            rotate_k(tile + 2, ST + 2, table);
            table = table_nxt;
        }
        landed(tile + D >= n_tiles);        // tile + 2 (ROPE, KV8: tile + 3)
        __syncthreads();
    };
    auto periods = [&](int tile, auto... st) {      // up to kPfStages periods, stopping at the last tile
        bool more = true;
        ((more = more && tile + decltype(st)::value < n_tiles && (period(st, tile + decltype(st)::value), true)), ...);
    };
    for (int tile = 0; tile < n_tiles; tile += kPfStages) {
        if constexpr (kPfStages == 3)
            periods(tile, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{},
                    std::integral_constant<int, 2>{});
        else if constexpr (kPfStages == 4)
            periods(tile, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{},
                    std::integral_constant<int, 2>{}, std::integral_constant<int, 3>{});
        else if constexpr (kPfStages == 5)
            periods(tile, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{},
                    std::integral_constant<int, 2>{}, std::integral_constant<int, 3>{}, std::integral_constant<int, 4>{});
        else
            periods(tile, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{},
                    std::integral_constant<int, 2>{}, std::integral_constant<int, 3>{}, std::integral_constant<int, 4>{},
                    std::integral_constant<int, 5>{});
    }

    float l = l_run;
    l += __shfl_xor(l, 32, 64);
    const float inv = KV8 ? a.v_scale / l : 1.0f / l;
    const int64_t row = ((int64_t)pr.b * a.ge.Hq + h) * a.ge.Tq + q0 + n;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            uint2 w;
            w.x = f32_to_bf16_bits(o[dt][r4 * 4 + 0] * inv) | (f32_to_bf16_bits(o[dt][r4 * 4 + 1] * inv) << 16);
            w.y = f32_to_bf16_bits(o[dt][r4 * 4 + 2] * inv) | (f32_to_bf16_bits(o[dt][r4 * 4 + 3] * inv) << 16);
            *reinterpret_cast<uint2 *>(a.out + row * kD + dt * 32 + r4 * 8 + half * 4) = w;
        }
    if (a.out_lse != nullptr && half == 0)
        a.out_lse[row] = (m_run + log2f(l)) * 0.69314718055994530942f;
}

}  // namespace ihip
