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
#include "prune_prefill.h"
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

// 32-bit element offsets (one VGPR per address, full-rate 24-bit multiply) when every row of a
// (batch, head) slab of Q and K lies within 2^31 elements of its base and positions and strides are
// below 2^24; 64-bit offsets otherwise.
template <int MT>
static void launch_prefill(const PruneArgs &a, int P, int64_t max_seq_len, const RopeView *rope, int style,
                           hipStream_t st)
{
    const int64_t lim = (int64_t)1 << 31;
    const int64_t lim24 = (int64_t)1 << 24;         // narrow offsets are formed by a 24-bit multiply
    // (row x byte stride, as an unsigned 32-bit byte offset from a scalar base)
    const bool wide = max_seq_len * a.k_st + kD >= lim || (int64_t)a.ge.b_q * a.q_st + kD >= lim ||
                      a.k_st < 0 || a.q_st < 0 || max_seq_len >= lim24 || a.k_st * 2 >= lim24 || a.q_st * 2 >= lim24;
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
void launch_prune_prefill_fp8(const PruneArgs &a, int P, int b_q, const RopeView *rope, int style, hipStream_t st);

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
    if (s.b_q != 16 && s.b_q != 32 && s.b_q != 64)
        return fail(IHIP_ERR_UNSUPPORTED, "prune_stage: b_q = %d not in {1, 16, 32, 64}", s.b_q);
    if (fp8) {
        launch_prune_prefill_fp8(a, P, s.b_q, rv, rope_style, st);
        return check_launch("prune_stage (prefill, E4M3 keys)");
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
