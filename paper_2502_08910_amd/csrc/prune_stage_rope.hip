// Decode pruning stage with dynamic RoPE (Sec. 4 "Dynamic RoPE for OOL
// generalization"; ApplyRopeQ / ApplyRopeK after Alg. 3).  Q and K are stored
// unrotated.  Same mapping as the plain decode kernel (16 lanes per K row, a
// 16-lane group walks the searches of all G query heads of U chunk slots); the
// rotations are folded into the query, using  R(a)q . R(b)k = R(a-b)q . k  for
// a table of true rotations (cos and sin of position x angle), so no K row is
// ever rotated and the rows read are exactly those of the plain kernel:
//
//  relative style:       the query sits at n_stream+1, a left-branch key at 0,
//                        a right-branch key (and the representative in the
//                        chunk score) at 1: two rotated copies of q per head,
//                        q_L = R(n_stream+1) q and q_R = R(n_stream) q.  Every
//                        row read is dotted with both, because a key that wins
//                        as the right branch is the left branch of the next
//                        iteration.
//  chunk-indexed style:  every key of chunk j (index in the stage's chunk
//                        list) sits at j, the query at
//                        min(its own position, n_chunk - 1 + n_stream): one
//                        rotated copy of q per chunk, R(qpos - j) q, and the
//                        carried-score search of the plain kernel.
// SRC 0: K through strides, 1: host tier (a resident block is read from its bank, the touch and
// miss bookkeeping is done by one lane per row read), 2: paged pool; KV8: rows are 128
// bytes of E4M3, the scores are multiplied by the K scale at the end (a positive factor: the
// searches do not depend on it).
#include "prune_args.h"
#include <type_traits>

namespace ihip {

// lane l16 of a 16-lane group holds dims 8*l16 .. 8*l16+7 = pairs 4*l16 .. 4*l16+3
__device__ inline void rotate8(const float (&x)[8], const RopeView &rope, int pos, int l16, float (&out)[8])
{
    const float4 c = *reinterpret_cast<const float4 *>(rope.cos + (int64_t)pos * (kD / 2) + l16 * 4);
    const float4 s = *reinterpret_cast<const float4 *>(rope.sin + (int64_t)pos * (kD / 2) + l16 * 4);
    const float cc[4] = {c.x, c.y, c.z, c.w}, ss[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = x[2 * i] * cc[i] - x[2 * i + 1] * ss[i];
        out[2 * i + 1] = x[2 * i] * ss[i] + x[2 * i + 1] * cc[i];
    }
}

template <int G, int U, int STYLE, int SRC, bool KV8>   // STYLE 1: relative, 2: chunk-indexed
__global__ __launch_bounds__(256) void prune_decode_rope_kernel(const PruneArgs a, const RopeView rope)
{
    using piece_t = typename std::conditional<KV8, uint2, uint4>::type;     // a lane's share of a row
    constexpr int kLaneOff = KV8 ? 4 : 8;                                   // in 2-byte units
    const int p = blockIdx.y;
    const Problem pr = problem_of(a.ge, p);
    const int l16 = threadIdx.x & 15;
    const int grp = threadIdx.x >> 4;
    const int j0 = (blockIdx.x * 16 + grp) * U;

    // chunk-indexed: the number of chunks this stage really has for this problem
    __shared__ int sh_n_chunk;
    int n_chunk = 0;
    if (STYLE == 2) n_chunk = stage_n_chunk(a, pr, p, 256, &sh_n_chunk);
    if (j0 >= a.max_chunks) return;

    float qf[G][8];
    {
        const uint16_t *qb = a.q + pr.b * a.q_sb + (int64_t)(pr.g * G) * a.q_sh +
                             (int64_t)(pr.m * a.ge.b_q) * a.q_st;
#pragma unroll
        for (int h = 0; h < G; ++h) unpack8(load_row16(qb, h * a.q_sh, l16), qf[h]);
    }
    const typename KeySource<SRC>::type src = KeySource<SRC>::make(a, pr);

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
    // group, and handed round by shuffles (all shuffles of a search level before its row loads), as
    // in the plain kernel.
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
    auto load_row = [&](int pos, int page) {
        if constexpr (SRC == 2)
            return *reinterpret_cast<const piece_t *>(src.row_in_page(page, pos) + l16 * kLaneOff);
        else
            return *reinterpret_cast<const piece_t *>(src.row(pos, l16 == 0) + l16 * kLaneOff);
    };

    int off[U][G];
    float score[U][G];       // what the chunk score takes from head h

    if (STYLE == 1) {
        float qL[G][8], qR[G][8];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            rotate8(qf[h], rope, a.ge.n_stream + 1, l16, qL[h]);
            rotate8(qf[h], rope, a.ge.n_stream, l16, qR[h]);
        }
        float sL[U][G];      // the current left key against q_L; score[][] holds it against q_R
        {
            // first key of the chunk and of its right half: common to all heads
            piece_t r0[U], r1[U];
            const int mid = a.chunk >> 1;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                r0[u] = piece_t{};
                r1[u] = piece_t{};
                const int pg0 = page_of(max(start[u], 0), u), pg1 = page_of(max(start[u], 0) + mid, u);
                if (valid[u]) r0[u] = load_row(start[u], pg0);
                if (mid >= 1 && mid < len[u]) r1[u] = load_row(start[u] + mid, pg1);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float l0 = row16_sum(dot8(r0[u], qL[h])), l0r = row16_sum(dot8(r0[u], qR[h]));
                    const float r1l = row16_sum(dot8(r1[u], qL[h])), r1r = row16_sum(dot8(r1[u], qR[h]));
                    const bool right = (mid >= 1 && mid < len[u]) && r1r > l0;   // strict: tie keeps left
                    off[u][h] = right ? mid : 0;
                    sL[u][h] = right ? r1l : l0;
                    score[u][h] = right ? r1r : l0r;
                }
            }
        }
        for (int half = a.chunk >> 2; half >= 1; half >>= 1) {
            piece_t r[U][G];
            bool ok[U][G];
            int page[U][G];
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
                    r[u][h] = piece_t{};
                    if (ok[u][h]) r[u][h] = load_row(start[u] + mid, page[u][h]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float tl = row16_sum(dot8(r[u][h], qL[h])), tr = row16_sum(dot8(r[u][h], qR[h]));
                    if (ok[u][h] && tr > sL[u][h]) {
                        off[u][h] += half;
                        sL[u][h] = tl;
                        score[u][h] = tr;
                    }
                }
            }
        }
    } else {
        const int qpos = min(pr.E - 1, n_chunk - 1 + a.ge.n_stream);
        float qr[U][G][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // empty slots rotate by 0: their scores are never written
            const int delta = valid[u] ? qpos - (j0 + u) : 0;
#pragma unroll
            for (int h = 0; h < G; ++h) rotate8(qf[h], rope, delta, l16, qr[u][h]);
        }
        {
            piece_t r0[U], r1[U];
            const int mid = a.chunk >> 1;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                r0[u] = piece_t{};
                r1[u] = piece_t{};
                const int pg0 = page_of(max(start[u], 0), u), pg1 = page_of(max(start[u], 0) + mid, u);
                if (valid[u]) r0[u] = load_row(start[u], pg0);
                if (mid >= 1 && mid < len[u]) r1[u] = load_row(start[u] + mid, pg1);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float s0 = row16_sum(dot8(r0[u], qr[u][h]));
                    const float s1 = row16_sum(dot8(r1[u], qr[u][h]));
                    const bool right = (mid >= 1 && mid < len[u]) && s1 > s0;
                    off[u][h] = right ? mid : 0;
                    score[u][h] = right ? s1 : s0;
                }
            }
        }
        for (int half = a.chunk >> 2; half >= 1; half >>= 1) {
            piece_t r[U][G];
            bool ok[U][G];
            int page[U][G];
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
                    r[u][h] = piece_t{};
                    if (ok[u][h]) r[u][h] = load_row(start[u] + mid, page[u][h]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float s = row16_sum(dot8(r[u][h], qr[u][h]));
                    if (ok[u][h] && s > score[u][h]) {
                        off[u][h] += half;
                        score[u][h] = s;
                    }
                }
            }
        }
    }

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int j = j0 + u;
        if (j >= a.max_chunks) break;
        float best = score[u][0];
#pragma unroll
        for (int h = 1; h < G; ++h) best = fmaxf(best, score[u][h]);
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

template <int G, int SRC, bool KV8, int U>
static void launch_rope_u(const PruneArgs &a, const RopeView &rope, int style, int P, hipStream_t st)
{
    dim3 grid((a.max_chunks + 16 * U - 1) / (16 * U), P);
    KernelTimer timer(stage_name(kNamePruneDecode, a.parent_starts == nullptr, a.chunk), st);
    if (style == 1) hipLaunchKernelGGL((prune_decode_rope_kernel<G, U, 1, SRC, KV8>), grid, dim3(256), 0, st, a, rope);
    else hipLaunchKernelGGL((prune_decode_rope_kernel<G, U, 2, SRC, KV8>), grid, dim3(256), 0, st, a, rope);
}

// U chunks per 16-lane group: one everywhere (most waves per SIMD, finest cut of the work) except on
// a large first stage over contiguous E4M3 rows, where three chunks per group put more of the short
// rows in flight (cfg3: 193 us against 207 us).
template <int G, int SRC, bool KV8>
static void launch_rope(const PruneArgs &a, const RopeView &rope, int style, int P, hipStream_t st)
{
    if constexpr (SRC == 0 && KV8) {
        if (a.parent_starts == nullptr && a.chunk >= 128 && (int64_t)P * a.max_chunks >= 65536) {
            launch_rope_u<G, SRC, KV8, 3>(a, rope, style, P, st);
            return;
        }
    }
    launch_rope_u<G, SRC, KV8, 1>(a, rope, style, P, st);
}

template <int G>
static void launch_rope_g(const PruneArgs &a, const RopeView &rope, int style, int P, bool fp8, hipStream_t st)
{
    const bool paged = a.paged.block_table != nullptr;
    if (a.bank.page_table != nullptr && fp8) launch_rope<G, 1, true>(a, rope, style, P, st);   // host tier
    else if (a.bank.page_table != nullptr) launch_rope<G, 1, false>(a, rope, style, P, st);
    else if (paged && fp8) launch_rope<G, 2, true>(a, rope, style, P, st);
    else if (paged) launch_rope<G, 2, false>(a, rope, style, P, st);
    else if (fp8) launch_rope<G, 0, true>(a, rope, style, P, st);
    else launch_rope<G, 0, false>(a, rope, style, P, st);
}

int32_t launch_prune_stage_rope(const PruneArgs &a, const RopeView &rope, int style, int P, bool fp8, hipStream_t st)
{
    switch (a.ge.G) {
    case 1: launch_rope_g<1>(a, rope, style, P, fp8, st); break;
    case 2: launch_rope_g<2>(a, rope, style, P, fp8, st); break;
    case 4: launch_rope_g<4>(a, rope, style, P, fp8, st); break;
    case 8: launch_rope_g<8>(a, rope, style, P, fp8, st); break;
    default: return fail(IHIP_ERR_UNSUPPORTED, "Hq/Hkv = %d not in {1,2,4,8}", a.ge.G);
    }
    return check_launch("prune_stage (decode, dynamic RoPE)");
}

}  // namespace ihip
