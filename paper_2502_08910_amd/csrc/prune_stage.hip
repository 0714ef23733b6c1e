// Pruning-stage scoring: representative search (Alg. 3) + chunk score (Alg. 2).
//
// Decode kernel (b_q == 1).  HBM-latency/bandwidth bound gather: each chunk
// needs 1 + log2(l_c) dependent 256-byte row reads per query head.  Mapping:
// 16 lanes share one K row (16 B per lane -> one fully coalesced 256 B read),
// so a wave works on 4 chunk slots at a time and a 16-lane group walks the
// searches of all G query heads of its KV head together (the first two rows
// of a chunk are common to the heads, the rest are G independent loads in
// flight).  U slots per group are interleaved to put more loads in flight.
#include "common.h"

namespace ihip {

struct PruneArgs {
    Geometry ge;
    const uint16_t *q; int64_t q_sb, q_sh, q_st;
    const uint16_t *k; int64_t k_sb, k_sh, k_st;
    const int32_t *parent_starts;
    int n_parent, ratio_log2, chunk, max_chunks;
    float *out_scores;
    int32_t *out_rep;
};

template <int G, int U>
__global__ __launch_bounds__(256) void prune_decode_kernel(const PruneArgs a)
{
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
    const uint16_t *kb = a.k + pr.b * a.k_sb + pr.g * a.k_sh;

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

    int off[U][G];
    float sigma[U][G];

    // first key of the chunk, and the first key of its right half: common to all heads
    {
        uint4 r0[U], r1[U];
        const int mid = a.chunk >> 1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            r0[u] = make_uint4(0, 0, 0, 0);
            r1[u] = make_uint4(0, 0, 0, 0);
            if (valid[u]) r0[u] = load_row16(kb, (int64_t)start[u] * a.k_st, l16);
            if (mid >= 1 && mid < len[u]) r1[u] = load_row16(kb, (int64_t)(start[u] + mid) * a.k_st, l16);
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
        uint4 r[U][G];
        bool ok[U][G];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const int mid = off[u][h] + half;
                ok[u][h] = mid < len[u];
                r[u][h] = make_uint4(0, 0, 0, 0);
                if (ok[u][h]) r[u][h] = load_row16(kb, (int64_t)(start[u] + mid) * a.k_st, l16);
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

template <int G>
static void launch_decode(const PruneArgs &a, int P, hipStream_t st)
{
    constexpr int U = 2;
    dim3 grid((a.max_chunks + 16 * U - 1) / (16 * U), P);
    KernelTimer timer(stage_name(kNamePruneDecode, a.parent_starts == nullptr, a.chunk), st);
    hipLaunchKernelGGL((prune_decode_kernel<G, U>), grid, dim3(256), 0, st, a);
}

int32_t launch_prune_stage(const ihip_shape &s, const ihip_tensor &q, const ihip_tensor &k,
                           const int32_t *parent_starts, int n_parent, int parent_chunk, int chunk,
                           int max_chunks, float *out_scores, int32_t *out_rep, hipStream_t st)
{
    PruneArgs a;
    a.ge = make_geometry(s);
    a.q = (const uint16_t *)q.ptr; a.q_sb = q.stride_b; a.q_sh = q.stride_h; a.q_st = q.stride_t;
    a.k = (const uint16_t *)k.ptr; a.k_sb = k.stride_b; a.k_sh = k.stride_h; a.k_st = k.stride_t;
    a.parent_starts = parent_starts;
    a.n_parent = n_parent;
    a.ratio_log2 = parent_starts ? __builtin_ctz(parent_chunk / chunk) : 0;
    a.chunk = chunk;
    a.max_chunks = max_chunks;
    a.out_scores = out_scores;
    a.out_rep = out_rep;
    const int P = s.B * s.Hkv * (s.Tq / s.b_q);
    if (max_chunks == 0 || P == 0) return IHIP_OK;
    if (s.b_q == 1) {
        switch (a.ge.G) {
        case 1: launch_decode<1>(a, P, st); break;
        case 2: launch_decode<2>(a, P, st); break;
        case 4: launch_decode<4>(a, P, st); break;
        case 8: launch_decode<8>(a, P, st); break;
        default: return fail(IHIP_ERR_UNSUPPORTED, "Hq/Hkv = %d not in {1,2,4,8}", a.ge.G);
        }
        return check_launch("prune_stage (decode)");
    }
    return fail(IHIP_ERR_UNSUPPORTED, "prune_stage: b_q = %d not built yet", s.b_q);
}

}  // namespace ihip
