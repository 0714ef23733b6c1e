// Block-sparse chunked-prefill attention on the matrix cores.
//
// One workgroup per problem (sequence, KV head, query block of 64), one wave
// per query head of the group, so the gathered K/V tiles are staged in LDS
// once and shared by the G heads.  The attended keys form the virtual slot
// list [sink | kept blocks | window]; it is consumed 32 slots per step.
//
// "Transposed" flash attention, so that every per-query quantity lives in the
// lanes that own that query and nothing has to be shuffled between the two
// matrix products:
//     S^T = K Q^T   (A = K tile from LDS,  B = Q, resident in registers)
//     O^T = V^T P^T (A = V^T tile from LDS, B = P^T = the lanes' own S^T values)
// v_mfma_f32_16x16x32_bf16 layouts: A/B lane l holds 8 consecutive k of
// row/column l%16 (k group l/16); C lane l holds column l%16, rows 4*(l/16)..+3.
// The k order of the second product (keys) is free as long as V^T and P^T
// agree: k slot (kq, j) is key kq*4+j of the first 16-key tile for j < 4 and
// key kq*4+j-4 of the second for j >= 4 -- exactly what a lane's two S^T
// accumulators hold.  V is transposed on its way into LDS.
#include "attn_prefill_args.h"
#include <type_traits>

namespace ihip {

// ROPE: streaming-style dynamic RoPE; the queries are rotated once, a K piece on its way from the
// staging registers into LDS (its table row is fetched along with it), both rounded to bf16.
// PAGED: K and V are page pools; a piece's page is looked up in the block table right before it is fetched.
// KV8: K and V rows are 128 bytes of E4M3 (strides in 2-byte units); a piece stays 8 bytes in the
// staging registers and is repacked as bf16 (exact) on its way into LDS.  The K scale is folded into
// the softmax scale, the V scale into the final normalisation.
template <int QT, int G, bool ROPE, bool PAGED, bool KV8 = false>   // query tiles of 16 (b_q = 16*QT); G query heads = G waves per workgroup
__global__ __launch_bounds__(64 * G) void attn_prefill_kernel(const AttnPrefillArgs a)
{
    using raw_t = typename std::conditional<KV8, uint2, uint4>::type;     // 8 elements of a row as fetched
    constexpr int kPiece = KV8 ? 4 : 8;                                   // ... in 2-byte units
    __shared__ __attribute__((aligned(16))) uint16_t sK[kPfTile * kPfKStride];
    __shared__ __attribute__((aligned(16))) uint16_t sVt[kD * kPfVStride];
    __shared__ int sPos[kPfTile];
    __shared__ int sFlag[2];             // "this tile needs masking", alternating by tile parity

    const int p = blockIdx.x;
    const Problem pr = problem_of(a.ge, p);
    constexpr int nthreads = 64 * G;
    const int tid = threadIdx.x;
    const int lane = tid & 63, hh = tid >> 6;
    const int n = lane & 15, kq = lane >> 4;
    const int h = pr.g * G + hh;
    const int b_q = 16 * QT;
    const int q0 = pr.m * b_q;                 // first query row of the block
    const int qpos0 = pr.E - b_q;              // its absolute position

    const int n_sink_eff = min(a.ge.n_sink, pr.E);
    const int w0 = max(pr.hi, a.ge.n_sink);
    const int total = n_sink_eff + (a.n_blocks << a.block_log2) + max(0, pr.E - w0);
    const int n_tiles = (total + kPfTile - 1) / kPfTile;
    StreamIds ids{n_sink_eff, a.n_blocks << a.block_log2, 0, w0};
    if constexpr (ROPE) {
        __shared__ int sh_tokens;
        ids.block_tokens = pf_block_tokens(a, pr, p, nthreads, &sh_tokens);
    }

    // B operands of the first product: this head's queries
    bf16x8 qb[QT][4];
    {
        const uint16_t *qp = a.q + pr.b * a.q_sb + (int64_t)h * a.q_sh + (int64_t)q0 * a.q_st;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                qb[qt][ks] = *reinterpret_cast<const bf16x8 *>(qp + (int64_t)(qt * 16 + n) * a.q_st + ks * 32 + kq * 8);
                if constexpr (ROPE) {
                    const int64_t at = (int64_t)ids.query(a.ge.n_sink, qpos0 + qt * 16 + n) * (kD / 2) + ks * 16 + kq * 4;
                    qb[qt][ks] = __builtin_bit_cast(
                        bf16x8, rotate_bf16x8(__builtin_bit_cast(uint4, qb[qt][ks]), a.rope_cos + at, a.rope_sin + at));
                }
            }
    }
    const uint16_t *kb = PAGED ? a.k + pr.g * a.k_sh : a.k + pr.b * a.k_sb + pr.g * a.k_sh;
    const uint16_t *vb = PAGED ? a.v + pr.g * a.v_sh : a.v + pr.b * a.v_sb + pr.g * a.v_sh;

    f32x4 o[8][QT];
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m_run[qt] = kNegBigPf; l_run[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[dt][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // loader role: item = (key pair a2, dim group c); 16 pairs x 16 groups per tile
    constexpr int kItems = (kPfTile / 2) * 16;
    constexpr int kMaxPerThread = (kItems + nthreads - 1) / nthreads;
    raw_t rk[kMaxPerThread][2], rv[kMaxPerThread][2];
    int rpos[kMaxPerThread][2];
    float4 rc[ROPE ? kMaxPerThread : 1][2], rs[ROPE ? kMaxPerThread : 1][2];     // table row piece of each K piece

    auto fetch = [&](int tile) {
#pragma unroll
        for (int r = 0; r < kMaxPerThread; ++r) {
            const int item = tid + r * nthreads;
            if (item >= kItems) break;
            const int a2 = item >> 4, c = item & 15;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int slot = tile * kPfTile + a2 * 2 + e;
                const int pos = slot < total ? pf_slot_to_pos(a, pr, p, slot, n_sink_eff, w0) : -1;
                rpos[r][e] = pos;
                rk[r][e] = raw_t{};
                rv[r][e] = raw_t{};
                if (pos >= 0) {
                    if constexpr (PAGED) {
                        const int64_t page = a.paged.block_table[(int64_t)pr.b * a.paged.table_stride + (pos >> a.paged.page_log2)];
                        const int64_t tok = pos & ((1 << a.paged.page_log2) - 1);
                        rk[r][e] = *reinterpret_cast<const raw_t *>(kb + page * a.k_sb + tok * a.k_st + c * kPiece);
                        rv[r][e] = *reinterpret_cast<const raw_t *>(vb + page * a.v_sb + tok * a.v_st + c * kPiece);
                    } else {
                        rk[r][e] = *reinterpret_cast<const raw_t *>(kb + (int64_t)pos * a.k_st + c * kPiece);
                        rv[r][e] = *reinterpret_cast<const raw_t *>(vb + (int64_t)pos * a.v_st + c * kPiece);
                    }
                }
                if constexpr (ROPE) {
                    const int64_t at = (int64_t)(pos >= 0 ? ids.key(slot) : 0) * (kD / 2) + c * 4;
                    rc[r][e] = *reinterpret_cast<const float4 *>(a.rope_cos + at);
                    rs[r][e] = *reinterpret_cast<const float4 *>(a.rope_sin + at);
                }
            }
        }
    };
    auto stash = [&](int tile) {
        bool need_mask = false;
#pragma unroll
        for (int r = 0; r < kMaxPerThread; ++r) {
            const int item = tid + r * nthreads;
            if (item >= kItems) break;
            const int a2 = item >> 4, c = item & 15;
            const int key0 = a2 * 2;                                   // keys key0, key0+1 of the 32
            uint4 wv[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                uint4 wk;
                if constexpr (KV8) {
                    if constexpr (ROPE) wk = rotate_fp8x8(rk[r][e], rc[r][e], rs[r][e]);
                    else wk = fp8x8_to_bf16x8(rk[r][e]);
                    wv[e] = fp8x8_to_bf16x8(rv[r][e]);
                } else {
                    wk = rk[r][e];
                    wv[e] = rv[r][e];
                    if constexpr (ROPE) wk = rotate_bf16x8(wk, rc[r][e], rs[r][e]);
                }
                *reinterpret_cast<uint4 *>(&sK[(key0 + e) * kPfKStride + c * 8]) = wk;
            }
            // k slot of key kk: tile t = kk/16, kq = (kk%16)/4, j = kk%4 + 4*t
            const int t = key0 >> 4, kk = key0 & 15;
            const int kslot = (kk >> 2) * 8 + (kk & 3) + 4 * t;        // even; key0+1 sits at kslot+1
            const uint32_t v0[4] = {wv[0].x, wv[0].y, wv[0].z, wv[0].w};
            const uint32_t v1[4] = {wv[1].x, wv[1].y, wv[1].z, wv[1].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // dims c*8+2i (low halves) and c*8+2i+1 (high halves)
                const uint32_t lo = (v0[i] & 0xffffu) | (v1[i] << 16);
                const uint32_t hi = (v0[i] >> 16) | (v1[i] & 0xffff0000u);
                *reinterpret_cast<uint32_t *>(&sVt[(c * 8 + 2 * i) * kPfVStride + kslot]) = lo;
                *reinterpret_cast<uint32_t *>(&sVt[(c * 8 + 2 * i + 1) * kPfVStride + kslot]) = hi;
            }
            if (c == 0) { sPos[key0] = rpos[r][0]; sPos[key0 + 1] = rpos[r][1]; }
            need_mask |= rpos[r][0] < 0 || rpos[r][1] < 0 || rpos[r][0] >= qpos0 || rpos[r][1] >= qpos0;
        }
        if (need_mask) sFlag[tile & 1] = 1;
    };

    if (n_tiles > 0) fetch(0);
    for (int tile = 0; tile < n_tiles; ++tile) {
        if (tid == 0) sFlag[tile & 1] = 0;     // last read two tiles (and two barriers) ago
        __syncthreads();                       // previous tile fully consumed, flag cleared
        stash(tile);
        __syncthreads();
        if (tile + 1 < n_tiles) fetch(tile + 1);
        const bool masked = sFlag[tile & 1] != 0;

        // V^T operands of this tile: dims dt*16+n, k slots kq*8..+8
        bf16x8 va[8];
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            va[dt] = *reinterpret_cast<const bf16x8 *>(&sVt[(dt * 16 + n) * kPfVStride + kq * 8]);
        // K operands: key kt*16+n, dims ks*32+kq*8..+8
        bf16x8 ka[2][4];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                ka[kt][ks] = *reinterpret_cast<const bf16x8 *>(&sK[(kt * 16 + n) * kPfKStride + ks * 32 + kq * 8]);
        int kpos[2][4];
        if (masked) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int i = 0; i < 4; ++i) kpos[kt][i] = sPos[kt * 16 + kq * 4 + i];
        }

#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            // S^T for 32 keys x 16 queries: lane holds keys kt*16 + kq*4 + i of query qt*16 + n
            f32x4 s[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[kt][ks], qb[qt][ks], c, 0, 0, 0);
                s[kt] = c * a.scale_log2e;
            }
            if (masked) {
                const int qpos = qpos0 + qt * 16 + n;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (kpos[kt][i] < 0 || kpos[kt][i] > qpos) s[kt][i] = -INFINITY;
            }
            float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                             fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
            mx = max_over_rows(mx);        // over the four key groups of the lane's query
            const float mn = fmaxf(m_run[qt], mx);
            const float corr = exp2f(m_run[qt] - mn);
            m_run[qt] = mn;
            float ps = 0.f;
            bf16x8 pb;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float pw = exp2f(s[kt][i] - mn);      // exp2(-inf) = 0 for masked keys
                    ps += pw;
                    pb[kt * 4 + i] = (__bf16)pw;
                }
            l_run[qt] = l_run[qt] * corr + ps;                  // partial over this lane's keys
            if (__any(corr != 1.0f)) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[dt][qt] *= corr;
            }
#pragma unroll
            for (int dt = 0; dt < 8; ++dt)
                o[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pb, o[dt][qt], 0, 0, 0);
        }
    }

    // epilogue: O[q][dim] = O^T / l
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        float l = l_run[qt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const float inv = KV8 ? a.v_scale / l : 1.0f / l;
        const int64_t row = ((int64_t)pr.b * a.ge.Hq + h) * a.ge.Tq + q0 + qt * 16 + n;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            const f32x4 x = o[dt][qt] * inv;
            uint2 w;
            w.x = f32_to_bf16_bits(x[0]) | (f32_to_bf16_bits(x[1]) << 16);
            w.y = f32_to_bf16_bits(x[2]) | (f32_to_bf16_bits(x[3]) << 16);
            *reinterpret_cast<uint2 *>(a.out + row * kD + dt * 16 + kq * 4) = w;
        }
        if (a.out_lse != nullptr && kq == 0)
            a.out_lse[row] = (m_run[qt] + log2f(l)) * 0.69314718055994530942f;
    }
}

int32_t launch_attn_prefill(const ihip_shape &s, const ihip_tensor &q, const ihip_tensor &k,
                            const ihip_tensor &v, const int32_t *block_starts, int n_blocks, int block,
                            float sm_scale, void *out, float *out_lse, const ihip_rope *rope, hipStream_t st,
                            const KvFormat *fmt)
{
    AttnPrefillArgs a;
    const bool fp8 = fmt && fmt->fp8;
    a.paged = (fmt && fmt->paged.block_table) ? fmt->paged : PagedView{nullptr, 0, 0};
    const bool paged = a.paged.block_table != nullptr;
    const bool use_rope = rope && rope->attn_style != IHIP_ROPE_NONE;
    a.rope_cos = a.rope_sin = nullptr;
    if (use_rope) {
        if (rope->attn_style != IHIP_ROPE_STREAMING)
            return fail(IHIP_ERR_INVALID_ARG, "sparse_attn_prefill: rope attn_style = %d", rope->attn_style);
        if (!rope->cos || !rope->sin) return fail(IHIP_ERR_INVALID_ARG, "sparse_attn_prefill: rope tables are NULL");
        // largest id: a query that attends to every slot
        const int64_t need = (int64_t)s.n_sink + (int64_t)n_blocks * block + s.n_stream;
        if (rope->n_pos < need)
            return fail(IHIP_ERR_INVALID_ARG, "sparse_attn_prefill: rope table has %d positions, %lld needed",
                        rope->n_pos, (long long)need);
        a.rope_cos = rope->cos;
        a.rope_sin = rope->sin;
    }
    a.ge = make_geometry(s);
    a.q = (const uint16_t *)q.ptr; a.q_sb = q.stride_b; a.q_sh = q.stride_h; a.q_st = q.stride_t;
    a.k = (const uint16_t *)k.ptr; a.k_sb = k.stride_b; a.k_sh = k.stride_h; a.k_st = k.stride_t;
    a.v = (const uint16_t *)v.ptr; a.v_sb = v.stride_b; a.v_sh = v.stride_h; a.v_st = v.stride_t;
    a.v_scale = 1.0f;
    if (fp8) {      // byte strides (even) in 2-byte units
        a.k_sb /= 2; a.k_sh /= 2; a.k_st /= 2;
        a.v_sb /= 2; a.v_sh /= 2; a.v_st /= 2;
        a.v_scale = fmt->v_scale;
    }
    a.block_starts = block_starts;
    a.n_blocks = n_blocks;
    a.block = block;
    a.block_log2 = __builtin_ctz(block);
    a.scale_log2e = sm_scale * 1.44269504088896340736f * (fp8 ? fmt->k_scale : 1.0f);
    a.out = (uint16_t *)out;
    a.out_lse = out_lse;
    const int P = s.B * s.Hkv * (s.Tq / s.b_q);
    if (P == 0) return IHIP_OK;
    KernelTimer timer("attn_prefill", st);
    const dim3 block_dim(64 * a.ge.G), grid(P);
#define IHIP_PF_BY_G3(KERNEL, QT, RP, PG, F8)                                                      \
    switch (a.ge.G) {                                                                              \
    case 1: hipLaunchKernelGGL((KERNEL<QT, 1, RP, PG, F8>), grid, block_dim, 0, st, a); break;     \
    case 2: hipLaunchKernelGGL((KERNEL<QT, 2, RP, PG, F8>), grid, block_dim, 0, st, a); break;     \
    case 4: hipLaunchKernelGGL((KERNEL<QT, 4, RP, PG, F8>), grid, block_dim, 0, st, a); break;     \
    default: hipLaunchKernelGGL((KERNEL<QT, 8, RP, PG, F8>), grid, block_dim, 0, st, a); break;    \
    }
#define IHIP_PF_BY_G2(KERNEL, QT, RP, PG)                                                          \
    if (fp8) { IHIP_PF_BY_G3(KERNEL, QT, RP, PG, true) } else { IHIP_PF_BY_G3(KERNEL, QT, RP, PG, false) }
#define IHIP_PF_BY_G(KERNEL, QT)                                                                   \
    if (use_rope && paged) { IHIP_PF_BY_G2(KERNEL, QT, true, true) }                               \
    else if (use_rope) { IHIP_PF_BY_G2(KERNEL, QT, true, false) }                                  \
    else if (paged) { IHIP_PF_BY_G2(KERNEL, QT, false, true) }                                     \
    else { IHIP_PF_BY_G2(KERNEL, QT, false, false) }
    // the 32x32 kernel keeps every slot's position in LDS; longer key lists take the 16x16 one
    const int slot_limit = use_rope ? (paged ? kPf32MaxSlotsRopePaged : kPf32MaxSlotsRope)
                                    : (paged ? kPf32MaxSlotsPaged : kPf32MaxSlots);
    if (fp8 && s.b_q >= 32 && s.n_sink + n_blocks * block + s.n_stream <= (paged ? kPf32MaxSlotsFp8Paged : kPf32MaxSlotsFp8)) {
        launch_attn_prefill32_fp8(a, P, st);
        return check_launch("sparse_attn_prefill");
    }
    if (!fp8 && s.b_q >= 32 && s.n_sink + n_blocks * block + s.n_stream <= slot_limit) {
        launch_attn_prefill32(a, P, s.max_seq_len, st);
        return check_launch("sparse_attn_prefill");
    }
    switch (s.b_q) {
    case 16: IHIP_PF_BY_G(attn_prefill_kernel, 1); break;
    case 32: IHIP_PF_BY_G(attn_prefill_kernel, 2); break;
    case 64: IHIP_PF_BY_G(attn_prefill_kernel, 4); break;
    default: return fail(IHIP_ERR_UNSUPPORTED, "sparse_attn_prefill: b_q = %d not in {16, 32, 64}", s.b_q);
    }
#undef IHIP_PF_BY_G
#undef IHIP_PF_BY_G2
#undef IHIP_PF_BY_G3
    return check_launch("sparse_attn_prefill");
}

}  // namespace ihip
