// Block-sparse decode attention over sink + kept blocks + window.
//
// HBM-bound gather of K and V rows (512 B per attended token, shared by the G
// query heads of the KV head).  Flash-decoding layout: the attended tokens of
// a problem form a virtual slot list  [sink | kept blocks | window];  the list
// is cut into splits, one workgroup each; inside a workgroup every 16-lane
// group owns one token at a time (16 B of the K row and of the V row per
// lane) and keeps an online-softmax state for all G heads; groups are merged
// through LDS, splits by a second small kernel (log-sum-exp merge).
#include "common.h"
#include <algorithm>
#include <type_traits>

namespace ihip {

constexpr int kAttnThreads = 256;
constexpr int kAttnGroups = kAttnThreads / kRowLanes;   // 16 tokens in flight per step
constexpr int kAttnMinSplit = 256, kAttnMaxSplit = 1024;   // slots of one split (a multiple of 16)
constexpr float kNegBig = -1.0e30f;                      // finite stand-in for -inf in running maxima

struct AttnDecodeArgs {
    Geometry ge;
    const uint16_t *q; int64_t q_sb, q_sh, q_st;
    const uint16_t *k; int64_t k_sb, k_sh, k_st;
    const uint16_t *v; int64_t v_sb, v_sh, v_st;
    const int32_t *block_starts;
    int n_blocks, block, block_log2;
    float scale_log2e;
    int n_splits, slots_per_split;
    float *part_ml;      // [P, n_splits, G, 2]   (running max in log2 units, sum)
    float *part_acc;     // [P, n_splits, G, 128]
    uint16_t *out;       // bf16 [B, Hq, 1, d]
    float *out_lse;      // [B, Hq] or null
    BankView bank;       // used by the cached instantiations only (K/V then point to host memory)
    const float *rope_cos, *rope_sin;   // streaming-style RoPE instantiations only: fp32 [n_pos][d/2]
    PagedView paged;     // paged instantiations only: K and V are page pools, *_sb the page strides
    float v_scale;       // FP8 instantiations: the output is multiplied by it (the K scale is folded into
                         // scale_log2e; K/V strides then count 2-byte units of the byte rows)
};

__device__ inline uint4 as_bf16x8(const uint4 &k) { return k; }
__device__ inline uint4 as_bf16x8(const uint2 &k) { return fp8x8_to_bf16x8(k); }

// SRC 0: K/V in HBM through strides; 1: host tier with the on-GPU bank; 2: paged pools
template <int SRC> struct KvSource;
template <> struct KvSource<0> {
    typedef DirectRows type;
    static __device__ type k(const AttnDecodeArgs &a, const Problem &pr)
    {
        return DirectRows{a.k + pr.b * a.k_sb + pr.g * a.k_sh, a.k_st};
    }
    static __device__ type v(const AttnDecodeArgs &a, const Problem &pr)
    {
        return DirectRows{a.v + pr.b * a.v_sb + pr.g * a.v_sh, a.v_st};
    }
};
template <> struct KvSource<1> {
    typedef CachedRows type;
    static __device__ type k(const AttnDecodeArgs &a, const Problem &pr)
    {
        return cached_rows(a.bank, a.k, a.k_sb, a.k_sh, a.k_st, a.bank.bank_k, pr.b, pr.g, a.ge.Hkv);
    }
    static __device__ type v(const AttnDecodeArgs &a, const Problem &pr)
    {
        return cached_rows(a.bank, a.v, a.v_sb, a.v_sh, a.v_st, a.bank.bank_v, pr.b, pr.g, a.ge.Hkv);
    }
};

template <> struct KvSource<2> {
    typedef PagedRows type;
    static __device__ type k(const AttnDecodeArgs &a, const Problem &pr)
    {
        return PagedRows{a.k + pr.g * a.k_sh, a.paged.block_table + (int64_t)pr.b * a.paged.table_stride, a.k_sb,
                         a.k_st, a.paged.page_log2};
    }
    static __device__ type v(const AttnDecodeArgs &a, const Problem &pr)
    {
        return PagedRows{a.v + pr.g * a.v_sh, a.paged.block_table + (int64_t)pr.b * a.paged.table_stride, a.v_sb,
                         a.v_st, a.paged.page_log2};
    }
};

// slot -> key position, or -1
__device__ inline int slot_to_pos(const AttnDecodeArgs &a, const Problem &pr, int p, int slot,
                                  int n_sink_eff, int w0)
{
    if (slot < n_sink_eff) return slot;
    slot -= n_sink_eff;
    const int nb = a.n_blocks << a.block_log2;
    if (slot < nb) {
        const int bs = a.block_starts[(int64_t)p * a.n_blocks + (slot >> a.block_log2)];
        if (bs < 0) return -1;
        const int pos = bs + (slot & (a.block - 1));
        return pos < pr.hi ? pos : -1;
    }
    const int pos = w0 + (slot - nb);
    return pos < pr.E ? pos : -1;
}

// ROPE: streaming-style positions (Sec. 4 "Dynamic RoPE ..."): the attended keys, in position
// order, are rotated to positions 0, 1, ..., n-1 and the query to n-1.  Attended slots are a
// prefix of the block part of the slot list (blocks are ascending, empty ones last, only the last
// one can be cut short), so a key's id is its slot, less the empty block slots for window keys.
// KV8: K and V rows are 128 bytes of E4M3 (8 bytes per lane), repacked exactly as bf16 for the dot.
template <int G, int SRC, bool ROPE, bool KV8>
__global__ __launch_bounds__(kAttnThreads) void attn_decode_split_kernel(const AttnDecodeArgs a)
{
    using piece_t = typename std::conditional<KV8, uint2, uint4>::type;     // a lane's share of a row
    constexpr int kLaneOff = KV8 ? 4 : 8;                                   // in 2-byte units
    const int p = blockIdx.y, split = blockIdx.x;
    const Problem pr = problem_of(a.ge, p);
    const int l16 = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int n_sink_eff = min(a.ge.n_sink, pr.E);
    const int w0 = max(pr.hi, a.ge.n_sink);

    // this lane's 8 dims of the G query vectors, kept packed (bf16 pairs) for the dot2 instruction
    uint4 qp[G];
    {
        const uint16_t *qb = a.q + pr.b * a.q_sb + (int64_t)(pr.g * G) * a.q_sh;
#pragma unroll
        for (int h = 0; h < G; ++h) qp[h] = load_row16(qb, h * a.q_sh, l16);
    }
    // ROPE: tokens in the kept blocks (so that window keys and the query know their ids) and the
    // rotated queries, fp32
    __shared__ int sh_block_tokens;
    float qr[ROPE ? G : 1][8];
    int block_slots = 0, block_tokens = 0;
    if (ROPE) {
        if (threadIdx.x == 0) sh_block_tokens = 0;
        __syncthreads();
        int mine = 0;
        for (int i = threadIdx.x; i < a.n_blocks; i += kAttnThreads) {
            const int bs = a.block_starts[(int64_t)p * a.n_blocks + i];
            if (bs >= 0 && bs < pr.hi) mine += min(a.block, pr.hi - bs);
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
        if ((threadIdx.x & 63) == 0 && mine > 0) atomicAdd(&sh_block_tokens, mine);
        __syncthreads();
        block_slots = a.n_blocks << a.block_log2;
        block_tokens = sh_block_tokens;
        const int n_sel = n_sink_eff + block_tokens + max(0, pr.E - w0);
        const float4 c = *reinterpret_cast<const float4 *>(a.rope_cos + (int64_t)(n_sel - 1) * (kD / 2) + l16 * 4);
        const float4 sn = *reinterpret_cast<const float4 *>(a.rope_sin + (int64_t)(n_sel - 1) * (kD / 2) + l16 * 4);
        const float cc[4] = {c.x, c.y, c.z, c.w}, ss[4] = {sn.x, sn.y, sn.z, sn.w};
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float x[8];
            unpack8(qp[h], x);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                qr[h][2 * i] = x[2 * i] * cc[i] - x[2 * i + 1] * ss[i];
                qr[h][2 * i + 1] = x[2 * i] * ss[i] + x[2 * i + 1] * cc[i];
            }
        }
    }
    const typename KvSource<SRC>::type ksrc = KvSource<SRC>::k(a, pr);
    const typename KvSource<SRC>::type vsrc = KvSource<SRC>::v(a, pr);

    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = kNegBig; l[h] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[h][i] = 0.f;
    }

    constexpr int UNR = 4;
    const int s0 = split * a.slots_per_split;
    const int s1 = s0 + a.slots_per_split;
    // key position of every slot of this split, computed up front, so that the main loop has no
    // dependent global loads (block start -> row address)
    __shared__ int sh_pos[kAttnMaxSplit];
    __shared__ int sh_page[SRC == 2 ? kAttnMaxSplit : 1];    // paged K/V: the slot's page id, looked up here once
    for (int i = threadIdx.x; i < a.slots_per_split; i += kAttnThreads) {
        const int pos = slot_to_pos(a, pr, p, s0 + i, n_sink_eff, w0);
        sh_pos[i] = pos;
        if constexpr (SRC == 2) sh_page[i] = pos >= 0 ? ksrc.table_entry(pos) : 0;
    }
    __syncthreads();
    for (int base = s0 + grp; base < s1; base += kAttnGroups * UNR) {
        piece_t kr[UNR], vr[UNR];
        bool ok[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int slot = base + u * kAttnGroups;
            const int pos = slot < s1 ? sh_pos[slot - s0] : -1;
            ok[u] = pos >= 0;
            kr[u] = piece_t{};
            vr[u] = piece_t{};
            if (ok[u]) {
                if constexpr (SRC == 2) {
                    const int page = sh_page[slot - s0];
                    kr[u] = *reinterpret_cast<const piece_t *>(ksrc.row_in_page(page, pos) + l16 * kLaneOff);
                    vr[u] = *reinterpret_cast<const piece_t *>(vsrc.row_in_page(page, pos) + l16 * kLaneOff);
                } else {
                    kr[u] = *reinterpret_cast<const piece_t *>(ksrc.row(pos, l16 == 0) + l16 * kLaneOff);
                    vr[u] = *reinterpret_cast<const piece_t *>(vsrc.row(pos, false) + l16 * kLaneOff);   // K did the bookkeeping
                }
            }
        }
        // scores of the UNR tokens for all heads (log2 units), then one running-max update per batch
        float sc[UNR][G];
        if (ROPE) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int slot = base + u * kAttnGroups;
                // id of the key: its slot, less the empty block slots if it is a window key
                const int id = ok[u] ? (slot < n_sink_eff + block_slots ? slot : slot - (block_slots - block_tokens)) : 0;
                const float4 c = *reinterpret_cast<const float4 *>(a.rope_cos + (int64_t)id * (kD / 2) + l16 * 4);
                const float4 sn = *reinterpret_cast<const float4 *>(a.rope_sin + (int64_t)id * (kD / 2) + l16 * 4);
                const float cc[4] = {c.x, c.y, c.z, c.w}, ss[4] = {sn.x, sn.y, sn.z, sn.w};
                float x[8], kt[8];
                unpack8(kr[u], x);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    kt[2 * i] = x[2 * i] * cc[i] - x[2 * i + 1] * ss[i];
                    kt[2 * i + 1] = x[2 * i] * ss[i] + x[2 * i + 1] * cc[i];
                }
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    float d8 = kt[0] * qr[h][0];
#pragma unroll
                    for (int i = 1; i < 8; ++i) d8 = fmaf(kt[i], qr[h][i], d8);
                    sc[u][h] = ok[u] ? row16_sum(d8) * a.scale_log2e : kNegBig;
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int h = 0; h < G; ++h)
                    sc[u][h] = ok[u] ? row16_sum(dot8_bf16(as_bf16x8(kr[u]), qp[h])) * a.scale_log2e : kNegBig;
        }
        float pw[UNR][G], corr[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float mn = m[h];
#pragma unroll
            for (int u = 0; u < UNR; ++u) mn = fmaxf(mn, sc[u][h]);
            corr[h] = __builtin_amdgcn_exp2f(m[h] - mn);
            m[h] = mn;
            float ps = 0.f;
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                pw[u][h] = ok[u] ? __builtin_amdgcn_exp2f(sc[u][h] - mn) : 0.f;
                ps += pw[u][h];
            }
            l[h] = l[h] * corr[h] + ps;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[h][i] *= corr[h];
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            float vf[8];
            unpack8(vr[u], vf);
#pragma unroll
            for (int h = 0; h < G; ++h)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[h][i] = fmaf(pw[u][h], vf[i], acc[h][i]);
        }
    }

    // merge the 4 groups of each wave in registers (lanes l, l^16, l^32, l^48 hold the same dims): a
    // row swap hands every lane its own and its partner's value (which of the two is which differs
    // between the partners; the merge is symmetric in them, so both compute the same bits)
    auto both = [](float x, int d, float &a, float &b) {
        const unsigned u = __float_as_uint(x);
        if (d == 16) {
            const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
            a = __uint_as_float(r[0]); b = __uint_as_float(r[1]);
        } else {
            const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
            a = __uint_as_float(r[0]); b = __uint_as_float(r[1]);
        }
    };
#pragma unroll
    for (int d = 16; d <= 32; d <<= 1) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float ma, mb, la, lb;
            both(m[h], d, ma, mb);
            both(l[h], d, la, lb);
            const float mn = fmaxf(ma, mb);
            const float wa = __builtin_amdgcn_exp2f(ma - mn), wb = __builtin_amdgcn_exp2f(mb - mn);
            l[h] = la * wa + lb * wb;
            m[h] = mn;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float xa, xb;
                both(acc[h][i], d, xa, xb);
                acc[h][i] = xa * wa + xb * wb;
            }
        }
    }
    // then the waves through LDS
    constexpr int NW = kAttnThreads / kWave;
    __shared__ float sh_m[NW][G], sh_l[NW][G];
    __shared__ float sh_acc[NW][G][kD];
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) { sh_m[wv][h] = m[h]; sh_l[wv][h] = l[h]; }
    }
    if (lane < 16) {
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
            for (int i = 0; i < 8; ++i) sh_acc[wv][h][l16 * 8 + i] = acc[h][i];
    }
    __syncthreads();

    const int64_t pbase = ((int64_t)p * a.n_splits + split) * G;
    for (int idx = threadIdx.x; idx < G * kD; idx += kAttnThreads) {
        const int h = idx / kD, c = idx % kD;
        float M = kNegBig;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) M = fmaxf(M, sh_m[w2][h]);
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) {
            const float w = __builtin_amdgcn_exp2f(sh_m[w2][h] - M);
            L = fmaf(w, sh_l[w2][h], L);
            A = fmaf(w, sh_acc[w2][h][c], A);
        }
        a.part_acc[(pbase + h) * kD + c] = A;
        if (c == 0) {
            a.part_ml[(pbase + h) * 2 + 0] = M;
            a.part_ml[(pbase + h) * 2 + 1] = L;
        }
    }
}

// merge the splits: one workgroup of 128 threads per (problem, head), a thread per dim.  The partial
// results of the first 16 splits (all of them in the usual shapes) are requested at once, before
// anything is computed, and every thread takes the maximum over the splits itself: one trip to
// memory and no barrier, where a reduction of the maxima first and the sums after it made two
// dependent trips.  The sums run over the splits in order, so the result does not depend on this.
constexpr int kMergeAhead = 16;
__global__ __launch_bounds__(kD) void attn_decode_merge_kernel(const AttnDecodeArgs a)
{
    const int G = a.ge.G;
    const int p = blockIdx.x / G, h = blockIdx.x % G;
    const int c = threadIdx.x;
    const int b = p / a.ge.Hkv, g = p % a.ge.Hkv;            // decode: one problem per (sequence, KV head)
    const int64_t pbase = (int64_t)p * a.n_splits * G;
    const float2 *ml = reinterpret_cast<const float2 *>(a.part_ml);
    float2 mlv[kMergeAhead];
    float av[kMergeAhead];
#pragma unroll
    for (int s = 0; s < kMergeAhead; ++s) {
        const int64_t r = pbase + (int64_t)min(s, a.n_splits - 1) * G + h;      // clamped: ignored beyond the last split
        mlv[s] = ml[r];
        av[s] = a.part_acc[r * kD + c];
    }
    float M = kNegBig;
#pragma unroll
    for (int s = 0; s < kMergeAhead; ++s)
        if (s < a.n_splits) M = fmaxf(M, mlv[s].x);
    for (int s = kMergeAhead; s < a.n_splits; ++s) M = fmaxf(M, ml[pbase + (int64_t)s * G + h].x);
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int s = 0; s < kMergeAhead; ++s) {
        if (s < a.n_splits) {
            const float w = __builtin_amdgcn_exp2f(mlv[s].x - M);
            L = fmaf(w, mlv[s].y, L);
            A = fmaf(w, av[s], A);
        }
    }
#pragma unroll 8
    for (int s = kMergeAhead; s < a.n_splits; ++s) {
        const int64_t r = pbase + (int64_t)s * G + h;
        const float2 x = ml[r];
        const float w = __builtin_amdgcn_exp2f(x.x - M);
        L = fmaf(w, x.y, L);
        A = fmaf(w, a.part_acc[r * kD + c], A);
    }
    const int hq = g * G + h;
    a.out[((int64_t)b * a.ge.Hq + hq) * kD + c] = (uint16_t)f32_to_bf16_bits(A / L * a.v_scale);
    if (a.out_lse != nullptr && c == 0)
        a.out_lse[(int64_t)b * a.ge.Hq + hq] = (M + log2f(L)) * 0.69314718055994530942f;
}

// Splits of the slot list: as many workgroups as the chip holds at once (4 workgroups of 4 waves
// per CU with the plain kernel's registers), so that no workgroup has to wait for a free slot and
// run its whole latency chain after the others have drained -- with 256-slot splits the cfg3 shape
// had 1344 workgroups for 1024 places.  Between 256 and 1024 slots per split, a multiple of 16.
// wg_per_cu: 4 for the plain kernels, 3 for the RoPE instantiations (more registers).  The workspace
// is sized for 4, which gives the most splits.
static int decode_splits(const ihip_shape &s, int n_blocks, int block, int *slots_per_split, int wg_per_cu = 4)
{
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
            n_cu = 256;
    }
    const int total = s.n_sink + n_blocks * block + s.n_stream;
    const int P = std::max(1, s.B * s.Hkv);
    const int places = std::max(1, n_cu * wg_per_cu / P);      // splits per problem that run at once
    int per = ((total + places - 1) / places + 15) / 16 * 16;
    per = std::min(kAttnMaxSplit, std::max(kAttnMinSplit, per));
    *slots_per_split = per;
    return (total + per - 1) / per;
}

size_t attn_decode_workspace(const ihip_shape &s, int n_blocks, int block)
{
    int per;
    const int ns = decode_splits(s, n_blocks, block, &per);
    const size_t P = (size_t)s.B * s.Hkv;
    const size_t G = s.Hq / s.Hkv;
    return P * ns * G * (2 + kD) * sizeof(float);
}

int32_t launch_attn_decode(const ihip_shape &s, const ihip_tensor &q, const ihip_tensor &k,
                           const ihip_tensor &v, const int32_t *block_starts, int n_blocks, int block,
                           float sm_scale, void *out, float *out_lse, void *ws, const BankView *bank,
                           const ihip_rope *rope, hipStream_t st, const KvFormat *fmt)
{
    AttnDecodeArgs a;
    const bool fp8 = fmt && fmt->fp8;
    a.v_scale = fp8 ? fmt->v_scale : 1.0f;
    a.paged = (fmt && fmt->paged.block_table) ? fmt->paged : PagedView{nullptr, 0, 0};
    const bool paged = a.paged.block_table != nullptr;
    if (paged && bank)
        return fail(IHIP_ERR_UNSUPPORTED, "sparse_attn_decode: paged K/V and the host tier exclude each other");
    const bool use_rope = rope && rope->attn_style != IHIP_ROPE_NONE;
    a.rope_cos = a.rope_sin = nullptr;
    if (use_rope) {
        if (rope->attn_style != IHIP_ROPE_STREAMING)
            return fail(IHIP_ERR_INVALID_ARG, "sparse_attn_decode: rope attn_style = %d", rope->attn_style);
        if (!rope->cos || !rope->sin) return fail(IHIP_ERR_INVALID_ARG, "sparse_attn_decode: rope tables are NULL");
        const int64_t need = (int64_t)s.n_sink + (int64_t)n_blocks * block + s.n_stream;   // most keys a query can attend
        if (rope->n_pos < need)
            return fail(IHIP_ERR_INVALID_ARG, "sparse_attn_decode: rope table has %d positions, %lld needed",
                        rope->n_pos, (long long)need);
        a.rope_cos = rope->cos;
        a.rope_sin = rope->sin;
    }
    if (bank && (bank->row_units == kD) == fp8)
        return fail(IHIP_ERR_INVALID_ARG, "sparse_attn_decode: the host tier holds %s rows", fp8 ? "bf16" : "E4M3");
    a.bank = bank ? *bank : BankView{};
    a.ge = make_geometry(s);
    a.q = (const uint16_t *)q.ptr; a.q_sb = q.stride_b; a.q_sh = q.stride_h; a.q_st = q.stride_t;
    a.k = (const uint16_t *)k.ptr; a.k_sb = k.stride_b; a.k_sh = k.stride_h; a.k_st = k.stride_t;
    a.v = (const uint16_t *)v.ptr; a.v_sb = v.stride_b; a.v_sh = v.stride_h; a.v_st = v.stride_t;
    if (fp8) {
        a.k_sb /= 2; a.k_sh /= 2; a.k_st /= 2;      // byte strides (even) in 2-byte units
        a.v_sb /= 2; a.v_sh /= 2; a.v_st /= 2;
    }
    a.block_starts = block_starts;
    a.n_blocks = n_blocks;
    a.block = block;
    a.block_log2 = __builtin_ctz(block);
    a.scale_log2e = sm_scale * 1.44269504088896340736f * (fp8 ? fmt->k_scale : 1.0f);
    a.n_splits = decode_splits(s, n_blocks, block, &a.slots_per_split, use_rope ? 3 : 4);
    const int P = s.B * s.Hkv;
    const int G = a.ge.G;
    a.part_ml = (float *)ws;
    a.part_acc = a.part_ml + (size_t)P * a.n_splits * G * 2;
    a.out = (uint16_t *)out;
    a.out_lse = out_lse;
    if (P == 0) return IHIP_OK;
    dim3 grid(a.n_splits, P);
    {
    KernelTimer timer("attn_decode_split", st);
    switch (G) {
#define IHIP_AD_KERNEL(GG, SRCV, RV, F8V)                                                                           \
    hipLaunchKernelGGL((attn_decode_split_kernel<GG, SRCV, RV, F8V>), grid, dim3(kAttnThreads), 0, st, a)
#define IHIP_AD_BY_FMT(GG, SRCV)                                                                                    \
    if (use_rope && fp8) IHIP_AD_KERNEL(GG, SRCV, true, true);                                                      \
    else if (use_rope) IHIP_AD_KERNEL(GG, SRCV, true, false);                                                       \
    else if (fp8) IHIP_AD_KERNEL(GG, SRCV, false, true);                                                            \
    else IHIP_AD_KERNEL(GG, SRCV, false, false)
#define IHIP_AD_LAUNCH(GG)                                                                                          \
    if (bank) { IHIP_AD_BY_FMT(GG, 1); }                                                                            \
    else if (paged) { IHIP_AD_BY_FMT(GG, 2); }                                                                      \
    else { IHIP_AD_BY_FMT(GG, 0); }
    case 1: IHIP_AD_LAUNCH(1); break;
    case 2: IHIP_AD_LAUNCH(2); break;
    case 4: IHIP_AD_LAUNCH(4); break;
    case 8: IHIP_AD_LAUNCH(8); break;
#undef IHIP_AD_LAUNCH
#undef IHIP_AD_BY_FMT
#undef IHIP_AD_KERNEL
    default: return fail(IHIP_ERR_UNSUPPORTED, "Hq/Hkv = %d not in {1,2,4,8}", G);
    }
    }
    int32_t rc = check_launch("sparse_attn_decode (split)");
    if (rc != IHIP_OK) return rc;
    KernelTimer timer("attn_decode_merge", st);
    hipLaunchKernelGGL(attn_decode_merge_kernel, dim3(P * G), dim3(kD), 0, st, a);
    return check_launch("sparse_attn_decode (merge)");
}

}  // namespace ihip
