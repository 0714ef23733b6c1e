// Shared device/host helpers of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ihip.h"
#include "../../include/ihip_measure.h"

struct ihip_cache;

namespace ihip {

constexpr int kD = 128;            // head dimension: 16 lanes x 8 bf16 (16 B) per row
constexpr int kRowLanes = 16;      // lanes that share one K/V row
constexpr int kWave = 64;

// ---- error plumbing (api.hip) ------------------------------------------
int32_t fail(int32_t code, const char *fmt, ...);
int32_t check_launch(const char *what);

// ---- optional per-kernel timing (api.hip) ----------------------------------
// When profiling is on, a KernelTimer brackets one kernel launch with two HIP
// events on the launch stream; ihip_profile_read() sums them up per name.
void profile_begin(const char *name, hipStream_t st);
void profile_end(hipStream_t st);
// Static name "<prefix>.l<chunk>" (or "<prefix>.first.l<chunk>") for the timing table.
const char *stage_name(int which, bool first, int chunk);
enum { kNamePruneDecode = 0, kNamePrunePrefill = 1, kNameSelect = 2 };
struct KernelTimer {
    hipStream_t st;
    KernelTimer(const char *name, hipStream_t s) : st(s) { profile_begin(name, s); }
    ~KernelTimer() { profile_end(st); }
};

// ---- matrix-core throughput probe (mfma_rate.hip) ---------------------------
double measure_mfma_rate(int kind, int iters, float *sink, hipStream_t st);

// ---- geometry of one problem ---------------------------------------------
struct Geometry {
    const int32_t *seq_lens;
    int32_t B, Hq, Hkv, G, Tq, b_q, Mq, n_sink, n_stream;
    int32_t b_q_range;      // block size that defines the candidate range (>= b_q; b_q unless the stages differ)
};

__host__ __device__ inline Geometry make_geometry(const ihip_shape &s)
{
    Geometry g;
    g.seq_lens = s.seq_lens;
    g.B = s.B; g.Hq = s.Hq; g.Hkv = s.Hkv; g.G = s.Hq / s.Hkv;
    g.Tq = s.Tq; g.b_q = s.b_q; g.Mq = s.Tq / s.b_q;
    g.n_sink = s.n_sink; g.n_stream = s.n_stream;
    g.b_q_range = s.b_q_range > 0 ? s.b_q_range : s.b_q;
    return g;
}

struct Problem {
    int b, g, m;
    int lo, hi, E;      // middle range [lo, hi), visible keys [0, E)
};

__device__ inline Problem problem_of(const Geometry &ge, int p)
{
    Problem r;
    r.m = p % ge.Mq;
    const int bg = p / ge.Mq;
    r.g = bg % ge.Hkv;
    r.b = bg / ge.Hkv;
    const int T = ge.seq_lens[r.b];
    r.E = (T - ge.Tq) + (r.m + 1) * ge.b_q;
    r.lo = ge.n_sink;
    // Alg. 1 step 1 defines the candidate range with the first stage's query block: a finer block
    // inherits the range of the coarse block that holds it (and a window that starts there)
    const int E_range = ge.b_q_range == ge.b_q ? r.E
                                               : (T - ge.Tq) + (r.m * ge.b_q / ge.b_q_range + 1) * ge.b_q_range;
    r.hi = E_range - ge.n_stream;
    return r;
}

// Start position of chunk slot j (or -1) -- first stage: implicit; later
// stages: child c of parent i.
__device__ inline int slot_start(const Problem &pr, const int32_t *parent_starts, int n_parent,
                                 int ratio_log2, int chunk, int p, int j)
{
    int start;
    if (parent_starts == nullptr) {
        start = pr.lo + j * chunk;
    } else {
        const int ps = parent_starts[(int64_t)p * n_parent + (j >> ratio_log2)];
        if (ps < 0) return -1;
        start = ps + (j & ((1 << ratio_log2) - 1)) * chunk;
    }
    return start < pr.hi ? start : -1;
}

// ---- where a K or V row lives ------------------------------------------------
// Kernels read rows through a "source".  DirectRows: the tensor is in HBM.
// CachedRows: the tensor is in pinned host memory and 2^block_log2-token
// blocks of it may have a copy in an on-GPU bank; a page table maps the global
// block id to a bank slot (Sec. 4 "KV Cache Offloading").  Every access marks
// the block as touched; a hit refreshes the slot's LRU stamp, a miss reads the
// host copy over the host link and flags the block for insertion.
struct DirectRows {
    const uint16_t *base;     // row 0 of this (sequence, KV head)
    int64_t st;               // elements between rows
    __device__ const uint16_t *row(int pos, bool) const { return base + (int64_t)pos * st; }
};

// PagedRows: the tensor is a pool of fixed-size pages, [page][KV head][token in page][d] through
// the strides; a per-sequence block table maps logical page -> page id (paged KV cache).
struct PagedView {
    const int32_t *block_table;  // [B][table_stride]
    int table_stride;
    int page_log2;               // tokens per page = 1 << page_log2
};
struct PagedRows {
    const uint16_t *pool;        // page 0, this KV head, token 0
    const int32_t *table;        // this sequence's row of the block table
    int64_t page_st, st;         // elements between pages / between tokens of a page
    int page_log2;
    __device__ const uint16_t *row_in_page(int page, int pos) const
    {
        return pool + (int64_t)page * page_st + (int64_t)(pos & ((1 << page_log2) - 1)) * st;
    }
    __device__ int table_entry(int pos) const { return table[pos >> page_log2]; }
    __device__ const uint16_t *row(int pos, bool) const { return row_in_page(table_entry(pos), pos); }
};

struct BankView {
    const int32_t *page_table;   // [n_blocks_total] slot or -1
    uint32_t *slot_stamp;        // [n_slots] call counter of the last touch
    uint8_t *touch_flag;         // [n_blocks_total] touched during this call
    uint8_t *miss_flag;          // [n_blocks_total] touched and not resident
    const uint16_t *bank_k;      // [n_slots][block][d]
    const uint16_t *bank_v;      // same for V, or null (bank holds keys only)
    int block_log2;
    int blocks_per_head;         // blocks of one (sequence, KV head)
    uint32_t stamp;              // this call's counter value
    int row_units;               // 2-byte units of one row: d for bf16 rows, d/2 for E4M3 rows
    // the host tier is a page pool read through a block table (device int32 [B][host_table_stride]),
    // or contiguous per sequence (host_table == nullptr)
    const int32_t *host_table;
    int host_table_stride, host_page_log2;
};

struct CachedRows {
    BankView c;
    const uint16_t *host_base;   // row 0 of this (sequence, KV head) in host memory (paged: of this head in page 0)
    int64_t host_st;
    const uint16_t *bank;        // bank_k or bank_v
    int gb0;                     // global id of this (sequence, KV head)'s block 0
    const int32_t *host_pages;   // paged host tier: this sequence's row of the block table, else nullptr
    int64_t host_page_stride;
    // leader: one lane per row does the bookkeeping stores
    __device__ const uint16_t *row(int pos, bool leader) const
    {
        const int gb = gb0 + (pos >> c.block_log2);
        const int slot = c.page_table[gb];
        if (leader) {
            c.touch_flag[gb] = 1;
            if (slot >= 0) c.slot_stamp[slot] = c.stamp;
            else c.miss_flag[gb] = 1;
        }
        if (slot >= 0)
            return bank + ((((int64_t)slot << c.block_log2) | (pos & ((1 << c.block_log2) - 1))) * c.row_units);
        if (host_pages != nullptr)
            return host_base + (int64_t)host_pages[pos >> c.host_page_log2] * host_page_stride +
                   (int64_t)(pos & ((1 << c.host_page_log2) - 1)) * host_st;
        return host_base + (int64_t)pos * host_st;
    }
};

// Rows of (sequence b, KV head g) behind the host tier.  base / sb / sh / st: the host tensor (paged:
// the pool, sb = elements between pages); bank: the bank's K or V rows.
__device__ inline CachedRows cached_rows(const BankView &c, const uint16_t *base, int64_t sb, int64_t sh, int64_t st,
                                         const uint16_t *bank, int b, int g, int Hkv)
{
    const bool paged = c.host_table != nullptr;
    return CachedRows{c, paged ? base + g * sh : base + b * sb + g * sh, st, bank, (b * Hkv + g) * c.blocks_per_head,
                      paged ? c.host_table + (int64_t)b * c.host_table_stride : nullptr, sb};
}

// ---- bf16 ------------------------------------------------------------------
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 (finite inputs)
__device__ inline uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Two fp32 -> a packed pair of bf16 (a in the low half), round to nearest even: one
// v_cvt_pk_bf16_f32, where the integer form above takes a dozen instructions for the pair.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack_bf16x2(float a, float b)
{
    const bf16x2_t v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}

// 8 bf16 = 4 (even, odd) dim pairs, each turned by the angle whose cos and sin are given (fp32
// arithmetic, every product and sum rounded on its own -- no fused multiply-add, so that the value
// does not depend on the compiler's contraction --, results rounded to bf16, nearest-even):
// ApplyRope of Sec. 4 on a 16-byte piece of a row
__device__ inline uint4 rotate_f32x8(const float (&f)[8], const float4 c, const float4 sn)
{
    const float cc[4] = {c.x, c.y, c.z, c.w}, ss[4] = {sn.x, sn.y, sn.z, sn.w};
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float e = f[2 * i], o = f[2 * i + 1];
        w[i] = pack_bf16x2(__fsub_rn(__fmul_rn(e, cc[i]), __fmul_rn(o, ss[i])),
                           __fadd_rn(__fmul_rn(e, ss[i]), __fmul_rn(o, cc[i])));
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ inline void unpack_bf16x8(const uint4 x, float (&f)[8])
{
    const uint32_t in[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(in[i] << 16);
        f[2 * i + 1] = __uint_as_float(in[i] & 0xffff0000u);
    }
}
__device__ inline uint4 rotate_bf16x8(const uint4 x, const float4 c, const float4 sn)
{
    float f[8];
    unpack_bf16x8(x, f);
    return rotate_f32x8(f, c, sn);
}
// The same rotation kept to twice the mantissa: hi = the rotated values rounded to bf16 (what
// rotate_bf16x8 returns), lo = what the rounding dropped, itself rounded to bf16 (the difference is
// exact in fp32).  A product with hi + lo on one side is the fp32 rotation's to about 2^-17 relative.
__device__ inline void rotate_f32x8_split(const float (&f)[8], const float4 c, const float4 sn, uint4 &hi, uint4 &lo)
{
    const float cc[4] = {c.x, c.y, c.z, c.w}, ss[4] = {sn.x, sn.y, sn.z, sn.w};
    uint32_t wh[4], wl[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float e = f[2 * i], o = f[2 * i + 1];
        const float re = __fsub_rn(__fmul_rn(e, cc[i]), __fmul_rn(o, ss[i]));
        const float ro = __fadd_rn(__fmul_rn(e, ss[i]), __fmul_rn(o, cc[i]));
        wh[i] = pack_bf16x2(re, ro);
        wl[i] = pack_bf16x2(__fsub_rn(re, __uint_as_float(wh[i] << 16)),
                            __fsub_rn(ro, __uint_as_float(wh[i] & 0xffff0000u)));
    }
    hi = make_uint4(wh[0], wh[1], wh[2], wh[3]);
    lo = make_uint4(wl[0], wl[1], wl[2], wl[3]);
}
__device__ inline void rotate_bf16x8_split(const uint4 x, const float4 c, const float4 sn, uint4 &hi, uint4 &lo)
{
    float f[8];
    unpack_bf16x8(x, f);
    rotate_f32x8_split(f, c, sn, hi, lo);
}
__device__ inline uint4 rotate_bf16x8(const uint4 x, const float *cos4, const float *sin4)
{
    return rotate_bf16x8(x, *reinterpret_cast<const float4 *>(cos4), *reinterpret_cast<const float4 *>(sin4));
}

// 8 bf16 (one lane's 16-byte share of a row) dotted with 8 fp32
__device__ inline float dot8(const uint4 &k, const float (&q)[8])
{
    float s = bf16_lo(k.x) * q[0];
    s = fmaf(bf16_hi(k.x), q[1], s);
    s = fmaf(bf16_lo(k.y), q[2], s);
    s = fmaf(bf16_hi(k.y), q[3], s);
    s = fmaf(bf16_lo(k.z), q[4], s);
    s = fmaf(bf16_hi(k.z), q[5], s);
    s = fmaf(bf16_lo(k.w), q[6], s);
    s = fmaf(bf16_hi(k.w), q[7], s);
    return s;
}

// the same with both sides packed bf16: four v_dot2_f32_bf16 (products exact, fp32 sums)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ inline float dot8_bf16(const uint4 &k, const uint4 &q)
{
    float s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.x), __builtin_bit_cast(bf16x2_t, q.x), 0.f, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.y), __builtin_bit_cast(bf16x2_t, q.y), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.z), __builtin_bit_cast(bf16x2_t, q.z), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.w), __builtin_bit_cast(bf16x2_t, q.w), s, false);
    return s;
}

__device__ inline void unpack8(const uint4 &k, float (&f)[8])
{
    f[0] = bf16_lo(k.x); f[1] = bf16_hi(k.x);
    f[2] = bf16_lo(k.y); f[3] = bf16_hi(k.y);
    f[4] = bf16_lo(k.z); f[5] = bf16_hi(k.z);
    f[6] = bf16_lo(k.w); f[7] = bf16_hi(k.w);
}

// ---- FP8 (OCP E4M3) K/V ------------------------------------------------------
// An FP8 row is 128 bytes: 8 bytes per lane of a 16-lane row group.  The hardware
// converter handles two bytes of one 16-bit half of a word at a time; E4M3 values
// are a subset of bf16, so repacking them as bf16 is exact.
struct KvFormat {             // nullptr: bf16 K and V in HBM through strides
    bool fp8;
    float k_scale, v_scale;   // fp8: value = scale * decoded byte (one scale per tensor)
    PagedView paged;          // block_table != nullptr: K and V are page pools
};
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ inline void unpack8_fp8(const uint2 &k, float (&f)[8])
{
    const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8(k.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8(k.x, true);
    const f32x2_t c = __builtin_amdgcn_cvt_pk_f32_fp8(k.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8(k.y, true);
    f[0] = a[0]; f[1] = a[1]; f[2] = b[0]; f[3] = b[1];
    f[4] = c[0]; f[5] = c[1]; f[6] = d[0]; f[7] = d[1];
}
__device__ inline float dot8(const uint2 &k, const float (&q)[8])
{
    float f[8];
    unpack8_fp8(k, f);
    float s = f[0] * q[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) s = fmaf(f[i], q[i], s);
    return s;
}
// 8 E4M3 bytes -> 8 bf16 (exact: E4M3 is a subset of bf16), two values per instruction
// (v_cvt_scalef32_pk_bf16_fp8 with scale 1; the way over fp32 takes two to three times as many)
__device__ inline uint4 fp8x8_to_bf16x8(const uint2 &k)
{
    uint4 r;
    r.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(k.x, 1.0f, false));
    r.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(k.x, 1.0f, true));
    r.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(k.y, 1.0f, false));
    r.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(k.y, 1.0f, true));
    return r;
}
__device__ inline void unpack8(const uint2 &k, float (&f)[8]) { unpack8_fp8(k, f); }
// 8 E4M3 bytes decoded and turned: the rotation takes the decoded fp32 values as they are (widening
// to bf16 first and unpacking again costs a dozen instructions more and, in the chunk-indexed
// pruning kernel, a third of its time)
__device__ inline uint4 rotate_fp8x8(const uint2 &k, const float4 c, const float4 sn)
{
    float f[8];
    unpack8_fp8(k, f);
    return rotate_f32x8(f, c, sn);
}
__device__ inline void rotate_fp8x8_split(const uint2 &k, const float4 c, const float4 sn, uint4 &hi, uint4 &lo)
{
    float f[8];
    unpack8_fp8(k, f);
    rotate_f32x8_split(f, c, sn, hi, lo);
}

// ---- cross-lane -----------------------------------------------------------
template <int CTRL>
__device__ inline float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a DPP row; every lane of the row gets the same
// bits (each step adds a value to its mirror image, and fp add commutes).
__device__ inline float row16_sum(float v)
{
    v += dpp_f32<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f32<0x141>(v);   // row_half_mirror
    v += dpp_f32<0x140>(v);   // row_mirror
    return v;
}

// Maximum over the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48), in every lane.  Two
// in-register row swaps (v_permlane16_swap: odd rows of one copy against even rows of the other;
// v_permlane32_swap: upper half against lower half) instead of two round trips through LDS.
__device__ inline float max_over_rows(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    const unsigned w = __float_as_uint(x);
    const auto s = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    return fmaxf(__uint_as_float(s[0]), __uint_as_float(s[1]));
}

// Reductions and an inclusive scan over the 64 lanes of a wave that stay in the vector registers:
// four DPP steps inside each 16-lane row, then the two row swaps above (reductions) or the three
// row totals read as scalars (scan).  The shuffle-based forms go through the LDS crossbar once per
// step, six dependent steps of ~100 cycles each.
template <int CTRL>
__device__ inline uint32_t dpp_u32(uint32_t v)      // lanes without a source lane read 0
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
template <class Op>
__device__ inline uint32_t wave_reduce_bits(uint32_t v, Op op)      // op: commutative and associative on the bit patterns
{
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true));     // quad_perm [1,0,3,2]
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true));     // quad_perm [2,3,0,1]
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true));    // row_half_mirror
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, true));    // row_mirror
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = op(r[0], r[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return op(q[0], q[1]);
}
__device__ inline float wave_max_f32(float x)
{
    return __uint_as_float(wave_reduce_bits(__float_as_uint(x), [](uint32_t a, uint32_t b) {
        return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b)));
    }));
}
__device__ inline float wave_min_f32(float x)
{
    return __uint_as_float(wave_reduce_bits(__float_as_uint(x), [](uint32_t a, uint32_t b) {
        return __float_as_uint(fminf(__uint_as_float(a), __uint_as_float(b)));
    }));
}
__device__ inline uint32_t wave_sum_u32(uint32_t x)
{
    return wave_reduce_bits(x, [](uint32_t a, uint32_t b) { return a + b; });
}
// inclusive prefix sum over the wave's lanes
__device__ inline uint32_t wave_scan_u32(uint32_t v, int lane)
{
    v += dpp_u32<0x111>(v);      // row_shr:1
    v += dpp_u32<0x112>(v);      // row_shr:2
    v += dpp_u32<0x114>(v);      // row_shr:4
    v += dpp_u32<0x118>(v);      // row_shr:8
    const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
    const uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
    const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
    return v + (lane >= 16 ? t0 : 0u) + (lane >= 32 ? t1 : 0u) + (lane >= 48 ? t2 : 0u);
}

__device__ inline int ilog2(int x) { return 31 - __builtin_clz(x); }

// 16-byte row fragment load for lane l16 of a row group
__device__ inline uint4 load_row16(const uint16_t *base, int64_t row_elem_offset, int l16)
{
    return *reinterpret_cast<const uint4 *>(base + row_elem_offset + l16 * 8);
}

}  // namespace ihip
