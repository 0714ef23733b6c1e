// Block-sparse chunked-prefill attention on v_mfma_f32_32x32x16_bf16.
//
// One workgroup per problem (sequence, KV head, query block); one wave per
// (query head of the group, 32 queries of the block), i.e. G * b_q/32 waves
// (8 for Llama-shaped GQA with b_q = 64), two per SIMD, so that one wave's
// softmax arithmetic overlaps the other's matrix work.  The gathered K/V tile
// (32 key slots) is staged in LDS once and shared by all waves.
//
// Same "transposed" scheme as the 16x16 kernel:  S^T = K Q^T,  O^T = V^T P^T.
// Layouts: A/B lane l holds 8 consecutive k (group half = l/32) of row/column
// n = l%32; C lane l holds column n, element r = row 8*(r/4) + 4*half + r%4.
// A lane's 16 S^T values are keys {8*(r/4) + 4*half + r%4}; taken 8 at a time
// (r < 8: keys 0..15, r >= 8: keys 16..31) they are the B operand of the second
// product, and V^T is laid out in LDS to match: k slot half*8 + j of step kk is
// key 16*kk + 8*(j/4) + 4*half + j%4.
//
// Latency hiding.  The position of every key slot is computed once into LDS
// (so the steady state has no dependent global loads); K/V rows travel
// global -> registers -> LDS with two register buffers and three LDS stages:
// the rows of tile t+4 are requested while tile t is being multiplied, and
// there is one barrier per tile.  Inside a wave the first product of tile t+1
// is issued before the softmax arithmetic of tile t, so the matrix pipe works
// while the vector pipe does exponentials.  V^T granules (8 keys = 16 B) are
// XOR-swizzled by the row's dim group so the transposing stores spread over
// the LDS banks.
#include "attn_prefill_args.h"

namespace ihip {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kPfStageK = kPfTile * kPfKStride;    // elements per LDS stage
constexpr int kPfStageV = kD * kPfVStride;

template <int NQ, int G>   // NQ = b_q / 32 query tiles, G query heads: NQ*G waves
__global__ __launch_bounds__(64 * NQ * G) void attn_prefill32_kernel(const AttnPrefillArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *sK = smem;                                   // 3 stages
    uint16_t *sVt = smem + 3 * kPfStageK;                  // 3 stages
    int *sPos = reinterpret_cast<int *>(smem + 3 * (kPfStageK + kPfStageV));   // one int per key slot

    const int p = blockIdx.x;
    const Problem pr = problem_of(a.ge, p);
    constexpr int nthreads = 64 * NQ * G;
    constexpr int b_q = 32 * NQ;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int hh = wave % G, qt = wave / G;          // this wave's head and query tile
    const int n = lane & 31, half = lane >> 5;
    const int h = pr.g * G + hh;
    const int q0 = pr.m * b_q + qt * 32;             // first query row of this wave
    const int qpos0 = pr.E - b_q;                    // absolute position of the block's first query
    const int qpos = qpos0 + qt * 32 + n;            // ... of this lane's query

    const int n_sink_eff = min(a.ge.n_sink, pr.E);
    const int w0 = max(pr.hi, a.ge.n_sink);
    const int total = n_sink_eff + (a.n_blocks << a.block_log2) + max(0, pr.E - w0);
    const int n_tiles = (total + kPfTile - 1) / kPfTile;     // host guarantees n_tiles*32 <= kPf32MaxSlots

    for (int slot = tid; slot < n_tiles * kPfTile; slot += nthreads)
        sPos[slot] = slot < total ? pf_slot_to_pos(a, pr, p, slot, n_sink_eff, w0) : -1;

    bf16x8 qb[8];
    {
        const uint16_t *qp = a.q + pr.b * a.q_sb + (int64_t)h * a.q_sh + (int64_t)(q0 + n) * a.q_st + half * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qb[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
    }
    const uint16_t *kb = a.k + pr.b * a.k_sb + pr.g * a.k_sh;
    const uint16_t *vb = a.v + pr.b * a.v_sb + pr.g * a.v_sh;

    f32x16 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m_run = kNegBigPf, l_run = 0.f;

    // loader roles.  K: item = (key, dim group c), 32 x 16 = 512 sixteen-byte pieces.
    // V: item = (key pair, dim group c), 16 x 16 = 256 pairs of pieces (a pair packs into 32-bit V^T stores).
    constexpr int kItemsK = kPfTile * 16, kItemsV = (kPfTile / 2) * 16;
    constexpr int kPerK = (kItemsK + nthreads - 1) / nthreads, kPerV = (kItemsV + nthreads - 1) / nthreads;
    struct RowBuf { uint4 k[kPerK], v[kPerV][2]; };
    RowBuf bufA, bufB;

    auto fetch = [&](RowBuf &buf, int tile) {
        if (tile >= n_tiles) return;
#pragma unroll
        for (int r = 0; r < kPerK; ++r) {
            const int item = tid + r * nthreads;
            if (item >= kItemsK) break;
            const int pos = sPos[tile * kPfTile + (item >> 4)];
            buf.k[r] = make_uint4(0, 0, 0, 0);
            if (pos >= 0) buf.k[r] = *reinterpret_cast<const uint4 *>(kb + (int64_t)pos * a.k_st + (item & 15) * 8);
        }
#pragma unroll
        for (int r = 0; r < kPerV; ++r) {
            const int item = tid + r * nthreads;
            if (item >= kItemsV) break;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int pos = sPos[tile * kPfTile + (item >> 4) * 2 + e];
                buf.v[r][e] = make_uint4(0, 0, 0, 0);
                if (pos >= 0) buf.v[r][e] = *reinterpret_cast<const uint4 *>(vb + (int64_t)pos * a.v_st + (item & 15) * 8);
            }
        }
    };
    auto stash = [&](const RowBuf &buf, int tile) {
        if (tile >= n_tiles) return;
        uint16_t *dK = sK + (tile % 3) * kPfStageK;
        uint16_t *dV = sVt + (tile % 3) * kPfStageV;
#pragma unroll
        for (int r = 0; r < kPerK; ++r) {
            const int item = tid + r * nthreads;
            if (item >= kItemsK) break;
            *reinterpret_cast<uint4 *>(&dK[(item >> 4) * kPfKStride + (item & 15) * 8]) = buf.k[r];
        }
#pragma unroll
        for (int r = 0; r < kPerV; ++r) {
            const int item = tid + r * nthreads;
            if (item >= kItemsV) break;
            const int key0 = (item >> 4) * 2, c = item & 15;
            // position of key kappa in a V^T row: 16*(kappa/16) + 8*half + j,
            // half = (kappa%8)/4, j = 4*((kappa%16)/8) + kappa%4
            const int k16 = key0 & 15;
            int vslot = (key0 & 16) + ((k16 & 7) >> 2) * 8 + (k16 >> 3) * 4 + (k16 & 3);   // even
            vslot ^= ((c >> 1) & 3) << 3;                     // granule swizzle by dim group
            const uint32_t v0[4] = {buf.v[r][0].x, buf.v[r][0].y, buf.v[r][0].z, buf.v[r][0].w};
            const uint32_t v1[4] = {buf.v[r][1].x, buf.v[r][1].y, buf.v[r][1].z, buf.v[r][1].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = (v0[i] & 0xffffu) | (v1[i] << 16);            // dim c*8+2i of both keys
                const uint32_t hi = (v0[i] >> 16) | (v1[i] & 0xffff0000u);        // dim c*8+2i+1
                *reinterpret_cast<uint32_t *>(&dV[(c * 8 + 2 * i) * kPfVStride + vslot]) = lo;
                *reinterpret_cast<uint32_t *>(&dV[(c * 8 + 2 * i + 1) * kPfVStride + vslot]) = hi;
            }
        }
    };

    // first product of a tile: S^T = K Q^T for this wave's 32 queries
    auto scores = [&](int tile) -> f32x16 {
        const uint16_t *cK = sK + (tile % 3) * kPfStageK;
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(&cK[n * kPfKStride + ks * 16 + half * 8]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[ks], s, 0, 0, 0);
        }
        return s;
    };
    // softmax update and second product of a tile
    auto finish = [&](int tile, f32x16 s) {
        const uint16_t *cV = sVt + (tile % 3) * kPfStageV;
        // a tile needs masking if it has an empty slot or a key at or after the block's first query
        const int myp = sPos[tile * kPfTile + n];
        if (__any(myp < 0 || myp >= qpos0)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kp = sPos[tile * kPfTile + 8 * (r >> 2) + 4 * half + (r & 3)];
                if (kp < 0 || kp > qpos) s[r] = -INFINITY;
            }
        }
        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float mn = fmaxf(m_run, mx * a.scale_log2e);       // running max in scaled (log2) units
        const float corr = __builtin_amdgcn_exp2f(m_run - mn);
        m_run = mn;
        float ps = 0.f;
        bf16x8 pb[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float pw = __builtin_amdgcn_exp2f(fmaf(s[r], a.scale_log2e, -mn));   // exp2(-inf) = 0
            ps += pw;
            pb[r >> 3][r & 7] = (__bf16)pw;
        }
        l_run = l_run * corr + ps;                                // partial over this lane's keys
        if (__any(corr != 1.0f)) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) o[dt] *= corr;
        }
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const int row = dt * 32 + n;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int g = (kk * 2 + half) ^ ((row >> 4) & 3);     // swizzled 16-byte granule
                const bf16x8 va = *reinterpret_cast<const bf16x8 *>(&cV[row * kPfVStride + g * 8]);
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[kk], o[dt], 0, 0, 0);
            }
        }
    };

    __syncthreads();                        // sPos complete
    fetch(bufA, 0);
    fetch(bufB, 1);
    stash(bufA, 0);
    stash(bufB, 1);
    fetch(bufA, 2);
    fetch(bufB, 3);
    __syncthreads();
    f32x16 s_cur = scores(0);
    // At the top of iteration t: stage t%3 holds tile t, stage (t+1)%3 tile t+1 (visible after the
    // barrier), the buffer of t's parity holds tile t+2 and the other one tile t+3.
    for (int tile = 0; tile < n_tiles; tile += 2) {
        __syncthreads();
        f32x16 s_next = s_cur;
        if (tile + 1 < n_tiles) s_next = scores(tile + 1);
        finish(tile, s_cur);
        stash(bufA, tile + 2);              // stage (tile+2)%3 was last read for tile-1: everyone is past it
        fetch(bufA, tile + 4);
        if (tile + 1 >= n_tiles) break;
        __syncthreads();
        if (tile + 2 < n_tiles) s_cur = scores(tile + 2);
        finish(tile + 1, s_next);
        stash(bufB, tile + 3);
        fetch(bufB, tile + 5);
    }

    float l = l_run;
    l += __shfl_xor(l, 32, 64);
    const float inv = 1.0f / l;
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

void launch_attn_prefill32(const AttnPrefillArgs &a, int P, hipStream_t st)
{
    const int NQ = a.ge.b_q / 32;
    const dim3 block_dim(64 * NQ * a.ge.G), grid(P);
    const int slots = (a.ge.n_sink + a.n_blocks * a.block + a.ge.n_stream + kPfTile - 1) / kPfTile * kPfTile;
    const size_t lds = 3 * (kPfStageK + kPfStageV) * sizeof(uint16_t) + (size_t)slots * sizeof(int);
#define IHIP_PF32(NQV, GV)                                                                               \
    {                                                                                                    \
        static bool attr_set = false;     /* allow more than 64 KiB of dynamic LDS, once per kernel */   \
        if (!attr_set) {                                                                                 \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_prefill32_kernel<NQV, GV>),  \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kPf32MaxLds);         \
            attr_set = true;                                                                             \
        }                                                                                                \
        hipLaunchKernelGGL((attn_prefill32_kernel<NQV, GV>), grid, block_dim, lds, st, a);              \
    }
#define IHIP_PF32_BY_G(NQV)             \
    switch (a.ge.G) {                   \
    case 1: IHIP_PF32(NQV, 1); break;   \
    case 2: IHIP_PF32(NQV, 2); break;   \
    case 4: IHIP_PF32(NQV, 4); break;   \
    default: IHIP_PF32(NQV, 8); break;  \
    }
    if (NQ == 1) { IHIP_PF32_BY_G(1) } else { IHIP_PF32_BY_G(2) }
#undef IHIP_PF32_BY_G
#undef IHIP_PF32
}

}  // namespace ihip
