// Shared by the two block-sparse prefill attention kernels.
#pragma once

#include "common.h"

namespace ihip {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPfTile = 32;             // key slots per step
constexpr int kPfKStride = kD + 8;      // K tile row stride in LDS (elements): 272 B, conflict-free 16-B reads
constexpr int kPfVStride = kPfTile + 8; // V^T row stride (elements): 80 B
constexpr float kNegBigPf = -1.0e30f;

struct AttnPrefillArgs {
    Geometry ge;
    const uint16_t *q; int64_t q_sb, q_sh, q_st;
    const uint16_t *k; int64_t k_sb, k_sh, k_st;
    const uint16_t *v; int64_t v_sb, v_sh, v_st;
    const int32_t *block_starts;
    int n_blocks, block, block_log2;
    float scale_log2e;
    uint16_t *out;       // bf16 [B, Hq, Tq, d]
    float *out_lse;      // [B, Hq, Tq] or null
    const float *rope_cos, *rope_sin;   // streaming-style RoPE instantiations only: fp32 [n_pos][d/2]
    PagedView paged;                    // paged instantiations only: k / v are the page pools, k_sb / v_sb
                                        // the page strides
    float v_scale;                      // E4M3 instantiations only (K, V strides then count 2-byte units)
};

// Streaming-style positions (Sec. 4 "Dynamic RoPE for OOL generalization"): the keys a query
// attends to, in position order, sit at 0, 1, ..., n-1 and the query at n-1.  Attended slots are a
// prefix of the block part of the slot list (blocks are ascending, empty ones last, only the last
// one can be cut short), so a key's id is its slot, less the empty block slots for window keys;
// n_stream >= b_q keeps every block key before every query of the block, so the id does not depend
// on the query.
struct StreamIds {
    int n_sink_eff, block_slots, block_tokens, w0;
    __device__ int key(int slot) const
    {
        return slot < n_sink_eff + block_slots ? slot : slot - (block_slots - block_tokens);
    }
    __device__ int query(int n_sink, int qpos) const      // = (number of keys the query attends to) - 1
    {
        return min(n_sink, qpos + 1) + block_tokens + max(0, qpos - w0 + 1) - 1;
    }
};

// tokens in the kept blocks of problem p; every thread of the workgroup calls it (uses *sh, barriers)
__device__ inline int pf_block_tokens(const AttnPrefillArgs &a, const Problem &pr, int p, int nthreads, int *sh)
{
    if (threadIdx.x == 0) *sh = 0;
    __syncthreads();
    int mine = 0;
    for (int i = threadIdx.x; i < a.n_blocks; i += nthreads) {
        const int bs = a.block_starts[(int64_t)p * a.n_blocks + i];
        if (bs >= 0 && bs < pr.hi) mine += min(a.block, pr.hi - bs);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
    if ((threadIdx.x & 63) == 0 && mine > 0) atomicAdd(sh, mine);
    __syncthreads();
    return *sh;
}

__device__ inline int pf_slot_to_pos(const AttnPrefillArgs &a, const Problem &pr, int p, int slot,
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

// LDS of the 32x32 kernel: K/V stages of 16 KB (32 rows of 256 bytes each), for E4M3 also raw stages of
// 8 KB; then an int per key slot (two with paged K/V: the page id) and a flag per tile.  The most key
// slots a kernel can take follow from the 160 KB of a CU (64 bytes are left for static variables).
constexpr int kPfStagesPlain = 3, kPfStagesRope = 4, kPfStagesFp8 = 3;
constexpr int kPfRawStages = 3;                     // E4M3: raw stages of one K or V tile's size
constexpr int kPfTileEl = kPfTile * kD;             // elements of one K (or V) tile: 32 rows of 256 bytes
constexpr int kPfStageEl = 2 * kPfTileEl;           // K tile, then V tile
constexpr int kPf32MaxLds = 160 * 1024;             // LDS per workgroup the 32x32 kernel may ask for
constexpr int pf32_max_slots(int stage_bytes, int ints_per_slot)
{
    // slots * 4 * ints_per_slot + slots / 32 <= room, slots a multiple of the tile
    return (int)((int64_t)(kPf32MaxLds - 64 - stage_bytes) * kPfTile / (4 * ints_per_slot * kPfTile + 1)) / kPfTile * kPfTile;
}
constexpr int kPfStageBytes = kPfStageEl * 2, kPfRawBytes = kPfTileEl * 2;
constexpr int kPfFp8StageBytes = kPfStagesFp8 * kPfStageBytes + kPfRawStages * kPfRawBytes;
constexpr int kPf32MaxSlots = pf32_max_slots(kPfStagesPlain * kPfStageBytes, 1);            // 28,416
constexpr int kPf32MaxSlotsRope = pf32_max_slots(kPfStagesRope * kPfStageBytes, 1);         // 24,352
constexpr int kPf32MaxSlotsPaged = pf32_max_slots(kPfStagesPlain * kPfStageBytes, 2);       // 14,272: a page id per slot as well
constexpr int kPf32MaxSlotsRopePaged = pf32_max_slots(kPfStagesRope * kPfStageBytes, 2);
constexpr int kPf32MaxSlotsFp8 = pf32_max_slots(kPfFp8StageBytes, 1);                      // E4M3, with or without RoPE
constexpr int kPf32MaxSlotsFp8Paged = pf32_max_slots(kPfFp8StageBytes, 2);
static_assert(kPf32MaxSlots * 4 + kPf32MaxSlots / kPfTile + kPfStagesPlain * kPfStageBytes + 64 <= kPf32MaxLds, "LDS");
static_assert(kPf32MaxSlotsFp8Paged * 8 + kPf32MaxSlotsFp8Paged / kPfTile + kPfFp8StageBytes + 64 <= kPf32MaxLds, "LDS");

void launch_attn_prefill32(const AttnPrefillArgs &a, int P, int64_t max_seq_len, hipStream_t st);
void launch_attn_prefill32_fp8(const AttnPrefillArgs &a, int P, hipStream_t st);   // E4M3 K and V


}  // namespace ihip
