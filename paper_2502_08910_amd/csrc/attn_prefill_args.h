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
};

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

constexpr int kPf32MaxLds = 160 * 1024;  // LDS per workgroup the 32x32 kernel may ask for
constexpr int kPf32MaxSlots = 24320;    // key slots whose positions (and per-tile flags) the 32x32 kernel keeps in LDS

void launch_attn_prefill32(const AttnPrefillArgs &a, int P, int64_t max_seq_len, hipStream_t st);

}  // namespace ihip
