// Block-sparse chunked-prefill attention on v_mfma_f32_32x32x16_bf16 over E4M3 K and V: the
// instantiations that widen raw 8-bit tiles in LDS (a translation unit of their own, so that the two
// sets of instantiations compile side by side).  64-bit row offsets throughout.
#include "attn_prefill32.h"

namespace ihip {

// K / V strides of `a` count 2-byte units; a.v_scale and the K scale (inside a.scale_log2e) are set.
// The caller keeps n_sink + n_blocks * block + n_stream within kPf32MaxSlotsFp8 (paged: ...Fp8Paged).
void launch_attn_prefill32_fp8(const AttnPrefillArgs &a, int P, hipStream_t st)
{
    const int NQ = a.ge.b_q / 32;
    const int heads_per_wg = NQ * a.ge.G > 8 ? a.ge.G / 2 : a.ge.G;
    const int parts = a.ge.G / heads_per_wg;
    const dim3 block_dim(64 * NQ * heads_per_wg), grid(parts == 1 ? P : (P + 7) / 8 * 8 * parts);
    const int slots = (a.ge.n_sink + a.n_blocks * a.block + a.ge.n_stream + kPfTile - 1) / kPfTile * kPfTile;
    const bool use_rope = a.rope_cos != nullptr, paged = a.paged.block_table != nullptr;
    const size_t lds = (size_t)(kPfStagesFp8 * kPfStageEl + kPfRawStages * kPfTileEl) * sizeof(uint16_t) +
                       (size_t)slots * sizeof(int) * (paged ? 2 : 1) + slots / kPfTile;
#define IHIP_PF32_R(NQV, GV, RV, PV)                                                                         \
    {                                                                                                        \
        static bool attr_set = false;     /* allow more than 64 KiB of dynamic LDS, once per kernel */       \
        if (!attr_set) {                                                                                     \
            (void)hipFuncSetAttribute(                                                                       \
                reinterpret_cast<const void *>(&attn_prefill32_kernel<NQV, GV, true, RV, PV, true>),         \
                hipFuncAttributeMaxDynamicSharedMemorySize, kPf32MaxLds - (RV ? 64 : 0));                    \
            attr_set = true;                                                                                 \
        }                                                                                                    \
        hipLaunchKernelGGL((attn_prefill32_kernel<NQV, GV, true, RV, PV, true>), grid, block_dim, lds, st, a); \
    }
#define IHIP_PF32(NQV, GV)                                                                                   \
    if (paged) {                                                                                             \
        if (use_rope) IHIP_PF32_R(NQV, GV, true, true) else IHIP_PF32_R(NQV, GV, false, true)                \
    } else if (use_rope) IHIP_PF32_R(NQV, GV, true, false) else IHIP_PF32_R(NQV, GV, false, false)
    // at most 8 waves: a workgroup of 64-query blocks has at most 4 heads
    if (NQ == 1) {
        switch (heads_per_wg) {
        case 1: IHIP_PF32(1, 1); break;
        case 2: IHIP_PF32(1, 2); break;
        case 4: IHIP_PF32(1, 4); break;
        default: IHIP_PF32(1, 8); break;
        }
    } else {
        switch (heads_per_wg) {
        case 1: IHIP_PF32(2, 1); break;
        case 2: IHIP_PF32(2, 2); break;
        default: IHIP_PF32(2, 4); break;
        }
    }
#undef IHIP_PF32
#undef IHIP_PF32_R
}

}  // namespace ihip
