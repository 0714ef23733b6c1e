// Block-sparse chunked-prefill attention on v_mfma_f32_32x32x16_bf16: the bf16 instantiations and
// their launcher (the kernel template is in attn_prefill32.h).
#include "attn_prefill32.h"

namespace ihip {

void launch_attn_prefill32(const AttnPrefillArgs &a, int P, int64_t max_seq_len, hipStream_t st)
{
    const int NQ = a.ge.b_q / 32;
    const int heads_per_wg = NQ * a.ge.G > 8 ? a.ge.G / 2 : a.ge.G;
    const int parts = a.ge.G / heads_per_wg;
    const dim3 block_dim(64 * NQ * heads_per_wg), grid(parts == 1 ? P : (P + 7) / 8 * 8 * parts);
    const int slots = (a.ge.n_sink + a.n_blocks * a.block + a.ge.n_stream + kPfTile - 1) / kPfTile * kPfTile;
    const bool use_rope = a.rope_cos != nullptr, paged = a.paged.block_table != nullptr;
    const size_t lds = (size_t)(use_rope ? kPfStagesRope : kPfStagesPlain) * kPfStageEl * sizeof(uint16_t) +
                       (size_t)slots * sizeof(int) * (paged ? 2 : 1) + slots / kPfTile;   // stages, slot positions (and pages), per-tile flags
    const int64_t lim = (int64_t)1 << 31, lim24 = (int64_t)1 << 24;
    const bool wide = paged || max_seq_len >= lim24 || a.k_st < 0 || a.v_st < 0 || a.k_st >= lim24 || a.v_st >= lim24 ||
                      max_seq_len * a.k_st + kD >= lim || max_seq_len * a.v_st + kD >= lim;
#define IHIP_PF32_R(NQV, GV, WV, RV, PV)                                                                     \
    {                                                                                                        \
        static bool attr_set = false;     /* allow more than 64 KiB of dynamic LDS, once per kernel */       \
        if (!attr_set) {                                                                                     \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_prefill32_kernel<NQV, GV, WV, RV, PV>), \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kPf32MaxLds - (RV ? 64 : 0)); \
            attr_set = true;                                                                                 \
        }                                                                                                    \
        hipLaunchKernelGGL((attn_prefill32_kernel<NQV, GV, WV, RV, PV>), grid, block_dim, lds, st, a);      \
    }
#define IHIP_PF32(NQV, GV, WV)                                                                               \
    if (WV && paged) {                                                                                       \
        if (use_rope) IHIP_PF32_R(NQV, GV, true, true, true) else IHIP_PF32_R(NQV, GV, true, false, true)    \
    } else if (use_rope) IHIP_PF32_R(NQV, GV, WV, true, false) else IHIP_PF32_R(NQV, GV, WV, false, false)
#define IHIP_PF32_BY_G(NQV, WV)             \
    switch (heads_per_wg) {                 \
    case 1: IHIP_PF32(NQV, 1, WV); break;   \
    case 2: IHIP_PF32(NQV, 2, WV); break;   \
    case 4: IHIP_PF32(NQV, 4, WV); break;   \
    default: IHIP_PF32(NQV, 8, WV); break;  \
    }
    if (wide) {
        if (NQ == 1) { IHIP_PF32_BY_G(1, true) } else { IHIP_PF32_BY_G(2, true) }
    } else {
        if (NQ == 1) { IHIP_PF32_BY_G(1, false) } else { IHIP_PF32_BY_G(2, false) }
    }
#undef IHIP_PF32_BY_G
#undef IHIP_PF32
#undef IHIP_PF32_R
}

}  // namespace ihip
