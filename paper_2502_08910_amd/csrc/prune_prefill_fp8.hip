// Pruning-stage scoring for chunked prefill over E4M3 keys: the instantiations of the prefill kernel
// that repack 8-bit rows on their way into LDS (a translation unit of their own, so that the two
// sets of instantiations compile side by side).  64-bit row offsets throughout.
#include "prune_prefill.h"

namespace ihip {

template <int MT>
static void launch_fp8(const PruneArgs &a, int P, const RopeView *rope, int style, hipStream_t st)
{
    const RopeView none{nullptr, nullptr, 0};
    if (a.paged.block_table) {
        if (rope && style == 2) launch_prefill_w<MT, true, 2, true, true>(a, P, *rope, st);
        else if (rope) launch_prefill_w<MT, true, 1, true, true>(a, P, *rope, st);
        else launch_prefill_w<MT, true, 0, true, true>(a, P, none, st);
    } else {
        if (rope && style == 2) launch_prefill_w<MT, true, 2, false, true>(a, P, *rope, st);
        else if (rope) launch_prefill_w<MT, true, 1, false, true>(a, P, *rope, st);
        else launch_prefill_w<MT, true, 0, false, true>(a, P, none, st);
    }
}

// b_q in {16, 32, 64} (checked by the caller); K strides of `a` count 2-byte units
void launch_prune_prefill_fp8(const PruneArgs &a, int P, int b_q, const RopeView *rope, int style, hipStream_t st)
{
    switch (b_q) {
    case 16: launch_fp8<1>(a, P, rope, style, st); break;
    case 32: launch_fp8<2>(a, P, rope, style, st); break;
    default: launch_fp8<4>(a, P, rope, style, st); break;
    }
}

}  // namespace ihip
