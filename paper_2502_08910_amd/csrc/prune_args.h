// Arguments of the pruning-stage kernels (Alg. 2 / Alg. 3), shared by the plain and the
// dynamic-RoPE translation units.
#pragma once

#include "common.h"

namespace ihip {

// Rotary table handed in by the caller: cos and sin of (position x angle of frequency j),
// fp32 [n_pos][d/2].
struct RopeView {
    const float *cos, *sin;
    int n_pos;
};

struct PruneArgs {
    Geometry ge;
    const uint16_t *q; int64_t q_sb, q_sh, q_st;
    const uint16_t *k; int64_t k_sb, k_sh, k_st;
    const int32_t *parent_starts;
    int n_parent, ratio_log2, chunk, max_chunks;
    float *out_scores;
    int32_t *out_rep;
    BankView bank;            // used by the cached instantiations only (K then points to host memory)
    PagedView paged;          // paged instantiations only: K is the page pool, k_sb the page stride
    float k_scale;            // FP8 instantiations only: the scores are multiplied by it (K strides then
                              // count 2-byte units of the byte rows)
};

// Chunk-indexed RoPE needs the number of chunks this stage really has for problem p (valid slots are
// a prefix of the slot list: parents are ascending with the empty ones last, and only the last chunk
// before the end of the middle range can be cut short).  Every thread of the workgroup calls it
// (uses *sh and barriers).
__device__ inline int stage_n_chunk(const PruneArgs &a, const Problem &pr, int p, int nthreads, int *sh)
{
    if (a.parent_starts == nullptr) return max(0, (pr.hi - pr.lo + a.chunk - 1) / a.chunk);
    if (threadIdx.x == 0) *sh = 0;
    __syncthreads();
    const int32_t *ps = a.parent_starts + (int64_t)p * a.n_parent;
    const int parent_chunk = a.chunk << a.ratio_log2;
    for (int i = threadIdx.x; i < a.n_parent; i += nthreads) {
        const int s0 = ps[i];
        const bool here = s0 >= 0 && s0 < pr.hi;
        const int s1 = i + 1 < a.n_parent ? ps[i + 1] : -1;
        if (here && !(s1 >= 0 && s1 < pr.hi))       // the last parent that holds keys
            *sh = (i << a.ratio_log2) + (min(parent_chunk, pr.hi - s0) + a.chunk - 1) / a.chunk;
    }
    __syncthreads();
    return *sh;
}

// SRC 0: K in HBM through strides; 1: host tier with the on-GPU bank; 2: paged pool
template <int SRC> struct KeySource;
template <> struct KeySource<0> {
    typedef DirectRows type;
    static __device__ type make(const PruneArgs &a, const Problem &pr)
    {
        return DirectRows{a.k + pr.b * a.k_sb + pr.g * a.k_sh, a.k_st};
    }
};
template <> struct KeySource<1> {
    typedef CachedRows type;
    static __device__ type make(const PruneArgs &a, const Problem &pr)
    {
        return cached_rows(a.bank, a.k, a.k_sb, a.k_sh, a.k_st, a.bank.bank_k, pr.b, pr.g, a.ge.Hkv);
    }
};

template <> struct KeySource<2> {
    typedef PagedRows type;
    static __device__ type make(const PruneArgs &a, const Problem &pr)
    {
        return PagedRows{a.k + pr.g * a.k_sh, a.paged.block_table + (int64_t)pr.b * a.paged.table_stride, a.k_sb,
                         a.k_st, a.paged.page_log2};
    }
};

}  // namespace ihip
