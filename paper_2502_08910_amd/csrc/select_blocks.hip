// arg-top-K of the chunk scores (Alg. 2) -- one workgroup per problem.
//
// Scores become order-preserving 32-bit keys (held in LDS when they fit); the
// workgroup-wide radix select of block_select.h keeps the K best under the
// order (score descending, slot ascending) and emits them in ascending slot
// order, i.e. ascending position.
#include "block_select.h"

namespace ihip {

constexpr int kSelThreads = 256;
constexpr int kSelLdsKeys = 12288;     // keys cached in LDS (48 KiB); larger inputs re-read global memory

struct SelectArgs {
    Geometry ge;
    const float *scores;
    int max_chunks;
    const int32_t *parent_starts;
    int n_parent, ratio_log2, chunk, keep;
    int32_t *out_starts;
};

// Monotone map fp32 -> u32 (larger float <=> larger key); -0.0 maps with +0.0.
__device__ inline uint32_t order_key(float f)
{
    const uint32_t u = __float_as_uint(f + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
constexpr uint32_t kKeyNegInf = 0x007fffffu;   // order_key(-inf): empty slot

__global__ __launch_bounds__(kSelThreads) void select_blocks_kernel(const SelectArgs a)
{
    __shared__ uint32_t keys[kSelLdsKeys];
    __shared__ SelectScratch<kSelThreads> scratch;
    __shared__ uint32_t sh_valid;

    const int p = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = a.max_chunks;
    const float *sc = a.scores + (int64_t)p * n;
    const bool cached = n <= kSelLdsKeys;

    // load keys, count non-empty slots
    uint32_t my_valid = 0;
    for (int i = tid; i < n; i += kSelThreads) {
        const uint32_t kk = order_key(sc[i]);
        if (cached) keys[i] = kk;
        my_valid += kk != kKeyNegInf;
    }
    if (tid == 0) sh_valid = 0;
    __syncthreads();
    {
        uint32_t v = my_valid;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
        if (lane == 0) atomicAdd(&sh_valid, v);
    }
    __syncthreads();
    const int keep_eff = min((int)sh_valid, a.keep);
    int32_t *out = a.out_starts + (int64_t)p * a.keep;

    if (keep_eff > 0) {
        const Problem pr = problem_of(a.ge, p);
        block_select_largest<kSelThreads>(
            n, keep_eff,
            [&](int i) -> uint32_t { return cached ? keys[i] : order_key(sc[i]); },
            [&](uint32_t rank, int i) {
                out[rank] = slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, i);
            },
            scratch);
    }
    for (int i = keep_eff + tid; i < a.keep; i += kSelThreads) out[i] = -1;
}

int32_t launch_select_blocks(const ihip_shape &s, const float *scores, int max_chunks,
                             const int32_t *parent_starts, int n_parent, int parent_chunk, int chunk,
                             int keep, int32_t *out_starts, hipStream_t st)
{
    SelectArgs a;
    a.ge = make_geometry(s);
    a.scores = scores;
    a.max_chunks = max_chunks;
    a.parent_starts = parent_starts;
    a.n_parent = n_parent;
    a.ratio_log2 = parent_starts ? __builtin_ctz(parent_chunk / chunk) : 0;
    a.chunk = chunk;
    a.keep = keep;
    a.out_starts = out_starts;
    const int P = s.B * s.Hkv * (s.Tq / s.b_q);
    if (P == 0 || keep == 0) return IHIP_OK;
    KernelTimer timer(stage_name(kNameSelect, parent_starts == nullptr, chunk), st);
    hipLaunchKernelGGL(select_blocks_kernel, dim3(P), dim3(kSelThreads), 0, st, a);
    return check_launch("select_blocks");
}

}  // namespace ihip
