// arg-top-K of the chunk scores (Alg. 2) -- one workgroup per problem.
//
// Scores become order-preserving 32-bit keys (held in LDS when they fit); the
// workgroup-wide radix select of block_select.h keeps the K best under the
// order (score descending, slot ascending) and emits them in ascending slot
// order, i.e. ascending position.
#include "select_fast.h"

namespace ihip {

constexpr int kSelThreads = 256;
constexpr int kSelLdsKeys = 12288;     // keys cached in LDS (48 KiB); larger inputs re-read global memory

__global__ __launch_bounds__(kSelThreads) void select_blocks_kernel(const SelectArgs a)
{
    __shared__ uint32_t keys[kSelLdsKeys];
    __shared__ SelectScratch<kSelThreads> scratch;
    __shared__ uint32_t sh_valid;

    const SelView view(a, blockIdx.x);
    const int p = view.p;
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = a.max_chunks;
    const bool cached = n <= kSelLdsKeys;

    // load keys, count non-empty slots
    uint32_t my_valid = 0;
    for (int i = tid; i < n; i += kSelThreads) {
        const uint32_t kk = order_key(view.score(i));
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

    if (keep_eff > 0) {
        const Problem pr = problem_of(a.ge, p);
        block_select_largest<kSelThreads>(
            n, keep_eff,
            [&](int i) -> uint32_t { return cached ? keys[i] : order_key(view.score(i)); },
            [&](uint32_t rank, int i) {
                view.put(rank, slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, i));
            },
            scratch);
    }
    for (int i = keep_eff + tid; i < a.keep; i += kSelThreads) view.put(i, -1);
}

// Fast path for up to 16 slots per thread (select_fast.h), in the smallest shape that holds the slots.
template <int NT, int ITEMS>
__global__ __launch_bounds__(NT) void select_blocks_fast_kernel(const SelectArgs a)
{
    __shared__ SelectFastShared<NT> sh;
    select_blocks_fast<NT, ITEMS>(a, blockIdx.x, sh);
}

// Alg. 1 "subdivide query blocks for the next stage": row p of dst (one per block of b_q / ratio
// queries) is a copy of the row of the coarse block that holds it.
__global__ __launch_bounds__(256) void subdivide_blocks_kernel(const int32_t *src, int32_t *dst, int n, int Mq_fine,
                                                              int ratio)
{
    const int pf = blockIdx.x;                       // (sequence, KV head, fine block)
    const int bg = pf / Mq_fine, m = pf % Mq_fine;
    const int32_t *from = src + ((int64_t)bg * (Mq_fine / ratio) + m / ratio) * n;
    int32_t *to = dst + (int64_t)pf * n;
    for (int i = threadIdx.x; i < n; i += blockDim.x) to[i] = from[i];
}

// s: the shape of the coarse stage (b_q = its block size)
int32_t launch_subdivide_blocks(const ihip_shape &s, const int32_t *starts, int n, int b_q_fine, int32_t *out,
                                hipStream_t st)
{
    const int ratio = s.b_q / b_q_fine;
    const int Mq_fine = s.Tq / b_q_fine;
    const int P = s.B * s.Hkv * Mq_fine;
    if (P == 0 || n == 0) return IHIP_OK;
    KernelTimer timer("subdivide_blocks", st);
    hipLaunchKernelGGL(subdivide_blocks_kernel, dim3(P), dim3(256), 0, st, starts, out, n, Mq_fine, ratio);
    return check_launch("subdivide_blocks");
}

int32_t launch_select_blocks(const ihip_shape &s, const float *scores, int max_chunks,
                             const int32_t *parent_starts, int n_parent, int parent_chunk, int chunk,
                             int keep, int32_t *out_starts, bool all_heads, hipStream_t st)
{
    SelectArgs a;
    a.pool = all_heads ? s.Hkv : 1;
    a.ge = make_geometry(s);
    a.scores = scores;
    a.max_chunks = max_chunks;
    a.parent_starts = parent_starts;
    a.n_parent = n_parent;
    a.ratio_log2 = parent_starts ? __builtin_ctz(parent_chunk / chunk) : 0;
    a.chunk = chunk;
    a.keep = keep;
    a.out_starts = out_starts;
    const int P = s.B * (all_heads ? 1 : s.Hkv) * (s.Tq / s.b_q);      // workgroups
    if (P == 0 || keep == 0) return IHIP_OK;
    KernelTimer timer(stage_name(kNameSelect, parent_starts == nullptr, chunk), st);
    // Workgroup shape.  A few problems (at most one workgroup per CU, all running at once): the
    // kernel is a chain of latencies, and 4 slots per thread in as many threads as that takes is
    // the shortest (cfg3's 4,092 first-stage slots: 1024 x 4 9.0 us, 512 x 8 10.2, 256 x 16 11.3).
    // Many problems (chunked prefill: one per query block): the workgroups queue for the CUs, and
    // the fewest threads that hold the slots win (cfg4's 4,143 slots: 512 threads 13.6 us, 1024
    // threads 16.4).
#define IHIP_SEL(NTV, ITV) hipLaunchKernelGGL((select_blocks_fast_kernel<NTV, ITV>), dim3(P), dim3(NTV), 0, st, a)
    const bool few = P <= 256;
    if (max_chunks <= 256 * 4) IHIP_SEL(256, 4);
    else if (few && max_chunks <= 512 * 4) IHIP_SEL(512, 4);
    else if (few && max_chunks <= 1024 * 4) IHIP_SEL(1024, 4);
    else if (few && max_chunks <= 1024 * 8) IHIP_SEL(1024, 8);
    else if (max_chunks <= 256 * 8) IHIP_SEL(256, 8);
    else if (max_chunks <= 256 * kFastItems) IHIP_SEL(256, kFastItems);
    else if (max_chunks <= 512 * kFastItems) IHIP_SEL(512, kFastItems);
    else if (max_chunks <= 1024 * kFastItems) IHIP_SEL(1024, kFastItems);
#undef IHIP_SEL
    else
        hipLaunchKernelGGL(select_blocks_kernel, dim3(P), dim3(kSelThreads), 0, st, a);
    return check_launch("select_blocks");
}

}  // namespace ihip
