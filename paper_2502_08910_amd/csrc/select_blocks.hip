// arg-top-K of the chunk scores (Alg. 2) -- one workgroup per problem.
//
// Radix select on order-preserving 32-bit keys held in LDS (4 passes of 8
// bits find the K-th largest key), then one ordered compaction: a single
// block-wide scan of per-thread (greater, equal) counts gives every kept slot
// its output position, so the result comes out in ascending position order
// with ties resolved to the lowest slot, without any sort.
#include "common.h"

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

__device__ inline uint32_t wave_incl_scan_u32(uint32_t v, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

__global__ __launch_bounds__(kSelThreads) void select_blocks_kernel(const SelectArgs a)
{
    __shared__ uint32_t keys[kSelLdsKeys];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_tot[kSelThreads / 64];
    __shared__ uint32_t sh_prefix, sh_remaining, sh_valid;

    const int p = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = a.max_chunks;
    const float *sc = a.scores + (int64_t)p * n;
    const bool cached = n <= kSelLdsKeys;

    auto key_at = [&](int i) -> uint32_t { return cached ? keys[i] : order_key(sc[i]); };

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
        // ---- K-th largest key by 4 radix passes, most significant digit first
        if (tid == 0) { sh_prefix = 0; sh_remaining = keep_eff; }
        uint32_t mask = 0;
        for (int shift = 24; shift >= 0; shift -= 8) {
            hist[tid] = 0;
            __syncthreads();
            const uint32_t prefix = sh_prefix;
            for (int i = tid; i < n; i += kSelThreads) {
                const uint32_t kk = key_at(i);
                if ((kk & mask) == prefix) atomicAdd(&hist[(kk >> shift) & 255u], 1u);
            }
            __syncthreads();
            // suffix[t] = candidates with digit >= t
            const uint32_t h = hist[255 - tid];                // thread tid looks at digit 255-tid
            uint32_t incl = wave_incl_scan_u32(h, lane);
            if (lane == 63) wave_tot[wv] = incl;
            __syncthreads();
            for (int w = 0; w < wv; ++w) incl += wave_tot[w];
            const uint32_t remaining = sh_remaining;
            __syncthreads();
            // digit D = 255-tid is the K-th key's digit iff suffix[D] >= remaining > suffix[D+1]
            if (incl >= remaining && incl - h < remaining) {
                sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
                sh_remaining = remaining - (incl - h);
            }
            mask |= 255u << shift;
            __syncthreads();
        }
        const uint32_t thr = sh_prefix;            // the K-th largest key
        const uint32_t need_eq = sh_remaining;     // how many keys equal to it are kept (lowest slots first)

        // ---- ordered compaction: thread t owns slots [t*c, (t+1)*c)
        const int c = (n + kSelThreads - 1) / kSelThreads;
        const int i0 = tid * c, i1 = min(n, i0 + c);
        uint32_t gt = 0, eq = 0;
        for (int i = i0; i < i1; ++i) {
            const uint32_t kk = key_at(i);
            gt += kk > thr;
            eq += kk == thr;
        }
        // block-wide exclusive scan of (gt, eq); c <= 4096 so both fit 16 bits... use two scans for safety
        uint32_t gt_incl = wave_incl_scan_u32(gt, lane);
        uint32_t eq_incl = wave_incl_scan_u32(eq, lane);
        __shared__ uint32_t wt_gt[kSelThreads / 64], wt_eq[kSelThreads / 64];
        if (lane == 63) { wt_gt[wv] = gt_incl; wt_eq[wv] = eq_incl; }
        __syncthreads();
        uint32_t gt_base = gt_incl - gt, eq_base = eq_incl - eq;
        for (int w = 0; w < wv; ++w) { gt_base += wt_gt[w]; eq_base += wt_eq[w]; }

        uint32_t pos = gt_base + min(eq_base, need_eq);
        uint32_t eq_seen = eq_base;
        const Problem pr = problem_of(a.ge, p);
        for (int i = i0; i < i1; ++i) {
            const uint32_t kk = key_at(i);
            bool take = kk > thr;
            if (kk == thr) { take = eq_seen < need_eq; ++eq_seen; }
            if (take) {
                out[pos++] = slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, i);
            }
        }
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
