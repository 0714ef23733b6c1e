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
    int pool;                 // 1: one selection per KV head; Hkv: scores max-pooled over the KV heads
                              // of a (sequence, query block), one selection written to all of them
};

// Which problem a workgroup selects for, how it reads a (possibly pooled) score and where the
// selection goes.  With pooling the Hkv problems of a (sequence, query block) have identical
// slots, so the first one's parent list describes them all.
struct SelView {
    int p;                    // first problem of the pooled set (the problem itself without pooling)
    int pool;
    int64_t in_stride, out_stride;   // elements between consecutive KV heads' rows
    const float *sc;
    int32_t *out;
    __device__ SelView(const SelectArgs &a, int wg)
    {
        pool = a.pool;
        p = pool > 1 ? (wg / a.ge.Mq) * a.ge.Hkv * a.ge.Mq + wg % a.ge.Mq : wg;
        in_stride = (int64_t)a.ge.Mq * a.max_chunks;
        out_stride = (int64_t)a.ge.Mq * a.keep;
        sc = a.scores + (int64_t)p * a.max_chunks;
        out = a.out_starts + (int64_t)p * a.keep;
    }
    __device__ float score(int i) const
    {
        float v = sc[i];
        for (int g = 1; g < pool; ++g) v = fmaxf(v, sc[g * in_stride + i]);
        return v;
    }
    __device__ void put(int rank, int value) const
    {
        out[rank] = value;
        if (pool > 1)
            for (int g = 1; g < pool; ++g) out[g * out_stride + rank] = value;
    }
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

// ---------------------------------------------------------------------------
// Fast path for up to 16 slots per thread.  Scores are bucketed into 2048
// linear bins between the problem's smallest and largest score (monotone in
// the key order, so the K-th best lies in one identifiable bin); only the few
// candidates of that bin are ranked exactly, by (key descending, slot
// ascending).  One pass over the scores, no contended atomics, ~10 barriers.
// If the threshold bin holds more candidates than threads (heavy ties), the
// radix select above finishes the job on the keys already in LDS.
// ---------------------------------------------------------------------------
constexpr int kFastItems = 16;
constexpr int kFastBins = 2048;

template <int NT>
__global__ __launch_bounds__(NT) void select_blocks_fast_kernel(const SelectArgs a)
{
    constexpr int NW = NT / 64;
    __shared__ uint32_t keys[NT * kFastItems];          // all keys (for the tie fallback and the ranking)
    __shared__ uint32_t hist[kFastBins];
    __shared__ uint8_t sel[NT * kFastItems];            // candidate of the threshold bin that is kept
    __shared__ uint32_t cand[NT];                       // slots of the threshold bin's candidates
    __shared__ float red_min[NW], red_max[NW];
    __shared__ uint32_t red_cnt[NW], wave_tot[NW];
    __shared__ uint32_t sh_bin, sh_above, sh_ncand;
    __shared__ SelectScratch<NT> scratch;

    const SelView view(a, blockIdx.x);
    const int p = view.p;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = a.max_chunks;
    const int per = (n + NT - 1) / NT;                  // <= kFastItems, slots [tid*per, tid*per + per)
    const int i0 = tid * per;

    // The start positions of this thread's slots depend on nothing the selection computes: the
    // sequence length and the parents' starts are requested now, next to the scores, and are there
    // when the kept slots are written at the end (asked for then, they would be two more dependent
    // trips to memory on a path that consists of little else).
    if (n == 0) {                                       // no slots at all: only the padding is written
        for (int i = tid; i < a.keep; i += NT) view.put(i, -1);
        return;
    }
    // All of these loads are written without a branch or a loop between them, so that they are in
    // flight together: with a per-item loop over the pooled rows, or an early return per slot, the
    // compiler waits for every load before it issues the next, and 16 trips to L2 one after the
    // other were half of this kernel's time.
    const Problem pr = problem_of(a.ge, p);
    const bool has_parents = a.parent_starts != nullptr;
    const int32_t *parents = has_parents ? a.parent_starts + (int64_t)p * a.n_parent : nullptr;
    int start_of[kFastItems];
    float v[kFastItems];
#pragma unroll
    for (int i = 0; i < kFastItems; ++i) {
        const int idx = min(i0 + i, n - 1);              // clamped: the value is ignored when out of range
        start_of[i] = has_parents ? parents[idx >> a.ratio_log2] : 0;
        v[i] = view.sc[idx];
    }
    if (view.pool > 1) {
#pragma unroll
        for (int i = 0; i < kFastItems; ++i)
            for (int g = 1; g < view.pool; ++g) v[i] = fmaxf(v[i], view.sc[g * view.in_stride + min(i0 + i, n - 1)]);
    }
    float mn = INFINITY, mx = -INFINITY;
    uint32_t valid = 0;
#pragma unroll
    for (int i = 0; i < kFastItems; ++i) {
        const int idx = i0 + i;
        const bool in = i < per && idx < n;
        // the slot's start position (as slot_start computes it), -1 for a slot without keys
        const int st = has_parents ? start_of[i] + (idx & ((1 << a.ratio_log2) - 1)) * a.chunk : pr.lo + idx * a.chunk;
        start_of[i] = in && (!has_parents || start_of[i] >= 0) && st < pr.hi ? st : -1;
        v[i] = in ? v[i] + 0.0f : -INFINITY;                                    // -0.0 -> +0.0
        if (in) keys[idx] = order_key(v[i]);
        if (v[i] > -INFINITY) { mn = fminf(mn, v[i]); mx = fmaxf(mx, v[i]); ++valid; }
    }
    mn = wave_min_f32(mn);
    mx = wave_max_f32(mx);
    valid = wave_sum_u32(valid);
    if (lane == 0) { red_min[wv] = mn; red_max[wv] = mx; red_cnt[wv] = valid; }
    for (int i = tid; i < kFastBins; i += NT) hist[i] = 0;
    for (int i = tid; i < NT * kFastItems / 4; i += NT) reinterpret_cast<uint32_t *>(sel)[i] = 0;
    if (tid == 0) sh_ncand = 0;
    __syncthreads();
    uint32_t n_valid = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { mn = fminf(mn, red_min[w]); mx = fmaxf(mx, red_max[w]); n_valid += red_cnt[w]; }
    const int keep_eff = min((int)n_valid, a.keep);

    if (keep_eff > 0) {
        const float scale = mx > mn ? (float)(kFastBins - 1) / (mx - mn) : 0.f;
        int bin[kFastItems];
#pragma unroll
        for (int i = 0; i < kFastItems; ++i) {
            bin[i] = -1;
            if (v[i] > -INFINITY) {
                bin[i] = min(kFastBins - 1, (int)((v[i] - mn) * scale));
                atomicAdd(&hist[bin[i]], 1u);
            }
        }
        __syncthreads();
        // suffix sums over the bins: thread t owns bins [t*bp, t*bp + bp), highest bins = lowest threads
        constexpr int bp = kFastBins / NT > 0 ? kFastBins / NT : 1;
        const bool owns = tid * bp < kFastBins;
        uint32_t mine = 0, hv[bp];
#pragma unroll
        for (int j = 0; j < bp; ++j) {
            hv[j] = owns ? hist[kFastBins - 1 - (tid * bp + j)] : 0u;
            mine += hv[j];
        }
        uint32_t incl = wave_incl_scan_u32(mine, lane);
        if (lane == 63) wave_tot[wv] = incl;
        __syncthreads();
        for (int w = 0; w < wv; ++w) incl += wave_tot[w];
        // the K-th best lies in the first bin (from the top) where the running count reaches keep_eff
        if (owns && incl >= (uint32_t)keep_eff && incl - mine < (uint32_t)keep_eff) {
            uint32_t run = incl - mine;
            bool found = false;
#pragma unroll
            for (int j = 0; j < bp; ++j) {
                if (!found && run + hv[j] >= (uint32_t)keep_eff) {
                    sh_bin = kFastBins - 1 - (tid * bp + j);
                    sh_above = run;
                    found = true;
                }
                run += hv[j];
            }
        }
        __syncthreads();
        const int tb = sh_bin;
        const uint32_t need = keep_eff - sh_above;         // kept from the threshold bin
        const uint32_t n_cand = hist[tb];
        if (n_cand <= (uint32_t)NT) {
            // list the candidates, then rank each exactly among them
#pragma unroll
            for (int i = 0; i < kFastItems; ++i)
                if (bin[i] == tb) cand[atomicAdd(&sh_ncand, 1u)] = i0 + i;
            __syncthreads();
            if ((uint32_t)tid < n_cand) {
                const uint32_t me = cand[tid], mk = keys[me];
                uint32_t rank = 0;
                for (uint32_t j = 0; j < n_cand; ++j) {
                    const uint32_t o = cand[j], ok = keys[o];
                    rank += (ok > mk) || (ok == mk && o < me);
                }
                if (rank < need) sel[me] = 1;
            }
            __syncthreads();
            // ordered compaction (the flags are read without conditions, all at once)
            bool take[kFastItems];
#pragma unroll
            for (int i = 0; i < kFastItems; ++i) take[i] = sel[min(i0 + i, NT * kFastItems - 1)] != 0;
            uint32_t cnt = 0;
#pragma unroll
            for (int i = 0; i < kFastItems; ++i) {
                take[i] = bin[i] > tb || (bin[i] == tb && take[i]);
                cnt += take[i];
            }
            uint32_t cincl = wave_incl_scan_u32(cnt, lane);
            if (lane == 63) red_cnt[wv] = cincl;
            __syncthreads();
            uint32_t pos = cincl - cnt;
            for (int w = 0; w < wv; ++w) pos += red_cnt[w];
#pragma unroll
            for (int i = 0; i < kFastItems; ++i)
                if (take[i]) view.put(pos++, start_of[i]);
        } else {
            // heavy ties: exact radix select over the keys in LDS
            block_select_largest<NT>(
                n, keep_eff, [&](int i) -> uint32_t { return keys[i]; },
                [&](uint32_t rank, int i) {
                    view.put(rank, slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, i));
                },
                scratch);
        }
    }
    for (int i = keep_eff + tid; i < a.keep; i += NT) view.put(i, -1);
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
    if (max_chunks <= 256 * kFastItems)
        hipLaunchKernelGGL(select_blocks_fast_kernel<256>, dim3(P), dim3(256), 0, st, a);
    else if (max_chunks <= 512 * kFastItems)
        hipLaunchKernelGGL(select_blocks_fast_kernel<512>, dim3(P), dim3(512), 0, st, a);
    else if (max_chunks <= 1024 * kFastItems)
        hipLaunchKernelGGL(select_blocks_fast_kernel<1024>, dim3(P), dim3(1024), 0, st, a);
    else
        hipLaunchKernelGGL(select_blocks_kernel, dim3(P), dim3(kSelThreads), 0, st, a);
    return check_launch("select_blocks");
}

}  // namespace ihip
