// arg-top-K of one problem's chunk scores (Alg. 2) by one workgroup of NT threads with up to ITEMS
// slots per thread.
//
// Scores are bucketed into 2048 linear bins between the problem's smallest and largest score
// (monotone in the key order, so the K-th best lies in one identifiable bin); only the few
// candidates of that bin are ranked exactly, by (key descending, slot ascending).  One pass over
// the scores, no contended atomics, ~10 barriers.  If the threshold bin holds more candidates than
// threads (heavy ties), the radix select of block_select.h finishes the job on keys re-read from
// the scores.
#pragma once

#include "block_select.h"

namespace ihip {

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

constexpr int kFastItems = 16;                 // most slots per thread
constexpr int kFastBins = 2048;

template <int NT>
struct SelectFastShared {
    uint32_t hist[kFastBins];
    uint32_t cand[NT], cand_key[NT];           // slots and keys of the threshold bin's candidates
    uint32_t cand_keep[NT];                    // ... and whether each is kept
    float red_min[NT / 64], red_max[NT / 64];
    uint32_t red_cnt[NT / 64], wave_tot[NT / 64];
    uint32_t bin, above, ncand;
    SelectScratch<NT> scratch;
};

// All NT threads of workgroup call it; `wg` says which problem (or pooled set) is selected.  Up to
// ITEMS slots per thread (a.max_chunks <= NT * ITEMS): the slots' scores and start positions live
// in registers, so ITEMS sets the register cost.
template <int NT, int ITEMS>
__device__ inline void select_blocks_fast(const SelectArgs &a, int wg, SelectFastShared<NT> &sh)
{
    constexpr int NW = NT / 64;
    const SelView view(a, wg);
    const int p = view.p;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = a.max_chunks;
    const int per = (n + NT - 1) / NT;                  // <= ITEMS, slots [tid*per, tid*per + per)
    const int i0 = tid * per;

    if (n == 0) {                                       // no slots at all: only the padding is written
        for (int i = tid; i < a.keep; i += NT) view.put(i, -1);
        return;
    }
    // The start positions of this thread's slots depend on nothing the selection computes: the
    // sequence length and the parents' starts are requested now, next to the scores, and are there
    // when the kept slots are written at the end (asked for then, they would be two more dependent
    // trips to memory on a path that consists of little else).
    // All of these loads are written without a branch or a loop between them, so that they are in
    // flight together: with a per-item loop over the pooled rows, or an early return per slot, the
    // compiler waits for every load before it issues the next, and 16 trips to L2 one after the
    // other were half of this kernel's time.
    const Problem pr = problem_of(a.ge, p);
    const bool has_parents = a.parent_starts != nullptr;
    const int32_t *parents = has_parents ? a.parent_starts + (int64_t)p * a.n_parent : nullptr;
    int start_of[ITEMS];
    float v[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int idx = min(i0 + i, n - 1);              // clamped: the value is ignored when out of range
        start_of[i] = has_parents ? parents[idx >> a.ratio_log2] : 0;
        v[i] = view.sc[idx];
    }
    if (view.pool > 1) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
            for (int g = 1; g < view.pool; ++g) v[i] = fmaxf(v[i], view.sc[g * view.in_stride + min(i0 + i, n - 1)]);
    }
    float mn = INFINITY, mx = -INFINITY;
    uint32_t valid = 0;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int idx = i0 + i;
        const bool in = i < per && idx < n;
        // the slot's start position (as slot_start computes it), -1 for a slot without keys
        const int st = has_parents ? start_of[i] + (idx & ((1 << a.ratio_log2) - 1)) * a.chunk : pr.lo + idx * a.chunk;
        start_of[i] = in && (!has_parents || start_of[i] >= 0) && st < pr.hi ? st : -1;
        v[i] = in ? v[i] + 0.0f : -INFINITY;                                    // -0.0 -> +0.0
        if (v[i] > -INFINITY) { mn = fminf(mn, v[i]); mx = fmaxf(mx, v[i]); ++valid; }
    }
    mn = wave_min_f32(mn);
    mx = wave_max_f32(mx);
    valid = wave_sum_u32(valid);
    if (lane == 0) { sh.red_min[wv] = mn; sh.red_max[wv] = mx; sh.red_cnt[wv] = valid; }
    for (int i = tid; i < kFastBins; i += NT) sh.hist[i] = 0;
    if (tid == 0) sh.ncand = 0;
    __syncthreads();
    uint32_t n_valid = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { mn = fminf(mn, sh.red_min[w]); mx = fmaxf(mx, sh.red_max[w]); n_valid += sh.red_cnt[w]; }
    const int keep_eff = min((int)n_valid, a.keep);

    if (keep_eff > 0) {
        const float scale = mx > mn ? (float)(kFastBins - 1) / (mx - mn) : 0.f;
        // a score's bin, -1 for an empty slot; computed again where it is needed rather than kept (a
        // register per slot less)
        auto bin_of = [&](float x) { return x > -INFINITY ? min(kFastBins - 1, (int)((x - mn) * scale)) : -1; };
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
            if (v[i] > -INFINITY) atomicAdd(&sh.hist[bin_of(v[i])], 1u);
        __syncthreads();
        // suffix sums over the bins: thread t owns bins [t*bp, t*bp + bp), highest bins = lowest threads
        constexpr int bp = kFastBins / NT > 0 ? kFastBins / NT : 1;
        const bool owns = tid * bp < kFastBins;
        uint32_t mine = 0, hv[bp];
#pragma unroll
        for (int j = 0; j < bp; ++j) {
            hv[j] = owns ? sh.hist[kFastBins - 1 - (tid * bp + j)] : 0u;
            mine += hv[j];
        }
        uint32_t incl = wave_incl_scan_u32(mine, lane);
        if (lane == 63) sh.wave_tot[wv] = incl;
        __syncthreads();
        for (int w = 0; w < wv; ++w) incl += sh.wave_tot[w];
        // the K-th best lies in the first bin (from the top) where the running count reaches keep_eff
        if (owns && incl >= (uint32_t)keep_eff && incl - mine < (uint32_t)keep_eff) {
            uint32_t run = incl - mine;
            bool found = false;
#pragma unroll
            for (int j = 0; j < bp; ++j) {
                if (!found && run + hv[j] >= (uint32_t)keep_eff) {
                    sh.bin = kFastBins - 1 - (tid * bp + j);
                    sh.above = run;
                    found = true;
                }
                run += hv[j];
            }
        }
        __syncthreads();
        const int tb = sh.bin;
        const uint32_t need = keep_eff - sh.above;         // kept from the threshold bin
        const uint32_t n_cand = sh.hist[tb];
        if (n_cand <= (uint32_t)NT) {
            // list the candidates, then rank each exactly among them.  code: where in the list the
            // slot went, or -1 for a slot above the threshold bin (kept), -2 below it or empty
            int code[ITEMS];
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                const int b = bin_of(v[i]);
                code[i] = b > tb ? -1 : -2;
                if (b == tb) {
                    code[i] = atomicAdd(&sh.ncand, 1u);
                    sh.cand[code[i]] = i0 + i;
                    sh.cand_key[code[i]] = order_key(v[i]);
                }
            }
            __syncthreads();
            if ((uint32_t)tid < n_cand) {
                const uint32_t me = sh.cand[tid], mk = sh.cand_key[tid];
                uint32_t rank = 0;
                for (uint32_t j = 0; j < n_cand; ++j) {
                    const uint32_t o = sh.cand[j], ok = sh.cand_key[j];
                    rank += (ok > mk) || (ok == mk && o < me);
                }
                sh.cand_keep[tid] = rank < need;
            }
            __syncthreads();
            // ordered compaction (the flags are read without conditions, all at once)
            bool take[ITEMS];
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) take[i] = sh.cand_keep[max(code[i], 0)] != 0;
            uint32_t cnt = 0;
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                take[i] = code[i] == -1 || (code[i] >= 0 && take[i]);
                cnt += take[i];
            }
            uint32_t cincl = wave_incl_scan_u32(cnt, lane);
            if (lane == 63) sh.red_cnt[wv] = cincl;
            __syncthreads();
            uint32_t pos = cincl - cnt;
            for (int w = 0; w < wv; ++w) pos += sh.red_cnt[w];
#pragma unroll
            for (int i = 0; i < ITEMS; ++i)
                if (take[i]) view.put(pos++, start_of[i]);
        } else {
            // heavy ties: exact radix select over the keys, re-read from the scores
            block_select_largest<NT>(
                n, keep_eff, [&](int i) -> uint32_t { return order_key(view.score(i)); },
                [&](uint32_t rank, int i) {
                    view.put(rank, slot_start(pr, a.parent_starts, a.n_parent, a.ratio_log2, a.chunk, p, i));
                },
                sh.scratch);
        }
    }
    for (int i = keep_eff + tid; i < a.keep; i += NT) view.put(i, -1);
}

}  // namespace ihip
