// Workgroup-wide selection of the `keep` largest of n 32-bit keys.
//
// Radix select (4 passes of 8 bits, most significant first) finds the keep-th
// largest key; one block scan of per-thread (greater, equal) counts then gives
// every selected index its rank, so results are emitted in ascending index
// order with ties going to the lowest index -- no sort.  Used by the arg-top-K
// of the chunk scores and by the LRU victim choice of the hot-block cache.
#pragma once

#include "common.h"

namespace ihip {

template <int NT>
struct SelectScratch {
    uint32_t hist[256];
    uint32_t wave_tot[NT / 64];
    uint32_t wt_gt[NT / 64], wt_eq[NT / 64];
    uint32_t prefix, remaining;
};

__device__ inline uint32_t wave_incl_scan_u32(uint32_t v, int lane) { return wave_scan_u32(v, lane); }

// All NT threads of the workgroup must call this with the same n, keep
// (1 <= keep <= n).  key_at(i) returns the key of index i; emit(rank, i) is
// called once per selected index, rank = its position among the selected in
// ascending index order.
template <int NT, class KeyAt, class Emit>
__device__ inline void block_select_largest(int n, int keep, KeyAt key_at, Emit emit, SelectScratch<NT> &sh)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) { sh.prefix = 0; sh.remaining = keep; }
    uint32_t mask = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = tid; i < 256; i += NT) sh.hist[i] = 0;
        __syncthreads();
        const uint32_t prefix = sh.prefix;
        for (int i = tid; i < n; i += NT) {
            const uint32_t kk = key_at(i);
            if ((kk & mask) == prefix) atomicAdd(&sh.hist[(kk >> shift) & 255u], 1u);
        }
        __syncthreads();
        // threads 0..255 look at digit 255-tid; suffix[D] = candidates with digit >= D
        uint32_t h = 0, incl = 0;
        if (tid < 256) {
            h = sh.hist[255 - tid];
            incl = wave_incl_scan_u32(h, lane);
            if (lane == 63) sh.wave_tot[wv] = incl;
        }
        __syncthreads();
        const uint32_t remaining = sh.remaining;
        if (tid < 256)
            for (int w = 0; w < wv; ++w) incl += sh.wave_tot[w];
        __syncthreads();
        // digit D is the keep-th key's digit iff suffix[D] >= remaining > suffix[D+1]
        if (tid < 256 && incl >= remaining && incl - h < remaining) {
            sh.prefix = prefix | ((uint32_t)(255 - tid) << shift);
            sh.remaining = remaining - (incl - h);
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    const uint32_t thr = sh.prefix;            // the keep-th largest key
    const uint32_t need_eq = sh.remaining;     // keys equal to it that are kept (lowest indices first)

    // ordered compaction: thread t owns indices [t*c, (t+1)*c)
    const int c = (n + NT - 1) / NT;
    const int i0 = tid * c, i1 = min(n, i0 + c);
    uint32_t gt = 0, eq = 0;
    for (int i = i0; i < i1; ++i) {
        const uint32_t kk = key_at(i);
        gt += kk > thr;
        eq += kk == thr;
    }
    const uint32_t gt_incl = wave_incl_scan_u32(gt, lane);
    const uint32_t eq_incl = wave_incl_scan_u32(eq, lane);
    if (lane == 63) { sh.wt_gt[wv] = gt_incl; sh.wt_eq[wv] = eq_incl; }
    __syncthreads();
    uint32_t gt_base = gt_incl - gt, eq_base = eq_incl - eq;
    for (int w = 0; w < wv; ++w) { gt_base += sh.wt_gt[w]; eq_base += sh.wt_eq[w]; }
    uint32_t pos = gt_base + min(eq_base, need_eq);
    uint32_t eq_seen = eq_base;
    for (int i = i0; i < i1; ++i) {
        const uint32_t kk = key_at(i);
        bool take = kk > thr;
        if (kk == thr) { take = eq_seen < need_eq; ++eq_seen; }
        if (take) emit(pos++, i);
    }
    __syncthreads();
}

}  // namespace ihip
