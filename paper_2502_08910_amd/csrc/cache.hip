// Host-memory KV tier with two on-GPU hot-block banks (Sec. 4 "KV Cache
// Offloading"; Alg. 4: per-layer miss lists, then LRU replacement after the
// layer's attention).
//
// K/V of the layer live in pinned host memory that kernels can read directly
// over the host link.  Two banks in HBM hold copies of 2^k-token blocks: the
// mask-selection bank (keys only, read by the pruning stages) and the
// sparse-attention bank (keys and values).  A page table maps a global block
// id (sequence, KV head, block) to a bank slot.  During a layer call kernels
// only mark blocks (touched / missed) and refresh LRU stamps; after the call
// ihip_cache_update turns the miss flags into an ascending miss list, picks as
// many least-recently-used slots (oldest stamp first, lowest slot on a tie,
// never a slot touched in this same call) and copies the missed blocks from
// host memory into them.  Everything is
// deterministic, so a CPU simulation of the same policy reproduces the tables.
//
// The call counter that stamps touches is a host variable copied into the
// kernel arguments at enqueue time: a captured graph would replay a frozen
// stamp (every slot would look "touched in this call" and replacement would
// stop), so calls on a stream under capture are refused (refuse_capture).
#include "block_select.h"

namespace ihip {

struct Bank {
    int n_slots;
    int32_t *page_table;      // [n_gb]
    int32_t *slot_block;      // [n_slots] global block id or -1
    uint32_t *slot_stamp;     // [n_slots]
    uint8_t *touch_flag;      // [n_gb_pad]
    uint8_t *miss_flag;       // [n_gb_pad]
    int32_t *miss_list;       // [n_gb]
    int32_t *victims;         // [n_slots]
    unsigned long long *counters;   // [8]: hit blocks, missed blocks (cumulative), last call's misses, touches, insertions
    uint16_t *bank_k, *bank_v;      // [n_slots][block][row]; bank_v null for the keys-only bank
};

}  // namespace ihip

struct ihip_cache {
    int B, Hkv;
    int64_t T_alloc;
    int block_tokens, block_log2, blocks_per_head, n_gb;
    ihip_tensor host_k, host_v;   // as given: strides in elements (bf16) or bytes (E4M3)
    int row_units;                // 2-byte units per row: d (bf16) or d/2 (E4M3)
    const int32_t *host_table;    // paged host tier: device int32 [B][host_table_stride] page ids, else nullptr
    int host_table_stride, host_page_log2;
    ihip::Bank bank[2];
    uint32_t stamp;           // counter of the current layer call (starts at 1)
};

namespace ihip {

constexpr int kCacheThreads = 1024;

static size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }

// carve one bank out of dev memory starting at *off (or just measure when base == nullptr)
static void carve_bank(Bank &b, char *base, size_t &off, int n_gb, int n_slots, int block_tokens, bool has_v,
                       int row_units)
{
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += a256(bytes); return p; };
    b.n_slots = n_slots;
    b.page_table = (int32_t *)take((size_t)n_gb * 4);
    b.slot_block = (int32_t *)take((size_t)n_slots * 4);
    b.slot_stamp = (uint32_t *)take((size_t)n_slots * 4);
    b.touch_flag = (uint8_t *)take((size_t)n_gb + 16);
    b.miss_flag = (uint8_t *)take((size_t)n_gb + 16);
    b.miss_list = (int32_t *)take((size_t)n_gb * 4);
    b.victims = (int32_t *)take((size_t)n_slots * 4);
    b.counters = (unsigned long long *)take(8 * 8);
    b.bank_k = (uint16_t *)take((size_t)n_slots * block_tokens * row_units * 2);
    b.bank_v = has_v ? (uint16_t *)take((size_t)n_slots * block_tokens * row_units * 2) : nullptr;
}

__global__ void cache_init_kernel(const Bank b, const int n_gb)
{
    const int stride = gridDim.x * blockDim.x;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_gb; i += stride) b.page_table[i] = -1;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < ((n_gb + 15) & ~15); i += stride) {
        b.touch_flag[i] = 0;          // including the padding up to a multiple of 16
        b.miss_flag[i] = 0;
    }
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slots; i += stride) {
        b.slot_block[i] = -1;
        b.slot_stamp[i] = 0;
    }
    if (blockIdx.x == 0 && threadIdx.x < 8) b.counters[threadIdx.x] = 0;
}

// miss flags -> ascending miss list; counts; clears the flags.  One workgroup;
// the 0/1 byte flags are read 16 at a time (the arrays are padded and zeroed
// to a multiple of 16).
__global__ __launch_bounds__(kCacheThreads) void cache_collect_kernel(const Bank b, const int n_gb)
{
    __shared__ uint32_t wave_miss[kCacheThreads / 64], wave_touch[kCacheThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n16 = (n_gb + 15) >> 4;
    const int c = (n16 + kCacheThreads - 1) / kCacheThreads;
    const int g0 = min(n16, tid * c), g1 = min(n16, g0 + c);
    uint4 *mf = reinterpret_cast<uint4 *>(b.miss_flag);
    uint4 *tf = reinterpret_cast<uint4 *>(b.touch_flag);
    auto ones = [](const uint4 &x) { return __popc(x.x) + __popc(x.y) + __popc(x.z) + __popc(x.w); };
    uint32_t miss = 0, touch = 0;
    for (int g = g0; g < g1; ++g) { miss += ones(mf[g]); touch += ones(tf[g]); }
    const uint32_t miss_incl = wave_incl_scan_u32(miss, lane);
    uint32_t t = touch;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) t += __shfl_xor(t, d, 64);
    if (lane == 63) wave_miss[wv] = miss_incl;
    if (lane == 0) wave_touch[wv] = t;
    __syncthreads();
    uint32_t base = miss_incl - miss, total_miss = 0, total_touch = 0;
    for (int w = 0; w < kCacheThreads / 64; ++w) {
        if (w < wv) base += wave_miss[w];
        total_miss += wave_miss[w];
        total_touch += wave_touch[w];
    }
    const uint4 zero = make_uint4(0, 0, 0, 0);
    for (int g = g0; g < g1; ++g) {
        const uint4 m = mf[g];
        const uint32_t w4[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if ((w4[j >> 2] >> ((j & 3) * 8)) & 1u) b.miss_list[base++] = g * 16 + j;
        mf[g] = zero;
        tf[g] = zero;
    }
    if (tid == 0) {
        b.counters[0] += total_touch - total_miss;
        b.counters[1] += total_miss;
        b.counters[2] = total_miss;
        b.counters[3] = total_touch;
    }
}

// The least recently used slots that will be replaced, ascending slot order:
// as many as there were misses, but only slots not touched in this call
// (swapping two blocks that were both just used would only burn host-link
// bandwidth).  One workgroup.
__global__ __launch_bounds__(kCacheThreads) void cache_victims_kernel(const Bank b, const uint32_t stamp)
{
    __shared__ SelectScratch<kCacheThreads> scratch;
    __shared__ uint32_t sh_eligible;
    if (threadIdx.x == 0) sh_eligible = 0;
    __syncthreads();
    uint32_t mine = 0;
    for (int i = threadIdx.x; i < b.n_slots; i += kCacheThreads) mine += b.slot_stamp[i] != stamp;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
    if ((threadIdx.x & 63) == 0) atomicAdd(&sh_eligible, mine);
    __syncthreads();
    const int m_eff = (int)min((unsigned long long)sh_eligible, b.counters[2]);
    if (threadIdx.x == 0) b.counters[4] = m_eff;
    if (m_eff == 0) return;
    block_select_largest<kCacheThreads>(
        b.n_slots, m_eff,
        [&](int i) -> uint32_t { return ~b.slot_stamp[i]; },          // oldest stamp = largest key
        [&](uint32_t rank, int i) { b.victims[rank] = i; },
        scratch);
}

// workgroup i: evict victims[i], install miss_list[i] there and copy its rows from host memory
__global__ __launch_bounds__(256) void cache_insert_kernel(const Bank b, const ihip_tensor hk, const ihip_tensor hv,
                                                           const int Hkv, const int64_t T_alloc, const int block_log2,
                                                           const int blocks_per_head, const uint32_t stamp,
                                                           const int row_units, const int32_t *host_table,
                                                           const int host_table_stride, const int host_page_log2)
{
    const int i = blockIdx.x;
    if (i >= (int)b.counters[4]) return;
    const int gb = b.miss_list[i];
    const int slot = b.victims[i];
    if (threadIdx.x == 0) {
        const int old = b.slot_block[slot];
        if (old >= 0) b.page_table[old] = -1;
        b.slot_block[slot] = gb;
        b.page_table[gb] = slot;
        b.slot_stamp[slot] = stamp;
    }
    const int bg = gb / blocks_per_head, blk = gb % blocks_per_head;
    const int bb = bg / Hkv, g = bg % Hkv;
    const int bt = 1 << block_log2;
    const int lanes = row_units >> 3;                 // 16-byte pieces per row: 16 (bf16) or 8 (E4M3)
    const int piece = threadIdx.x % lanes;
    const bool paged = host_table != nullptr;      // the host tensors are page pools: stride_b between pages
    const uint16_t *src_k = (const uint16_t *)hk.ptr + (paged ? 0 : bb * hk.stride_b) + g * hk.stride_h;
    const uint16_t *src_v = (const uint16_t *)hv.ptr + (paged ? 0 : bb * hv.stride_b) + g * hv.stride_h;
    for (int r = threadIdx.x / lanes; r < bt; r += 256 / lanes) {
        const int64_t pos = ((int64_t)blk << block_log2) + r;
        if (pos >= T_alloc) break;
        const int64_t dst = (((int64_t)slot << block_log2) + r) * row_units + piece * 8;
        int64_t at_k = pos * hk.stride_t, at_v = pos * hv.stride_t;
        if (paged) {
            const int64_t page = host_table[(int64_t)bb * host_table_stride + (pos >> host_page_log2)];
            const int64_t tok = pos & ((1 << host_page_log2) - 1);
            at_k = page * hk.stride_b + tok * hk.stride_t;
            at_v = page * hv.stride_b + tok * hv.stride_t;
        }
        *reinterpret_cast<uint4 *>(b.bank_k + dst) = *reinterpret_cast<const uint4 *>(src_k + at_k + piece * 8);
        if (b.bank_v != nullptr)
            *reinterpret_cast<uint4 *>(b.bank_v + dst) = *reinterpret_cast<const uint4 *>(src_v + at_v + piece * 8);
    }
}

BankView cache_bank_view(const ihip_cache *c, int which)
{
    const Bank &b = c->bank[which];
    BankView v;
    v.page_table = b.page_table;
    v.slot_stamp = b.slot_stamp;
    v.touch_flag = b.touch_flag;
    v.miss_flag = b.miss_flag;
    v.bank_k = b.bank_k;
    v.bank_v = b.bank_v;
    v.block_log2 = c->block_log2;
    v.blocks_per_head = c->blocks_per_head;
    v.stamp = c->stamp;
    v.row_units = c->row_units;
    v.host_table = c->host_table;
    v.host_table_stride = c->host_table_stride;
    v.host_page_log2 = c->host_page_log2;
    return v;
}

bool cache_holds_fp8(const ihip_cache *c) { return c->row_units != kD; }

// IHIP_ERR_UNSUPPORTED if `stream` is being captured into a graph (see the header of this file)
int32_t refuse_capture(const char *who, hipStream_t st)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &status) != hipSuccess) {
        (void)hipGetLastError();            // the query itself failed: nothing is known, go on
        return IHIP_OK;
    }
    if (status != hipStreamCaptureStatusNone)
        return fail(IHIP_ERR_UNSUPPORTED,
                    "%s: the host tier stamps its calls with a host-side counter and cannot be captured into a graph",
                    who);
    return IHIP_OK;
}

void cache_describe(const ihip_cache *c, int32_t *B, int32_t *Hkv, int64_t *T_alloc, ihip_tensor *hk, ihip_tensor *hv)
{
    *B = c->B; *Hkv = c->Hkv; *T_alloc = c->T_alloc; *hk = c->host_k; *hv = c->host_v;
}

static int32_t init_banks(ihip_cache *c, hipStream_t st)
{
    for (int w = 0; w < 2; ++w)
        hipLaunchKernelGGL(cache_init_kernel, dim3(256), dim3(256), 0, st, c->bank[w], c->n_gb);
    c->stamp = 1;
    return check_launch("cache init");
}

}  // namespace ihip

using namespace ihip;

extern "C" {

static size_t cache_device_bytes(int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens, int32_t mask_slots,
                                 int32_t sa_slots, int row_units)
{
    if (B <= 0 || Hkv <= 0 || T_alloc <= 0 || block_tokens <= 0 || (block_tokens & (block_tokens - 1)) ||
        mask_slots <= 0 || sa_slots <= 0)
        return 0;
    const int64_t n_gb = (int64_t)B * Hkv * ((T_alloc + block_tokens - 1) / block_tokens);
    if (n_gb > 0x7fffffff) return 0;
    Bank b;
    size_t off = 0;
    carve_bank(b, nullptr, off, (int)n_gb, mask_slots, block_tokens, false, row_units);
    carve_bank(b, nullptr, off, (int)n_gb, sa_slots, block_tokens, true, row_units);
    return off;
}

size_t ihip_cache_device_bytes(int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens, int32_t mask_slots,
                               int32_t sa_slots)
{
    return cache_device_bytes(B, Hkv, T_alloc, block_tokens, mask_slots, sa_slots, kD);
}

size_t ihip_cache_device_bytes_fp8(int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens, int32_t mask_slots,
                                   int32_t sa_slots)
{
    return cache_device_bytes(B, Hkv, T_alloc, block_tokens, mask_slots, sa_slots, kD / 2);
}

static int32_t cache_create(const char *who, int row_units, ihip_cache **out, void *dev_mem, size_t dev_bytes,
                            ihip_tensor host_k, ihip_tensor host_v, int32_t B, int32_t Hkv, int64_t T_alloc,
                            int32_t block_tokens, int32_t mask_slots, int32_t sa_slots, void *stream,
                            const ihip_paged_kv *host_pages = nullptr)
{
    if (!out) return fail(IHIP_ERR_INVALID_ARG, "%s: out is NULL", who);
    if (host_pages) {
        if (!host_pages->block_table || host_pages->page_tokens <= 0 ||
            (host_pages->page_tokens & (host_pages->page_tokens - 1)))
            return fail(IHIP_ERR_INVALID_ARG, "%s: block_table is NULL or page_tokens = %d is no power of two", who,
                        host_pages->page_tokens);
        if ((int64_t)host_pages->table_stride * host_pages->page_tokens < T_alloc)
            return fail(IHIP_ERR_INVALID_ARG, "%s: the block table covers %lld tokens, T_alloc is %lld", who,
                        (long long)host_pages->table_stride * host_pages->page_tokens, (long long)T_alloc);
    }
    const size_t need = cache_device_bytes(B, Hkv, T_alloc, block_tokens, mask_slots, sa_slots, row_units);
    if (need == 0) return fail(IHIP_ERR_INVALID_ARG, "%s: bad sizes (block_tokens must be a power of two)", who);
    if (mask_slots > 65536 * 16 || sa_slots > 65536 * 16)
        return fail(IHIP_ERR_UNSUPPORTED, "%s: at most 1,048,576 slots per bank", who);
    if (!dev_mem || dev_bytes < need || ((uintptr_t)dev_mem & 255))
        return fail(IHIP_ERR_WORKSPACE, "%s: %zu bytes of 256-byte aligned device memory needed, %zu given", who, need,
                    dev_bytes);
    // strides: elements for bf16 rows (multiples of 8), bytes for E4M3 rows (multiples of 16)
    const int64_t sm = row_units == kD ? 7 : 15;
    if (!host_k.ptr || !host_v.ptr || ((uintptr_t)host_k.ptr & 15) || ((uintptr_t)host_v.ptr & 15) ||
        (host_k.stride_t & sm) || (host_v.stride_t & sm) || (host_k.stride_h & sm) || (host_v.stride_h & sm) ||
        (host_k.stride_b & sm) || (host_v.stride_b & sm))
        return fail(IHIP_ERR_INVALID_ARG, "%s: host K/V must be non-NULL with 16-byte aligned rows", who);

    // the kernels dereference these pointers: insist on pinned, GPU-addressable host memory
    for (ihip_tensor *t : {&host_k, &host_v}) {
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, t->ptr) != hipSuccess) {
            (void)hipGetLastError();
            return fail(IHIP_ERR_INVALID_ARG, "%s: host K/V is not memory HIP knows (allocate it with hipHostMalloc)", who);
        }
        if (attr.type != hipMemoryTypeHost || attr.devicePointer == nullptr)
            return fail(IHIP_ERR_INVALID_ARG, "%s: host K/V must be pinned host memory the GPU can address", who);
        t->ptr = attr.devicePointer;
    }
    ihip_cache *c = new ihip_cache();
    c->B = B; c->Hkv = Hkv; c->T_alloc = T_alloc;
    c->block_tokens = block_tokens;
    c->block_log2 = __builtin_ctz(block_tokens);
    c->blocks_per_head = (int)((T_alloc + block_tokens - 1) / block_tokens);
    c->n_gb = B * Hkv * c->blocks_per_head;
    c->host_k = host_k; c->host_v = host_v;
    c->row_units = row_units;
    c->host_table = host_pages ? host_pages->block_table : nullptr;
    c->host_table_stride = host_pages ? host_pages->table_stride : 0;
    c->host_page_log2 = host_pages ? __builtin_ctz(host_pages->page_tokens) : 0;
    size_t off = 0;
    carve_bank(c->bank[0], (char *)dev_mem, off, c->n_gb, mask_slots, block_tokens, false, row_units);
    carve_bank(c->bank[1], (char *)dev_mem, off, c->n_gb, sa_slots, block_tokens, true, row_units);
    const int32_t rc = init_banks(c, (hipStream_t)stream);
    if (rc != IHIP_OK) { delete c; return rc; }
    *out = c;
    return IHIP_OK;
}

int32_t ihip_cache_create(ihip_cache **out, void *dev_mem, size_t dev_bytes, ihip_tensor host_k, ihip_tensor host_v,
                          int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens, int32_t mask_slots,
                          int32_t sa_slots, void *stream)
{
    return cache_create("ihip_cache_create", kD, out, dev_mem, dev_bytes, host_k, host_v, B, Hkv, T_alloc,
                        block_tokens, mask_slots, sa_slots, stream);
}

int32_t ihip_cache_create_fp8(ihip_cache **out, void *dev_mem, size_t dev_bytes, ihip_tensor host_k,
                              ihip_tensor host_v, int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens,
                              int32_t mask_slots, int32_t sa_slots, void *stream)
{
    return cache_create("ihip_cache_create_fp8", kD / 2, out, dev_mem, dev_bytes, host_k, host_v, B, Hkv, T_alloc,
                        block_tokens, mask_slots, sa_slots, stream);
}

int32_t ihip_cache_create_paged(ihip_cache **out, void *dev_mem, size_t dev_bytes, ihip_tensor host_k_pool,
                                ihip_tensor host_v_pool, const ihip_paged_kv *host_pages, int32_t kv_fp8, int32_t B,
                                int32_t Hkv, int64_t T_alloc, int32_t block_tokens, int32_t mask_slots,
                                int32_t sa_slots, void *stream)
{
    if (!host_pages) return fail(IHIP_ERR_INVALID_ARG, "ihip_cache_create_paged: host_pages is NULL");
    return cache_create("ihip_cache_create_paged", kv_fp8 ? kD / 2 : kD, out, dev_mem, dev_bytes, host_k_pool,
                        host_v_pool, B, Hkv, T_alloc, block_tokens, mask_slots, sa_slots, stream, host_pages);
}

void ihip_cache_destroy(ihip_cache *c) { delete c; }

int32_t ihip_cache_reset(ihip_cache *c, void *stream)
{
    if (!c) return fail(IHIP_ERR_INVALID_ARG, "ihip_cache_reset: cache is NULL");
    return init_banks(c, (hipStream_t)stream);
}

int32_t ihip_cache_update(ihip_cache *c, void *stream)
{
    if (!c) return fail(IHIP_ERR_INVALID_ARG, "ihip_cache_update: cache is NULL");
    hipStream_t st = (hipStream_t)stream;
    const int32_t rc = refuse_capture("ihip_cache_update", st);
    if (rc != IHIP_OK) return rc;
    for (int w = 0; w < 2; ++w) {
        const Bank &b = c->bank[w];
        {
            KernelTimer t(w == 0 ? "cache_collect.mask" : "cache_collect.sa", st);
            hipLaunchKernelGGL(cache_collect_kernel, dim3(1), dim3(kCacheThreads), 0, st, b, c->n_gb);
        }
        {
            KernelTimer t(w == 0 ? "cache_victims.mask" : "cache_victims.sa", st);
            hipLaunchKernelGGL(cache_victims_kernel, dim3(1), dim3(kCacheThreads), 0, st, b, c->stamp);
        }
        {
            KernelTimer t(w == 0 ? "cache_insert.mask" : "cache_insert.sa", st);
            ihip_tensor hk = c->host_k, hv = c->host_v;      // the kernel counts in 2-byte units
            if (c->row_units != kD)
                for (ihip_tensor *x : {&hk, &hv}) { x->stride_b /= 2; x->stride_h /= 2; x->stride_t /= 2; }
            hipLaunchKernelGGL(cache_insert_kernel, dim3(b.n_slots), dim3(256), 0, st, b, hk, hv, c->Hkv,
                               c->T_alloc, c->block_log2, c->blocks_per_head, c->stamp, c->row_units,
                               c->host_table, c->host_table_stride, c->host_page_log2);
        }
    }
    c->stamp += 1;
    return check_launch("cache update");
}

int32_t ihip_cache_stats(ihip_cache *c, uint64_t *stats8)
{
    if (!c || !stats8) return fail(IHIP_ERR_INVALID_ARG, "ihip_cache_stats: NULL argument");
    if (hipDeviceSynchronize() != hipSuccess) return fail(IHIP_ERR_HIP, "ihip_cache_stats: device synchronise failed");
    for (int w = 0; w < 2; ++w)
        if (hipMemcpy(stats8 + 4 * w, c->bank[w].counters, 32, hipMemcpyDeviceToHost) != hipSuccess)
            return fail(IHIP_ERR_HIP, "ihip_cache_stats: copy failed");
    return IHIP_OK;
}

int32_t ihip_cache_read_tables(ihip_cache *c, int32_t bank, int32_t *host_page_table, int32_t *host_slot_block)
{
    if (!c || bank < 0 || bank > 1) return fail(IHIP_ERR_INVALID_ARG, "ihip_cache_read_tables: bad argument");
    if (hipDeviceSynchronize() != hipSuccess) return fail(IHIP_ERR_HIP, "ihip_cache_read_tables: synchronise failed");
    const Bank &b = c->bank[bank];
    if (host_page_table &&
        hipMemcpy(host_page_table, b.page_table, (size_t)c->n_gb * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(IHIP_ERR_HIP, "ihip_cache_read_tables: copy failed");
    if (host_slot_block &&
        hipMemcpy(host_slot_block, b.slot_block, (size_t)b.n_slots * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(IHIP_ERR_HIP, "ihip_cache_read_tables: copy failed");
    return IHIP_OK;
}

int32_t ihip_cache_geometry(const ihip_cache *c, int32_t *n_blocks_total, int32_t *mask_slots, int32_t *sa_slots)
{
    if (!c) return fail(IHIP_ERR_INVALID_ARG, "ihip_cache_geometry: cache is NULL");
    if (n_blocks_total) *n_blocks_total = c->n_gb;
    if (mask_slots) *mask_slots = c->bank[0].n_slots;
    if (sa_slots) *sa_slots = c->bank[1].n_slots;
    return IHIP_OK;
}

}  // extern "C"
