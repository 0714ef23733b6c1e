// C ABI of the library: argument checks, error text, workspace layout and the
// multi-stage drivers (Alg. 1; the per-layer sequence of Alg. 4 with every
// stage refreshed).  Kernels live in the other translation units.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "common.h"

namespace ihip {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int32_t check_launch(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(IHIP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return IHIP_OK;
}

// ---- per-kernel event timing -------------------------------------------------
namespace {
struct Span { const char *name; hipEvent_t t0, t1; };
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<Span> g_spans;                 // recorded, not yet read
std::vector<hipEvent_t> g_free_events;     // recycled
hipEvent_t take_event()
{
    hipEvent_t e;
    if (!g_free_events.empty()) { e = g_free_events.back(); g_free_events.pop_back(); return e; }
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

const char *stage_name(int which, bool first, int chunk)
{
    static char names[3][2][11][40];
    static const char *prefix[3] = {"prune_decode", "prune_prefill", "select_blocks"};
    const int lg = __builtin_ctz(chunk);
    char *n = names[which][first][lg];
    if (n[0] == 0) snprintf(n, 40, first ? "%s.first.l%d" : "%s.l%d", prefix[which], chunk);
    return n;
}

void profile_begin(const char *name, hipStream_t st)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_prof_on) return;
    Span s{name, take_event(), take_event()};
    if (!s.t0 || !s.t1) return;
    (void)hipEventRecord(s.t0, st);
    g_spans.push_back(s);
}

void profile_end(hipStream_t st)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_prof_on || g_spans.empty()) return;
    (void)hipEventRecord(g_spans.back().t1, st);
}

// kernels' host launchers
int32_t launch_prune_stage(const ihip_shape &, const ihip_tensor &, const ihip_tensor &, const int32_t *,
                           int, int, int, int, float *, int32_t *, const BankView *, const ihip_rope *, hipStream_t,
                           const KvFormat * = nullptr);
int32_t launch_subdivide_blocks(const ihip_shape &, const int32_t *, int, int, int32_t *, hipStream_t);
int32_t launch_select_blocks(const ihip_shape &, const float *, int, const int32_t *, int, int, int, int,
                             int32_t *, bool, hipStream_t);
int32_t launch_attn_decode(const ihip_shape &, const ihip_tensor &, const ihip_tensor &,
                           const ihip_tensor &, const int32_t *, int, int, float, void *, float *,
                           void *, const BankView *, const ihip_rope *, hipStream_t, const KvFormat * = nullptr);
BankView cache_bank_view(const ihip_cache *, int);
void cache_describe(const ihip_cache *, int32_t *, int32_t *, int64_t *, ihip_tensor *, ihip_tensor *);
bool cache_holds_fp8(const ihip_cache *);
int32_t refuse_capture(const char *, hipStream_t);
size_t attn_decode_workspace(const ihip_shape &, int, int);
int32_t launch_attn_prefill(const ihip_shape &, const ihip_tensor &, const ihip_tensor &,
                            const ihip_tensor &, const int32_t *, int, int, float, void *, float *,
                            const ihip_rope *, hipStream_t, const KvFormat * = nullptr);

static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// FP8 K/V tensors: strides count bytes; rows 16-byte aligned like the bf16 ones
static int32_t check_tensor8(const ihip_tensor &t, const char *who, const char *name)
{
    if (!t.ptr) return fail(IHIP_ERR_INVALID_ARG, "%s: %s.ptr is NULL", who, name);
    if (((uintptr_t)t.ptr | (uintptr_t)t.stride_b | (uintptr_t)t.stride_h | (uintptr_t)t.stride_t) & 15)
        return fail(IHIP_ERR_INVALID_ARG, "%s: %s rows must be 16-byte aligned", who, name);
    if (t.stride_t < kD) return fail(IHIP_ERR_INVALID_ARG, "%s: %s.stride_t = %lld < d", who, name, (long long)t.stride_t);
    return IHIP_OK;
}
// paged K/V: pools through strides (stride_b = elements between pages) + a block table
static int32_t check_paged(const char *who, const ihip_shape *shape, const ihip_paged_kv *pg, KvFormat *fmt)
{
    if (!pg || !pg->block_table) return fail(IHIP_ERR_INVALID_ARG, "%s: paged / block_table is NULL", who);
    if (!pow2(pg->page_tokens)) return fail(IHIP_ERR_INVALID_ARG, "%s: page_tokens = %d is not a power of two", who, pg->page_tokens);
    if (shape && (int64_t)pg->table_stride * pg->page_tokens < shape->max_seq_len)
        return fail(IHIP_ERR_INVALID_ARG, "%s: the block table covers %lld tokens, max_seq_len is %d", who,
                    (long long)pg->table_stride * pg->page_tokens, shape->max_seq_len);
    *fmt = KvFormat{false, 1.0f, 1.0f, PagedView{pg->block_table, pg->table_stride, __builtin_ctz(pg->page_tokens)}};
    return IHIP_OK;
}

static int32_t check_scales(const char *who, float k_scale, float v_scale)
{
    if (!(k_scale > 0.f) || !(v_scale > 0.f) || k_scale > 3.0e38f || v_scale > 3.0e38f)
        return fail(IHIP_ERR_INVALID_ARG, "%s: scales must be positive and finite", who);
    return IHIP_OK;
}

static int32_t check_shape(const ihip_shape *s, const char *who)
{
    if (!s) return fail(IHIP_ERR_INVALID_ARG, "%s: shape is NULL", who);
    if (s->B < 0 || s->Hq <= 0 || s->Hkv <= 0 || s->Hq % s->Hkv != 0)
        return fail(IHIP_ERR_INVALID_ARG, "%s: bad B/Hq/Hkv = %d/%d/%d", who, s->B, s->Hq, s->Hkv);
    const int G = s->Hq / s->Hkv;
    if (G != 1 && G != 2 && G != 4 && G != 8)
        return fail(IHIP_ERR_UNSUPPORTED, "%s: Hq/Hkv = %d not in {1,2,4,8}", who, G);
    if (s->d != kD) return fail(IHIP_ERR_UNSUPPORTED, "%s: d = %d, only 128 is built", who, s->d);
    if (s->Tq <= 0 || s->b_q <= 0 || s->Tq % s->b_q != 0)
        return fail(IHIP_ERR_INVALID_ARG, "%s: Tq = %d must be a positive multiple of b_q = %d", who, s->Tq, s->b_q);
    if (s->n_sink < 0 || s->n_stream < s->b_q)
        return fail(IHIP_ERR_INVALID_ARG, "%s: need n_sink >= 0 and n_stream >= b_q (got %d, %d, b_q %d)", who,
                    s->n_sink, s->n_stream, s->b_q);
    if (s->b_q_range != 0 && (s->b_q_range < s->b_q || s->b_q_range % s->b_q != 0 || s->Tq % s->b_q_range != 0 ||
                              s->n_stream < s->b_q_range))
        return fail(IHIP_ERR_INVALID_ARG,
                    "%s: b_q_range = %d must be 0 or a multiple of b_q = %d that divides Tq = %d and is <= n_stream = %d",
                    who, s->b_q_range, s->b_q, s->Tq, s->n_stream);
    if (s->max_seq_len < s->Tq)
        return fail(IHIP_ERR_INVALID_ARG, "%s: max_seq_len = %d < Tq = %d", who, s->max_seq_len, s->Tq);
    if (!s->seq_lens && s->B > 0) return fail(IHIP_ERR_INVALID_ARG, "%s: seq_lens is NULL", who);
    return IHIP_OK;
}

static int32_t check_tensor(const ihip_tensor &t, const char *who, const char *name)
{
    if (!t.ptr) return fail(IHIP_ERR_INVALID_ARG, "%s: %s.ptr is NULL", who, name);
    if (((uintptr_t)t.ptr & 15) || (t.stride_b & 7) || (t.stride_h & 7) || (t.stride_t & 7))
        return fail(IHIP_ERR_INVALID_ARG, "%s: %s rows must be 16-byte aligned", who, name);
    if (t.stride_t < kD && t.stride_t != 0)
        return fail(IHIP_ERR_INVALID_ARG, "%s: %s.stride_t = %lld < d", who, name, (long long)t.stride_t);
    return IHIP_OK;
}

static int32_t check_slots(const char *who, const int32_t *parent_starts, int n_parent, int parent_chunk,
                           int chunk, int max_chunks)
{
    if (!pow2(chunk) || chunk > 1024)
        return fail(IHIP_ERR_INVALID_ARG, "%s: chunk = %d must be a power of two <= 1024", who, chunk);
    if (max_chunks < 0) return fail(IHIP_ERR_INVALID_ARG, "%s: max_chunks = %d", who, max_chunks);
    if (parent_starts) {
        if (!pow2(parent_chunk) || parent_chunk % chunk != 0)
            return fail(IHIP_ERR_INVALID_ARG, "%s: parent_chunk = %d must be a power of two multiple of chunk = %d",
                        who, parent_chunk, chunk);
        if (n_parent < 0 || (int64_t)n_parent * (parent_chunk / chunk) != max_chunks)
            return fail(IHIP_ERR_INVALID_ARG, "%s: max_chunks = %d must equal n_parent * parent_chunk / chunk = %lld",
                        who, max_chunks, (long long)n_parent * (parent_chunk / chunk));
    }
    return IHIP_OK;
}

static int stage1_slots(const ihip_shape &s, int chunk)
{
    const int64_t mid = (int64_t)s.max_seq_len - s.n_stream - s.n_sink;
    return mid > 0 ? (int)((mid + chunk - 1) / chunk) : 0;
}

static int32_t check_plan(const char *who, const ihip_shape *s, int n_stages, const int32_t *chunks,
                          const int32_t *keeps)
{
    if (n_stages < 1 || n_stages > 8 || !chunks || !keeps)
        return fail(IHIP_ERR_INVALID_ARG, "%s: need 1..8 stages with chunk_sizes and keeps", who);
    for (int i = 0; i < n_stages; ++i) {
        if (!pow2(chunks[i]) || chunks[i] > 1024 || keeps[i] < 1)
            return fail(IHIP_ERR_INVALID_ARG, "%s: stage %d: chunk %d / keep %d invalid", who, i, chunks[i], keeps[i]);
        if (i > 0 && chunks[i - 1] % chunks[i] != 0)
            return fail(IHIP_ERR_INVALID_ARG, "%s: stage %d: chunk %d does not divide %d", who, i, chunks[i],
                        chunks[i - 1]);
    }
    (void)s;
    return IHIP_OK;
}

// ---- workspace layout of prune_all: [scores | starts ping | starts pong] ----
struct PlanLayout {
    size_t scores_off, scores_bytes;
    size_t starts_off[2], starts_bytes;
    size_t total;
};

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static PlanLayout plan_layout(const ihip_shape &s, int n_stages, const int32_t *chunks, const int32_t *keeps)
{
    const size_t P = (size_t)s.B * s.Hkv * (s.Tq / s.b_q);
    size_t max_slots = stage1_slots(s, chunks[0]);
    size_t max_keep = 0;
    for (int i = 0; i < n_stages; ++i) {
        if (i > 0) max_slots = std::max(max_slots, (size_t)keeps[i - 1] * (chunks[i - 1] / chunks[i]));
        if (i + 1 < n_stages) max_keep = std::max(max_keep, (size_t)keeps[i]);
    }
    PlanLayout L;
    L.scores_off = 0;
    L.scores_bytes = align256(P * max_slots * sizeof(float));
    L.starts_bytes = align256(P * max_keep * sizeof(int32_t));
    L.starts_off[0] = L.scores_off + L.scores_bytes;
    L.starts_off[1] = L.starts_off[0] + L.starts_bytes;
    L.total = L.starts_off[1] + L.starts_bytes;
    return L;
}

// The stages of Alg. 1 whose bit is set in `due`.  stage_out[i] receives stage i's kept starts; a
// stage that is re-run reads the list of the stage before it as it stands, re-run in this call or
// cached from an earlier one (Alg. 4: a stage is re-run when its counter says so, with the current
// lists of the earlier stages; a stage that is not due keeps its list).
static int32_t prune_stages_impl(const ihip_shape &s, const ihip_tensor &q, const ihip_tensor &k, int n_stages,
                                 const int32_t *chunks, const int32_t *keeps, uint32_t due,
                                 int32_t *const *stage_out, float *scores, const BankView *bank,
                                 const ihip_rope *rope, bool all_heads, hipStream_t st,
                                 const KvFormat *fmt = nullptr)
{
    for (int i = 0; i < n_stages; ++i) {
        if (!((due >> i) & 1u)) continue;
        const int32_t *parents = i == 0 ? nullptr : stage_out[i - 1];
        const int n_parent = i == 0 ? 0 : keeps[i - 1];
        const int parent_chunk = i == 0 ? 0 : chunks[i - 1];
        const int slots = i == 0 ? stage1_slots(s, chunks[0]) : n_parent * (parent_chunk / chunks[i]);
        int32_t rc = launch_prune_stage(s, q, k, parents, n_parent, parent_chunk, chunks[i], slots, scores,
                                        nullptr, bank, rope, st, fmt);
        if (rc != IHIP_OK) return rc;
        rc = launch_select_blocks(s, scores, slots, parents, n_parent, parent_chunk, chunks[i], keeps[i],
                                  stage_out[i], all_heads, st);
        if (rc != IHIP_OK) return rc;
    }
    return IHIP_OK;
}

// Alg. 1 with a query-block size per stage (Sec. 4, the m' rule): stage i runs on blocks of
// stage_b_q[i] queries inside the candidate ranges of the first stage's blocks; where the next stage's
// blocks are smaller its kept lists are copied to every block inside.  s.b_q is the last stage's
// block size: the workspace of that shape has room for every stage.
static int32_t prune_all_subdivided(const ihip_shape &s, const ihip_tensor &q, const ihip_tensor &k, int n_stages,
                                    const int32_t *chunks, const int32_t *keeps, const int32_t *stage_b_q,
                                    int32_t *out_block_starts, char *ws, const ihip_rope *rope, bool all_heads,
                                    hipStream_t st, const KvFormat *fmt)
{
    const PlanLayout L = plan_layout(s, n_stages, chunks, keeps);
    int32_t *buf[2] = {(int32_t *)(ws + L.starts_off[0]), (int32_t *)(ws + L.starts_off[1])};
    float *scores = (float *)(ws + L.scores_off);
    const int32_t *parents = nullptr;
    for (int i = 0; i < n_stages; ++i) {
        ihip_shape si = s;
        si.b_q = stage_b_q[i];
        si.b_q_range = stage_b_q[0];
        const int n_parent = i == 0 ? 0 : keeps[i - 1];
        const int parent_chunk = i == 0 ? 0 : chunks[i - 1];
        const int slots = i == 0 ? stage1_slots(si, chunks[0]) : n_parent * (parent_chunk / chunks[i]);
        int32_t *out = i + 1 == n_stages ? out_block_starts : (parents == buf[0] ? buf[1] : buf[0]);
        int32_t rc = launch_prune_stage(si, q, k, parents, n_parent, parent_chunk, chunks[i], slots, scores, nullptr,
                                        nullptr, rope, st, fmt);
        if (rc != IHIP_OK) return rc;
        rc = launch_select_blocks(si, scores, slots, parents, n_parent, parent_chunk, chunks[i], keeps[i], out,
                                  all_heads, st);
        if (rc != IHIP_OK) return rc;
        parents = out;
        if (i + 1 < n_stages && stage_b_q[i + 1] != stage_b_q[i]) {
            int32_t *finer = out == buf[0] ? buf[1] : buf[0];
            if ((rc = launch_subdivide_blocks(si, out, keeps[i], stage_b_q[i + 1], finer, st)) != IHIP_OK) return rc;
            parents = finer;
        }
    }
    return IHIP_OK;
}

static int32_t prune_all_impl(const ihip_shape &s, const ihip_tensor &q, const ihip_tensor &k, int n_stages,
                              const int32_t *chunks, const int32_t *keeps, int32_t *out_block_starts,
                              char *ws, const BankView *bank, const ihip_rope *rope, bool all_heads, hipStream_t st,
                              const KvFormat *fmt = nullptr)
{
    const PlanLayout L = plan_layout(s, n_stages, chunks, keeps);
    int32_t *stage_out[8];
    for (int i = 0; i < n_stages; ++i)
        stage_out[i] = (i + 1 == n_stages) ? out_block_starts : (int32_t *)(ws + L.starts_off[i & 1]);
    return prune_stages_impl(s, q, k, n_stages, chunks, keeps, ~0u, stage_out, (float *)(ws + L.scores_off), bank, rope, all_heads, st, fmt);
}

}  // namespace ihip

using namespace ihip;

extern "C" {

const char *ihip_last_error(void) { return g_err; }
int32_t ihip_version(void) { return 100; }

int32_t ihip_mfma_rate(int32_t kind, int32_t iters, float *scratch, double *tflops, void *stream)
{
    if ((kind != 0 && kind != 1) || iters <= 0 || iters > (1 << 22) || !scratch || !tflops)
        return fail(IHIP_ERR_INVALID_ARG, "ihip_mfma_rate: kind in {0,1}, 1 <= iters <= 2^22, scratch and tflops non-NULL");
    const double r = measure_mfma_rate(kind, iters, scratch, (hipStream_t)stream);
    if (r < 0.0) return fail(IHIP_ERR_HIP, "ihip_mfma_rate: HIP error while timing");
    *tflops = r;
    return IHIP_OK;
}

int32_t ihip_stage1_slots(const ihip_shape *shape, int32_t chunk)
{
    if (check_shape(shape, "ihip_stage1_slots") != IHIP_OK || !pow2(chunk)) return -1;
    return stage1_slots(*shape, chunk);
}

static int32_t prune_stage_entry(const char *who, const ihip_rope *rope, const KvFormat *fmt, const ihip_shape *shape, ihip_tensor q, ihip_tensor k, const int32_t *parent_starts,
                         int32_t n_parent, int32_t parent_chunk, int32_t chunk, int32_t max_chunks,
                         float *out_scores, int32_t *out_rep, void *stream, const BankView *bank = nullptr)
{
    int32_t rc;
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;          // an empty batch: nothing to do, no pointer is looked at
    if ((rc = check_tensor(q, who, "q")) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(k, who, "k") : check_tensor(k, who, "k"))) != IHIP_OK) return rc;
    if ((rc = check_slots(who, parent_starts, n_parent, parent_chunk, chunk, max_chunks)) != IHIP_OK) return rc;
    if (!parent_starts && max_chunks < stage1_slots(*shape, chunk))
        return fail(IHIP_ERR_INVALID_ARG, "%s: max_chunks = %d < %d slots of the first stage", who, max_chunks,
                    stage1_slots(*shape, chunk));
    if (!out_scores && max_chunks > 0) return fail(IHIP_ERR_INVALID_ARG, "%s: out_scores is NULL", who);
    if (shape->b_q == 1 && shape->Tq != 1)
        return fail(IHIP_ERR_INVALID_ARG, "%s: b_q == 1 is the decode path and needs Tq == 1", who);
    return launch_prune_stage(*shape, q, k, parent_starts, n_parent, parent_chunk, chunk, max_chunks, out_scores,
                              out_rep, bank, rope, (hipStream_t)stream, fmt);
}

int32_t ihip_prune_stage(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, const int32_t *parent_starts,
                         int32_t n_parent, int32_t parent_chunk, int32_t chunk, int32_t max_chunks,
                         float *out_scores, int32_t *out_rep, void *stream)
{
    return prune_stage_entry("ihip_prune_stage", nullptr, nullptr, shape, q, k, parent_starts, n_parent, parent_chunk, chunk,
                             max_chunks, out_scores, out_rep, stream);
}

int32_t ihip_prune_stage_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, const int32_t *parent_starts,
                              int32_t n_parent, int32_t parent_chunk, int32_t chunk, int32_t max_chunks,
                              const ihip_rope *rope, float *out_scores, int32_t *out_rep, void *stream)
{
    if (!rope) return fail(IHIP_ERR_INVALID_ARG, "ihip_prune_stage_rope: rope is NULL");
    return prune_stage_entry("ihip_prune_stage_rope", rope, nullptr, shape, q, k, parent_starts, n_parent, parent_chunk, chunk,
                             max_chunks, out_scores, out_rep, stream);
}

static int32_t select_blocks_entry(const char *who, bool all_heads, const ihip_shape *shape, const float *scores, int32_t max_chunks,
                           const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk, int32_t chunk,
                           int32_t keep, int32_t *out_starts, void *stream)
{
    int32_t rc;
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;          // an empty batch: nothing to do, no pointer is looked at
    if ((rc = check_slots(who, parent_starts, n_parent, parent_chunk, chunk, max_chunks)) != IHIP_OK) return rc;
    if (keep < 0) return fail(IHIP_ERR_INVALID_ARG, "%s: keep = %d", who, keep);
    if (max_chunks > 65535 * 16) return fail(IHIP_ERR_UNSUPPORTED, "%s: max_chunks = %d too large", who, max_chunks);
    if ((!scores && max_chunks > 0) || (!out_starts && keep > 0))
        return fail(IHIP_ERR_INVALID_ARG, "%s: scores / out_starts is NULL", who);
    return launch_select_blocks(*shape, scores, max_chunks, parent_starts, n_parent, parent_chunk, chunk, keep,
                                out_starts, all_heads, (hipStream_t)stream);
}

int32_t ihip_prune_stage_fp8kv(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, const int32_t *parent_starts,
                               int32_t n_parent, int32_t parent_chunk, int32_t chunk, int32_t max_chunks,
                               float k_scale, float *out_scores, int32_t *out_rep, void *stream)
{
    const int32_t rc = check_scales("ihip_prune_stage_fp8kv", k_scale, 1.0f);
    if (rc != IHIP_OK) return rc;
    const KvFormat fmt{true, k_scale, 1.0f};
    return prune_stage_entry("ihip_prune_stage_fp8kv", nullptr, &fmt, shape, q, k, parent_starts, n_parent,
                             parent_chunk, chunk, max_chunks, out_scores, out_rep, stream);
}

int32_t ihip_prune_stage_paged(const ihip_shape *shape, ihip_tensor q, ihip_tensor k_pool, const ihip_paged_kv *paged,
                               const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk, int32_t chunk,
                               int32_t max_chunks, float *out_scores, int32_t *out_rep, void *stream)
{
    KvFormat fmt;
    const int32_t rc = check_paged("ihip_prune_stage_paged", shape, paged, &fmt);
    if (rc != IHIP_OK) return rc;
    return prune_stage_entry("ihip_prune_stage_paged", nullptr, &fmt, shape, q, k_pool, parent_starts, n_parent,
                             parent_chunk, chunk, max_chunks, out_scores, out_rep, stream);
}

int32_t ihip_subdivide_blocks(const ihip_shape *shape, const int32_t *starts, int32_t n, int32_t b_q_fine,
                              int32_t *out_starts, void *stream)
{
    const char *who = "ihip_subdivide_blocks";
    int32_t rc;
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;          // an empty batch: nothing to do, no pointer is looked at
    if (b_q_fine <= 0 || shape->b_q % b_q_fine != 0)
        return fail(IHIP_ERR_INVALID_ARG, "%s: b_q_fine = %d must divide b_q = %d", who, b_q_fine, shape->b_q);
    if (n < 0 || (n > 0 && (!starts || !out_starts)) || starts == out_starts)
        return fail(IHIP_ERR_INVALID_ARG, "%s: n = %d, starts / out_starts NULL or the same buffer", who, n);
    return launch_subdivide_blocks(*shape, starts, n, b_q_fine, out_starts, (hipStream_t)stream);
}

int32_t ihip_select_blocks(const ihip_shape *shape, const float *scores, int32_t max_chunks,
                           const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk, int32_t chunk,
                           int32_t keep, int32_t *out_starts, void *stream)
{
    return select_blocks_entry("ihip_select_blocks", false, shape, scores, max_chunks, parent_starts, n_parent,
                               parent_chunk, chunk, keep, out_starts, stream);
}

static int32_t check_pooling(const char *who, int32_t pooling)
{
    if (pooling != IHIP_POOL_KV_HEAD && pooling != IHIP_POOL_ALL_HEADS)
        return fail(IHIP_ERR_INVALID_ARG, "%s: pooling = %d", who, pooling);
    return IHIP_OK;
}

int32_t ihip_select_blocks_pooled(const ihip_shape *shape, const float *scores, int32_t max_chunks,
                                  const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk,
                                  int32_t chunk, int32_t keep, int32_t pooling, int32_t *out_starts, void *stream)
{
    const int32_t rc = check_pooling("ihip_select_blocks_pooled", pooling);
    if (rc != IHIP_OK) return rc;
    return select_blocks_entry("ihip_select_blocks_pooled", pooling == IHIP_POOL_ALL_HEADS, shape, scores, max_chunks,
                               parent_starts, n_parent, parent_chunk, chunk, keep, out_starts, stream);
}

static int32_t attn_decode_entry(const char *who, const ihip_rope *rope, const KvFormat *fmt, const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                const int32_t *block_starts, int32_t n_blocks, int32_t block, float sm_scale,
                                void *out, float *out_lse, void *ws, size_t ws_bytes, void *stream,
                                const BankView *bank = nullptr)
{
    int32_t rc;
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;          // an empty batch: nothing to do, no pointer is looked at
    if (shape->Tq != 1 || shape->b_q != 1) return fail(IHIP_ERR_INVALID_ARG, "%s: needs Tq == b_q == 1", who);
    if ((rc = check_tensor(q, who, "q")) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(k, who, "k") : check_tensor(k, who, "k"))) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(v, who, "v") : check_tensor(v, who, "v"))) != IHIP_OK) return rc;
    if (n_blocks < 0 || !pow2(block)) return fail(IHIP_ERR_INVALID_ARG, "%s: n_blocks = %d, block = %d", who, n_blocks, block);
    if (n_blocks > 0 && !block_starts) return fail(IHIP_ERR_INVALID_ARG, "%s: block_starts is NULL", who);
    if (!out) return fail(IHIP_ERR_INVALID_ARG, "%s: out is NULL", who);
    const size_t need = attn_decode_workspace(*shape, n_blocks, block);
    if (!ws || ws_bytes < need)
        return fail(IHIP_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need, ws_bytes);
    return launch_attn_decode(*shape, q, k, v, block_starts, n_blocks, block, sm_scale, out, out_lse, ws,
                              bank, rope, (hipStream_t)stream, fmt);
}

int32_t ihip_sparse_attn_decode(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                const int32_t *block_starts, int32_t n_blocks, int32_t block, float sm_scale,
                                void *out, float *out_lse, void *ws, size_t ws_bytes, void *stream)
{
    return attn_decode_entry("ihip_sparse_attn_decode", nullptr, nullptr, shape, q, k, v, block_starts, n_blocks, block,
                             sm_scale, out, out_lse, ws, ws_bytes, stream);
}

int32_t ihip_sparse_attn_decode_fp8kv(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                      const int32_t *block_starts, int32_t n_blocks, int32_t block, float sm_scale,
                                      float k_scale, float v_scale, void *out, float *out_lse, void *ws,
                                      size_t ws_bytes, void *stream)
{
    const int32_t rc = check_scales("ihip_sparse_attn_decode_fp8kv", k_scale, v_scale);
    if (rc != IHIP_OK) return rc;
    const KvFormat fmt{true, k_scale, v_scale};
    return attn_decode_entry("ihip_sparse_attn_decode_fp8kv", nullptr, &fmt, shape, q, k, v, block_starts, n_blocks,
                             block, sm_scale, out, out_lse, ws, ws_bytes, stream);
}

int32_t ihip_sparse_attn_decode_paged(const ihip_shape *shape, ihip_tensor q, ihip_tensor k_pool, ihip_tensor v_pool,
                                      const ihip_paged_kv *paged, const int32_t *block_starts, int32_t n_blocks,
                                      int32_t block, float sm_scale, void *out, float *out_lse, void *ws,
                                      size_t ws_bytes, void *stream)
{
    KvFormat fmt;
    const int32_t rc = check_paged("ihip_sparse_attn_decode_paged", shape, paged, &fmt);
    if (rc != IHIP_OK) return rc;
    return attn_decode_entry("ihip_sparse_attn_decode_paged", nullptr, &fmt, shape, q, k_pool, v_pool, block_starts,
                             n_blocks, block, sm_scale, out, out_lse, ws, ws_bytes, stream);
}

int32_t ihip_sparse_attn_decode_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                     const int32_t *block_starts, int32_t n_blocks, int32_t block, float sm_scale,
                                     const ihip_rope *rope, void *out, float *out_lse, void *ws, size_t ws_bytes,
                                     void *stream)
{
    if (!rope) return fail(IHIP_ERR_INVALID_ARG, "ihip_sparse_attn_decode_rope: rope is NULL");
    return attn_decode_entry("ihip_sparse_attn_decode_rope", rope, nullptr, shape, q, k, v, block_starts, n_blocks, block,
                             sm_scale, out, out_lse, ws, ws_bytes, stream);
}

static int32_t attn_prefill_entry(const char *who, const ihip_rope *rope, const KvFormat *fmt, const ihip_shape *shape, ihip_tensor q,
                                  ihip_tensor k, ihip_tensor v, const int32_t *block_starts, int32_t n_blocks,
                                  int32_t block, float sm_scale, void *out, float *out_lse, void *ws,
                                  size_t ws_bytes, void *stream)
{
    int32_t rc;
    (void)ws; (void)ws_bytes;       // this kernel needs no scratch
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;          // an empty batch: nothing to do, no pointer is looked at
    if (shape->b_q != 16 && shape->b_q != 32 && shape->b_q != 64)
        return fail(IHIP_ERR_UNSUPPORTED, "%s: b_q = %d not in {16, 32, 64}", who, shape->b_q);
    if ((rc = check_tensor(q, who, "q")) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(k, who, "k") : check_tensor(k, who, "k"))) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(v, who, "v") : check_tensor(v, who, "v"))) != IHIP_OK) return rc;
    if (n_blocks < 0 || !pow2(block)) return fail(IHIP_ERR_INVALID_ARG, "%s: n_blocks = %d, block = %d", who, n_blocks, block);
    if (n_blocks > 0 && !block_starts) return fail(IHIP_ERR_INVALID_ARG, "%s: block_starts is NULL", who);
    if (!out) return fail(IHIP_ERR_INVALID_ARG, "%s: out is NULL", who);
    return launch_attn_prefill(*shape, q, k, v, block_starts, n_blocks, block, sm_scale, out, out_lse, rope,
                               (hipStream_t)stream, fmt);
}

int32_t ihip_sparse_attn_prefill_fp8kv(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                       const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                       float sm_scale, float k_scale, float v_scale, const ihip_rope *rope,
                                       void *out, float *out_lse, void *ws, size_t ws_bytes, void *stream)
{
    const int32_t rc = check_scales("ihip_sparse_attn_prefill_fp8kv", k_scale, v_scale);
    if (rc != IHIP_OK) return rc;
    const KvFormat fmt{true, k_scale, v_scale, PagedView{nullptr, 0, 0}};
    return attn_prefill_entry("ihip_sparse_attn_prefill_fp8kv", rope, &fmt, shape, q, k, v, block_starts, n_blocks,
                              block, sm_scale, out, out_lse, ws, ws_bytes, stream);
}

int32_t ihip_sparse_attn_prefill_paged(const ihip_shape *shape, ihip_tensor q, ihip_tensor k_pool, ihip_tensor v_pool,
                                       const ihip_paged_kv *paged, const int32_t *block_starts, int32_t n_blocks,
                                       int32_t block, float sm_scale, const ihip_rope *rope, void *out,
                                       float *out_lse, void *ws, size_t ws_bytes, void *stream)
{
    KvFormat fmt;
    const int32_t rc = check_paged("ihip_sparse_attn_prefill_paged", shape, paged, &fmt);
    if (rc != IHIP_OK) return rc;
    return attn_prefill_entry("ihip_sparse_attn_prefill_paged", rope, &fmt, shape, q, k_pool, v_pool, block_starts,
                              n_blocks, block, sm_scale, out, out_lse, ws, ws_bytes, stream);
}

int32_t ihip_sparse_attn_prefill(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                 const int32_t *block_starts, int32_t n_blocks, int32_t block, float sm_scale,
                                 void *out, float *out_lse, void *ws, size_t ws_bytes, void *stream)
{
    return attn_prefill_entry("ihip_sparse_attn_prefill", nullptr, nullptr, shape, q, k, v, block_starts, n_blocks, block,
                              sm_scale, out, out_lse, ws, ws_bytes, stream);
}

int32_t ihip_sparse_attn_prefill_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                      const int32_t *block_starts, int32_t n_blocks, int32_t block, float sm_scale,
                                      const ihip_rope *rope, void *out, float *out_lse, void *ws, size_t ws_bytes,
                                      void *stream)
{
    if (!rope) return fail(IHIP_ERR_INVALID_ARG, "ihip_sparse_attn_prefill_rope: rope is NULL");
    return attn_prefill_entry("ihip_sparse_attn_prefill_rope", rope, nullptr, shape, q, k, v, block_starts, n_blocks, block,
                              sm_scale, out, out_lse, ws, ws_bytes, stream);
}

int32_t ihip_prune_all(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, int32_t n_stages,
                       const int32_t *chunk_sizes, const int32_t *keeps, int32_t *out_block_starts, void *ws,
                       size_t ws_bytes, void *stream)
{
    const char *who = "ihip_prune_all";
    int32_t rc;
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;          // an empty batch: nothing to do, no pointer is looked at
    if ((rc = check_tensor(q, who, "q")) != IHIP_OK) return rc;
    if ((rc = check_tensor(k, who, "k")) != IHIP_OK) return rc;
    if ((rc = check_plan(who, shape, n_stages, chunk_sizes, keeps)) != IHIP_OK) return rc;
    if (!out_block_starts) return fail(IHIP_ERR_INVALID_ARG, "%s: out_block_starts is NULL", who);
    const size_t need = plan_layout(*shape, n_stages, chunk_sizes, keeps).total;
    if (!ws || ws_bytes < need)
        return fail(IHIP_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need, ws_bytes);
    return prune_all_impl(*shape, q, k, n_stages, chunk_sizes, keeps, out_block_starts, (char *)ws, nullptr, nullptr,
                          false, (hipStream_t)stream);
}

// stage_starts != NULL: mask caching (the caller's per-stage lists; stages first_stage.. are recomputed,
// or, with stage_due, exactly the stages whose entry is non-zero)
static int32_t decode_layer_impl(const char *who, const ihip_shape *shape, ihip_tensor q, ihip_tensor k,
                                 ihip_tensor v, const ihip_cache *cache, const ihip_rope *rope, bool all_heads,
                                 const KvFormat *fmt, int32_t n_stages,
                                 const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale, void *out,
                                 float *out_lse, int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream,
                                 int32_t first_stage = 0, int32_t *stage_starts = nullptr,
                                 const int32_t *stage_due = nullptr)
{
    int32_t rc;
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;          // an empty batch: nothing to do, no pointer is looked at
    if (shape->Tq != 1 || shape->b_q != 1) return fail(IHIP_ERR_INVALID_ARG, "%s: needs Tq == b_q == 1", who);
    if ((rc = check_tensor(q, who, "q")) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(k, who, "k") : check_tensor(k, who, "k"))) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(v, who, "v") : check_tensor(v, who, "v"))) != IHIP_OK) return rc;
    if ((rc = check_plan(who, shape, n_stages, chunk_sizes, keeps)) != IHIP_OK) return rc;
    if (!out) return fail(IHIP_ERR_INVALID_ARG, "%s: out is NULL", who);
    const int last = n_stages - 1;
    const PlanLayout L = plan_layout(*shape, n_stages, chunk_sizes, keeps);
    const size_t P = (size_t)shape->B * shape->Hkv;
    const size_t blocks_bytes = align256(P * keeps[last] * sizeof(int32_t));
    const size_t attn_bytes = attn_decode_workspace(*shape, keeps[last], chunk_sizes[last]);
    BankView mask_bank, sa_bank;
    if (cache) {
        if ((rc = refuse_capture(who, (hipStream_t)stream)) != IHIP_OK) return rc;
        mask_bank = cache_bank_view(cache, 0);
        sa_bank = cache_bank_view(cache, 1);
    }
    if (stage_starts) {
        if (first_stage < 0 || first_stage > n_stages)
            return fail(IHIP_ERR_INVALID_ARG, "%s: first_stage = %d not in 0..%d", who, first_stage, n_stages);
        const size_t need = L.scores_bytes + attn_bytes;
        if (!ws || ws_bytes < need)
            return fail(IHIP_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need, ws_bytes);
        int32_t *stage_out[8];
        size_t off = 0;
        for (int i = 0; i < n_stages; ++i) { stage_out[i] = stage_starts + off; off += P * (size_t)keeps[i]; }
        uint32_t due = 0;
        for (int i = 0; i < n_stages; ++i)
            if (stage_due ? stage_due[i] != 0 : i >= first_stage) due |= 1u << i;
        rc = prune_stages_impl(*shape, q, k, n_stages, chunk_sizes, keeps, due, stage_out, (float *)ws,
                               cache ? &mask_bank : nullptr, rope, all_heads, (hipStream_t)stream, fmt);
        if (rc != IHIP_OK) return rc;
        if (out_block_starts &&
            hipMemcpyAsync(out_block_starts, stage_out[last], P * keeps[last] * sizeof(int32_t),
                           hipMemcpyDeviceToDevice, (hipStream_t)stream) != hipSuccess)
            return fail(IHIP_ERR_HIP, "%s: copy of the final block list failed", who);
        return launch_attn_decode(*shape, q, k, v, stage_out[last], keeps[last], chunk_sizes[last], sm_scale, out,
                                  out_lse, (char *)ws + L.scores_bytes, cache ? &sa_bank : nullptr, rope,
                                  (hipStream_t)stream, fmt);
    }
    if (first_stage != 0 || stage_due)
        return fail(IHIP_ERR_INVALID_ARG, "%s: first_stage = %d / stage_due without stage_starts", who, first_stage);
    const size_t need = L.total + blocks_bytes + attn_bytes;
    if (!ws || ws_bytes < need)
        return fail(IHIP_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need, ws_bytes);
    char *w = (char *)ws;
    int32_t *blocks = out_block_starts ? out_block_starts : (int32_t *)(w + L.total);
    rc = prune_all_impl(*shape, q, k, n_stages, chunk_sizes, keeps, blocks, w, cache ? &mask_bank : nullptr, rope,
                        all_heads, (hipStream_t)stream, fmt);
    if (rc != IHIP_OK) return rc;
    return launch_attn_decode(*shape, q, k, v, blocks, keeps[last], chunk_sizes[last], sm_scale, out, out_lse,
                              w + L.total + blocks_bytes, cache ? &sa_bank : nullptr, rope, (hipStream_t)stream, fmt);
}

int32_t ihip_decode_layer(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v, int32_t n_stages,
                          const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale, void *out,
                          float *out_lse, int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream)
{
    return decode_layer_impl("ihip_decode_layer", shape, q, k, v, nullptr, nullptr, false, nullptr, n_stages, chunk_sizes,
                             keeps, sm_scale, out, out_lse, out_block_starts, ws, ws_bytes, stream);
}

// ---- the decode layer for callers that cannot allocate -----------------------
// Its scratch (scores, the kept lists between the stages, the final block list and the attention's
// split partials) is a device array of the library itself; every GPU holds its own copy at its own
// address, looked up once per device.  The array's name is only a host-side handle of the symbol:
// host code uses the looked-up address.
static __device__ __align__(256) unsigned char scratch[IHIP_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

int32_t static_scratch(const char *who, void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(IHIP_ERR_HIP, "%s: hipGetDevice: %s", who, hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(IHIP_ERR_UNSUPPORTED, "%s: device %d beyond %d", who, dev, kMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(IHIP_ERR_HIP, "%s: hipGetSymbolAddress(scratch): %s", who, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return IHIP_OK;
}
}  // namespace

int32_t ihip_decode_layer_static(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                 int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                 float sm_scale, void *out, float *out_lse, int32_t *out_block_starts, void *stream)
{
    const char *who = "ihip_decode_layer_static";
    int32_t rc;
    // sizes first: a plan that does not fit the array is refused before anything is looked up or enqueued
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;
    if (shape->Tq != 1 || shape->b_q != 1) return fail(IHIP_ERR_INVALID_ARG, "%s: needs Tq == b_q == 1", who);
    if ((rc = check_plan(who, shape, n_stages, chunk_sizes, keeps)) != IHIP_OK) return rc;
    const size_t need = plan_layout(*shape, n_stages, chunk_sizes, keeps).total +
                        align256((size_t)shape->B * shape->Hkv * keeps[n_stages - 1] * sizeof(int32_t)) +
                        attn_decode_workspace(*shape, keeps[n_stages - 1], chunk_sizes[n_stages - 1]);
    if (need > (size_t)IHIP_STATIC_SCRATCH_BYTES)
        return fail(IHIP_ERR_WORKSPACE, "%s: this shape and plan need %zu bytes of scratch, the static array holds %zu",
                    who, need, (size_t)IHIP_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    if ((rc = static_scratch(who, &ws)) != IHIP_OK) return rc;
    // nothing in the scratch has to start at zero: every score, list entry and partial that a kernel
    // reads was written earlier in the same call
    return decode_layer_impl(who, shape, q, k, v, nullptr, nullptr, false, nullptr, n_stages, chunk_sizes, keeps,
                             sm_scale, out, out_lse, out_block_starts, ws, IHIP_STATIC_SCRATCH_BYTES, stream);
}

int32_t ihip_decode_layer_pooled(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                 int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps, int32_t pooling,
                                 float sm_scale, void *out, float *out_lse, int32_t *out_block_starts, void *ws,
                                 size_t ws_bytes, void *stream)
{
    const int32_t rc = check_pooling("ihip_decode_layer_pooled", pooling);
    if (rc != IHIP_OK) return rc;
    return decode_layer_impl("ihip_decode_layer_pooled", shape, q, k, v, nullptr, nullptr,
                             pooling == IHIP_POOL_ALL_HEADS, nullptr, n_stages, chunk_sizes, keeps, sm_scale, out, out_lse,
                             out_block_starts, ws, ws_bytes, stream);
}

int32_t ihip_decode_layer_fp8kv(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v, int32_t n_stages,
                                const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale, float k_scale,
                                float v_scale, void *out, float *out_lse, int32_t *out_block_starts, void *ws,
                                size_t ws_bytes, void *stream)
{
    const int32_t rc = check_scales("ihip_decode_layer_fp8kv", k_scale, v_scale);
    if (rc != IHIP_OK) return rc;
    const KvFormat fmt{true, k_scale, v_scale};
    return decode_layer_impl("ihip_decode_layer_fp8kv", shape, q, k, v, nullptr, nullptr, false, &fmt, n_stages,
                             chunk_sizes, keeps, sm_scale, out, out_lse, out_block_starts, ws, ws_bytes, stream);
}

int32_t ihip_decode_layer_paged(const ihip_shape *shape, ihip_tensor q, ihip_tensor k_pool, ihip_tensor v_pool,
                                const ihip_paged_kv *paged, int32_t n_stages, const int32_t *chunk_sizes,
                                const int32_t *keeps, float sm_scale, void *out, float *out_lse,
                                int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream)
{
    KvFormat fmt;
    const int32_t rc = check_paged("ihip_decode_layer_paged", shape, paged, &fmt);
    if (rc != IHIP_OK) return rc;
    return decode_layer_impl("ihip_decode_layer_paged", shape, q, k_pool, v_pool, nullptr, nullptr, false, &fmt,
                             n_stages, chunk_sizes, keeps, sm_scale, out, out_lse, out_block_starts, ws, ws_bytes,
                             stream);
}

int32_t ihip_decode_layer_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v, int32_t n_stages,
                               const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale, const ihip_rope *rope,
                               void *out, float *out_lse, int32_t *out_block_starts, void *ws, size_t ws_bytes,
                               void *stream)
{
    if (!rope) return fail(IHIP_ERR_INVALID_ARG, "ihip_decode_layer_rope: rope is NULL");
    return decode_layer_impl("ihip_decode_layer_rope", shape, q, k, v, nullptr, rope, false, nullptr, n_stages, chunk_sizes, keeps,
                             sm_scale, out, out_lse, out_block_starts, ws, ws_bytes, stream);
}

int32_t ihip_decode_layer_cached(const ihip_shape *shape, ihip_tensor q, ihip_cache *cache, int32_t n_stages,
                                 const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale, void *out,
                                 float *out_lse, int32_t *out_block_starts, void *ws, size_t ws_bytes,
                                 void *stream)
{
    const char *who = "ihip_decode_layer_cached";
    if (!cache) return fail(IHIP_ERR_INVALID_ARG, "%s: cache is NULL", who);
    if (cache_holds_fp8(cache))
        return fail(IHIP_ERR_INVALID_ARG, "%s: the host tier holds E4M3 rows: pass the scales through ihip_decode_layer_ex", who);
    int32_t B, Hkv;
    int64_t T_alloc;
    ihip_tensor hk, hv;
    cache_describe(cache, &B, &Hkv, &T_alloc, &hk, &hv);
    if (shape && (shape->B != B || shape->Hkv != Hkv || shape->max_seq_len > T_alloc))
        return fail(IHIP_ERR_INVALID_ARG, "%s: shape (B %d, Hkv %d, max_seq_len %d) does not fit the cache (%d, %d, %lld)",
                    who, shape->B, shape->Hkv, shape->max_seq_len, B, Hkv, (long long)T_alloc);
    return decode_layer_impl(who, shape, q, hk, hv, cache, nullptr, false, nullptr, n_stages, chunk_sizes, keeps, sm_scale, out, out_lse,
                             out_block_starts, ws, ws_bytes, stream);
}

// what the stage-by-stage calls through the host tier share: the cache fits the shape; E4M3 tiers
// bring their scales
static int32_t cached_stage_setup(const char *who, const ihip_shape *shape, const ihip_cache *cache, float k_scale,
                                  float v_scale, ihip_tensor *hk, ihip_tensor *hv, KvFormat *fmt, bool *fp8)
{
    if (!cache) return fail(IHIP_ERR_INVALID_ARG, "%s: cache is NULL", who);
    int32_t B, Hkv;
    int64_t T_alloc;
    cache_describe(cache, &B, &Hkv, &T_alloc, hk, hv);
    if (shape && (shape->B != B || shape->Hkv != Hkv || shape->max_seq_len > T_alloc))
        return fail(IHIP_ERR_INVALID_ARG, "%s: shape (B %d, Hkv %d, max_seq_len %d) does not fit the cache (%d, %d, %lld)",
                    who, shape->B, shape->Hkv, shape->max_seq_len, B, Hkv, (long long)T_alloc);
    *fp8 = cache_holds_fp8(cache);
    *fmt = KvFormat{*fp8, 1.0f, 1.0f, PagedView{nullptr, 0, 0}};
    if (*fp8) {
        const int32_t rc = check_scales(who, k_scale, v_scale);
        if (rc != IHIP_OK) return rc;
        fmt->k_scale = k_scale;
        fmt->v_scale = v_scale;
    }
    return IHIP_OK;
}

int32_t ihip_prune_stage_cached(const ihip_shape *shape, ihip_tensor q, ihip_cache *cache, const int32_t *parent_starts,
                                int32_t n_parent, int32_t parent_chunk, int32_t chunk, int32_t max_chunks,
                                const ihip_rope *rope, float k_scale, float *out_scores, int32_t *out_rep,
                                void *stream)
{
    const char *who = "ihip_prune_stage_cached";
    ihip_tensor hk, hv;
    KvFormat fmt;
    bool fp8;
    int32_t rc = cached_stage_setup(who, shape, cache, k_scale, 1.0f, &hk, &hv, &fmt, &fp8);
    if (rc != IHIP_OK) return rc;
    if ((rc = refuse_capture(who, (hipStream_t)stream)) != IHIP_OK) return rc;
    const BankView bank = cache_bank_view(cache, 0);
    return prune_stage_entry(who, rope, fp8 ? &fmt : nullptr, shape, q, hk, parent_starts, n_parent, parent_chunk,
                             chunk, max_chunks, out_scores, out_rep, stream, &bank);
}

int32_t ihip_sparse_attn_decode_cached(const ihip_shape *shape, ihip_tensor q, ihip_cache *cache,
                                       const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                       float sm_scale, const ihip_rope *rope, float k_scale, float v_scale,
                                       void *out, float *out_lse, void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "ihip_sparse_attn_decode_cached";
    ihip_tensor hk, hv;
    KvFormat fmt;
    bool fp8;
    int32_t rc = cached_stage_setup(who, shape, cache, k_scale, v_scale, &hk, &hv, &fmt, &fp8);
    if (rc != IHIP_OK) return rc;
    if ((rc = refuse_capture(who, (hipStream_t)stream)) != IHIP_OK) return rc;
    const BankView bank = cache_bank_view(cache, 1);
    return attn_decode_entry(who, rope, fp8 ? &fmt : nullptr, shape, q, hk, hv, block_starts, n_blocks, block,
                             sm_scale, out, out_lse, ws, ws_bytes, stream, &bank);
}

size_t ihip_mask_state_elems(const ihip_shape *shape, int32_t n_stages, const int32_t *keeps)
{
    if (check_shape(shape, "ihip_mask_state_elems") != IHIP_OK || n_stages < 1 || n_stages > 8 || !keeps) return 0;
    const size_t P = (size_t)shape->B * shape->Hkv * (shape->Tq / shape->b_q);
    size_t n = 0;
    for (int i = 0; i < n_stages; ++i) n += P * (size_t)keeps[i];
    return n;
}

int32_t ihip_decode_layer_masked(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                 int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                 int32_t first_stage, int32_t *stage_starts, float sm_scale, void *out,
                                 float *out_lse, void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "ihip_decode_layer_masked";
    if (!stage_starts) return fail(IHIP_ERR_INVALID_ARG, "%s: out / stage_starts is NULL", who);
    return decode_layer_impl(who, shape, q, k, v, nullptr, nullptr, false, nullptr, n_stages, chunk_sizes, keeps,
                             sm_scale, out, out_lse, nullptr, ws, ws_bytes, stream, first_stage, stage_starts);
}

int32_t ihip_decode_layer_ex(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v, int32_t n_stages,
                             const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale,
                             const ihip_decode_options *opt, void *out, float *out_lse, int32_t *out_block_starts,
                             void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "ihip_decode_layer_ex";
    if (!opt) return fail(IHIP_ERR_INVALID_ARG, "%s: options are NULL", who);
    int32_t rc;
    KvFormat fmt{false, 1.0f, 1.0f, PagedView{nullptr, 0, 0}};
    if (opt->paged && (rc = check_paged(who, shape, opt->paged, &fmt)) != IHIP_OK) return rc;
    if (opt->kv_fp8) {
        if ((rc = check_scales(who, opt->k_scale, opt->v_scale)) != IHIP_OK) return rc;
        fmt.fp8 = true; fmt.k_scale = opt->k_scale; fmt.v_scale = opt->v_scale;
    }
    if ((rc = check_pooling(who, opt->pooling)) != IHIP_OK) return rc;
    if ((opt->first_stage != 0 || opt->stage_due) && !opt->stage_starts)
        return fail(IHIP_ERR_INVALID_ARG, "%s: first_stage = %d / stage_due without stage_starts", who, opt->first_stage);
    if (opt->stage_due && opt->first_stage != 0)
        return fail(IHIP_ERR_INVALID_ARG, "%s: stage_due and first_stage = %d exclude each other", who, opt->first_stage);
    if (opt->cache) {
        if (opt->paged) return fail(IHIP_ERR_UNSUPPORTED, "%s: the host tier holds contiguous K/V", who);
        if (cache_holds_fp8(opt->cache) != (opt->kv_fp8 != 0))
            return fail(IHIP_ERR_INVALID_ARG, "%s: the host tier holds %s rows", who,
                        cache_holds_fp8(opt->cache) ? "E4M3" : "bf16");
        int32_t B, Hkv;
        int64_t T_alloc;
        cache_describe(opt->cache, &B, &Hkv, &T_alloc, &k, &v);
        if (shape && (shape->B != B || shape->Hkv != Hkv || shape->max_seq_len > T_alloc))
            return fail(IHIP_ERR_INVALID_ARG, "%s: shape (B %d, Hkv %d, max_seq_len %d) does not fit the cache (%d, %d, %lld)",
                        who, shape->B, shape->Hkv, shape->max_seq_len, B, Hkv, (long long)T_alloc);
    }
    const bool plain = !opt->paged && !opt->kv_fp8;
    return decode_layer_impl(who, shape, q, k, v, opt->cache, opt->rope, opt->pooling == IHIP_POOL_ALL_HEADS,
                             plain ? nullptr : &fmt, n_stages, chunk_sizes, keeps, sm_scale, out, out_lse,
                             out_block_starts, ws, ws_bytes, stream, opt->first_stage, opt->stage_starts, opt->stage_due);
}

int32_t ihip_refresh_due(int32_t n_stages, const int32_t *n_refresh, int64_t step, int32_t *stage_due)
{
    const char *who = "ihip_refresh_due";
    if (n_stages < 1 || n_stages > 8 || !n_refresh || step < 0)
        return fail(IHIP_ERR_INVALID_ARG, "%s: need 1..8 stages, their intervals and step >= 0", who);
    int32_t first = n_stages;
    for (int i = 0; i < n_stages; ++i) {
        if (n_refresh[i] < 1) return fail(IHIP_ERR_INVALID_ARG, "%s: n_refresh[%d] = %d", who, i, n_refresh[i]);
        // the counter of stage i starts at 0 and advances by one per step modulo its interval
        const bool due = step % n_refresh[i] == 0;
        if (stage_due) stage_due[i] = due ? 1 : 0;
        if (due && first == n_stages) first = i;
    }
    return first;
}

static int32_t prefill_layer_impl(const char *who, bool all_heads, const ihip_rope *rope, const KvFormat *fmt, const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v, int32_t n_stages,
                           const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale, void *out,
                           float *out_lse, int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream,
                           const int32_t *stage_b_q = nullptr)
{
    int32_t rc;
    if ((rc = check_shape(shape, who)) != IHIP_OK) return rc;
    if (shape->B == 0) return IHIP_OK;          // an empty batch: nothing to do, no pointer is looked at
    if (shape->b_q != 16 && shape->b_q != 32 && shape->b_q != 64)
        return fail(IHIP_ERR_UNSUPPORTED, "%s: b_q = %d not in {16, 32, 64}", who, shape->b_q);
    if ((rc = check_tensor(q, who, "q")) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(k, who, "k") : check_tensor(k, who, "k"))) != IHIP_OK) return rc;
    if ((rc = (fmt && fmt->fp8 ? check_tensor8(v, who, "v") : check_tensor(v, who, "v"))) != IHIP_OK) return rc;
    if ((rc = check_plan(who, shape, n_stages, chunk_sizes, keeps)) != IHIP_OK) return rc;
    if (!out) return fail(IHIP_ERR_INVALID_ARG, "%s: out is NULL", who);
    const int last = n_stages - 1;
    const PlanLayout L = plan_layout(*shape, n_stages, chunk_sizes, keeps);
    const size_t P = (size_t)shape->B * shape->Hkv * (shape->Tq / shape->b_q);
    const size_t blocks_bytes = align256(P * keeps[last] * sizeof(int32_t));
    const size_t need = L.total + blocks_bytes;
    if (!ws || ws_bytes < need)
        return fail(IHIP_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need, ws_bytes);
    char *w = (char *)ws;
    int32_t *blocks = out_block_starts ? out_block_starts : (int32_t *)(w + L.total);
    ihip_shape attn_shape = *shape;
    if (stage_b_q) {
        for (int i = 0; i < n_stages; ++i) {
            const int bq = stage_b_q[i];
            if ((bq != 16 && bq != 32 && bq != 64) || (i > 0 && (bq > stage_b_q[i - 1] || stage_b_q[i - 1] % bq != 0)))
                return fail(IHIP_ERR_INVALID_ARG, "%s: stage_b_q[%d] = %d: need 16, 32 or 64, not above the stage before", who, i, bq);
        }
        if (stage_b_q[last] != shape->b_q)
            return fail(IHIP_ERR_INVALID_ARG, "%s: the last stage's block size %d must be shape.b_q = %d", who,
                        stage_b_q[last], shape->b_q);
        if (shape->b_q_range != 0 && shape->b_q_range != stage_b_q[0])
            return fail(IHIP_ERR_INVALID_ARG, "%s: shape.b_q_range = %d, the first stage's block size is %d", who,
                        shape->b_q_range, stage_b_q[0]);
        attn_shape.b_q_range = stage_b_q[0];
        if ((rc = check_shape(&attn_shape, who)) != IHIP_OK) return rc;
        rc = prune_all_subdivided(attn_shape, q, k, n_stages, chunk_sizes, keeps, stage_b_q, blocks, w, rope, all_heads,
                                  (hipStream_t)stream, fmt);
    } else {
        rc = prune_all_impl(*shape, q, k, n_stages, chunk_sizes, keeps, blocks, w, nullptr, rope, all_heads,
                            (hipStream_t)stream, fmt);
    }
    if (rc != IHIP_OK) return rc;
    return launch_attn_prefill(attn_shape, q, k, v, blocks, keeps[last], chunk_sizes[last], sm_scale, out, out_lse,
                               rope, (hipStream_t)stream, fmt);
}

int32_t ihip_prefill_layer(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v, int32_t n_stages,
                           const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale, void *out,
                           float *out_lse, int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream)
{
    return prefill_layer_impl("ihip_prefill_layer", false, nullptr, nullptr, shape, q, k, v, n_stages, chunk_sizes, keeps, sm_scale, out,
                              out_lse, out_block_starts, ws, ws_bytes, stream);
}

int32_t ihip_prefill_layer_pooled(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                  int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                  int32_t pooling, float sm_scale, void *out, float *out_lse,
                                  int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream)
{
    const int32_t rc = check_pooling("ihip_prefill_layer_pooled", pooling);
    if (rc != IHIP_OK) return rc;
    return prefill_layer_impl("ihip_prefill_layer_pooled", pooling == IHIP_POOL_ALL_HEADS, nullptr, nullptr, shape, q, k, v, n_stages,
                              chunk_sizes, keeps, sm_scale, out, out_lse, out_block_starts, ws, ws_bytes, stream);
}

int32_t ihip_prefill_layer_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale,
                                const ihip_rope *rope, void *out, float *out_lse, int32_t *out_block_starts,
                                void *ws, size_t ws_bytes, void *stream)
{
    if (!rope) return fail(IHIP_ERR_INVALID_ARG, "ihip_prefill_layer_rope: rope is NULL");
    return prefill_layer_impl("ihip_prefill_layer_rope", false, rope, nullptr, shape, q, k, v, n_stages, chunk_sizes, keeps,
                              sm_scale, out, out_lse, out_block_starts, ws, ws_bytes, stream);
}

int32_t ihip_prefill_layer_ex(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v, int32_t n_stages,
                              const int32_t *chunk_sizes, const int32_t *keeps, float sm_scale,
                              const ihip_prefill_options *opt, void *out, float *out_lse, int32_t *out_block_starts,
                              void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "ihip_prefill_layer_ex";
    if (!opt) return fail(IHIP_ERR_INVALID_ARG, "%s: options are NULL", who);
    int32_t rc;
    KvFormat fmt{false, 1.0f, 1.0f, PagedView{nullptr, 0, 0}};
    if (opt->paged && (rc = check_paged(who, shape, opt->paged, &fmt)) != IHIP_OK) return rc;
    if ((rc = check_pooling(who, opt->pooling)) != IHIP_OK) return rc;
    if (opt->kv_fp8) {
        if ((rc = check_scales(who, opt->k_scale, opt->v_scale)) != IHIP_OK) return rc;
        fmt.fp8 = true; fmt.k_scale = opt->k_scale; fmt.v_scale = opt->v_scale;
    }
    return prefill_layer_impl(who, opt->pooling == IHIP_POOL_ALL_HEADS, opt->rope,
                              opt->paged || opt->kv_fp8 ? &fmt : nullptr, shape,
                              q, k, v, n_stages, chunk_sizes, keeps, sm_scale, out, out_lse, out_block_starts, ws,
                              ws_bytes, stream, opt->stage_b_q);
}

int32_t ihip_profile_enable(int32_t on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = on != 0;
    return IHIP_OK;
}

int32_t ihip_profile_read(int32_t max_entries, const char **names, double *total_ms, int64_t *launches)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    int n = 0;
    for (const Span &s : g_spans) {
        float ms = 0.f;
        if (hipEventSynchronize(s.t1) != hipSuccess || hipEventElapsedTime(&ms, s.t0, s.t1) != hipSuccess)
            return fail(IHIP_ERR_HIP, "ihip_profile_read: event query failed");
        int i = 0;
        while (i < n && names[i] != s.name) ++i;
        if (i == n) {
            if (n == max_entries) continue;
            names[n] = s.name; total_ms[n] = 0.0; launches[n] = 0; ++n;
        }
        total_ms[i] += ms;
        launches[i] += 1;
        g_free_events.push_back(s.t0);
        g_free_events.push_back(s.t1);
    }
    g_spans.clear();
    return n;
}

size_t ihip_workspace_bytes(int32_t op, const ihip_shape *shape, int32_t n_stages, const int32_t *chunk_sizes,
                            const int32_t *keeps)
{
    if (check_shape(shape, "ihip_workspace_bytes") != IHIP_OK) return 0;
    if (check_plan("ihip_workspace_bytes", shape, n_stages, chunk_sizes, keeps) != IHIP_OK) return 0;
    const int last = n_stages - 1;
    const size_t P = (size_t)shape->B * shape->Hkv * (shape->Tq / shape->b_q);
    switch (op) {
    case IHIP_OP_ATTN_DECODE:
        return std::max<size_t>(256, attn_decode_workspace(*shape, keeps[last], chunk_sizes[last]));
    case IHIP_OP_ATTN_PREFILL:
        return 256;
    case IHIP_OP_PRUNE_ALL:         // (never 0, which stands for an error: an empty batch needs nothing)
        return std::max<size_t>(256, plan_layout(*shape, n_stages, chunk_sizes, keeps).total);
    case IHIP_OP_DECODE_LAYER:
        return std::max<size_t>(256, plan_layout(*shape, n_stages, chunk_sizes, keeps).total +
                                         align256(P * keeps[last] * sizeof(int32_t)) +
                                         attn_decode_workspace(*shape, keeps[last], chunk_sizes[last]));
    case IHIP_OP_PREFILL_LAYER:
        return std::max<size_t>(256, plan_layout(*shape, n_stages, chunk_sizes, keeps).total +
                                         align256(P * keeps[last] * sizeof(int32_t)));
    default:
        fail(IHIP_ERR_INVALID_ARG, "ihip_workspace_bytes: unknown op %d", op);
        return 0;
    }
}

}  // extern "C"
