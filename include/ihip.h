/*
 * ihip.h -- C ABI of the MI355X (gfx950) implementation of InfiniteHiP's
 * attention hot path (arXiv 2502.08910): modular hierarchical context pruning
 * (Sec. 4 "Efficient Modular Context Pruning"; App. A, Alg. 1-3) followed by
 * block-sparse attention over sink + kept blocks + sliding window (Sec. 4,
 * first paragraph of the pruning description; Alg. 4, "perform block sparse
 * attention").
 *
 * General rules
 *  - Every pointer marked "device" is GPU memory owned by the caller; the
 *    library never allocates, frees or keeps it.  Pointers marked "host" are
 *    ordinary host memory read during the call only.
 *  - All work is enqueued on the HIP stream passed last (a hipStream_t cast to
 *    void*, NULL = the default stream); no call synchronises the device.
 *  - Tensors are bf16 with the last dimension (d) contiguous; strides are in
 *    elements.  Rows must be 16-byte aligned (ptr and every stride a multiple
 *    of 8 elements).
 *  - Every function returns 0 on success or a negative IHIP_ERR_* code; the
 *    text of the last error of the calling thread is in ihip_last_error().
 *    Nothing is enqueued when an argument check fails.
 *  - An empty batch (shape->B == 0) is no error: the call returns IHIP_OK
 *    after checking the shape, enqueues nothing and looks at no pointer.
 *  - Preconditions the library cannot check: inputs hold no NaN or Inf;
 *    seq_lens[b] <= max_seq_len <= the allocated token count of K and V.
 *
 * Problem indexing.  One "problem" is (sequence b, KV head g, query block m),
 * p = (b*Hkv + g)*Mq + m with Mq = Tq / b_q.  Query head h reads KV head
 * h / (Hq/Hkv); the mask is chosen per KV head and pooled over the Hq/Hkv query
 * heads that share it and over the b_q queries of the block (Alg. 2, chunk
 * score s_{m,j}).  For problem p with T = seq_lens[b]:
 *     E  = (T - Tq) + (m+1)*b_q        one past the last key the block may see
 *     lo = n_sink,  hi = E - n_stream  the middle range [lo, hi) that is pruned
 * (Alg. 1, first step).  Sink [0, n_sink) and window [max(hi,lo), E) are always
 * attended, the window causally.  n_stream >= b_q is required so that every
 * middle key precedes every query of the block.  (With shape->b_q_range set,
 * hi is taken from the b_q_range-sized block that holds block m instead: see
 * ihip_shape.)
 */
#ifndef IHIP_H
#define IHIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IHIP_OK                 0
#define IHIP_ERR_INVALID_ARG   (-1)
#define IHIP_ERR_WORKSPACE     (-2)
#define IHIP_ERR_HIP           (-3)
#define IHIP_ERR_UNSUPPORTED   (-4)

/* A bf16 tensor [B, H, T, d] on the device. */
typedef struct {
    const void *ptr;                       /* device */
    int64_t stride_b, stride_h, stride_t;  /* elements; stride of d is 1 */
} ihip_tensor;

typedef struct {
    int32_t B, Hq, Hkv, d;       /* d must be 128; Hq/Hkv in {1,2,4,8} */
    int32_t Tq, b_q;             /* new query tokens and query block size; decode: 1, 1 */
    const int32_t *seq_lens;     /* device [B]: keys visible per sequence, the Tq new tokens included */
    int32_t max_seq_len;         /* host-side upper bound of seq_lens (sizes the launch) */
    int32_t n_sink, n_stream;
    int32_t b_q_range;           /* 0 or b_q: every query block has its own candidate range.  Otherwise a
                                  * multiple of b_q that divides Tq (and is <= n_stream): the block size
                                  * of the first pruning stage when the stages use different block sizes
                                  * (Sec. 4, the m' rule; Alg. 1 "subdivide query blocks"): the middle
                                  * range of block m ends n_stream before the end of the b_q_range-sized
                                  * block that holds it, and its window runs from there to its queries. */
} ihip_shape;

/*
 * Dynamic RoPE (Sec. 4 "Dynamic RoPE for OOL generalization"; ApplyRopeQ /
 * ApplyRopeK after Alg. 3).  With it, Q and K are stored without positional
 * rotation and the kernels rotate them on the fly with position ids of the
 * method's own choosing.  cos / sin: device fp32 [n_pos][d/2], cos and sin of
 * (position i) x (angle of frequency j), the table of Su et al.; dims (2j, 2j+1)
 * of a vector form pair j.  The kernels rely on the table being one of true
 * rotations (they fold R(a)q . R(b)k into R(a-b)q . k).
 *   prune_style  IHIP_ROPE_RELATIVE: the query at n_stream+1, a left-branch key of
 *                SelectRep at 0, a right-branch key and the representative in the
 *                chunk score at 1 (needs n_pos >= n_stream + 2).
 *                IHIP_ROPE_CHUNK_INDEXED: every key of chunk j (index in the stage's
 *                list of non-empty chunks) at j, the query at min(its own position,
 *                n_chunk - 1 + n_stream) (needs n_pos >= max_chunks + n_stream).
 *   attn_style   IHIP_ROPE_STREAMING: the keys a query attends to, in position
 *                order, at 0..n-1, the query at n-1 (needs n_pos >= n_sink +
 *                n_blocks*block + n_stream).
 * Built for decode (Tq == b_q == 1), also behind the host tier, and for chunked
 * prefill from device memory (all queries of a block share the relative
 * position; query t of a block gets its own chunk-indexed position and its own
 * streaming id, the latter from the number of keys it attends to).  The prefill
 * kernels round the rotated Q and K operands to bf16 for the matrix cores.
 * Other uses return IHIP_ERR_UNSUPPORTED.
 */
#define IHIP_ROPE_NONE          0
#define IHIP_ROPE_RELATIVE      1
#define IHIP_ROPE_CHUNK_INDEXED 2
#define IHIP_ROPE_STREAMING     1
typedef struct ihip_rope {
    const float *cos;
    const float *sin;
    int32_t n_pos;
    int32_t prune_style;         /* IHIP_ROPE_NONE / _RELATIVE / _CHUNK_INDEXED */
    int32_t attn_style;          /* IHIP_ROPE_NONE / _STREAMING */
} ihip_rope;

/* Handle of a host-memory KV tier (see "Host-memory KV tier" below); owned by the library. */
typedef struct ihip_cache ihip_cache;

/* Operation ids for ihip_workspace_bytes. */
#define IHIP_OP_ATTN_DECODE   1
#define IHIP_OP_ATTN_PREFILL  2
#define IHIP_OP_PRUNE_ALL     3
#define IHIP_OP_DECODE_LAYER  4
#define IHIP_OP_PREFILL_LAYER 5

/* ==========================================================================
 * Variants of the storage and of the scores, used by the calls below
 * ========================================================================== */

/*
 * FP8 KV cache (the paper's end-to-end runs keep K and V in 8 bits): the
 * *_fp8kv entry points take K and V as bytes in the OCP FP8 format E4M3 (1 sign,
 * 4 exponent bits with bias 7, 3 mantissa bits, no infinities), one positive
 * scale per tensor: element = scale * decoded byte.  Their ihip_tensor strides
 * count bytes; rows are 128 bytes, 16-byte aligned.  Q and the output stay
 * bf16.  Chunk scores are k_scale * (q . decoded k) in fp32 (the selection does
 * not depend on the scale); the attention multiplies its scores by k_scale and
 * its output by v_scale.  ihip_prune_stage_fp8kv serves decode and chunked
 * prefill (b_q in {1, 16, 32, 64}); the prefill kernels repack a row as bf16
 * (exact) on its way into LDS and multiply in bf16 as before.  These entry
 * points read contiguous (strided) device memory; ihip_decode_layer_ex and
 * ihip_prefill_layer_ex combine E4M3 rows with RoPE, page pools, the pooling
 * rule or (decode) the host tier.
 */

/*
 * Paged KV cache (the serving systems the paper runs in keep K and V in
 * fixed-size pages): the *_paged entry points take K and V as page pools plus a
 * block table.  k_pool / v_pool: ptr = page 0, stride_b = elements between
 * pages, stride_h = between the KV heads of a page, stride_t = between the
 * tokens of a page.  block_table: device int32 [B][table_stride], the page id
 * of logical page i (tokens [i*page_tokens, (i+1)*page_tokens)) of sequence b;
 * entries beyond a sequence's length are never read.  page_tokens is a power
 * of two and table_stride * page_tokens >= max_seq_len.  Everything else as in
 * the entry points of the same names without the suffix.  Built for decode
 * and chunked prefill from bf16 pools; FP8 pools and the other variants
 * combine through ihip_decode_layer_ex / ihip_prefill_layer_ex.
 */
typedef struct ihip_paged_kv {
    const int32_t *block_table;
    int32_t table_stride;
    int32_t page_tokens;
} ihip_paged_kv;

/*
 * Pooling of the chunk scores before the arg-top-K.  IHIP_POOL_KV_HEAD: one
 * selection per (sequence, KV head, query block), the scores as ihip_prune_stage
 * writes them (pooled over the query heads of the KV head) -- what every other
 * entry point does.  IHIP_POOL_ALL_HEADS: the paper's own rule (Sec. 4 and
 * Alg. 2: max over all attention heads h = 1..H): the Hkv score rows of a
 * (sequence, query block) are max-pooled and one selection is written to all
 * Hkv rows of out_starts, i.e. one mask per layer.  Requires the Hkv problems
 * to have identical slots (true when every earlier stage was pooled the same way).
 */
#define IHIP_POOL_KV_HEAD   0
#define IHIP_POOL_ALL_HEADS 1

/* ==========================================================================
 * The path, stage by stage: prune_stage -> select_blocks -> ... -> sparse_attn_{decode,prefill}
 * ========================================================================== */

/*
 * One pruning stage up to the arg-top-K (Alg. 2 with SelectRep of Alg. 3 inside):
 * for every chunk slot j of every problem, finds a representative key per query
 * head by the halving search (first key of each half, left half on a tie) and
 * writes the chunk score = max over the group's heads and the block's queries
 * of q . k_rep (fp32, unscaled).
 *
 * Chunk slots.  parent_starts == NULL: first stage, slot j is
 * [lo + j*chunk, min(lo + (j+1)*chunk, hi)).  Otherwise parent_starts is device
 * int32 [P, n_parent], ascending start positions of the previous stage's kept
 * chunks of size parent_chunk (-1 = none, only at the tail); slot
 * j = i*(parent_chunk/chunk) + c is child c of parent i, cut at hi.  A slot that
 * holds no key gets score -INFINITY (this is how later calls recognise it).
 *
 *   max_chunks   slots per problem: >= ihip_stage1_slots(shape, chunk) for the first
 *                stage, = n_parent*(parent_chunk/chunk) otherwise
 *   out_scores   device fp32 [P, max_chunks]
 *   out_rep      device int32 [B, Hq, Mq, max_chunks] representative positions
 *                (-1 for empty slots); may be NULL
 * chunk and parent_chunk are powers of two, chunk <= 1024, parent_chunk % chunk == 0.
 * b_q == 1 requires Tq == 1 (decode); b_q in {16, 32, 64} is chunked prefill.
 */
int32_t ihip_prune_stage(const ihip_shape *shape, ihip_tensor q, ihip_tensor k,
                         const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk,
                         int32_t chunk, int32_t max_chunks,
                         float *out_scores, int32_t *out_rep, void *stream);

/* Slots the first stage needs per problem: ceil((max_seq_len - n_stream - n_sink) / chunk), >= 0. */
int32_t ihip_stage1_slots(const ihip_shape *shape, int32_t chunk);

/*
 * arg-top-K of the chunk scores (Alg. 2, "discard chunks with low estimated
 * scores"): per problem keeps the min(keep, #non-empty slots) best slots under
 * the order (score descending, slot ascending; -0.0 == +0.0) and writes their
 * start positions in ascending order to out_starts (device int32 [P, keep]),
 * padding with -1.  scores is device fp32 [P, max_chunks] as written by
 * ihip_prune_stage; parent_starts / n_parent / parent_chunk / chunk describe the
 * slots exactly as there.  max_chunks <= 65535 * 16.
 */
int32_t ihip_select_blocks(const ihip_shape *shape, const float *scores, int32_t max_chunks,
                           const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk,
                           int32_t chunk, int32_t keep, int32_t *out_starts, void *stream);

/*
 * Alg. 1 "subdivide query blocks for the next stage" (Sec. 4: a stage's result
 * for block m goes to the blocks m' of the next, smaller block size that lie
 * inside it).  starts: device int32 [P, n], the kept chunk starts of a stage run
 * with shape->b_q queries per block; out_starts: device int32 [P * b_q /
 * b_q_fine, n], row (b, g, m') a copy of row (b, g, m' * b_q_fine / b_q).  The
 * next stage is then called with b_q = b_q_fine and b_q_range = the first
 * stage's block size.  b_q_fine divides shape->b_q; the buffers must differ.
 */
int32_t ihip_subdivide_blocks(const ihip_shape *shape, const int32_t *starts, int32_t n, int32_t b_q_fine,
                              int32_t *out_starts, void *stream);

/*
 * Block-sparse decode attention (Tq == b_q == 1): for every query head,
 *   O = softmax(sm_scale * q K_S^T) V_S,
 *   S = [0, min(n_sink,E)) u kept blocks u [max(hi,n_sink), E)
 * with fp32 scores, exp and accumulation (flash-decoding style split over S and
 * a log-sum-exp merge), bf16 result.
 *   block_starts device int32 [P, n_blocks], start positions of blocks of
 *                `block` tokens (power of two) inside [lo, hi), -1 = none; a block
 *                is cut at hi.  Blocks must not overlap.
 *   out          device bf16 [B, Hq, 1, d] contiguous
 *   out_lse      device fp32 [B, Hq] natural-log sum-exp of the scaled scores; may be NULL
 *   ws, ws_bytes device scratch of at least ihip_workspace_bytes(IHIP_OP_ATTN_DECODE, ...)
 */
int32_t ihip_sparse_attn_decode(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                float sm_scale, void *out, float *out_lse,
                                void *ws, size_t ws_bytes, void *stream);

/*
 * Block-sparse chunked-prefill attention: the same key set per query block m,
 * every query of the block attending causally inside the window (keys after
 * its own position are masked).  b_q in {16, 32, 64}.  block_starts is
 * [P, n_blocks] with P = B*Hkv*Mq; out is bf16 [B, Hq, Tq, d] contiguous;
 * out_lse fp32 [B, Hq, Tq] or NULL.  QK^T and PV run on the matrix cores
 * (bf16 inputs, fp32 accumulation), softmax in fp32.
 */
int32_t ihip_sparse_attn_prefill(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                 const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                 float sm_scale, void *out, float *out_lse,
                                 void *ws, size_t ws_bytes, void *stream);

/*
 * Scratch bytes an operation needs.  n_stages / chunk_sizes / keeps describe
 * the stage plan (for the attention-only ops pass n_stages = 1 with
 * chunk_sizes[0] = block and keeps[0] = n_blocks).  Returns 0 on bad arguments.
 */
size_t ihip_workspace_bytes(int32_t op, const ihip_shape *shape, int32_t n_stages,
                            const int32_t *chunk_sizes, const int32_t *keeps);

/* ==========================================================================
 * The path in one enqueue: every stage, every selection and the attention (what bench.py times)
 * ========================================================================== */

/*
 * Alg. 1: every pruning stage and its arg-top-K, coarse to fine, in one
 * enqueue.  chunk_sizes / keeps are host int32 [n_stages] (l_c and K = k/l_c per
 * stage; each chunk size divides the previous one).  out_block_starts is
 * device int32 [P, keeps[n_stages-1]]: the last stage's kept blocks, as
 * ihip_sparse_attn_* take them.  Scratch from ihip_workspace_bytes(IHIP_OP_PRUNE_ALL, ...).
 */
int32_t ihip_prune_all(const ihip_shape *shape, ihip_tensor q, ihip_tensor k,
                       int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                       int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);

/*
 * One decode layer call: ihip_prune_all followed by ihip_sparse_attn_decode
 * (Alg. 4 with every stage refreshed at every step).  out / out_lse as in
 * ihip_sparse_attn_decode; out_block_starts device int32 [P, keeps[last]] or NULL.
 */
int32_t ihip_decode_layer(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                          int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                          float sm_scale, void *out, float *out_lse, int32_t *out_block_starts,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * One chunked-prefill layer call: ihip_prune_all followed by
 * ihip_sparse_attn_prefill (Alg. 1 per query block, then block-sparse
 * attention).  out / out_lse as in ihip_sparse_attn_prefill; out_block_starts
 * device int32 [P, keeps[last]] or NULL.
 */
int32_t ihip_prefill_layer(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                           int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                           float sm_scale, void *out, float *out_lse, int32_t *out_block_starts,
                           void *ws, size_t ws_bytes, void *stream);

/*
 * The decode layer with any combination of the variants above that the kernels
 * are built for, chosen by one options struct (zero-initialise it: every zero
 * field means "off"):
 *   rope          dynamic RoPE (pruning and attention styles inside), or NULL
 *   cache         host tier: k and v are ignored, the handle's host tensors and
 *                 banks are used, or NULL
 *   paged         k and v are page pools read through this block table, or NULL
 *   kv_fp8        non-zero: k and v hold E4M3 bytes with the scales k_scale, v_scale
 *   pooling       IHIP_POOL_KV_HEAD / IHIP_POOL_ALL_HEADS
 *   stage_starts  mask-caching state as in ihip_decode_layer_masked, or NULL;
 *   first_stage   first stage to recompute (needs stage_starts unless 0)
 *   stage_due     host int32 [n_stages] or NULL (needs stage_starts; first_stage must be 0): Alg. 4's
 *                 per-stage test as it is printed -- stage i is re-run iff stage_due[i] != 0, reading
 *                 the list of stage i-1 as it stands (re-run in this call or cached), and a stage that
 *                 is not due keeps its cached list even when an earlier stage was re-run.
 *                 ihip_refresh_due fills it from the refresh intervals and the step number.
 * Paged, FP8 and RoPE combine freely with each other, with either pooling rule
 * and with mask caching; the host tier (contiguous K/V) combines with FP8 (a
 * cache made by ihip_cache_create_fp8), RoPE, pooling and mask caching
 * (IHIP_ERR_UNSUPPORTED otherwise).  With stage_starts the scratch is the
 * scores buffer plus the attention partials (IHIP_OP_DECODE_LAYER covers it);
 * out_block_starts, if given, receives a copy of the final list.
 */
typedef struct ihip_decode_options {
    const ihip_rope *rope;
    const ihip_cache *cache;
    const ihip_paged_kv *paged;
    int32_t kv_fp8;
    float k_scale, v_scale;
    int32_t pooling;
    int32_t first_stage;
    int32_t *stage_starts;
    const int32_t *stage_due;
} ihip_decode_options;
int32_t ihip_decode_layer_ex(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                             int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                             float sm_scale, const ihip_decode_options *opt, void *out, float *out_lse,
                             int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);

/*
 * The prefill layer with the variants in any combination: dynamic RoPE
 * (relative style in the pruning stages, streaming style in the attention),
 * paged K/V (k and v are then the page pools), the pooling rule and E4M3
 * K/V (kv_fp8 != 0: k and v, or the pools, hold bytes, strides count bytes,
 * k_scale / v_scale as in the *_fp8kv entry points).
 * Zero-initialise the struct: every zero field means "off".
 */
typedef struct ihip_prefill_options {
    const ihip_rope *rope;
    const ihip_paged_kv *paged;
    int32_t pooling;
    int32_t kv_fp8;
    float k_scale, v_scale;
    const int32_t *stage_b_q;   /* host [n_stages] or NULL: query-block size of every stage (Sec. 4, the m'
                                 * rule): 16, 32 or 64, non-increasing, each dividing the one before, the
                                 * last equal to shape.b_q (the attention's block).  The candidate ranges
                                 * are those of the first stage's blocks (see ihip_shape.b_q_range, which
                                 * the call sets itself); where the block size drops, a block's kept
                                 * chunks are handed to every finer block inside it. */
} ihip_prefill_options;
int32_t ihip_prefill_layer_ex(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                              int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                              float sm_scale, const ihip_prefill_options *opt, void *out, float *out_lse,
                              int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);

/*
 * Decode layer with per-stage mask caching (Sec. 4 "Sparse Attention Mask
 * Caching"; Alg. 4: a stage is re-run only every n_refresh steps, otherwise
 * its cached index list is reused).  stage_starts is device int32, owned and
 * kept by the caller between the decode steps of one layer: every stage's
 * kept chunk starts, [P, keeps[0]] then [P, keeps[1]] ... back to back
 * (ihip_mask_state_elems elements).  Stages first_stage .. n_stages-1 are
 * recomputed with the current q and stored; stages before first_stage are
 * taken as cached (first_stage = 0 recomputes everything, = n_stages only
 * runs the attention over the cached final blocks).  The window and the
 * cut of blocks at the end of the middle range always follow the current
 * seq_lens.  Which stage is due at which step (c mod n_refresh == 0):
 * ihip_refresh_due; schedules in which a later stage is not due while an
 * earlier one is go through ihip_decode_layer_ex (stage_due).  Scratch as
 * for IHIP_OP_DECODE_LAYER.
 */
size_t  ihip_mask_state_elems(const ihip_shape *shape, int32_t n_stages, const int32_t *keeps);
int32_t ihip_decode_layer_masked(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                 int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                 int32_t first_stage, int32_t *stage_starts, float sm_scale, void *out,
                                 float *out_lse, void *ws, size_t ws_bytes, void *stream);

/*
 * Alg. 4's counters (c^(i) starts at 0 and advances by one per generated token modulo n_refresh^(i);
 * stage i is re-run when c^(i) = 0): for decode step `step` (0 = the first) writes
 * stage_due[i] = (step mod n_refresh[i] == 0) to the host array stage_due (may be NULL) and returns
 * the first due stage, n_stages if none is, or a negative error.  Host arithmetic only.  With nested
 * intervals (each a multiple of the next) every stage after the first due one is due as well and the
 * return value is all ihip_decode_layer_masked needs.
 */
int32_t ihip_refresh_due(int32_t n_stages, const int32_t *n_refresh, int64_t step, int32_t *stage_due);

/*
 * ihip_decode_layer for callers that cannot allocate device memory or hand a
 * workspace over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results, but the scratch (scores, the kept lists between the
 * stages, the final block list, the attention's split partials) is a device
 * array inside the library of IHIP_STATIC_SCRATCH_BYTES bytes, which every GPU
 * the library runs on holds until the process ends.  The call allocates and
 * frees nothing.  A shape and plan whose scratch
 * (ihip_workspace_bytes(IHIP_OP_DECODE_LAYER, ...)) exceeds the array returns
 * IHIP_ERR_WORKSPACE and enqueues nothing; the batch-8, 1M-token plan with
 * four stages needs about 4 MiB.  Every call on a GPU shares that GPU's array
 * (nothing in it has to survive or be cleared between calls): calls that
 * overlap on one GPU, on different streams or threads, race.  The GPU the
 * stream belongs to must be the calling thread's current device (the array
 * of that device is the one used).
 */
#define IHIP_STATIC_SCRATCH_BYTES (8u << 20)
int32_t ihip_decode_layer_static(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                 int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                 float sm_scale, void *out, float *out_lse, int32_t *out_block_starts,
                                 void *stream);

/* ==========================================================================
 * Host-memory KV tier with the on-GPU hot-block cache
 * ========================================================================== */

/*
 * Host-memory KV tier with an on-GPU hot-block cache (Sec. 4 "KV Cache
 * Offloading"; Alg. 4, the miss lists and the LRU replacement after the layer).
 *
 * K and V of the layer, bf16 [B,Hkv,T_alloc,d], live in pinned host memory
 * that the GPU can address (hipHostMalloc): host_k / host_v carry such
 * pointers.  The cache keeps copies of block_tokens-token blocks (a power of
 * two) in two banks carved out of dev_mem (device memory owned by the caller,
 * 256-byte aligned, at least ihip_cache_device_bytes(...) long): the
 * mask-selection bank (keys only, mask_slots blocks) read by the pruning
 * stages, and the sparse-attention bank (keys and values, sa_slots blocks).
 * The handle itself is a small host object owned by the library; the caller
 * keeps dev_mem and the host tensors alive until ihip_cache_destroy.
 *
 * ihip_decode_layer_cached is ihip_decode_layer reading K/V through the cache:
 * a resident block is read from its bank, any other row straight from host
 * memory over the host link; the results are bit-identical to the uncached
 * call on the same data whatever the cache holds.  It records which blocks
 * were touched and which were missing.  ihip_cache_update (same stream, after
 * the layer call) then, per bank, evicts as many least-recently-used slots as
 * there were missed blocks (oldest last-touch call first, lowest slot on a
 * tie; never-used slots first; never a slot touched in this same call) and
 * copies the missed blocks in, in ascending block order; if more blocks were
 * missed than there are such slots, only the lowest-numbered ones are inserted.  Layer calls and updates on one cache
 * must not overlap.  The counter that stamps the calls lives on the host, so
 * the calls that read or update a cache (the *_cached calls, ihip_decode_layer_ex
 * with a cache, ihip_cache_update) cannot be captured into a HIP graph: on a
 * stream under capture they return IHIP_ERR_UNSUPPORTED.
 *
 * ihip_cache_stats (synchronises the device) fills stats8 (host):
 * [0..3] mask bank, [4..7] sparse-attention bank: blocks hit (cumulative over
 * calls, a block counts once per call), blocks missed (cumulative), blocks
 * missed in the last call, blocks touched in the last call.
 * ihip_cache_read_tables (synchronises) copies a bank's page table (int32 per
 * global block id (b*Hkv+g)*blocks_per_head + block: slot or -1) and slot
 * table (block id per slot or -1) to host arrays; either may be NULL.
 */
size_t  ihip_cache_device_bytes(int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens,
                                int32_t mask_slots, int32_t sa_slots);
int32_t ihip_cache_create(ihip_cache **out, void *dev_mem, size_t dev_bytes, ihip_tensor host_k,
                          ihip_tensor host_v, int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens,
                          int32_t mask_slots, int32_t sa_slots, void *stream);
/*
 * The same tier over E4M3 K/V (FP8 KV cache, see ihip_*_fp8kv): host_k / host_v hold bytes, their
 * strides count bytes (multiples of 16), the banks hold 128-byte rows.  Such a cache is read through
 * ihip_decode_layer_ex with kv_fp8 set and the scales given there.
 */
size_t  ihip_cache_device_bytes_fp8(int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens,
                                    int32_t mask_slots, int32_t sa_slots);
int32_t ihip_cache_create_fp8(ihip_cache **out, void *dev_mem, size_t dev_bytes, ihip_tensor host_k,
                              ihip_tensor host_v, int32_t B, int32_t Hkv, int64_t T_alloc,
                              int32_t block_tokens, int32_t mask_slots, int32_t sa_slots, void *stream);
/*
 * The same tier with the host memory organised in pages (the serving systems
 * the paper runs in keep K and V in fixed-size pages, also when they are
 * offloaded): host_k_pool / host_v_pool are pinned host page pools laid out as
 * in ihip_paged_kv (stride_b = between pages), host_pages->block_table is a
 * DEVICE int32 [B][table_stride] array of page ids that must stay valid and
 * unchanged while the cache is in use, table_stride * page_tokens >= T_alloc.
 * kv_fp8 != 0: E4M3 pools (strides in bytes).  The banks, their block ids
 * (logical positions) and the LRU policy are those of the contiguous tier;
 * only the address of a row in host memory goes through the table.
 */
int32_t ihip_cache_create_paged(ihip_cache **out, void *dev_mem, size_t dev_bytes, ihip_tensor host_k_pool,
                                ihip_tensor host_v_pool, const ihip_paged_kv *host_pages, int32_t kv_fp8,
                                int32_t B, int32_t Hkv, int64_t T_alloc, int32_t block_tokens,
                                int32_t mask_slots, int32_t sa_slots, void *stream);
void    ihip_cache_destroy(ihip_cache *cache);
int32_t ihip_cache_reset(ihip_cache *cache, void *stream);
int32_t ihip_cache_update(ihip_cache *cache, void *stream);
int32_t ihip_cache_stats(ihip_cache *cache, uint64_t *stats8);
int32_t ihip_cache_read_tables(ihip_cache *cache, int32_t bank, int32_t *host_page_table,
                               int32_t *host_slot_block);
int32_t ihip_cache_geometry(const ihip_cache *cache, int32_t *n_blocks_total, int32_t *mask_slots,
                            int32_t *sa_slots);

/*
 * The stage-by-stage calls through the host tier: ihip_prune_stage (decode,
 * Tq == b_q == 1) reading K through the cache's mask bank, and
 * ihip_sparse_attn_decode reading K and V through its sparse-attention bank;
 * everything else as in the calls without the suffix, results bit-identical to
 * them on the same data.  They record touched and missed blocks like the layer
 * call, for a later ihip_cache_update.  rope may be NULL (the pruning call uses
 * rope->prune_style, the attention rope->attn_style); k_scale / v_scale are
 * used by an E4M3 tier only.
 */
int32_t ihip_prune_stage_cached(const ihip_shape *shape, ihip_tensor q, ihip_cache *cache,
                                const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk,
                                int32_t chunk, int32_t max_chunks, const ihip_rope *rope, float k_scale,
                                float *out_scores, int32_t *out_rep, void *stream);
int32_t ihip_sparse_attn_decode_cached(const ihip_shape *shape, ihip_tensor q, ihip_cache *cache,
                                       const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                       float sm_scale, const ihip_rope *rope, float k_scale, float v_scale,
                                       void *out, float *out_lse, void *ws, size_t ws_bytes, void *stream);

/* ==========================================================================
 * The stage-by-stage calls with one variant of the storage or of the scores
 * ========================================================================== */

/* ihip_prune_stage / ihip_sparse_attn_decode / ihip_sparse_attn_prefill over E4M3 K and V ("FP8 KV cache" above);
 * the prefill attention takes rope as well (may be NULL). */
int32_t ihip_prune_stage_fp8kv(const ihip_shape *shape, ihip_tensor q, ihip_tensor k,
                               const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk,
                               int32_t chunk, int32_t max_chunks, float k_scale,
                               float *out_scores, int32_t *out_rep, void *stream);
int32_t ihip_sparse_attn_decode_fp8kv(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                      const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                      float sm_scale, float k_scale, float v_scale, void *out,
                                      float *out_lse, void *ws, size_t ws_bytes, void *stream);
int32_t ihip_sparse_attn_prefill_fp8kv(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                       const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                       float sm_scale, float k_scale, float v_scale, const ihip_rope *rope,
                                       void *out, float *out_lse, void *ws, size_t ws_bytes, void *stream);

/* ... reading K and V from page pools (ihip_paged_kv above); the prefill attention takes rope as well (may be NULL). */
int32_t ihip_prune_stage_paged(const ihip_shape *shape, ihip_tensor q, ihip_tensor k_pool,
                               const ihip_paged_kv *paged, const int32_t *parent_starts, int32_t n_parent,
                               int32_t parent_chunk, int32_t chunk, int32_t max_chunks,
                               float *out_scores, int32_t *out_rep, void *stream);
int32_t ihip_sparse_attn_decode_paged(const ihip_shape *shape, ihip_tensor q, ihip_tensor k_pool,
                                      ihip_tensor v_pool, const ihip_paged_kv *paged,
                                      const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                      float sm_scale, void *out, float *out_lse, void *ws, size_t ws_bytes,
                                      void *stream);
int32_t ihip_sparse_attn_prefill_paged(const ihip_shape *shape, ihip_tensor q, ihip_tensor k_pool,
                                       ihip_tensor v_pool, const ihip_paged_kv *paged,
                                       const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                       float sm_scale, const ihip_rope *rope, void *out, float *out_lse,
                                       void *ws, size_t ws_bytes, void *stream);

/* ... with dynamic RoPE: the pruning call applies rope->prune_style, the attention calls rope->attn_style to q and K
 * (V is not rotated); rope must not be NULL. */
int32_t ihip_prune_stage_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k,
                              const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk,
                              int32_t chunk, int32_t max_chunks, const ihip_rope *rope,
                              float *out_scores, int32_t *out_rep, void *stream);
int32_t ihip_sparse_attn_decode_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                     const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                     float sm_scale, const ihip_rope *rope, void *out, float *out_lse,
                                     void *ws, size_t ws_bytes, void *stream);
int32_t ihip_sparse_attn_prefill_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                      const int32_t *block_starts, int32_t n_blocks, int32_t block,
                                      float sm_scale, const ihip_rope *rope, void *out, float *out_lse,
                                      void *ws, size_t ws_bytes, void *stream);

/* ihip_select_blocks with a pooling rule (IHIP_POOL_* above). */
int32_t ihip_select_blocks_pooled(const ihip_shape *shape, const float *scores, int32_t max_chunks,
                                  const int32_t *parent_starts, int32_t n_parent, int32_t parent_chunk,
                                  int32_t chunk, int32_t keep, int32_t pooling, int32_t *out_starts,
                                  void *stream);

/* ==========================================================================
 * Conveniences: a layer call with exactly one variant.  Each is ihip_decode_layer_ex /
 * ihip_prefill_layer_ex with that one option set (same checks, same kernels, same results); new code
 * can use the _ex calls alone.
 * ========================================================================== */

int32_t ihip_decode_layer_pooled(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                 int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                 int32_t pooling, float sm_scale, void *out, float *out_lse,
                                 int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);
int32_t ihip_prefill_layer_pooled(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                  int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                  int32_t pooling, float sm_scale, void *out, float *out_lse,
                                  int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);
int32_t ihip_decode_layer_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                               int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                               float sm_scale, const ihip_rope *rope, void *out, float *out_lse,
                               int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);
int32_t ihip_prefill_layer_rope(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                float sm_scale, const ihip_rope *rope, void *out, float *out_lse,
                                int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);
int32_t ihip_decode_layer_fp8kv(const ihip_shape *shape, ihip_tensor q, ihip_tensor k, ihip_tensor v,
                                int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                float sm_scale, float k_scale, float v_scale, void *out, float *out_lse,
                                int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);
int32_t ihip_decode_layer_paged(const ihip_shape *shape, ihip_tensor q, ihip_tensor k_pool, ihip_tensor v_pool,
                                const ihip_paged_kv *paged, int32_t n_stages, const int32_t *chunk_sizes,
                                const int32_t *keeps, float sm_scale, void *out, float *out_lse,
                                int32_t *out_block_starts, void *ws, size_t ws_bytes, void *stream);
int32_t ihip_decode_layer_cached(const ihip_shape *shape, ihip_tensor q, ihip_cache *cache,
                                 int32_t n_stages, const int32_t *chunk_sizes, const int32_t *keeps,
                                 float sm_scale, void *out, float *out_lse, int32_t *out_block_starts,
                                 void *ws, size_t ws_bytes, void *stream);

/* Text of the calling thread's last error ("" if none).  Never NULL. */
const char *ihip_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int32_t ihip_version(void);

#ifdef __cplusplus
}
#endif
#endif /* IHIP_H */

