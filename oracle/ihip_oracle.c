/*
 * CPU oracle for InfiniteHiP's attention hot path (arXiv 2502.08910).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, sequential C that follows the
 * paper's algorithms step by step; it shares no code with the HIP library and
 * must never be called from the product path.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may load it.
 *
 * What is here (one (sequence b, KV head g, query block) problem at a time;
 * the multi-stage loop of Alg. 1 lives in pipeline.py beside this file):
 *   orc_score            q.k score of one key against a query block  (Sec. 4, eq. for s_{m,j}; Alg. 3 step "compute scores")
 *   orc_select_rep       SelectRep, hierarchical top-1 search          (Alg. 3)
 *   orc_prune_stage      representative + chunk score per chunk        (Alg. 2, up to the arg-top-K)
 *   orc_topk             arg-top-K of the chunk scores                  (Alg. 2, arg top_{k/l_c})
 *   orc_sparse_attention softmax attention over sink + kept blocks + window (Sec. 4 "Background", BSA of Alg. 4)
 *   orc_*_rope           the same steps with dynamic RoPE (Sec. 4 "Dynamic RoPE ..."; second half of this file)
 *
 * Conventions (the paper is silent or garbled on these; same readings as the
 * design notes list): 0-based positions; chunk sizes are powers of two; the
 * two halves of a range are [first, first+size/2) and [first+size/2, last];
 * ties keep the left branch / the lowest index; a chunk that is cut short by
 * the end of the middle range scores -inf for positions past its end.  In the
 * first half of the file RoPE adjustment is off; with RoPE off the left
 * branch's first key is the previous winner, so its score is carried over
 * instead of being recomputed.
 * Scores that decide a selection are fp32 (bf16 inputs, fp32 products and
 * sums, summed in index order); the attention itself is fp64.
 *
 * Layouts: Q [B,Hq,Tq,d], K and V [B,Hkv,T_alloc,d], contiguous, bf16 bit
 * patterns in uint16 (K and V optionally E4M3 bytes with a scale each, see
 * orc_tensors).  Query head h reads KV head h / (Hq/Hkv).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    const uint16_t *Q, *K, *V;
    int32_t B, Hq, Hkv, d, Tq;
    int64_t T_alloc;
    /* FP8 KV cache (the paper's end-to-end runs keep K and V in 8 bits): when kv_fp8 != 0, K and V
     * point to bytes in the OCP 8-bit float format E4M3 and an element's value is its scale times
     * the decoded byte (one scale per tensor).  Q stays bf16. */
    int32_t kv_fp8;
    float k_scale, v_scale;
} orc_tensors;

static float bf16_to_f32(uint16_t x)
{
    uint32_t u = (uint32_t)x << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/*
 * OCP FP8 E4M3: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; no
 * infinities; exponent 15 with mantissa 7 is NaN; exponent 0 holds the
 * subnormals m/8 * 2^-6.
 */
float orc_e4m3_to_f32(uint8_t x)
{
    const int sign = x >> 7, e = (x >> 3) & 15, m = x & 7;
    float v;
    if (e == 15 && m == 7) v = NAN;
    else if (e == 0) v = ldexpf((float)m, -9);
    else v = ldexpf((float)(8 + m), e - 10);
    return sign ? -v : v;
}

/* element c of key / value row p of (sequence b, KV head g), as a float */
static float k_elem(const orc_tensors *t, int b, int g, int64_t p, int c)
{
    const int64_t i = (((int64_t)b * t->Hkv + g) * t->T_alloc + p) * t->d + c;
    if (t->kv_fp8) return t->k_scale * orc_e4m3_to_f32(((const uint8_t *)t->K)[i]);
    return bf16_to_f32(t->K[i]);
}
static float v_elem(const orc_tensors *t, int b, int g, int64_t p, int c)
{
    const int64_t i = (((int64_t)b * t->Hkv + g) * t->T_alloc + p) * t->d + c;
    if (t->kv_fp8) return t->v_scale * orc_e4m3_to_f32(((const uint8_t *)t->V)[i]);
    return bf16_to_f32(t->V[i]);
}

static const uint16_t *q_row(const orc_tensors *t, int b, int h, int64_t tq)
{
    return t->Q + (((int64_t)b * t->Hq + h) * t->Tq + tq) * t->d;
}

/* max over the queries t of the block [q0, q0+bq) of  q_t . k_p   (fp32). */
float orc_score(const orc_tensors *t, int b, int h, int64_t q0, int bq, int64_t p)
{
    const int g = h / (t->Hq / t->Hkv);
    float best = -INFINITY;
    for (int i = 0; i < bq; ++i) {
        const uint16_t *q = q_row(t, b, h, q0 + i);
        float acc = 0.0f;
        for (int c = 0; c < t->d; ++c)
            acc += bf16_to_f32(q[c]) * k_elem(t, b, g, p, c);
        if (acc > best)
            best = acc;
    }
    return best;
}

/*
 * SelectRep (Alg. 3) for head h on the chunk [start, start+len), nominal size
 * l_c (a power of two, len <= l_c).  Binary search: at each of the log2(l_c)
 * iterations the current range is cut in two equal halves and the first key
 * of each half is scored; the better half survives (left on a tie).
 * exhaustive != 0 replaces the search by the true in-chunk arg-max (lowest
 * index on ties) -- used only to pin the search against brute force.
 * touched (nullable): byte map over positions of this (b, g); every key that
 * is scored is marked.
 */
void orc_select_rep(const orc_tensors *t, int b, int h, int64_t q0, int bq,
                    int64_t start, int len, int l_c, int exhaustive,
                    int64_t *r_out, float *sigma_out, uint8_t *touched)
{
    if (exhaustive) {
        int best_off = 0;
        float best = -INFINITY;
        for (int off = 0; off < len; ++off) {
            float s = orc_score(t, b, h, q0, bq, start + off);
            if (touched) touched[start + off] = 1;
            if (off == 0 || s > best) { best = s; best_off = off; }
        }
        *r_out = start + best_off;
        *sigma_out = best;
        return;
    }
    int off = 0;            /* first position of the current range, relative to start */
    int size = l_c;         /* its nominal size */
    float sigma = orc_score(t, b, h, q0, bq, start);   /* first key of the whole chunk */
    if (touched) touched[start] = 1;
    while (size > 1) {
        const int half = size / 2;
        const int mid = off + half;             /* first key of the right half */
        float sigma_right = -INFINITY;
        if (mid < len) {
            sigma_right = orc_score(t, b, h, q0, bq, start + mid);
            if (touched) touched[start + mid] = 1;
        }
        if (sigma_right > sigma) {              /* strict: a tie keeps the left half */
            off = mid;
            sigma = sigma_right;
        }
        size = half;
    }
    *r_out = start + off;
    *sigma_out = sigma;
}

/*
 * One pruning stage up to (not including) the arg-top-K (Alg. 2): for every
 * chunk j, a representative per query head of the KV group g, and the chunk
 * score = max over the group's heads (and over the block's queries, inside
 * orc_score) of q . k_rep.
 * rep (nullable) is [G][n_chunk].
 */
void orc_prune_stage(const orc_tensors *t, int b, int g, int64_t q0, int bq,
                     int n_chunk, const int64_t *starts, const int32_t *lens,
                     int l_c, int exhaustive,
                     float *score, int64_t *rep, uint8_t *touched)
{
    const int G = t->Hq / t->Hkv;
    for (int j = 0; j < n_chunk; ++j) {
        float s = -INFINITY;
        for (int hh = 0; hh < G; ++hh) {
            int64_t r;
            float sigma;
            orc_select_rep(t, b, g * G + hh, q0, bq, starts[j], lens[j], l_c,
                           exhaustive, &r, &sigma, touched);
            if (rep) rep[(int64_t)hh * n_chunk + j] = r;
            if (sigma > s) s = sigma;
        }
        score[j] = s;
    }
}

typedef struct { float s; int32_t j; } scored;

static int by_score_desc_then_index(const void *a, const void *b)
{
    const scored *x = a, *y = b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}
static int by_index(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * arg-top-K: ids of the min(keep, n) largest scores, a tie going to the lower
 * id, returned in ascending id order.  Returns how many were kept.
 */
int orc_topk(int n, const float *score, int keep, int32_t *ids_out)
{
    scored *v = malloc(sizeof(scored) * (n > 0 ? n : 1));
    for (int j = 0; j < n; ++j) { v[j].s = score[j]; v[j].j = j; }
    qsort(v, n, sizeof(scored), by_score_desc_then_index);
    const int kept = keep < n ? keep : n;
    for (int i = 0; i < kept; ++i) ids_out[i] = v[i].j;
    qsort(ids_out, kept, sizeof(int32_t), by_index);
    free(v);
    return kept;
}

/*
 * Attention of the query block [q0, q0+bq) of KV group g over
 *   sink  [0, min(n_sink, p+1))
 *   kept  every token of the blocks (block_starts[i], block_lens[i])
 *   window [w0, p]
 * where p = pos0 + i is the absolute position of query q0+i (causal: no key
 * after p).  Kept blocks must lie in [n_sink, w0).  O = softmax(scale q K^T) V
 * in fp64.  out is [G][bq][d] doubles, lse (nullable) [G][bq] natural-log
 * sum-exp of the scaled scores.
 */
void orc_sparse_attention(const orc_tensors *t, int b, int g, int64_t q0, int bq,
                          int64_t pos0, int64_t n_sink, int64_t w0,
                          int n_blocks, const int64_t *block_starts,
                          const int32_t *block_lens, double scale,
                          double *out, double *lse)
{
    const int G = t->Hq / t->Hkv, d = t->d;
    /* the key list of the last query is the longest */
    int64_t cap = n_sink + (pos0 + bq - w0 > 0 ? pos0 + bq - w0 : 0) + 1;
    for (int i = 0; i < n_blocks; ++i) cap += block_lens[i];
    int64_t *keys = malloc(sizeof(int64_t) * cap);
    double *s = malloc(sizeof(double) * cap);

    for (int hh = 0; hh < G; ++hh) {
        for (int i = 0; i < bq; ++i) {
            const int64_t p = pos0 + i;
            int64_t n = 0;
            for (int64_t x = 0; x < n_sink && x <= p; ++x) keys[n++] = x;
            for (int j = 0; j < n_blocks; ++j)
                for (int c = 0; c < block_lens[j]; ++c) keys[n++] = block_starts[j] + c;
            for (int64_t x = w0; x <= p; ++x) keys[n++] = x;

            const uint16_t *q = q_row(t, b, g * G + hh, q0 + i);
            double mx = -INFINITY;
            for (int64_t a = 0; a < n; ++a) {
                double acc = 0.0;
                for (int c = 0; c < d; ++c)
                    acc += (double)bf16_to_f32(q[c]) * (double)k_elem(t, b, g, keys[a], c);
                s[a] = scale * acc;
                if (s[a] > mx) mx = s[a];
            }
            double denom = 0.0;
            double *o = out + ((int64_t)hh * bq + i) * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            for (int64_t a = 0; a < n; ++a) {
                const double w = exp(s[a] - mx);
                denom += w;
                for (int c = 0; c < d; ++c) o[c] += w * (double)v_elem(t, b, g, keys[a], c);
            }
            for (int c = 0; c < d; ++c) o[c] /= denom;
            if (lse) lse[(int64_t)hh * bq + i] = mx + log(denom);
        }
    }
    free(keys);
    free(s);
}

/* ===========================================================================
 * Dynamic RoPE (Sec. 4 "Dynamic RoPE for OOL generalization"; the ApplyRopeQ /
 * ApplyRopeK definitions after Alg. 3).  Q and K are stored without positional
 * rotation; the pruning stages and the attention rotate them on the fly with
 * position ids of their own choosing.
 *
 * Readings (the paper cites RoFormer for ApplyRope and is terse on the ids):
 *  - ApplyRope(x, p_i): dims (2j, 2j+1) form a pair that is turned by the angle
 *    of position i at frequency j; the table gives cos and sin of that angle,
 *    rope->cos[i*(d/2) + j], rope->sin[...].
 *  - Relative style (layers after the third): the query block is at position
 *    n_stream + 1; in SelectRep the left branch's key is at position 0 and the
 *    right branch's at position 1; the chunk score puts the representative at
 *    position 1 (ApplyRopeK_{l,2}).  The two branches use different positions,
 *    so both scores are computed at every iteration (no carried score).
 *  - Chunk-indexed style (first three layers): every key of chunk j of the
 *    stage's chunk list (0-based, in position order) is at position j; query t
 *    of the block is at min(original position, (n_chunk - 1) + n_stream), i.e.
 *    the last chunk is n_stream behind the query.
 *  - Streaming style (attention): the keys a query attends to, in position
 *    order, are at positions 0, 1, ..., n-1 and the query at n-1 (the position
 *    of the most recent key, which is the query's own token).
 * Rotations for the selection scores are fp32 (products and sums rounded one
 * by one; the paper does not fix the precision of the rotated vectors, fp32 is
 * that of every other selection score here), the attention is fp64 throughout.
 * =========================================================================== */
typedef struct {
    const float *cos, *sin;     /* [n_pos][d/2] */
    int32_t n_pos;
} orc_rope;

static void rope_f32(const float *x, const orc_rope *r, int64_t pos, int d, float *out)
{
    const float *c = r->cos + pos * (d / 2), *s = r->sin + pos * (d / 2);
    for (int j = 0; j < d / 2; ++j) {
        const float a = x[2 * j], b = x[2 * j + 1];
        out[2 * j] = a * c[j] - b * s[j];
        out[2 * j + 1] = a * s[j] + b * c[j];
    }
}

/* max over the block's queries t of ApplyRope(q_t, qpos[t]) . ApplyRope(k_p, kpos)   (fp32) */
float orc_score_rope(const orc_tensors *t, int b, int h, int64_t q0, int bq, int64_t p,
                     const orc_rope *rope, const int64_t *qpos, int64_t kpos)
{
    const int g = h / (t->Hq / t->Hkv), d = t->d;
    float *kr = malloc(sizeof(float) * d), *qr = malloc(sizeof(float) * d), *x = malloc(sizeof(float) * d);
    for (int c = 0; c < d; ++c) x[c] = k_elem(t, b, g, p, c);
    rope_f32(x, rope, kpos, d, kr);
    float best = -INFINITY;
    for (int i = 0; i < bq; ++i) {
        for (int c = 0; c < d; ++c) x[c] = bf16_to_f32(q_row(t, b, h, q0 + i)[c]);
        rope_f32(x, rope, qpos[i], d, qr);
        float acc = 0.0f;
        for (int c = 0; c < d; ++c) acc += qr[c] * kr[c];
        if (acc > best) best = acc;
    }
    free(kr);
    free(qr);
    free(x);
    return best;
}

/*
 * SelectRep (Alg. 3) with ApplyRopeQ / ApplyRopeK: style 1 = relative (branch j's
 * key at position j-1), style 2 = chunk-indexed (both branches' keys at
 * position chunk_index).  Same halving, tie and ragged-end rules as
 * orc_select_rep; both branches are scored at every iteration.
 */
void orc_select_rep_rope(const orc_tensors *t, int b, int h, int64_t q0, int bq,
                         int64_t start, int len, int l_c, const orc_rope *rope, int style,
                         const int64_t *qpos, int64_t chunk_index, int64_t *r_out, uint8_t *touched)
{
    int off = 0, size = l_c;
    if (touched) touched[start] = 1;
    while (size > 1) {
        const int half = size / 2, mid = off + half;
        const int64_t pos_left = style == 1 ? 0 : chunk_index, pos_right = style == 1 ? 1 : chunk_index;
        const float sigma_left = orc_score_rope(t, b, h, q0, bq, start + off, rope, qpos, pos_left);
        float sigma_right = -INFINITY;
        if (mid < len) {
            sigma_right = orc_score_rope(t, b, h, q0, bq, start + mid, rope, qpos, pos_right);
            if (touched) touched[start + mid] = 1;
        }
        if (sigma_right > sigma_left) off = mid;    /* strict: a tie keeps the left half */
        size = half;
    }
    *r_out = start + off;
}

/*
 * One pruning stage (Alg. 2) with dynamic RoPE.  pos0 = original position of
 * the block's first query.  The chunk score rotates the representative as
 * branch 2 (relative: position 1; chunk-indexed: its chunk's index).
 */
void orc_prune_stage_rope(const orc_tensors *t, int b, int g, int64_t q0, int bq, int64_t pos0,
                          int n_chunk, const int64_t *starts, const int32_t *lens, int l_c,
                          const orc_rope *rope, int style, int64_t n_stream,
                          float *score, int64_t *rep, uint8_t *touched)
{
    const int G = t->Hq / t->Hkv;
    int64_t *qpos = malloc(sizeof(int64_t) * bq);
    for (int i = 0; i < bq; ++i) {
        if (style == 1) qpos[i] = n_stream + 1;
        else {
            const int64_t cap = (int64_t)(n_chunk - 1) + n_stream;
            qpos[i] = pos0 + i < cap ? pos0 + i : cap;
        }
    }
    for (int j = 0; j < n_chunk; ++j) {
        float s = -INFINITY;
        for (int hh = 0; hh < G; ++hh) {
            int64_t r;
            orc_select_rep_rope(t, b, g * G + hh, q0, bq, starts[j], lens[j], l_c, rope, style,
                                qpos, j, &r, touched);
            if (rep) rep[(int64_t)hh * n_chunk + j] = r;
            const float sigma = orc_score_rope(t, b, g * G + hh, q0, bq, r, rope, qpos, style == 1 ? 1 : j);
            if (sigma > s) s = sigma;
        }
        score[j] = s;
    }
    free(qpos);
}

/*
 * orc_sparse_attention with streaming-style positions: key a of a query's key
 * list (position order) is rotated to position a, the query to position n-1.
 */
void orc_sparse_attention_rope(const orc_tensors *t, int b, int g, int64_t q0, int bq,
                               int64_t pos0, int64_t n_sink, int64_t w0,
                               int n_blocks, const int64_t *block_starts,
                               const int32_t *block_lens, double scale, const orc_rope *rope,
                               double *out, double *lse)
{
    const int G = t->Hq / t->Hkv, d = t->d;
    int64_t cap = n_sink + (pos0 + bq - w0 > 0 ? pos0 + bq - w0 : 0) + 1;
    for (int i = 0; i < n_blocks; ++i) cap += block_lens[i];
    int64_t *keys = malloc(sizeof(int64_t) * cap);
    double *s = malloc(sizeof(double) * cap);
    double *qr = malloc(sizeof(double) * d), *kr = malloc(sizeof(double) * d);

    for (int hh = 0; hh < G; ++hh) {
        for (int i = 0; i < bq; ++i) {
            const int64_t p = pos0 + i;
            int64_t n = 0;
            for (int64_t x = 0; x < n_sink && x <= p; ++x) keys[n++] = x;
            for (int j = 0; j < n_blocks; ++j)
                for (int c = 0; c < block_lens[j]; ++c) keys[n++] = block_starts[j] + c;
            for (int64_t x = w0; x <= p; ++x) keys[n++] = x;

            const uint16_t *q = q_row(t, b, g * G + hh, q0 + i);
            const float *cq = rope->cos + (n - 1) * (d / 2), *sq = rope->sin + (n - 1) * (d / 2);
            for (int j = 0; j < d / 2; ++j) {
                const double x0 = bf16_to_f32(q[2 * j]), x1 = bf16_to_f32(q[2 * j + 1]);
                qr[2 * j] = x0 * cq[j] - x1 * sq[j];
                qr[2 * j + 1] = x0 * sq[j] + x1 * cq[j];
            }
            double mx = -INFINITY;
            for (int64_t a = 0; a < n; ++a) {
                const float *ck = rope->cos + a * (d / 2), *sk = rope->sin + a * (d / 2);
                double acc = 0.0;
                for (int j = 0; j < d / 2; ++j) {
                    const double x0 = k_elem(t, b, g, keys[a], 2 * j), x1 = k_elem(t, b, g, keys[a], 2 * j + 1);
                    kr[2 * j] = x0 * ck[j] - x1 * sk[j];
                    kr[2 * j + 1] = x0 * sk[j] + x1 * ck[j];
                }
                for (int c = 0; c < d; ++c) acc += qr[c] * kr[c];
                s[a] = scale * acc;
                if (s[a] > mx) mx = s[a];
            }
            double denom = 0.0;
            double *o = out + ((int64_t)hh * bq + i) * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            for (int64_t a = 0; a < n; ++a) {
                const double w = exp(s[a] - mx);
                denom += w;
                for (int c = 0; c < d; ++c) o[c] += w * (double)v_elem(t, b, g, keys[a], c);
            }
            for (int c = 0; c < d; ++c) o[c] /= denom;
            if (lse) lse[(int64_t)hh * bq + i] = mx + log(denom);
        }
    }
    free(keys); free(s); free(qr); free(kr);
}
