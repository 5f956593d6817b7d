/*
 * Plain CPU oracle for one embedding-table shard's prioritized-update path.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the HIP library; nothing in the
 * product path may call it.  It is written for obviousness, not speed: one thread,
 * no blocking, no fusion, fp64 accumulation, one rounding per output element.  It
 * shares no source, header, table or helper with the HIP library.
 *
 * What each function follows (FreeScale paper, Section 3.2 "Prioritized Embedding
 * Updates" and its Algorithm 2 "Prioritized Embedding Autograd Function"):
 *   fso_gather_jagged          Lookup(I): rows of the shard-major table selected by a
 *                              jagged ID tensor (Section 2.1 describes the lookup, Section
 *                              4.2 the jagged layout).
 *   fso_unique_ids             the distinct rows of one iteration's IDs; collisions are
 *                              defined on rows (Section 2.3).
 *   fso_collision_split        compute_collision(I^i, I^{i+1}) -> I_co^i, I_ex^i, I_ex^{i+1}
 *                              (Algorithm 2; the collision definition below it).
 *   fso_segment_reduce_grads   first half of update_embedding(I, G): one summed gradient
 *                              per distinct row.
 *   fso_rowwise_adagrad_update second half of update_embedding(I, G): the sparse optimizer
 *                              step.  The paper does not name the optimizer; this build
 *                              fixes row-wise Adagrad (one accumulator per row that adds
 *                              the MEAN over columns of the squared summed gradient, eps
 *                              outside the square root, no decay, no clipping).
 *   fso_gather_jagged_class    the lookup of Algorithm 2 taken in its two parts: Forward fetches the
 *                              rows of I_ex^{i+1} ahead of time (they are untouched by iteration
 *                              i), Backward returns the collision rows E_co^{i+1} as the priority
 *                              update leaves them, and merge() puts both into one input batch.
 *                              One call copies the occurrences of one of the two kinds of row.
 *   fso_split_grads            split(G~^i, I~_co^i, I~_ex^i) at the start of Backward of Algorithm 2: the
 *                              batch-major gradient rows separated into the collision part and the exclusive
 *                              part, each in batch order.
 *   fso_partition_fbs          the Fixed Batch Size partitioner of Section 4.1 ("Partitioning
 *                              Algorithms"): samples sorted by UIH length, dealt to the ranks in a
 *                              zig-zag.
 *   fso_partition_vbs          the Variable Batch Size partitioner of the same section: samples sorted by
 *                              length, cut into n runs of about equal total weight (weight = a function
 *                              of the length, L^alpha in the paper; here an integer table so that every
 *                              cut is exact).
 *   fso_jagged_indexed_permute the indexed permute of Section 4.2 ("Triton Kernel Optimizations"):
 *                              the samples of a jagged tensor laid out in a given order.
 *   fso_jagged_keyed_transpose, fso_jagged_ranged_dispatch, fso_jagged_ranged_combine
 *                              the other jagged shuffles Section 4.2 names.  The paper states their
 *                              purpose only (feature-major to batch-major; input and output tensors of
 *                              the ID and embedding AllToAll); the layouts are this build's reading,
 *                              spelled out at each function.
 *
 * Pins (tests/test_oracle_pins.py): brute-force set logic on tiny inputs, dense one-hot
 * reduction, hand-computed Adagrad steps, element-wise Adagrad of a library on the
 * special case where both coincide, a closed form over T steps, and the invariants of
 * the partition (union, disjointness, schedule independence).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { FSO_OK = 0, FSO_EINVAL = -1, FSO_ENOMEM = -2, FSO_ERANGE = -5 };
enum { FSO_F32 = 0, FSO_BF16 = 1 };

/* Set to 0 to accumulate the SUM (not the mean) of squared gradients per row. */
#ifndef FSO_ADAGRAD_MEAN
#define FSO_ADAGRAD_MEAN 1
#endif

/* ---- bf16 <-> f32 ------------------------------------------------------------------- */
static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round to nearest, ties to even; NaN stays NaN */
static uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

static size_t elem_size(int dt) { return dt == FSO_BF16 ? 2 : 4; }

/* ---- O1: gather ---------------------------------------------------------------------- */
/* out[j, :] = table[values[j], :] for every j in [0, n_values).  offsets describes how the
 * n_values occurrences are grouped into `batch` sequences; the output keeps that grouping,
 * so offsets is only validated. */
int fso_gather_jagged(const void *table, int64_t num_rows, int32_t dim, int dt,
                      const int64_t *values, const int64_t *offsets, int64_t batch,
                      int64_t n_values, void *out)
{
    if (num_rows < 0 || dim <= 0 || batch < 0 || n_values < 0) return FSO_EINVAL;
    if (dt != FSO_F32 && dt != FSO_BF16) return FSO_EINVAL;
    if (offsets) {
        if (offsets[0] != 0 || offsets[batch] != n_values) return FSO_ERANGE;
        for (int64_t b = 0; b < batch; ++b)
            if (offsets[b + 1] < offsets[b]) return FSO_ERANGE;
    }
    size_t row_bytes = (size_t)dim * elem_size(dt);
    for (int64_t j = 0; j < n_values; ++j) {
        int64_t r = values[j];
        if (r < 0 || r >= num_rows) return FSO_ERANGE;
        memcpy((char *)out + (size_t)j * row_bytes, (const char *)table + (size_t)r * row_bytes, row_bytes);
    }
    return FSO_OK;
}

/* ---- O1b: lookup of one kind of row ---------------------------------------------------------- */
/* For every occurrence j whose row values[j] IS (which = 1) or IS NOT (which = 0) a member of the
 * ascending distinct list u_t: out[j, :] = table[values[j], :].  The other occurrences of `out` are
 * left as they are: calling it for both kinds, in either order, on tables that agree on the rows
 * each call reads, is merge() of Algorithm 2. */
static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

int fso_gather_jagged_class(const void *table, int64_t num_rows, int32_t dim, int dt,
                            const int64_t *values, int64_t n_values, const int64_t *u_t, int64_t n_t,
                            int which, void *out)
{
    if (num_rows < 0 || dim <= 0 || n_values < 0 || n_t < 0) return FSO_EINVAL;
    if (dt != FSO_F32 && dt != FSO_BF16) return FSO_EINVAL;
    if (which != 0 && which != 1) return FSO_EINVAL;
    for (int64_t i = 1; i < n_t; ++i) if (u_t[i] <= u_t[i - 1]) return FSO_EINVAL;
    size_t row_bytes = (size_t)dim * elem_size(dt);
    for (int64_t j = 0; j < n_values; ++j) {
        int64_t r = values[j];
        if (r < 0 || r >= num_rows) return FSO_ERANGE;
        int member = n_t > 0 && bsearch(&r, u_t, (size_t)n_t, sizeof(int64_t), cmp_i64) != NULL;
        if (member == which)
            memcpy((char *)out + (size_t)j * row_bytes, (const char *)table + (size_t)r * row_bytes, row_bytes);
    }
    return FSO_OK;
}

/* ---- O2: unique ---------------------------------------------------------------------- */
typedef struct { int64_t key; int32_t idx; } keyidx;

static int cmp_keyidx(const void *a, const void *b)
{
    const keyidx *x = (const keyidx *)a, *y = (const keyidx *)b;
    if (x->key < y->key) return -1;
    if (x->key > y->key) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);   /* ties by ascending position */
}

/* unique      : ascending distinct IDs, *n_unique of them
 * seg_offsets : seg_offsets[k]..seg_offsets[k+1] is the range of sorted positions of unique[k]
 * perm        : perm[p] = original position of the occurrence at sorted position p
 *               (sorted by ID, equal IDs in ascending original position)
 * inverse     : ids[j] == unique[inverse[j]]
 * num_rows > 0 bounds the legal IDs to [0, num_rows); 0 means any non-negative int64. */
int fso_unique_ids(const int64_t *ids, int64_t n, int64_t num_rows, int64_t *unique,
                   int32_t *seg_offsets, int32_t *perm, int32_t *inverse, int64_t *n_unique)
{
    if (n < 0 || n > INT32_MAX || num_rows < 0) return FSO_EINVAL;
    *n_unique = 0;
    seg_offsets[0] = 0;
    if (n == 0) return FSO_OK;
    for (int64_t j = 0; j < n; ++j)
        if (ids[j] < 0 || (num_rows > 0 && ids[j] >= num_rows)) return FSO_ERANGE;
    keyidx *a = (keyidx *)malloc((size_t)n * sizeof(keyidx));
    if (!a) return FSO_ENOMEM;
    for (int64_t j = 0; j < n; ++j) { a[j].key = ids[j]; a[j].idx = (int32_t)j; }
    qsort(a, (size_t)n, sizeof(keyidx), cmp_keyidx);
    int64_t u = 0;
    for (int64_t p = 0; p < n; ++p) {
        if (p == 0 || a[p].key != a[p - 1].key) {
            unique[u] = a[p].key;
            seg_offsets[u] = (int32_t)p;
            ++u;
        }
        perm[p] = a[p].idx;
        inverse[a[p].idx] = (int32_t)(u - 1);
    }
    seg_offsets[u] = (int32_t)n;
    *n_unique = u;
    free(a);
    return FSO_OK;
}

/* ---- O3: collision split --------------------------------------------------------------- */
/* u_t, u_t1: ascending distinct IDs of iterations t and t+1.
 * co      = u_t  intersect u_t1   (rows updated at t AND read at t+1: update first)
 * ex      = u_t  minus     u_t1   (rows whose update may be deferred)
 * ex_next = u_t1 minus     u_t    (rows of t+1 that are safe to read before t's updates)
 * co_slot/ex_slot index u_t, ex_next_slot indexes u_t1.  counts = {|co|, |ex|, |ex_next|}. */
int fso_collision_split(const int64_t *u_t, int64_t n_t, const int64_t *u_t1, int64_t n_t1,
                        int64_t *co, int32_t *co_slot, int64_t *ex, int32_t *ex_slot,
                        int64_t *ex_next, int32_t *ex_next_slot, int64_t *counts)
{
    if (n_t < 0 || n_t1 < 0) return FSO_EINVAL;
    for (int64_t i = 1; i < n_t; ++i) if (u_t[i] <= u_t[i - 1]) return FSO_EINVAL;
    for (int64_t i = 1; i < n_t1; ++i) if (u_t1[i] <= u_t1[i - 1]) return FSO_EINVAL;
    int64_t i = 0, j = 0, nco = 0, nex = 0, nexn = 0;
    while (i < n_t || j < n_t1) {
        if (j >= n_t1 || (i < n_t && u_t[i] < u_t1[j])) {
            ex[nex] = u_t[i]; ex_slot[nex] = (int32_t)i; ++nex; ++i;
        } else if (i >= n_t || u_t1[j] < u_t[i]) {
            ex_next[nexn] = u_t1[j]; ex_next_slot[nexn] = (int32_t)j; ++nexn; ++j;
        } else {
            co[nco] = u_t[i]; co_slot[nco] = (int32_t)i; ++nco; ++i; ++j;
        }
    }
    counts[0] = nco; counts[1] = nex; counts[2] = nexn;
    return FSO_OK;
}

/* ---- O4: gradient segment reduce ------------------------------------------------------- */
/* reduced[k, :] = sum of grads[j, :] over the occurrences j of distinct row k, accumulated
 * in fp64 in ascending j (perm is stable), rounded once to fp32. */
int fso_segment_reduce_grads(const float *grads, int64_t n, int32_t dim, const int32_t *perm,
                             const int32_t *seg_offsets, int64_t n_unique, float *reduced)
{
    if (n < 0 || dim <= 0 || n_unique < 0) return FSO_EINVAL;
    double *acc = (double *)malloc((size_t)dim * sizeof(double));
    if (!acc) return FSO_ENOMEM;
    for (int64_t k = 0; k < n_unique; ++k) {
        for (int32_t d = 0; d < dim; ++d) acc[d] = 0.0;
        for (int32_t p = seg_offsets[k]; p < seg_offsets[k + 1]; ++p) {
            const float *g = grads + (size_t)perm[p] * (size_t)dim;
            for (int32_t d = 0; d < dim; ++d) acc[d] += (double)g[d];
        }
        for (int32_t d = 0; d < dim; ++d) reduced[(size_t)k * (size_t)dim + d] = (float)acc[d];
    }
    free(acc);
    return FSO_OK;
}

/* ---- O5: row-wise Adagrad ---------------------------------------------------------------- */
/* For every listed pair (r = rows[i], k = slots[i]):
 *     m    = mean over columns of reduced[k, d]^2            (fp64 sum, rounded once to fp32)
 *     S[r] = S[r] + m                                         (fp32)
 *     c    = lr / (sqrt(S[r]) + eps)                          (fp32)
 *     W[r, d] = W[r, d] - c * reduced[k, d]                   (fp32; bf16 tables: widen, update, RNE)
 * Rows not listed are untouched. */
int fso_rowwise_adagrad_update(void *table, int dt, float *state, int64_t num_rows, int32_t dim,
                               const int64_t *rows, const int32_t *slots, int64_t n_rows,
                               const float *reduced, float lr, float eps)
{
    if (num_rows < 0 || dim <= 0 || n_rows < 0) return FSO_EINVAL;
    if (dt != FSO_F32 && dt != FSO_BF16) return FSO_EINVAL;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t r = rows[i];
        if (r < 0 || r >= num_rows) return FSO_ERANGE;
        const float *g = reduced + (size_t)slots[i] * (size_t)dim;
        double ss = 0.0;
        for (int32_t d = 0; d < dim; ++d) ss += (double)g[d] * (double)g[d];
#if FSO_ADAGRAD_MEAN
        float m = (float)(ss / (double)dim);
#else
        float m = (float)ss;
#endif
        float s_new = state[r] + m;
        state[r] = s_new;
        float c = lr / (sqrtf(s_new) + eps);
        if (dt == FSO_F32) {
            float *w = (float *)table + (size_t)r * (size_t)dim;
            for (int32_t d = 0; d < dim; ++d) {
                float step = c * g[d];
                w[d] = w[d] - step;
            }
        } else {
            uint16_t *w = (uint16_t *)table + (size_t)r * (size_t)dim;
            for (int32_t d = 0; d < dim; ++d) {
                float step = c * g[d];
                float v = bf16_to_f32(w[d]) - step;
                w[d] = f32_to_bf16_rne(v);
            }
        }
    }
    return FSO_OK;
}

/* ---- O6: split of the batch-major gradients ---------------------------------------------------- */
/* Backward of Algorithm 2 begins with split(G~^i, I~_co^i, I~_ex^i): the gradient rows of the batch arrive in
 * batch order, one row per occurrence, and are separated into the rows of collision occurrences and the rows of
 * exclusive occurrences, each part keeping batch order.  (The collision part is what the exposed gradient
 * AllToAll carries, the exclusive part travels with the deferred one.)  An occurrence j is a collision
 * occurrence iff its row values[j] is a member of u_t1, the ascending distinct rows of the lookahead batch.
 *   co_index [n_co], ex_index [n_ex]   the occurrence numbers of the two parts, ascending (I~_co^i, I~_ex^i)
 *   g_co [n_co, dim], g_ex [n_ex, dim] the gradient rows in that order (G~_co^i, G~_ex^i)
 *   counts = {n_co, n_ex} */
int fso_split_grads(const float *grads, int64_t n, int32_t dim, const int64_t *values, const int64_t *u_t1,
                    int64_t n_t1, int32_t *co_index, float *g_co, int32_t *ex_index, float *g_ex, int64_t *counts)
{
    if (n < 0 || n > INT32_MAX || dim <= 0 || n_t1 < 0) return FSO_EINVAL;
    for (int64_t i = 1; i < n_t1; ++i) if (u_t1[i] <= u_t1[i - 1]) return FSO_EINVAL;
    int64_t n_co = 0, n_ex = 0;
    size_t row_bytes = (size_t)dim * sizeof(float);
    for (int64_t j = 0; j < n; ++j) {
        int64_t r = values[j];
        int member = n_t1 > 0 && bsearch(&r, u_t1, (size_t)n_t1, sizeof(int64_t), cmp_i64) != NULL;
        if (member) {
            co_index[n_co] = (int32_t)j;
            memcpy(g_co + (size_t)n_co * (size_t)dim, grads + (size_t)j * (size_t)dim, row_bytes);
            ++n_co;
        } else {
            ex_index[n_ex] = (int32_t)j;
            memcpy(g_ex + (size_t)n_ex * (size_t)dim, grads + (size_t)j * (size_t)dim, row_bytes);
            ++n_ex;
        }
    }
    counts[0] = n_co; counts[1] = n_ex;
    return FSO_OK;
}

/* ---- O7: FBS partitioner --------------------------------------------------------------------- */
/* Samples are sorted by length (ascending; equal lengths keep their sample order) and rank i of n takes
 * the sorted positions  i, 2n-1-i, 2n+i, 4n-1-i, 4n+i, ...  that exist: forth in even rounds of n, back
 * in odd ones.  (The index list printed in Section 4.1 starts its backward rounds one position too far:
 * taken literally rank 0 would get position 2n twice and nobody position n; the zig-zag the section
 * describes in words is the one above.)
 * sample_of [B]: the samples of rank 0 in the order they were dealt, then those of rank 1, ...;
 * rank_offsets [n+1]: where each rank's samples start in sample_of. */
typedef struct { int64_t len; int64_t idx; } lenidx;

static int cmp_lenidx(const void *a, const void *b)
{
    const lenidx *x = (const lenidx *)a, *y = (const lenidx *)b;
    if (x->len != y->len) return x->len < y->len ? -1 : 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

int fso_partition_fbs(const int64_t *lengths, int64_t B, int32_t n_ranks, int32_t *sample_of,
                      int64_t *rank_offsets)
{
    if (B < 0 || n_ranks <= 0) return FSO_EINVAL;
    lenidx *order = (lenidx *)malloc((size_t)(B > 0 ? B : 1) * sizeof(lenidx));
    if (!order) return FSO_ENOMEM;
    for (int64_t b = 0; b < B; ++b) {
        if (lengths[b] < 0) { free(order); return FSO_ERANGE; }
        order[b].len = lengths[b]; order[b].idx = b;
    }
    qsort(order, (size_t)B, sizeof(lenidx), cmp_lenidx);
    int64_t n = n_ranks, at = 0;
    for (int64_t i = 0; i < n; ++i) {
        rank_offsets[i] = at;
        for (int64_t k = 0;; ++k) {
            int64_t pos = (k % 2 == 0) ? k * n + i : (k + 1) * n - 1 - i;
            if (k * n >= B) break;                  /* no sample left in round k for anybody */
            if (pos < B) sample_of[at++] = (int32_t)order[pos].idx;
        }
    }
    rank_offsets[n] = at;
    free(order);
    return at == B ? FSO_OK : FSO_EINVAL;
}

/* ---- O7b: VBS partitioner ---------------------------------------------------------------------- */
/* Samples sorted as for FBS.  weight_of_len[L] >= 0 is the weight of a sample of length L (the caller tabulates
 * its L^alpha, scaled to integers).  With W the total weight and w_before(s) the weight of the sorted
 * positions before s, position s goes to rank min(n-1, floor(n * w_before(s) / W)) - every rank takes the
 * run of samples whose starts fall into its n-th of the total weight (Section 4.1 asks for n runs whose
 * summed weights are about equal and does not state the rule; this one keeps every rank within one
 * sample's weight of W/n).  W == 0: everything goes to rank 0.
 * sample_of [B]: the sorted order; rank_offsets [n+1]: where each rank's run starts. */
int fso_partition_vbs(const int64_t *lengths, int64_t B, const int64_t *weight_of_len, int64_t max_len,
                      int32_t n_ranks, int32_t *sample_of, int64_t *rank_offsets)
{
    if (B < 0 || n_ranks <= 0 || max_len < 0) return FSO_EINVAL;
    lenidx *order = (lenidx *)malloc((size_t)(B > 0 ? B : 1) * sizeof(lenidx));
    if (!order) return FSO_ENOMEM;
    unsigned __int128 total = 0;
    for (int64_t b = 0; b < B; ++b) {
        if (lengths[b] < 0 || lengths[b] > max_len || weight_of_len[lengths[b]] < 0) { free(order); return FSO_ERANGE; }
        order[b].len = lengths[b]; order[b].idx = b;
        total += (unsigned __int128)weight_of_len[lengths[b]];
    }
    qsort(order, (size_t)B, sizeof(lenidx), cmp_lenidx);
    unsigned __int128 before = 0;
    int64_t n = n_ranks, next_rank = 0;               /* ranks below next_rank have their start written */
    for (int64_t s = 0; s < B; ++s) {
        int64_t r = 0;
        if (total > 0) {
            unsigned __int128 q = (unsigned __int128)n * before / total;
            r = q >= (unsigned __int128)n ? n - 1 : (int64_t)q;
        }
        while (next_rank <= r) rank_offsets[next_rank++] = s;
        sample_of[s] = (int32_t)order[s].idx;
        before += (unsigned __int128)weight_of_len[order[s].len];
    }
    while (next_rank <= n) rank_offsets[next_rank++] = B;
    free(order);
    return FSO_OK;
}

/* ---- O8: indexed permute of a jagged tensor ---------------------------------------------------- */
/* out = the samples sample_of[0], sample_of[1], ... of (values, offsets) one after another;
 * out_offsets [n_out + 1] their boundaries.  Elements are elem_bytes wide. */
int fso_jagged_indexed_permute(const void *values, int32_t elem_bytes, const int64_t *offsets, int64_t B,
                               const int32_t *sample_of, int64_t n_out, void *out_values, int64_t *out_offsets)
{
    if (B < 0 || n_out < 0 || elem_bytes <= 0) return FSO_EINVAL;
    if (B > 0 && offsets[0] != 0) return FSO_ERANGE;
    for (int64_t b = 0; b < B; ++b) if (offsets[b + 1] < offsets[b]) return FSO_ERANGE;
    int64_t at = 0;
    out_offsets[0] = 0;
    for (int64_t k = 0; k < n_out; ++k) {
        int64_t p = sample_of[k];
        if (p < 0 || p >= B) return FSO_ERANGE;
        int64_t len = offsets[p + 1] - offsets[p];
        memcpy((char *)out_values + (size_t)at * elem_bytes, (const char *)values + (size_t)offsets[p] * elem_bytes,
               (size_t)len * elem_bytes);
        at += len;
        out_offsets[k + 1] = at;
    }
    return FSO_OK;
}

/* ---- O9: keyed transpose, ranged dispatch, ranged combine -------------------------------------- */
/* A keyed jagged tensor has F keys (features) and B samples: F * B segments.  Feature-major: segment
 * (f, b) is number f * B + b; batch-major: number b * F + f.  A partition of the samples into ranks is
 * given as ranges: rank r owns the samples [rank_offsets[r], rank_offsets[r + 1]). */
static void copy_segment(const void *values, int32_t elem_bytes, const int64_t *offsets, int64_t seg,
                         void *out_values, int64_t *at)
{
    int64_t len = offsets[seg + 1] - offsets[seg];
    memcpy((char *)out_values + (size_t)*at * elem_bytes, (const char *)values + (size_t)offsets[seg] * elem_bytes,
           (size_t)len * elem_bytes);
    *at += len;
}

static int check_segments(const int64_t *offsets, int64_t n_seg)
{
    if (n_seg > 0 && offsets[0] != 0) return FSO_ERANGE;
    for (int64_t i = 0; i < n_seg; ++i) if (offsets[i + 1] < offsets[i]) return FSO_ERANGE;
    return FSO_OK;
}

static int check_ranges(const int64_t *rank_offsets, int32_t n_ranks, int64_t B)
{
    if (n_ranks <= 0 || rank_offsets[0] != 0 || rank_offsets[n_ranks] != B) return FSO_ERANGE;
    for (int32_t r = 0; r < n_ranks; ++r) if (rank_offsets[r + 1] < rank_offsets[r]) return FSO_ERANGE;
    return FSO_OK;
}

/* feature-major in, batch-major out: the segments of sample 0 for every key, then those of sample 1, ... */
int fso_jagged_keyed_transpose(const void *values, int32_t elem_bytes, const int64_t *offsets, int64_t F, int64_t B,
                               void *out_values, int64_t *out_offsets)
{
    if (F < 0 || B < 0 || elem_bytes <= 0) return FSO_EINVAL;
    if (check_segments(offsets, F * B) != FSO_OK) return FSO_ERANGE;
    int64_t at = 0, j = 0;
    out_offsets[0] = 0;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t f = 0; f < F; ++f) {
            copy_segment(values, elem_bytes, offsets, f * B + b, out_values, &at);
            out_offsets[++j] = at;
        }
    return FSO_OK;
}

/* Input of the AllToAll: feature-major in; out holds, rank after rank, what each rank is sent - itself a
 * feature-major keyed jagged tensor over that rank's samples.  splits[r] = elements sent to rank r. */
int fso_jagged_ranged_dispatch(const void *values, int32_t elem_bytes, const int64_t *offsets, int64_t F, int64_t B,
                               const int64_t *rank_offsets, int32_t n_ranks, void *out_values, int64_t *out_offsets,
                               int64_t *splits)
{
    if (F < 0 || B < 0 || elem_bytes <= 0) return FSO_EINVAL;
    if (check_segments(offsets, F * B) != FSO_OK || check_ranges(rank_offsets, n_ranks, B) != FSO_OK) return FSO_ERANGE;
    int64_t at = 0, j = 0;
    out_offsets[0] = 0;
    for (int32_t r = 0; r < n_ranks; ++r) {
        int64_t start = at;
        for (int64_t f = 0; f < F; ++f)
            for (int64_t b = rank_offsets[r]; b < rank_offsets[r + 1]; ++b) {
                copy_segment(values, elem_bytes, offsets, f * B + b, out_values, &at);
                out_offsets[++j] = at;
            }
        splits[r] = at - start;
    }
    return FSO_OK;
}

/* Output of the AllToAll: `values` holds, source rank after source rank, a feature-major keyed jagged tensor
 * over that rank's samples (what fso_jagged_ranged_dispatch lays out); out is one feature-major tensor over
 * all B samples. */
int fso_jagged_ranged_combine(const void *values, int32_t elem_bytes, const int64_t *offsets, int64_t F, int64_t B,
                              const int64_t *rank_offsets, int32_t n_ranks, void *out_values, int64_t *out_offsets)
{
    if (F < 0 || B < 0 || elem_bytes <= 0) return FSO_EINVAL;
    if (check_segments(offsets, F * B) != FSO_OK || check_ranges(rank_offsets, n_ranks, B) != FSO_OK) return FSO_ERANGE;
    int64_t at = 0, j = 0;
    out_offsets[0] = 0;
    for (int64_t f = 0; f < F; ++f)
        for (int32_t r = 0; r < n_ranks; ++r) {
            int64_t first = rank_offsets[r], count = rank_offsets[r + 1] - first;
            for (int64_t i = 0; i < count; ++i) {
                copy_segment(values, elem_bytes, offsets, F * first + f * count + i, out_values, &at);
                out_offsets[++j] = at;
            }
        }
    return FSO_OK;
}

/* exposed for the bf16 conversion pins */
uint16_t fso_f32_to_bf16(float f) { return f32_to_bf16_rne(f); }
float fso_bf16_to_f32(uint16_t h) { return bf16_to_f32(h); }
