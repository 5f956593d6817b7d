/*
 * freescale.h - C ABI of the MI355X (gfx950) library for one embedding-table shard's
 * prioritized embedding updates (FreeScale paper, Section 3.2 and its Algorithm 2,
 * "Prioritized Embedding Autograd Function", with the collectives removed: one GPU, one
 * shard, shard-major IDs).
 *
 * Conventions that hold for every call unless a comment says otherwise
 *   - Every pointer except fs_ctx* and the *_host out-parameters is CALLER-OWNED DEVICE
 *     memory on the context's GPU.  The library neither frees nor keeps it past the stream
 *     work it enqueues.
 *   - Calls are ASYNCHRONOUS: they enqueue kernels on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) and return.  Data-dependent sizes (number of
 *     distinct rows, sizes of the collision / exclusive sets) are written to device scalars
 *     and read from device scalars by the calls that consume them; no call synchronises.
 *   - The return value is a status code.  No call aborts, throws or prints.  Errors that the
 *     host can see (NULL pointer, negative size, unsupported dim/dtype, size beyond the
 *     context capacity) are returned at once and nothing is enqueued.  Errors only the
 *     device can see (row ID outside [0, num_rows), malformed offsets) never fault: the
 *     offending access is suppressed (gathered row zero-filled, update skipped) and a flag is
 *     raised that fs_check_async() reports as FS_ERANGE.
 *   - n == 0 is a valid no-op everywhere.
 *   - Row layout: tables are row-major [num_rows, dim], 16-byte aligned, fp32 or bf16; the
 *     Adagrad state is one fp32 per row; gradients are fp32 [n, dim].  dim must be a
 *     multiple of 4 (fp32) or 8 (bf16) and at most FS_MAX_DIM.
 *   - One context serves one GPU and one caller thread at a time.  Calls that use the
 *     context workspace (fs_unique_ids, fs_collision_split, fs_segment_reduce_grads,
 *     fs_prioritized_step) must not overlap each other on different streams.
 */
#ifndef FREESCALE_H
#define FREESCALE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FS_MAX_DIM 256

typedef struct fs_ctx fs_ctx;            /* opaque: workspace, side streams, events, last error */
typedef void *fs_stream;                 /* a hipStream_t */

typedef enum { FS_F32 = 0, FS_BF16 = 1 } fs_dtype;

enum {
    FS_OK = 0,
    FS_EINVAL = -1,      /* bad argument visible to the host */
    FS_ENOMEM = -2,      /* size beyond the context capacity, or allocation failure */
    FS_EHIP = -3,        /* a HIP runtime call failed; fs_last_error() has its text */
    FS_ENOTIMPL = -4,
    FS_ERANGE = -5       /* device-detected: row ID out of range / malformed offsets */
};

/* ---- context ------------------------------------------------------------------------- */

/* Allocates the workspace for inputs of at most max_ids IDs per iteration and rows of at
 * most max_dim columns on GPU `device` (sort double buffers, histograms, scan partials,
 * fp64 partial rows of the segment reduce), two side streams at default priority and the
 * events that order the passes.  This is the only call that allocates device memory. */
int fs_ctx_create(fs_ctx **out, int device, int64_t max_ids, int32_t max_dim);
int fs_ctx_destroy(fs_ctx *ctx);

/* Text of the last host-visible error on this context ("" if none).  Never NULL.  ctx == NULL: the text of
 * the calling thread's last failed call that takes no context. */
const char *fs_last_error(const fs_ctx *ctx);

/* Waits for `stream`, then reports and clears the device-side error flags:
 * FS_OK, or FS_ERANGE if any kernel since the last check suppressed an access. */
int fs_check_async(fs_ctx *ctx, fs_stream stream);

/* Bytes of device workspace held by the context. */
size_t fs_ctx_workspace_bytes(const fs_ctx *ctx);

/* ---- the five operations ---------------------------------------------------------------- */

/* Lookup(I) of Algorithm 2 (embedding lookup of Section 2.1 on the jagged ID layout of
 * Section 4.2):  out[j, :] = table[values[j], :]  for j in [0, n_values), bit-exact.
 * values  [n_values] int64 row IDs of `batch` sequences laid end to end;
 * offsets [batch+1]  int64, offsets[b]..offsets[b+1] is sequence b (may be empty); may be NULL,
 *         otherwise it is validated on the device (offsets[0]==0, non-decreasing,
 *         offsets[batch]==n_values) - the output keeps the same jagged grouping.
 * out     [n_values, dim] of the table's dtype.  An out-of-range ID yields a zero row. */
int fs_gather_jagged(fs_ctx *ctx, const void *table, int64_t num_rows, int32_t dim, fs_dtype dt,
                     const int64_t *values, const int64_t *offsets, int64_t batch, int64_t n_values,
                     void *out, fs_stream stream);

/* Distinct rows of one iteration's IDs (collisions are defined on rows, Section 2.3).
 * ids          [n] int64, each in [0, num_rows) when num_rows > 0; num_rows == 0 sorts on all
 *              63 value bits of non-negative IDs.
 * unique       [>= n]   ascending distinct IDs; entries past *n_unique_dev are unspecified
 * seg_offsets  [>= n+1] sorted positions seg_offsets[k]..seg_offsets[k+1] hold unique[k]
 * perm         [n]      original position of the occurrence at each sorted position (stable:
 *                       equal IDs keep ascending original position)
 * inverse      [n]      ids[j] == unique[inverse[j]]          (may be NULL)
 * n_unique_dev [1]      int64 device scalar
 * n <= context max_ids. */
int fs_unique_ids(fs_ctx *ctx, const int64_t *ids, int64_t n, int64_t num_rows,
                  int64_t *unique, int32_t *seg_offsets, int32_t *perm, int32_t *inverse,
                  int64_t *n_unique_dev, fs_stream stream);

/* compute_collision(I^i, I^{i+1}) -> I_co^i, I_ex^i, I_ex^{i+1} of Algorithm 2, on distinct
 * ascending row lists:
 *   co      = u_t  intersect u_t1   rows updated at t and read at t+1 (update these first)
 *   ex      = u_t  minus u_t1       rows whose update may be deferred
 *   ex_next = u_t1 minus u_t        rows of t+1 that may be fetched before t's updates land
 * u_t [*n_t_dev], u_t1 [*n_t1_dev] ascending; cap_t / cap_t1 bound the two counts (host
 * values used to size the launch; the outputs need that many entries).
 * co_slot / ex_slot index u_t (and so the reduced-gradient rows), ex_next_slot indexes u_t1.
 * n_t1_dev may be NULL with cap_t1 == 0: no lookahead batch, everything is exclusive.
 * counts_dev [3] int64 = |co|, |ex|, |ex_next|.  All outputs ascending. */
int fs_collision_split(fs_ctx *ctx, const int64_t *u_t, const int64_t *n_t_dev,
                       const int64_t *u_t1, const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1,
                       int64_t *co, int32_t *co_slot, int64_t *ex, int32_t *ex_slot,
                       int64_t *ex_next, int32_t *ex_next_slot, int64_t *counts_dev, fs_stream stream);

/* fs_collision_split for callers that cannot allocate device memory or create a context where they stand:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (no
 * context), same outputs bit for bit.  The membership flags and per-tile counts that fs_collision_split keeps
 * in the context's workspace live in a fixed device array of the library instead (about 2.1 MB per GPU, held
 * until the process ends); the call allocates and frees nothing.  Works on the CURRENT device, which must
 * own every pointer.
 *   cap_t, cap_t1 <= FS_STATIC_SPLIT_MAX_ROWS, else FS_ENOMEM and nothing is enqueued (use the context form).
 *   Every call on a GPU shares that GPU's array: calls whose stream work may overlap on one GPU race with
 *   each other - order them (one stream, or events).  Nothing in the array has to be cleared between calls.
 *   The array's address is looked up once per GPU, by fs_ctx_create for its device or else by the first call
 *   here on that GPU; make that first call outside a capture.
 * Errors are returned as status codes; fs_last_error(NULL) has the text of the calling thread's last one. */
#define FS_STATIC_SPLIT_MAX_ROWS (1 << 20)
int fs_collision_split_static(const int64_t *u_t, const int64_t *n_t_dev, const int64_t *u_t1,
                              const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1, int64_t *co,
                              int32_t *co_slot, int64_t *ex, int32_t *ex_slot, int64_t *ex_next,
                              int32_t *ex_next_slot, int64_t *counts_dev, fs_stream stream);

/* First half of update_embedding(I, G) of Algorithm 2: one summed gradient per distinct row,
 *   reduced[k, :] = sum over sorted positions p in [seg_offsets[k], seg_offsets[k+1]) of
 *                   grads[perm[p], :]
 * accumulated in fp64 in a fixed order (results do not vary run to run) and rounded once to
 * fp32.  grads [n, dim] fp32; reduced needs *n_unique_dev rows (at most n).
 * inverse [n] is OPTIONAL (NULL allowed): the inverse map that fs_unique_ids wrote next to perm
 * and seg_offsets.  With it every wavefront reads the segment of its positions directly instead
 * of searching seg_offsets; the results are bit-identical either way. */
int fs_segment_reduce_grads(fs_ctx *ctx, const float *grads, int64_t n, int32_t dim,
                            const int32_t *perm, const int32_t *seg_offsets, const int32_t *inverse,
                            const int64_t *n_unique_dev, float *reduced, fs_stream stream);

/* Second half of update_embedding(I, G): fused row-wise Adagrad on the listed rows, in place.
 * For i < *n_rows_dev, r = rows[i], k = slots[i]:
 *     S[r] += mean over columns of reduced[k, :]^2
 *     W[r, :] -= lr * reduced[k, :] / (sqrt(S[r]) + eps)        (bf16: widen, update, round
 *                                                                to nearest even)
 * Called once with the collision rows (priority pass) and once with the exclusive rows
 * (deferred pass); rows must be distinct within and across concurrent calls.  cap bounds
 * *n_rows_dev (host value used to size the launch).  Out-of-range rows are skipped and
 * flagged. */
int fs_rowwise_adagrad_update(fs_ctx *ctx, void *table, fs_dtype dt, float *state, int64_t num_rows,
                              int32_t dim, const int64_t *rows, const int32_t *slots,
                              const int64_t *n_rows_dev, int64_t cap, const float *reduced,
                              float lr, float eps, fs_stream stream);

/* One part of the lookup of Algorithm 2.  Forward fetches the rows of I_ex^{i+1} ahead of time (no
 * update of iteration i touches them), Backward returns the collision rows E_co^{i+1} as the priority
 * update leaves them, and merge() makes one input batch of both.  On one shard both parts land directly
 * in the batch (`out`, [n, dim] in the order of `values`), so merge() is the two calls having finished:
 *   which = 0: out[j, :] = table[values[j], :] for the occurrences j of rows NOT flagged (exclusive rows)
 *   which = 1: the same for the occurrences of flagged rows (collision rows)
 * where the flag of occurrence j is co_flag[inverse[j]]; the other occurrences of `out` are left alone.
 * inverse [n] is the inverse map of fs_unique_ids(values); co_flag [n_unique] is the co_flag_t1 a step
 * call wrote, or any byte per distinct row.  offsets (NULL allowed), range checks and errors as in
 * fs_gather_jagged. */
int fs_gather_jagged_class(fs_ctx *ctx, const void *table, int64_t num_rows, int32_t dim, fs_dtype dt,
                           const int64_t *values, const int64_t *offsets, int64_t batch, int64_t n,
                           const int32_t *inverse, const uint8_t *co_flag, int which, void *out,
                           fs_stream stream);

/* ---- the load balancer's data path on one GPU ------------------------------------------------ */

/* Fixed Batch Size partitioner (Section 4.1, "Partitioning Algorithms"): the B samples are sorted by UIH
 * length (ascending, equal lengths in sample order) and dealt to n_ranks ranks in a zig-zag - rank i takes
 * the sorted positions i, 2n-1-i, 2n+i, 4n-1-i, ... that exist (forth in even rounds of n, back in odd ones;
 * the index list printed in Section 4.1 starts the backward rounds one position later, which is not a
 * partition).  Every rank gets B/n samples (one more for
 * some when n does not divide B), and long and short samples are spread evenly.
 *   lengths      [B] int64, device; each in [0, max_len] (max_len: host value that sizes the sort; a length
 *                outside is reported as FS_ERANGE by fs_check_async)
 *   sample_of    [B] int32 out: the samples of rank 0 in the order dealt, then those of rank 1, ...
 *   rank_offsets [n_ranks + 1] int64 out: where each rank's samples start in sample_of
 * B <= context max_ids.  Uses the context's index workspace like fs_unique_ids. */
int fs_partition_fbs(fs_ctx *ctx, const int64_t *lengths, int64_t B, int64_t max_len, int32_t n_ranks,
                     int32_t *sample_of, int64_t *rank_offsets, fs_stream stream);

/* Variable Batch Size partitioner (same section): the samples sorted as for FBS are cut into n_ranks runs of
 * about equal total weight, so that ranks get different numbers of samples of similar length.  The weight of
 * a sample is a function of its length - L^alpha in the paper, here weight_of_len [max_len + 1] int64 on the
 * device, tabulated and scaled to integers by the caller, which makes every cut exact.  With W the total and
 * w_before(s) the weight of the sorted positions before s, position s goes to rank
 * min(n_ranks - 1, floor(n_ranks * w_before(s) / W)) (the paper does not state its rule; this one keeps every
 * rank within one sample's weight of W / n_ranks).  W == 0: rank 0 takes everything.
 *   sample_of    [B] int32 out: the sorted order;  rank_offsets [n_ranks + 1] int64 out: the cuts
 * n_ranks * W must stay below 2^63; that, a negative weight or a length outside [0, max_len] are reported as
 * FS_ERANGE by fs_check_async.  The paper's AutoTune (batch sizes corrected from measured step times) is the
 * caller's business: it changes the weights.  B <= context max_ids. */
int fs_partition_vbs(fs_ctx *ctx, const int64_t *lengths, int64_t B, const int64_t *weight_of_len, int64_t max_len,
                     int32_t n_ranks, int32_t *sample_of, int64_t *rank_offsets, fs_stream stream);

/* Indexed permute of a jagged tensor (Section 4.2, "Triton Kernel Optimizations": the kernel that applies a
 * partitioning to the gathered IDs): output sample k is input sample sample_of[k], k < n_out.
 *   values       [n_values] elements of elem_bytes bytes each (a multiple of 4: 8 for IDs, a row of
 *                embeddings otherwise), offsets [B + 1] int64: the input
 *   sample_of    [n_out] int32: any selection of input samples (a permutation, a rank's share, repeats)
 *   out_values   [cap_out] elements, out_offsets [n_out + 1] int64: the output; cap_out is a host-side bound
 *                on the number of output elements (it sizes the copy; for a permutation n_values)
 * A sample index outside [0, B), a sample whose boundaries do not lie inside the values, or more output
 * elements than cap_out (the copy stops there) are reported as FS_ERANGE by fs_check_async.
 * n_out <= context max_ids. */
int fs_jagged_indexed_permute(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                              const int64_t *offsets, int64_t B, const int32_t *sample_of, int64_t n_out,
                              void *out_values, int64_t cap_out, int64_t *out_offsets, fs_stream stream);

/* The other jagged shuffles Section 4.2 names, on a keyed jagged tensor: F keys (features) x B samples, F * B
 * segments described by offsets [F * B + 1] over values [n_values] of elem_bytes bytes each (a multiple of 4).
 * Feature-major: segment (f, b) is number f * B + b; batch-major: number b * F + f.  The paper states what
 * these kernels are for, not their layouts; the layouts below are this library's.  Each writes out_values
 * [n_values] and out_offsets [F * B + 1]; F * B <= context max_ids; malformed offsets or ranges are reported
 * as FS_ERANGE by fs_check_async (the segments concerned come out empty).
 *
 * Keyed transpose: feature-major in, batch-major out. */
int fs_jagged_keyed_transpose(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                              const int64_t *offsets, int64_t F, int64_t B, void *out_values, int64_t *out_offsets,
                              fs_stream stream);

/* Ranged dispatch: the input of the ID or embedding AllToAll.  Rank r of n_ranks owns the samples
 * [rank_offsets[r], rank_offsets[r + 1]) (rank_offsets [n_ranks + 1] int64 on the device, ascending from 0 to
 * B - what fs_partition_fbs and fs_jagged_indexed_permute leave).  Feature-major in; out holds, rank after
 * rank, the feature-major tensor over that rank's samples; splits [n_ranks] int64 = elements sent to each. */
int fs_jagged_ranged_dispatch(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                              const int64_t *offsets, int64_t F, int64_t B, const int64_t *rank_offsets,
                              int32_t n_ranks, void *out_values, int64_t *out_offsets, int64_t *splits,
                              fs_stream stream);

/* Ranged combine: the output of the AllToAll.  `values` / `offsets` hold, source rank after source rank, the
 * feature-major tensor over that rank's samples (the layout fs_jagged_ranged_dispatch produces); out is one
 * feature-major tensor over all B samples.  Undoes fs_jagged_ranged_dispatch for the same ranges. */
int fs_jagged_ranged_combine(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                             const int64_t *offsets, int64_t F, int64_t B, const int64_t *rank_offsets,
                             int32_t n_ranks, void *out_values, int64_t *out_offsets, fs_stream stream);

/* ---- the fused update path of the whole iteration ------------------------------------------ */

/* Rows with at most this many occurrences in a batch take the short path of the fused update (all
 * their gradient rows are requested at once by one group of lanes); rows with more go through the
 * class order below. */
#define FS_SHORT_SEGMENT 8

/* Class order of the occurrences of batch t (input of fs_reduce_update_class), for the rows with
 * more than FS_SHORT_SEGMENT occurrences: the occurrences of such collision rows first (class
 * 0), then those of such exclusive rows (class 1); inside a class by ascending row, inside a row
 * in batch order.  Does fs_collision_split (same arguments, same outputs) and then lays the
 * batch out:
 *   cperm [n_t]          occurrence (row of G_t) at each class position
 *   cslot [n_t]          slot in u_t of the row at each class position
 *   cstart[cap_t]        class position of the first occurrence of u_t[k] (rows in the class
 *                        order only; other entries are unspecified)
 *   class_pos_dev [2]    int32: number of class-0 positions, number of class positions
 *   short_rec [2 * cap_t * 12] int32: one 12-word record per row of U_t, at the row's place in
 *                        its class list (co rows from word 0, ex rows from word 12 * cap_t):
 *                        row (2 words, low first), slot, number of occurrences, and for rows
 *                        with at most FS_SHORT_SEGMENT occurrences the occurrences (rows of G_t)
 *                        in batch order
 * seg_offsets_t, perm_t: the layout of batch t as written by fs_unique_ids (both required; inverse_t is
 * not read and may be NULL: the row of a sorted position is found in seg_offsets_t, which costs no random
 * access); cap_t is also the capacity of cstart.  This is the prioritization of Section 3.2
 * carried down to the gradient rows: the priority pass reads only what collision rows need. */
int fs_collision_split_classes(fs_ctx *ctx, const int64_t *u_t, const int64_t *n_t_dev,
                               const int64_t *u_t1, const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1,
                               const int32_t *seg_offsets_t, const int32_t *perm_t, const int32_t *inverse_t,
                               int64_t n_t, int64_t *co, int32_t *co_slot, int64_t *ex, int32_t *ex_slot,
                               int64_t *ex_next, int32_t *ex_next_slot, int64_t *counts_dev, int32_t *cperm,
                               int32_t *cslot, int32_t *cstart, int32_t *class_pos_dev, int32_t *short_rec,
                               fs_stream stream);

/* split(G~^i, I~_co^i, I~_ex^i) at the start of Backward of Algorithm 2: the batch-major gradient rows (one per
 * occurrence, in batch order) packed into the collision part and the exclusive part, each in batch order - the
 * tensors that the exposed and the deferred gradient AllToAll of Section 3.2 are fed with.  An occurrence belongs
 * to the collision part iff its row is a collision row of the batch (co_slot / counts_dev[0] as fs_collision_split
 * left them; inverse_t [n] is the inverse map of fs_unique_ids for the batch, REQUIRED here; cap_u bounds the
 * number of distinct rows and is at most n).
 *   co_index [n] / ex_index [n]   int32 out: occurrence numbers of the two parts, ascending (I~_co^i, I~_ex^i)
 *   g_co [n, dim] / g_ex [n, dim] fp32 out: the gradient rows in that order (only the first counts are written)
 *   part_pos [n]                  int32 out: for occurrence j its row number in g_co, or -1 - its row number in g_ex
 *   part_counts_dev [2]           int64 out: occurrences in the collision part, in the exclusive part
 * n <= context max_ids; uses the context's index workspace like fs_collision_split. */
int fs_split_grads(fs_ctx *ctx, const float *grads, int64_t n, int32_t dim, const int32_t *inverse_t,
                   const int32_t *co_slot, const int64_t *n_co_dev, int64_t cap_u, int32_t *co_index, float *g_co,
                   int32_t *ex_index, float *g_ex, int32_t *part_pos, int64_t *part_counts_dev, fs_stream stream);

/* Lets the fused passes read the packed parts of fs_split_grads instead of the batch-major gradients: rewrites
 * the class order (cperm) and the occurrence lists of the records (short_rec, both as fs_collision_split_classes
 * left them for a batch of n_t occurrences; counts_dev its row counts) through part_pos into cperm_parts [n_t] and
 * short_rec_parts [2 * n_t * 12].  fs_reduce_update_class(0, grads = g_co, ..., short_rec_parts, cperm_parts) and
 * fs_reduce_update_class(1, grads = g_ex, ..., short_rec_parts + 12 * n_t, cperm_parts) then give the results of
 * the same calls on the batch-major tensor bit for bit (pass n = n_t to both). */
int fs_class_order_for_parts(fs_ctx *ctx, const int32_t *part_pos, int64_t n_t, const int32_t *cperm,
                             const int32_t *class_pos_dev, const int32_t *short_rec, const int64_t *counts_dev,
                             int32_t *cperm_parts, int32_t *short_rec_parts, fs_stream stream);

/* update_embedding(I, G) of Algorithm 2 for one class of rows: the segment reduce of
 * fs_segment_reduce_grads and the Adagrad update of fs_rowwise_adagrad_update fused, same
 * arithmetic (fp64 sums in a fixed order, one rounding to fp32, then the update), restricted to
 * the rows of class `cls` (0: collision rows = priority pass, 1: exclusive rows = deferred
 * pass).  short_rec_cls / n_rows_dev: the records of this class (short_rec + cls * 12 * cap_t)
 * and the number of its rows (counts_dev + cls).  One launch: its first workgroups take the
 * position-cut path over the class order, the others the short path over the records.
 * The summed gradients do not go through memory unless `reduced` (OPTIONAL, [n_unique, dim]
 * fp32) is given, in which case the rows of this class are also written there.
 * Calls for the two classes may run side by side on different streams; calls for the same class
 * on one context must be ordered. */
int fs_reduce_update_class(fs_ctx *ctx, int cls, void *table, fs_dtype dt, float *state, int64_t num_rows,
                           int32_t dim, float lr, float eps, const float *grads, int64_t n,
                           const int64_t *u_t, const int32_t *seg_offsets, const int32_t *short_rec_cls,
                           const int64_t *n_rows_dev, const int32_t *cperm, const int32_t *cslot, const int32_t *cstart,
                           const int32_t *class_pos_dev, float *reduced, fs_stream stream);

/* ---- one whole iteration ------------------------------------------------------------------ */

/* Arguments of fs_prioritized_step (plain pointers; `t` is the iteration whose gradients
 * arrive, `t1` the lookahead batch whose rows are fetched). */
typedef struct fs_step_args {
    void *table; float *state; int64_t num_rows; int32_t dim; int32_t dtype; /* fs_dtype */
    float lr, eps;
    /* iteration t: layout produced by the previous step (or by fs_unique_ids), gradients.  inverse_t is not
     * read by the step calls and may be NULL */
    const int64_t *u_t; const int32_t *seg_offsets_t; const int32_t *perm_t; const int32_t *inverse_t;
    const int64_t *n_unique_t_dev;
    const float *grads_t; int64_t n_t;
    /* lookahead batch t+1 (values_t1 == NULL: last iteration, every row is exclusive) */
    const int64_t *values_t1; const int64_t *offsets_t1; int64_t batch_t1; int64_t n_t1;
    /* outputs: layout of t+1 (already there if fs_unique_ids_ahead was called on these buffers).  inverse_t1
     * is OPTIONAL (NULL: not written - a scattered 4-byte write per occurrence saved); only the two-part
     * lookup reads it */
    int64_t *u_t1; int32_t *seg_offsets_t1; int32_t *perm_t1; int32_t *inverse_t1; int64_t *n_unique_t1_dev;
    /* outputs: the split of U_t */
    int64_t *co; int32_t *co_slot; int64_t *ex; int32_t *ex_slot; int64_t *ex_next; int32_t *ex_next_slot;
    int64_t *counts_dev;        /* [3] */
    /* outputs: class order of batch t: [n_t], [n_t], [n_t], [2] (see fs_collision_split_classes) */
    int32_t *cperm; int32_t *cslot; int32_t *cstart; int32_t *class_pos_dev; int32_t *short_rec /* [24 * n_t] */;
    /* outputs: reduced gradients [n_t, dim] capacity (OPTIONAL, may be NULL: the step does not need
     * them in memory), and gathered rows of t+1 [n_t1, dim] */
    float *reduced; void *emb_t1;
    /* output (OPTIONAL, may be NULL; needed by the two-part lookup): [n_t1] bytes, for every row of u_t1
     * 1 if it is a collision row (also in u_t), else 0; written with the split */
    uint8_t *co_flag_t1;
    /* output (OPTIONAL, may be NULL): [n_t1] the IDs of the lookahead batch in ascending order, every occurrence
     * listed (sorted_ids_t1[p] is the row of the occurrence perm_t1[p]); written with the layout of t+1.  Given,
     * the lookup of the lookahead batch walks the batch row by row instead of occurrence by occurrence: all
     * occurrences of a row are neighbours, so a row is fetched once however far apart its occurrences lie */
    int64_t *sorted_ids_t1;
} fs_step_args;

/* Iteration t on one shard, scheduled as Section 3.2 prescribes (strict write-read ordering
 * on collision rows only):
 *   side stream A : fs_unique_ids(values_t1) -> fs_collision_split_classes(U_t, U_t1)
 *   `stream`      : wait A; fs_reduce_update_class(0)  [priority pass: collision rows];
 *                   fs_gather_jagged(values_t1)
 *   side stream B : after A: fs_reduce_update_class(1) [deferred pass: exclusive rows],
 *                   overlapping the gather, which is race-free because ex and U_t1 are disjoint
 * and `stream` finally waits for B, so the step is complete when `stream` is.  Results are
 * identical to running the five operations one after another. */
int fs_prioritized_step(fs_ctx *ctx, const fs_step_args *args, fs_stream stream);

/* The index half of an iteration alone - what Forward of Algorithm 2 does with the prefetched
 * indices of the next batch, long before the gradients arrive: on side stream A (forked from
 * `stream`, joined back into it) dedup values_t1 into the layout of t+1 (unless
 * fs_unique_ids_ahead already did), split U_t against U_t1 and lay batch t out in class order.
 * Uses only the index fields of `args` (no gradients, no table access). */
int fs_step_forward(fs_ctx *ctx, const fs_step_args *args, fs_stream stream);

/* Dedup of a prefetched batch ahead of time: fs_unique_ids on one of the context's two index
 * streams (used in turn), ordered after the work queued on `stream` so far and after nothing
 * else.  Indices arrive batches ahead of the gradients (Forward of Algorithm 2 consumes
 * prefetched indices), and the dedup is a chain of small latency-bound launches: started early
 * it hides behind the bandwidth-bound passes of earlier iterations.  The results are consumed by
 * a step call whose u_t1 is this `unique` buffer (it waits for them instead of doing the dedup
 * itself); anyone else must call fs_step_join or fs_check_async first.  The outputs must not be
 * in use by work that is not ordered before `stream`'s current position, and `ids` must stay in
 * place until the dedup has run (it is only enqueued when the call returns); in a loop of pipelined
 * calls that means five layout buffers in rotation when the dedup runs two batches ahead of the
 * call that consumes it as u_t1.  When more ahead-of-time results are outstanding than the context
 * tracks, the oldest finished one that no call has asked for is forgotten (its data stay valid).
 * stream == FS_STREAM_LAST_STEP: no event is recorded on any stream of the caller; the dedup is
 * ordered after the position the caller's stream had at the START of the most recent
 * fs_prioritized_step_pipelined call (its deferred pass may still be running: one more layout
 * buffer in the rotation, six).  The caller vouches that `ids` are complete by then. */
#define FS_STREAM_LAST_STEP ((fs_stream)(intptr_t)-1)
int fs_unique_ids_ahead(fs_ctx *ctx, const int64_t *ids, int64_t n, int64_t num_rows,
                        int64_t *unique, int32_t *seg_offsets, int32_t *perm, int32_t *inverse,
                        int64_t *n_unique_dev, fs_stream stream);

/* The whole index half of an iteration ahead of time - fs_step_forward on one of the context's
 * index streams, ordered like fs_unique_ids_ahead (`stream`, or FS_STREAM_LAST_STEP).  It dedups
 * args->values_t1 (unless fs_unique_ids_ahead already did), waits for the layout of batch t if that
 * is still in the making (the index half of t-1 produces it), splits, and lays batch t out in class
 * order with its records.  fs_prioritized_step_pipelined then finds the index half of its `next`
 * (or of its `cur`, on the first call) done and only waits for it; its side stream is left with
 * the deferred pass alone.  Issued for iteration t+2 before the pipelined call of iteration t,
 * the chain of a dozen small launches has two iterations' time to finish.  Buffers in rotation
 * for that pattern: six layouts and five split/class bundles with FS_STREAM_LAST_STEP, five and
 * four with `stream`.  A chain of launches per iteration costs the bandwidth-bound passes more
 * than chains shared by several iterations: prefer fs_step_forward_ahead_batch. */
int fs_step_forward_ahead(fs_ctx *ctx, const fs_step_args *args, fs_stream stream);

/* The index halves of `count` (1..FS_MAX_AHEAD_BATCH) argument records ahead of time in SHARED
 * launches: every kernel of the chain (three radix passes, compaction, split, class order) runs once
 * for all of them.  A launch disturbs whatever runs beside it on the chip by about as much however
 * small it is, so what the index work costs the bandwidth-bound passes falls with the number of
 * iterations - or tables - that share a chain.  The records may be consecutive iterations of one table
 * (args[k+1].u_t == args[k].u_t1: the layout that record k+1 splits is the one the dedup of record k
 * produces in this very call) or belong to different tables; each is found and waited for by the
 * pipelined call that names its counts_dev, like the result of fs_step_forward_ahead, which is this
 * call with count == 1.  Ordering, `stream` and the lifetime of the inputs are as for
 * fs_step_forward_ahead.  Buffers in rotation when a batch of K consecutive iterations is issued D
 * iterations before the pipelined call of its first one, with FS_STREAM_LAST_STEP: K + D + 3 layouts
 * and K + D + 2 split/class bundles. */
#define FS_MAX_AHEAD_BATCH 8
int fs_step_forward_ahead_batch(fs_ctx *ctx, const fs_step_args *args, int count, fs_stream stream);

/* Steady-state form of the iteration, software-pipelined by one batch exactly as Algorithm 2
 * interleaves its Forward and Backward.  For iteration `cur`:
 *   `stream`      : wait for the side work of the previous call; priority pass of cur
 *                   (fs_reduce_update_class(0)); gather of cur's lookahead rows
 *   side stream A : (after the work queued on `stream` before the call, i.e. cur's gradients)
 *                   deferred pass of cur (fs_reduce_update_class(1)); then the index half of
 *                   `next`: dedup of next's lookahead IDs (or a wait for fs_unique_ids_ahead),
 *                   split of next's U_t, class order of next's batch
 * The split and class order of `cur` must already exist: they were produced by the previous call
 * of this function (as its `next`) or by fs_step_forward.  `next` may be NULL (last iteration).
 * Nothing on A is waited for when the call returns: the next pipelined call waits for it before
 * its priority pass (its gather may read rows the deferred pass writes), and so do fs_step_join,
 * fs_check_async and every call that reuses the index workspace.  Use consecutive pipelined
 * calls on ONE stream.  The buffers of consecutive calls must be distinct: three split/class
 * buffers in rotation, and three layout buffers (five with fs_unique_ids_ahead two batches
 * ahead; see fs_step_forward_ahead for its rotation).  If the index half of `next` (or, on the
 * first call of a run, of `cur`) was done ahead of time with fs_step_forward_ahead, the call only
 * waits for it. */
int fs_prioritized_step_pipelined(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next,
                                  fs_stream stream);

/* The same for `count` (1..FS_MAX_STEP_TABLES) tables of one shard in ONE call: cur[k] / next[k] are the
 * records of table k (next == NULL: last iteration of all of them).  The tables are independent
 * problems (table-local IDs, own buffers); what they share is the schedule: one fork event, one wait for
 * the side stream per call instead of one per table - the cross-stream waits are what a call costs the
 * host - priority pass and gather of every table on `stream`, the deferred passes of all of them on
 * side stream A; and the launches: tables of one dtype and row width take their priority passes in
 * one launch, their deferred passes in one and their gathers in one (as many as fit the context's
 * partial-row space at a time).  With fs_step_forward_ahead_batch taking the index halves of the same tables in shared
 * launches, an iteration of a shard with eight tables is two calls.  Results are those of one
 * fs_prioritized_step_pipelined call per table, bit for bit; the context must be sized for the largest
 * table's batch and dim. */
#define FS_MAX_STEP_TABLES 16
int fs_prioritized_step_pipelined_multi(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next,
                                        int count, fs_stream stream);

/* fs_prioritized_step_pipelined_multi with the lookup in its two parts, as Forward and Backward of
 * Algorithm 2 have it:
 *   `stream`      : wait for the side work of the previous call; priority pass of cur; lookup of the
 *                   COLLISION rows of cur's lookahead batch (fs_gather_jagged_class, which = 1) - the
 *                   only rows whose values the priority pass decides
 *   side stream A : deferred pass of cur; index half of `next` (or the wait for it); then the lookup of
 *                   the EXCLUSIVE rows of next's lookahead batch (which = 0) into next's emb_t1 - they are
 *                   rows of neither cur's nor next's update sets, and every older deferred pass has landed
 * so that between the arrival of the gradients and the complete input batch lie the priority pass and
 * the collision rows only.  A lookahead batch of `cur` whose exclusive rows the previous call of this
 * function did not fetch (first call of a run; another pipelined or self-contained step, a stand-alone
 * update or a table initialisation on the context in between; fs_two_part_forget) gets its whole lookup on
 * `stream`.  fs_check_async, fs_step_join and the ahead-of-time index calls keep what was fetched.  Whoever
 * changes table rows or the output batch by other means between two calls must call fs_two_part_forget.  Every record with a lookahead batch needs co_flag_t1.  Results are those of
 * fs_prioritized_step_pipelined_multi, bit for bit; emb_t1 of cur is complete when `stream` is.  The output
 * batches of three consecutive iterations must be distinct buffers: while the caller consumes one, this call
 * completes the next and the side stream already fills the one after. */
int fs_prioritized_step_two_part_multi(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next,
                                       int count, fs_stream stream);

/* Forget what the last fs_prioritized_step_two_part_multi call fetched ahead of time: the next call does the
 * whole lookup of its lookahead batch (host-side bookkeeping only). */
int fs_two_part_forget(fs_ctx *ctx);

/* Makes `stream` wait for everything earlier calls left running on the context's own streams
 * (side work of the last pipelined call, outstanding ahead-of-time dedups); no-op if there is
 * none. */
int fs_step_join(fs_ctx *ctx, fs_stream stream);

/* The pipelined call and fs_unique_ids_ahead hand the enqueueing of their side-stream work to
 * host threads owned by the context (on by default; started on first use, joined by
 * fs_ctx_destroy), because the host cost of the launches and cross-stream waits would otherwise
 * exceed the GPU time of an iteration.  on == 0 makes the calling thread enqueue everything.
 * The results do not depend on this setting. */
int fs_ctx_set_threaded_enqueue(fs_ctx *ctx, int on);

/* ---- the pipelined iteration as a HIP graph ---------------------------------------------------- */

/* fs_graph_capture_pipelined records exactly the work of fs_prioritized_step_pipelined(cur,
 * next) (same kernels, same dependencies, pointers baked in: the buffers must stay alive and in
 * place; the dedup of next's lookahead IDs is part of the graph) on an internal stream; nothing
 * runs during capture.  fs_graph_launch replays it on `stream`.  A graph holds no memset node.
 * Replays of graphs that share a context must be ordered on one stream.  On this hardware the
 * replay of a multi-stream graph costs the host more than the eager calls do; the eager
 * pipelined call is the faster way to drive the step. */
typedef struct fs_graph fs_graph;
int fs_graph_capture_pipelined(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next, fs_graph **out);
int fs_graph_launch(fs_ctx *ctx, fs_graph *graph, fs_stream stream);
int fs_graph_destroy(fs_graph *graph);

/* Library version as major*10000 + minor*100 + patch. */
int fs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FREESCALE_H */
