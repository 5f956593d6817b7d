// Internal declarations shared by the HIP translation units of libfreescale_hip.so.
// gfx950 only: 64-wide wavefronts, 16 bytes per lane per memory instruction.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "freescale_aux.h"

namespace fs {

constexpr int kWave = 64;

// radix sort geometry
#ifndef FS_RADIX_BITS
#define FS_RADIX_BITS 9
#endif
constexpr int kRadixBits = FS_RADIX_BITS;                 // most bits one pass may sort (11 would sort 22-bit row IDs in
                                                          // two passes, but every scatter workgroup then scans a
                                                          // [tile][2048] table and lives four times as long beside the
                                                          // class passes: measured slower, 105.2 against 103.0 us per step)
constexpr int kRadix = 1 << kRadixBits;                   // most bins of one pass
#ifndef FS_SORT_THREADS
#define FS_SORT_THREADS 1024
#endif
constexpr int kSortThreads = FS_SORT_THREADS;
constexpr int kSortTile = 4096;                           // keys per tile
constexpr int kSortKpt = kSortTile / kSortThreads;        // keys per thread
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kSortScan = kSortThreads > kRadix ? kSortThreads : kRadix;

// unique / split compaction geometry
constexpr int kScanThreads = 256;
constexpr int kScanIpt = 4;
constexpr int kScanTile = kScanThreads * kScanIpt;

// segment reduce: sorted positions owned by one wavefront (one 64-bit tail mask, one permutation
// entry per lane).  Short chunks = many wavefronts with short dependent-load chains.
constexpr int kReduceChunk = 64;
constexpr int kReduceWavesPerBlock = 4;
constexpr int kShortRecInts = 12;                         // row (2), slot, occurrences, occurrence list (FS_SHORT_SEGMENT)
static_assert(FS_SHORT_SEGMENT == 8, "record layout");
constexpr int kFusedMinChunk = 16;                        // smallest chunk the fused pass may be built with

// device-side error flag bits (ctx->d_flags[0])
constexpr int kFlagRowRange = 1;
constexpr int kFlagOffsets = 2;
constexpr int kFlagInternal = 4;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

}  // namespace fs

// scratch of one dedup (radix sort + compaction); one set per stream that may run a dedup
struct fs_sort_scratch {
    uint64_t *keys[2];        // [max_ids] each (also used as uint32 keys)
    int32_t *idx[2];          // [max_ids] each
    uint32_t *tile_hist;      // [tiles * bins] per-tile digit counts
    int32_t *tile_heads;      // [scan tiles] heads per compaction tile
};
#ifndef FS_INDEX_STREAMS
#define FS_INDEX_STREAMS 2
#endif
constexpr int kIndexStreams = FS_INDEX_STREAMS;   // streams that run ahead-of-time index work, used in turn
constexpr int kMaxBatch = FS_MAX_AHEAD_BATCH;     // index halves that may share their launches (freescale.h)
// scratch sets: 0 for the caller's stream / side stream, then kMaxBatch per index stream
constexpr int kSortSets = 1 + kIndexStreams * kMaxBatch;

// scratch between the launches of one split + class order (same stream); one set per stream that may run one
struct fs_split_scratch {
    uint8_t *flag_t;          // [max_ids] membership flags of U_t
    uint8_t *flag_t1;         // [max_ids] membership flags of U_t1
    int32_t *cnt;             // [2 * scan tiles] collisions per tile
    int32_t *cstart_local;    // [max_ids] occurrences of same-class rows before this row inside its split tile
    int32_t *tile_len;        // [2 * scan tiles] occurrences per split tile: collision rows, then exclusive rows
    int32_t *cidx;            // [max_ids] place of every row of U_t in its class list
};

// one dedup / one collision split / one class order of a batch that shares its launches (host side)
struct fs_unique_job {
    const int64_t *ids;
    int64_t n, num_rows;
    int64_t *unique;
    int32_t *seg_offsets, *perm, *inverse;
    int64_t *n_unique_dev;
    int64_t *sorted_ids = nullptr;  // optional [n]: all IDs in ascending order
};
struct fs_split_job {
    const int64_t *u_t, *n_t_dev, *u_t1, *n_t1_dev;
    int64_t cap_t, cap_t1;
    int64_t *co;
    int32_t *co_slot;
    int64_t *ex;
    int32_t *ex_slot;
    int64_t *ex_next;
    int32_t *ex_next_slot;
    int64_t *counts_dev;
    const int32_t *seg_offsets_t;   // optional; given, the per-tile occurrence counts the class order needs are left in the scratch
    uint8_t *flag_t1_out = nullptr; // optional [cap_t1]: 1 where the row of u_t1 is also in u_t (a collision row), else 0
};
struct fs_class_job {
    const int32_t *perm;
    const int64_t *n_unique_dev;    // rows of the batch (bounds seg_offsets)
    const int32_t *seg_offsets;
    int64_t n, cap_u;
    int32_t *cperm, *cslot, *cstart, *class_pos_dev;
    const int64_t *u_t;
    int32_t *short_rec;
};

// one class pass / one gather of a launch shared by several tables (host side)
struct fs_class_pass_job {
    const float *grads;
    int64_t n;
    int32_t dim;
    const int32_t *cperm, *cslot, *class_pos, *seg_offsets, *cstart;
    const int64_t *u_t;
    void *table;
    int dt;
    float *state;
    int64_t num_rows;
    float lr, eps;
    float *reduced;
    const int32_t *short_rec;       // the records of the class
    const int64_t *n_rows_dev;      // the number of rows of the class
};
struct fs_gather_job {
    const void *table;
    int64_t num_rows;
    int row_bytes;
    const int64_t *values, *offsets;
    int64_t batch, n;
    void *out;
    // one part of the two-part lookup (optional): only the occurrences j with (row_flag[inverse[j]] != 0) ==
    // (which != 0) are copied; which < 0 or a null pointer: every occurrence
    const int32_t *inverse = nullptr;
    const uint8_t *row_flag = nullptr;
    int which = -1;
    // row order (optional, whole lookups only): position p of the ascending list holds row sorted_ids[p], whose
    // occurrence is perm[p]
    const int64_t *sorted_ids = nullptr;
    const int32_t *perm = nullptr;
};

struct fs_ctx {
    int device;
    int64_t max_ids;
    int32_t max_dim;
    char err[512];

    // one slab of device workspace, carved into the pointers below
    void *slab;
    size_t slab_bytes;

    int *d_flags;             // [4] device error flags
    fs_sort_scratch sort[kSortSets];
    fs_split_scratch split[kSortSets];
    // segment reduce
    double *part_head;        // [chunks, max_dim] fp64 partial of the first run of each chunk
    double *part_last;        // [chunks, max_dim] fp64 partial of the last run of each chunk
    int32_t *chunk_desc;      // [chunks * 4]
    // fused reduce+update, one set per class (0 = collision rows, 1 = exclusive rows) so that the
    // priority pass of one iteration and the deferred pass of another may run side by side
    double *fpart_head[2];    // [chunks, max_dim] piece of a cut segment that came in from the previous chunk
    double *fpart_last[2];    // [chunks, max_dim] first piece of a cut segment that continues into the next chunk
    int *fcounters[2];        // [chunks] arrivals per cut segment (indexed by its first chunk); at 0 between launches
    int *fcounters_sup[2];    // [chunks] arrivals per group of sixteen pieces (indexed by its first chunk)
    const int32_t *reduce_inverse;   // host-side: the caller's optional inverse map for the launch being enqueued
    int64_t *d_zero;          // device scalar that stays 0 (stands in for a missing lookahead)
    // partitioner and jagged shuffles
    int64_t *jag_unique;      // [max_ids] by-products of sorting the lengths (distinct lengths, their extents, count)
    int32_t *jag_seg;         // [max_ids + 1]
    int64_t *jag_n;           // [1]
    int32_t *jag_sorted;      // [max_ids] samples in ascending order of length
    int64_t *jag_tile_sum;    // [scan tiles] output elements per tile of output samples
    int32_t *jag_sel;         // [max_ids] computed segment order of a keyed shuffle

    hipStream_t stream_a;     // side stream: index half of the lookahead batch; deferred pass of a pipelined call
    hipStream_t stream_b;     // deferred pass of the self-contained step
    hipStream_t stream_x[kIndexStreams];   // ahead-of-time dedups and index halves, used in turn
    hipEvent_t ev_fork, ev_split, ev_ex;   // self-contained step and fs_step_forward
    hipEvent_t ev_pfork[2];   // position of the caller's stream at the start of a pipelined call (alternating)
    hipEvent_t ev_side[2];    // side-stream work of a pipelined call (deferred pass of cur, index half of next) done
    int pipe_parity;          // event set used by the last pipelined call
    bool pfork_valid;         // host-side: ev_pfork[pipe_parity] has been recorded
    bool side_pending;        // host-side: side-stream work is in flight and not yet joined
    // two-part lookup: the lookahead batches whose exclusive rows the last pipelined call fetched on the side
    // stream (output buffer, IDs, count), per table; forgotten whenever anything else touches the context
    const void *fetched_emb[FS_MAX_STEP_TABLES];
    const void *fetched_values[FS_MAX_STEP_TABLES];
    int64_t fetched_n[FS_MAX_STEP_TABLES];
    double host_us[7];        // host-side time spent in the phases of the pipelined call (measurement aid)
    struct fs_host *host;     // host threads and the table of outstanding ahead-of-time dedups
    bool use_worker;
    hipStream_t stream_cap;   // capture stream of fs_graph_capture_pipelined
    bool capturing;           // host-side: a step is being recorded into a graph (no timing events)
    int timing_slots;
    int timing_every;         // bracket the kernels of one step in `timing_every`
    bool timing_now;          // host-side: the step being enqueued is a sampled one
    int64_t step_counter;
    int64_t timing_steps;
    hipEvent_t *timing_events;
};

namespace fs {

inline int set_err(fs_ctx *ctx, int code, const char *msg) {
    if (ctx) snprintf(ctx->err, sizeof(ctx->err), "%s", msg);
    return code;
}

// error text of the calls that take no context (kept per calling thread; fs_last_error(NULL) returns it)
char *static_err_buf();
int set_static_err(int code, const char *msg);
// looks up this GPU's copy of the fixed scratch array of fs_collision_split_static (`device` must be current)
int static_split_prepare(int device);

inline int hip_err(fs_ctx *ctx, hipError_t e, const char *what) {
    if (ctx) snprintf(ctx->err, sizeof(ctx->err), "%s: %s", what, hipGetErrorString(e));
    return FS_EHIP;
}

#define FS_HIP(ctx, call)                                        \
    do {                                                         \
        hipError_t e__ = (call);                                 \
        if (e__ != hipSuccess) return fs::hip_err(ctx, e__, #call); \
    } while (0)

#define FS_LAUNCH_CHECK(ctx, name)                               \
    do {                                                         \
        hipError_t e__ = hipGetLastError();                      \
        if (e__ != hipSuccess) return fs::hip_err(ctx, e__, name); \
    } while (0)

inline bool dim_ok(int32_t dim, int dt) {
    if (dim <= 0 || dim > FS_MAX_DIM) return false;
    return dt == FS_F32 ? (dim % 4 == 0) : (dim % 8 == 0);
}

// lanes that cover one row of `granules` 16-byte pieces: next power of two, at most 64
inline int lanes_per_row(int granules) {
    int l = 1;
    while (l < granules) l <<= 1;
    return l;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// launchers implemented in the kernel translation units (host side, argument-checked callers)
int launch_gather(fs_ctx *, const void *table, int64_t num_rows, int row_bytes, const int64_t *values,
                  const int64_t *offsets, int64_t batch, int64_t n, void *out, hipStream_t s);
int launch_partition_fbs(fs_ctx *, const int64_t *lengths, int64_t B, int64_t max_len, int32_t n_ranks,
                         int32_t *sample_of, int64_t *rank_offsets, hipStream_t s);
int launch_partition_vbs(fs_ctx *, const int64_t *lengths, int64_t B, const int64_t *weight_of_len, int64_t max_len,
                         int32_t n_ranks, int32_t *sample_of, int64_t *rank_offsets, hipStream_t s);
int launch_indexed_permute(fs_ctx *, const void *values, int64_t n_values, int32_t elem_bytes, const int64_t *offsets,
                           int64_t B, const int32_t *sample_of, int64_t n_out, void *out_values, int64_t cap_out,
                           int64_t *out_offsets, hipStream_t s);
// mode 0 keyed transpose, 1 ranged dispatch, 2 ranged combine (rank_offsets / splits unused by the transpose)
int launch_keyed_shuffle(fs_ctx *, int mode, const void *values, int64_t n_values, int32_t elem_bytes,
                         const int64_t *offsets, int64_t F, int64_t B, const int64_t *rank_offsets, int32_t n_ranks,
                         void *out_values, int64_t *out_offsets, int64_t *splits, hipStream_t s);
// event pair of timing kind `kind` for the step being enqueued, or nullptr when timing is off
inline hipEvent_t *timing_pair(fs_ctx *ctx, int kind) {
    if (!ctx->timing_now) return nullptr;
    const int slot = (int)(ctx->timing_steps % ctx->timing_slots);
    return ctx->timing_events + ((size_t)kind * ctx->timing_slots + slot) * 2;
}
int launch_unique(fs_ctx *, const int64_t *ids, int64_t n, int64_t num_rows, int64_t *unique,
                  int32_t *seg_offsets, int32_t *perm, int32_t *inverse, int64_t *n_unique_dev, hipStream_t s,
                  int set = 0);
// `count` (1..kMaxBatch) independent jobs in shared launches; job k uses scratch set set0 + k
int launch_unique_batch(fs_ctx *, int count, const fs_unique_job *jobs, hipStream_t s, int set0);
int launch_split_batch(fs_ctx *, int count, const fs_split_job *jobs, hipStream_t s, int set0);
// right after launch_split_batch(..., seg_offsets_t given) with the same jobs order and sets, on the same stream
int launch_class_order_batch(fs_ctx *, int count, const fs_class_job *jobs, hipStream_t s, int set0);
// seg_offsets_t: optional; given, the per-tile occurrence counts that launch_class_order needs are left in
// the context scratch
int launch_split(fs_ctx *, const int64_t *u_t, const int64_t *n_t_dev, const int64_t *u_t1,
                 const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1, int64_t *co, int32_t *co_slot,
                 int64_t *ex, int32_t *ex_slot, int64_t *ex_next, int32_t *ex_next_slot, int64_t *counts_dev,
                 hipStream_t s, const int32_t *seg_offsets_t = nullptr, int set = 0);
// right after launch_split(..., seg_offsets_t) on the same stream: occurrences of the batch in class order
int launch_class_order(fs_ctx *, const int32_t *perm, const int64_t *n_unique_dev, const int32_t *seg_offsets, int64_t n,
                       int64_t cap_u, int32_t *cperm, int32_t *cslot, int32_t *cstart, int32_t *class_pos_dev,
                       const int64_t *u_t, int32_t *short_rec, hipStream_t s, int set = 0);
int launch_reduce_update(fs_ctx *, int cls, const float *grads, int64_t n, int32_t dim, const int32_t *cperm,
                         const int32_t *cslot, const int32_t *class_pos, const int32_t *seg_offsets,
                         const int32_t *cstart, const int64_t *u_t, void *table, int dt, float *state,
                         int64_t num_rows, float lr, float eps, float *reduced, hipStream_t s,
                         const int32_t *short_rec, const int64_t *n_rows_dev);
// the class passes (class `cls`) / the gathers of `count` tables: tables of one dtype and row width share launches
int launch_reduce_update_batch(fs_ctx *, int cls, int count, const fs_class_pass_job *jobs, hipStream_t s);
int launch_gather_batch(fs_ctx *, int count, const fs_gather_job *jobs, hipStream_t s);
// `timing`: optional event pair recorded around the main (chunk) kernel only
int launch_reduce(fs_ctx *, const float *grads, int64_t n, int32_t dim, const int32_t *perm,
                  const int32_t *seg_offsets, const int64_t *n_unique_dev, float *reduced, hipStream_t s,
                  hipEvent_t *timing = nullptr);
int launch_adagrad(fs_ctx *, void *table, int dt, float *state, int64_t num_rows, int32_t dim,
                   const int64_t *rows, const int32_t *slots, const int64_t *n_rows_dev, int64_t cap,
                   const float *reduced, float lr, float eps, hipStream_t s);
int launch_split_grads(fs_ctx *, const float *grads, int64_t n, int32_t dim, const int32_t *inverse,
                       const int32_t *co_slot, const int64_t *n_co_dev, int64_t cap_u, int32_t *co_index, float *g_co,
                       int32_t *ex_index, float *g_ex, int32_t *part_pos, int64_t *counts_dev, hipStream_t s);
int launch_class_order_for_parts(fs_ctx *, const int32_t *part_pos, int64_t n, int64_t cap_u, const int32_t *cperm,
                                 const int32_t *class_pos_dev, const int32_t *short_rec, const int64_t *counts_dev,
                                 int32_t *cperm_parts, int32_t *short_rec_parts, hipStream_t s);
int launch_init_hash(fs_ctx *, void *table, int64_t num_rows, int32_t dim, int dt, hipStream_t s);
int launch_copy(fs_ctx *, const void *src, void *dst, int64_t n_bytes, hipStream_t s);
int launch_row_read(fs_ctx *, const void *rows, int64_t num_rows, int row_bytes, const int64_t *index, int64_t n,
                    uint32_t *sink, hipStream_t s);

}  // namespace fs
