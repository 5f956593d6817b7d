// C-ABI entry points: argument validation, context/workspace management and the two-stream
// schedule of one prioritized iteration (Section 3.2 / Algorithm 2 of the paper, collectives
// removed).  No kernel lives here.
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <new>
#include <thread>

#include "fs_common.h"

using namespace fs;

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Carver {
    char *base;
    size_t off;
    template <typename T>
    T *take(size_t count) {
        off = align_up(off, 256);
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
};

void carve(fs_ctx *c, char *base, size_t *total) {
    Carver cv{base, 0};
    const size_t n = (size_t)c->max_ids;
    const size_t sort_tiles = (size_t)ceil_div(c->max_ids, kSortTile) + 1;
    const size_t scan_tiles = (size_t)ceil_div(c->max_ids, kScanTile) + 2;
    const size_t chunks = (size_t)ceil_div(c->max_ids, kReduceChunk) + 2;
    c->d_flags = cv.take<int>(4);
    c->d_zero = cv.take<int64_t>(1);
    c->keys[0] = cv.take<uint64_t>(n);
    c->keys[1] = cv.take<uint64_t>(n);
    c->idx[0] = cv.take<int32_t>(n);
    c->idx[1] = cv.take<int32_t>(n);
    c->tile_hist = cv.take<uint32_t>(sort_tiles * kRadix);
    c->digit_base = cv.take<uint32_t>(kRadix);
    c->tile_heads = cv.take<int32_t>(scan_tiles);
    c->split_flag_t = cv.take<uint8_t>(n + 16);
    c->split_flag_t1 = cv.take<uint8_t>(n + 16);
    c->split_cnt = cv.take<int32_t>(2 * scan_tiles);
    c->part_head = cv.take<double>(chunks * (size_t)c->max_dim);
    c->part_last = cv.take<double>(chunks * (size_t)c->max_dim);
    c->chunk_desc = cv.take<int32_t>(chunks * 4);
    *total = align_up(cv.off, 256);
}

hipStream_t as_stream(fs_stream s) { return reinterpret_cast<hipStream_t>(s); }

double now_us() {
    return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

void worker_stop(fs_ctx *ctx);
int join_pending_work(fs_ctx *ctx, hipStream_t s);

#define FS_REQUIRE(ctx, cond, msg)                          \
    do {                                                    \
        if (!(cond)) return set_err(ctx, FS_EINVAL, msg);   \
    } while (0)

}  // namespace

extern "C" {

int fs_version(void) { return 100; }

int fs_ctx_create(fs_ctx **out, int device, int64_t max_ids, int32_t max_dim) {
    if (!out) return FS_EINVAL;
    *out = nullptr;
    if (device < 0 || max_ids < 1 || max_ids > (1ll << 30) || max_dim < 4 || max_dim > FS_MAX_DIM) return FS_EINVAL;
    fs_ctx *c = new (std::nothrow) fs_ctx();
    if (!c) return FS_ENOMEM;
    memset(c, 0, sizeof(*c));
    c->device = device;
    c->max_ids = max_ids;
    c->max_dim = max_dim;
    c->use_worker = true;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) {
        delete c;
        return FS_EHIP;
    }
    if (hipSetDevice(device) != hipSuccess) {
        delete c;
        return FS_EHIP;
    }
    carve(c, nullptr, &c->slab_bytes);
    if (hipMalloc(&c->slab, c->slab_bytes) != hipSuccess) {
        (void)hipGetLastError();
        delete c;
        return FS_ENOMEM;
    }
    size_t total;
    carve(c, static_cast<char *>(c->slab), &total);
    bool ok = hipMemset(c->slab, 0, 4096) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&c->stream_a, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&c->stream_b, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&c->stream_cap, hipStreamNonBlocking) == hipSuccess;
    hipEvent_t *evs[] = {&c->ev_fork, &c->ev_split, &c->ev_reduce, &c->ev_co, &c->ev_ex, &c->ev_idx[0], &c->ev_idx[1],
                         &c->ev_red[0], &c->ev_red[1], &c->ev_side[0], &c->ev_side[1]};
    for (hipEvent_t *e : evs) ok = ok && hipEventCreateWithFlags(e, hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        fs_ctx_destroy(c);
        return FS_EHIP;
    }
    *out = c;
    return FS_OK;
}

int fs_ctx_destroy(fs_ctx *c) {
    if (!c) return FS_OK;
    (void)hipSetDevice(c->device);
    worker_stop(c);
    if (c->stream_a) { (void)hipStreamSynchronize(c->stream_a); (void)hipStreamDestroy(c->stream_a); }
    if (c->stream_b) { (void)hipStreamSynchronize(c->stream_b); (void)hipStreamDestroy(c->stream_b); }
    if (c->stream_cap) (void)hipStreamDestroy(c->stream_cap);
    hipEvent_t evs[] = {c->ev_fork, c->ev_split, c->ev_reduce, c->ev_co, c->ev_ex, c->ev_idx[0], c->ev_idx[1],
                        c->ev_red[0], c->ev_red[1], c->ev_side[0], c->ev_side[1]};
    for (hipEvent_t e : evs)
        if (e) (void)hipEventDestroy(e);
    (void)fs_ctx_set_kernel_timing(c, 0, 1);
    if (c->slab) (void)hipFree(c->slab);
    delete c;
    return FS_OK;
}

const char *fs_last_error(const fs_ctx *ctx) { return ctx ? ctx->err : "null context"; }

size_t fs_ctx_workspace_bytes(const fs_ctx *ctx) { return ctx ? ctx->slab_bytes : 0; }

int fs_check_async(fs_ctx *ctx, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    const int jrc = join_pending_work(ctx, as_stream(stream));
    if (jrc != FS_OK) return jrc;
    FS_HIP(ctx, hipStreamSynchronize(as_stream(stream)));
    FS_HIP(ctx, hipStreamSynchronize(ctx->stream_a));
    FS_HIP(ctx, hipStreamSynchronize(ctx->stream_b));
    int flags[4] = {0, 0, 0, 0};
    FS_HIP(ctx, hipMemcpy(flags, ctx->d_flags, sizeof(flags), hipMemcpyDeviceToHost));
    if (flags[0] == 0) return FS_OK;
    FS_HIP(ctx, hipMemset(ctx->d_flags, 0, sizeof(flags)));
    snprintf(ctx->err, sizeof(ctx->err), "device flags 0x%x:%s%s%s", flags[0],
             (flags[0] & kFlagRowRange) ? " row id out of range" : "",
             (flags[0] & kFlagOffsets) ? " malformed offsets" : "", (flags[0] & kFlagInternal) ? " internal" : "");
    return FS_ERANGE;
}

int fs_ctx_set_kernel_timing(fs_ctx *ctx, int slots, int every) {
    if (!ctx || slots < 0 || slots > 65536 || every < 1) return FS_EINVAL;
    if (ctx->timing_events) {
        const size_t cnt = (size_t)FS_TIME_KINDS * ctx->timing_slots * 2;
        for (size_t i = 0; i < cnt; ++i)
            if (ctx->timing_events[i]) (void)hipEventDestroy(ctx->timing_events[i]);
        delete[] ctx->timing_events;
        ctx->timing_events = nullptr;
    }
    ctx->timing_slots = 0;
    ctx->timing_steps = 0;
    ctx->step_counter = 0;
    ctx->timing_every = every;
    ctx->timing_now = false;
    if (slots == 0) return FS_OK;
    const size_t cnt = (size_t)FS_TIME_KINDS * slots * 2;
    ctx->timing_events = new (std::nothrow) hipEvent_t[cnt]();
    if (!ctx->timing_events) return FS_ENOMEM;
    ctx->timing_slots = slots;
    for (size_t i = 0; i < cnt; ++i) FS_HIP(ctx, hipEventCreate(&ctx->timing_events[i]));
    return FS_OK;
}

int fs_ctx_get_kernel_timing(fs_ctx *ctx, int which, float *ms_out_host, int max_out, int *n_out_host) {
    if (!ctx || which < 0 || which >= FS_TIME_KINDS || !ms_out_host || !n_out_host || max_out < 0) return FS_EINVAL;
    *n_out_host = 0;
    if (ctx->timing_slots <= 0) return FS_OK;
    FS_HIP(ctx, hipDeviceSynchronize());
    const int64_t have = ctx->timing_steps < ctx->timing_slots ? ctx->timing_steps : ctx->timing_slots;
    const int64_t first = ctx->timing_steps - have;
    int n = 0;
    for (int64_t i = 0; i < have && n < max_out; ++i) {
        const int slot = (int)((first + i) % ctx->timing_slots);
        hipEvent_t *pair = ctx->timing_events + ((size_t)which * ctx->timing_slots + slot) * 2;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, pair[0], pair[1]) != hipSuccess) {
            (void)hipGetLastError();
            continue;                     // this kernel was not launched in that step
        }
        ms_out_host[n++] = ms;
    }
    *n_out_host = n;
    return FS_OK;
}

int fs_gather_jagged(fs_ctx *ctx, const void *table, int64_t num_rows, int32_t dim, fs_dtype dt,
                     const int64_t *values, const int64_t *offsets, int64_t batch, int64_t n_values, void *out,
                     fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, dt == FS_F32 || dt == FS_BF16, "gather: unknown dtype");
    FS_REQUIRE(ctx, dim_ok(dim, dt), "gather: dim must be a multiple of 4 (fp32) / 8 (bf16), at most FS_MAX_DIM");
    FS_REQUIRE(ctx, num_rows >= 0 && batch >= 0 && n_values >= 0, "gather: negative size");
    FS_REQUIRE(ctx, n_values <= (1ll << 31) - 1, "gather: more than 2^31-1 values");
    if (n_values == 0) return FS_OK;
    FS_REQUIRE(ctx, table && values && out, "gather: null pointer");
    const int row_bytes = dim * (dt == FS_F32 ? 4 : 2);
    return launch_gather(ctx, table, num_rows, row_bytes, values, offsets, batch, n_values, out, as_stream(stream));
}

int fs_unique_ids(fs_ctx *ctx, const int64_t *ids, int64_t n, int64_t num_rows, int64_t *unique,
                  int32_t *seg_offsets, int32_t *perm, int32_t *inverse, int64_t *n_unique_dev, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, n >= 0 && num_rows >= 0, "unique: negative size");
    if (n > ctx->max_ids) return set_err(ctx, FS_ENOMEM, "unique: n beyond the context capacity");
    FS_REQUIRE(ctx, seg_offsets && n_unique_dev, "unique: null pointer");
    if (n > 0) FS_REQUIRE(ctx, ids && unique && perm, "unique: null pointer");
    const int jrc = join_pending_work(ctx, as_stream(stream));      // the workspace may still be in use on A
    if (jrc != FS_OK) return jrc;
    return launch_unique(ctx, ids, n, num_rows, unique, seg_offsets, perm, inverse, n_unique_dev, as_stream(stream));
}

int fs_collision_split(fs_ctx *ctx, const int64_t *u_t, const int64_t *n_t_dev, const int64_t *u_t1,
                       const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1, int64_t *co, int32_t *co_slot,
                       int64_t *ex, int32_t *ex_slot, int64_t *ex_next, int32_t *ex_next_slot, int64_t *counts_dev,
                       fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, cap_t >= 0 && cap_t1 >= 0, "split: negative capacity");
    if (cap_t > ctx->max_ids || cap_t1 > ctx->max_ids)
        return set_err(ctx, FS_ENOMEM, "split: capacity beyond the context capacity");
    FS_REQUIRE(ctx, counts_dev, "split: null counts");
    if (cap_t > 0) FS_REQUIRE(ctx, u_t && n_t_dev && co && co_slot && ex && ex_slot, "split: null pointer (t side)");
    if (cap_t1 > 0) FS_REQUIRE(ctx, u_t1 && n_t1_dev && ex_next && ex_next_slot, "split: null pointer (t+1 side)");
    const int jrc = join_pending_work(ctx, as_stream(stream));      // the workspace may still be in use on A
    if (jrc != FS_OK) return jrc;
    return launch_split(ctx, u_t, cap_t > 0 ? n_t_dev : nullptr, u_t1, cap_t1 > 0 ? n_t1_dev : nullptr, cap_t, cap_t1,
                        co, co_slot, ex, ex_slot, ex_next, ex_next_slot, counts_dev, as_stream(stream));
}

int fs_segment_reduce_grads(fs_ctx *ctx, const float *grads, int64_t n, int32_t dim, const int32_t *perm,
                            const int32_t *seg_offsets, const int32_t *inverse, const int64_t *n_unique_dev,
                            float *reduced, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, n >= 0, "reduce: negative size");
    FS_REQUIRE(ctx, dim_ok(dim, FS_F32), "reduce: dim must be a multiple of 4, at most FS_MAX_DIM");
    if (n > ctx->max_ids || dim > ctx->max_dim) return set_err(ctx, FS_ENOMEM, "reduce: beyond the context capacity");
    if (n == 0) return FS_OK;
    FS_REQUIRE(ctx, grads && perm && seg_offsets && n_unique_dev && reduced, "reduce: null pointer");
    ctx->reduce_inverse = inverse;
    const int rc = launch_reduce(ctx, grads, n, dim, perm, seg_offsets, n_unique_dev, reduced, as_stream(stream));
    ctx->reduce_inverse = nullptr;
    return rc;
}

int fs_rowwise_adagrad_update(fs_ctx *ctx, void *table, fs_dtype dt, float *state, int64_t num_rows, int32_t dim,
                              const int64_t *rows, const int32_t *slots, const int64_t *n_rows_dev, int64_t cap,
                              const float *reduced, float lr, float eps, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, dt == FS_F32 || dt == FS_BF16, "adagrad: unknown dtype");
    FS_REQUIRE(ctx, dim_ok(dim, dt), "adagrad: dim must be a multiple of 4 (fp32) / 8 (bf16), at most FS_MAX_DIM");
    FS_REQUIRE(ctx, num_rows >= 0 && cap >= 0, "adagrad: negative size");
    if (cap == 0) return FS_OK;
    FS_REQUIRE(ctx, table && state && rows && slots && n_rows_dev && reduced, "adagrad: null pointer");
    return launch_adagrad(ctx, table, dt, state, num_rows, dim, rows, slots, n_rows_dev, cap, reduced, lr, eps,
                          as_stream(stream));
}

int fs_init_table_hash(fs_ctx *ctx, void *table, int64_t num_rows, int32_t dim, fs_dtype dt, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, dt == FS_F32 || dt == FS_BF16, "init: unknown dtype");
    FS_REQUIRE(ctx, dim_ok(dim, dt) && num_rows >= 0, "init: bad shape");
    if (num_rows == 0) return FS_OK;
    FS_REQUIRE(ctx, table, "init: null pointer");
    return launch_init_hash(ctx, table, num_rows, dim, dt, as_stream(stream));
}

int fs_stream_copy(fs_ctx *ctx, const void *src, void *dst, int64_t n_bytes, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, n_bytes >= 0 && n_bytes % 16 == 0, "copy: size must be a non-negative multiple of 16");
    if (n_bytes == 0) return FS_OK;
    FS_REQUIRE(ctx, src && dst, "copy: null pointer");
    return launch_copy(ctx, src, dst, n_bytes, as_stream(stream));
}

}  // extern "C"

namespace {

// host-visible checks shared by the step entry points; `need_t`: iteration t is used (reduce,
// updates), `need_t1`: the lookahead batch is used (dedup, gather)
int check_step_args(fs_ctx *ctx, const fs_step_args *a, bool *have_t, bool *have_t1) {
    FS_REQUIRE(ctx, a, "step: null args");
    const int dt = a->dtype;
    FS_REQUIRE(ctx, dt == FS_F32 || dt == FS_BF16, "step: unknown dtype");
    FS_REQUIRE(ctx, dim_ok(a->dim, dt), "step: unsupported dim");
    FS_REQUIRE(ctx, a->num_rows >= 0 && a->n_t >= 0 && a->n_t1 >= 0 && a->batch_t1 >= 0, "step: negative size");
    if (a->n_t > ctx->max_ids || a->n_t1 > ctx->max_ids || a->dim > ctx->max_dim)
        return set_err(ctx, FS_ENOMEM, "step: beyond the context capacity");
    FS_REQUIRE(ctx, a->table && a->state && a->counts_dev, "step: null table/state/counts");
    *have_t = a->n_t > 0;
    *have_t1 = a->values_t1 != nullptr && a->n_t1 > 0;
    if (*have_t)
        FS_REQUIRE(ctx, a->u_t && a->seg_offsets_t && a->perm_t && a->n_unique_t_dev && a->grads_t && a->reduced &&
                            a->co && a->co_slot && a->ex && a->ex_slot,
                   "step: null pointer (iteration t)");
    if (*have_t1)
        FS_REQUIRE(ctx, a->u_t1 && a->seg_offsets_t1 && a->perm_t1 && a->n_unique_t1_dev && a->ex_next &&
                            a->ex_next_slot && a->emb_t1,
                   "step: null pointer (lookahead)");
    return FS_OK;
}

// Forward of Algorithm 2 (index work): dedup of the lookahead IDs, then the collision split
int enqueue_index_work(fs_ctx *ctx, const fs_step_args *a, bool have_t, bool have_t1, hipStream_t s) {
    int rc;
    if (have_t1) {
        rc = launch_unique(ctx, a->values_t1, a->n_t1, a->num_rows, a->u_t1, a->seg_offsets_t1, a->perm_t1,
                           a->inverse_t1, a->n_unique_t1_dev, s);
        if (rc != FS_OK) return rc;
    }
    return launch_split(ctx, a->u_t, have_t ? a->n_unique_t_dev : nullptr, a->u_t1,
                        have_t1 ? a->n_unique_t1_dev : nullptr, have_t ? a->n_t : 0, have_t1 ? a->n_t1 : 0, a->co,
                        a->co_slot, a->ex, a->ex_slot, a->ex_next, a->ex_next_slot, a->counts_dev, s);
}

// one step in `timing_every` gets its kernels bracketed by event pairs (an event record costs the
// host more than a kernel launch, so bracketing every step would slow the very thing it measures)
void begin_step_timing(fs_ctx *ctx) {
    ctx->timing_now = ctx->timing_slots > 0 && !ctx->capturing && (ctx->step_counter % ctx->timing_every) == 0;
    if (ctx->timing_slots > 0 && !ctx->capturing) ++ctx->step_counter;
}

int enqueue_reduce(fs_ctx *ctx, const fs_step_args *a, hipStream_t sp) {
    ctx->reduce_inverse = a->inverse_t;
    const int rc = launch_reduce(ctx, a->grads_t, a->n_t, a->dim, a->perm_t, a->seg_offsets_t, a->n_unique_t_dev,
                                 a->reduced, sp, timing_pair(ctx, FS_TIME_REDUCE));
    ctx->reduce_inverse = nullptr;
    return rc;
}

// Backward of Algorithm 2 after the reduce: priority pass on `sp`, deferred pass on B (which
// already waits for the reduce and the split), gather of the lookahead rows on `sp`, join of B.
// ex_done == nullptr: B is joined into `sp` at the end; otherwise the deferred pass records it
// and the caller decides who waits for it.
int enqueue_updates_and_gather(fs_ctx *ctx, const fs_step_args *a, bool have_t, bool have_t1, hipStream_t sp,
                               hipEvent_t ex_done = nullptr) {
    hipStream_t sb = ctx->stream_b;
    const fs_dtype fdt = (fs_dtype)a->dtype;
    int rc;
    if (have_t) {
        // priority pass: collision rows, strictly before the lookahead rows are read
        hipEvent_t *tco = timing_pair(ctx, FS_TIME_UPDATE_CO), *tex = timing_pair(ctx, FS_TIME_UPDATE_EX);
        if (tco) (void)hipEventRecord(tco[0], sp);
        rc = launch_adagrad(ctx, a->table, fdt, a->state, a->num_rows, a->dim, a->co, a->co_slot, a->counts_dev + 0,
                            a->n_t, a->reduced, a->lr, a->eps, sp);
        if (rc != FS_OK) return rc;
        if (tco) (void)hipEventRecord(tco[1], sp);
        if (tex) (void)hipEventRecord(tex[0], sb);
        rc = launch_adagrad(ctx, a->table, fdt, a->state, a->num_rows, a->dim, a->ex, a->ex_slot, a->counts_dev + 1,
                            a->n_t, a->reduced, a->lr, a->eps, sb);
        if (rc != FS_OK) return rc;
        if (tex) (void)hipEventRecord(tex[1], sb);
    }
    FS_HIP(ctx, hipEventRecord(ex_done ? ex_done : ctx->ev_ex, sb));
    if (have_t1) {
        // exclusive rows and lookahead rows are disjoint, so this may overlap the deferred pass
        const int row_bytes = a->dim * (a->dtype == FS_F32 ? 4 : 2);
        hipEvent_t *tg = timing_pair(ctx, FS_TIME_GATHER);
        if (tg) (void)hipEventRecord(tg[0], sp);
        rc = launch_gather(ctx, a->table, a->num_rows, row_bytes, a->values_t1, a->offsets_t1, a->batch_t1, a->n_t1,
                           a->emb_t1, sp);
        if (rc != FS_OK) return rc;
        if (tg) (void)hipEventRecord(tg[1], sp);
    }
    if (!ex_done) FS_HIP(ctx, hipStreamWaitEvent(sp, ctx->ev_ex, 0));
    if (ctx->timing_now) ++ctx->timing_steps;
    return FS_OK;
}

// pipelined form: priority pass and gather on `sp` (the deferred pass goes to the side stream)
int enqueue_priority_and_gather(fs_ctx *ctx, const fs_step_args *a, bool have_t, bool have_t1, hipStream_t sp) {
    int rc;
    if (have_t) {
        hipEvent_t *tco = timing_pair(ctx, FS_TIME_UPDATE_CO);
        if (tco) (void)hipEventRecord(tco[0], sp);
        rc = launch_adagrad(ctx, a->table, (fs_dtype)a->dtype, a->state, a->num_rows, a->dim, a->co, a->co_slot,
                            a->counts_dev + 0, a->n_t, a->reduced, a->lr, a->eps, sp);
        if (rc != FS_OK) return rc;
        if (tco) (void)hipEventRecord(tco[1], sp);
    }
    if (have_t1) {
        const int row_bytes = a->dim * (a->dtype == FS_F32 ? 4 : 2);
        hipEvent_t *tg = timing_pair(ctx, FS_TIME_GATHER);
        if (tg) (void)hipEventRecord(tg[0], sp);
        rc = launch_gather(ctx, a->table, a->num_rows, row_bytes, a->values_t1, a->offsets_t1, a->batch_t1, a->n_t1,
                           a->emb_t1, sp);
        if (rc != FS_OK) return rc;
        if (tg) (void)hipEventRecord(tg[1], sp);
    }
    return FS_OK;
}

}  // namespace

struct fs_graph {
    hipGraph_t graph;
    hipGraphExec_t exec;
};

// A second host thread that enqueues the index half of an iteration on side stream A while the
// calling thread enqueues the gradient half: an iteration is about sixteen launches and a dozen
// event operations, and at a few microseconds each the host, not the GPU, would set the pace.
struct fs_worker {
    std::thread thread;
    std::mutex mu;
    std::condition_variable cv;
    bool has_job = false, done = true, quit = false;
    // the job: index half of `next` (if has_next), then the deferred pass of `cur` (if has_cur)
    fs_step_args next, cur;
    bool has_next = false, nxt_t = false, nxt_t1 = false, has_cur = false;
    int parity = 0;               // event set of the call that posted the job
    hipEvent_t first_after = nullptr;   // A waits for this before the job's first kernel (may be null)
    std::atomic<bool> red_recorded{false};   // set by the posting thread once ev_red[parity] is recorded
    hipEvent_t *ex_timing = nullptr;
    int rc = FS_OK;
};

namespace {

// Side stream A, in this order: index half of the next iteration (needs nothing of the current
// one), then - once the reduce of the current iteration is done - its deferred pass, then the
// event that the next call waits for before its priority pass.
int enqueue_side_stream(fs_ctx *ctx, const fs_step_args *next, bool nxt_t, bool nxt_t1, const fs_step_args *cur,
                        int parity, hipEvent_t first_after, std::atomic<bool> *red_recorded, hipEvent_t *ex_timing) {
    hipStream_t sa = ctx->stream_a;
    int rc = FS_OK;
    if (first_after) FS_HIP(ctx, hipStreamWaitEvent(sa, first_after, 0));
    if (next) rc = enqueue_index_work(ctx, next, nxt_t, nxt_t1, sa);
    if (rc != FS_OK) return rc;
    if (cur) {
        if (red_recorded)
            while (!red_recorded->load(std::memory_order_acquire)) std::this_thread::yield();
        FS_HIP(ctx, hipStreamWaitEvent(sa, ctx->ev_red[parity], 0));
        if (ex_timing) (void)hipEventRecord(ex_timing[0], sa);
        rc = launch_adagrad(ctx, cur->table, (fs_dtype)cur->dtype, cur->state, cur->num_rows, cur->dim, cur->ex,
                            cur->ex_slot, cur->counts_dev + 1, cur->n_t, cur->reduced, cur->lr, cur->eps, sa);
        if (rc != FS_OK) return rc;
        if (ex_timing) (void)hipEventRecord(ex_timing[1], sa);
    }
    FS_HIP(ctx, hipEventRecord(ctx->ev_side[parity], sa));
    return FS_OK;
}

void worker_main(fs_ctx *ctx) {
    fs_worker *w = ctx->worker;
    (void)hipSetDevice(ctx->device);
    std::unique_lock<std::mutex> lk(w->mu);
    for (;;) {
        w->cv.wait(lk, [w] { return w->has_job || w->quit; });
        if (w->quit) return;
        w->has_job = false;
        lk.unlock();
        const double j0 = now_us();
        const int rc = enqueue_side_stream(ctx, w->has_next ? &w->next : nullptr, w->nxt_t, w->nxt_t1,
                                           w->has_cur ? &w->cur : nullptr, w->parity, w->first_after,
                                           &w->red_recorded, w->ex_timing);
        ctx->host_us[5] += now_us() - j0;                    // the worker's enqueueing
        lk.lock();
        w->rc = rc;
        w->done = true;
        w->cv.notify_all();
    }
}

// hands the side-stream work of one call to the worker (started on first use); false if no worker
bool worker_post(fs_ctx *ctx, const fs_step_args *next, bool nxt_t, bool nxt_t1, const fs_step_args *cur, int parity,
                 hipEvent_t first_after, hipEvent_t *ex_timing) {
    if (!ctx->worker) {
        ctx->worker = new (std::nothrow) fs_worker();
        if (!ctx->worker) return false;
        ctx->worker->thread = std::thread(worker_main, ctx);
    }
    fs_worker *w = ctx->worker;
    std::lock_guard<std::mutex> lk(w->mu);
    w->has_next = next != nullptr;
    if (next) w->next = *next;
    w->nxt_t = nxt_t;
    w->nxt_t1 = nxt_t1;
    w->has_cur = cur != nullptr;
    if (cur) w->cur = *cur;
    w->parity = parity;
    w->first_after = first_after;
    w->ex_timing = ex_timing;
    w->red_recorded.store(false, std::memory_order_relaxed);
    w->has_job = true;
    w->done = false;
    w->cv.notify_all();
    return true;
}

int worker_wait(fs_ctx *ctx) {
    fs_worker *w = ctx->worker;
    if (!w) return FS_OK;
    std::unique_lock<std::mutex> lk(w->mu);
    w->cv.wait(lk, [w] { return w->done; });
    return w->rc;
}

void worker_stop(fs_ctx *ctx) {
    fs_worker *w = ctx->worker;
    if (!w) return;
    {
        std::lock_guard<std::mutex> lk(w->mu);
        w->quit = true;
        w->cv.notify_all();
    }
    if (w->thread.joinable()) w->thread.join();
    delete w;
    ctx->worker = nullptr;
}

// Makes `s` wait for what an earlier pipelined call left running on side stream A: the index half
// of its `next` and the deferred pass of its `cur`.
int join_pending_work(fs_ctx *ctx, hipStream_t s) {
    int wrc = FS_OK;
    if (ctx->side_pending) {
        wrc = worker_wait(ctx);                              // its enqueueing (and event record) is complete
        ctx->side_pending = false;
        FS_HIP(ctx, hipStreamWaitEvent(s, ctx->ev_side[ctx->pipe_parity], 0));
    }
    ctx->red_valid = false;                                  // the next pipelined call forks from its stream
    return wrc;
}

}  // namespace

extern "C" {

int fs_step_forward(fs_ctx *ctx, const fs_step_args *a, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    bool have_t, have_t1;
    int rc = check_step_args(ctx, a, &have_t, &have_t1);
    if (rc != FS_OK) return rc;
    hipStream_t sp = as_stream(stream), sa = ctx->stream_a;
    rc = join_pending_work(ctx, sp);
    if (rc != FS_OK) return rc;
    FS_HIP(ctx, hipEventRecord(ctx->ev_fork, sp));
    FS_HIP(ctx, hipStreamWaitEvent(sa, ctx->ev_fork, 0));
    rc = enqueue_index_work(ctx, a, have_t, have_t1, sa);
    if (rc != FS_OK) return rc;
    FS_HIP(ctx, hipEventRecord(ctx->ev_split, sa));
    FS_HIP(ctx, hipStreamWaitEvent(sp, ctx->ev_split, 0));
    return FS_OK;
}

int fs_prioritized_step(fs_ctx *ctx, const fs_step_args *a, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    bool have_t, have_t1;
    int rc = check_step_args(ctx, a, &have_t, &have_t1);
    if (rc != FS_OK) return rc;
    hipStream_t sp = as_stream(stream), sa = ctx->stream_a, sb = ctx->stream_b;
    rc = join_pending_work(ctx, sp);
    if (rc != FS_OK) return rc;
    begin_step_timing(ctx);
    // fork: the side streams start after whatever the caller already queued on `stream`
    FS_HIP(ctx, hipEventRecord(ctx->ev_fork, sp));
    FS_HIP(ctx, hipStreamWaitEvent(sa, ctx->ev_fork, 0));
    FS_HIP(ctx, hipStreamWaitEvent(sb, ctx->ev_fork, 0));
    // main stream first (the host enqueues the bandwidth-heavy kernel before the many small ones):
    // reduce the gradients of t while A works on the indices of t+1
    if (have_t) {
        rc = enqueue_reduce(ctx, a, sp);
        if (rc != FS_OK) return rc;
    }
    FS_HIP(ctx, hipEventRecord(ctx->ev_reduce, sp));
    rc = enqueue_index_work(ctx, a, have_t, have_t1, sa);
    if (rc != FS_OK) return rc;
    FS_HIP(ctx, hipEventRecord(ctx->ev_split, sa));
    FS_HIP(ctx, hipStreamWaitEvent(sp, ctx->ev_split, 0));
    // deferred pass on B: needs the split and the reduced gradients, nothing else
    FS_HIP(ctx, hipStreamWaitEvent(sb, ctx->ev_split, 0));
    FS_HIP(ctx, hipStreamWaitEvent(sb, ctx->ev_reduce, 0));
    return enqueue_updates_and_gather(ctx, a, have_t, have_t1, sp);
}

int fs_prioritized_step_pipelined(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    bool have_t, have_t1, nxt_t = false, nxt_t1 = false;
    int rc = check_step_args(ctx, cur, &have_t, &have_t1);
    if (rc != FS_OK) return rc;
    if (next) {
        rc = check_step_args(ctx, next, &nxt_t, &nxt_t1);
        if (rc != FS_OK) return rc;
    }
    hipStream_t sp = as_stream(stream);
    begin_step_timing(ctx);
    // Side stream A still runs what the previous call left there: the index half that produced the
    // split of `cur`, then the previous deferred pass.  It is not waited for at the call boundary -
    // the big kernels of consecutive iterations follow each other without a barrier packet - but
    // once, right before the priority pass.  Cross-stream waits are the expensive host operation
    // here (each makes the runtime flush the producer queue), so there are two per call: A waits
    // for the reduce, `stream` waits for A.
    const bool prev_side = ctx->side_pending;
    const int pp = ctx->pipe_parity, p = pp ^ 1;            // event set of the previous / this call
    const double h0 = now_us();
    if (prev_side) {
        rc = worker_wait(ctx);                               // host side only: its enqueueing is complete
        if (rc != FS_OK) return rc;
    }
    const double h1 = now_us();
    // The reduce overwrites cur->reduced: if the caller did not alternate that buffer, the
    // previous deferred pass (which reads it) has to finish first.
    bool joined_early = false;
    if (prev_side && cur->reduced == ctx->prev_reduced) {
        FS_HIP(ctx, hipStreamWaitEvent(sp, ctx->ev_side[pp], 0));
        joined_early = true;
    }
    // Without a previous pipelined call the side stream forks from `stream`; otherwise its order
    // after the previous deferred pass (which waited for the previous reduce) is all it needs.
    hipEvent_t first_after = nullptr;
    if (!ctx->red_valid) {
        FS_HIP(ctx, hipEventRecord(ctx->ev_fork, sp));
        first_after = ctx->ev_fork;
    }
    hipEvent_t *tex = have_t ? timing_pair(ctx, FS_TIME_UPDATE_EX) : nullptr;
    const bool threaded = !ctx->capturing && ctx->use_worker &&
                          worker_post(ctx, next, nxt_t, nxt_t1, have_t ? cur : nullptr, p, first_after, tex);
    const double h2 = now_us();
    rc = FS_OK;
    if (have_t) rc = enqueue_reduce(ctx, cur, sp);
    if (rc == FS_OK && hipEventRecord(ctx->ev_red[p], sp) != hipSuccess) rc = FS_EHIP;
    if (threaded) ctx->worker->red_recorded.store(true, std::memory_order_release);
    ctx->red_valid = (rc == FS_OK) && !ctx->capturing;
    const double h3 = now_us();
    // from here on the split of `cur` is needed, and the rows the previous deferred pass wrote
    // must be in place before the gather reads the table
    if (rc == FS_OK && prev_side && !joined_early && hipStreamWaitEvent(sp, ctx->ev_side[pp], 0) != hipSuccess)
        rc = FS_EHIP;
    ctx->side_pending = false;
    const double h4 = now_us();
    if (rc == FS_OK) rc = enqueue_priority_and_gather(ctx, cur, have_t, have_t1, sp);
    const double h5 = now_us();
    if (!threaded && rc == FS_OK)
        rc = enqueue_side_stream(ctx, next, nxt_t, nxt_t1, have_t ? cur : nullptr, p, first_after, nullptr, tex);
    if (ctx->timing_now) ++ctx->timing_steps;
    ctx->host_us[0] += h1 - h0;      // waiting for the worker
    ctx->host_us[1] += h2 - h1;      // posting the side-stream work
    ctx->host_us[2] += h3 - h2;      // enqueueing the reduce, recording its event
    ctx->host_us[3] += h4 - h3;      // waiting for the side stream
    ctx->host_us[4] += h5 - h4;      // priority pass and gather
    ctx->host_us[6] += 1.0;
    ctx->pipe_parity = p;
    ctx->prev_reduced = cur->reduced;
    ctx->side_pending = (rc == FS_OK);
    // a captured graph must end with every stream joined
    if (ctx->capturing && rc == FS_OK) rc = join_pending_work(ctx, sp);
    return rc;
}

int fs_step_join(fs_ctx *ctx, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    return join_pending_work(ctx, as_stream(stream));
}

int fs_ctx_host_times(fs_ctx *ctx, double *out7_host, int reset) {
    if (!ctx || !out7_host) return FS_EINVAL;
    (void)worker_wait(ctx);
    for (int i = 0; i < 7; ++i) out7_host[i] = ctx->host_us[i];
    if (reset)
        for (int i = 0; i < 7; ++i) ctx->host_us[i] = 0.0;
    return FS_OK;
}

int fs_ctx_set_threaded_enqueue(fs_ctx *ctx, int on) {
    if (!ctx) return FS_EINVAL;
    ctx->use_worker = on != 0;
    return FS_OK;
}

int fs_graph_capture_pipelined(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next, fs_graph **out) {
    if (!ctx || !out) return FS_EINVAL;
    *out = nullptr;
    fs_graph *g = new (std::nothrow) fs_graph();
    if (!g) return FS_ENOMEM;
    g->graph = nullptr;
    g->exec = nullptr;
    if (ctx->side_pending) {                                 // nothing from outside may leak into the capture
        (void)worker_wait(ctx);
        ctx->side_pending = false;
        (void)hipStreamSynchronize(ctx->stream_a);
    }
    ctx->red_valid = false;
    hipError_t e = hipStreamBeginCapture(ctx->stream_cap, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) {
        delete g;
        return hip_err(ctx, e, "hipStreamBeginCapture");
    }
    ctx->capturing = true;
    const int rc = fs_prioritized_step_pipelined(ctx, cur, next, ctx->stream_cap);
    ctx->capturing = false;
    e = hipStreamEndCapture(ctx->stream_cap, &g->graph);       // always end the capture, also after an error
    if (rc != FS_OK || e != hipSuccess || g->graph == nullptr) {
        if (g->graph) (void)hipGraphDestroy(g->graph);
        delete g;
        (void)hipGetLastError();
        return rc != FS_OK ? rc : hip_err(ctx, e, "hipStreamEndCapture");
    }
    e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        (void)hipGraphDestroy(g->graph);
        delete g;
        return hip_err(ctx, e, "hipGraphInstantiate");
    }
    *out = g;
    return FS_OK;
}

int fs_graph_launch(fs_ctx *ctx, fs_graph *graph, fs_stream stream) {
    if (!ctx || !graph || !graph->exec) return FS_EINVAL;
    FS_HIP(ctx, hipGraphLaunch(graph->exec, as_stream(stream)));
    return FS_OK;
}

int fs_graph_destroy(fs_graph *graph) {
    if (!graph) return FS_OK;
    if (graph->exec) (void)hipGraphExecDestroy(graph->exec);
    if (graph->graph) (void)hipGraphDestroy(graph->graph);
    delete graph;
    return FS_OK;
}

}  // extern "C"
