// C-ABI entry points: argument validation, context/workspace management and the schedules of one
// prioritized iteration (Section 3.2 / Algorithm 2 of the paper, collectives removed): which stream
// runs what, which event orders whom, which host thread enqueues it.  No kernel lives here.
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <functional>
#include <memory>
#include <mutex>
#include <new>
#include <thread>

#include "fs_common.h"

using namespace fs;

static double now_us() {
    return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

struct fs_graph {
    hipGraph_t graph;
    hipGraphExec_t exec;
};

// A host thread that enqueues work on the context's own streams while the calling thread enqueues
// on the caller's: an iteration is a dozen launches plus cross-stream waits, and at several
// microseconds each the host, not the GPU, would set the pace.
struct fs_worker {
    std::thread thread;
    std::mutex mu;
    std::condition_variable cv;
    std::deque<std::function<int()>> jobs;
    bool busy = false, quit = false;
    int rc = FS_OK;               // first failure since the last wait()
    double busy_us = 0.0;
    uint64_t posted = 0, completed = 0;

    void main_loop(int device) {
        (void)hipSetDevice(device);
        std::unique_lock<std::mutex> lk(mu);
        for (;;) {
            cv.wait(lk, [this] { return !jobs.empty() || quit; });
            if (jobs.empty() && quit) return;
            std::function<int()> job = std::move(jobs.front());
            jobs.pop_front();
            busy = true;
            lk.unlock();
            const double t0 = now_us();
            const int r = job();
            const double t1 = now_us();
            lk.lock();
            busy_us += t1 - t0;
            if (r != FS_OK && rc == FS_OK) rc = r;
            busy = false;
            ++completed;
            cv.notify_all();
        }
    }
    void post(std::function<int()> job) {
        std::lock_guard<std::mutex> lk(mu);
        jobs.push_back(std::move(job));
        ++posted;
        cv.notify_all();
    }
    uint64_t posted_so_far() {
        std::lock_guard<std::mutex> lk(mu);
        return posted;
    }
    int wait_for(uint64_t count) {    // the first `count` jobs ever posted have been enqueued on their streams
        std::unique_lock<std::mutex> lk(mu);
        cv.wait(lk, [this, count] { return completed >= count; });
        const int r = rc;
        rc = FS_OK;
        return r;
    }
    int wait() {                  // everything posted so far has been enqueued on its stream
        std::unique_lock<std::mutex> lk(mu);
        cv.wait(lk, [this] { return jobs.empty() && !busy; });
        const int r = rc;
        rc = FS_OK;
        return r;
    }
};

// Work done ahead of time on an index stream whose results a later call consumes: a dedup (key: its
// `unique` output buffer) or the whole index half of an iteration (key: its `counts_dev`).
enum { kAheadFree = 0, kAheadPosted = 1, kAheadRecorded = 2 };
struct fs_ahead {
    const void *key = nullptr;         // calling thread only; null once a consumer has claimed the entry
    hipEvent_t fork = nullptr, done = nullptr;
    std::atomic<int> state{kAheadFree};
    uint64_t stamp = 0;                // calling thread only: allocation order
};
constexpr int kAheadSlots = 8 * kMaxBatch;

struct fs_host {
    fs_worker *worker[2] = {nullptr, nullptr};   // 0: side stream A, 1: index streams
    fs_ahead ahead[kAheadSlots];
    uint64_t ahead_clock = 0;
    uint64_t x_posted_before_call[2] = {0, 0};   // index-stream jobs posted before the pipelined call of each parity
    int x_turn = 0;
};

namespace fs {
char *static_err_buf() {
    static thread_local char buf[256] = "";
    return buf;
}
int set_static_err(int code, const char *msg) {
    snprintf(static_err_buf(), 256, "%s", msg);
    return code;
}
}  // namespace fs

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
    for (int k = 0; k < kSortSets; ++k) {
        fs_sort_scratch &ws = c->sort[k];
        ws.keys[0] = cv.take<uint64_t>(n);
        ws.keys[1] = cv.take<uint64_t>(n);
        ws.idx[0] = cv.take<int32_t>(n);
        ws.idx[1] = cv.take<int32_t>(n);
        ws.tile_hist = cv.take<uint32_t>(sort_tiles * kRadix);
        ws.tile_heads = cv.take<int32_t>(scan_tiles);
    }
    for (int k = 0; k < kSortSets; ++k) {
        fs_split_scratch &ws = c->split[k];
        ws.flag_t = cv.take<uint8_t>(n + 16);
        ws.flag_t1 = cv.take<uint8_t>(n + 16);
        ws.cnt = cv.take<int32_t>(2 * scan_tiles);
        ws.cstart_local = cv.take<int32_t>(n + 16);
        ws.tile_len = cv.take<int32_t>(2 * scan_tiles);
        ws.cidx = cv.take<int32_t>(n + 16);
    }
    c->part_head = cv.take<double>(chunks * (size_t)c->max_dim);
    c->part_last = cv.take<double>(chunks * (size_t)c->max_dim);
    c->chunk_desc = cv.take<int32_t>(chunks * 4);
    const size_t fchunks = (size_t)ceil_div(c->max_ids, kFusedMinChunk) + 2;
    for (int k = 0; k < 2; ++k) {
        c->fpart_head[k] = cv.take<double>(fchunks * (size_t)c->max_dim);
        c->fpart_last[k] = cv.take<double>(fchunks * (size_t)c->max_dim);
        c->fcounters[k] = cv.take<int>(fchunks);
        c->fcounters_sup[k] = cv.take<int>(fchunks);
    }
    c->jag_unique = cv.take<int64_t>(n + 16);
    c->jag_seg = cv.take<int32_t>(n + 16);
    c->jag_n = cv.take<int64_t>(1);
    c->jag_sorted = cv.take<int32_t>(n + 16);
    c->jag_tile_sum = cv.take<int64_t>(scan_tiles);
    c->jag_sel = cv.take<int32_t>(n + 16);
    *total = align_up(cv.off, 256);
}

hipStream_t as_stream(fs_stream s) { return reinterpret_cast<hipStream_t>(s); }

// two-part lookup: what the last call fetched ahead is void once anything else may have written a table
void forget_fetched(fs_ctx *ctx) {
    for (int k = 0; k < FS_MAX_STEP_TABLES; ++k) ctx->fetched_emb[k] = nullptr;
}

void worker_stop(fs_ctx *ctx);
int join_pending_work(fs_ctx *ctx, hipStream_t s);
void drop_ahead(fs_ctx *ctx, const void *key);

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
    (void)static_split_prepare(device);      // fs_collision_split_static's array on this GPU: looked up here, or at its first call
    carve(c, nullptr, &c->slab_bytes);
    if (hipMalloc(&c->slab, c->slab_bytes) != hipSuccess) {
        (void)hipGetLastError();
        delete c;
        return FS_ENOMEM;
    }
    size_t total;
    carve(c, static_cast<char *>(c->slab), &total);
    bool ok = hipMemset(c->slab, 0, 4096) == hipSuccess;
    for (int k = 0; k < 2; ++k) {
        const size_t bytes = ((size_t)ceil_div(c->max_ids, kFusedMinChunk) + 2) * sizeof(int);
        ok = ok && hipMemset(c->fcounters[k], 0, bytes) == hipSuccess;
        ok = ok && hipMemset(c->fcounters_sup[k], 0, bytes) == hipSuccess;
    }
    c->host = new (std::nothrow) fs_host();
    ok = ok && c->host != nullptr;
    // The chip gives a process four hardware queues; streams beyond that share them, and two streams on one
    // queue run one after the other.  Only the streams of the steady-state step exist from the start (side
    // stream, index streams: with the caller's stream that makes four); the self-contained step's second side
    // stream and the capture stream are created when first needed.
    ok = ok && hipStreamCreateWithFlags(&c->stream_a, hipStreamNonBlocking) == hipSuccess;
    for (hipStream_t &st : c->stream_x) ok = ok && hipStreamCreateWithFlags(&st, hipStreamNonBlocking) == hipSuccess;
    hipEvent_t *evs[] = {&c->ev_fork, &c->ev_split, &c->ev_ex, &c->ev_pfork[0], &c->ev_pfork[1], &c->ev_side[0],
                         &c->ev_side[1]};
    // These events order work of this device's streams among themselves and nothing else: nobody reads through
    // them what a kernel wrote (the host only asks whether one has passed, to skip a wait).  Without the
    // system-scope fence that a recorded event otherwise brings, the kernel behind a wait keeps the caches as the
    // kernels before it left them (measured: 2 to 3 us per step on every workload).
    constexpr unsigned kOrderEvent = hipEventDisableTiming | hipEventDisableSystemFence;
    for (hipEvent_t *e : evs) ok = ok && hipEventCreateWithFlags(e, kOrderEvent) == hipSuccess;
    if (c->host)
        for (fs_ahead &a : c->host->ahead) {
            ok = ok && hipEventCreateWithFlags(&a.fork, kOrderEvent) == hipSuccess;
            ok = ok && hipEventCreateWithFlags(&a.done, kOrderEvent) == hipSuccess;
        }
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
    hipStream_t streams[] = {c->stream_a, c->stream_b, c->stream_cap};
    for (hipStream_t st : streams)
        if (st) { (void)hipStreamSynchronize(st); (void)hipStreamDestroy(st); }
    for (hipStream_t st : c->stream_x)
        if (st) { (void)hipStreamSynchronize(st); (void)hipStreamDestroy(st); }
    hipEvent_t evs[] = {c->ev_fork, c->ev_split, c->ev_ex, c->ev_pfork[0], c->ev_pfork[1], c->ev_side[0], c->ev_side[1]};
    for (hipEvent_t e : evs)
        if (e) (void)hipEventDestroy(e);
    if (c->host) {
        for (fs_ahead &a : c->host->ahead) {
            if (a.fork) (void)hipEventDestroy(a.fork);
            if (a.done) (void)hipEventDestroy(a.done);
        }
        delete c->host;
        c->host = nullptr;
    }
    (void)fs_ctx_set_kernel_timing(c, 0, 1);
    if (c->slab) (void)hipFree(c->slab);
    delete c;
    return FS_OK;
}

const char *fs_last_error(const fs_ctx *ctx) { return ctx ? ctx->err : static_err_buf(); }

size_t fs_ctx_workspace_bytes(const fs_ctx *ctx) { return ctx ? ctx->slab_bytes : 0; }

int fs_check_async(fs_ctx *ctx, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    const int jrc = join_pending_work(ctx, as_stream(stream));
    if (jrc != FS_OK) return jrc;
    FS_HIP(ctx, hipStreamSynchronize(as_stream(stream)));
    FS_HIP(ctx, hipStreamSynchronize(ctx->stream_a));
    if (ctx->stream_b) FS_HIP(ctx, hipStreamSynchronize(ctx->stream_b));
    for (hipStream_t sx : ctx->stream_x) FS_HIP(ctx, hipStreamSynchronize(sx));
    int flags[4] = {0, 0, 0, 0};
    FS_HIP(ctx, hipMemcpy(flags, ctx->d_flags, sizeof(flags), hipMemcpyDeviceToHost));
    if (flags[0] == 0) return FS_OK;
    FS_HIP(ctx, hipMemset(ctx->d_flags, 0, sizeof(flags)));
    if (flags[0] & kFlagInternal) {
        // a fused pass that met an inconsistent class order left cut segments half counted in: the arrival
        // counters must stand at zero again before the next pass (every stream is idle here)
        const size_t bytes = ((size_t)ceil_div(ctx->max_ids, kFusedMinChunk) + 2) * sizeof(int);
        for (int k = 0; k < 2; ++k) {
            FS_HIP(ctx, hipMemset(ctx->fcounters[k], 0, bytes));
            FS_HIP(ctx, hipMemset(ctx->fcounters_sup[k], 0, bytes));
        }
    }
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

int fs_gather_jagged_class(fs_ctx *ctx, const void *table, int64_t num_rows, int32_t dim, fs_dtype dt,
                           const int64_t *values, const int64_t *offsets, int64_t batch, int64_t n_values,
                           const int32_t *inverse, const uint8_t *co_flag, int which, void *out, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, dt == FS_F32 || dt == FS_BF16, "gather: unknown dtype");
    FS_REQUIRE(ctx, dim_ok(dim, dt), "gather: dim must be a multiple of 4 (fp32) / 8 (bf16), at most FS_MAX_DIM");
    FS_REQUIRE(ctx, num_rows >= 0 && batch >= 0 && n_values >= 0, "gather: negative size");
    FS_REQUIRE(ctx, n_values <= (1ll << 31) - 1, "gather: more than 2^31-1 values");
    FS_REQUIRE(ctx, which == 0 || which == 1, "gather: which must be 0 (exclusive rows) or 1 (collision rows)");
    if (n_values == 0) return FS_OK;
    FS_REQUIRE(ctx, table && values && out && inverse && co_flag, "gather: null pointer");
    fs_gather_job job;
    job.table = table; job.num_rows = num_rows; job.row_bytes = dim * (dt == FS_F32 ? 4 : 2); job.values = values;
    job.offsets = offsets; job.batch = batch; job.n = n_values; job.out = out;
    job.inverse = inverse; job.row_flag = co_flag; job.which = which;
    return launch_gather_batch(ctx, 1, &job, as_stream(stream));
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
    drop_ahead(ctx, unique);
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
    forget_fetched(ctx);
    return launch_adagrad(ctx, table, dt, state, num_rows, dim, rows, slots, n_rows_dev, cap, reduced, lr, eps,
                          as_stream(stream));
}

int fs_partition_fbs(fs_ctx *ctx, const int64_t *lengths, int64_t B, int64_t max_len, int32_t n_ranks,
                     int32_t *sample_of, int64_t *rank_offsets, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, B >= 0 && max_len >= 0 && n_ranks >= 1, "fbs: negative size or no rank");
    if (B > ctx->max_ids) return set_err(ctx, FS_ENOMEM, "fbs: B beyond the context capacity");
    FS_REQUIRE(ctx, rank_offsets && (B == 0 || (lengths && sample_of)), "fbs: null pointer");
    const int jrc = join_pending_work(ctx, as_stream(stream));      // the index workspace may still be in use
    if (jrc != FS_OK) return jrc;
    return launch_partition_fbs(ctx, lengths, B, max_len, n_ranks, sample_of, rank_offsets, as_stream(stream));
}

int fs_partition_vbs(fs_ctx *ctx, const int64_t *lengths, int64_t B, const int64_t *weight_of_len, int64_t max_len,
                     int32_t n_ranks, int32_t *sample_of, int64_t *rank_offsets, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, B >= 0 && max_len >= 0 && n_ranks >= 1, "vbs: negative size or no rank");
    if (B > ctx->max_ids) return set_err(ctx, FS_ENOMEM, "vbs: B beyond the context capacity");
    FS_REQUIRE(ctx, rank_offsets && (B == 0 || (lengths && sample_of && weight_of_len)), "vbs: null pointer");
    const int jrc = join_pending_work(ctx, as_stream(stream));      // the index workspace may still be in use
    if (jrc != FS_OK) return jrc;
    return launch_partition_vbs(ctx, lengths, B, weight_of_len, max_len, n_ranks, sample_of, rank_offsets,
                                as_stream(stream));
}

int fs_jagged_indexed_permute(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                              const int64_t *offsets, int64_t B, const int32_t *sample_of, int64_t n_out,
                              void *out_values, int64_t cap_out, int64_t *out_offsets, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, n_values >= 0 && B >= 0 && n_out >= 0 && cap_out >= 0, "indexed permute: negative size");
    FS_REQUIRE(ctx, elem_bytes > 0 && elem_bytes % 4 == 0, "indexed permute: elem_bytes must be a multiple of 4");
    if (n_out > ctx->max_ids) return set_err(ctx, FS_ENOMEM, "indexed permute: n_out beyond the context capacity");
    FS_REQUIRE(ctx, out_offsets && (n_out == 0 || (offsets && sample_of)), "indexed permute: null pointer");
    FS_REQUIRE(ctx, cap_out == 0 || n_out == 0 || (values && out_values), "indexed permute: null pointer");
    const int jrc = join_pending_work(ctx, as_stream(stream));
    if (jrc != FS_OK) return jrc;
    return launch_indexed_permute(ctx, values, n_values, elem_bytes, offsets, B, sample_of, n_out, out_values, cap_out,
                                  out_offsets, as_stream(stream));
}

namespace {
int keyed_shuffle(fs_ctx *ctx, int mode, const void *values, int64_t n_values, int32_t elem_bytes, const int64_t *offsets,
                  int64_t F, int64_t B, const int64_t *rank_offsets, int32_t n_ranks, void *out_values,
                  int64_t *out_offsets, int64_t *splits, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, n_values >= 0 && F >= 0 && B >= 0, "keyed shuffle: negative size");
    FS_REQUIRE(ctx, elem_bytes > 0 && elem_bytes % 4 == 0, "keyed shuffle: elem_bytes must be a multiple of 4");
    if (F > 0 && B > ctx->max_ids / F) return set_err(ctx, FS_ENOMEM, "keyed shuffle: F * B beyond the context capacity");
    FS_REQUIRE(ctx, offsets && out_offsets && (n_values == 0 || (values && out_values)), "keyed shuffle: null pointer");
    if (mode != 0) FS_REQUIRE(ctx, n_ranks >= 1 && rank_offsets, "keyed shuffle: no ranks");
    const int jrc = join_pending_work(ctx, as_stream(stream));
    if (jrc != FS_OK) return jrc;
    return launch_keyed_shuffle(ctx, mode, values, n_values, elem_bytes, offsets, F, B, rank_offsets, n_ranks, out_values,
                                out_offsets, splits, as_stream(stream));
}
}  // namespace

int fs_jagged_keyed_transpose(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                              const int64_t *offsets, int64_t F, int64_t B, void *out_values, int64_t *out_offsets,
                              fs_stream stream) {
    return keyed_shuffle(ctx, 0, values, n_values, elem_bytes, offsets, F, B, nullptr, 0, out_values, out_offsets, nullptr,
                         stream);
}

int fs_jagged_ranged_dispatch(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                              const int64_t *offsets, int64_t F, int64_t B, const int64_t *rank_offsets, int32_t n_ranks,
                              void *out_values, int64_t *out_offsets, int64_t *splits, fs_stream stream) {
    if (ctx && !splits) return set_err(ctx, FS_EINVAL, "ranged dispatch: null splits");
    return keyed_shuffle(ctx, 1, values, n_values, elem_bytes, offsets, F, B, rank_offsets, n_ranks, out_values,
                         out_offsets, splits, stream);
}

int fs_jagged_ranged_combine(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                             const int64_t *offsets, int64_t F, int64_t B, const int64_t *rank_offsets, int32_t n_ranks,
                             void *out_values, int64_t *out_offsets, fs_stream stream) {
    return keyed_shuffle(ctx, 2, values, n_values, elem_bytes, offsets, F, B, rank_offsets, n_ranks, out_values,
                         out_offsets, nullptr, stream);
}

int fs_init_table_hash(fs_ctx *ctx, void *table, int64_t num_rows, int32_t dim, fs_dtype dt, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, dt == FS_F32 || dt == FS_BF16, "init: unknown dtype");
    FS_REQUIRE(ctx, dim_ok(dim, dt) && num_rows >= 0, "init: bad shape");
    if (num_rows == 0) return FS_OK;
    FS_REQUIRE(ctx, table, "init: null pointer");
    forget_fetched(ctx);
    return launch_init_hash(ctx, table, num_rows, dim, dt, as_stream(stream));
}

int fs_stream_row_read(fs_ctx *ctx, const void *rows, int64_t num_rows, int32_t row_bytes, const int64_t *index,
                       int64_t n, uint32_t *sink, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, num_rows >= 0 && n >= 0, "row read: negative size");
    FS_REQUIRE(ctx, row_bytes > 0 && row_bytes % 16 == 0 && row_bytes <= 1024, "row read: rows of 16..1024 bytes, a multiple of 16");
    if (n == 0 || num_rows == 0) return FS_OK;
    FS_REQUIRE(ctx, rows && index && sink, "row read: null pointer");
    return launch_row_read(ctx, rows, num_rows, row_bytes, index, n, sink, as_stream(stream));
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

// host-visible checks shared by the step entry points; `have_t`: iteration t is used (updates),
// `have_t1`: the lookahead batch is used (dedup, gather)
int check_step_args(fs_ctx *ctx, const fs_step_args *a, bool *have_t, bool *have_t1) {
    FS_REQUIRE(ctx, a, "step: null args");
    const int dt = a->dtype;
    FS_REQUIRE(ctx, dt == FS_F32 || dt == FS_BF16, "step: unknown dtype");
    FS_REQUIRE(ctx, dim_ok(a->dim, dt), "step: unsupported dim");
    FS_REQUIRE(ctx, a->num_rows >= 0 && a->n_t >= 0 && a->n_t1 >= 0 && a->batch_t1 >= 0, "step: negative size");
    if (a->n_t > ctx->max_ids || a->n_t1 > ctx->max_ids || a->dim > ctx->max_dim)
        return set_err(ctx, FS_ENOMEM, "step: beyond the context capacity");
    FS_REQUIRE(ctx, a->table && a->state && a->counts_dev && a->class_pos_dev, "step: null table/state/counts");
    *have_t = a->n_t > 0;
    *have_t1 = a->values_t1 != nullptr && a->n_t1 > 0;
    if (*have_t)
        FS_REQUIRE(ctx, a->u_t && a->seg_offsets_t && a->perm_t && a->n_unique_t_dev && a->grads_t &&
                            a->co && a->co_slot && a->ex && a->ex_slot && a->cperm && a->cslot && a->cstart && a->short_rec,
                   "step: null pointer (iteration t)");
    if (*have_t1)
        FS_REQUIRE(ctx, a->u_t1 && a->seg_offsets_t1 && a->perm_t1 && a->n_unique_t1_dev &&
                            a->ex_next && a->ex_next_slot && a->emb_t1,
                   "step: null pointer (lookahead)");
    return FS_OK;
}

// one step in `timing_every` gets its kernels bracketed by event pairs (an event record costs the
// host more than a kernel launch, so bracketing every step would slow the very thing it measures)
void begin_step_timing(fs_ctx *ctx) {
    ctx->timing_now = ctx->timing_slots > 0 && !ctx->capturing && (ctx->step_counter % ctx->timing_every) == 0;
    if (ctx->timing_slots > 0 && !ctx->capturing) ++ctx->step_counter;
}

}  // namespace

namespace {

fs_worker *get_worker(fs_ctx *ctx, int which) {
    fs_host *h = ctx->host;
    if (!h->worker[which]) {
        fs_worker *w = new (std::nothrow) fs_worker();
        if (!w) return nullptr;
        const int device = ctx->device;
        w->thread = std::thread([w, device] { w->main_loop(device); });
        h->worker[which] = w;
    }
    return h->worker[which];
}

int workers_wait(fs_ctx *ctx) {
    int rc = FS_OK;
    for (int k = 0; k < 2; ++k)
        if (ctx->host && ctx->host->worker[k]) {
            const int r = ctx->host->worker[k]->wait();
            if (rc == FS_OK) rc = r;
        }
    if (rc != FS_OK && ctx->err[0] == 0) snprintf(ctx->err, sizeof(ctx->err), "side-stream enqueue failed");
    return rc;
}

void worker_stop(fs_ctx *ctx) {
    if (!ctx->host) return;
    for (int k = 0; k < 2; ++k) {
        fs_worker *w = ctx->host->worker[k];
        if (!w) continue;
        {
            std::lock_guard<std::mutex> lk(w->mu);
            w->quit = true;
            w->cv.notify_all();
        }
        if (w->thread.joinable()) w->thread.join();
        delete w;
        ctx->host->worker[k] = nullptr;
    }
}

// the outstanding ahead-of-time work registered under `key`, if any (calling thread only)
fs_ahead *find_ahead(fs_ctx *ctx, const void *key) {
    if (!key) return nullptr;
    for (fs_ahead &e : ctx->host->ahead)
        if (e.key == key && e.state.load(std::memory_order_acquire) != kAheadFree) return &e;
    return nullptr;
}

// find_ahead + claim: the caller hands the entry to exactly one consumer (consume_ahead)
fs_ahead *claim_ahead(fs_ctx *ctx, const void *key) {
    fs_ahead *e = find_ahead(ctx, key);
    if (e) e->key = nullptr;
    return e;
}

// a free entry, registered under `key` (calling thread only).  When all are taken, the oldest finished
// one that nobody claimed is given up: its results are complete, whoever names its buffers later
// simply finds no entry and redoes or skips the work as if it had never been done ahead.
fs_ahead *alloc_ahead(fs_ctx *ctx, const void *key) {
    fs_host *h = ctx->host;
    fs_ahead *e = nullptr;
    for (fs_ahead &c : h->ahead)
        if (c.state.load(std::memory_order_acquire) == kAheadFree) { e = &c; break; }
    if (!e) {
        (void)workers_wait(ctx);
        for (fs_ahead &c : h->ahead)
            if (c.key != nullptr && c.state.load(std::memory_order_acquire) == kAheadRecorded &&
                (e == nullptr || c.stamp < e->stamp))
                e = &c;
        if (!e) return nullptr;
        (void)hipEventSynchronize(e->done);
        e->state.store(kAheadFree, std::memory_order_release);
    }
    e->key = key;
    e->stamp = ++h->ahead_clock;
    e->state.store(kAheadPosted, std::memory_order_release);
    return e;
}

// stream `s` waits for the work of `e`; the slot is free afterwards (any thread; `e` was claimed)
int consume_ahead(fs_ctx *ctx, fs_ahead *e, hipStream_t s) {
    while (e->state.load(std::memory_order_acquire) != kAheadRecorded) std::this_thread::yield();
    // Work issued iterations ahead has usually finished by now: asking costs a microsecond, a cross-stream
    // wait twenty (it makes the runtime flush the producer's queue)
    hipError_t err = hipEventQuery(e->done);
    if (err != hipSuccess) {
        (void)hipGetLastError();                              // "not ready" is not an error to keep
        err = hipStreamWaitEvent(s, e->done, 0);
    }
    e->state.store(kAheadFree, std::memory_order_release);
    if (err != hipSuccess) return hip_err(ctx, err, "hipStreamWaitEvent(ahead)");
    return FS_OK;
}

// Forward of Algorithm 2 (index work) for `count` argument records in shared launches: dedup of the
// lookahead IDs (unless done ahead of time), the collision split of U_t, the class order of batch t.
// Per record: `ahead` = its dedup was done by fs_unique_ids_ahead (only waited for); `dedup_out` =
// entry to signal once its layout of t+1 stands; `layout_in` = the layout of t is still in the making
// on another index stream.  Record k works in scratch set set0 + k.
int enqueue_index_work_batch(fs_ctx *ctx, int count, const fs_step_args *a, const bool *have_t, const bool *have_t1,
                             fs_ahead *const *ahead, hipStream_t s, int set0, fs_ahead *const *dedup_out,
                             fs_ahead *const *layout_in) {
    int rc = FS_OK;
    // dedups: those not done ahead of time share their launches (each keeps the scratch set of its record:
    // a job list with gaps is passed as separate runs)
    for (int k = 0; k < count; ++k)
        if (have_t1[k] && ahead && ahead[k]) {
            const int r = consume_ahead(ctx, ahead[k], s);
            if (rc == FS_OK) rc = r;
            // fs_unique_ids_ahead has no place for the ascending ID list: a lookup that walked it would read junk
            if (a[k].sorted_ids_t1 != nullptr && rc == FS_OK)
                rc = set_err(ctx, FS_EINVAL, "step: sorted_ids_t1 given, but the dedup of this batch was done by "
                                             "fs_unique_ids_ahead, which does not write it");
        }
    for (int k0 = 0; k0 < count && rc == FS_OK;) {
        if (!(have_t1[k0] && !(ahead && ahead[k0]))) { ++k0; continue; }
        fs_unique_job jobs[kMaxBatch];
        int m = 0;
        while (k0 + m < count && have_t1[k0 + m] && !(ahead && ahead[k0 + m])) {
            const fs_step_args &x = a[k0 + m];
            jobs[m] = fs_unique_job{x.values_t1, x.n_t1, x.num_rows, x.u_t1, x.seg_offsets_t1, x.perm_t1, x.inverse_t1,
                                    x.n_unique_t1_dev, x.sorted_ids_t1};
            ++m;
        }
        rc = launch_unique_batch(ctx, m, jobs, s, set0 + k0);
        k0 += m;
    }
    if (dedup_out)
        for (int k = 0; k < count; ++k)
            if (dedup_out[k]) {
                // the layout of t+1 stands from here on: the index half of t+1 (other stream) waits for this
                const hipError_t e = hipEventRecord(dedup_out[k]->done, s);
                dedup_out[k]->state.store(kAheadRecorded, std::memory_order_release);
                if (e != hipSuccess && rc == FS_OK) rc = hip_err(ctx, e, "hipEventRecord(dedup)");
            }
    if (layout_in)
        for (int k = 0; k < count; ++k)
            if (layout_in[k]) {                               // the layout of t comes from another index stream
                const int r = consume_ahead(ctx, layout_in[k], s);
                if (rc == FS_OK) rc = r;
            }
    if (rc != FS_OK) return rc;
    fs_split_job sj[kMaxBatch];
    fs_class_job cj[kMaxBatch];
    for (int k = 0; k < count; ++k) {
        const fs_step_args &x = a[k];
        const bool t = have_t[k], t1 = have_t1[k];
        sj[k] = fs_split_job{x.u_t, t ? x.n_unique_t_dev : nullptr, x.u_t1, t1 ? x.n_unique_t1_dev : nullptr,
                             t ? x.n_t : 0, t1 ? x.n_t1 : 0, x.co, x.co_slot, x.ex, x.ex_slot, x.ex_next,
                             x.ex_next_slot, x.counts_dev, t ? x.seg_offsets_t : nullptr, t1 ? x.co_flag_t1 : nullptr};
        cj[k] = fs_class_job{x.perm_t, x.n_unique_t_dev, x.seg_offsets_t, t ? x.n_t : 0, t ? x.n_t : 0, x.cperm, x.cslot,
                             x.cstart, x.class_pos_dev, x.u_t, x.short_rec};
    }
    rc = launch_split_batch(ctx, count, sj, s, set0);
    if (rc != FS_OK) return rc;
    return launch_class_order_batch(ctx, count, cj, s, set0);
}

int enqueue_index_work(fs_ctx *ctx, const fs_step_args *a, bool have_t, bool have_t1, fs_ahead *ahead,
                       hipStream_t s, int set = 0, fs_ahead *dedup_out = nullptr, fs_ahead *layout_in = nullptr) {
    return enqueue_index_work_batch(ctx, 1, a, &have_t, &have_t1, &ahead, s, set, &dedup_out, &layout_in);
}

// update_embedding for one class of rows of iteration t (0: priority pass, 1: deferred pass) of `count`
// tables (`use[k]`: table k has gradients); tables of one row width share their launches
fs_class_pass_job class_job(const fs_step_args *a, int cls) {
    return fs_class_pass_job{a->grads_t, a->n_t, a->dim, a->cperm, a->cslot, a->class_pos_dev, a->seg_offsets_t,
                             a->cstart, a->u_t, a->table, a->dtype, a->state, a->num_rows, a->lr, a->eps, a->reduced,
                             a->short_rec + (int64_t)cls * a->n_t * kShortRecInts, a->counts_dev + cls};
}

int enqueue_class_passes(fs_ctx *ctx, const fs_step_args *a, const bool *use, int count, int cls, hipStream_t s,
                         hipEvent_t *timing) {
    fs_class_pass_job jobs[FS_MAX_STEP_TABLES];
    int m = 0;
    for (int k = 0; k < count; ++k)
        if (use[k]) jobs[m++] = class_job(&a[k], cls);
    if (m == 0) return FS_OK;
    if (timing) (void)hipEventRecord(timing[0], s);
    const int rc = launch_reduce_update_batch(ctx, cls, m, jobs, s);
    if (timing && rc == FS_OK) (void)hipEventRecord(timing[1], s);
    return rc;
}

int enqueue_class_pass(fs_ctx *ctx, const fs_step_args *a, int cls, hipStream_t s, hipEvent_t *timing) {
    const bool use = true;
    return enqueue_class_passes(ctx, a, &use, 1, cls, s, timing);
}

// `part` (optional): per table -1 = the whole lookup, 0 / 1 = the exclusive / collision rows only
int enqueue_gathers(fs_ctx *ctx, const fs_step_args *a, const bool *use, int count, hipStream_t s,
                    const int *part = nullptr, bool timed = true) {
    fs_gather_job jobs[FS_MAX_STEP_TABLES];
    int m = 0;
    for (int k = 0; k < count; ++k)
        if (use[k]) {
            fs_gather_job &j = jobs[m++];
            j = fs_gather_job{a[k].table, a[k].num_rows, a[k].dim * (a[k].dtype == FS_F32 ? 4 : 2), a[k].values_t1,
                              a[k].offsets_t1, a[k].batch_t1, a[k].n_t1, a[k].emb_t1};
            if (part && part[k] >= 0) {
                j.inverse = a[k].inverse_t1; j.row_flag = a[k].co_flag_t1; j.which = part[k];
            } else if (a[k].sorted_ids_t1 != nullptr) {
                j.sorted_ids = a[k].sorted_ids_t1; j.perm = a[k].perm_t1;
            }
        }
    if (m == 0) return FS_OK;
    hipEvent_t *tg = timed ? timing_pair(ctx, FS_TIME_GATHER) : nullptr;
    if (tg) (void)hipEventRecord(tg[0], s);
    const int rc = launch_gather_batch(ctx, m, jobs, s);
    if (tg && rc == FS_OK) (void)hipEventRecord(tg[1], s);
    return rc;
}

int enqueue_gather(fs_ctx *ctx, const fs_step_args *a, hipStream_t s) {
    const bool use = true;
    return enqueue_gathers(ctx, a, &use, 1, s);
}

// What one pipelined call hands to side stream A: for each of its tables the deferred pass of `cur` and the
// index half of `next` (done ahead of time on an index stream: only waited for; else done here).
constexpr int kMaxTables = FS_MAX_STEP_TABLES;
struct side_work {
    int count = 0, parity = 0;
    hipEvent_t *ex_timing = nullptr;
    fs_step_args cur[kMaxTables], next[kMaxTables];
    bool have_t[kMaxTables], has_next[kMaxTables], nxt_t[kMaxTables], nxt_t1[kMaxTables];
    fs_ahead *ahead[kMaxTables], *index_ahead[kMaxTables];
    bool fetch_next[kMaxTables];    // two-part lookup: fetch the exclusive rows of next's lookahead batch
};

// Side stream A for one pipelined call: after the caller's earlier work (the gradients of `cur`), the
// deferred passes, then the index halves of `next`, then the event the next call waits for.
int enqueue_side_stream(fs_ctx *ctx, const side_work &w) {
    hipStream_t sa = ctx->stream_a;
    int rc = FS_OK;
    FS_HIP(ctx, hipStreamWaitEvent(sa, ctx->ev_pfork[w.parity], 0));
    rc = enqueue_class_passes(ctx, w.cur, w.have_t, w.count, 1, sa, w.ex_timing);
    for (int k = 0; k < w.count; ++k) {
        if (w.index_ahead[k]) {
            const int r = consume_ahead(ctx, w.index_ahead[k], sa);
            if (rc == FS_OK) rc = r;
        } else if (rc == FS_OK && w.has_next[k]) {
            rc = enqueue_index_work(ctx, &w.next[k], w.nxt_t[k], w.nxt_t1[k], w.ahead[k], sa);
        } else if (w.ahead[k]) {
            (void)consume_ahead(ctx, w.ahead[k], sa);
        }
    }
    if (rc != FS_OK) return rc;
    // Forward of Algorithm 2 ends with Lookup(I_ex^{i+1}): every deferred pass so far has landed on this
    // stream, and no priority pass writes a row that is not a collision row
    int part[kMaxTables];
    for (int k = 0; k < w.count; ++k) part[k] = 0;
    rc = enqueue_gathers(ctx, w.next, w.fetch_next, w.count, sa, part, false);
    if (rc != FS_OK) return rc;
    FS_HIP(ctx, hipEventRecord(ctx->ev_side[w.parity], sa));
    return FS_OK;
}

// Makes `s` wait for what earlier calls left running on the context's own streams: the side work of
// the last pipelined call, and every ahead-of-time dedup no step has claimed yet (those stay
// registered: a later step may still name their buffers).
int join_pending_work(fs_ctx *ctx, hipStream_t s) {
    const int wrc = workers_wait(ctx);
    if (ctx->side_pending) {
        ctx->side_pending = false;
        FS_HIP(ctx, hipStreamWaitEvent(s, ctx->ev_side[ctx->pipe_parity], 0));
    }
    if (!ctx->capturing)
        for (fs_ahead &e : ctx->host->ahead)
            if (e.key != nullptr && e.state.load(std::memory_order_acquire) == kAheadRecorded)
                FS_HIP(ctx, hipStreamWaitEvent(s, e.done, 0));
    return wrc;
}

// forget ahead-of-time work registered under `key` (its buffers are about to be rewritten by someone
// else); only after join_pending_work, so the entry is finished
void drop_ahead(fs_ctx *ctx, const void *key) {
    fs_ahead *e = find_ahead(ctx, key);
    if (e) {
        e->key = nullptr;
        e->state.store(kAheadFree, std::memory_order_release);
    }
}

}  // namespace

extern "C" {

int fs_collision_split_classes(fs_ctx *ctx, const int64_t *u_t, const int64_t *n_t_dev, const int64_t *u_t1,
                               const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1, const int32_t *seg_offsets_t,
                               const int32_t *perm_t, const int32_t *inverse_t, int64_t n_t, int64_t *co,
                               int32_t *co_slot, int64_t *ex, int32_t *ex_slot, int64_t *ex_next,
                               int32_t *ex_next_slot, int64_t *counts_dev, int32_t *cperm, int32_t *cslot,
                               int32_t *cstart, int32_t *class_pos_dev, int32_t *short_rec, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    (void)inverse_t;
    FS_REQUIRE(ctx, cap_t >= 0 && cap_t1 >= 0 && n_t >= 0, "split: negative size");
    if (cap_t > ctx->max_ids || cap_t1 > ctx->max_ids || n_t > ctx->max_ids)
        return set_err(ctx, FS_ENOMEM, "split: capacity beyond the context capacity");
    FS_REQUIRE(ctx, counts_dev && class_pos_dev, "split: null counts");
    FS_REQUIRE(ctx, (n_t == 0) == (cap_t == 0), "split: n_t and cap_t must both be zero or both positive");
    if (cap_t > 0)
        FS_REQUIRE(ctx, u_t && n_t_dev && co && co_slot && ex && ex_slot && seg_offsets_t && perm_t &&
                            cperm && cslot && cstart && short_rec,
                   "split: null pointer (t side)");
    if (cap_t1 > 0) FS_REQUIRE(ctx, u_t1 && n_t1_dev && ex_next && ex_next_slot, "split: null pointer (t+1 side)");
    int rc = join_pending_work(ctx, as_stream(stream));      // the workspace may still be in use on A
    if (rc != FS_OK) return rc;
    rc = launch_split(ctx, u_t, cap_t > 0 ? n_t_dev : nullptr, u_t1, cap_t1 > 0 ? n_t1_dev : nullptr, cap_t, cap_t1,
                      co, co_slot, ex, ex_slot, ex_next, ex_next_slot, counts_dev, as_stream(stream),
                      cap_t > 0 ? seg_offsets_t : nullptr);
    if (rc != FS_OK) return rc;
    return launch_class_order(ctx, perm_t, n_t_dev, seg_offsets_t, n_t, cap_t, cperm, cslot, cstart, class_pos_dev,
                              u_t, short_rec, as_stream(stream));
}

int fs_reduce_update_class(fs_ctx *ctx, int cls, void *table, fs_dtype dt, float *state, int64_t num_rows,
                           int32_t dim, float lr, float eps, const float *grads, int64_t n, const int64_t *u_t,
                           const int32_t *seg_offsets, const int32_t *short_rec_cls, const int64_t *n_rows_dev,
                           const int32_t *cperm, const int32_t *cslot, const int32_t *cstart,
                           const int32_t *class_pos_dev, float *reduced, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, cls == 0 || cls == 1, "reduce+update: class must be 0 or 1");
    forget_fetched(ctx);
    FS_REQUIRE(ctx, dt == FS_F32 || dt == FS_BF16, "reduce+update: unknown dtype");
    FS_REQUIRE(ctx, dim_ok(dim, dt), "reduce+update: dim must be a multiple of 4 (fp32) / 8 (bf16), at most FS_MAX_DIM");
    FS_REQUIRE(ctx, num_rows >= 0 && n >= 0, "reduce+update: negative size");
    if (n > ctx->max_ids || dim > ctx->max_dim)
        return set_err(ctx, FS_ENOMEM, "reduce+update: beyond the context capacity");
    if (n == 0) return FS_OK;
    FS_REQUIRE(ctx, table && state && grads && u_t && seg_offsets && short_rec_cls && n_rows_dev && cperm && cslot &&
                        cstart && class_pos_dev,
               "reduce+update: null pointer");
    return launch_reduce_update(ctx, cls, grads, n, dim, cperm, cslot, class_pos_dev, seg_offsets, cstart, u_t, table,
                                dt, state, num_rows, lr, eps, reduced, as_stream(stream), short_rec_cls, n_rows_dev);
}

int fs_split_grads(fs_ctx *ctx, const float *grads, int64_t n, int32_t dim, const int32_t *inverse_t,
                   const int32_t *co_slot, const int64_t *n_co_dev, int64_t cap_u, int32_t *co_index, float *g_co,
                   int32_t *ex_index, float *g_ex, int32_t *part_pos, int64_t *part_counts_dev, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, n >= 0 && cap_u >= 0 && cap_u <= n, "split grads: negative size, or more distinct rows than occurrences");
    FS_REQUIRE(ctx, dim_ok(dim, FS_F32), "split grads: dim must be a multiple of 4, at most FS_MAX_DIM");
    if (n > ctx->max_ids) return set_err(ctx, FS_ENOMEM, "split grads: n beyond the context capacity");
    FS_REQUIRE(ctx, part_counts_dev, "split grads: null counts");
    if (n > 0)
        FS_REQUIRE(ctx, grads && inverse_t && co_slot && n_co_dev && co_index && g_co && ex_index && g_ex && part_pos,
                   "split grads: null pointer");
    const int jrc = join_pending_work(ctx, as_stream(stream));      // the index workspace may still be in use
    if (jrc != FS_OK) return jrc;
    return launch_split_grads(ctx, grads, n, dim, inverse_t, co_slot, n_co_dev, cap_u, co_index, g_co, ex_index, g_ex,
                              part_pos, part_counts_dev, as_stream(stream));
}

int fs_class_order_for_parts(fs_ctx *ctx, const int32_t *part_pos, int64_t n_t, const int32_t *cperm,
                             const int32_t *class_pos_dev, const int32_t *short_rec, const int64_t *counts_dev,
                             int32_t *cperm_parts, int32_t *short_rec_parts, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, n_t >= 0, "class order for parts: negative size");
    if (n_t > ctx->max_ids) return set_err(ctx, FS_ENOMEM, "class order for parts: n_t beyond the context capacity");
    if (n_t == 0) return FS_OK;
    FS_REQUIRE(ctx, part_pos && cperm && class_pos_dev && short_rec && counts_dev && cperm_parts && short_rec_parts,
               "class order for parts: null pointer");
    return launch_class_order_for_parts(ctx, part_pos, n_t, n_t, cperm, class_pos_dev, short_rec, counts_dev,
                                        cperm_parts, short_rec_parts, as_stream(stream));
}

int fs_unique_ids_ahead(fs_ctx *ctx, const int64_t *ids, int64_t n, int64_t num_rows, int64_t *unique,
                        int32_t *seg_offsets, int32_t *perm, int32_t *inverse, int64_t *n_unique_dev,
                        fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, n >= 0 && num_rows >= 0, "unique: negative size");
    if (n > ctx->max_ids) return set_err(ctx, FS_ENOMEM, "unique: n beyond the context capacity");
    FS_REQUIRE(ctx, unique && seg_offsets && n_unique_dev, "unique: null pointer");
    if (n > 0) FS_REQUIRE(ctx, ids && perm, "unique: null pointer");
    FS_REQUIRE(ctx, !ctx->capturing, "unique ahead: not while a graph is being captured");
    fs_host *h = ctx->host;
    if (find_ahead(ctx, unique)) {
        (void)workers_wait(ctx);
        drop_ahead(ctx, unique);
    }
    fs_ahead *e = alloc_ahead(ctx, unique);
    if (!e) return set_err(ctx, FS_EINVAL, "unique ahead: too much ahead-of-time work is outstanding");
    const int x = h->x_turn;
    h->x_turn = (x + 1) % kIndexStreams;
    hipStream_t sx = ctx->stream_x[x];
    // what the dedup is ordered after: the caller's stream as it stands, or - no new event on the
    // caller's stream - its position at the start of the most recent pipelined call
    hipEvent_t after = e->fork;
    if (stream == FS_STREAM_LAST_STEP) {
        FS_REQUIRE(ctx, ctx->pfork_valid, "unique ahead: FS_STREAM_LAST_STEP before any pipelined call");
        after = ctx->ev_pfork[ctx->pipe_parity];
    } else {
        FS_HIP(ctx, hipEventRecord(e->fork, as_stream(stream)));
    }
    auto job = [=]() -> int {
        int rc = FS_OK;
        if (hipStreamWaitEvent(sx, after, 0) != hipSuccess) rc = FS_EHIP;
        if (rc == FS_OK)
            rc = launch_unique(ctx, ids, n, num_rows, unique, seg_offsets, perm, inverse, n_unique_dev, sx, 1 + x * kMaxBatch);
        if (hipEventRecord(e->done, sx) != hipSuccess && rc == FS_OK) rc = FS_EHIP;
        e->state.store(kAheadRecorded, std::memory_order_release);   // also after a failure: nobody may spin forever
        return rc;
    };
    fs_worker *w = ctx->use_worker ? get_worker(ctx, 1) : nullptr;
    if (w) {
        w->post(job);
        return FS_OK;
    }
    return job();
}

int fs_step_forward_ahead(fs_ctx *ctx, const fs_step_args *a, fs_stream stream) {
    return fs_step_forward_ahead_batch(ctx, a, 1, stream);
}

int fs_step_forward_ahead_batch(fs_ctx *ctx, const fs_step_args *a, int count, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, a && count >= 1 && count <= FS_MAX_AHEAD_BATCH, "index half ahead: batch of 1..FS_MAX_AHEAD_BATCH records");
    struct batch_state {
        fs_step_args args[kMaxBatch];
        bool have_t[kMaxBatch], have_t1[kMaxBatch];
        fs_ahead *dedup_in[kMaxBatch], *layout_in[kMaxBatch], *e_idx[kMaxBatch], *e_ded[kMaxBatch];
    } b;
    for (int k = 0; k < count; ++k) {
        const int rc = check_step_args(ctx, &a[k], &b.have_t[k], &b.have_t1[k]);
        if (rc != FS_OK) return rc;
        b.args[k] = a[k];
        b.dedup_in[k] = b.layout_in[k] = b.e_idx[k] = b.e_ded[k] = nullptr;
    }
    FS_REQUIRE(ctx, !ctx->capturing, "index half ahead: not while a graph is being captured");
    if (stream == FS_STREAM_LAST_STEP)
        FS_REQUIRE(ctx, ctx->pfork_valid, "index half ahead: FS_STREAM_LAST_STEP before any pipelined call");
    fs_host *h = ctx->host;
    for (int k = 0; k < count; ++k)
        if (find_ahead(ctx, a[k].counts_dev)) {
            (void)workers_wait(ctx);
            drop_ahead(ctx, a[k].counts_dev);
        }
    // the dedup of a lookahead batch may already be under way (fs_unique_ids_ahead); the layout of a
    // batch t may still be in the making (index half of t-1 on the other index stream) unless an earlier
    // record of this very batch produces it
    bool failed = false;
    for (int k = 0; k < count && !failed; ++k) {
        bool internal = false;
        for (int q = 0; q < k; ++q) internal = internal || (b.have_t1[q] && a[q].u_t1 == a[k].u_t);
        b.dedup_in[k] = b.have_t1[k] ? claim_ahead(ctx, a[k].u_t1) : nullptr;
        b.layout_in[k] = (b.have_t[k] && !internal) ? claim_ahead(ctx, a[k].u_t) : nullptr;
    }
    for (int k = 0; k < count && !failed; ++k) {
        // a layout that a later record of this batch splits needs no entry of its own: nobody else waits
        // for it before that record's index half is done
        bool wanted = b.have_t1[k];
        for (int q = k + 1; q < count; ++q) wanted = wanted && a[q].u_t != a[k].u_t1;
        b.e_idx[k] = alloc_ahead(ctx, a[k].counts_dev);
        b.e_ded[k] = (b.e_idx[k] && wanted) ? alloc_ahead(ctx, a[k].u_t1) : nullptr;
        failed = !b.e_idx[k] || (wanted && !b.e_ded[k]);
    }
    if (failed) {
        // the claimed entries still have to be waited for by somebody: let the index streams do it
        for (int k = 0; k < count; ++k) {
            if (b.dedup_in[k]) (void)consume_ahead(ctx, b.dedup_in[k], ctx->stream_x[0]);
            if (b.layout_in[k]) (void)consume_ahead(ctx, b.layout_in[k], ctx->stream_x[0]);
            fs_ahead *mine[2] = {b.e_idx[k], b.e_ded[k]};
            for (fs_ahead *e : mine)
                if (e) { e->key = nullptr; e->state.store(kAheadFree, std::memory_order_release); }
        }
        return set_err(ctx, FS_EINVAL, "index half ahead: too much ahead-of-time work is outstanding");
    }
    const int x = h->x_turn;
    h->x_turn = (x + 1) % kIndexStreams;
    hipStream_t sx = ctx->stream_x[x];
    hipEvent_t after = b.e_idx[0]->fork;
    if (stream == FS_STREAM_LAST_STEP) after = ctx->ev_pfork[ctx->pipe_parity];
    else FS_HIP(ctx, hipEventRecord(b.e_idx[0]->fork, as_stream(stream)));
    auto job = [=]() -> int {
        int jrc = FS_OK;
        if (hipStreamWaitEvent(sx, after, 0) != hipSuccess) jrc = FS_EHIP;
        const int irc = enqueue_index_work_batch(ctx, count, b.args, b.have_t, b.have_t1, b.dedup_in, sx,
                                                 1 + x * kMaxBatch, b.e_ded, b.layout_in);
        if (jrc == FS_OK) jrc = irc;
        for (int k = 0; k < count; ++k) {
            fs_ahead *e = b.e_ded[k];
            if (e && e->state.load(std::memory_order_acquire) != kAheadRecorded) {
                (void)hipEventRecord(e->done, sx);            // only after an early failure: nobody may spin forever
                e->state.store(kAheadRecorded, std::memory_order_release);
            }
        }
        for (int k = 0; k < count; ++k) {
            if (hipEventRecord(b.e_idx[k]->done, sx) != hipSuccess && jrc == FS_OK) jrc = FS_EHIP;
            b.e_idx[k]->state.store(kAheadRecorded, std::memory_order_release);
        }
        return jrc;
    };
    fs_worker *w = ctx->use_worker ? get_worker(ctx, 1) : nullptr;
    if (w) {
        w->post(job);
        return FS_OK;
    }
    return job();
}

int fs_step_forward(fs_ctx *ctx, const fs_step_args *a, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    bool have_t, have_t1;
    int rc = check_step_args(ctx, a, &have_t, &have_t1);
    if (rc != FS_OK) return rc;
    hipStream_t sp = as_stream(stream), sa = ctx->stream_a;
    rc = join_pending_work(ctx, sp);
    if (rc != FS_OK) return rc;
    // already done ahead of time (and joined above): nothing left to do but to give the entry back
    fs_ahead *index_ahead = claim_ahead(ctx, a->counts_dev);
    fs_ahead *ahead = (!index_ahead && have_t1) ? claim_ahead(ctx, a->u_t1) : nullptr;
    FS_HIP(ctx, hipEventRecord(ctx->ev_fork, sp));
    FS_HIP(ctx, hipStreamWaitEvent(sa, ctx->ev_fork, 0));
    rc = index_ahead ? consume_ahead(ctx, index_ahead, sa) : enqueue_index_work(ctx, a, have_t, have_t1, ahead, sa);
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
    if (!ctx->stream_b) FS_HIP(ctx, hipStreamCreateWithFlags(&ctx->stream_b, hipStreamNonBlocking));
    hipStream_t sp = as_stream(stream), sa = ctx->stream_a, sb = ctx->stream_b;
    forget_fetched(ctx);
    rc = join_pending_work(ctx, sp);
    if (rc != FS_OK) return rc;
    begin_step_timing(ctx);
    fs_ahead *index_ahead = claim_ahead(ctx, a->counts_dev);
    fs_ahead *ahead = (!index_ahead && have_t1) ? claim_ahead(ctx, a->u_t1) : nullptr;
    // fork: the side streams start after whatever the caller already queued on `stream`
    FS_HIP(ctx, hipEventRecord(ctx->ev_fork, sp));
    FS_HIP(ctx, hipStreamWaitEvent(sa, ctx->ev_fork, 0));
    FS_HIP(ctx, hipStreamWaitEvent(sb, ctx->ev_fork, 0));
    rc = index_ahead ? consume_ahead(ctx, index_ahead, sa) : enqueue_index_work(ctx, a, have_t, have_t1, ahead, sa);
    if (rc != FS_OK) return rc;
    FS_HIP(ctx, hipEventRecord(ctx->ev_split, sa));
    FS_HIP(ctx, hipStreamWaitEvent(sp, ctx->ev_split, 0));
    FS_HIP(ctx, hipStreamWaitEvent(sb, ctx->ev_split, 0));
    if (have_t) {
        // priority pass: collision rows, strictly before the lookahead rows are read
        rc = enqueue_class_pass(ctx, a, 0, sp, timing_pair(ctx, FS_TIME_UPDATE_CO));
        if (rc != FS_OK) return rc;
        // deferred pass on B: exclusive rows and lookahead rows are disjoint, so it may overlap the gather
        rc = enqueue_class_pass(ctx, a, 1, sb, timing_pair(ctx, FS_TIME_UPDATE_EX));
        if (rc != FS_OK) return rc;
    }
    FS_HIP(ctx, hipEventRecord(ctx->ev_ex, sb));
    if (have_t1) {
        rc = enqueue_gather(ctx, a, sp);
        if (rc != FS_OK) return rc;
    }
    FS_HIP(ctx, hipStreamWaitEvent(sp, ctx->ev_ex, 0));
    if (ctx->timing_now) ++ctx->timing_steps;
    return FS_OK;
}

int fs_prioritized_step_pipelined(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next, fs_stream stream) {
    return fs_prioritized_step_pipelined_multi(ctx, cur, next, 1, stream);
}

static int pipelined_impl(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next, int count, fs_stream stream,
                          bool two_part);

int fs_prioritized_step_pipelined_multi(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next, int count,
                                        fs_stream stream) {
    return pipelined_impl(ctx, cur, next, count, stream, false);
}

int fs_prioritized_step_two_part_multi(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next, int count,
                                       fs_stream stream) {
    return pipelined_impl(ctx, cur, next, count, stream, true);
}

static int pipelined_impl(fs_ctx *ctx, const fs_step_args *cur, const fs_step_args *next, int count, fs_stream stream,
                          bool two_part) {
    if (!ctx) return FS_EINVAL;
    FS_REQUIRE(ctx, cur && count >= 1 && count <= FS_MAX_STEP_TABLES, "pipelined step: 1..FS_MAX_STEP_TABLES tables");
    std::shared_ptr<side_work> w = std::make_shared<side_work>();
    bool have_t1[kMaxTables];
    w->count = count;
    for (int k = 0; k < count; ++k) {
        int rc = check_step_args(ctx, &cur[k], &w->have_t[k], &have_t1[k]);
        if (rc != FS_OK) return rc;
        w->has_next[k] = next != nullptr;
        w->nxt_t[k] = w->nxt_t1[k] = false;
        if (next) {
            rc = check_step_args(ctx, &next[k], &w->nxt_t[k], &w->nxt_t1[k]);
            if (rc != FS_OK) return rc;
        }
        w->cur[k] = cur[k];
        w->next[k] = next ? next[k] : cur[k];
        w->ahead[k] = w->index_ahead[k] = nullptr;
        w->fetch_next[k] = two_part && next && w->nxt_t1[k];
        if (two_part) {
            FS_REQUIRE(ctx, !ctx->capturing, "two-part step: not while a graph is being captured");
            FS_REQUIRE(ctx, !have_t1[k] || (cur[k].co_flag_t1 && cur[k].inverse_t1),
                       "two-part step: co_flag_t1 or inverse_t1 missing");
            FS_REQUIRE(ctx, !w->fetch_next[k] || (next[k].co_flag_t1 && next[k].inverse_t1),
                       "two-part step: co_flag_t1 or inverse_t1 missing (next)");
        }
    }
    // which part of cur's lookup is left to do: the collision rows if the previous call fetched the rest
    int part[kMaxTables];
    for (int k = 0; k < count; ++k) {
        const bool fetched = two_part && have_t1[k] && ctx->fetched_emb[k] == cur[k].emb_t1 &&
                             ctx->fetched_values[k] == cur[k].values_t1 && ctx->fetched_n[k] == cur[k].n_t1;
        part[k] = fetched ? 1 : -1;
    }
    hipStream_t sp = as_stream(stream);
    begin_step_timing(ctx);
    // Side stream A still runs what the previous call left there (its deferred passes, the index halves
    // that produced the split and class order of `cur`).  It is waited for once, right before the first
    // priority pass.  Cross-stream waits are the expensive host operation here (each makes the
    // runtime flush the producer queue): two per call, whatever the number of tables - A waits for `stream`
    // as it stands at the start of the call (the gradients), `stream` waits for A's previous job.
    const bool prev_side = ctx->side_pending;
    const int pp = ctx->pipe_parity, p = pp ^ 1;            // event set of the previous / this call
    int rc = FS_OK;
    const double h0 = now_us();
    fs_worker *w0 = (!ctx->capturing && ctx->use_worker) ? get_worker(ctx, 0) : nullptr;
    if (ctx->host->worker[0]) {
        rc = ctx->host->worker[0]->wait();                   // host side only: the previous job is enqueued
        if (rc != FS_OK) return set_err(ctx, rc, "side-stream enqueue of the previous call failed");
    }
    if (ctx->host->worker[1]) {
        // Ahead-of-time jobs posted before the PREVIOUS pipelined call may refer to the fork event that is
        // recorded again below (FS_STREAM_LAST_STEP): their waits must be on their streams by now.  Jobs
        // posted since then refer to the other event of the pair and are left alone.
        rc = ctx->host->worker[1]->wait_for(ctx->host->x_posted_before_call[pp]);
        if (rc != FS_OK) return set_err(ctx, rc, "index-stream enqueue failed");
        ctx->host->x_posted_before_call[p] = ctx->host->worker[1]->posted_so_far();
    }
    const double h1 = now_us();
    if (!ctx->capturing) {
        // index halves of `cur` done ahead of time and not yet waited for by anybody (first call of a
        // run): the caller's stream waits for them, and through the fork event so does the side stream
        for (int k = 0; k < count; ++k) {
            fs_ahead *index_cur = claim_ahead(ctx, cur[k].counts_dev);
            if (index_cur) {
                rc = consume_ahead(ctx, index_cur, sp);
                if (rc != FS_OK) return rc;
            }
        }
    }
    FS_HIP(ctx, hipEventRecord(ctx->ev_pfork[p], sp));
    ctx->pfork_valid = true;
    // claimed entries: the side job waits for them and gives them back
    if (next && !ctx->capturing)
        for (int k = 0; k < count; ++k) {
            w->index_ahead[k] = claim_ahead(ctx, next[k].counts_dev);
            w->ahead[k] = (w->nxt_t1[k] && !w->index_ahead[k]) ? claim_ahead(ctx, next[k].u_t1) : nullptr;
        }
    w->parity = p;
    w->ex_timing = timing_pair(ctx, FS_TIME_UPDATE_EX);
    auto side_job = [ctx, w]() -> int { return enqueue_side_stream(ctx, *w); };
    if (w0) w0->post(side_job);
    const double h2 = now_us();
    rc = FS_OK;
    if (prev_side && hipStreamWaitEvent(sp, ctx->ev_side[pp], 0) != hipSuccess) rc = FS_EHIP;
    ctx->side_pending = false;
    const double h3 = now_us();
    // every priority pass before every gather: a gather may only read what its table's priority pass left
    if (rc == FS_OK) rc = enqueue_class_passes(ctx, cur, w->have_t, count, 0, sp, timing_pair(ctx, FS_TIME_UPDATE_CO));
    if (rc == FS_OK) rc = enqueue_gathers(ctx, cur, have_t1, count, sp, part);
    const double h4 = now_us();
    if (!w0) {
        const int src = side_job();
        if (rc == FS_OK) rc = src;
    }
    if (ctx->timing_now) ++ctx->timing_steps;
    ctx->host_us[0] += h1 - h0;      // waiting for the side-stream thread
    ctx->host_us[1] += h2 - h1;      // fork event, handing over the side work
    ctx->host_us[2] += h3 - h2;      // wait for the previous side work
    ctx->host_us[3] += h4 - h3;      // priority passes and gathers
    ctx->host_us[6] += 1.0;
    ctx->pipe_parity = p;
    ctx->side_pending = true;        // also after a failure: a posted job still records its event
    for (int k = 0; k < kMaxTables; ++k) {
        const bool f = rc == FS_OK && k < count && w->fetch_next[k];
        ctx->fetched_emb[k] = f ? next[k].emb_t1 : nullptr;
        ctx->fetched_values[k] = f ? next[k].values_t1 : nullptr;
        ctx->fetched_n[k] = f ? next[k].n_t1 : 0;
    }
    // a captured graph must end with every stream joined
    if (ctx->capturing && rc == FS_OK) rc = join_pending_work(ctx, sp);
    return rc;
}

int fs_two_part_forget(fs_ctx *ctx) {
    if (!ctx) return FS_EINVAL;
    forget_fetched(ctx);
    return FS_OK;
}

int fs_step_join(fs_ctx *ctx, fs_stream stream) {
    if (!ctx) return FS_EINVAL;
    return join_pending_work(ctx, as_stream(stream));
}

#ifdef FS_TRACE
// Diagnostic builds only: `buf_dev` = zeroed device array of 64-bit words with [1] = records per lane
// (layout beside the tracer in fs_device.h); nullptr switches the trace off.
void fs_set_trace_unique(unsigned long long *);
void fs_set_trace_split(unsigned long long *);
void fs_set_trace_gather(unsigned long long *);
void fs_set_trace_fused(unsigned long long *);
int fs_debug_trace(fs_ctx *ctx, void *buf_dev) {
    if (!ctx) return FS_EINVAL;
    FS_HIP(ctx, hipDeviceSynchronize());
    fs_set_trace_unique((unsigned long long *)buf_dev);
    fs_set_trace_split((unsigned long long *)buf_dev);
    fs_set_trace_gather((unsigned long long *)buf_dev);
    fs_set_trace_fused((unsigned long long *)buf_dev);
    FS_HIP(ctx, hipDeviceSynchronize());
    return FS_OK;
}
#endif

int fs_ctx_host_times(fs_ctx *ctx, double *out7_host, int reset) {
    if (!ctx || !out7_host) return FS_EINVAL;
    (void)workers_wait(ctx);
    for (int k = 0; k < 2; ++k) {
        fs_worker *w = ctx->host->worker[k];
        if (!w) continue;
        std::lock_guard<std::mutex> lk(w->mu);
        ctx->host_us[k == 0 ? 5 : 4] = w->busy_us;
        if (reset) w->busy_us = 0.0;
    }
    for (int i = 0; i < 7; ++i) out7_host[i] = ctx->host_us[i];
    if (reset)
        for (int i = 0; i < 7; ++i) ctx->host_us[i] = 0.0;
    return FS_OK;
}

int fs_ctx_set_threaded_enqueue(fs_ctx *ctx, int on) {
    if (!ctx) return FS_EINVAL;
    (void)workers_wait(ctx);
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
    // nothing from outside may leak into the capture
    (void)workers_wait(ctx);
    ctx->side_pending = false;
    (void)hipStreamSynchronize(ctx->stream_a);
    for (hipStream_t sx : ctx->stream_x) (void)hipStreamSynchronize(sx);
    if (!ctx->stream_cap && hipStreamCreateWithFlags(&ctx->stream_cap, hipStreamNonBlocking) != hipSuccess) {
        delete g;
        return set_err(ctx, FS_EHIP, "hipStreamCreateWithFlags(capture stream)");
    }
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
    if (ctx) forget_fetched(ctx);
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
