// split(G~^i, I~_co^i, I~_ex^i) at the start of Backward of Algorithm 2: the gradient rows of a batch arrive in
// batch order, one per occurrence, and are packed into the rows of collision occurrences and the rows of
// exclusive occurrences, each part in batch order (the collision part is what the exposed gradient AllToAll of
// Section 3.2 carries, the exclusive part travels with the deferred one).  On one shard batch-major and
// shard-major coincide, so the occurrence lists I~_co, I~_ex are occurrence numbers of the batch.
//
// Whether an occurrence is a collision occurrence is decided per distinct row (the collision split's co_slot
// list) and reaches the occurrences through the inverse map of the batch.  Four launches: row flags, collision
// occurrences per tile of 1024, the numbering (tile prefixes, block scan), the copy.  The copy reads the
// gradient rows front to back and writes two streams that only move forward: both sides stay as sequential as a
// plain copy.  A second, small entry point rewrites a class order so that the fused passes can read the packed
// parts instead of the batch-major tensor.
#include "fs_common.h"
#include "fs_device.h"

namespace fs {

__device__ __forceinline__ int clamp_i64(const int64_t *dev, int64_t cap) {
    int64_t v = dev ? *dev : 0;
    if (v < 0) v = 0;
    if (v > cap) v = cap;
    return (int)v;
}

// flag[slot] = 1 iff slot is in the ascending list co_slot[0, n_co)
__global__ __launch_bounds__(256) void gs_row_flag_kernel(const int32_t *__restrict__ co_slot,
                                                          const int64_t *__restrict__ n_co_dev, int cap,
                                                          uint8_t *__restrict__ flag) {
    const int n_co = clamp_i64(n_co_dev, cap);
    const int slot = blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= cap) return;
    int lo = 0, hi = n_co;                                   // first index with co_slot[i] >= slot
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (co_slot[mid] < slot) lo = mid + 1; else hi = mid;
    }
    flag[slot] = (lo < n_co && co_slot[lo] == slot) ? 1 : 0;
}

__device__ __forceinline__ bool occurrence_is_co(const int32_t *__restrict__ inverse, const uint8_t *__restrict__ flag,
                                                 int j, int cap, bool &bad) {
    const int s = inverse[j];
    if ((unsigned)s >= (unsigned)cap) { bad = true; return false; }
    return flag[s] != 0;
}

__global__ __launch_bounds__(kScanThreads) void gs_count_kernel(const int32_t *__restrict__ inverse,
                                                                const uint8_t *__restrict__ flag, int n, int cap,
                                                                int32_t *__restrict__ tile_cnt, int *__restrict__ flags) {
    __shared__ int sh[kScanThreads / kWave];
    const int p0 = blockIdx.x * kScanTile + threadIdx.x * kScanIpt;
    int c = 0;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i)
        if (p0 + i < n) c += occurrence_is_co(inverse, flag, p0 + i, cap, bad) ? 1 : 0;
    int total;
    (void)block_exclusive_scan<int>(c, sh, total);
    if (threadIdx.x == 0) tile_cnt[blockIdx.x] = total;
    if (bad) atomicOr(flags, kFlagInternal);
}

// part_pos[j]: a collision occurrence's number in the collision part; for an exclusive occurrence -1 - its number
// in the exclusive part
__global__ __launch_bounds__(kScanThreads) void gs_number_kernel(const int32_t *__restrict__ inverse,
                                                                 const uint8_t *__restrict__ flag, int n, int cap,
                                                                 const int32_t *__restrict__ tile_cnt, int tiles,
                                                                 int32_t *__restrict__ co_index,
                                                                 int32_t *__restrict__ ex_index,
                                                                 int32_t *__restrict__ part_pos,
                                                                 int64_t *__restrict__ counts_dev) {
    __shared__ int sh[kScanThreads / kWave];
    int before = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += kScanThreads) before += tile_cnt[t];
    int co_before;
    (void)block_exclusive_scan<int>(before, sh, co_before);
    const int p0 = blockIdx.x * kScanTile + threadIdx.x * kScanIpt;
    bool f[kScanIpt], bad = false;
    int c = 0;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        f[i] = (p0 + i < n) && occurrence_is_co(inverse, flag, p0 + i, cap, bad);
        c += f[i] ? 1 : 0;
    }
    int tile_total;
    int r_co = co_before + block_exclusive_scan<int>(c, sh, tile_total);     // collision occurrences before p0
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        const int j = p0 + i;
        if (j < n) {
            if (f[i]) { co_index[r_co] = j; part_pos[j] = r_co; }
            else { ex_index[j - r_co] = j; part_pos[j] = -1 - (j - r_co); }
            r_co += f[i] ? 1 : 0;
        }
    }
    if ((int)blockIdx.x == tiles - 1 && threadIdx.x == 0) {
        const int n_co = co_before + tile_total;
        counts_dev[0] = n_co;
        counts_dev[1] = n - n_co;
    }
}

__global__ void gs_empty_kernel(int64_t *counts_dev) {
    counts_dev[0] = 0;
    counts_dev[1] = 0;
}

template <int LPR, int UNR>
__global__ __launch_bounds__(256) void gs_copy_kernel(const u32x4 *__restrict__ grads, int n, int gvec,
                                                      const int32_t *__restrict__ part_pos, u32x4 *__restrict__ g_co,
                                                      u32x4 *__restrict__ g_ex) {
    constexpr int GPW = kWave / LPR;
    constexpr int ROWS_PER_WAVE = GPW * UNR;
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int64_t waves = (int64_t)gridDim.x * (blockDim.x / kWave);
    for (int64_t j0 = wave * ROWS_PER_WAVE; j0 < n; j0 += waves * ROWS_PER_WAVE) {
        int pos[UNR];
        bool live[UNR];
        u32x4 v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t j = j0 + u * GPW + grp;
            live[u] = (j < n) && (lig < gvec);
            pos[u] = live[u] ? part_pos[j] : 0;
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (live[u]) v[u] = __builtin_nontemporal_load(&grads[j * gvec + lig]);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
            if (live[u]) {
                const bool co = pos[u] >= 0;
                const int64_t r = co ? pos[u] : -1 - pos[u];
                store_streaming(v[u], (co ? g_co : g_ex) + r * gvec + lig);
            }
    }
}

int launch_split_grads(fs_ctx *ctx, const float *grads, int64_t n, int32_t dim, const int32_t *inverse,
                       const int32_t *co_slot, const int64_t *n_co_dev, int64_t cap_u, int32_t *co_index, float *g_co,
                       int32_t *ex_index, float *g_ex, int32_t *part_pos, int64_t *counts_dev, hipStream_t s) {
    if (n == 0) {
        hipLaunchKernelGGL(gs_empty_kernel, dim3(1), dim3(1), 0, s, counts_dev);
        FS_LAUNCH_CHECK(ctx, "gs_empty_kernel");
        return FS_OK;
    }
    const fs_split_scratch &ws = ctx->split[0];
    const int tiles = (int)ceil_div(n, kScanTile);
    hipLaunchKernelGGL(gs_row_flag_kernel, dim3((unsigned)ceil_div(cap_u, 256)), dim3(256), 0, s, co_slot, n_co_dev,
                       (int)cap_u, ws.flag_t);
    hipLaunchKernelGGL(gs_count_kernel, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, inverse, ws.flag_t, (int)n,
                       (int)cap_u, ws.cnt, ctx->d_flags);
    hipLaunchKernelGGL(gs_number_kernel, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, inverse, ws.flag_t, (int)n,
                       (int)cap_u, ws.cnt, tiles, co_index, ex_index, part_pos, counts_dev);
    const int gvec = dim / 4;
#define FS_CASE(L)                                                                                                 \
    case L: {                                                                                                      \
        constexpr int UNR = 4;                                                                                     \
        const int64_t blocks = ceil_div(n, (int64_t)(kWave / L) * UNR * 4);                                        \
        hipLaunchKernelGGL((gs_copy_kernel<L, UNR>), dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), \
                           0, s, (const u32x4 *)grads, (int)n, gvec, part_pos, (u32x4 *)g_co, (u32x4 *)g_ex);      \
        break;                                                                                                     \
    }
    switch (lanes_per_row(gvec)) {
        FS_CASE(1) FS_CASE(2) FS_CASE(4) FS_CASE(8) FS_CASE(16) FS_CASE(32) FS_CASE(64)
        default: return set_err(ctx, FS_EINVAL, "split grads: dim beyond 256");
    }
#undef FS_CASE
    FS_LAUNCH_CHECK(ctx, "split grads kernels");
    return FS_OK;
}

// ---- a class order that addresses the packed parts ---------------------------------------------------------------
// The class order and the records of a batch name occurrences (rows of the batch-major gradient tensor).  Rewritten
// through part_pos they name rows of the packed parts instead: class 0 (collision rows) reads g_co, class 1 g_ex.
__device__ __forceinline__ int part_row(int pos) { return pos >= 0 ? pos : -1 - pos; }

__global__ __launch_bounds__(256) void gs_remap_cperm_kernel(const int32_t *__restrict__ cperm,
                                                             const int32_t *__restrict__ class_pos, int n,
                                                             const int32_t *__restrict__ part_pos,
                                                             int32_t *__restrict__ cperm_parts, int *__restrict__ flags) {
    int n_pos = class_pos[1];
    if (n_pos > n) n_pos = n;
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n_pos) return;
    const int j = cperm[p];
    if ((unsigned)j >= (unsigned)n) { atomicOr(flags, kFlagInternal); cperm_parts[p] = 0; return; }
    const int pos = part_pos[j];
    // a position of class 0 must lie in the collision part, one of class 1 in the exclusive part
    if ((pos >= 0) != (p < class_pos[0])) atomicOr(flags, kFlagInternal);
    cperm_parts[p] = part_row(pos);
}

__global__ __launch_bounds__(256) void gs_remap_records_kernel(const int32_t *__restrict__ recs,
                                                               const int64_t *__restrict__ counts_dev, int cap, int n,
                                                               const int32_t *__restrict__ part_pos,
                                                               int32_t *__restrict__ recs_parts, int *__restrict__ flags) {
    const int cls = blockIdx.y;
    const int n_rows = clamp_i64(counts_dev + cls, cap);
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    const int32_t *src = recs + ((int64_t)cls * cap + i) * kShortRecInts;
    int32_t *dst = recs_parts + ((int64_t)cls * cap + i) * kShortRecInts;
    int w[kShortRecInts];
#pragma unroll
    for (int q = 0; q < kShortRecInts; ++q) w[q] = src[q];
    const int len = w[3];
    if (len >= 1 && len <= FS_SHORT_SEGMENT) {
#pragma unroll
        for (int q = 0; q < FS_SHORT_SEGMENT; ++q)
            if (q < len) {
                const int j = w[4 + q];
                if ((unsigned)j >= (unsigned)n) { atomicOr(flags, kFlagInternal); w[4 + q] = 0; continue; }
                const int pos = part_pos[j];
                if ((pos >= 0) != (cls == 0)) atomicOr(flags, kFlagInternal);
                w[4 + q] = part_row(pos);
            }
    }
#pragma unroll
    for (int q = 0; q < kShortRecInts; ++q) dst[q] = w[q];
}

int launch_class_order_for_parts(fs_ctx *ctx, const int32_t *part_pos, int64_t n, int64_t cap_u, const int32_t *cperm,
                                 const int32_t *class_pos_dev, const int32_t *short_rec, const int64_t *counts_dev,
                                 int32_t *cperm_parts, int32_t *short_rec_parts, hipStream_t s) {
    if (n == 0) return FS_OK;
    hipLaunchKernelGGL(gs_remap_cperm_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, cperm, class_pos_dev,
                       (int)n, part_pos, cperm_parts, ctx->d_flags);
    hipLaunchKernelGGL(gs_remap_records_kernel, dim3((unsigned)ceil_div(cap_u, 256), 2u), dim3(256), 0, s, short_rec,
                       counts_dev, (int)cap_u, (int)n, part_pos, short_rec_parts, ctx->d_flags);
    FS_LAUNCH_CHECK(ctx, "class order for parts");
    return FS_OK;
}

}  // namespace fs
