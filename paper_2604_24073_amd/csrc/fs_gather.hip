// Jagged row gather (Lookup(I) of Algorithm 2) plus the two helper kernels that only move or
// generate bytes: the hash table initialiser and the plain stream copy.
//
// Gather layout: a row is `granules` 16-byte pieces.  LPR = next power of two >= granules lanes
// cover one row, so one wavefront instruction moves 64/LPR rows (2 rows of 128 fp32, 4 rows of
// 64 fp32 or 128 bf16, 1 row of 256 fp32).  Work is flat over the N occurrences, never one
// workgroup per user, so a 16K-item sequence costs the same per item as a short one.
#include "fs_common.h"
#include "fs_device.h"

#ifndef FS_GATHER_UNR
#define FS_GATHER_UNR 4
#endif
#ifndef FS_PART_CHUNK
#define FS_PART_CHUNK 64
#endif
#ifndef FS_GATHER_MAX_BLOCKS
#define FS_GATHER_MAX_BLOCKS 16384
#endif

namespace fs {

// one gather of a launch shared by several tables of one row width (blockIdx.y picks the table)
struct gather_dev_job {
    const u32x4 *table;
    int64_t num_rows;
    const int64_t *values, *offsets;
    int64_t batch, n;
    u32x4 *out;
    int granules, blocks;
    const int32_t *inverse;       // gather_part_kernel: occurrence -> slot of its row in the distinct list
    const uint8_t *row_flag;      //                     slot -> 1 for a collision row
    int which;                    //                     copy the occurrences whose flag equals this
    const int64_t *sorted_ids;    // gather_rows_kernel: row at each position of the ascending list
    const int32_t *perm;          //                     occurrence at each position of the ascending list
};
struct gather_dev_batch {
    gather_dev_job j[kMaxBatch];
};

template <int LPR, int UNR>
__global__ __launch_bounds__(256) void gather_kernel(const gather_dev_batch jobs, int *__restrict__ flags) {
    const gather_dev_job &job = jobs.j[blockIdx.y];
    FS_WG_TRACE(10);
    if ((int)blockIdx.x >= job.blocks) return;
    const u32x4 *__restrict__ table = job.table;
    const int64_t num_rows = job.num_rows;
    const int granules = job.granules;
    const int64_t *__restrict__ values = job.values;
    const int64_t *__restrict__ offsets = job.offsets;
    const int64_t batch = job.batch, n = job.n;
    u32x4 *__restrict__ out = job.out;
    constexpr int GPW = kWave / LPR;                  // rows per wavefront instruction
    constexpr int ROWS_PER_WAVE = GPW * UNR;
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int64_t waves = (int64_t)job.blocks * (blockDim.x / kWave);

    // offsets validation rides along (grid-stride over the batch; almost free)
    if (offsets != nullptr) {
        const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
        const int64_t gsz = (int64_t)job.blocks * blockDim.x;
        bool bad = false;
        for (int64_t b = gtid; b < batch; b += gsz) bad |= offsets[b + 1] < offsets[b];
        if (gtid == 0) bad |= (offsets[0] != 0) || (offsets[batch] != n);
        if (bad) atomicOr(flags, kFlagOffsets);
    }
    bool oob = false;
    for (int64_t row0 = wave * ROWS_PER_WAVE; row0 < n; row0 += waves * ROWS_PER_WAVE) {
        int64_t id[UNR];
        bool live[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t j = row0 + u * GPW + grp;
            live[u] = (j < n) && (lig < granules);
            id[u] = live[u] ? values[j] : 0;
        }
        u32x4 v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const bool in = (id[u] >= 0) && (id[u] < num_rows);
            oob |= live[u] && !in;
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (live[u] && in) v[u] = table[id[u] * granules + lig];
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t j = row0 + u * GPW + grp;
            if (live[u]) store_streaming(v[u], &out[j * granules + lig]);
        }
    }
    if (oob) atomicOr(flags, kFlagRowRange);
}


// The same lookup walked in ROW order: position p of the ascending ID list (every occurrence listed) holds row
// sorted_ids[p] and belongs to occurrence perm[p] of the batch, so out[perm[p], :] = table[sorted_ids[p], :].
// All occurrences of a row are neighbours in this order - the same wavefront, or the next one - so a row comes
// from HBM once however far apart its occurrences lie in the batch (in batch order the occurrences of a row of
// middling popularity meet in no cache: measured 62 MB fetched where 41 MB are distinct rows).  The output rows
// are whole 128-byte lines either way; only their order in time changes.  Offsets are validated as in the
// batch-order kernel.
template <int LPR, int UNR>
__device__ __forceinline__ void gather_rows_body(const gather_dev_job &job, int *__restrict__ flags) {
    if ((int)blockIdx.x >= job.blocks) return;
    const u32x4 *__restrict__ table = job.table;
    const int64_t num_rows = job.num_rows;
    const int granules = job.granules;
    const int64_t *__restrict__ sorted_ids = job.sorted_ids;
    const int32_t *__restrict__ perm = job.perm;
    const int64_t *__restrict__ offsets = job.offsets;
    const int64_t batch = job.batch, n = job.n;
    u32x4 *__restrict__ out = job.out;
    constexpr int GPW = kWave / LPR;
    constexpr int ROWS_PER_WAVE = GPW * UNR;
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int64_t waves = (int64_t)job.blocks * (blockDim.x / kWave);
    if (offsets != nullptr) {
        const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
        const int64_t gsz = (int64_t)job.blocks * blockDim.x;
        bool bad = false;
        for (int64_t b = gtid; b < batch; b += gsz) bad |= offsets[b + 1] < offsets[b];
        if (gtid == 0) bad |= (offsets[0] != 0) || (offsets[batch] != n);
        if (bad) atomicOr(flags, kFlagOffsets);
    }
    bool oob = false, bad_perm = false;
    for (int64_t p0 = wave * ROWS_PER_WAVE; p0 < n; p0 += waves * ROWS_PER_WAVE) {
        int64_t id[UNR];
        int32_t dst[UNR];
        bool live[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t p = p0 + u * GPW + grp;
            live[u] = (p < n) && (lig < granules);
            id[u] = live[u] ? sorted_ids[p] : 0;
            dst[u] = live[u] ? perm[p] : 0;
        }
        u32x4 v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const bool in = (id[u] >= 0) && (id[u] < num_rows);
            const bool dst_ok = (unsigned)dst[u] < (unsigned)n;     // a consistent layout never trips this
            oob |= live[u] && !in;
            bad_perm |= live[u] && !dst_ok;
            live[u] = live[u] && dst_ok;
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (live[u] && in) v[u] = table[id[u] * granules + lig];
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
            if (live[u]) store_streaming(v[u], &out[(int64_t)dst[u] * granules + lig]);
    }
    if (oob) atomicOr(flags, kFlagRowRange);
    if (bad_perm) atomicOr(flags, kFlagInternal);
}

template <int LPR, int UNR>
__global__ __launch_bounds__(256) void gather_rows_kernel(const gather_dev_batch jobs, int *__restrict__ flags) {
    FS_WG_TRACE(10);
    gather_rows_body<LPR, UNR>(jobs.j[blockIdx.y], flags);
}


// One part of the two-part lookup of Algorithm 2 (the rows Forward fetches ahead of time, or the collision
// rows the priority update of Backward returns): only the occurrences whose row flag equals `which` are
// copied, the output rows of the others are left alone.  A wavefront takes FS_PART_CHUNK consecutive occurrences, one
// per lane and round (coalesced reads of the IDs, the inverse map and the byte flags), squeezes the ones
// of its part into a list in LDS and then copies rows from that list exactly as the plain kernel does -
// the row traffic stays as dense as if the other part did not exist.
constexpr int kPartChunk = FS_PART_CHUNK;
template <int LPR, int UNR>
__global__ __launch_bounds__(256) void gather_part_kernel(const gather_dev_batch jobs, int *__restrict__ flags) {
    const gather_dev_job &job = jobs.j[blockIdx.y];
    FS_WG_TRACE(10);
    if ((int)blockIdx.x >= job.blocks) return;
    const u32x4 *__restrict__ table = job.table;
    const int64_t num_rows = job.num_rows;
    const int granules = job.granules;
    const int64_t *__restrict__ values = job.values;
    const int64_t *__restrict__ offsets = job.offsets;
    const int32_t *__restrict__ inverse = job.inverse;
    const uint8_t *__restrict__ row_flag = job.row_flag;
    const bool want = job.which != 0;
    const int64_t batch = job.batch, n = job.n;
    u32x4 *__restrict__ out = job.out;
    constexpr int GPW = kWave / LPR;
    constexpr int ROWS_PER_WAVE = GPW * UNR;
    constexpr int WAVES = 256 / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    __shared__ int64_t l_id[WAVES][kPartChunk];
    __shared__ int32_t l_pos[WAVES][kPartChunk];

    if (offsets != nullptr) {
        const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
        const int64_t gsz = (int64_t)job.blocks * blockDim.x;
        bool bad = false;
        for (int64_t b = gtid; b < batch; b += gsz) bad |= offsets[b + 1] < offsets[b];
        if (gtid == 0) bad |= (offsets[0] != 0) || (offsets[batch] != n);
        if (bad) atomicOr(flags, kFlagOffsets);
    }
    bool oob = false;
    const uint64_t lt = (1ull << lane) - 1ull;
    const int64_t chunks = (n + kPartChunk - 1) / kPartChunk;
    // every wavefront of the workgroup makes the same number of rounds (the barriers below are met by all)
    for (int64_t c0 = (int64_t)blockIdx.x * WAVES; c0 < chunks; c0 += (int64_t)job.blocks * WAVES) {
        const int64_t base = (c0 + w) * kPartChunk;
        int count = 0;
#pragma unroll
        for (int q = 0; q < kPartChunk / kWave; ++q) {
            const int64_t j = base + q * kWave + lane;
            int64_t id = 0;
            bool mine = false;
            if (j < n) {
                id = values[j];
                mine = (row_flag[inverse[j]] != 0) == want;
            }
            const uint64_t m = __ballot(mine);
            if (mine) {
                const int at = count + __popcll(m & lt);
                l_id[w][at] = id;
                l_pos[w][at] = (int32_t)j;
            }
            count += __popcll(m);
        }
        __syncthreads();
        for (int r0 = 0; r0 < count; r0 += ROWS_PER_WAVE) {
            int64_t id[UNR];
            int32_t pos[UNR];
            bool live[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int k = r0 + u * GPW + grp;
                live[u] = (k < count) && (lig < granules);
                id[u] = live[u] ? l_id[w][k] : 0;
                pos[u] = live[u] ? l_pos[w][k] : 0;
            }
            u32x4 v[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const bool in = (id[u] >= 0) && (id[u] < num_rows);
                oob |= live[u] && !in;
                v[u] = u32x4{0u, 0u, 0u, 0u};
                if (live[u] && in) v[u] = table[id[u] * granules + lig];
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                if (live[u]) store_streaming(v[u], &out[(int64_t)pos[u] * granules + lig]);
        }
        __syncthreads();
    }
    if (oob) atomicOr(flags, kFlagRowRange);
}

template <int LPR>
static void gather_launch(const fs_gather_job *jobs, const int *idx, int m, bool part, bool rows, int *flags,
                          hipStream_t s) {
    // One round of rows per workgroup when the cap allows: the chip writes faster the more workgroups share
    // the job (a write-only kernel: 4.6 TB/s from 1024 workgroups, 5.8 TB/s from 65536), and the small
    // latency-bound kernels that used to queue behind a long grid now run iterations ahead of it.
    constexpr int UNR = FS_GATHER_UNR;
    const int ROWS_PER_BLOCK = part ? 4 * kPartChunk : (kWave / LPR) * UNR * 4;
    for (int at = 0; at < m; at += kMaxBatch) {
        const int k = (m - at) < kMaxBatch ? (m - at) : kMaxBatch;
        gather_dev_batch batch;
        memset(&batch, 0, sizeof(batch));
        // the tables of a launch share the chip: FS_GATHER_MAX_BLOCKS workgroups in all, by their sizes
        int64_t total = 0;
        for (int i = 0; i < k; ++i) total += jobs[idx[at + i]].n;
        int blocks = 0;
        for (int i = 0; i < k; ++i) {
            const fs_gather_job &in = jobs[idx[at + i]];
            gather_dev_job &j = batch.j[i];
            int64_t b = ceil_div(in.n, ROWS_PER_BLOCK);
            int64_t share = ceil_div((int64_t)FS_GATHER_MAX_BLOCKS * in.n, total);
            if (share < 1) share = 1;
            if (b > share) b = share;
            j.table = (const u32x4 *)in.table; j.num_rows = in.num_rows; j.values = in.values; j.offsets = in.offsets;
            j.batch = in.batch; j.n = in.n; j.out = (u32x4 *)in.out; j.granules = in.row_bytes / 16; j.blocks = (int)b;
            j.inverse = in.inverse; j.row_flag = in.row_flag; j.which = in.which;
            j.sorted_ids = in.sorted_ids; j.perm = in.perm;
            blocks = j.blocks > blocks ? j.blocks : blocks;
        }
        if (part)
            hipLaunchKernelGGL((gather_part_kernel<LPR, UNR>), dim3((unsigned)blocks, (unsigned)k), dim3(256), 0, s, batch, flags);
        else if (rows)
            hipLaunchKernelGGL((gather_rows_kernel<LPR, UNR>), dim3((unsigned)blocks, (unsigned)k), dim3(256), 0, s, batch, flags);
        else
            hipLaunchKernelGGL((gather_kernel<LPR, UNR>), dim3((unsigned)blocks, (unsigned)k), dim3(256), 0, s, batch, flags);
    }
}

static bool is_part(const fs_gather_job &j) { return j.which >= 0 && j.inverse != nullptr && j.row_flag != nullptr; }
static bool is_rows(const fs_gather_job &j) { return !is_part(j) && j.sorted_ids != nullptr && j.perm != nullptr; }

int launch_gather_batch(fs_ctx *ctx, int count, const fs_gather_job *jobs, hipStream_t s) {
    bool done[FS_MAX_STEP_TABLES];
    if (count < 0 || count > FS_MAX_STEP_TABLES) return set_err(ctx, FS_EINVAL, "gather: too many tables");
    for (int k = 0; k < count; ++k) done[k] = jobs[k].n == 0;
    for (int k0 = 0; k0 < count; ++k0) {
        if (done[k0]) continue;
        const int lpr = lanes_per_row(jobs[k0].row_bytes / 16);
        const bool part = is_part(jobs[k0]), rows = is_rows(jobs[k0]);
        int idx[FS_MAX_STEP_TABLES], m = 0;
        for (int k = k0; k < count; ++k)
            if (!done[k] && lanes_per_row(jobs[k].row_bytes / 16) == lpr && is_part(jobs[k]) == part &&
                is_rows(jobs[k]) == rows) {
                idx[m++] = k;
                done[k] = true;
            }
        switch (lpr) {
            case 1: gather_launch<1>(jobs, idx, m, part, rows, ctx->d_flags, s); break;
            case 2: gather_launch<2>(jobs, idx, m, part, rows, ctx->d_flags, s); break;
            case 4: gather_launch<4>(jobs, idx, m, part, rows, ctx->d_flags, s); break;
            case 8: gather_launch<8>(jobs, idx, m, part, rows, ctx->d_flags, s); break;
            case 16: gather_launch<16>(jobs, idx, m, part, rows, ctx->d_flags, s); break;
            case 32: gather_launch<32>(jobs, idx, m, part, rows, ctx->d_flags, s); break;
            case 64: gather_launch<64>(jobs, idx, m, part, rows, ctx->d_flags, s); break;
            default: return set_err(ctx, FS_EINVAL, "gather: row wider than 1024 bytes");
        }
    }
    FS_LAUNCH_CHECK(ctx, "gather_kernel");
    return FS_OK;
}

int launch_gather(fs_ctx *ctx, const void *table, int64_t num_rows, int row_bytes, const int64_t *values,
                  const int64_t *offsets, int64_t batch, int64_t n, void *out, hipStream_t s) {
    fs_gather_job job;
    job.table = table; job.num_rows = num_rows; job.row_bytes = row_bytes; job.values = values; job.offsets = offsets;
    job.batch = batch; job.n = n; job.out = out;
    return launch_gather_batch(ctx, 1, &job, s);
}

// ---- hash initialiser (input generator; mirrors the rule of the synthetic workloads) --------
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

__device__ __forceinline__ uint32_t elem_hash(uint64_t e) {
    return mix32((uint32_t)e ^ mix32((uint32_t)(e >> 32) + 0x9E3779B9u));
}

__global__ __launch_bounds__(256) void init_hash_f32_kernel(f32x4 *__restrict__ table, int64_t n_vec) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
        const uint64_t e = (uint64_t)i * 4;
        f32x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            v[c] = (float)((int)(elem_hash(e + c) & 0xFFFFu) - 32768) * 0x1p-22f;
        __builtin_nontemporal_store(v, &table[i]);
    }
}

__global__ __launch_bounds__(256) void init_hash_bf16_kernel(u32x4 *__restrict__ table, int64_t n_vec) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
        const uint64_t e = (uint64_t)i * 8;
        u32x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            // values are exact in bf16 (8 significant bits): the high half of the fp32 pattern
            const float lo = (float)((int)(elem_hash(e + 2 * c) & 0xFFu) - 128) * 0x1p-14f;
            const float hi = (float)((int)(elem_hash(e + 2 * c + 1) & 0xFFu) - 128) * 0x1p-14f;
            v[c] = (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
        }
        __builtin_nontemporal_store(v, &table[i]);
    }
}

int launch_init_hash(fs_ctx *ctx, void *table, int64_t num_rows, int32_t dim, int dt, hipStream_t s) {
    const int64_t elems = num_rows * (int64_t)dim;
    if (elems == 0) return FS_OK;
    const int64_t n_vec = elems / (dt == FS_F32 ? 4 : 8);
    const int64_t blocks = ceil_div(n_vec, 256) < 16384 ? ceil_div(n_vec, 256) : 16384;
    if (dt == FS_F32)
        hipLaunchKernelGGL(init_hash_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (f32x4 *)table, n_vec);
    else
        hipLaunchKernelGGL(init_hash_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (u32x4 *)table, n_vec);
    FS_LAUNCH_CHECK(ctx, "init_hash_kernel");
    return FS_OK;
}

// ---- plain copy (bandwidth calibration) -------------------------------------------------------
__global__ __launch_bounds__(256) void copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n_vec) {
    const int64_t base = ((int64_t)blockIdx.x * blockDim.x) * 4 + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t i = base + (int64_t)u * blockDim.x;
        if (i < n_vec) v[u] = __builtin_nontemporal_load(&src[i]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t i = base + (int64_t)u * blockDim.x;
        if (i < n_vec) __builtin_nontemporal_store(v[u], &dst[i]);
    }
}

int launch_copy(fs_ctx *ctx, const void *src, void *dst, int64_t n_bytes, hipStream_t s) {
    const int64_t n_vec = n_bytes / 16;
    if (n_vec == 0) return FS_OK;
    const int64_t blocks = ceil_div(n_vec, 1024);
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const u32x4 *)src, (u32x4 *)dst, n_vec);
    FS_LAUNCH_CHECK(ctx, "copy_kernel");
    return FS_OK;
}

// ---- rows read and thrown away (bandwidth calibration) ----------------------------------------------------
// What the memory system gives the access pattern of the step - whole rows at addresses that follow an index
// list - with nothing else in the way: a wavefront takes 64 consecutive entries of `index`, requests the rows in
// rounds of UNR row groups exactly as the position-cut pass does, and folds them into one word per wavefront.
template <int LPR, int UNR>
__global__ __launch_bounds__(256) void row_read_kernel(const u32x4 *__restrict__ rows, int64_t num_rows, int granules,
                                                       const int64_t *__restrict__ index, int64_t n,
                                                       uint32_t *__restrict__ sink) {
    constexpr int GPW = kWave / LPR;
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int64_t a = wave * kWave;
    if (a >= n) return;
    const int span = (int)((n - a) < kWave ? (n - a) : kWave);
    int64_t id = lane < span ? index[a + lane] : 0;
    if (id < 0 || id >= num_rows) id = 0;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int k = 0; k * GPW * UNR < span; ++k) {
        u32x4 v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int q = k * GPW * UNR + u * GPW + grp;
            const int64_t r = __shfl(id, q & (kWave - 1), kWave);
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (q < span && lig < granules) v[u] = __builtin_nontemporal_load(&rows[r * granules + lig]);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) acc ^= v[u];
    }
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) x ^= __shfl_xor(x, m, kWave);
    if (lane == 0) sink[wave & 1023] = x;
}

int launch_row_read(fs_ctx *ctx, const void *rows, int64_t num_rows, int row_bytes, const int64_t *index, int64_t n,
                    uint32_t *sink, hipStream_t s) {
    if (n == 0) return FS_OK;
    const int granules = row_bytes / 16;
    const unsigned blocks = (unsigned)ceil_div(n, 4 * kWave);
#define FS_CASE(L)                                                                                            \
    case L:                                                                                                   \
        hipLaunchKernelGGL((row_read_kernel<L, 4>), dim3(blocks), dim3(256), 0, s, (const u32x4 *)rows, num_rows, \
                           granules, index, n, sink);                                                         \
        break;
    switch (lanes_per_row(granules)) {
        FS_CASE(1) FS_CASE(2) FS_CASE(4) FS_CASE(8) FS_CASE(16) FS_CASE(32) FS_CASE(64)
        default: return set_err(ctx, FS_EINVAL, "row read: row wider than 1024 bytes");
    }
#undef FS_CASE
    FS_LAUNCH_CHECK(ctx, "row_read_kernel");
    return FS_OK;
}

FS_TRACE_SETTER(gather)

}  // namespace fs
