// compute_collision(I^i, I^{i+1}) of Algorithm 2 on ascending distinct row lists:
//   co = U_t & U_t1, ex = U_t \ U_t1, ex_next = U_t1 \ U_t, each ascending, each with the slot of
//   the row in its source list (the slot addresses the reduced-gradient row).
// Sorted-merge intersect by tiles: a tile of 1024 elements of one list only needs the window of
// the other list between its first and last element.  One wavefront finds that window with two
// 64-ary searches, the workgroup stages it in LDS and every element binary-searches LDS (global
// binary search only if the window does not fit).  Membership flags are counted per tile and a
// second launch compacts with tile prefixes.  The list lengths are device scalars; the launch is
// sized by the host-side caps and tiles past the end do nothing.
#include <mutex>

#include "fs_common.h"
#include "fs_device.h"

namespace fs {

constexpr int kSplitWindow = 4096;       // elements of the other list staged in LDS (32 KB)

// number of elements of a[0, n) that are < key; executed by one whole wavefront (64-ary search)
__device__ __forceinline__ int wave_lower_bound(const int64_t *__restrict__ a, int n, int64_t key) {
    const int lane = threadIdx.x & (kWave - 1);
    int lo = 0, hi = n;                      // a[i] < key for i < lo, a[i] >= key for i >= hi
    while (lo < hi) {
        const int step = (hi - lo + kWave - 1) / kWave;
        const int probe = lo + (lane + 1) * step - 1;          // last element of my sub-block
        const bool less = (probe < hi) && (a[probe] < key);
        const int cnt = __popcll(__ballot(less));
        lo += cnt * step;
        const int nhi = lo + step - 1;
        hi = nhi < hi ? nhi : hi;
    }
    return lo;
}

// number of entries of a[0, n) that are <= key; executed by one whole wavefront (64-ary search)
template <typename T>
__device__ __forceinline__ int wave_upper_bound(const T *__restrict__ a, int n, T key) {
    const int lane = threadIdx.x & (kWave - 1);
    int lo = 0, hi = n;                      // a[i] <= key for i < lo, a[i] > key for i >= hi
    while (lo < hi) {
        const int step = (hi - lo + kWave - 1) / kWave;
        const int probe = lo + (lane + 1) * step - 1;          // last entry of my sub-block
        const bool le = (probe < hi) && (a[probe] <= key);
        const int cnt = __popcll(__ballot(le));
        lo += cnt * step;
        const int nhi = lo + step - 1;
        hi = nhi < hi ? nhi : hi;
    }
    return lo;
}

template <typename P>
__device__ __forceinline__ bool sorted_contains(P a, int lo, int hi, int64_t key) {
    const int end = hi;
    while (lo < hi) {                        // first index with a[i] >= key
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo < end && a[lo] == key;
}

__device__ __forceinline__ int clamp_count(const int64_t *dev, int64_t cap) {
    if (dev == nullptr) return 0;
    int64_t v = *dev;
    if (v < 0) v = 0;
    if (v > cap) v = cap;
    return (int)v;
}

// One collision split + class order of a batch that shares its launches (blockIdx.y picks the job), as
// the kernels see it.
struct split_dev_job {
    const int64_t *u_t, *n_t_dev, *u_t1, *n_t1_dev;
    int64_t cap_t, cap_t1;
    int tiles_t, tiles_t1;        // tiles_t is at least 1: an empty U_t still has its counts written
    uint8_t *flag_t, *flag_t1;
    int32_t *tile_cnt;
    int64_t *co;
    int32_t *co_slot;
    int64_t *ex;
    int32_t *ex_slot;
    int64_t *ex_next;
    int32_t *ex_next_slot;
    int64_t *counts_dev;
    const int32_t *seg_offsets_t;
    int32_t *cstart_local, *tile_len, *cidx;
};
struct split_dev_batch {
    split_dev_job j[kMaxBatch];
};
struct class_dev_job {
    const int32_t *perm, *seg_offsets;
    const int64_t *n_unique_dev;
    int n, tiles_t, blocks, cap;  // blocks is at least 1: an empty batch still has its class extents written
    const uint8_t *flag_t;
    const int32_t *cstart_local, *tile_len, *cidx;
    int32_t *cperm, *cslot, *cstart, *class_pos_dev;
    const int64_t *u_t;
    int32_t *short_rec;
};
struct class_dev_batch {
    class_dev_job j[kMaxBatch];
};

// blocks [0, tiles_t) flag U_t against U_t1; blocks [tiles_t, tiles_t + tiles_t1) flag U_t1 against U_t
__global__ __launch_bounds__(kScanThreads) void split_flag_kernel(const split_dev_batch batch) {
    FS_WG_TRACE(5);
    const split_dev_job &job = batch.j[blockIdx.y];
    if ((int)blockIdx.x >= job.tiles_t + job.tiles_t1) return;
    const int64_t *__restrict__ u_t = job.u_t, *__restrict__ u_t1 = job.u_t1;
    const int64_t *__restrict__ n_t_dev = job.n_t_dev, *__restrict__ n_t1_dev = job.n_t1_dev;
    const int64_t cap_t = job.cap_t, cap_t1 = job.cap_t1;
    const int tiles_t = job.tiles_t;
    uint8_t *__restrict__ flag_t = job.flag_t, *__restrict__ flag_t1 = job.flag_t1;
    int32_t *__restrict__ tile_cnt = job.tile_cnt;
    __shared__ int sh[kScanThreads / kWave];
    __shared__ int win[2];
    __shared__ int64_t window[kSplitWindow];
    const int n_t = clamp_count(n_t_dev, cap_t), n_t1 = clamp_count(n_t1_dev, cap_t1);
    const bool side_t = (int)blockIdx.x < tiles_t;
    const int tile = side_t ? blockIdx.x : blockIdx.x - tiles_t;
    const int64_t *mine = side_t ? u_t : u_t1;
    const int64_t *other = side_t ? u_t1 : u_t;
    const int n_mine = side_t ? n_t : n_t1, n_other = side_t ? n_t1 : n_t;
    uint8_t *flag = side_t ? flag_t : flag_t1;
    const int t_lo = tile * kScanTile;
    if (t_lo >= n_mine) {                                    // whole workgroup: tile past the end
        if (threadIdx.x == 0) tile_cnt[blockIdx.x] = 0;
        return;
    }
    const int t_hi = (t_lo + kScanTile < n_mine) ? t_lo + kScanTile : n_mine;
    if (threadIdx.x < kWave) {
        const int j0 = wave_lower_bound(other, n_other, mine[t_lo]);
        // upper end: the entries <= the tile's last element (a search for "last + 1" would wrap around at the
        // top of the ID range, which is legal when the table size is not given)
        const int j1 = wave_upper_bound<int64_t>(other, n_other, mine[t_hi - 1]);
        if (threadIdx.x == 0) { win[0] = j0; win[1] = j1; }
    }
    __syncthreads();
    const int j0 = win[0], j1 = win[1];
    const bool staged = (j1 - j0) <= kSplitWindow;
    if (staged)
        for (int i = threadIdx.x; i < j1 - j0; i += kScanThreads) window[i] = other[j0 + i];
    __syncthreads();
    const int p0 = t_lo + threadIdx.x * kScanIpt;
    int found = 0;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        const int p = p0 + i;
        if (p < t_hi) {
            const int64_t key = mine[p];
            const bool f = staged ? sorted_contains((const int64_t *)window, 0, j1 - j0, key)
                                  : sorted_contains(other, j0, j1, key);
            flag[p] = f ? 1 : 0;
            found += f ? 1 : 0;
        }
    }
    int total;
    (void)block_exclusive_scan<int>(found, sh, total);
    if (threadIdx.x == 0) tile_cnt[blockIdx.x] = total;      // number of collisions in this tile
}

__global__ __launch_bounds__(kScanThreads) void split_compact_kernel(const split_dev_batch batch) {
    FS_WG_TRACE(6);
    const split_dev_job &job = batch.j[blockIdx.y];
    if ((int)blockIdx.x >= job.tiles_t + job.tiles_t1) return;
    const int64_t *__restrict__ u_t = job.u_t, *__restrict__ u_t1 = job.u_t1;
    const int64_t *__restrict__ n_t_dev = job.n_t_dev, *__restrict__ n_t1_dev = job.n_t1_dev;
    const int64_t cap_t = job.cap_t, cap_t1 = job.cap_t1;
    const int tiles_t = job.tiles_t;
    const uint8_t *__restrict__ flag_t = job.flag_t, *__restrict__ flag_t1 = job.flag_t1;
    const int32_t *__restrict__ tile_cnt = job.tile_cnt;
    int64_t *__restrict__ co = job.co, *__restrict__ ex = job.ex, *__restrict__ ex_next = job.ex_next;
    int32_t *__restrict__ co_slot = job.co_slot, *__restrict__ ex_slot = job.ex_slot;
    int32_t *__restrict__ ex_next_slot = job.ex_next_slot;
    int64_t *__restrict__ counts_dev = job.counts_dev;
    const int32_t *__restrict__ seg_offsets_t = job.seg_offsets_t;
    int32_t *__restrict__ cstart_local = job.cstart_local, *__restrict__ tile_len = job.tile_len;
    int32_t *__restrict__ cidx = job.cidx;
    __shared__ int sh[kScanThreads / kWave];
    const int n_t = clamp_count(n_t_dev, cap_t), n_t1 = clamp_count(n_t1_dev, cap_t1);
    const bool side_t = (int)blockIdx.x < tiles_t;
    const int tile = side_t ? blockIdx.x : blockIdx.x - tiles_t;
    const int first = side_t ? 0 : tiles_t;
    // collisions in the earlier tiles of my side
    int before = 0;
    for (int t = threadIdx.x; t < tile; t += kScanThreads) before += tile_cnt[first + t];
    int found_before;
    (void)block_exclusive_scan<int>(before, sh, found_before);

    const int64_t *mine = side_t ? u_t : u_t1;
    const uint8_t *flag = side_t ? flag_t : flag_t1;
    const int n_mine = side_t ? n_t : n_t1;
    const int p0 = tile * kScanTile + threadIdx.x * kScanIpt;
    bool f[kScanIpt];
    int found = 0;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        const int p = p0 + i;
        f[i] = (p < n_mine) && flag[p] != 0;
        found += f[i] ? 1 : 0;
    }
    int tile_total;
    int r_found = found_before + block_exclusive_scan<int>(found, sh, tile_total);   // collisions before p0
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        const int p = p0 + i;
        if (p < n_mine) {
            const int64_t id = mine[p];
            if (side_t) {
                if (f[i]) { co[r_found] = id; co_slot[r_found] = p; }
                else { ex[p - r_found] = id; ex_slot[p - r_found] = p; }
                if (seg_offsets_t != nullptr) cidx[p] = f[i] ? r_found : p - r_found;   // place in its class list
            } else if (!f[i]) {
                ex_next[p - r_found] = id; ex_next_slot[p - r_found] = p;
            }
            r_found += f[i] ? 1 : 0;
        }
    }
    // For the class order of the batch (rows with more than FS_SHORT_SEGMENT occurrences only):
    // occurrences of the same-class rows that precede each row inside this tile, and the tile's
    // occurrence totals per class.
    if (side_t && seg_offsets_t != nullptr) {
        int len[kScanIpt];
        int co_len = 0, ex_len = 0;
#pragma unroll
        for (int i = 0; i < kScanIpt; ++i) {
            const int p = p0 + i;
            len[i] = (p < n_mine) ? seg_offsets_t[p + 1] - seg_offsets_t[p] : 0;
            if (len[i] <= FS_SHORT_SEGMENT) len[i] = 0;      // short segments are not part of the class order
            co_len += f[i] ? len[i] : 0;
            ex_len += f[i] ? 0 : len[i];
        }
        int co_total, ex_total;
        int co_before = block_exclusive_scan<int>(co_len, sh, co_total);
        int ex_before = block_exclusive_scan<int>(ex_len, sh, ex_total);
#pragma unroll
        for (int i = 0; i < kScanIpt; ++i) {
            const int p = p0 + i;
            if (p < n_mine) cstart_local[p] = f[i] ? co_before : ex_before;
            co_before += f[i] ? len[i] : 0;
            ex_before += f[i] ? 0 : len[i];
        }
        if (threadIdx.x == 0) {
            tile_len[tile] = co_total;
            tile_len[tiles_t + tile] = ex_total;
        }
    }
    // the last tile of side t knows |co|; |ex| and |ex_next| follow from the list lengths
    if (side_t && tile == tiles_t - 1 && threadIdx.x == 0) {
        const int n_co = found_before + tile_total;
        counts_dev[0] = n_co;
        counts_dev[1] = n_t - n_co;
        counts_dev[2] = n_t1 - n_co;
    }
}

// Class order of the occurrences of batch t that belong to rows with more than FS_SHORT_SEGMENT
// occurrences: sorted position q (row slot s, the j-th occurrence of that row) goes to  [start of the class] + [occurrences of same-class rows before s] + j.
// Every workgroup first turns the per-tile totals into tile bases (a few hundred values).  The row slot of a
// sorted position is found in the segment boundaries themselves: a workgroup's 1024 consecutive sorted
// positions touch at most 1024 consecutive rows, whose boundaries it stages in LDS (the inverse map would
// give the same slot at the price of one random 4-byte read per occurrence).
__global__ __launch_bounds__(kScanThreads) void class_scatter_kernel(const class_dev_batch batch,
                                                                     int *__restrict__ flags) {
    FS_WG_TRACE(7);
    const class_dev_job &job = batch.j[blockIdx.y];
    if ((int)blockIdx.x >= job.blocks) return;
    const int32_t *__restrict__ perm = job.perm;
    const int32_t *__restrict__ seg_offsets = job.seg_offsets;
    const int n = job.n, tiles_t = job.tiles_t, cap = job.cap;
    const int n_u = clamp_count(job.n_unique_dev, cap);
    const uint8_t *__restrict__ flag_t = job.flag_t;
    const int32_t *__restrict__ cstart_local = job.cstart_local, *__restrict__ tile_len = job.tile_len;
    const int32_t *__restrict__ cidx = job.cidx;
    int32_t *__restrict__ cperm = job.cperm, *__restrict__ cslot = job.cslot, *__restrict__ cstart = job.cstart;
    int32_t *__restrict__ class_pos_dev = job.class_pos_dev;
    const int64_t *__restrict__ u_t = job.u_t;
    int32_t *__restrict__ short_rec = job.short_rec;
    extern __shared__ int tile_base[];                      // [2 * tiles_t]
    __shared__ int sh[kScanThreads / kWave];
    __shared__ int32_t seg_win[kScanTile + 2];              // seg_offsets[slot_a .. slot_b + 1]
    __shared__ int win[2];
    const int qa = blockIdx.x * kScanTile;
    const int qb = (qa + kScanTile < n ? qa + kScanTile : n) - 1;          // last sorted position of the workgroup
    if (threadIdx.x < 2 * kWave) {
        // the row of a sorted position q: the last slot whose segment starts at or before q
        const int w = threadIdx.x / kWave;
        int k = 0;
        if (qa < n && n_u > 0) k = wave_upper_bound<int32_t>(seg_offsets, n_u + 1, w == 0 ? qa : qb) - 1;
        k = k < 0 ? 0 : (k > n_u - 1 ? n_u - 1 : k);
        if ((threadIdx.x & (kWave - 1)) == 0) win[w] = k;
    }
    __syncthreads();
    const int slot_a = win[0];
    int wn = (qa < n && n_u > 0) ? win[1] - slot_a + 2 : 0; // boundaries staged
    if (wn > kScanTile + 2 || wn < 0) {                     // cannot happen: every row has an occurrence
        if (threadIdx.x == 0) atomicOr(flags, kFlagInternal);
        wn = 0;
    }
    for (int j = threadIdx.x; j < wn; j += kScanThreads) seg_win[j] = seg_offsets[slot_a + j];
    int class_total[2];
    for (int c = 0; c < 2; ++c) {
        int carry = 0;
        for (int t0 = 0; t0 < tiles_t; t0 += kScanThreads) {
            const int t = t0 + threadIdx.x;
            const int v = (t < tiles_t) ? tile_len[c * tiles_t + t] : 0;
            int total;
            const int before = block_exclusive_scan<int>(v, sh, total);
            if (t < tiles_t) tile_base[c * tiles_t + t] = carry + before;
            carry += total;
        }
        class_total[c] = carry;
    }
    __syncthreads();
    const int n_co_pos = class_total[0];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        class_pos_dev[0] = n_co_pos;
        class_pos_dev[1] = n_co_pos + class_total[1];
    }
    const int q0 = blockIdx.x * kScanTile + threadIdx.x;
    int i[kScanIpt], s[kScanIpt];
#pragma unroll
    for (int k = 0; k < kScanIpt; ++k) {
        const int q = q0 + k * kScanThreads;
        i[k] = (q < n) ? perm[q] : 0;
    }
#pragma unroll
    for (int k = 0; k < kScanIpt; ++k) {
        const int q = q0 + k * kScanThreads;
        s[k] = -1;
        if (q < n && wn >= 2) {
            int lo = 0, hi = wn - 1;                         // first j with seg_win[j] > q, among the row starts
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (seg_win[mid] <= q) lo = mid + 1; else hi = mid;
            }
            s[k] = lo - 1;                                   // place in the window, -1: before its first row
        }
    }
#pragma unroll
    for (int k = 0; k < kScanIpt; ++k) {
        const int q = q0 + k * kScanThreads;
        if (q < n) {
            if (s[k] < 0 || q >= seg_win[s[k] + 1]) {        // layout and batch do not fit each other
                atomicOr(flags, kFlagInternal);
                continue;
            }
            const int slot = slot_a + s[k];
            const bool is_co = flag_t[slot] != 0;
            const int tile = slot / kScanTile;
            const int first = seg_win[s[k]];
            const int len = seg_win[s[k] + 1] - first;
            // one record per row of the batch, at the row's place in its class list: header (row,
            // slot, occurrences) from the row's first position, occurrences only for short segments
            const int li = cidx[slot];
            if (li < 0 || li >= cap) {
                atomicOr(flags, kFlagInternal);
                continue;
            }
            int32_t *rec = short_rec + ((int64_t)(is_co ? 0 : cap) + li) * kShortRecInts;
            if (q == first) {
                const int64_t row = u_t[slot];
                typedef int i32x4 __attribute__((ext_vector_type(4)));
                *reinterpret_cast<i32x4 *>(rec) = i32x4{(int)(row & 0xFFFFFFFFll), (int)(row >> 32), slot, len};
            }
            if (len <= FS_SHORT_SEGMENT) {
                rec[4 + (q - first)] = i[k];
                continue;
            }
            const int dest = (is_co ? tile_base[tile] : n_co_pos + tile_base[tiles_t + tile]) + cstart_local[slot] +
                             (q - first);
            if (dest < 0 || dest >= n) {                     // cannot happen with a consistent layout and split
                atomicOr(flags, kFlagInternal);
                continue;
            }
            cperm[dest] = i[k];
            cslot[dest] = slot;
            if (q == first) cstart[slot] = dest;
        }
    }
}

__global__ void class_empty_kernel(int32_t *class_pos_dev) {
    class_pos_dev[0] = 0;
    class_pos_dev[1] = 0;
}

__global__ void split_empty_kernel(const int64_t *n_t1_dev, int64_t cap_t1, int64_t *counts_dev) {
    counts_dev[0] = 0;
    counts_dev[1] = 0;
    counts_dev[2] = clamp_count(n_t1_dev, cap_t1);
}

int launch_split_batch(fs_ctx *ctx, int count, const fs_split_job *jobs, hipStream_t s, int set0) {
    if (count < 1 || count > kMaxBatch || set0 < 0 || set0 + count > kSortSets)
        return set_err(ctx, FS_EINVAL, "split: batch size");
    if (count == 1 && jobs[0].cap_t == 0 && jobs[0].cap_t1 == 0) {
        hipLaunchKernelGGL(split_empty_kernel, dim3(1), dim3(1), 0, s, jobs[0].n_t1_dev, jobs[0].cap_t1,
                           jobs[0].counts_dev);
        FS_LAUNCH_CHECK(ctx, "split_empty_kernel");
        return FS_OK;
    }
    split_dev_batch batch;
    memset(&batch, 0, sizeof(batch));
    int blocks = 0;
    for (int k = 0; k < count; ++k) {
        const fs_split_job &in = jobs[k];
        const fs_split_scratch &ws = ctx->split[set0 + k];
        split_dev_job &j = batch.j[k];
        const int tiles_t = (int)ceil_div(in.cap_t, kScanTile);
        j.u_t = in.u_t; j.n_t_dev = in.n_t_dev; j.u_t1 = in.u_t1; j.n_t1_dev = in.n_t1_dev;
        j.cap_t = in.cap_t; j.cap_t1 = in.cap_t1;
        // With cap_t == 0 a single (empty) tile on side t keeps the count logic in one place.
        j.tiles_t = tiles_t > 0 ? tiles_t : 1;
        j.tiles_t1 = (int)ceil_div(in.cap_t1, kScanTile);
        j.flag_t = ws.flag_t; j.flag_t1 = in.flag_t1_out ? in.flag_t1_out : ws.flag_t1; j.tile_cnt = ws.cnt;
        j.co = in.co; j.co_slot = in.co_slot; j.ex = in.ex; j.ex_slot = in.ex_slot;
        j.ex_next = in.ex_next; j.ex_next_slot = in.ex_next_slot; j.counts_dev = in.counts_dev;
        j.seg_offsets_t = in.seg_offsets_t;
        j.cstart_local = ws.cstart_local; j.tile_len = ws.tile_len; j.cidx = ws.cidx;
        blocks = (j.tiles_t + j.tiles_t1) > blocks ? (j.tiles_t + j.tiles_t1) : blocks;
    }
    const dim3 grid((unsigned)blocks, (unsigned)count);
    hipLaunchKernelGGL(split_flag_kernel, grid, dim3(kScanThreads), 0, s, batch);
    hipLaunchKernelGGL(split_compact_kernel, grid, dim3(kScanThreads), 0, s, batch);
    FS_LAUNCH_CHECK(ctx, "split kernels");
    return FS_OK;
}

int launch_split(fs_ctx *ctx, const int64_t *u_t, const int64_t *n_t_dev, const int64_t *u_t1,
                 const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1, int64_t *co, int32_t *co_slot,
                 int64_t *ex, int32_t *ex_slot, int64_t *ex_next, int32_t *ex_next_slot, int64_t *counts_dev,
                 hipStream_t s, const int32_t *seg_offsets_t, int set) {
    const fs_split_job job = {u_t, n_t_dev, u_t1, n_t1_dev, cap_t, cap_t1, co, co_slot, ex, ex_slot,
                              ex_next, ex_next_slot, counts_dev, seg_offsets_t};
    return launch_split_batch(ctx, 1, &job, s, set);
}

int launch_class_order_batch(fs_ctx *ctx, int count, const fs_class_job *jobs, hipStream_t s, int set0) {
    if (count < 1 || count > kMaxBatch || set0 < 0 || set0 + count > kSortSets)
        return set_err(ctx, FS_EINVAL, "class order: batch size");
    if (count == 1 && jobs[0].n == 0) {
        hipLaunchKernelGGL(class_empty_kernel, dim3(1), dim3(1), 0, s, jobs[0].class_pos_dev);
        FS_LAUNCH_CHECK(ctx, "class_empty_kernel");
        return FS_OK;
    }
    class_dev_batch batch;
    memset(&batch, 0, sizeof(batch));
    int blocks = 1, max_tiles = 0;
    for (int k = 0; k < count; ++k) {
        const fs_class_job &in = jobs[k];
        const fs_split_scratch &ws = ctx->split[set0 + k];
        class_dev_job &j = batch.j[k];
        j.perm = in.perm; j.n_unique_dev = in.n_unique_dev; j.seg_offsets = in.seg_offsets;
        j.n = (int)in.n;
        j.tiles_t = (int)ceil_div(in.cap_u, kScanTile);      // the same tiling the split used for side t
        j.blocks = in.n > 0 ? (int)ceil_div(in.n, kScanTile) : 1;
        j.cap = (int)in.cap_u;
        j.flag_t = ws.flag_t; j.cstart_local = ws.cstart_local; j.tile_len = ws.tile_len; j.cidx = ws.cidx;
        j.cperm = in.cperm; j.cslot = in.cslot; j.cstart = in.cstart; j.class_pos_dev = in.class_pos_dev;
        j.u_t = in.u_t; j.short_rec = in.short_rec;
        blocks = j.blocks > blocks ? j.blocks : blocks;
        max_tiles = j.tiles_t > max_tiles ? j.tiles_t : max_tiles;
    }
    if ((size_t)max_tiles * 2 * sizeof(int) > 60 * 1024)
        return set_err(ctx, FS_ERANGE, "class order: more than 7.8M distinct rows in one batch");
    hipLaunchKernelGGL(class_scatter_kernel, dim3((unsigned)blocks, (unsigned)count), dim3(kScanThreads),
                       (size_t)max_tiles * 2 * sizeof(int), s, batch, ctx->d_flags);
    FS_LAUNCH_CHECK(ctx, "class_scatter_kernel");
    return FS_OK;
}

int launch_class_order(fs_ctx *ctx, const int32_t *perm, const int64_t *n_unique_dev, const int32_t *seg_offsets,
                       int64_t n, int64_t cap_u, int32_t *cperm, int32_t *cslot, int32_t *cstart,
                       int32_t *class_pos_dev, const int64_t *u_t, int32_t *short_rec, hipStream_t s, int set) {
    const fs_class_job job = {perm, n_unique_dev, seg_offsets, n, cap_u, cperm, cslot, cstart, class_pos_dev, u_t, short_rec};
    return launch_class_order_batch(ctx, 1, &job, s, set);
}

FS_TRACE_SETTER(split)

// ---- the collision split for callers that cannot allocate ----------------------------------------------------
// Same two kernels as launch_split_batch; the membership flags and per-tile counts live in a fixed device array
// instead of a context's slab.
constexpr int64_t kStaticSplitRows = FS_STATIC_SPLIT_MAX_ROWS;
constexpr size_t kStaticFlagBytes = ((size_t)kStaticSplitRows + 16 + 255) / 256 * 256;
constexpr size_t kStaticTiles = (size_t)(kStaticSplitRows / kScanTile) + 2;
constexpr size_t kStaticCntBytes = (2 * kStaticTiles * sizeof(int32_t) + 255) / 256 * 256;
constexpr size_t kStaticScratchBytes = 2 * kStaticFlagBytes + kStaticCntBytes;
static_assert(kStaticSplitRows % kScanTile == 0, "whole tiles");

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kStaticMaxDevices = 64;
static std::mutex g_static_mu;
static unsigned char *g_static_ptr[kStaticMaxDevices];      // device address of `scratch` on each GPU, once asked for

// the address of this GPU's copy of `scratch` (each GPU holds its own); `device` must be current
static hipError_t static_scratch_for(int device, unsigned char **out) {
    std::lock_guard<std::mutex> lk(g_static_mu);
    if (g_static_ptr[device] == nullptr) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_static_ptr[device] = static_cast<unsigned char *>(p);
    }
    *out = g_static_ptr[device];
    return hipSuccess;
}

int static_split_prepare(int device) {
    if (device < 0 || device >= kStaticMaxDevices) return FS_EINVAL;
    unsigned char *p = nullptr;
    return static_scratch_for(device, &p) == hipSuccess ? FS_OK : FS_EHIP;
}

}  // namespace fs

extern "C" int fs_collision_split_static(const int64_t *u_t, const int64_t *n_t_dev, const int64_t *u_t1,
                                         const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1, int64_t *co,
                                         int32_t *co_slot, int64_t *ex, int32_t *ex_slot, int64_t *ex_next,
                                         int32_t *ex_next_slot, int64_t *counts_dev, fs_stream stream) {
    using namespace fs;
    if (cap_t < 0 || cap_t1 < 0) return set_static_err(FS_EINVAL, "static split: negative capacity");
    if (cap_t > kStaticSplitRows || cap_t1 > kStaticSplitRows)
        return set_static_err(FS_ENOMEM, "static split: a list of more than FS_STATIC_SPLIT_MAX_ROWS rows does not fit "
                                         "the fixed scratch array; use fs_collision_split with a context");
    if (!counts_dev) return set_static_err(FS_EINVAL, "static split: null counts");
    if (cap_t > 0 && !(u_t && n_t_dev && co && co_slot && ex && ex_slot))
        return set_static_err(FS_EINVAL, "static split: null pointer (t side)");
    if (cap_t1 > 0 && !(u_t1 && n_t1_dev && ex_next && ex_next_slot))
        return set_static_err(FS_EINVAL, "static split: null pointer (t+1 side)");
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kStaticMaxDevices)
        return set_static_err(FS_EHIP, "static split: no current device");
    unsigned char *base = nullptr;
    const hipError_t se = static_scratch_for(device, &base);
    if (se != hipSuccess) return set_static_err(FS_EHIP, hipGetErrorString(se));
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (cap_t == 0 && cap_t1 == 0) {
        hipLaunchKernelGGL(split_empty_kernel, dim3(1), dim3(1), 0, s, (const int64_t *)nullptr, (int64_t)0, counts_dev);
    } else {
        // Nothing has to start at zero: the flag launch writes every flag and every per-tile count that the
        // compaction launch reads (tiles past the end of a list write a zero count).
        split_dev_batch batch;
        memset(&batch, 0, sizeof(batch));
        split_dev_job &j = batch.j[0];
        const int tiles_t = (int)ceil_div(cap_t, kScanTile);
        j.u_t = u_t; j.n_t_dev = cap_t > 0 ? n_t_dev : nullptr;
        j.u_t1 = u_t1; j.n_t1_dev = cap_t1 > 0 ? n_t1_dev : nullptr;
        j.cap_t = cap_t; j.cap_t1 = cap_t1;
        j.tiles_t = tiles_t > 0 ? tiles_t : 1;
        j.tiles_t1 = (int)ceil_div(cap_t1, kScanTile);
        j.flag_t = base;
        j.flag_t1 = base + kStaticFlagBytes;
        j.tile_cnt = reinterpret_cast<int32_t *>(base + 2 * kStaticFlagBytes);
        j.co = co; j.co_slot = co_slot; j.ex = ex; j.ex_slot = ex_slot;
        j.ex_next = ex_next; j.ex_next_slot = ex_next_slot; j.counts_dev = counts_dev;
        j.seg_offsets_t = nullptr; j.cstart_local = nullptr; j.tile_len = nullptr; j.cidx = nullptr;
        const dim3 grid((unsigned)(j.tiles_t + j.tiles_t1), 1u);
        hipLaunchKernelGGL(split_flag_kernel, grid, dim3(kScanThreads), 0, s, batch);
        hipLaunchKernelGGL(split_compact_kernel, grid, dim3(kScanThreads), 0, s, batch);
    }
    const hipError_t le = hipGetLastError();
    if (le != hipSuccess) return set_static_err(FS_EHIP, hipGetErrorString(le));
    return FS_OK;
}
