// compute_collision(I^i, I^{i+1}) of Algorithm 2 on ascending distinct row lists:
//   co = U_t & U_t1, ex = U_t \ U_t1, ex_next = U_t1 \ U_t, each ascending, each with the slot of
//   the row in its source list (the slot addresses the reduced-gradient row).
// Sorted-merge intersect by tiles: a tile of 1024 elements of one list only needs the window of
// the other list between its first and last element.  One wavefront finds that window with two
// 64-ary searches, the workgroup stages it in LDS and every element binary-searches LDS (global
// binary search only if the window does not fit).  Membership flags are counted per tile and a
// second launch compacts with tile prefixes.  The list lengths are device scalars; the launch is
// sized by the host-side caps and tiles past the end do nothing.
#include "fs_common.h"

namespace fs {

constexpr int kSplitWindow = 4096;       // elements of the other list staged in LDS (32 KB)

__device__ __forceinline__ int wave_incl_scan_i(int v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int t = __shfl_up(v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

__device__ __forceinline__ int block_excl_scan_i(int v, int *sh, int &total) {
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const int inc = wave_incl_scan_i(v);
    if (lane == kWave - 1) sh[w] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kScanThreads / kWave; ++i) {
        const int x = sh[i];
        if (i < w) base += x;
        tot += x;
    }
    __syncthreads();
    total = tot;
    return base + inc - v;
}

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

// blocks [0, tiles_t) flag U_t against U_t1; blocks [tiles_t, tiles_t + tiles_t1) flag U_t1 against U_t
__global__ __launch_bounds__(kScanThreads) void split_flag_kernel(const int64_t *__restrict__ u_t,
                                                                  const int64_t *__restrict__ n_t_dev,
                                                                  const int64_t *__restrict__ u_t1,
                                                                  const int64_t *__restrict__ n_t1_dev, int64_t cap_t,
                                                                  int64_t cap_t1, int tiles_t,
                                                                  uint8_t *__restrict__ flag_t,
                                                                  uint8_t *__restrict__ flag_t1,
                                                                  int32_t *__restrict__ tile_cnt) {
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
        const int j1 = wave_lower_bound(other, n_other, mine[t_hi - 1] + 1);
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
    (void)block_excl_scan_i(found, sh, total);
    if (threadIdx.x == 0) tile_cnt[blockIdx.x] = total;      // number of collisions in this tile
}

__global__ __launch_bounds__(kScanThreads) void split_compact_kernel(
    const int64_t *__restrict__ u_t, const int64_t *__restrict__ n_t_dev, const int64_t *__restrict__ u_t1,
    const int64_t *__restrict__ n_t1_dev, int64_t cap_t, int64_t cap_t1, int tiles_t, int tiles_t1,
    const uint8_t *__restrict__ flag_t, const uint8_t *__restrict__ flag_t1, const int32_t *__restrict__ tile_cnt,
    int64_t *__restrict__ co, int32_t *__restrict__ co_slot, int64_t *__restrict__ ex, int32_t *__restrict__ ex_slot,
    int64_t *__restrict__ ex_next, int32_t *__restrict__ ex_next_slot, int64_t *__restrict__ counts_dev) {
    __shared__ int sh[kScanThreads / kWave];
    const int n_t = clamp_count(n_t_dev, cap_t), n_t1 = clamp_count(n_t1_dev, cap_t1);
    const bool side_t = (int)blockIdx.x < tiles_t;
    const int tile = side_t ? blockIdx.x : blockIdx.x - tiles_t;
    const int first = side_t ? 0 : tiles_t;
    // collisions in the earlier tiles of my side
    int before = 0;
    for (int t = threadIdx.x; t < tile; t += kScanThreads) before += tile_cnt[first + t];
    int found_before;
    (void)block_excl_scan_i(before, sh, found_before);

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
    int r_found = found_before + block_excl_scan_i(found, sh, tile_total);   // collisions before p0
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        const int p = p0 + i;
        if (p < n_mine) {
            const int64_t id = mine[p];
            if (side_t) {
                if (f[i]) { co[r_found] = id; co_slot[r_found] = p; }
                else { ex[p - r_found] = id; ex_slot[p - r_found] = p; }
            } else if (!f[i]) {
                ex_next[p - r_found] = id; ex_next_slot[p - r_found] = p;
            }
            r_found += f[i] ? 1 : 0;
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

__global__ void split_empty_kernel(const int64_t *n_t1_dev, int64_t cap_t1, int64_t *counts_dev) {
    counts_dev[0] = 0;
    counts_dev[1] = 0;
    counts_dev[2] = clamp_count(n_t1_dev, cap_t1);
}

int launch_split(fs_ctx *ctx, const int64_t *u_t, const int64_t *n_t_dev, const int64_t *u_t1,
                 const int64_t *n_t1_dev, int64_t cap_t, int64_t cap_t1, int64_t *co, int32_t *co_slot,
                 int64_t *ex, int32_t *ex_slot, int64_t *ex_next, int32_t *ex_next_slot, int64_t *counts_dev,
                 hipStream_t s) {
    const int tiles_t = (int)ceil_div(cap_t, kScanTile);
    const int tiles_t1 = (int)ceil_div(cap_t1, kScanTile);
    if (tiles_t == 0 && tiles_t1 == 0) {
        hipLaunchKernelGGL(split_empty_kernel, dim3(1), dim3(1), 0, s, n_t1_dev, cap_t1, counts_dev);
        FS_LAUNCH_CHECK(ctx, "split_empty_kernel");
        return FS_OK;
    }
    // With cap_t == 0 a single (empty) tile on side t keeps the count logic in one place.
    const int tt = tiles_t > 0 ? tiles_t : 1;
    hipLaunchKernelGGL(split_flag_kernel, dim3(tt + tiles_t1), dim3(kScanThreads), 0, s, u_t, n_t_dev, u_t1, n_t1_dev,
                       cap_t, cap_t1, tt, ctx->split_flag_t, ctx->split_flag_t1, ctx->split_cnt);
    hipLaunchKernelGGL(split_compact_kernel, dim3(tt + tiles_t1), dim3(kScanThreads), 0, s, u_t, n_t_dev, u_t1,
                       n_t1_dev, cap_t, cap_t1, tt, tiles_t1, (const uint8_t *)ctx->split_flag_t,
                       (const uint8_t *)ctx->split_flag_t1, (const int32_t *)ctx->split_cnt, co, co_slot, ex, ex_slot,
                       ex_next, ex_next_slot, counts_dev);
    FS_LAUNCH_CHECK(ctx, "split kernels");
    return FS_OK;
}

}  // namespace fs
