// Dedup of one iteration's row IDs: stable LSD radix sort of (ID, position) pairs followed by a
// head-flag compaction that yields the ascending distinct rows, the segment offsets, the stable
// permutation and the inverse map.  (Collisions are defined on rows, Section 2.3 of the paper;
// compute_collision of Algorithm 2 consumes the distinct lists.)
//
// Only ceil(log2(num_rows)) key bits are sorted, in the fewest passes of at most 9 bits; keys
// travel as 32-bit words when they fit.  The inputs are small (a few hundred thousand keys), so
// the passes are latency bound: tiles are large (4096 keys, 1024 threads) to keep the
// [tile][digit] table small enough that every scatter workgroup scans it by itself - a pass is
// two launches (histogram, scan+rank+scatter) and no workgroup ever waits for another.  Ranking
// uses wavefront ballots, so equal digits keep their order.
//
// Every launch handles up to kMaxBatch independent dedups (blockIdx.y picks the job): the lookahead
// batches of several iterations, or of several tables, share their launches - what a launch costs the
// rest of the chip (its start and end disturb every kernel that runs beside it) is paid once.
#include "fs_common.h"
#include "fs_device.h"

namespace fs {

// ---- one dedup of a batch, as the kernels see it ----------------------------------------------------
struct unique_dev_job {
    const int64_t *ids;
    int n, tiles, stiles;         // IDs, sort tiles, compaction tiles (at least 1: the empty dedup writes its counts too)
    int64_t num_rows;
    void *keys[2];                // ping-pong key buffers (K words)
    int32_t *idx[2];              // ping-pong position buffers
    uint32_t *tile_hist;
    int32_t *tile_heads;
    int64_t *unique;
    int32_t *seg_offsets, *perm, *inverse;
    int64_t *n_unique_dev;
    int64_t *sorted_ids;
};
struct unique_dev_batch {
    unique_dev_job j[kMaxBatch];
};

// Workgroups go to the eight XCDs in turn, each with an L2 of its own.  Neighbouring tiles write neighbouring
// runs of every bin; taken by the same XCD one after the other, their runs meet in one L2 and leave it as
// whole lines instead of as eight partly filled ones.  XCD x takes the x-th eighth of the tiles; the grid is a
// multiple of eight workgroups wide.  Returns -1 for a workgroup without a tile.
__device__ __forceinline__ int xcd_tile(int tiles) {
    const int per = (tiles + 7) / 8;
    const int b = (int)blockIdx.x;
    if (b / 8 >= per) return -1;
    const int t = (b % 8) * per + b / 8;
    return t < tiles ? t : -1;
}

// ---- radix pass 1/2: per-tile digit histogram ---------------------------------------------------
template <typename K, bool FIRST>
__global__ __launch_bounds__(kSortThreads) void radix_hist_kernel(const unique_dev_batch batch, int src, int shift,
                                                                  int bits, int *__restrict__ flags) {
    FS_WG_TRACE(1);
    const unique_dev_job &job = batch.j[blockIdx.y];
    const int tile_id = xcd_tile(job.tiles);
    if (tile_id < 0) return;
    const int64_t *__restrict__ ids = job.ids;
    const K *__restrict__ keys_in = (const K *)job.keys[src];
    const int n = job.n;
    const int64_t num_rows = job.num_rows;
    uint32_t *__restrict__ tile_hist = job.tile_hist;
    __shared__ uint32_t hist[kRadix];
    const int bins = 1 << bits;
    for (int d = threadIdx.x; d < bins; d += kSortThreads) hist[d] = 0;
    __syncthreads();
    const int base = tile_id * kSortTile;
    bool bad = false;
#pragma unroll
    for (int r = 0; r < kSortKpt; ++r) {
        const int e = base + r * kSortThreads + threadIdx.x;
        if (e < n) {
            K key;
            if (FIRST) {
                const int64_t id = ids[e];
                bad |= (id < 0) || (num_rows > 0 && id >= num_rows);
                key = (K)id;
            } else {
                key = keys_in[e];
            }
            atomicAdd(&hist[(uint32_t)(key >> shift) & (bins - 1)], 1u);
        }
    }
    __syncthreads();
    for (int d = threadIdx.x; d < bins; d += kSortThreads) tile_hist[tile_id * bins + d] = hist[d];
    if (bad) atomicOr(flags, kFlagRowRange);
}

// ---- radix pass 2/2: scan of the [tile][digit] table, stable ranking, scatter ---------------------
// Tile order is (wave, round, lane): wave w owns 64*KPT consecutive keys, read 64 at a time.
template <typename K, bool FIRST>
__global__ __launch_bounds__(kSortThreads) void radix_scatter_kernel(const unique_dev_batch batch, int src, int shift,
                                                                     int bits, int last) {
    FS_WG_TRACE(2);
    const unique_dev_job &job = batch.j[blockIdx.y];
    const int tile_id = xcd_tile(job.tiles);
    if (tile_id < 0) return;
    const int64_t *__restrict__ ids = job.ids;
    const K *__restrict__ keys_in = (const K *)job.keys[src];
    const int32_t *__restrict__ idx_in = job.idx[src];
    K *__restrict__ keys_out = (K *)job.keys[src ^ 1];
    int32_t *__restrict__ idx_out = last ? job.perm : job.idx[src ^ 1];
    const int n = job.n, tiles = job.tiles;
    const uint32_t *__restrict__ tile_hist = job.tile_hist;
    __shared__ uint16_t cnt[kSortWaves][kRadix];       // per-wave digit counters, then the waves' starts inside the
                                                       // tile's share of the digit (a tile has 4096 keys: 16 bits do)
    __shared__ uint32_t sh_below[kSortScan];
    __shared__ uint32_t sh_total[kSortScan];
    __shared__ uint32_t gbase[kRadix];
    const int bins = 1 << bits;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const int tile = tile_id;

    // keys first: their latency overlaps the table scan
    const int base = tile * kSortTile + w * (kWave * kSortKpt);
    K key[kSortKpt];
#pragma unroll
    for (int r = 0; r < kSortKpt; ++r) {
        const int e = base + r * kWave + lane;
        key[r] = 0;
        if (e < n) key[r] = FIRST ? (K)ids[e] : keys_in[e];
    }
    for (int i = threadIdx.x; i < kSortWaves * kRadix / 2; i += kSortThreads)
        reinterpret_cast<uint32_t *>(&cnt[0][0])[i] = 0u;

    // (1) every workgroup scans the table by itself: virtual thread (q, d) adds the tiles t = q, q+groups, ...
    // (a thread stands for several virtual threads when there are more digits than threads)
    {
        const int groups = kSortThreads >= bins ? kSortThreads / bins : 1;
        for (int vt = threadIdx.x; vt < groups * bins; vt += kSortThreads) {
            const int d = vt & (bins - 1);
            const int q = vt / bins;
            uint32_t below = 0, total = 0;
            for (int t = q; t < tiles; t += groups * 8) {       // eight independent loads in flight
                uint32_t v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int tt = t + j * groups;
                    v[j] = (tt < tiles) ? tile_hist[tt * bins + d] : 0u;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    total += v[j];
                    below += (t + j * groups < tile) ? v[j] : 0u;
                }
            }
            sh_below[vt] = below;
            sh_total[vt] = total;
        }
        __syncthreads();
        for (int d = threadIdx.x; d < bins; d += kSortThreads) {
            uint32_t below = sh_below[d], total = sh_total[d];
            for (int g = 1; g < groups; ++g) {
                below += sh_below[g * bins + d];
                total += sh_total[g * bins + d];
            }
            sh_below[d] = below;       // only this thread reads or writes entry d of group 0 in this loop
            sh_total[d] = total;
        }
        __syncthreads();
        // exclusive scan of the digit totals by the first wave: each lane owns bins/64 consecutive digits
        if (w == 0) {
            const int per = (bins + kWave - 1) / kWave;    // <= 8
            uint32_t loc[kRadix / kWave];
            uint32_t s = 0;
#pragma unroll
            for (int i = 0; i < kRadix / kWave; ++i) {
                const int dd = lane * per + i;
                loc[i] = (i < per && dd < bins) ? sh_total[dd] : 0u;
                s += loc[i];
            }
            const uint32_t incl = (uint32_t)wave_inclusive_scan((int)s);
            uint32_t run = incl - s;
#pragma unroll
            for (int i = 0; i < kRadix / kWave; ++i) {
                const int dd = lane * per + i;
                if (i < per && dd < bins) gbase[dd] = run + sh_below[dd];
                run += loc[i];
            }
        }
    }
    __syncthreads();

    // (2) stable rank of every key among the keys of its wave with the same digit
    const uint64_t lt = (1ull << lane) - 1ull;
    uint32_t rank[kSortKpt];
#pragma unroll
    for (int r = 0; r < kSortKpt; ++r) {
        const int e = base + r * kWave + lane;
        const bool valid = e < n;
        const uint32_t digit = (uint32_t)(key[r] >> shift) & (bins - 1);
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < bits; ++b) {
            const bool bit = (digit >> b) & 1u;
            const uint64_t bal = __ballot(bit);
            peers &= bit ? bal : ~bal;
        }
        const uint32_t before = __popcll(peers & lt);
        const uint32_t old = valid ? cnt[w][digit] : 0u;              // all peers read ...
        if (valid && before == 0) cnt[w][digit] = (uint16_t)(old + (uint32_t)__popcll(peers));   // ... then the first one writes
        rank[r] = old + before;
    }
    __syncthreads();
    // (3) exclusive prefix over the waves of this tile, per digit
    for (int d = threadIdx.x; d < bins; d += kSortThreads) {
        uint32_t run = 0;
#pragma unroll
        for (int i = 0; i < kSortWaves; ++i) {
            const uint32_t v = cnt[i][d];
            cnt[i][d] = (uint16_t)run;
            run += v;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortKpt; ++r) {
        const int e = base + r * kWave + lane;
        if (e < n) {
            const uint32_t digit = (uint32_t)(key[r] >> shift) & (bins - 1);
            const uint32_t pos = gbase[digit] + cnt[w][digit] + rank[r];
            keys_out[pos] = key[r];
            idx_out[pos] = FIRST ? e : idx_in[e];
        }
    }
}

// ---- unique 1/2: heads per compaction tile ---------------------------------------------------------
template <typename K>
__device__ __forceinline__ int load_heads(const K *__restrict__ keys, int n, int p0, K (&k)[kScanIpt], bool (&head)[kScanIpt]) {
    K prev = 0;
    if (p0 > 0 && p0 < n) prev = keys[p0 - 1];
    int c = 0;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        const int p = p0 + i;
        k[i] = (p < n) ? keys[p] : 0;
        head[i] = (p < n) && (p == 0 || k[i] != prev);
        prev = k[i];
        c += head[i] ? 1 : 0;
    }
    return c;
}

template <typename K>
__global__ __launch_bounds__(kScanThreads) void unique_count_kernel(const unique_dev_batch batch, int src) {
    FS_WG_TRACE(3);
    const unique_dev_job &job = batch.j[blockIdx.y];
    if ((int)blockIdx.x >= job.stiles) return;
    const K *__restrict__ keys = (const K *)job.keys[src];
    const int n = job.n;
    int32_t *__restrict__ tile_heads = job.tile_heads;
    __shared__ int sh[kScanThreads / kWave];
    K k[kScanIpt];
    bool head[kScanIpt];
    const int c = load_heads<K>(keys, n, blockIdx.x * kScanTile + threadIdx.x * kScanIpt, k, head);
    int total;
    (void)block_exclusive_scan(c, sh, total);
    if (threadIdx.x == 0) tile_heads[blockIdx.x] = total;
}

// ---- unique 2/2: compaction -------------------------------------------------------------------------
template <typename K>
__global__ __launch_bounds__(kScanThreads) void unique_compact_kernel(const unique_dev_batch batch, int src) {
    FS_WG_TRACE(4);
    const unique_dev_job &job = batch.j[blockIdx.y];
    if ((int)blockIdx.x >= job.stiles) return;
    const K *__restrict__ keys = (const K *)job.keys[src];
    const int32_t *__restrict__ perm = job.perm;
    const int n = job.n;
    const int32_t *__restrict__ tile_heads = job.tile_heads;
    int64_t *__restrict__ unique = job.unique;
    int32_t *__restrict__ seg_offsets = job.seg_offsets;
    int32_t *__restrict__ inverse = job.inverse;
    int64_t *__restrict__ n_unique_dev = job.n_unique_dev;
    int64_t *__restrict__ sorted_ids = job.sorted_ids;
    __shared__ int sh[kScanThreads / kWave];
    const int p0 = blockIdx.x * kScanTile + threadIdx.x * kScanIpt;
    int pm[kScanIpt];
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) pm[i] = (inverse != nullptr && p0 + i < n) ? perm[p0 + i] : 0;
    // heads in all earlier tiles: a cooperative sum (tiles is a few hundred)
    int before = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += kScanThreads) before += tile_heads[t];
    int tile_base;
    (void)block_exclusive_scan(before, sh, tile_base);

    K k[kScanIpt];
    bool head[kScanIpt];
    const int c = load_heads<K>(keys, n, p0, k, head);
    int tile_total;
    int rank = tile_base + block_exclusive_scan(c, sh, tile_total);    // heads strictly before p0
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        const int p = p0 + i;
        if (p < n) {
            if (head[i]) {
                unique[rank] = (int64_t)k[i];
                seg_offsets[rank] = p;
                ++rank;
            }
            if (inverse != nullptr) inverse[pm[i]] = rank - 1;
            if (sorted_ids != nullptr) sorted_ids[p] = (int64_t)k[i];
        }
    }
    if ((int)blockIdx.x == job.stiles - 1 && threadIdx.x == 0) {
        const int total = tile_base + tile_total;
        seg_offsets[total] = n;
        *n_unique_dev = total;
    }
}

__global__ void unique_empty_kernel(int32_t *seg_offsets, int64_t *n_unique_dev) {
    seg_offsets[0] = 0;
    *n_unique_dev = 0;
}

// ---- host side ------------------------------------------------------------------------------------------
template <typename K>
static int unique_batch_impl(fs_ctx *ctx, const unique_dev_batch &batch, int count, int key_bits, hipStream_t s) {
    int tiles = 0, stiles = 0;
    for (int k = 0; k < count; ++k) {
        tiles = batch.j[k].tiles > tiles ? batch.j[k].tiles : tiles;
        stiles = batch.j[k].stiles > stiles ? batch.j[k].stiles : stiles;
    }
    const int passes = (key_bits + kRadixBits - 1) / kRadixBits;
    const int bits = (key_bits + passes - 1) / passes;            // <= kRadixBits, evenly spread
    int cur = 0;   // buffer holding the input of the next pass (unused for the first pass)
    if (tiles > 0) {
        const dim3 grid((unsigned)((tiles + 7) / 8 * 8), (unsigned)count);
        for (int p = 0; p < passes; ++p) {
            const int shift = p * bits;
            const int last = (p == passes - 1) ? 1 : 0;
            if (p == 0) {
                hipLaunchKernelGGL((radix_hist_kernel<K, true>), grid, dim3(kSortThreads), 0, s, batch, cur, shift,
                                   bits, ctx->d_flags);
                hipLaunchKernelGGL((radix_scatter_kernel<K, true>), grid, dim3(kSortThreads), 0, s, batch, cur, shift,
                                   bits, last);
            } else {
                hipLaunchKernelGGL((radix_hist_kernel<K, false>), grid, dim3(kSortThreads), 0, s, batch, cur, shift,
                                   bits, ctx->d_flags);
                hipLaunchKernelGGL((radix_scatter_kernel<K, false>), grid, dim3(kSortThreads), 0, s, batch, cur,
                                   shift, bits, last);
            }
            cur ^= 1;
        }
    }
    const dim3 sgrid((unsigned)stiles, (unsigned)count);
    hipLaunchKernelGGL((unique_count_kernel<K>), sgrid, dim3(kScanThreads), 0, s, batch, cur);
    hipLaunchKernelGGL((unique_compact_kernel<K>), sgrid, dim3(kScanThreads), 0, s, batch, cur);
    FS_LAUNCH_CHECK(ctx, "unique kernels");
    return FS_OK;
}

int launch_unique_batch(fs_ctx *ctx, int count, const fs_unique_job *jobs, hipStream_t s, int set0) {
    if (count < 1 || count > kMaxBatch || set0 < 0 || set0 + count > kSortSets)
        return set_err(ctx, FS_EINVAL, "unique: batch size");
    if (count == 1 && jobs[0].n == 0) {
        hipLaunchKernelGGL(unique_empty_kernel, dim3(1), dim3(1), 0, s, jobs[0].seg_offsets, jobs[0].n_unique_dev);
        FS_LAUNCH_CHECK(ctx, "unique_empty_kernel");
        return FS_OK;
    }
    // one sort geometry for the whole batch: the widest key decides (sorting zero bits is harmless)
    int key_bits = 1;
    unique_dev_batch batch;
    memset(&batch, 0, sizeof(batch));
    for (int k = 0; k < count; ++k) {
        const fs_unique_job &in = jobs[k];
        int kb = 63;
        if (in.num_rows > 0) {
            kb = 1;
            while (kb < 63 && (1ll << kb) < in.num_rows) ++kb;
        }
        key_bits = kb > key_bits ? kb : key_bits;
        const fs_sort_scratch &ws = ctx->sort[set0 + k];
        unique_dev_job &j = batch.j[k];
        j.ids = in.ids;
        j.n = (int)in.n;
        j.tiles = (int)ceil_div(in.n, kSortTile);
        j.stiles = in.n > 0 ? (int)ceil_div(in.n, kScanTile) : 1;
        j.num_rows = in.num_rows;
        j.keys[0] = ws.keys[0];
        j.keys[1] = ws.keys[1];
        j.idx[0] = ws.idx[0];
        j.idx[1] = ws.idx[1];
        j.tile_hist = ws.tile_hist;
        j.tile_heads = ws.tile_heads;
        j.unique = in.unique;
        j.seg_offsets = in.seg_offsets;
        j.perm = in.perm;
        j.inverse = in.inverse;
        j.n_unique_dev = in.n_unique_dev;
        j.sorted_ids = in.sorted_ids;
    }
    if (key_bits <= 32) return unique_batch_impl<uint32_t>(ctx, batch, count, key_bits, s);
    return unique_batch_impl<uint64_t>(ctx, batch, count, key_bits, s);
}

int launch_unique(fs_ctx *ctx, const int64_t *ids, int64_t n, int64_t num_rows, int64_t *unique,
                  int32_t *seg_offsets, int32_t *perm, int32_t *inverse, int64_t *n_unique_dev, hipStream_t s,
                  int set) {
    const fs_unique_job job = {ids, n, num_rows, unique, seg_offsets, perm, inverse, n_unique_dev};
    return launch_unique_batch(ctx, 1, &job, s, set);
}

FS_TRACE_SETTER(unique)

}  // namespace fs
