// Load-balancer data path on one GPU: the Fixed Batch Size partitioner (Section 4.1 of the paper,
// "Partitioning Algorithms") and the indexed permute of a jagged tensor (Section 4.2, "Triton Kernel
// Optimizations": the kernel that applies a partitioning to the gathered IDs).
//
// FBS: samples sorted by UIH length (the stable radix sort of the dedup, on the lengths), then dealt to
// the ranks in a zig-zag - rank i takes sorted positions i, 2n-1-i, 2n+i, 4n-1-i, ...  The deal is a
// closed form per sorted position, one thread each.
//
// Indexed permute: output sample k is input sample sample_of[k].  Three launches: lengths summed per
// tile of samples, the output offsets by a scan with tile prefixes, and the copy.  The copy is driven
// by the OUTPUT (every lane writes consecutive pieces of the output, so a 16K-item sample costs per
// item what a short one costs): a workgroup takes 4096 or 8192 consecutive output pieces, finds the samples
// they belong to with two 64-ary searches, stages their boundaries in LDS and lets every piece
// binary-search LDS.
//
// VBS: the same sort, then the sorted order is cut into n runs of about equal total weight.
//
// Keyed transpose, ranged dispatch and ranged combine (same section of the paper) are the same copy
// under a computed order of the F x B segments of a keyed jagged tensor: one more launch writes that
// order down, then the three launches above run.
#include "fs_common.h"
#include "fs_device.h"

namespace fs {

// ---- FBS: the deal ------------------------------------------------------------------------------------
// full rounds R = B / n, m = B % n samples in the last, partial round (round R): forth if R is even
// (ranks 0..m-1 get one more), back if R is odd (ranks n-m..n-1 get one more)
__device__ __forceinline__ int64_t fbs_rank_start(int64_t i, int64_t n, int64_t R, int64_t m) {
    const int64_t extra = (R % 2 == 0) ? (i < m ? i : m) : (i > n - m ? i - (n - m) : 0);
    return i * R + extra;
}

__global__ __launch_bounds__(256) void fbs_deal_kernel(const int32_t *__restrict__ sorted, int64_t B, int64_t n,
                                                       int32_t *__restrict__ sample_of,
                                                       int64_t *__restrict__ rank_offsets) {
    const int64_t R = B / n, m = B % n;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = gtid; i <= n; i += stride) rank_offsets[i] = fbs_rank_start(i, n, R, m);
    for (int64_t s = gtid; s < B; s += stride) {
        const int64_t r = s / n, c = s % n;
        const int64_t i = (r % 2 == 0) ? c : n - 1 - c;
        sample_of[fbs_rank_start(i, n, R, m) + r] = sorted[s];
    }
}

int launch_partition_fbs(fs_ctx *ctx, const int64_t *lengths, int64_t B, int64_t max_len, int32_t n_ranks,
                         int32_t *sample_of, int64_t *rank_offsets, hipStream_t s) {
    if (B > 0) {
        const int rc = launch_unique(ctx, lengths, B, max_len + 1, ctx->jag_unique, ctx->jag_seg, ctx->jag_sorted,
                                     nullptr, ctx->jag_n, s, 0);
        if (rc != FS_OK) return rc;
    }
    const int64_t work = B > n_ranks ? B : (int64_t)n_ranks + 1;
    int64_t blocks = ceil_div(work, 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fbs_deal_kernel, dim3((unsigned)blocks), dim3(256), 0, s, ctx->jag_sorted, B, (int64_t)n_ranks,
                       sample_of, rank_offsets);
    FS_LAUNCH_CHECK(ctx, "fbs_deal_kernel");
    return FS_OK;
}

// ---- indexed permute ------------------------------------------------------------------------------------
struct jagged_in {
    const int64_t *offsets;   // [B + 1]
    int64_t B, n_values;      // samples, elements behind them
};

// length of output sample k (0 past the end; 0 and a flag for a sample index out of range or a sample whose
// boundaries are not inside the values: such a sample is never read)
__device__ __forceinline__ int64_t out_len(const jagged_in &in, const int32_t *__restrict__ sample_of, int64_t k,
                                           int64_t n_out, bool &bad) {
    if (k >= n_out) return 0;
    const int64_t p = sample_of[k];
    if (p < 0 || p >= in.B) { bad = true; return 0; }
    const int64_t a = in.offsets[p], b = in.offsets[p + 1];
    if (a < 0 || b < a || b > in.n_values) { bad = true; return 0; }
    return b - a;
}

__global__ __launch_bounds__(kScanThreads) void permute_tile_sum_kernel(const jagged_in in,
                                                                        const int32_t *__restrict__ sample_of,
                                                                        int64_t n_out, int64_t *__restrict__ tile_sum,
                                                                        int *__restrict__ flags) {
    __shared__ int64_t sh[kScanThreads / kWave];
    const int64_t k0 = (int64_t)blockIdx.x * kScanTile + threadIdx.x * kScanIpt;
    bool bad = false;
    int64_t v = 0;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) v += out_len(in, sample_of, k0 + i, n_out, bad);
    int64_t total;
    (void)block_exclusive_scan<int64_t>(v, sh, total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
    if (bad) atomicOr(flags, kFlagOffsets);
}

__global__ __launch_bounds__(kScanThreads) void permute_offsets_kernel(const jagged_in in,
                                                                       const int32_t *__restrict__ sample_of,
                                                                       int64_t n_out,
                                                                       const int64_t *__restrict__ tile_sum,
                                                                       int64_t cap_out, int64_t *__restrict__ out_offsets,
                                                                       int *__restrict__ flags) {
    __shared__ int64_t sh[kScanThreads / kWave];
    int64_t before = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += kScanThreads) before += tile_sum[t];
    int64_t tile_base;
    (void)block_exclusive_scan<int64_t>(before, sh, tile_base);
    const int64_t k0 = (int64_t)blockIdx.x * kScanTile + threadIdx.x * kScanIpt;
    bool bad = false;
    int64_t len[kScanIpt], v = 0;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        len[i] = out_len(in, sample_of, k0 + i, n_out, bad);
        v += len[i];
    }
    int64_t tile_total;
    int64_t run = tile_base + block_exclusive_scan<int64_t>(v, sh, tile_total);
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        if (k0 + i < n_out) out_offsets[k0 + i] = run;
        run += len[i];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const int64_t total = tile_base + tile_total;
        out_offsets[n_out] = total;
        if (total > cap_out) atomicOr(flags, kFlagOffsets);     // the copy stops at cap_out
    }
}

// number of entries of a[0, n) that are <= key; executed by one whole wavefront (64-ary search)
__device__ __forceinline__ int64_t wave_upper_bound(const int64_t *__restrict__ a, int64_t n, int64_t key) {
    const int lane = threadIdx.x & (kWave - 1);
    int64_t lo = 0, hi = n;                  // a[i] <= key for i < lo, a[i] > key for i >= hi
    while (lo < hi) {
        const int64_t step = (hi - lo + kWave - 1) / kWave;
        const int64_t probe = lo + (lane + 1) * step - 1;      // last entry of my sub-block
        const bool le = (probe < hi) && (a[probe] <= key);
        const int cnt = __popcll(__ballot(le));
        lo += cnt * step;
        const int64_t nhi = lo + step - 1;
        hi = nhi < hi ? nhi : hi;
    }
    return lo;
}

// pieces per workgroup: the searches that open a tile are a chain of dependent loads, paid once per tile, and
// the chip writes faster the more workgroups share a job.  Measured: 64 KB of output per workgroup for 8-byte
// pieces (16.7 M IDs: 75 us with twice that), 128 KB for 16-byte pieces (250 k rows of 512 bytes: 50 us, and
// 133 us with half of that)
template <typename V> constexpr int copy_tile() { return sizeof(V) == 16 ? 8192 : 4096; }
constexpr int kCopyWindow = 2048 + 2;                           // sample boundaries staged in LDS

// V: the piece, the widest of 4, 8, 16 bytes that divides the element; ppe pieces per element.
// Inside a tile everything is counted from the tile's first element in 32 bits (a 64-bit division per
// piece would cost more than the copy).
template <typename V, int PIECES>
__global__ __launch_bounds__(kScanThreads) void permute_copy_kernel(const V *__restrict__ values, const jagged_in in,
                                                                    const int32_t *__restrict__ sample_of,
                                                                    int64_t n_out, const int64_t *__restrict__ out_offsets,
                                                                    int64_t cap_out, int ppe, V *__restrict__ out) {
    constexpr int kCopyTile = copy_tile<V>();
    __shared__ int32_t w_rel[kCopyWindow];      // out_offsets[ka + j] minus the tile's first element (at least -1)
    __shared__ int64_t w_delta[kCopyWindow];    // first input element of sample ka + j minus its first output element
    __shared__ int64_t win[2];
    const int64_t *__restrict__ offsets = in.offsets;
    int64_t total = out_offsets[n_out];
    if (total > cap_out) total = cap_out;
    const int64_t pieces = total * ppe;
    const int64_t q0 = (int64_t)blockIdx.x * kCopyTile;
    if (q0 >= pieces) return;                                   // whole workgroup
    const uint32_t tile_pieces = (uint32_t)((q0 + kCopyTile < pieces ? q0 + kCopyTile : pieces) - q0);
    const int64_t e0 = q0 / ppe;                                // first element of the tile
    const uint32_t rem0 = (uint32_t)(q0 - e0 * ppe);            // pieces of it that belong to the tile before
    const int64_t e1 = (q0 + tile_pieces - 1) / ppe;            // last element of the tile
    if (threadIdx.x < 2 * kWave) {
        // sample of an element e: the last k with out_offsets[k] <= e (empty samples in between are skipped);
        // the first wavefront looks for the sample of the tile's first element, the second for that of its last
        const int w = threadIdx.x / kWave;
        const int64_t k = wave_upper_bound(out_offsets, n_out + 1, w == 0 ? e0 : e1) - 1;
        if ((threadIdx.x & (kWave - 1)) == 0) win[w] = k;
    }
    __syncthreads();
    const int64_t ka = win[0], kb = win[1];
    const bool staged = kb - ka + 1 <= kCopyWindow;             // else: the samples touched by the tile do not fit
    const int wn = staged ? (int)(kb - ka + 1) : 0;
    if (staged)
        for (int j = threadIdx.x; j < wn; j += kScanThreads) {
            const int64_t start = out_offsets[ka + j];
            const int64_t p = sample_of[ka + j];
            w_rel[j] = start < e0 ? -1 : (int32_t)(start - e0);                // start - e0 <= kCopyTile
            w_delta[j] = (p >= 0 && p < in.B) ? offsets[p] - start : 0;        // a flagged sample is empty: never used
        }
    __syncthreads();
    // Wavefront w copies the w-th quarter of the tile, 64 consecutive pieces per instruction, front to back:
    // the sample of a lane's piece only moves forward, so after one binary search per lane the boundary
    // list is walked (a step every few instructions for samples of a few hundred elements; never more
    // steps per lane and tile than the list is long).
    const uint32_t uppe = (uint32_t)ppe;
    constexpr uint32_t kWavePieces = kCopyTile / (kScanThreads / kWave);
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t w0 = (threadIdx.x / kWave) * kWavePieces;
    const int64_t wn_all = kb - ka + 1;
    int64_t j = 0;                                              // sample ka + j holds the lane's current piece
    {
        const uint32_t t = rem0 + w0 + lane;
        const int64_t le = uppe == 1 ? t : t / uppe;
        int64_t lo = 0, hi = wn_all;                            // first j with start[j] > element
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            const bool le_mid = staged ? (w_rel[mid] <= (int32_t)le) : (out_offsets[ka + mid] <= e0 + le);
            if (le_mid) lo = mid + 1; else hi = mid;
        }
        j = lo - 1;
    }
    static_assert(kWavePieces % (kWave * PIECES) == 0, "a wavefront's quarter is a whole number of rounds");
    for (uint32_t r0 = 0; r0 < kWavePieces; r0 += kWave * PIECES) {
        if (w0 + r0 >= tile_pieces) break;                      // whole wavefront
        V v[PIECES];                                            // 128 bytes per lane in flight whatever the piece
        bool live[PIECES];
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const uint32_t l = w0 + r0 + (uint32_t)i * kWave + lane;                // piece of the tile
            live[i] = l < tile_pieces;
            if (live[i]) {
                const uint32_t t = rem0 + l;
                const uint32_t le = uppe == 1 ? t : t / uppe;                       // element of the tile
                const uint32_t pin = t - le * uppe;                                 // piece of the element
                int64_t delta;
                if (staged) {
                    while (j + 1 < wn_all && w_rel[j + 1] <= (int32_t)le) ++j;
                    delta = w_delta[j];
                } else {
                    const int64_t e = e0 + le;
                    while (j + 1 < wn_all && out_offsets[ka + j + 1] <= e) ++j;
                    delta = offsets[sample_of[ka + j]] - out_offsets[ka + j];
                }
                v[i] = values[(e0 + le + delta) * ppe + pin];
            }
        }
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const uint32_t l = w0 + r0 + (uint32_t)i * kWave + lane;
            if (live[i]) out[q0 + l] = v[i];
        }
    }
}

int launch_indexed_permute(fs_ctx *ctx, const void *values, int64_t n_values, int32_t elem_bytes,
                           const int64_t *offsets, int64_t B, const int32_t *sample_of, int64_t n_out, void *out_values,
                           int64_t cap_out, int64_t *out_offsets, hipStream_t s) {
    const jagged_in in = {offsets, B, n_values};
    const int tiles = (int)(n_out > 0 ? ceil_div(n_out, kScanTile) : 1);
    hipLaunchKernelGGL(permute_tile_sum_kernel, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, in, sample_of,
                       n_out, ctx->jag_tile_sum, ctx->d_flags);
    hipLaunchKernelGGL(permute_offsets_kernel, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, in, sample_of,
                       n_out, ctx->jag_tile_sum, cap_out, out_offsets, ctx->d_flags);
    if (cap_out > 0 && n_out > 0) {
        const int piece = elem_bytes % 16 == 0 ? 16 : (elem_bytes % 8 == 0 ? 8 : 4);
        const int ppe = elem_bytes / piece;
        const int64_t blocks = ceil_div(cap_out * ppe, piece == 16 ? copy_tile<u32x4>() : copy_tile<uint64_t>());
        if (blocks > 0x7fffffffll) return set_err(ctx, FS_EINVAL, "indexed permute: output too large for one launch");
        const dim3 grid((unsigned)blocks);
        if (piece == 16)
            hipLaunchKernelGGL((permute_copy_kernel<u32x4, 8>), grid, dim3(kScanThreads), 0, s, (const u32x4 *)values,
                               in, sample_of, n_out, out_offsets, cap_out, ppe, (u32x4 *)out_values);
        else if (piece == 8)
            hipLaunchKernelGGL((permute_copy_kernel<uint64_t, 16>), grid, dim3(kScanThreads), 0, s, (const uint64_t *)values,
                               in, sample_of, n_out, out_offsets, cap_out, ppe, (uint64_t *)out_values);
        else
            hipLaunchKernelGGL((permute_copy_kernel<uint32_t, 16>), grid, dim3(kScanThreads), 0, s, (const uint32_t *)values,
                               in, sample_of, n_out, out_offsets, cap_out, ppe, (uint32_t *)out_values);
    }
    FS_LAUNCH_CHECK(ctx, "indexed permute kernels");
    return FS_OK;
}

// ---- VBS: cuts of about equal weight --------------------------------------------------------------------
// Sorted position s goes to rank min(n - 1, floor(n * w_before(s) / W)): weights are integers (a table per
// length), so every cut is exact.  Two launches after the sort: weights summed per tile of 1024 sorted
// positions; then every workgroup adds up the tile sums (the total W and its own start), scans its tile and
// writes the start of every rank whose first sample lies in it.
__device__ __forceinline__ int64_t vbs_weight(const int64_t *__restrict__ lengths, const int32_t *__restrict__ sorted,
                                              const int64_t *__restrict__ weight_of_len, int64_t max_len, int64_t s,
                                              int64_t B, bool &bad) {
    if (s < 0 || s >= B) return 0;
    const int64_t len = lengths[sorted[s]];
    if (len < 0 || len > max_len) return 0;              // the sort has reported it already
    const int64_t w = weight_of_len[len];
    if (w < 0) { bad = true; return 0; }
    return w;
}

__global__ __launch_bounds__(kScanThreads) void vbs_tile_sum_kernel(const int64_t *__restrict__ lengths,
                                                                    const int32_t *__restrict__ sorted, int64_t B,
                                                                    const int64_t *__restrict__ weight_of_len,
                                                                    int64_t max_len, int64_t *__restrict__ tile_sum,
                                                                    int *__restrict__ flags) {
    __shared__ int64_t sh[kScanThreads / kWave];
    const int64_t s0 = (int64_t)blockIdx.x * kScanTile + threadIdx.x * kScanIpt;
    bool bad = false;
    int64_t v = 0;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) v += vbs_weight(lengths, sorted, weight_of_len, max_len, s0 + i, B, bad);
    int64_t total;
    (void)block_exclusive_scan<int64_t>(v, sh, total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
    if (bad) atomicOr(flags, kFlagRowRange);
}

__device__ __forceinline__ int64_t vbs_rank(int64_t before, int64_t total, int64_t n) {
    if (total <= 0) return 0;
    const int64_t q = (int64_t)((uint64_t)n * (uint64_t)before / (uint64_t)total);      // n * total < 2^63 (checked)
    return q >= n ? n - 1 : q;
}

__global__ __launch_bounds__(kScanThreads) void vbs_cut_kernel(const int64_t *__restrict__ lengths,
                                                               const int32_t *__restrict__ sorted, int64_t B,
                                                               const int64_t *__restrict__ weight_of_len, int64_t max_len,
                                                               const int64_t *__restrict__ tile_sum, int tiles, int64_t n,
                                                               int64_t *__restrict__ rank_offsets,
                                                               int *__restrict__ flags) {
    __shared__ int64_t sh[kScanThreads / kWave];
    if (B == 0) {                                          // one workgroup: every rank starts (and ends) at 0
        for (int64_t r = threadIdx.x; r <= n; r += kScanThreads) rank_offsets[r] = 0;
        return;
    }
    int64_t mine = 0, all = 0;
    for (int t = threadIdx.x; t < tiles; t += kScanThreads) {
        const int64_t v = tile_sum[t];
        all += v;
        if (t < (int)blockIdx.x) mine += v;
    }
    int64_t tile_base, total;
    (void)block_exclusive_scan<int64_t>(mine, sh, tile_base);
    (void)block_exclusive_scan<int64_t>(all, sh, total);
    if (total < 0 || total > INT64_MAX / n) {              // n * w_before would not fit: refuse, one rank takes all
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(flags, kFlagRowRange);
        total = 0;
    }
    const int64_t s0 = (int64_t)blockIdx.x * kScanTile + threadIdx.x * kScanIpt;
    bool bad = false;
    int64_t w[kScanIpt], v = 0;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        w[i] = vbs_weight(lengths, sorted, weight_of_len, max_len, s0 + i, B, bad);
        v += w[i];
    }
    const int64_t w_prev = vbs_weight(lengths, sorted, weight_of_len, max_len, s0 - 1, B, bad);
    int64_t tile_total;
    int64_t before = tile_base + block_exclusive_scan<int64_t>(v, sh, tile_total);
    // rank of the position before mine (-1 before the first: rank 0 starts at position 0)
    int64_t r_prev = s0 > 0 ? vbs_rank(before - w_prev, total, n) : -1;
#pragma unroll
    for (int i = 0; i < kScanIpt; ++i) {
        const int64_t s = s0 + i;
        if (s < B) {
            const int64_t r = vbs_rank(before, total, n);
            for (int64_t x = r_prev + 1; x <= r; ++x) rank_offsets[x] = s;
            r_prev = r;
            before += w[i];
            if (s == B - 1)
                for (int64_t x = r + 1; x <= n; ++x) rank_offsets[x] = B;
        }
    }
}

int launch_partition_vbs(fs_ctx *ctx, const int64_t *lengths, int64_t B, const int64_t *weight_of_len, int64_t max_len,
                         int32_t n_ranks, int32_t *sample_of, int64_t *rank_offsets, hipStream_t s) {
    const int tiles = (int)(B > 0 ? ceil_div(B, kScanTile) : 1);
    if (B > 0) {
        const int rc = launch_unique(ctx, lengths, B, max_len + 1, ctx->jag_unique, ctx->jag_seg, sample_of, nullptr,
                                     ctx->jag_n, s, 0);
        if (rc != FS_OK) return rc;
        hipLaunchKernelGGL(vbs_tile_sum_kernel, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, lengths, sample_of, B,
                           weight_of_len, max_len, ctx->jag_tile_sum, ctx->d_flags);
    }
    hipLaunchKernelGGL(vbs_cut_kernel, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, lengths, sample_of, B,
                       weight_of_len, max_len, ctx->jag_tile_sum, tiles, (int64_t)n_ranks, rank_offsets, ctx->d_flags);
    FS_LAUNCH_CHECK(ctx, "vbs kernels");
    return FS_OK;
}

// ---- keyed transpose, ranged dispatch, ranged combine ---------------------------------------------------
// Segment (f, b) of a keyed jagged tensor with F keys and B samples is number f * B + b in feature-major
// form and b * F + f in batch-major form.  Ranks own sample ranges [ro[r], ro[r + 1]); what a rank is sent
// (dispatch) or has sent (combine) is a feature-major tensor over its own samples, rank after rank.
enum { kMapTranspose = 0, kMapDispatch = 1, kMapCombine = 2 };

// the last r in [0, n) with scale * ro[r] <= x (ro ascending, ro[0] == 0)
__device__ __forceinline__ int last_rank_at_or_before(const int64_t *__restrict__ ro, int n, int64_t scale, int64_t x) {
    int lo = 0, hi = n;                      // first r with scale * ro[r] > x
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (scale * ro[mid] <= x) lo = mid + 1; else hi = mid;
    }
    return lo > 0 ? lo - 1 : 0;
}

__global__ __launch_bounds__(256) void segment_map_kernel(int mode, int64_t F, int64_t B,
                                                          const int64_t *__restrict__ ro, int n_ranks,
                                                          int32_t *__restrict__ sel, int *__restrict__ flags) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (mode != kMapTranspose) {
        bool bad = false;
        for (int64_t r = gtid; r < n_ranks; r += stride) bad |= ro[r + 1] < ro[r];
        if (gtid == 0) bad |= ro[0] != 0 || ro[n_ranks] != B;
        if (bad) atomicOr(flags, kFlagOffsets);
    }
    for (int64_t j = gtid; j < F * B; j += stride) {
        int64_t in = -1;                     // stays -1 for ranges that make no sense: the copy skips and reports it
        if (mode == kMapTranspose) {
            in = (j % F) * B + j / F;
        } else if (mode == kMapDispatch) {
            const int r = last_rank_at_or_before(ro, n_ranks, F, j);
            const int64_t first = ro[r], cnt = ro[r + 1] - first, local = j - F * first;
            if (cnt > 0 && local >= 0 && local < F * cnt) in = (local / cnt) * B + first + local % cnt;
        } else {
            const int64_t f = j / B, b = j % B;
            const int r = last_rank_at_or_before(ro, n_ranks, 1, b);
            const int64_t first = ro[r], cnt = ro[r + 1] - first;
            if (cnt > 0 && b >= first && b < first + cnt) in = F * first + f * cnt + (b - first);
        }
        sel[j] = (in >= 0 && in < F * B) ? (int32_t)in : -1;
    }
}

// elements each rank is sent: the extent of its F * count segments in the dispatched tensor
__global__ __launch_bounds__(256) void dispatch_splits_kernel(int64_t F, int64_t B, const int64_t *__restrict__ ro,
                                                              int n_ranks, const int64_t *__restrict__ out_offsets,
                                                              int64_t *__restrict__ splits) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n_ranks; r += stride) {
        int64_t a = ro[r], b = ro[r + 1];
        a = a < 0 ? 0 : (a > B ? B : a);
        b = b < a ? a : (b > B ? B : b);
        splits[r] = out_offsets[F * b] - out_offsets[F * a];
    }
}

int launch_keyed_shuffle(fs_ctx *ctx, int mode, const void *values, int64_t n_values, int32_t elem_bytes,
                         const int64_t *offsets, int64_t F, int64_t B, const int64_t *rank_offsets, int32_t n_ranks,
                         void *out_values, int64_t *out_offsets, int64_t *splits, hipStream_t s) {
    const int64_t segs = F * B;
    if (segs > 0) {
        int64_t blocks = ceil_div(segs, 256);
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(segment_map_kernel, dim3((unsigned)blocks), dim3(256), 0, s, mode, F, B, rank_offsets,
                           (int)n_ranks, ctx->jag_sel, ctx->d_flags);
    }
    const int rc = launch_indexed_permute(ctx, values, n_values, elem_bytes, offsets, segs, ctx->jag_sel, segs,
                                          out_values, n_values, out_offsets, s);
    if (rc != FS_OK) return rc;
    if (splits != nullptr && n_ranks > 0) {
        hipLaunchKernelGGL(dispatch_splits_kernel, dim3((unsigned)ceil_div(n_ranks, 256)), dim3(256), 0, s, F, B,
                           rank_offsets, (int)n_ranks, out_offsets, splits);
        FS_LAUNCH_CHECK(ctx, "dispatch_splits_kernel");
    }
    return FS_OK;
}

}  // namespace fs
