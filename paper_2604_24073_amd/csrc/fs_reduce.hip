// Gradient segment reduce (first half of update_embedding(I, G) of Algorithm 2):
//   reduced[k, :] = sum of grads[perm[p], :] over the sorted positions p of distinct row k.
//
// Row popularity is Zipf: half of all occurrences sit in segments longer than a wavefront could
// own, the hottest row alone has tens of thousands.  So the work is cut by POSITION, not by
// segment: every wavefront owns 64 consecutive sorted positions and streams their gradient rows
// (16 bytes per lane, 64/LPR rows per instruction, up to 16 instructions = 16 KB in flight),
// accumulating in fp64.  On gfx9-family hardware loads and stores share one counter, so a
// wavefront that interleaves result stores with its loads cannot keep a second batch in flight;
// bandwidth comes from MANY short-lived wavefronts instead (short chunks, short dependent-load
// chains, first batch requested before the index work).  A 64-bit mask of the positions that
// end a segment drives wave-uniform flushes.  Runs cut by a chunk border go to fp64 partial
// rows, and a second launch adds the partials of each cut segment in a fixed order.  The
// summation order depends on the layout alone: results are reproducible.
#include "fs_common.h"
#include "fs_device.h"

namespace fs {

#ifndef FS_REDUCE_UNR
#define FS_REDUCE_UNR 4
#endif
constexpr int kFixThreads = 1024;
constexpr int kDescInts = 4;   // per chunk: first segment, number of flushes, last chunk of the cut segment that
                               // starts here (-1: none), flags
template <int LPR, int UNR, bool HAS_INV>
__global__ __launch_bounds__(kReduceWavesPerBlock *kWave) void reduce_chunk_kernel(
    const f32x4 *__restrict__ grads, int n, int gvec, const int32_t *__restrict__ perm,
    const int32_t *__restrict__ seg_offsets, const int32_t *__restrict__ inverse,
    const int64_t *__restrict__ n_unique_dev, f32x4 *__restrict__ reduced,
    double *__restrict__ part_head, double *__restrict__ part_last, int32_t *__restrict__ chunk_desc) {
    constexpr int GPW = kWave / LPR;          // rows per wavefront instruction
    constexpr int BP = GPW * UNR;             // positions per batch
    constexpr int NB = kReduceChunk / BP;     // batches per chunk
    static_assert(kReduceChunk == kWave && kReduceChunk % BP == 0, "one tail word, whole batches");
    __shared__ uint32_t tail_bits[kReduceWavesPerBlock][2];

    const int lane = threadIdx.x & (kWave - 1);
    const int wib = threadIdx.x / kWave;
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const int chunk = blockIdx.x * kReduceWavesPerBlock + wib;
    const int a = chunk * kReduceChunk;
    const bool active = a < n;                               // wave-uniform
    const int b = active ? ((a + kReduceChunk < n) ? a + kReduceChunk : n) : a;
    const int span = b - a;
    const bool col_ok = lig < gvec;

    // the gradient rows of the first batch are requested before anything else: the index work
    // below (search of the first segment, tail mask) then runs under their latency
    const int pr = (lane < span) ? perm[a + lane] : 0;
    int edge = 0;                                            // lane 0: position a-1, lane 1: position b
    if (HAS_INV && active && lane == 0 && a > 0) edge = perm[a - 1];
    if (HAS_INV && active && lane == 1 && b < n) edge = perm[b];
    auto load_batch = [&](f32x4(&v)[UNR], int k) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int q = k * BP + u * GPW + grp;             // position inside the chunk
            const int p = __shfl(pr, q, kWave);
            v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (col_ok && q < span) v[u] = __builtin_nontemporal_load(&grads[(int64_t)p * gvec + lig]);
        }
    };
    f32x4 v[UNR];
    load_batch(v, 0);

    int s0 = 0;
    bool head_complete = false;
    uint64_t tails = 0;
    if (HAS_INV) {
        // Segment of every position straight from the inverse map (one gathered 4-byte load per
        // position, issued together with the first batch of rows): a position ends a segment iff
        // its successor belongs to another one.  No search, no LDS, one dependent round.
        if (!active) return;
        const int inv = (lane < span) ? inverse[pr] : -1;
        const int inv_edge = (lane < 2) ? inverse[edge] : -1;
        const int inv_prev = __shfl(inv_edge, 0, kWave), inv_after = __shfl(inv_edge, 1, kWave);
        int nxt = __shfl_down(inv, 1, kWave);
        if (lane == span - 1) nxt = (b < n) ? inv_after : -1;
        tails = __ballot(lane < span && nxt != inv);
        s0 = __shfl(inv, 0, kWave);
        head_complete = (a == 0) || (inv_prev != s0);
    } else {
    const int U = (int)*n_unique_dev;
    if (lane < 2) tail_bits[wib][lane] = 0;
    // first segment of the chunk: the largest s with seg_offsets[s] <= a (64-ary search)
    if (active) {
        int lo = 0, hi = U;                                  // seg_offsets[lo] <= a < seg_offsets[hi]
        while (hi - lo > 1) {
            const int step = (hi - lo + kWave - 1) / kWave;
            const int probe = lo + (lane + 1) * step;
            const bool le = (probe < hi) && (seg_offsets[probe] <= a);
            const int cnt = __popcll(__ballot(le));
            const int nlo = lo + cnt * step;
            const int nhi = lo + (cnt + 1) * step;
            lo = nlo;
            hi = nhi < hi ? nhi : hi;
        }
        s0 = lo;
    }
    __syncthreads();
    if (active) {
        // segment ends inside (a, b]: at most 64 of them, strictly increasing
        const int s = s0 + 1 + lane;
        if (s <= U) {
            const int e = seg_offsets[s];
            if (e <= b) {
                const int bit = e - 1 - a;
                atomicOr(&tail_bits[wib][bit >> 5], 1u << (bit & 31));
            }
        }
        head_complete = seg_offsets[s0] == a;
    }
    __syncthreads();
    if (!active) return;
    const uint32_t w0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)tail_bits[wib][0]);
    const uint32_t w1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)tail_bits[wib][1]);
    tails = (uint64_t)w0 | ((uint64_t)w1 << 32);
    }
    s0 = __builtin_amdgcn_readfirstlane(s0);

    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    int seg = s0;
    int nflush = 0;
    const int dim = gvec * 4;

    auto flush = [&]() {
        double t[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = across_groups<LPR>(acc[c]);
        if (grp == 0 && col_ok) {
            if (nflush == 0 && !head_complete) {
                double *dst = part_head + (int64_t)chunk * dim + lig * 4;
#pragma unroll
                for (int c = 0; c < 4; ++c) dst[c] = t[c];
            } else {
                reduced[(int64_t)seg * gvec + lig] = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = 0.0;
        ++seg;
        ++nflush;
    };
    auto add_batch = [&](const f32x4(&vv)[UNR], int k) {
        const uint64_t shifted = tails >> ((k * BP) & 63);
        const uint64_t batch_tails = (BP == kWave) ? shifted : (shifted & ((1ull << (BP & 63)) - 1ull));
        if (batch_tails == 0) {                               // no segment ends in this batch
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] += (double)vv[u][c];
            return;
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint64_t tb = (batch_tails >> (u * GPW)) & (GPW == kWave ? ~0ull : ((1ull << (GPW & 63)) - 1ull));
            if (tb == 0) {
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] += (double)vv[u][c];
            } else {
#pragma unroll
                for (int g = 0; g < GPW; ++g) {
                    if (grp == g) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[c] += (double)vv[u][c];
                    }
                    if ((tb >> g) & 1ull) flush();
                }
            }
        }
    };

    add_batch(v, 0);
    for (int k = 1; k < NB; ++k) {
        if (k * BP >= span) break;                            // wave-uniform: ragged last chunk
        load_batch(v, k);
        add_batch(v, k);
    }

    // positions after the last segment end of the chunk (the chunk's last position is not a tail)
    const bool has_rest = ((tails >> (span - 1)) & 1ull) == 0;
    if (has_rest) {
        double t[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = across_groups<LPR>(acc[c]);
        if (grp == 0 && col_ok) {
            double *dst = (nflush == 0 ? part_head : part_last) + (int64_t)chunk * dim + lig * 4;
#pragma unroll
            for (int c = 0; c < 4; ++c) dst[c] = t[c];
        }
    }
    if (lane == 0) {
        // the second launch wants everything about this chunk's cut in ONE load: where the cut
        // segment (if one starts here) ends is looked up now, at the end of a wavefront's life
        const bool starts_cut = has_rest && (nflush != 0 || head_complete);
        const int c_last = starts_cut ? (seg_offsets[s0 + nflush + 1] - 1) / kReduceChunk : -1;
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        *reinterpret_cast<i32x4 *>(chunk_desc + (int64_t)chunk * kDescInts) =
            i32x4{s0, nflush, c_last, (head_complete ? 1 : 0) | (has_rest ? 2 : 0)};
    }
}

// Second launch: every cut segment gets its partial rows added in a fixed order.  One wavefront
// looks at one chunk; if a cut segment STARTS there, its partials are the chunk's own tail (or
// whole-chunk) partial plus the head partial of every later chunk it covers.  Short spans are
// finished by the wavefront itself (its 64/LPR groups fetch eight partial rows each per round);
// the few long ones (hot rows cover hundreds of chunks) are listed in LDS and then added by all
// groups of the workgroup together.  The order of the additions depends only on the layout.
constexpr int kFixWaves = kFixThreads / kWave;
constexpr int kFixLongSpan = 32;              // partial rows beyond which the whole workgroup helps

template <int LPR>
__device__ __forceinline__ void add_partials(double (&t)[4], const double *__restrict__ part_head, int dim, int lig,
                                             bool col_ok, int c_begin, int c_last, int stride, int fallback) {
    for (int c = c_begin; c <= c_last; c += 8 * stride) {
        double h[8][4];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int cj = c + j * stride;
            const bool ok = col_ok && cj <= c_last;
            const double *src = part_head + (int64_t)(ok ? cj : fallback) * dim + lig * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[j][i] = ok ? src[i] : 0.0;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) t[i] += h[j][i];
    }
}

template <int LPR>
__global__ __launch_bounds__(kFixThreads) void reduce_fix_kernel(int n_chunks, int gvec,
                                                         const int32_t *__restrict__ seg_offsets,
                                                         const double *__restrict__ part_head,
                                                         const double *__restrict__ part_last,
                                                         const int32_t *__restrict__ chunk_desc,
                                                         f32x4 *__restrict__ reduced) {
    constexpr int GPW = kWave / LPR;
    constexpr int GROUPS = kFixThreads / LPR;
    __shared__ double red[kFixThreads * 4];
    __shared__ int long_list[kFixWaves][3];       // chunk, segment, last chunk
    __shared__ int n_long;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const bool col_ok = lig < gvec;
    const int dim = gvec * 4;
    if (threadIdx.x == 0) n_long = 0;
    __syncthreads();

    const int chunk = blockIdx.x * kFixWaves + w;
    if (chunk < n_chunks) {
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        const i32x4 d = *reinterpret_cast<const i32x4 *>(chunk_desc + (int64_t)chunk * kDescInts);
        const int s0 = d[0], nflush = d[1], c_last = d[2];
        // c_last >= 0: a cut segment starts here (the chunk ends inside a run that began in it)
        if (c_last >= 0) {
            const int seg = s0 + nflush;
            if (c_last - chunk > kFixLongSpan) {
                if (lane == 0) {
                    const int slot = atomicAdd(&n_long, 1);
                    long_list[slot][0] = chunk;
                    long_list[slot][1] = seg;
                    long_list[slot][2] = c_last;
                }
            } else {
                double t[4] = {0.0, 0.0, 0.0, 0.0};
                if (grp == 0 && col_ok) {
                    const double *x = (nflush == 0 ? part_head : part_last) + (int64_t)chunk * dim + lig * 4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) t[i] = x[i];
                }
                add_partials<LPR>(t, part_head, dim, lig, col_ok, chunk + 1 + grp, c_last, GPW, chunk);
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] = across_groups<LPR>(t[i]);
                if (grp == 0 && col_ok)
                    reduced[(int64_t)seg * gvec + lig] = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
            }
        }
    }
    __syncthreads();
    // long spans: all groups of the workgroup, one span after the other (slot order is irrelevant
    // for the values: every span is summed in the same fixed group/stride order)
    const int bg = threadIdx.x / LPR;             // group index inside the workgroup
    for (int k = 0; k < n_long; ++k) {
        const int ch = long_list[k][0], seg = long_list[k][1], c_last = long_list[k][2];
        double t[4] = {0.0, 0.0, 0.0, 0.0};
        if (bg == 0 && col_ok) {
            const int32_t *d = chunk_desc + (int64_t)ch * kDescInts;
            const double *x = (d[1] == 0 ? part_head : part_last) + (int64_t)ch * dim + lig * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) t[i] = x[i];
        }
        add_partials<LPR>(t, part_head, dim, lig, col_ok, ch + 1 + bg, c_last, GROUPS, ch);
#pragma unroll
        for (int i = 0; i < 4; ++i) red[(bg * LPR + lig) * 4 + i] = t[i];
        __syncthreads();
        if (bg == 0 && col_ok) {
            for (int g = 1; g < GROUPS; ++g)
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] += red[(g * LPR + lig) * 4 + i];
            reduced[(int64_t)seg * gvec + lig] = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
        }
        __syncthreads();
    }
}

template <int LPR>
static void reduce_launch(fs_ctx *ctx, const float *grads, int n, int gvec, const int32_t *perm,
                          const int32_t *seg_offsets, const int64_t *n_unique_dev, float *reduced, hipStream_t s,
                          hipEvent_t *timing) {
    constexpr int GPW = kWave / LPR;
    // row-group loads one wavefront issues per round (build-time tuning knob)
    constexpr int UNR = (kReduceChunk / GPW) < FS_REDUCE_UNR ? (kReduceChunk / GPW) : FS_REDUCE_UNR;
    const int n_chunks = (int)ceil_div(n, kReduceChunk);
    const int blocks = (int)ceil_div(n_chunks, kReduceWavesPerBlock);
    const int32_t *inverse = ctx->reduce_inverse;            // optional accelerator, set by the caller
    if (timing) (void)hipEventRecord(timing[0], s);
    if (inverse)
        hipLaunchKernelGGL((reduce_chunk_kernel<LPR, UNR, true>), dim3(blocks), dim3(kReduceWavesPerBlock * kWave), 0,
                           s, (const f32x4 *)grads, n, gvec, perm, seg_offsets, inverse, n_unique_dev,
                           (f32x4 *)reduced, ctx->part_head, ctx->part_last, ctx->chunk_desc);
    else
        hipLaunchKernelGGL((reduce_chunk_kernel<LPR, UNR, false>), dim3(blocks), dim3(kReduceWavesPerBlock * kWave),
                           0, s, (const f32x4 *)grads, n, gvec, perm, seg_offsets, inverse, n_unique_dev,
                           (f32x4 *)reduced, ctx->part_head, ctx->part_last, ctx->chunk_desc);
    if (timing) (void)hipEventRecord(timing[1], s);
    hipLaunchKernelGGL((reduce_fix_kernel<LPR>), dim3((unsigned)ceil_div(n_chunks, kFixWaves)), dim3(kFixThreads), 0, s, n_chunks, gvec,
                       seg_offsets, (const double *)ctx->part_head, (const double *)ctx->part_last,
                       (const int32_t *)ctx->chunk_desc, (f32x4 *)reduced);
}

int launch_reduce(fs_ctx *ctx, const float *grads, int64_t n, int32_t dim, const int32_t *perm,
                  const int32_t *seg_offsets, const int64_t *n_unique_dev, float *reduced, hipStream_t s,
                  hipEvent_t *timing) {
    if (n == 0) return FS_OK;
    const int gvec = dim / 4;
    switch (lanes_per_row(gvec)) {
        case 1: reduce_launch<1>(ctx, grads, (int)n, gvec, perm, seg_offsets, n_unique_dev, reduced, s, timing); break;
        case 2: reduce_launch<2>(ctx, grads, (int)n, gvec, perm, seg_offsets, n_unique_dev, reduced, s, timing); break;
        case 4: reduce_launch<4>(ctx, grads, (int)n, gvec, perm, seg_offsets, n_unique_dev, reduced, s, timing); break;
        case 8: reduce_launch<8>(ctx, grads, (int)n, gvec, perm, seg_offsets, n_unique_dev, reduced, s, timing); break;
        case 16: reduce_launch<16>(ctx, grads, (int)n, gvec, perm, seg_offsets, n_unique_dev, reduced, s, timing); break;
        case 32: reduce_launch<32>(ctx, grads, (int)n, gvec, perm, seg_offsets, n_unique_dev, reduced, s, timing); break;
        case 64: reduce_launch<64>(ctx, grads, (int)n, gvec, perm, seg_offsets, n_unique_dev, reduced, s, timing); break;
        default: return set_err(ctx, FS_EINVAL, "reduce: dim beyond 256");
    }
    FS_LAUNCH_CHECK(ctx, "reduce kernels");
    return FS_OK;
}

}  // namespace fs
