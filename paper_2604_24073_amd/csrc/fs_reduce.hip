// Gradient segment reduce (first half of update_embedding(I, G) of Algorithm 2):
//   reduced[k, :] = sum of grads[perm[p], :] over the sorted positions p of distinct row k.
//
// Row popularity is Zipf: half of all occurrences sit in segments longer than a wavefront could
// own, the hottest row alone has tens of thousands.  So the work is cut by POSITION, not by
// segment: every wavefront owns kReduceChunk consecutive sorted positions and streams their
// gradient rows (16 bytes per lane, 64/LPR rows per instruction, UNR instructions in flight),
// accumulating in fp64.  A 128-bit tail mask (which positions end a segment) drives wave-uniform
// flushes.  Runs that are cut by a chunk border go to fp64 partial rows, and a second launch
// adds the partials of each cut segment in chunk order.  The summation order is fixed by the
// layout alone, so results are reproducible.
#include "fs_common.h"

namespace fs {

constexpr int kDescInts = 4;   // per chunk: first segment, number of flushes, head run complete, has tail run

template <int LPR>
__device__ __forceinline__ double across_groups(double x) {
#pragma unroll
    for (int m = LPR; m < kWave; m <<= 1) x += __shfl_xor(x, m, kWave);
    return x;
}

template <int LPR, int UNR>
__global__ __launch_bounds__(kReduceWavesPerBlock *kWave) void reduce_chunk_kernel(
    const f32x4 *__restrict__ grads, int n, int gvec, const int32_t *__restrict__ perm,
    const int32_t *__restrict__ seg_offsets, const int64_t *__restrict__ n_unique_dev, f32x4 *__restrict__ reduced,
    double *__restrict__ part_head, double *__restrict__ part_last, int32_t *__restrict__ chunk_desc) {
    constexpr int GPW = kWave / LPR;
    constexpr int ITERS = kReduceChunk / GPW;
    static_assert(kReduceChunk == 128, "tail mask is two 64-bit words");
    static_assert(ITERS % UNR == 0, "unroll must divide the chunk");
    __shared__ uint32_t tail_bits[kReduceWavesPerBlock][4];

    const int lane = threadIdx.x & (kWave - 1);
    const int wib = threadIdx.x / kWave;
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const int chunk = blockIdx.x * kReduceWavesPerBlock + wib;
    const int a = chunk * kReduceChunk;
    const bool active = a < n;                               // wave-uniform
    const int b = active ? ((a + kReduceChunk < n) ? a + kReduceChunk : n) : a;
    const int U = (int)*n_unique_dev;

    if (lane < 4) tail_bits[wib][lane] = 0;
    // first segment of the chunk: the largest s with seg_offsets[s] <= a (64-ary search)
    int s0 = 0;
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
    bool head_complete = false;
    if (active) {
        // segment ends inside (a, b]: at most kReduceChunk of them, strictly increasing
#pragma unroll
        for (int i = 0; i < kReduceChunk / kWave; ++i) {
            const int s = s0 + 1 + i * kWave + lane;
            if (s <= U) {
                const int e = seg_offsets[s];
                if (e <= b) {
                    const int bit = e - 1 - a;
                    atomicOr(&tail_bits[wib][bit >> 5], 1u << (bit & 31));
                }
            }
        }
        head_complete = seg_offsets[s0] == a;
    }
    __syncthreads();
    if (!active) return;
    uint64_t tails[2];
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (uint32_t)__builtin_amdgcn_readfirstlane((int)tail_bits[wib][i]);
        tails[0] = (uint64_t)w[0] | ((uint64_t)w[1] << 32);
        tails[1] = (uint64_t)w[2] | ((uint64_t)w[3] << 32);
    }

    // this chunk's slice of the permutation, one or two entries per lane
    int pr[kReduceChunk / kWave];
#pragma unroll
    for (int i = 0; i < kReduceChunk / kWave; ++i) {
        const int p = a + i * kWave + lane;
        pr[i] = (p < b) ? perm[p] : 0;
    }

    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    int seg = s0;
    int nflush = 0;
    const bool col_ok = lig < gvec;
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

    for (int it0 = 0; it0 < ITERS; it0 += UNR) {
        if (a + it0 * GPW >= b) break;                        // wave-uniform: ragged last chunk
        f32x4 v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int q0 = (it0 + u) * GPW;                   // wave-uniform first position of this instruction
            const int src = (q0 < kWave) ? pr[0] : pr[1];
            const int p = __shfl(src, (q0 & (kWave - 1)) + grp, kWave);
            v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (col_ok && (a + q0 + grp) < b) v[u] = __builtin_nontemporal_load(&grads[(int64_t)p * gvec + lig]);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int q0 = (it0 + u) * GPW;
            const uint64_t tw = (q0 < kWave) ? tails[0] : tails[1];
            const uint64_t tb = (tw >> (q0 & 63)) & (GPW == kWave ? ~0ull : ((1ull << (GPW & 63)) - 1ull));
            if (tb == 0) {
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] += (double)v[u][c];
            } else {
#pragma unroll
                for (int g = 0; g < GPW; ++g) {
                    if (grp == g) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[c] += (double)v[u][c];
                    }
                    if ((tb >> g) & 1ull) flush();
                }
            }
        }
    }
    // positions after the last segment end of the chunk (the chunk's last position is not a tail)
    const int last_bit = b - 1 - a;
    const bool has_rest = ((((last_bit < kWave) ? tails[0] : tails[1]) >> (last_bit & 63)) & 1ull) == 0;
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
        int32_t *d = chunk_desc + (int64_t)chunk * kDescInts;
        d[0] = s0;
        d[1] = nflush;
        d[2] = head_complete ? 1 : 0;
        d[3] = has_rest ? 1 : 0;
    }
}

// One group of LPR lanes per chunk: if a cut segment STARTS in this chunk, add its partial rows in
// chunk order and write the reduced row.
template <int LPR>
__global__ __launch_bounds__(256) void reduce_fix_kernel(int n_chunks, int gvec, const int32_t *__restrict__ seg_offsets,
                                                         const double *__restrict__ part_head,
                                                         const double *__restrict__ part_last,
                                                         const int32_t *__restrict__ chunk_desc,
                                                         f32x4 *__restrict__ reduced) {
    constexpr int GPW = kWave / LPR;
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const int chunk = (blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave) * GPW + grp;
    if (chunk >= n_chunks || lig >= gvec) return;
    const int dim = gvec * 4;
    const int32_t *d = chunk_desc + (int64_t)chunk * kDescInts;
    const int s0 = d[0], nflush = d[1], head_complete = d[2], has_rest = d[3];
    if (!has_rest) return;
    if (nflush == 0 && !head_complete) return;               // interior of a segment that started earlier
    const int seg = s0 + nflush;
    const double *x = (nflush == 0 ? part_head : part_last) + (int64_t)chunk * dim + lig * 4;
    double t[4] = {x[0], x[1], x[2], x[3]};
    const int c_last = (seg_offsets[seg + 1] - 1) / kReduceChunk;
    // partial rows are fetched eight at a time (independent loads) and added in chunk order
    for (int c = chunk + 1; c <= c_last; c += 8) {
        double h[8][4];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int cj = (c + j <= c_last) ? c + j : c_last;
            const double *src = part_head + (int64_t)cj * dim + lig * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[j][i] = src[i];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (c + j <= c_last) {
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] += h[j][i];
            }
        }
    }
    reduced[(int64_t)seg * gvec + lig] = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
}

template <int LPR>
static void reduce_launch(fs_ctx *ctx, const float *grads, int n, int gvec, const int32_t *perm,
                          const int32_t *seg_offsets, const int64_t *n_unique_dev, float *reduced, hipStream_t s,
                          hipEvent_t *timing) {
    constexpr int GPW = kWave / LPR;
    constexpr int UNR = (kReduceChunk / GPW) < 8 ? (kReduceChunk / GPW) : 8;
    const int n_chunks = (int)ceil_div(n, kReduceChunk);
    const int blocks = (int)ceil_div(n_chunks, kReduceWavesPerBlock);
    if (timing) (void)hipEventRecord(timing[0], s);
    hipLaunchKernelGGL((reduce_chunk_kernel<LPR, UNR>), dim3(blocks), dim3(kReduceWavesPerBlock * kWave), 0, s,
                       (const f32x4 *)grads, n, gvec, perm, seg_offsets, n_unique_dev, (f32x4 *)reduced,
                       ctx->part_head, ctx->part_last, ctx->chunk_desc);
    if (timing) (void)hipEventRecord(timing[1], s);
    const int chunks_per_block = 4 * GPW;
    hipLaunchKernelGGL((reduce_fix_kernel<LPR>), dim3((unsigned)ceil_div(n_chunks, chunks_per_block)), dim3(256), 0, s,
                       n_chunks, gvec, seg_offsets, (const double *)ctx->part_head, (const double *)ctx->part_last,
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
