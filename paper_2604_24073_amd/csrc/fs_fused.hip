// update_embedding(I, G) of Algorithm 2 for ONE class of rows (collision rows = priority pass,
// exclusive rows = deferred pass) in a single launch: gradient segment reduce and row-wise
// Adagrad fused, so the summed gradient of a row never travels through HBM.
//
// The index half of the step has laid the occurrences of the batch out class by class
// ("class order": all occurrences of collision rows first, then those of exclusive rows; inside a
// class by ascending row, inside a row in batch order).  A launch walks the positions of its
// class only, so the priority pass reads exactly the gradient rows of collision rows.
//
// Work is cut by POSITION (row popularity is Zipf, the hottest row has tens of thousands of
// occurrences): one wavefront owns 64 consecutive class positions, streams their gradient rows
// (16 bytes per lane, 64/LPR rows per instruction) into fp64 accumulators and, whenever a segment
// ends, parks the finished sum (rounded once to fp32) in LDS.  Parked rows are updated in rounds
// of eight or more, so the dependent loads of the update (table row, accumulator) of many rows
// are in flight together.  A segment cut by a chunk border leaves fp64 partial rows; every
// wavefront that contributed one counts itself in at the segment's counter, and the one that
// arrives last adds the partials in chunk order and updates the row.  No wavefront ever waits for
// another, and the order of every floating-point sum depends on the layout alone.
#include "fs_common.h"
#include "fs_device.h"

namespace fs {

#ifndef FS_FUSED_UNR
#define FS_FUSED_UNR 4
#endif
constexpr int kFusedWaves = 4;             // wavefronts per workgroup (they never synchronise)
constexpr int kFusedRound = 8;             // parked rows that trigger an update round

// Adagrad on `nrows` parked rows of one wavefront.  Group g of the wavefront takes rows g, g+GPW, ...
// stage: [row][LPR] fp32 sums (4 columns per lane), stage_row: table row, stage_slot: slot in U_t.
template <bool BF16, int LPR, int RU>
__device__ __forceinline__ void update_parked(const f32x4 *stage, const int64_t *stage_row, const int *stage_slot,
                                              int nrows, void *table, float *state, int64_t num_rows, int gvec,
                                              float lr, float eps, f32x4 *reduced, bool &oob) {
#pragma clang fp contract(off)
    constexpr int GPW = kWave / LPR;
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const bool col_ok = lig < gvec;
    const int dim = gvec * 4;
    u32x4 *t4 = reinterpret_cast<u32x4 *>(table);
    u32x2 *t2 = reinterpret_cast<u32x2 *>(table);
    for (int base = 0; base < nrows; base += GPW * RU) {
        int64_t r[RU];
        int k[RU];
        bool live[RU];
        f32x4 g[RU];
        u32x4 w[RU];
        float s_old[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int kk = base + u * GPW + grp;
            const bool in_list = kk < nrows;
            r[u] = in_list ? stage_row[kk] : 0;
            k[u] = in_list ? stage_slot[kk] : 0;
            g[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (in_list && col_ok) g[u] = stage[kk * LPR + lig];
            const bool in_table = (r[u] >= 0) && (r[u] < num_rows);
            oob |= in_list && !in_table;
            live[u] = in_list && in_table;
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            w[u] = u32x4{0u, 0u, 0u, 0u};
            if (live[u] && col_ok) {
                if (BF16) {
                    const u32x2 h = t2[r[u] * gvec + lig];
                    w[u][0] = h[0];
                    w[u][1] = h[1];
                } else {
                    w[u] = t4[r[u] * gvec + lig];
                }
            }
            s_old[u] = live[u] ? state[r[u]] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            double ss = 0.0;
#pragma unroll
            for (int c = 0; c < 4; ++c) ss += (double)g[u][c] * (double)g[u][c];
            ss = group_sum<LPR>(ss);
            const float m = (float)(ss / (double)dim);
            const float s_new = s_old[u] + m;
            const float c_step = __fdiv_rn(lr, __fsqrt_rn(s_new) + eps);
            const bool mine = live[u] && col_ok;
            if (BF16) {
                const float c0 = bf16_lo(w[u][0]) - c_step * g[u][0];
                const float c1 = bf16_hi(w[u][0]) - c_step * g[u][1];
                const float c2 = bf16_lo(w[u][1]) - c_step * g[u][2];
                const float c3 = bf16_hi(w[u][1]) - c_step * g[u][3];
                const u32x2 o = {f32_to_bf16_bits(c0) | (f32_to_bf16_bits(c1) << 16),
                                 f32_to_bf16_bits(c2) | (f32_to_bf16_bits(c3) << 16)};
                if (mine) t2[r[u] * gvec + lig] = o;
            } else {
                u32x4 o;
#pragma unroll
                for (int c = 0; c < 4; ++c) o[c] = __float_as_uint(__uint_as_float(w[u][c]) - c_step * g[u][c]);
                if (mine) t4[r[u] * gvec + lig] = o;
            }
            if (live[u] && lig == 0) state[r[u]] = s_new;
            if (reduced != nullptr && mine) reduced[(int64_t)k[u] * gvec + lig] = g[u];
        }
    }
}

// t += part[c] for c = c_begin, c_begin + stride, ... <= c_last (eight rows requested per round)
__device__ __forceinline__ void add_partial_rows(double (&t)[4], const double *part, int dim, int lig, bool col_ok,
                                                 int c_begin, int c_last, int stride) {
    for (int c = c_begin; c <= c_last; c += 8 * stride) {
        double h[8][4];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int cj = c + j * stride;
            const bool ok = col_ok && cj <= c_last;
            const double *src = part + (int64_t)(ok ? cj : c_begin) * dim + lig * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[j][i] = ok ? src[i] : 0.0;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) t[i] += h[j][i];
    }
}

// wave-private LDS hand-over between lanes: order the accesses for the compiler and the hardware
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <bool BF16, int LPR, int UNR>
__global__ __launch_bounds__(kFusedWaves *kWave) void reduce_update_kernel(
    const f32x4 *__restrict__ grads, const int32_t *__restrict__ cperm, const int32_t *__restrict__ cslot,
    const int32_t *__restrict__ class_pos, int cls, int n, const int32_t *__restrict__ seg_offsets,
    const int32_t *__restrict__ cstart, const int64_t *__restrict__ u_t, void *table, float *state, int64_t num_rows,
    int gvec, float lr, float eps, f32x4 *reduced, double *part_head, double *part_last, int *counters, int *flags) {
    constexpr int GPW = kWave / LPR;          // rows per wavefront instruction
    constexpr int BP = GPW * UNR;             // positions per batch
    constexpr int NB = kWave / BP;            // batches per chunk
    constexpr int ROUND = GPW > kFusedRound ? GPW : kFusedRound;
    constexpr int CAP = ROUND + BP;           // a batch can park BP more rows before the next check
    constexpr int RU = (ROUND / GPW) < 4 ? ((ROUND / GPW) < 1 ? 1 : (ROUND / GPW)) : 4;
    static_assert(kWave % BP == 0, "whole batches");
    __shared__ f32x4 stage[kFusedWaves][CAP * LPR];
    __shared__ int64_t stage_row[kFusedWaves][CAP];
    __shared__ int stage_slot[kFusedWaves][CAP];

    const int lane = threadIdx.x & (kWave - 1);
    const int wib = threadIdx.x / kWave;
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    int lo = cls == 0 ? 0 : class_pos[0];
    int hi = cls == 0 ? class_pos[0] : class_pos[1];
    // A consistent class order never trips the range checks below; they turn a corrupted one into
    // an error flag instead of a wild access.
    if (lo < 0) lo = 0;
    if (hi > n) hi = n;
    const int chunk = blockIdx.x * kFusedWaves + wib;        // chunk number inside the class
    const int64_t a64 = (int64_t)lo + (int64_t)chunk * kWave;
    if (a64 >= hi) return;                                   // wave-uniform; wavefronts share nothing
    const int a = (int)a64;
    const int b = (a + kWave < hi) ? a + kWave : hi;
    const int span = b - a;
    const bool col_ok = lig < gvec;
    const int dim = gvec * 4;

    int pr = (lane < span) ? cperm[a + lane] : 0;
    int sl = (lane < span) ? cslot[a + lane] : -1;
    bool bad = (lane < span) && ((unsigned)pr >= (unsigned)n || (unsigned)sl >= (unsigned)n);
    if (bad) { pr = 0; sl = 0; }
    int edge = -1;                                           // lane 0: slot of position a-1, lane 1: of position b
    if (lane == 0 && a > lo) edge = cslot[a - 1];
    if (lane == 1 && b < hi) edge = cslot[b];
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
    const int64_t rid = (lane < span) ? u_t[sl] : 0;          // table row of every position (used where a segment ends)

    const int sl_prev = __shfl(edge, 0, kWave), sl_after = __shfl(edge, 1, kWave);
    int nxt = __shfl_down(sl, 1, kWave);
    if (lane == span - 1) nxt = sl_after;
    const uint64_t tails = __ballot(lane < span && nxt != sl);
    const int s_first = __builtin_amdgcn_readfirstlane(sl);
    const bool head_complete = (a == lo) || (sl_prev != s_first);

    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    int nflush = 0;
    int nparked = 0;
    bool oob = false;
    const int n_chunks = (n + kWave - 1) / kWave;

    auto flush = [&](int q) {                                 // the segment that ends at chunk position q
        double t[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = across_groups<LPR>(acc[c]);
        if (nflush == 0 && !head_complete) {
            if (grp == 0 && col_ok) {
                double *dst = part_head + (int64_t)chunk * dim + lig * 4;
#pragma unroll
                for (int c = 0; c < 4; ++c) dst[c] = t[c];
            }
        } else {
            if (grp == 0 && col_ok)
                stage[wib][nparked * LPR + lig] = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
            const int s_q = __shfl(sl, q, kWave);
            const int64_t r_q = __shfl(rid, q, kWave);
            if (lane == 0) {
                stage_slot[wib][nparked] = s_q;
                stage_row[wib][nparked] = r_q;
            }
            ++nparked;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = 0.0;
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
                    if ((tb >> g) & 1ull) flush(k * BP + u * GPW + g);
                }
            }
        }
    };

    for (int k = 0; k < NB; ++k) {
        if (k > 0) {
            if (k * BP >= span) break;                        // wave-uniform: ragged last chunk
            load_batch(v, k);
        }
        add_batch(v, k);
        const bool last = (k + 1 == NB) || ((k + 1) * BP >= span);
        if (nparked >= ROUND || (last && nparked > 0)) {
            wave_lds_sync();
            update_parked<BF16, LPR, RU>(stage[wib], stage_row[wib], stage_slot[wib], nparked, table, state, num_rows,
                                         gvec, lr, eps, reduced, oob);
            wave_lds_sync();
            nparked = 0;
        }
    }

    // positions after the last segment end of the chunk (the chunk's last position is not a tail)
    const bool has_rest = ((tails >> (span - 1)) & 1ull) == 0;
    if (has_rest) {
        double t[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = across_groups<LPR>(acc[c]);
        if (grp == 0 && col_ok) {
            // a chunk wholly inside one segment is a middle piece (head buffer); otherwise this
            // chunk is the FIRST piece of the segment that continues (last buffer)
            double *dst = ((nflush == 0 && !head_complete) ? part_head : part_last) + (int64_t)chunk * dim + lig * 4;
#pragma unroll
            for (int c = 0; c < 4; ++c) dst[c] = t[c];
        }
    }

    // Count this chunk in at every cut segment it holds a piece of (at most two: the one that came
    // in from the left, the one that leaves to the right).  The last piece to arrive finishes the row.
    const bool head_cut = !head_complete;
    const bool tail_cut = has_rest && (nflush > 0 || head_complete);
    const int s_last = __shfl(sl, span - 1, kWave);
#pragma unroll 1
    for (int which = 0; which < 2; ++which) {
        if (!(which == 0 ? head_cut : tail_cut)) continue;    // wave-uniform
        const int s = which == 0 ? s_first : s_last;
        const int start = cstart[s];
        const int len = seg_offsets[s + 1] - seg_offsets[s];
        const int c_first = (start - lo) / kWave;
        const int c_last = (start + len - 1 - lo) / kWave;
        if (start < lo || c_first > chunk || c_last < chunk || c_last >= n_chunks) {
            bad = true;
            continue;
        }
        __threadfence();                                      // my partial rows before my count
        int old = 0;
        if (lane == 0) old = atomicAdd(&counters[c_first], 1);
        old = __builtin_amdgcn_readfirstlane(old);
        if (old != c_last - c_first) continue;                // wave-uniform
        __threadfence();                                      // everybody's partial rows after their counts
        if (lane == 0) counters[c_first] = 0;                 // ready for the next launch
        double t[4] = {0.0, 0.0, 0.0, 0.0};
        if (grp == 0 && col_ok) {
            const double *x = part_last + (int64_t)c_first * dim + lig * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) t[i] = x[i];
        }
        add_partial_rows(t, part_head, dim, lig, col_ok, c_first + 1 + grp, c_last, GPW);
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = across_groups<LPR>(t[i]);
        if (grp == 0 && col_ok) stage[wib][lig] = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
        if (lane == 0) {
            stage_slot[wib][0] = s;
            stage_row[wib][0] = u_t[s];
        }
        wave_lds_sync();
        update_parked<BF16, LPR, 1>(stage[wib], stage_row[wib], stage_slot[wib], 1, table, state, num_rows, gvec, lr,
                                    eps, reduced, oob);
        wave_lds_sync();
    }
    if (oob) atomicOr(flags, kFlagRowRange);
    if (bad) atomicOr(flags, kFlagInternal);
}

template <bool BF16, int LPR>
static void fused_launch(fs_ctx *ctx, int cls, const float *grads, int n, int gvec, const int32_t *cperm,
                         const int32_t *cslot, const int32_t *class_pos, const int32_t *seg_offsets,
                         const int32_t *cstart, const int64_t *u_t, void *table, float *state, int64_t num_rows,
                         float lr, float eps, float *reduced, hipStream_t s) {
    constexpr int GPW = kWave / LPR;
    constexpr int UNR = (kWave / GPW) < FS_FUSED_UNR ? (kWave / GPW) : FS_FUSED_UNR;
    const int n_chunks = (int)ceil_div(n, kWave);
    const int blocks = (int)ceil_div(n_chunks, kFusedWaves);
    hipLaunchKernelGGL((reduce_update_kernel<BF16, LPR, UNR>), dim3(blocks), dim3(kFusedWaves * kWave), 0, s,
                       (const f32x4 *)grads, cperm, cslot, class_pos, cls, n, seg_offsets, cstart, u_t, table, state,
                       num_rows, gvec, lr, eps, (f32x4 *)reduced, ctx->fpart_head[cls], ctx->fpart_last[cls],
                       ctx->fcounters[cls], ctx->d_flags);
}

int launch_reduce_update(fs_ctx *ctx, int cls, const float *grads, int64_t n, int32_t dim, const int32_t *cperm,
                         const int32_t *cslot, const int32_t *class_pos, const int32_t *seg_offsets,
                         const int32_t *cstart, const int64_t *u_t, void *table, int dt, float *state,
                         int64_t num_rows, float lr, float eps, float *reduced, hipStream_t s) {
    if (n == 0) return FS_OK;
    const int gvec = dim / 4;
    const bool bf = dt == FS_BF16;
#define FS_CASE(L)                                                                                                   \
    case L:                                                                                                          \
        if (bf) fused_launch<true, L>(ctx, cls, grads, (int)n, gvec, cperm, cslot, class_pos, seg_offsets, cstart,   \
                                      u_t, table, state, num_rows, lr, eps, reduced, s);                             \
        else fused_launch<false, L>(ctx, cls, grads, (int)n, gvec, cperm, cslot, class_pos, seg_offsets, cstart,     \
                                    u_t, table, state, num_rows, lr, eps, reduced, s);                               \
        break;
    switch (lanes_per_row(gvec)) {
        FS_CASE(1) FS_CASE(2) FS_CASE(4) FS_CASE(8) FS_CASE(16) FS_CASE(32) FS_CASE(64)
        default: return set_err(ctx, FS_EINVAL, "reduce+update: dim beyond 256");
    }
#undef FS_CASE
    FS_LAUNCH_CHECK(ctx, "reduce_update_kernel");
    return FS_OK;
}

}  // namespace fs
