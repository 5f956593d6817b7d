// update_embedding(I, G) of Algorithm 2 for ONE class of rows (collision rows = priority pass,
// exclusive rows = deferred pass) in a single launch: gradient segment reduce and row-wise
// Adagrad fused, so the summed gradient of a row never travels through HBM.
//
// The index half of the step has laid the occurrences of the batch out class by class
// ("class order": all occurrences of collision rows first, then those of exclusive rows; inside a
// class by ascending row, inside a row in batch order).  A launch walks the positions of its
// class only, so the priority pass reads exactly the gradient rows of collision rows.
//
// Rows with at most FS_SHORT_SEGMENT occurrences (the vast majority of rows) take the short path:
// one group of lanes per row requests all gradient rows of its segment and the table row at once,
// adds, updates, stores - four short dependent rounds, no LDS, nothing shared.  Only rows with more
// occurrences go through the class order and the position-cut path below.
//
// There work is cut by POSITION (row popularity is Zipf, the hottest row has tens of thousands of
// occurrences): one wavefront owns 64 consecutive class positions, streams their gradient rows
// (16 bytes per lane, 64/LPR rows per instruction) into fp64 accumulators and, whenever a segment
// ends, parks the finished sum (rounded once to fp32) in LDS.  The parked rows (a handful: every
// segment here is long) are updated together at the end of the chunk, so the dependent loads of
// the update (table row, accumulator) are in flight together.  A segment cut by a chunk border leaves fp64 partial rows; every
// wavefront that contributed one counts itself in at the segment's counter, and the one that
// arrives last adds the partials in chunk order and updates the row - in two levels for the hot
// rows (sixteen pieces at a time, then the sums of those), so that the last arriver of a row with
// tens of thousands of occurrences has two short rounds of loads to do, not dozens.  No wavefront
// ever waits for another, and the order of every floating-point sum depends on the layout alone.
//
// The pieces travel between wavefronts (possibly on different XCDs, each with its own L2) as
// device-scope relaxed atomic stores and loads, which go through to the coherent level, ordered
// against the counter by waiting for the stores to be acknowledged.  A device-scope fence would
// do the same but writes back the whole dirty L2 every time - measured 10x the kernel's time.
#include "fs_common.h"
#include "fs_device.h"

namespace fs {

// build-time tuning knobs: row-group loads one wavefront issues per round; class positions per
// wavefront in the priority / deferred pass (64, 32 or 16: collision rows have long segments,
// exclusive rows short ones, and a short chunk means more wavefronts with shorter lives)
#ifndef FS_FUSED_UNR
#define FS_FUSED_UNR 8
#endif
#ifndef FS_FUSED_RU
#define FS_FUSED_RU 2                      // parked rows one group of lanes updates per round
#endif
#ifndef FS_FUSED_CHUNK_CO
#define FS_FUSED_CHUNK_CO 64
#endif
#ifndef FS_FUSED_CHUNK_EX
#define FS_FUSED_CHUNK_EX 64
#endif
#ifndef FS_SHORT_MAX_BLOCKS
#define FS_SHORT_MAX_BLOCKS 1280
#endif
#ifndef FS_SHORT_UNR
#define FS_SHORT_UNR 2                     // short path: rows one group of lanes takes per iteration
#endif
constexpr int kFusedSuper = 16;            // pieces of a cut segment that are added in one go (first level)
constexpr int kFusedWaves = 4;             // wavefronts per workgroup (they never synchronise)

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
            const float c_step = __fdiv_rn(lr, sqrt_rn_f32(s_new) + eps);
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

// A partial row in memory: four planes of gvec doubles (column 4*l + c of the row at plane c, place l), so
// that each of the four instructions of a group of lanes writes or reads one contiguous run instead of
// eight bytes out of every thirty-two (which the write-through stores paid for four times over).
__device__ __forceinline__ void store_piece(double *row, int gvec, int lig, const double (&t)[4]) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
        __hip_atomic_store(row + c * gvec + lig, t[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ double load_piece(const double *row, int gvec, int lig, int c) {
    return __hip_atomic_load(row + c * gvec + lig, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// t += part[c] for c = c_begin, c_begin + stride, ... <= c_last (four rows requested per round)
__device__ __forceinline__ void add_partial_rows(double (&t)[4], const double *part, int dim, int lig, bool col_ok,
                                                 int c_begin, int c_last, int stride) {
    for (int c = c_begin; c <= c_last; c += 4 * stride) {
        double h[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int cj = c + j * stride;
            const bool ok = col_ok && cj <= c_last;
            const double *src = part + (int64_t)(ok ? cj : c_begin) * dim;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[j][i] = ok ? load_piece(src, dim / 4, lig, i) : 0.0;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
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

template <bool BF16, int LPR, int UNR, int CHUNK>
__device__ __forceinline__ void long_segments_body(
    const int block, const f32x4 *__restrict__ grads, const int32_t *__restrict__ cperm, const int32_t *__restrict__ cslot,
    const int32_t *__restrict__ class_pos, int cls, int n, const int32_t *__restrict__ seg_offsets,
    const int32_t *__restrict__ cstart, const int64_t *__restrict__ u_t, void *table, float *state, int64_t num_rows,
    int gvec, float lr, float eps, f32x4 *reduced, double *part_head, double *part_last, int *cnt_seg, int *cnt_sup,
    int *flags) {
    constexpr int GPW = kWave / LPR;          // rows per wavefront instruction
    constexpr int BP = GPW * UNR;             // positions per batch
    constexpr int NB = CHUNK / BP;            // batches per chunk
    // every segment here has more than FS_SHORT_SEGMENT positions, so only a few end inside one chunk:
    // their sums wait in LDS and are all applied in one round at the end of the chunk
    constexpr int CAP = CHUNK / (FS_SHORT_SEGMENT + 1) + 1;
    constexpr int RU = FS_FUSED_RU;
    static_assert(CHUNK <= kWave && CHUNK % BP == 0, "one tail word, whole batches");
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
    const int chunk = block * kFusedWaves + wib;             // chunk number inside the class
    const int64_t a64 = (int64_t)lo + (int64_t)chunk * CHUNK;
    if (a64 >= hi) return;                                   // wave-uniform; wavefronts share nothing
    const int a = (int)a64;
    const int b = (a + CHUNK < hi) ? a + CHUNK : hi;
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
    // extents of the first and the last segment of the chunk (lanes 0-2 / 3-5: class position of its
    // first occurrence, its sorted positions): only needed if the chunk border cuts them
    int meta = 0;
    {
        const int s_edge = __shfl(sl, lane < 3 ? 0 : span - 1, kWave);
        if (lane < 6) {
            const int f = lane % 3;
            meta = f == 0 ? cstart[s_edge] : seg_offsets[s_edge + (f - 1)];
        }
    }

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
    const int n_chunks = (n + CHUNK - 1) / CHUNK;

    auto flush = [&](int q) {                                 // the segment that ends at chunk position q
        double t[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = across_groups<LPR>(acc[c]);
        if (nflush == 0 && !head_complete) {
            if (grp == 0 && col_ok) store_piece(part_head + (int64_t)chunk * dim, gvec, lig, t);
        } else {
            if (nparked < CAP) {
                if (grp == 0 && col_ok)
                    stage[wib][nparked * LPR + lig] = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
                const int s_q = __shfl(sl, q, kWave);
                const int64_t r_q = __shfl(rid, q, kWave);
                if (lane == 0) {
                    stage_slot[wib][nparked] = s_q;
                    stage_row[wib][nparked] = r_q;
                }
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
    }
    if (nparked > CAP) {                                      // cannot happen with a consistent class order
        bad = true;
        nparked = 0;
    }
    if (nparked > 0) {
        wave_lds_sync();
        update_parked<BF16, LPR, RU>(stage[wib], stage_row[wib], stage_slot[wib], nparked, table, state, num_rows,
                                     gvec, lr, eps, reduced, oob);
        wave_lds_sync();
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
            store_piece(((nflush == 0 && !head_complete) ? part_head : part_last) + (int64_t)chunk * dim, gvec, lig, t);
        }
    }

    // Count this chunk in at every cut segment it holds a piece of (at most two: the one that came
    // in from the left, the one that leaves to the right).  A cut segment that starts in chunk f
    // and ends in chunk l has its first piece in part_last[f] and one piece in part_head[c] for
    // every c in (f, l].  Those are grouped sixteen at a time ("supers", the j-th starts at chunk
    // f+1+16j): the last piece of a super to arrive adds the super up (chunk order) and leaves the
    // sum in the super's first slot; the last of {first piece, supers} to arrive adds those up
    // (same order) and updates the row.
    // The extents of the two candidate segments were requested at the start of the chunk (meta, below
    // the first batch of loads); both first arrivals are counted with ONE atomic instruction (lane 0:
    // the piece of a super, lane 1: the first piece of the segment that leaves to the right), so the
    // common case costs one store acknowledgement and one atomic round trip per chunk.
    const bool head_cut = !head_complete;
    const bool tail_cut = has_rest && (nflush > 0 || head_complete);
    const int s_last = __shfl(sl, span - 1, kWave);
    int seg_s[2] = {s_first, s_last}, c_first[2], c_last[2];
    bool valid[2] = {head_cut, tail_cut};
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const int start = __shfl(meta, which * 3 + 0, kWave);
        const int len = __shfl(meta, which * 3 + 2, kWave) - __shfl(meta, which * 3 + 1, kWave);
        c_first[which] = (start - lo) / CHUNK;
        c_last[which] = (start + len - 1 - lo) / CHUNK;
        if (valid[which] && (start < lo || c_first[which] > chunk || c_last[which] < chunk || c_last[which] >= n_chunks ||
                             c_last[which] == c_first[which] || (which == 0) != (chunk > c_first[which]))) {
            bad = true;
            valid[which] = false;
        }
    }
    const int sup_first = c_first[0] + 1 + ((chunk - c_first[0] - 1) / kFusedSuper) * kFusedSuper;
    const int sup_last = (sup_first + kFusedSuper - 1 < c_last[0]) ? sup_first + kFusedSuper - 1 : c_last[0];
    int old = 0;
    if (valid[0] || valid[1]) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // my pieces are acknowledged before I count myself in
        if (lane == 0 && valid[0])
            old = __hip_atomic_fetch_add(&cnt_sup[sup_first], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (lane == 1 && valid[1])
            old = __hip_atomic_fetch_add(&cnt_seg[c_first[1]], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const int old_head = __shfl(old, 0, kWave), old_tail = __shfl(old, 1, kWave);

    // last arrival at a segment: first piece + the sums of the supers, in chunk order; update the row
    auto finish_segment = [&](int s, int cf, int cl) {
        if (lane == 0) __hip_atomic_store(&cnt_seg[cf], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        double t[4] = {0.0, 0.0, 0.0, 0.0};
        if (grp == 0 && col_ok) {
            const double *x = part_last + (int64_t)cf * dim;
#pragma unroll
            for (int i = 0; i < 4; ++i) t[i] = load_piece(x, gvec, lig, i);
        }
        add_partial_rows(t, part_head, dim, lig, col_ok, cf + 1 + grp * kFusedSuper, cl, GPW * kFusedSuper);
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
    };

    if (valid[0] && old_head == sup_last - sup_first) {       // wave-uniform: last piece of its super
        if (lane == 0) __hip_atomic_store(&cnt_sup[sup_first], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        double t[4] = {0.0, 0.0, 0.0, 0.0};
        add_partial_rows(t, part_head, dim, lig, col_ok, sup_first + grp, sup_last, GPW);
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = across_groups<LPR>(t[i]);
        if (grp == 0 && col_ok) store_piece(part_head + (int64_t)sup_first * dim, gvec, lig, t);
        const int n_sup = (c_last[0] - c_first[0] + kFusedSuper - 1) / kFusedSuper;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        int o2 = 0;
        if (lane == 0) o2 = __hip_atomic_fetch_add(&cnt_seg[c_first[0]], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        o2 = __builtin_amdgcn_readfirstlane(o2);
        if (o2 == n_sup) finish_segment(seg_s[0], c_first[0], c_last[0]);   // 1 + n_sup arrivals in all
    }
    if (valid[1]) {
        const int n_sup = (c_last[1] - c_first[1] + kFusedSuper - 1) / kFusedSuper;
        if (old_tail == n_sup) finish_segment(seg_s[1], c_first[1], c_last[1]);
    }
    if (oob) atomicOr(flags, kFlagRowRange);
    if (bad) atomicOr(flags, kFlagInternal);
}

// Short path: the rows of one class whose segment has at most FS_SHORT_SEGMENT occurrences.  The
// index half left one record per row of the class (row, slot, number of occurrences, the
// occurrences themselves), so a group of LPR lanes needs two dependent rounds per row: the record,
// then table row + accumulator + all gradient rows of the segment at once.  Rows with longer
// segments are skipped (the position-cut launch owns them).
template <bool BF16, int LPR, int UNR>
__device__ __forceinline__ void short_rows_body(
    const int block, const int nblocks, const f32x4 *__restrict__ grads, int n, const int32_t *__restrict__ recs, const int64_t *__restrict__ n_rows_dev,
    int64_t cap, void *table, float *state, int64_t num_rows, int gvec, float lr, float eps, f32x4 *reduced,
    int *flags) {
#pragma clang fp contract(off)
    constexpr int GPW = kWave / LPR;
    constexpr int T = FS_SHORT_SEGMENT;
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    const bool col_ok = lig < gvec;
    const int dim = gvec * 4;
    int64_t n_rows = *n_rows_dev;
    if (n_rows > cap) n_rows = cap;
    const int64_t waves = (int64_t)nblocks * kFusedWaves;
    const int64_t wave = (int64_t)block * kFusedWaves + (threadIdx.x / kWave);
    u32x4 *t4 = reinterpret_cast<u32x4 *>(table);
    u32x2 *t2 = reinterpret_cast<u32x2 *>(table);
    bool oob = false, bad = false;
    for (int64_t base = wave * (GPW * UNR); base < n_rows; base += waves * (GPW * UNR)) {
        i32x4 hd[UNR], pa[UNR], pb[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t i = base + u * GPW + grp;
            const i32x4 *rec = reinterpret_cast<const i32x4 *>(recs + i * kShortRecInts);
            hd[u] = i32x4{0, 0, 0, 0};
            pa[u] = i32x4{0, 0, 0, 0};
            pb[u] = i32x4{0, 0, 0, 0};
            if (i < n_rows) {
                hd[u] = rec[0];
                pa[u] = rec[1];
                pb[u] = rec[2];
            }
        }
        int64_t r[UNR];
        int len[UNR];
        bool mine[UNR];
        u32x4 w[UNR];
        float s_old[UNR];
        f32x4 g[UNR][4];
        bool any_more = false;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            r[u] = ((int64_t)hd[u][1] << 32) | (uint32_t)hd[u][0];
            len[u] = hd[u][3];
            const bool in_list = base + u * GPW + grp < n_rows;
            const bool in_table = (r[u] >= 0) && (r[u] < num_rows);
            oob |= in_list && !in_table;
            const bool is_short = len[u] >= 1 && len[u] <= T;
            const bool slot_ok = (unsigned)hd[u][2] < (unsigned)n;
            bad |= in_list && (len[u] < 1 || !slot_ok);
            const bool live = in_list && in_table && is_short && slot_ok;
            if (!live) len[u] = 0;
            mine[u] = live && col_ok;
            any_more |= len[u] > 4;
            w[u] = u32x4{0u, 0u, 0u, 0u};
            if (mine[u]) {
                if (BF16) {
                    const u32x2 h = t2[r[u] * gvec + lig];
                    w[u][0] = h[0];
                    w[u][1] = h[1];
                } else {
                    w[u] = t4[r[u] * gvec + lig];
                }
            }
            s_old[u] = live ? state[r[u]] : 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                g[u][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                int p = pa[u][j];
                if ((unsigned)p >= (unsigned)n) { bad |= j < len[u]; p = 0; }
                if (mine[u] && j < len[u]) g[u][j] = __builtin_nontemporal_load(&grads[(int64_t)p * gvec + lig]);
            }
        }
        double acc[UNR][4];
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc[u][c] = (double)g[u][0][c];
#pragma unroll
                for (int j = 1; j < 4; ++j) acc[u][c] += (double)g[u][j][c];
            }
        if (__ballot(any_more) != 0) {                        // wave-uniform: some row has 5..8 occurrences
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    g[u][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                    int p = pb[u][j];
                    if ((unsigned)p >= (unsigned)n) { bad |= 4 + j < len[u]; p = 0; }
                    if (mine[u] && 4 + j < len[u]) g[u][j] = __builtin_nontemporal_load(&grads[(int64_t)p * gvec + lig]);
                }
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[u][c] += (double)g[u][j][c];
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const f32x4 gs = {(float)acc[u][0], (float)acc[u][1], (float)acc[u][2], (float)acc[u][3]};
            double ss = 0.0;
#pragma unroll
            for (int c = 0; c < 4; ++c) ss += (double)gs[c] * (double)gs[c];
            ss = group_sum<LPR>(ss);
            const float m = (float)(ss / (double)dim);
            const float s_new = s_old[u] + m;
            const float c_step = __fdiv_rn(lr, sqrt_rn_f32(s_new) + eps);
            if (BF16) {
                const float c0 = bf16_lo(w[u][0]) - c_step * gs[0];
                const float c1 = bf16_hi(w[u][0]) - c_step * gs[1];
                const float c2 = bf16_lo(w[u][1]) - c_step * gs[2];
                const float c3 = bf16_hi(w[u][1]) - c_step * gs[3];
                const u32x2 o = {f32_to_bf16_bits(c0) | (f32_to_bf16_bits(c1) << 16),
                                 f32_to_bf16_bits(c2) | (f32_to_bf16_bits(c3) << 16)};
                if (mine[u]) t2[r[u] * gvec + lig] = o;
            } else {
                u32x4 o;
#pragma unroll
                for (int c = 0; c < 4; ++c) o[c] = __float_as_uint(__uint_as_float(w[u][c]) - c_step * gs[c]);
                if (mine[u]) t4[r[u] * gvec + lig] = o;
            }
            if (len[u] > 0 && lig == 0) state[r[u]] = s_new;
            if (reduced != nullptr && mine[u]) reduced[(int64_t)hd[u][2] * gvec + lig] = gs;
        }
    }
    if (oob) atomicOr(flags, kFlagRowRange);
    if (bad) atomicOr(flags, kFlagInternal);
}

// One launch per class: the first `long_blocks` workgroups walk the class order (rows with many
// occurrences, position-cut), the others the records of the rows with few.  The long part goes
// first because its last arrivers have the longest dependent chains; workgroups past the end of
// either part leave at once, so an empty part costs nothing but their dispatch.
// A launch takes the class passes of up to kMaxBatch tables of one row width (blockIdx.y picks the table):
// a pass is about one residency round of the chip however small it is, so the tables of a shard are
// better walked side by side than one after the other.
struct class_pass_job {
    const f32x4 *grads;
    int n, long_blocks, blocks, cls, gvec;
    float lr, eps;
    const int32_t *cperm, *cslot, *class_pos, *seg_offsets, *cstart, *recs;
    const int64_t *u_t, *n_rows_dev;
    void *table;
    float *state;
    int64_t num_rows;
    f32x4 *reduced;
    double *part_head, *part_last;      // this table's stretch of the class's partial rows and counters
    int *cnt_seg, *cnt_sup;
};
struct class_pass_batch {
    class_pass_job j[kMaxBatch];
};

// CLS (0: priority pass, 1: deferred pass) is a template parameter so that the two passes are two kernels by name
// in a profile; the code is the same.
template <bool BF16, int LPR, int UNR, int CHUNK, int SU, int CLS>
__global__ __launch_bounds__(kFusedWaves *kWave) void class_pass_kernel(const class_pass_batch batch, int *flags) {
    const class_pass_job &job = batch.j[blockIdx.y];
    FS_WG_TRACE(8 + CLS);
    if ((int)blockIdx.x >= job.blocks) return;
    if ((int)blockIdx.x < job.long_blocks)
        long_segments_body<BF16, LPR, UNR, CHUNK>((int)blockIdx.x, job.grads, job.cperm, job.cslot, job.class_pos, CLS,
                                                  job.n, job.seg_offsets, job.cstart, job.u_t, job.table, job.state,
                                                  job.num_rows, job.gvec, job.lr, job.eps, job.reduced, job.part_head,
                                                  job.part_last, job.cnt_seg, job.cnt_sup, flags);
    else
        short_rows_body<BF16, LPR, SU>((int)blockIdx.x - job.long_blocks, job.blocks - job.long_blocks, job.grads, job.n,
                                       job.recs, job.n_rows_dev, (int64_t)job.n, job.table, job.state, job.num_rows,
                                       job.gvec, job.lr, job.eps, job.reduced, flags);
}

// `idx[0..m)`: the jobs of `jobs` (all of one dtype and row width, all with n > 0) that share this launch
template <bool BF16, int LPR, int CHUNK, int CLS>
static void fused_launch(fs_ctx *ctx, const fs_class_pass_job *jobs, const int *idx, int m, hipStream_t s) {
    constexpr int cls = CLS;
    constexpr int GPW = kWave / LPR;
    constexpr int SU = FS_SHORT_UNR;
    constexpr int UNR = (CHUNK / GPW) < FS_FUSED_UNR ? ((CHUNK / GPW) < 1 ? 1 : (CHUNK / GPW)) : FS_FUSED_UNR;
    constexpr int CH = CHUNK < GPW ? GPW : CHUNK;             // at least one row group per chunk
    const size_t cap_chunks = (size_t)ceil_div(ctx->max_ids, kFusedMinChunk) + 2;
    const size_t cap_doubles = cap_chunks * (size_t)ctx->max_dim;
    int at = 0;
    while (at < m) {
        // as many jobs as fit the class's partial-row and counter space, each with its own stretch of it
        class_pass_batch batch;
        memset(&batch, 0, sizeof(batch));
        size_t chunks = 0, doubles = 0;
        int k = 0, blocks = 0;
        for (; at + k < m && k < kMaxBatch; ++k) {
            const fs_class_pass_job &in = jobs[idx[at + k]];
            const int n = (int)in.n;
            // Both parts are sized for the worst case the host can know (every occurrence in a long
            // segment / every occurrence a row of its own); the real sizes live on the device.
            const int long_blocks = (int)ceil_div(ceil_div(n, CH), kFusedWaves);
            const size_t my_chunks = (size_t)long_blocks * kFusedWaves;
            if (k > 0 && (chunks + my_chunks > cap_chunks || doubles + my_chunks * (size_t)in.dim > cap_doubles)) break;
            class_pass_job &j = batch.j[k];
            j.grads = (const f32x4 *)in.grads;
            j.n = n; j.long_blocks = long_blocks; j.cls = cls;
            j.gvec = in.dim / 4; j.lr = in.lr; j.eps = in.eps;
            j.cperm = in.cperm; j.cslot = in.cslot; j.class_pos = in.class_pos; j.seg_offsets = in.seg_offsets;
            j.cstart = in.cstart; j.recs = in.short_rec; j.u_t = in.u_t; j.n_rows_dev = in.n_rows_dev;
            j.table = in.table; j.state = in.state; j.num_rows = in.num_rows; j.reduced = (f32x4 *)in.reduced;
            j.part_head = ctx->fpart_head[cls] + doubles;
            j.part_last = ctx->fpart_last[cls] + doubles;
            j.cnt_seg = ctx->fcounters[cls] + chunks;
            j.cnt_sup = ctx->fcounters_sup[cls] + chunks;
            chunks += my_chunks;
            doubles += my_chunks * (size_t)in.dim;
        }
        // The short part walks its records with a grid stride: the tables of a launch share FS_SHORT_MAX_BLOCKS
        // workgroups (about five per compute unit, all resident from the start).  Measured on four workloads,
        // more and shorter-lived workgroups lose (16 k: +5 %, 64 k: +12 %), fewer than three per compute unit too.
        for (int q = 0; q < k; ++q) {
            class_pass_job &j = batch.j[q];
            int64_t short_blocks = ceil_div(j.n, (int64_t)GPW * SU * kFusedWaves);
            const int64_t cap = FS_SHORT_MAX_BLOCKS / k > 256 ? FS_SHORT_MAX_BLOCKS / k : 256;
            if (short_blocks > cap) short_blocks = cap;
            j.blocks = j.long_blocks + (int)short_blocks;
            blocks = j.blocks > blocks ? j.blocks : blocks;
        }
        hipLaunchKernelGGL((class_pass_kernel<BF16, LPR, UNR, CH, SU, CLS>), dim3((unsigned)blocks, (unsigned)k),
                           dim3(kFusedWaves * kWave), 0, s, batch, ctx->d_flags);
        at += k;
    }
}

int launch_reduce_update_batch(fs_ctx *ctx, int cls, int count, const fs_class_pass_job *jobs, hipStream_t s) {
    // one launch (or as few as fit) per dtype and row width; tables keep their order inside a launch
    bool done[FS_MAX_STEP_TABLES];
    if (count < 0 || count > FS_MAX_STEP_TABLES) return set_err(ctx, FS_EINVAL, "reduce+update: too many tables");
    for (int k = 0; k < count; ++k) done[k] = jobs[k].n == 0;
    for (int k0 = 0; k0 < count; ++k0) {
        if (done[k0]) continue;
        const bool bf = jobs[k0].dt == FS_BF16;
        const int lpr = lanes_per_row(jobs[k0].dim / 4);
        int idx[FS_MAX_STEP_TABLES], m = 0;
        for (int k = k0; k < count; ++k)
            if (!done[k] && (jobs[k].dt == FS_BF16) == bf && lanes_per_row(jobs[k].dim / 4) == lpr) {
                idx[m++] = k;
                done[k] = true;
            }
#define FS_CASE(L)                                                                              \
    case L:                                                                                     \
        if (cls == 0) {                                                                         \
            if (bf) fused_launch<true, L, FS_FUSED_CHUNK_CO, 0>(ctx, jobs, idx, m, s);          \
            else fused_launch<false, L, FS_FUSED_CHUNK_CO, 0>(ctx, jobs, idx, m, s);            \
        } else {                                                                                \
            if (bf) fused_launch<true, L, FS_FUSED_CHUNK_EX, 1>(ctx, jobs, idx, m, s);          \
            else fused_launch<false, L, FS_FUSED_CHUNK_EX, 1>(ctx, jobs, idx, m, s);            \
        }                                                                                       \
        break;
        switch (lpr) {
            FS_CASE(1) FS_CASE(2) FS_CASE(4) FS_CASE(8) FS_CASE(16) FS_CASE(32) FS_CASE(64)
            default: return set_err(ctx, FS_EINVAL, "reduce+update: dim beyond 256");
        }
#undef FS_CASE
    }
    FS_LAUNCH_CHECK(ctx, "class_pass_kernel");
    return FS_OK;
}

int launch_reduce_update(fs_ctx *ctx, int cls, const float *grads, int64_t n, int32_t dim, const int32_t *cperm,
                         const int32_t *cslot, const int32_t *class_pos, const int32_t *seg_offsets,
                         const int32_t *cstart, const int64_t *u_t, void *table, int dt, float *state,
                         int64_t num_rows, float lr, float eps, float *reduced, hipStream_t s,
                         const int32_t *short_rec, const int64_t *n_rows_dev) {
    const fs_class_pass_job job = {grads, n, dim, cperm, cslot, class_pos, seg_offsets, cstart, u_t, table, dt, state,
                                   num_rows, lr, eps, reduced, short_rec, n_rows_dev};
    return launch_reduce_update_batch(ctx, cls, 1, &job, s);
}

FS_TRACE_SETTER(fused)

}  // namespace fs
