// Fused row-wise Adagrad on a list of distinct rows (second half of update_embedding(I, G) of
// Algorithm 2).  The same kernel serves the priority pass (collision rows) and the deferred
// pass (exclusive rows); the passes differ only in the row list and the stream.
//
// One group of LPR lanes owns one row: each lane holds 16 bytes of the table row (4 fp32 or
// 8 bf16) and the matching fp32 summed gradients.  The mean of squares is summed in fp64
// (per-lane, then an xor butterfly inside the group), rounded once to fp32, added to the row's
// accumulator in fp32; the step is computed without FMA contraction so it rounds like the
// plain definition.  HBM traffic per row: read+write of the row, read of the gradient row,
// 8 bytes of state, 12 bytes of (row, slot).
#include "fs_common.h"
#include "fs_device.h"

namespace fs {

template <bool BF16, int LPR, int UNR>
__global__ __launch_bounds__(256) void adagrad_kernel(u32x4 *__restrict__ table, float *__restrict__ state,
                                                      int64_t num_rows, int dim, int granules,
                                                      const int64_t *__restrict__ rows,
                                                      const int32_t *__restrict__ slots,
                                                      const int64_t *__restrict__ n_rows_dev, int64_t cap,
                                                      const f32x4 *__restrict__ reduced, float lr, float eps,
                                                      int *__restrict__ flags) {
#pragma clang fp contract(off)
    constexpr int GPW = kWave / LPR;
    constexpr int GV = BF16 ? 2 : 1;                  // gradient float4s per lane
    const int lane = threadIdx.x & (kWave - 1);
    const int grp = lane / LPR;
    const int lig = lane % LPR;
    int64_t n_rows = *n_rows_dev;
    if (n_rows > cap) n_rows = cap;
    const int gvec_per_row = dim / 4;
    const int64_t waves = (int64_t)gridDim.x * (blockDim.x / kWave);
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    bool oob = false;

    for (int64_t base = wave * (GPW * UNR); base < n_rows; base += waves * (GPW * UNR)) {
        int64_t r[UNR];
        int32_t k[UNR];
        bool live[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t i = base + u * GPW + grp;
            const bool in_list = i < n_rows;
            r[u] = in_list ? rows[i] : 0;
            k[u] = in_list ? slots[i] : 0;
            const bool in_table = (r[u] >= 0) && (r[u] < num_rows);
            oob |= in_list && !in_table;
            live[u] = in_list && in_table;
        }
        f32x4 g[UNR][GV];
        u32x4 w[UNR];
        float s_old[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const bool mine = live[u] && (lig < granules);
#pragma unroll
            for (int q = 0; q < GV; ++q) {
                g[u][q] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (mine) g[u][q] = reduced[(int64_t)k[u] * gvec_per_row + lig * GV + q];
            }
            w[u] = u32x4{0u, 0u, 0u, 0u};
            if (mine) w[u] = table[r[u] * granules + lig];
            s_old[u] = live[u] ? state[r[u]] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            double ss = 0.0;
#pragma unroll
            for (int q = 0; q < GV; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c) ss += (double)g[u][q][c] * (double)g[u][q][c];
            ss = group_sum<LPR>(ss);
            const float m = (float)(ss / (double)dim);
            const float s_new = s_old[u] + m;
            const float c_step = __fdiv_rn(lr, sqrt_rn_f32(s_new) + eps);
            const bool mine = live[u] && (lig < granules);
            if (BF16) {
                u32x4 o;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float g_lo = g[u][c / 2][(c % 2) * 2], g_hi = g[u][c / 2][(c % 2) * 2 + 1];
                    const float lo = bf16_lo(w[u][c]) - c_step * g_lo;
                    const float hi = bf16_hi(w[u][c]) - c_step * g_hi;
                    o[c] = f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
                }
                if (mine) table[r[u] * granules + lig] = o;
            } else {
                u32x4 o;
#pragma unroll
                for (int c = 0; c < 4; ++c) o[c] = __float_as_uint(__uint_as_float(w[u][c]) - c_step * g[u][0][c]);
                if (mine) table[r[u] * granules + lig] = o;
            }
            if (live[u] && lig == 0) state[r[u]] = s_new;
        }
    }
    if (oob) atomicOr(flags, kFlagRowRange);
}

template <bool BF16, int LPR>
static void adagrad_launch(void *table, float *state, int64_t num_rows, int dim, int granules, const int64_t *rows,
                           const int32_t *slots, const int64_t *n_rows_dev, int64_t cap, const float *reduced,
                           float lr, float eps, int *flags, hipStream_t s) {
    constexpr int UNR = 2;
    constexpr int ROWS_PER_BLOCK = (kWave / LPR) * UNR * 4;
    int64_t blocks = ceil_div(cap, ROWS_PER_BLOCK);
    if (blocks > 4096) blocks = 4096;           // grid-stride beyond this; the list length lives on the device
    hipLaunchKernelGGL((adagrad_kernel<BF16, LPR, UNR>), dim3((unsigned)blocks), dim3(256), 0, s, (u32x4 *)table,
                       state, num_rows, dim, granules, rows, slots, n_rows_dev, cap, (const f32x4 *)reduced, lr, eps,
                       flags);
}

int launch_adagrad(fs_ctx *ctx, void *table, int dt, float *state, int64_t num_rows, int32_t dim,
                   const int64_t *rows, const int32_t *slots, const int64_t *n_rows_dev, int64_t cap,
                   const float *reduced, float lr, float eps, hipStream_t s) {
    if (cap == 0) return FS_OK;
    const bool bf = dt == FS_BF16;
    const int granules = bf ? dim / 8 : dim / 4;
    int *f = ctx->d_flags;
#define FS_CASE(L)                                                                                              \
    case L:                                                                                                     \
        if (bf) adagrad_launch<true, L>(table, state, num_rows, dim, granules, rows, slots, n_rows_dev, cap,   \
                                        reduced, lr, eps, f, s);                                                \
        else adagrad_launch<false, L>(table, state, num_rows, dim, granules, rows, slots, n_rows_dev, cap,     \
                                      reduced, lr, eps, f, s);                                                  \
        break;
    switch (lanes_per_row(granules)) {
        FS_CASE(1) FS_CASE(2) FS_CASE(4) FS_CASE(8) FS_CASE(16) FS_CASE(32) FS_CASE(64)
        default: return set_err(ctx, FS_EINVAL, "adagrad: row wider than 1024 bytes");
    }
#undef FS_CASE
    FS_LAUNCH_CHECK(ctx, "adagrad_kernel");
    return FS_OK;
}

}  // namespace fs
