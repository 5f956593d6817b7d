// Device-side helpers shared by the kernel translation units (wave64 cross-lane sums, bf16).
#pragma once

#include "fs_common.h"

namespace fs {

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// x + (x of the lane 32 away) in every lane: one cross-half swap per 32-bit word, no LDS traffic
__device__ __forceinline__ double add_xor32(double x) {
    const unsigned lo = (unsigned)__double2loint(x), hi = (unsigned)__double2hiint(x);
    const u32x2 a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const u32x2 b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}

// x + (x of the lane 16 away) in every lane
__device__ __forceinline__ double add_xor16(double x) {
    const unsigned lo = (unsigned)__double2loint(x), hi = (unsigned)__double2hiint(x);
    const u32x2 a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const u32x2 b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}

// sum over the 64/LPR groups of a wavefront, result in every lane; fixed order
template <int LPR>
__device__ __forceinline__ double across_groups(double x) {
    if (LPR == 32) return add_xor32(x);
    if (LPR == 16) return add_xor32(add_xor16(x));
#pragma unroll
    for (int m = LPR; m < kWave; m <<= 1) x += __shfl_xor(x, m, kWave);
    return x;
}

// sum over the LPR lanes of one group, result in every lane of the group; fixed order
template <int LPR>
__device__ __forceinline__ double group_sum(double x) {
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) x += __shfl_xor(x, m, kWave);
    return x;
}

// A 16-byte store for output that nobody on this chip reads again soon: the non-temporal hint keeps the lines
// from being left dirty in the L2 of the XCD for the write-back at the end of the kernel to find (the lookup
// with plain stores: 127 us per step instead of 102; asking for write-through on top of the hint changes nothing).
__device__ __forceinline__ void store_streaming(u32x4 v, u32x4 *p) { __builtin_nontemporal_store(v, p); }

// Correctly rounded fp32 square root.  The hardware's fp32 square-root instruction is good to one ulp only,
// and that bare instruction is what the __fsqrt_rn intrinsic compiles to here; the plain sqrtf builtin gets the
// compiler's IEEE lowering (the instruction, then the two neighbours of its result tested with exact fused
// residuals), which is what the update needs to agree with a host sqrtf bit for bit.
__device__ __forceinline__ float sqrt_rn_f32(float x) { return __builtin_sqrtf(x); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}


// ---- scans shared by the index kernels ----------------------------------------------------------------
// inclusive scan of one value per lane over the wavefront
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const T t = __shfl_up(v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

// exclusive scan of one value per thread over a workgroup of kScanThreads threads; the total is returned
// to all threads.  `sh` holds kScanThreads / kWave values.  Contains two barriers.
template <typename T>
__device__ __forceinline__ T block_exclusive_scan(T v, T *sh, T &total) {
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const T inc = wave_inclusive_scan<T>(v);
    if (lane == kWave - 1) sh[w] = inc;
    __syncthreads();
    T base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kScanThreads / kWave; ++i) {
        const T x = sh[i];
        if (i < w) base += x;
        tot += x;
    }
    __syncthreads();
    total = tot;
    return base + inc - v;
}

// ---- optional workgroup trace (diagnostic builds with -DFS_TRACE only) ------------------------------
// Every workgroup of a traced kernel appends {kind, workgroups of the launch << 32 | linear workgroup id, first and last reading
// of the 100 MHz wall clock by its thread 0} to a buffer the host sets with fs_debug_trace.  The buffer
// is cut into 1024 lanes with a counter each (128 bytes apart) so that the appends do not queue up on one
// address.  Layout in 64-bit words: [1] = records per lane; counter of lane l at [16 + 16 l]; record i of
// lane l at [16 + 16*1024 + 4 (l * per_lane + i)].  One variable per translation unit;
// fs_set_trace_<unit> stores the buffer into it.
#ifdef FS_TRACE
static __device__ unsigned long long *g_trace_buf;
struct wg_trace {
    unsigned long long t0;
    int kind;
    __device__ __forceinline__ wg_trace(int k) : t0(wall_clock64()), kind(k) {}
    __device__ __forceinline__ ~wg_trace() {
        unsigned long long *buf = g_trace_buf;
        if (threadIdx.x == 0 && buf != nullptr) {
            const unsigned long long per_lane = buf[1];
            const unsigned long long l = (blockIdx.x + 37u * blockIdx.y + 131u * (unsigned)kind) & 1023u;
            const unsigned long long i = atomicAdd(&buf[16 + 16 * l], 1ull);
            if (i < per_lane) {
                unsigned long long *r = buf + 16 + 16 * 1024 + 4 * (l * per_lane + i);
                r[0] = (unsigned long long)kind;
                r[1] = ((unsigned long long)(gridDim.x * gridDim.y) << 32) | (blockIdx.y * gridDim.x + blockIdx.x);
                r[2] = t0;
                r[3] = wall_clock64();
            }
        }
    }
};
#define FS_WG_TRACE(kind) fs::wg_trace wg_trace_((kind))
#define FS_TRACE_SETTER(unit)                                                                   \
    extern "C" void fs_set_trace_##unit(unsigned long long *buf) {                                            \
        (void)hipMemcpyToSymbol(HIP_SYMBOL(g_trace_buf), &buf, sizeof(buf), 0, hipMemcpyHostToDevice); \
    }
#else
#define FS_WG_TRACE(kind)
#define FS_TRACE_SETTER(unit)
#endif

}  // namespace fs
