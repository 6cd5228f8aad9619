// Shared device/host helpers of libstep (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "step.h"

namespace step {

typedef unsigned int u32;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kPageTokens = 16;

// First non-zero code wins and stays.
__device__ __forceinline__ void report(int32_t *status, int code)
{
    if (status) atomicCAS(status, 0, code);
}

__device__ __forceinline__ float bf16_lo(u32 w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(u32 w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ u32 f32_to_bf16_bits(float f)
{
    u32 u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// acc + a.lo*b.lo + a.hi*b.hi on packed bf16 pairs, fp32 accumulate (v_dot2c_f32_bf16).
__device__ __forceinline__ float dot2_bf16(u32 a, u32 b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}

// Value of `v` in another lane of the same 16-lane row, chosen by a DPP control word.
template <int CTRL>
__device__ __forceinline__ float dpp(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppRowMirror = 0x140;  // lane c <- lane 15 - c
constexpr int kDppHalfMirror = 0x141; // lane c <- lane 7 - c within each 8 lanes

// max without the NaN-quieting pass (inputs here are never signalling NaNs that matter)
__device__ __forceinline__ float max_nc(float x, float y) { return __builtin_amdgcn_fmed3f(x, y, INFINITY); }

// gfx950's v_permlane16_swap / v_permlane32_swap with both operands the same register: the first result holds, in
// both rows of a pair (both halves of the wave), the value of the even row (the lower half), the second that of the
// odd row (the upper half).  Combining the two gives every lane the combination of its own value with that of lane ^ 16
// (lane ^ 32), bit-identical in both lanes, as a vector-ALU operation instead of a trip through the LDS crossbar.
__device__ __forceinline__ void swap16(float x, float &even, float &odd)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    even = __uint_as_float(r[0]);
    odd = __uint_as_float(r[1]);
}
__device__ __forceinline__ void swap32(float x, float &lower, float &upper)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    lower = __uint_as_float(r[0]);
    upper = __uint_as_float(r[1]);
}
// over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (the same column of the four 16-lane rows), to all four
__device__ __forceinline__ float max_rows(float x)
{
    float a, b;
    swap16(x, a, b);
    x = max_nc(a, b);
    swap32(x, a, b);
    return max_nc(a, b);
}
__device__ __forceinline__ float sum_rows(float x)
{
    float a, b;
    swap16(x, a, b);
    x = a + b;
    swap32(x, a, b);
    return a + b;
}
// over the 16 lanes of a row, to all of them (xor 1, xor 2, half mirror, mirror)
__device__ __forceinline__ float max_row16(float x)
{
    x = max_nc(x, dpp<kDppXor1>(x));
    x = max_nc(x, dpp<kDppXor2>(x));
    x = max_nc(x, dpp<kDppHalfMirror>(x));
    return max_nc(x, dpp<kDppRowMirror>(x));
}
__device__ __forceinline__ float sum_row16(float x)
{
    x += dpp<kDppXor1>(x);
    x += dpp<kDppXor2>(x);
    x += dpp<kDppHalfMirror>(x);
    return x + dpp<kDppRowMirror>(x);
}
// over the 64 lanes of the wave, to all of them; the order of the additions is fixed
__device__ __forceinline__ float wave_max(float x) { return max_rows(max_row16(x)); }
__device__ __forceinline__ float wave_sum(float x) { return sum_rows(sum_row16(x)); }
constexpr int kDppRowRor4 = 0x124;
constexpr int kDppRowRor8 = 0x128;
#define STEP_DPP_QUAD_BCAST(k) ((k) * 0x55)

// Order-preserving image of an fp32 score: a < b as floats <=> order_key(a) < order_key(b) as unsigned
// (-0 counts as +0; NaN is the caller's business).
__device__ __forceinline__ u32 order_key(float s)
{
    u32 u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;  // -0 == +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum of one int per thread over a 1024-thread workgroup (wave shuffles, then the 16
// wave totals); *total receives the sum.  scratch: 32 ints of LDS; the barrier at the start orders this
// call's writes after the previous call's reads, so calls may follow each other directly.
__device__ __forceinline__ int block_excl_scan(int v, int *scratch /*[32]*/, int *total)
{
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    __syncthreads();
    if (lane == 63) scratch[wid] = x;
    __syncthreads();
    if (wid == 0) {
        int t = lane < 16 ? scratch[lane] : 0;
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            const int y = __shfl_up(t, off);
            if (lane >= off) t += y;
        }
        if (lane < 16) scratch[16 + lane] = t;
    }
    __syncthreads();
    const int base = wid > 0 ? scratch[16 + wid - 1] : 0;
    *total = scratch[31];
    return base + x - v;
}

// ---------------------------------------------------------------------------------------------
// Every kernel of the library is launched through launch_kernel.  While a profiling session is open
// (step_profile_begin, benchmarks only) the launch carries two HIP events that take the kernel's own begin
// and end timestamps on the stream it runs on; otherwise it is a plain launch.
// ---------------------------------------------------------------------------------------------
enum KernelId {
    kKernFront = 0, kKernPlanBlocks, kKernStage1, kKernMerge, kKernScore, kKernScoreFinish, kKernPruneFused,
    kKernPruneSelect, kKernPruneRelease, kKernPruneCompact, kKernReserve, kKernFreelist, kKernAppend, kKernVote, kKernCopy,
    kKernReadProbe, kKernCount
};

struct Profile {
    hipEvent_t *ev = nullptr;  // 2 * cap events
    int32_t *ids = nullptr;    // kernel id of each timed launch
    int cap = 0, used = 0;
};
Profile &profile();  // misc.hip

template <typename... KArgs, typename... Args>
inline void launch_kernel(int id, void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s, Args &&...args)
{
    Profile &p = profile();
    if (p.ev && p.used < p.cap) {
        const int i = p.used++;
        p.ids[i] = id;
        hipExtLaunchKernelGGL(kernel, grid, block, 0, s, p.ev[2 * i], p.ev[2 * i + 1], 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
    }
}

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? STEP_OK : STEP_ELAUNCH;
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace step
