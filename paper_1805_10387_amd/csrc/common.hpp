// Internal helpers shared by the HIP translation units of libmp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "mp.h"

namespace mp {

// ---- error reporting -------------------------------------------------------------------
void set_error(const char* fmt, ...);
int  hip_fail(hipError_t e, const char* what);

#define MP_REQUIRE(cond, ...)                 \
    do {                                      \
        if (!(cond)) {                        \
            ::mp::set_error(__VA_ARGS__);     \
            return MP_E_INVAL;                \
        }                                     \
    } while (0)

#define MP_LAUNCH_CHECK(what)                                 \
    do {                                                      \
        hipError_t e__ = hipGetLastError();                   \
        if (e__ != hipSuccess) return ::mp::hip_fail(e__, what); \
    } while (0)

// db[cols] = RNE16(sum over the nparts rows of part[nparts][cols]), summed in ascending order; sets st->found_inf (st may
// be NULL) if a stored value is non-finite.  Defined beside the column-sum kernels (glue.hip).
int finish_colsum_launch(const float* part, int nparts, int cols, mp_half* db, mp_scale_state* st, hipStream_t hs);

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline hipStream_t as_stream(mp_stream s) { return reinterpret_cast<hipStream_t>(s); }

// ---- fp16 storage ------------------------------------------------------------------------
// All conversions are plain casts: v_cvt_f16_f32 under the default rounding mode is
// round-to-nearest-even and overflows to inf.  Never use the round-toward-zero pack convert.
typedef _Float16 f16;
typedef f16   f16x2 __attribute__((ext_vector_type(2)));
typedef f16   f16x4 __attribute__((ext_vector_type(4)));
typedef f16   f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float h2f(uint16_t b) {
    union { uint16_t u; f16 h; } c; c.u = b; return (float)c.h;
}
__device__ __forceinline__ uint16_t f2h(float x) {
    union { uint16_t u; f16 h; } c; c.h = (f16)x; return c.u;
}
__device__ __forceinline__ float round16(float x) { return (float)(f16)x; }
__device__ __forceinline__ bool half_nonfinite(uint16_t b) { return (b & 0x7C00u) == 0x7C00u; }

// ---- wave / block reductions (wave64) -----------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
// Sum over a block of NW waves; every thread gets the result.  `red` is NW floats of LDS.
// Workgroup barrier that waits for the wave's LDS traffic only.  __syncthreads() is also a release fence: with global
// stores outstanding it waits for them to complete, and for every load issued before it, since loads and stores share
// one counter.  Where the waves of a workgroup communicate through LDS alone this barrier is enough, and global
// accesses stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += red[i];
    return t;
}
template <int NW>
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) t = fmaxf(t, red[i]);
    return t;
}

}  // namespace mp
