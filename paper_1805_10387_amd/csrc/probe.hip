// Measurement support: what the matrix cores sustain with operands held in registers.
//
// The dense fp16 peak of the chip assumes its top clock.  Under a full-chip MFMA load the clock follows the
// power the operands' bit activity draws, so the rate a contraction can reach at best depends on the data:
// all-zero operands run at the top clock, normally distributed ones markedly below it.  The benchmark reports
// this measured ceiling next to the published peak.
#include "common.hpp"

namespace mp {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float    f32x16 __attribute__((ext_vector_type(16)));

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_HALVES  = 8 * PROBE_THREADS * 8;  // 4 + 4 operand registers of 8 halves per lane

// Every wave keeps a 4 x 4 grid of 32x32 accumulators and multiplies 4 A by 4 B operand registers, over and over:
// 16 independent v_mfma_f32_32x32x16_f16 per iteration, nothing else in the loop.
__global__ __launch_bounds__(PROBE_THREADS) void mfma_rate_kernel(const f16x8* __restrict__ in, float* __restrict__ out,
                                                                  int iters) {
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    f16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = in[i * PROBE_THREADS + threadIdx.x];
        b[i] = in[(4 + i) * PROBE_THREADS + threadIdx.x];
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

}  // namespace mp

using namespace mp;

extern "C" int mp_mfma_sustained_rate(const mp_half* operands, size_t n_operands, float* sink, size_t n_sink,
                                      int workgroups, int iters, double* tflops, mp_stream stream) {
    MP_REQUIRE(operands != nullptr && sink != nullptr && tflops != nullptr, "mp_mfma_sustained_rate: NULL argument");
    MP_REQUIRE(n_operands >= (size_t)PROBE_HALVES, "mp_mfma_sustained_rate: %d operand halves needed", PROBE_HALVES);
    MP_REQUIRE(workgroups >= 1 && workgroups <= 4096 && iters >= 1 && iters <= (1 << 24),
               "mp_mfma_sustained_rate: workgroups in [1, 4096], iters in [1, 2^24]");
    MP_REQUIRE(n_sink >= (size_t)workgroups * PROBE_THREADS, "mp_mfma_sustained_rate: sink of %d floats needed",
               workgroups * PROBE_THREADS);
    MP_REQUIRE((reinterpret_cast<uintptr_t>(operands) & 15) == 0, "mp_mfma_sustained_rate: operands not 16-byte aligned");
    hipStream_t hs = as_stream(stream);
    hipEvent_t  e0, e1;
    MP_REQUIRE(hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess, "mp_mfma_sustained_rate: no events");
    const f16x8* in = reinterpret_cast<const f16x8*>(operands);
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(PROBE_THREADS), 0, hs, in, sink, 16);  // warm-up
    hipEventRecord(e0, hs);
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(PROBE_THREADS), 0, hs, in, sink, iters);
    hipEventRecord(e1, hs);
    const hipError_t err = hipEventSynchronize(e1);
    float            ms  = 0.f;
    if (err == hipSuccess) hipEventElapsedTime(&ms, e0, e1);
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    MP_REQUIRE(err == hipSuccess && ms > 0.f, "mp_mfma_sustained_rate: timing failed (%s)", hipGetErrorString(err));
    // 4 waves per workgroup, 16 instructions per iteration, 2 * 32 * 32 * 16 flops per instruction
    *tflops = (double)workgroups * 4.0 * iters * 16.0 * 32768.0 / (ms * 1e-3) * 1e-12;
    return MP_OK;
}
