// Measurement utility, not part of the method: the rate at which the chip sustains back-to-back bf16
// matrix instructions on given operand VALUES, with nothing else running.  The published matrix peak
// assumes the nominal shader clock; under dense matrix load with realistic operand values the chip
// lowers its clock (power management), and the rate this probe reaches is the ceiling any kernel built
// on the same instruction can approach on that day on that card.  bench.py reports it beside the
// roofline figures.
#include "bsfa_internal.h"

namespace bsfa {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeOperands = 4096;        // floats the operand registers are filled from

__global__ void __launch_bounds__(kProbeThreads, 2) mfma_rate_kernel(const float *operands, float *sink, int iters)
{
    bf16x8 a[4], b[4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[x][e] = (__bf16)operands[(threadIdx.x * 64 + x * 8 + e) & (kProbeOperands - 1)];
            b[x][e] = (__bf16)operands[(threadIdx.x * 64 + 32 + x * 8 + e) & (kProbeOperands - 1)];
        }
    f32x16 acc[4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[x][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < kProbeMfmaPerIter; ++n)
            acc[n & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n & 3], b[(n >> 2) & 3], acc[n & 3], 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e) r += acc[x][e];
    sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = r;
}

}  // namespace

hipError_t launch_mfma_rate_probe(const float *operands, float *sink, int workgroups, int iters, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)workgroups), dim3(kProbeThreads), 0, stream, operands, sink, iters);
    return hipGetLastError();
}

}  // namespace bsfa
