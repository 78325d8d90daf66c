// Calibration: what the matrix cores of the part this runs on sustain for the two binary16 MFMA shapes when fed
// operand data from memory and nothing else is going on.  With constant operands the published rate is nearly
// reached; with random operands the part clocks down and delivers well under it, which is the ceiling a real
// product kernel works against.  One workgroup of 4 wavefronts per compute unit and wavefront-per-SIMD count,
// 8 independent accumulator chains per wavefront, operands loaded once.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "aq_kernels.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// SHAPE 0: V_MFMA_F32_16X16X32_F16, 8 per iteration; SHAPE 1: V_MFMA_F32_32X32X16_F16, 4 per iteration
template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_probe_kernel(const half8* __restrict__ src, float* __restrict__ sink, int iters)
{
    half8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = src[(2 * i) * 256 + threadIdx.x];
        b[i] = src[(2 * i + 1) * 256 + threadIdx.x];
    }
    f32x16 c[4];
    f32x4 d[8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) c[i][v] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) d[i][v] = 0.f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (SHAPE == 1) {
                c[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[(i + 1) & 3], c[i], 0, 0, 0);
            } else {
                d[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], b[(i + 1) & 3], d[i], 0, 0, 0);
                d[i + 4] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[(i + 2) & 3], b[i], d[i + 4], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += c[i][v];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) s += d[i][v];
    if (blockIdx.x == 0) sink[threadIdx.x] = s;          // keeps the chains alive
}

}  // namespace

// operands: 8 * 256 * 16 bytes; sink: 256 floats.  *flops = the multiply-adds of the launch times two.
hipError_t aqk_probe_mfma(int shape, const void* operands, int iters, int waves_per_simd, float* sink, int64_t* flops,
                          hipStream_t s)
{
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    const int blocks = cus * waves_per_simd;
    const half8* src = static_cast<const half8*>(operands);
    if (shape == 1) hipLaunchKernelGGL(mfma_probe_kernel<1>, dim3(blocks), dim3(256), 0, s, src, sink, iters);
    else hipLaunchKernelGGL(mfma_probe_kernel<0>, dim3(blocks), dim3(256), 0, s, src, sink, iters);
    const int64_t per_mfma = shape == 1 ? 2LL * 32 * 32 * 16 : 2LL * 16 * 16 * 32;
    *flops = per_mfma * (shape == 1 ? 4 : 8) * iters * 4 * blocks;
    return hipGetLastError();
}
