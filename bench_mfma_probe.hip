// Bench-only calibration library (built to bench_mfma_probe.so by __graft_entry__.build(), loaded by bench.py
// alone; not part of libaq.so or its C ABI): what the matrix cores of the part this runs on sustain for the two binary16 MFMA shapes when fed
// operand data from memory and nothing else is going on.  With constant operands the published rate is nearly
// reached; with random operands the part clocks down and delivers well under it, which is the ceiling a real
// product kernel works against.  One workgroup of 4 wavefronts per compute unit and wavefront-per-SIMD count,
// 8 independent accumulator chains per wavefront, operands loaded once.
#include <hip/hip_runtime.h>
#include <stdint.h>

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

// One asynchronous launch on `stream` (time it with events).
//   shape           0: V_MFMA_F32_16X16X32_F16, 1: V_MFMA_F32_32X32X16_F16
//   operands        DEVICE, 16-byte aligned, 32768 bytes (8 * 256 * 16) of binary16 values of the caller's choice
//   iters           1 .. 2^24 loop trips per wavefront (8 resp. 4 independent MFMAs each)
//   waves_per_simd  1 or 2 (workgroups of 4 wavefronts launched per compute unit)
//   sink            DEVICE, 256 floats, overwritten
//   flops           HOST, receives the floating-point operations of the launch (2 per multiply-add)
// Returns 0, -1 for an invalid argument, -6 for a launch error.
extern "C" int bench_mfma_probe(int shape, const void* operands, int iters, int waves_per_simd, float* sink,
                                int64_t* flops, void* stream)
{
    if ((shape != 0 && shape != 1) || iters < 1 || iters > (1 << 24) || (waves_per_simd != 1 && waves_per_simd != 2))
        return -1;
    if (!operands || !sink || !flops || (reinterpret_cast<uintptr_t>(operands) & 15u)) return -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -6;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -6;
    const int blocks = cus * waves_per_simd;
    const half8* src = static_cast<const half8*>(operands);
    if (shape == 1) hipLaunchKernelGGL(mfma_probe_kernel<1>, dim3(blocks), dim3(256), 0, s, src, sink, iters);
    else hipLaunchKernelGGL(mfma_probe_kernel<0>, dim3(blocks), dim3(256), 0, s, src, sink, iters);
    const int64_t per_mfma = shape == 1 ? 2LL * 32 * 32 * 16 : 2LL * 16 * 16 * 32;
    *flops = per_mfma * (shape == 1 ? 4 : 8) * iters * 4 * blocks;
    return hipGetLastError() == hipSuccess ? 0 : -6;
}
