// Block-level scale optimisation (Section 4.2, "Block-Level Scale Optimization", Eq. 10-11): from fp32
// weights W[N, K] and per-element sensitivities F[N, K] to the block format of Eq. 1 -- codes in the
// canonical bitstream and one fp16 scale per block of 32 -- ready for aq_pack_weights.
//
// Per block:  omega_i = F_i sqrt(sigma_b^2 + w_i^2)  with sigma_b^2 the block's mean squared weight;
// start at s = max|w| / 2^(bits-1); `rounds` times: q_i = codebook entry nearest to w_i / s (codebook = the
// integers -2^(bits-1) .. 2^(bits-1)-1, the smaller entry on a tie), then s = sum(omega w q) / sum(omega q^2)
// (the loop of a block ends early when that quotient has a non-positive numerator or a zero denominator);
// the stored scale is d = binary16(s) (round to nearest even, capped at 65504) and the stored codes are one
// more assignment against d, plus the format's offset 2^(bits-1).
//
// Arithmetic is fp64 throughout: the codes are decisions (which integer is nearest), and in fp64 the
// summation order and the use of w * (1/s) for w / s move a decision only when w / s lies within ~1e-15 of
// a half-integer.  Roofline: HBM (8 bytes read per weight, b/8 + 1/16 written); fp64 VALU is a close second
// (about 12 fp64 instructions per weight and assignment).
//
// Work split: a lane owns 8 consecutive weights (a quarter block: two 16-byte loads of W and of F), the four
// lanes of a block meet through two xor-shuffles per sum; a lane's 8 codes are `bits` whole bytes of the
// block's bitstream.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "aq_kernels.h"

namespace {

__device__ __forceinline__ double quad_sum(double v)
{
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    return v;
}
__device__ __forceinline__ double quad_max(double v)
{
    v = fmax(v, __shfl_xor(v, 1));
    v = fmax(v, __shfl_xor(v, 2));
    return v;
}

// double -> binary16 bits, round to nearest even, for 0 <= a <= 65504
__device__ __forceinline__ uint32_t f64_to_f16_bits(double a)
{
    const uint64_t u = (uint64_t)__double_as_longlong(a);
    const int e = (int)(u >> 52) - 1023;                       // unbiased exponent (a is non-negative)
    if (e < -25) return 0u;                                    // below half of the smallest subnormal, or zero
    const uint64_t m = (u & 0xFFFFFFFFFFFFFull) | (1ull << 52); // 53-bit significand
    // keep 11 bits for normals, fewer for subnormals: drop `sh` low bits with round-to-nearest-even
    const int sh = 42 + (e < -14 ? -14 - e : 0);
    uint64_t kept = m >> sh;
    const uint64_t rem = m & ((1ull << sh) - 1), half = 1ull << (sh - 1);
    if (rem > half || (rem == half && (kept & 1))) ++kept;
    if (e < -14) return (uint32_t)kept;                        // subnormal (a carry into 0x400 is the smallest normal)
    // kept in [1024, 2048]: 2048 = carry into the next exponent
    return (uint32_t)(((uint64_t)(e + 15) << 10) + (kept - 1024));
}

template <int BITS>
__global__ __launch_bounds__(256) void scale_opt_kernel(const float* __restrict__ W, const float* __restrict__ F,
                                                        int64_t quarters, int rounds, uint8_t* __restrict__ codes,
                                                        uint16_t* __restrict__ scales)
{
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;    // quarter-block index = weights / 8
    // whole quads stay together: `quarters` is a multiple of 4 and the grid is rounded up to 256
    const bool live = id < quarters;
    const int64_t e0 = (live ? id : 0) * 8;
    constexpr double Z = (double)(1 << (BITS - 1));
    constexpr double QMIN = -Z, QMAX = Z - 1.0;

    float wf[8], ff[8];
    *reinterpret_cast<float4*>(&wf[0]) = *reinterpret_cast<const float4*>(W + e0);
    *reinterpret_cast<float4*>(&wf[4]) = *reinterpret_cast<const float4*>(W + e0 + 4);
    if (F) {
        *reinterpret_cast<float4*>(&ff[0]) = *reinterpret_cast<const float4*>(F + e0);
        *reinterpret_cast<float4*>(&ff[4]) = *reinterpret_cast<const float4*>(F + e0 + 4);
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) ff[i] = 1.f;
    }
    double w[8], ow[8], om[8];                                     // w, omega * w, omega
    double ss = 0.0, amax = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        w[i] = (double)wf[i];
        ss += w[i] * w[i];
        amax = fmax(amax, fabs(w[i]));
    }
    const double sigma2 = quad_sum(ss) * (1.0 / 32.0);
    amax = quad_max(amax);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        om[i] = (double)ff[i] * sqrt(sigma2 + w[i] * w[i]);        // Eq. 10, left
        ow[i] = om[i] * w[i];
    }
    double s = amax * (1.0 / Z);
    double q[8];
    auto assign = [&](double scale) {                              // Eq. 11, left; the smaller entry on a tie
        const double rs = 1.0 / scale;
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = fmin(fmax(ceil(w[i] * rs - 0.5), QMIN), QMAX);
    };
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = 0.0;
    bool going = s > 0.0;                                          // uniform inside a quad
    if (going) assign(s);
    for (int r = 0; r < rounds; ++r) {
        double num = 0.0, den = 0.0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            num += ow[i] * q[i];
            den += om[i] * q[i] * q[i];
        }
        num = quad_sum(num);                                       // every lane takes part in the shuffles
        den = quad_sum(den);
        going = going && num > 0.0 && den > 0.0;
        if (going) {
            s = num / den;                                         // Eq. 11, right
            assign(s);
        }
    }
    const uint32_t d_bits = f64_to_f16_bits(fmin(s, 65504.0));
    const int de = (int)(d_bits >> 10), dm = (int)(d_bits & 1023);
    const double d = de ? ldexp((double)(1024 + dm), de - 25) : ldexp((double)dm, -24);
    if (d > 0.0) {
        assign(d);
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = 0.0;
    }
    if (!live) return;
    uint32_t bitsword = 0;                                         // 8 codes = BITS whole bytes, little-endian
#pragma unroll
    for (int i = 0; i < 8; ++i) bitsword |= (uint32_t)(int)(q[i] + Z) << (i * BITS);
    uint8_t* out = codes + id * BITS;
    if (BITS == 4) {
        *reinterpret_cast<uint32_t*>(out) = bitsword;
    } else if (BITS == 2) {
        *reinterpret_cast<uint16_t*>(out) = (uint16_t)bitsword;
    } else {
        out[0] = (uint8_t)bitsword;
        out[1] = (uint8_t)(bitsword >> 8);
        out[2] = (uint8_t)(bitsword >> 16);
    }
    if ((id & 3) == 0) scales[id >> 2] = (uint16_t)d_bits;
}

}  // namespace

hipError_t aqk_optimize_scales(const float* W, const float* F, int64_t N, int64_t K, int bits, int rounds,
                               uint8_t* codes, uint16_t* scales, hipStream_t s)
{
    const int64_t quarters = N * K / 8;                            // K % 32 == 0
    const dim3 grid((unsigned)((quarters + 255) / 256)), block(256);
    if (bits == 2) hipLaunchKernelGGL(scale_opt_kernel<2>, grid, block, 0, s, W, F, quarters, rounds, codes, scales);
    else if (bits == 3) hipLaunchKernelGGL(scale_opt_kernel<3>, grid, block, 0, s, W, F, quarters, rounds, codes, scales);
    else hipLaunchKernelGGL(scale_opt_kernel<4>, grid, block, 0, s, W, F, quarters, rounds, codes, scales);
    return hipGetLastError();
}
