// Device pieces of the decode product on the block-scaled low-precision matrix instruction
// (V_MFMA_SCALE_F32_16X16X128_F8F6F4): the codes of Eq. 1 go to the matrix cores as they are stored.
//
//  * A operand = codes.  A b-bit code q sitting in the low bits of a 4-bit field IS the fp4 (E2M1) number q / 2
//    for q <= 3 (the patterns 0..3 run through the subnormal and the first normal binade, linearly).  The blob
//    keeps 2-bit fields, so `word & 0x33333333` and `(word >> 2) & 0x33333333` are A registers: 3 vector-ALU
//    instructions per 16 codes.  Wider codes are split into 2-bit (or 1-bit) planes, each plane one MFMA, the planes'
//    weights 2^p applied by the instruction's A-side scale.
//  * B operand = the activations as block floating point: per block of 32 along k one shared exponent e
//    (2^e <= max|x| < 2^(e+1)) and four signed fp6 (E2M3) digits per element, x = sum_j digit_j * 2^(e - 1 - 4j) up to
//    2^-17 of the block's largest magnitude (stage_convert).  Digit j of block b is one COLUMN of B, non-zero only in
//    the 32 k-slots of block b (block diagonal), and the instruction's B-side scale 2^(e - 1 - 4j) puts it at its
//    place: column (b, j) of the result is the exact partial sum  sum_k q[n, k] * digit_j(x[k]) * 2^(e - 1 - 4j).
//    One MFMA covers 4 blocks x 4 digits = 16 columns x 16 rows x 128 k.
//  * the zero point: sum x (q - z) = sum x q - z * sum x.  -z * (the block's sum of x) is the C operand of digit 0's
//    column.
//  * scale: lane (g, c) of the result holds rows 4g .. 4g+3 of column c = (block c / 4, digit c % 4); it multiplies its
//    four sums by the four rows' fp16 scale of that block in fp32 and keeps a running sum per row; the 16 columns
//    meet once, at the end of the row's walk over k.
//
// Error: the products and the column sums are exact; x is rounded to 16 bits below its block's leading bit
// (|error| <= 2^-17 of the block's largest magnitude per element: relative L2 of y around 1e-5 for any distribution
// of x, exact when every element of a block is within 2^-5 (fp16) or 2^-8 (bf16) of the block's largest); fp32
// rounding happens where a block sum is scaled and added.
#pragma once
#include <hip/hip_runtime.h>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"

namespace aqdev {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

// LDS image of the staged activations: one 48-byte record per (block, digit):
//   [0, 24)   the 32 fp6 digits of the block in A-slot order (slot s of the lane's A operand meets slot s here)
//   [24, 28)  byte 0 = the column's E8M0 scale (127 + e - 1 - 4j)
//   [32, 48)  the C operand, four copies: digit 0's record carries the block's zero-point term -z * (sum of the block),
//             the other three carry zero
constexpr int DG_REC = 48;
constexpr int DG_BLOCK = 4 * DG_REC;                 // 192 bytes per block of 32 k
constexpr int DG_CHUNK = AQ_CHUNK_BLOCKS * DG_BLOCK; // 1536 bytes per chunk of 256 k
constexpr int FMT_FP4 = 4, FMT_FP6 = 2;

// Which A slot element e (0..31) of a block occupies, per code layout (aq_layout.h):
//   2-bit words (also the planes of 3-bit codes): element 16h + 4n + 2f + o sits in register 2h + f, nibble n + 4o
//   4-bit words: element 8h + 2s + o sits in register h (of a plane), nibble s + 4o
// Both put the 8 consecutive elements [8a, 8a+8) of a block into the 6 bytes [6a, 6a+6) of the 24-byte digit string;
// inside them the order differs.

typedef _Float16 v32h __attribute__((ext_vector_type(32)));
typedef uint32_t v6u __attribute__((ext_vector_type(6)));
typedef uint32_t v16u __attribute__((ext_vector_type(16)));
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

// One thread's share of the staging: one block of 32 consecutive elements (64 bytes) of x.
struct StageLoad {
    u32x4 v[4];
};
// thread `it` of a staging team takes block blk0 + it (blocks at or beyond K / 32, and threads beyond nblk, get zeros)
__device__ __forceinline__ StageLoad stage_load(const uint16_t* x, int K, int blk0, int nblk, int it)
{
    StageLoad r;
    const int k = (blk0 + it) * AQ_BLOCK;
    const bool in = it < nblk && k < K;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        r.v[i] = u32x4{0u, 0u, 0u, 0u};
        if (in) r.v[i] = *(as_global<u32x4>(x + k + 8 * i));
    }
    return r;
}

// Convert the block stage_load(it) fetched and write its four digit records.  The digits come from the hardware's
// own fp6 conversion (V_CVT_SCALEF32_PK32_FP6_F16: 32 values per instruction, round to nearest even, saturating at
// +-7.5): digit 0 = fp6(x / 2^(e-1)) with 2^e <= max|x| < 2^(e+1), so |x| / 2^(e-1) < 4; the residual x - digit is exact
// in binary16, at most 1/8 of the scale, and is converted again at a scale 16 times smaller; four rounds leave a
// residual below 2^-17 of the block's largest magnitude.  Digits are signed (a residual can have either sign).
// `z`: the constant the block's sum is multiplied by (negated) for digit 0's C operand: the zero point 2^(BITS-1) of the
// base format; the codebook variant passes minus its table's constant term.  `all_digits`: write that value into every
// digit's record (the two-level variant reads it in all four lanes of a block).
template <int BITS>
__device__ __forceinline__ void stage_convert(const StageLoad& ld, int x_dtype, int nblk, uint8_t* xl, int it,
                                              const float z = (float)(1 << (BITS - 1)), const bool all_digits = false)
{
    if (it >= nblk) return;
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) { w[4 * i] = ld.v[i].x; w[4 * i + 1] = ld.v[i].y; w[4 * i + 2] = ld.v[i].z; w[4 * i + 3] = ld.v[i].w; }
    // the largest magnitude as a bit pattern (binary16 and bfloat16 magnitudes order like unsigned integers,
    // infinities and NaNs on top)
    u16x2 mx = {0, 0};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t mag = w[i] & 0x7FFF7FFFu;
        mx = __builtin_elementwise_max(mx, __builtin_bit_cast(u16x2, mag));
    }
    const uint32_t top = mx.x > mx.y ? mx.x : mx.y;
    const bool special = top >= (x_dtype == 1 ? 0x7C00u : 0x7F80u);          // an infinity or a NaN in the block
    int e;                                   // 2^e <= max < 2^(e+1); a subnormal maximum counts as the lowest normal binade
    if (x_dtype == 1) {
        e = (int)(top >> 10) - 15;
        e = e < -14 ? -14 : e;
    } else {
        e = (int)(top >> 7) - 127;
        e = e < -114 ? -114 : e;             // every column scale must fit E8M0
        // bfloat16 -> binary16 relative to the block: x * 2^-e lies in (-2, 2); exact unless an element is 2^14 times
        // smaller than the block's largest (then to 2^-25 of it)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float lo = ldexpf(__uint_as_float(w[i] << 16), -e), hi = ldexpf(__uint_as_float(w[i] & 0xFFFF0000u), -e);
            const half2v h = {(_Float16)lo, (_Float16)hi};
            w[i] = __builtin_bit_cast(uint32_t, h);
        }
    }
    const int eh = x_dtype == 1 ? e : 0;     // the block's exponent in the binary16 numbers held now
    // sum of the block (exact in fp32: multiples of one unit, 32 of them)
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t wi = w[i];
        sum = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, wi), half2v{(_Float16)1.f, (_Float16)1.f}, sum, false);
    }
    // elements into A-slot order: register pair sp holds slots 2 sp, 2 sp + 1
    uint32_t r[16];
    constexpr uint32_t LO = 0x05040100u, HI = 0x07060302u;       // (lo(a), lo(b)) and (hi(a), hi(b)) of perm(b, a, .)
    if (BITS == 4) {
        // slot 8h + s + 4o holds element 8h + 2s + o
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            r[4 * h + 0] = __builtin_amdgcn_perm(w[4 * h + 1], w[4 * h + 0], LO);
            r[4 * h + 1] = __builtin_amdgcn_perm(w[4 * h + 3], w[4 * h + 2], LO);
            r[4 * h + 2] = __builtin_amdgcn_perm(w[4 * h + 1], w[4 * h + 0], HI);
            r[4 * h + 3] = __builtin_amdgcn_perm(w[4 * h + 3], w[4 * h + 2], HI);
        }
    } else {
        // slot 8 (2h + f) + n + 4o holds element 16h + 4n + 2f + o
#pragma unroll
        for (int R = 0; R < 4; ++R) {
            const int h = R >> 1, f = R & 1;
            r[4 * R + 0] = __builtin_amdgcn_perm(w[8 * h + 2 + f], w[8 * h + f], LO);
            r[4 * R + 1] = __builtin_amdgcn_perm(w[8 * h + 6 + f], w[8 * h + 4 + f], LO);
            r[4 * R + 2] = __builtin_amdgcn_perm(w[8 * h + 2 + f], w[8 * h + f], HI);
            r[4 * R + 3] = __builtin_amdgcn_perm(w[8 * h + 6 + f], w[8 * h + 4 + f], HI);
        }
    }
    v16u rv;
#pragma unroll
    for (int i = 0; i < 16; ++i) rv[i] = r[i];
    v32h res = __builtin_bit_cast(v32h, rv);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float scale = __uint_as_float((uint32_t)(127 + eh - 1 - 4 * j) << 23);     // 2^(eh - 1 - 4j)
        const v6u p = __builtin_amdgcn_cvt_scalef32_pk32_fp6_f16(res, scale);
        if (j < 3) res -= __builtin_amdgcn_cvt_scalef32_pk32_f16_fp6(p, scale);
        uint8_t* rec = xl + (it * 4 + j) * DG_REC;
        *reinterpret_cast<u32x4*>(rec) = u32x4{p[0], p[1], p[2], p[3]};
        // bytes [16, 24): the last 8 digits; [24, 28): the column's E8M0 scale
        const int sb = special ? 255 : 127 + e - 1 - 4 * j;
        *reinterpret_cast<u32x4*>(rec + 16) = u32x4{p[4], p[5], (uint32_t)sb, 0u};
        // the zero point of the whole block rides in digit 0's column: -z * (sum of the block)
        const float cz = (j == 0 || all_digits) ? -z * (x_dtype == 1 ? sum : ldexpf(sum, e)) : 0.f;
        *reinterpret_cast<float4v*>(rec + 32) = float4v{cz, cz, cz, cz};
    }
}

// Stage the blocks [blk0, blk0 + nblk) of x (blocks at or beyond K/32 are zero) into `xl`, one block per thread, `T`
// threads with indices tid = 0 .. T-1.  The caller orders the LDS writes against the later reads (barrier).
template <int BITS, int T>
__device__ __forceinline__ void stage_digits(const uint16_t* x, int x_dtype, int K, int blk0, int nblk, uint8_t* xl, int tid,
                                             const float z = (float)(1 << (BITS - 1)), const bool all_digits = false)
{
    for (int it = tid; it < nblk; it += T) {
        const StageLoad ld = stage_load(x, K, blk0, nblk, it);
        stage_convert<BITS>(ld, x_dtype, nblk, xl, it, z, all_digits);
    }
}

// The operands lane (g, c) needs for one chunk: for each of the two MFMA slots m (slot m covers block 2g + m of every
// lane's two blocks, i.e. blocks m, 2 + m, 4 + m, 6 + m of the chunk): B digits (zero unless the column's block is the
// lane's k-range: c / 4 == g), the C operand and the column scale of column c = (block 2 (c / 4) + m, digit c % 4).
struct ChunkOperands {
    v8i B[2];
    float4v C[2];
    int sb[2];
};
// chl < 0: a chunk beyond the wavefront's range: every operand is the zero record (the product contributes zero).
__device__ __forceinline__ void load_chunk_operands(const uint8_t* xl, const uint8_t* zeros, int chl, int g, int c,
                                                    ChunkOperands& o)
{
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const uint8_t* rec = chl < 0 ? zeros : xl + ((chl * AQ_CHUNK_BLOCKS + 2 * (c >> 2) + m) * 4 + (c & 3)) * DG_REC;
        const uint8_t* bp = ((c >> 2) == g) ? rec : zeros;
        const v4i b0 = *reinterpret_cast<const v4i*>(bp);
        const v2i b1 = *reinterpret_cast<const v2i*>(bp + 16);
        o.B[m] = v8i{b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, 0, 0};
        o.C[m] = *reinterpret_cast<const float4v*>(rec + 32);
        o.sb[m] = *reinterpret_cast<const int*>(rec + 24);
    }
}

__device__ __forceinline__ float4v mfma_fp4_fp6(const v4i& a, const v8i& b, const float4v& c, int scale_a, int scale_b)
{
    const v8i a8 = {a.x, a.y, a.z, a.w, 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b, c, FMT_FP4, FMT_FP6, 0, scale_a, 0, scale_b);
}

// A-side scales (E8M0): an fp4 field holds (2-bit value) / 2
constexpr int SA_X2 = 128, SA_X4 = 129, SA_X8 = 130;

// Block sums of one block per lane: raw words of the block -> D (4 rows of this lane's column), C folded in.
template <int BITS> struct DigitUnit;

template <> struct DigitUnit<2> {
    __device__ static __forceinline__ float4v block(const uint32_t* w, const v8i& B, const float4v& C, int sb)
    {
        const uint32_t M = 0x33333333u;
        const v4i a = {(int)(w[0] & M), (int)((w[0] >> 2) & M), (int)(w[1] & M), (int)((w[1] >> 2) & M)};
        return mfma_fp4_fp6(a, B, C, SA_X2, sb);
    }
};

template <> struct DigitUnit<3> {
    // two planes: the upper two bits of every code (words 0, 1: 2-bit fields) and the lowest bit (word 2: one bit per
    // 4-bit field after the shifts below); q = 2 hi + lo
    __device__ static __forceinline__ float4v block(const uint32_t* w, const v8i& B, const float4v& C, int sb)
    {
        const uint32_t M = 0x33333333u, M1 = 0x11111111u;
        const v4i hi = {(int)(w[0] & M), (int)((w[0] >> 2) & M), (int)(w[1] & M), (int)((w[1] >> 2) & M)};
        const v4i lo = {(int)(w[2] & M1), (int)((w[2] >> 1) & M1), (int)((w[2] >> 2) & M1), (int)((w[2] >> 3) & M1)};
        const float4v d = mfma_fp4_fp6(lo, B, C, SA_X2, sb);
        return mfma_fp4_fp6(hi, B, d, SA_X4, sb);
    }
};

template <> struct DigitUnit<4> {
    // two planes: the low and the high two bits of every code; q = lo + 4 hi
    __device__ static __forceinline__ float4v block(const uint32_t* w, const v8i& B, const float4v& C, int sb)
    {
        const uint32_t M = 0x33333333u;
        const v4i lo = {(int)(w[0] & M), (int)(w[1] & M), (int)(w[2] & M), (int)(w[3] & M)};
        const v4i hi = {(int)((w[0] >> 2) & M), (int)((w[1] >> 2) & M), (int)((w[2] >> 2) & M), (int)((w[3] >> 2) & M)};
        const float4v d = mfma_fp4_fp6(lo, B, C, SA_X2, sb);
        return mfma_fp4_fp6(hi, B, d, SA_X8, sb);
    }
};

}  // namespace aqdev
