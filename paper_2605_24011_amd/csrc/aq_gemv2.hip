// Decode kernel for the two-level variant of the format:  y[n] = sum_k x[k] * (D_S a_b q[n,k] - M_S c_b)
// (Eq. 1 in its general form, a stored scale AND zero point per block, both compressed by the super-block).
//
// The arithmetic on the codes is the base kernel's: exact small integers on the matrix cores against the
// block-diagonal x, which leaves in lane (g, c) the sums  B[r] = sum_k (q - z) x  of block c for rows 4g .. 4g+3
// (z = 2^(bits-1), the offset the unpack constants are built around).  What changes is what happens to a block sum:
//     sum_k x (D a q - M c)  =  (D a) * (B[r] + z X_b)  -  (M c) * X_b,      X_b = sum of x over the block,
// two fp32 multiply-adds per row and block (each lane does two of the block's four rows: the lanes of the MFMA's
// eight empty block columns take half of their neighbours' work); X_b is computed once per workgroup while x is staged (next to the
// correction terms), z X_b rides in the MFMAs' C operand, and the two coefficients are formed from the lane's
// 4 bytes of codes and 4 (D, M) pairs.
// Same work split, ring and launch shapes as the base kernel; a unit is 64 bytes shorter.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"
#include "aq_gemv_core.h"

namespace {

using namespace aqdev;

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;

// X_b for the staged blocks: fp32 sum of the 32 binary16 values of block b
__device__ __forceinline__ void block_sums(const uint8_t* xl, float* xsum, int nblocks)
{
    for (int b = threadIdx.x; b < nblocks; b += THREADS) {
        float s = 0.f;
        const half2v one = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const u32x2 v = *reinterpret_cast<const u32x2*>(xl + x_lds_offset(b, q));
            const uint32_t p0 = v.x, p1 = v.y;
            s = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, p0), one, s, false);
            s = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, p1), one, s, false);
        }
        xsum[b] = s;
    }
}

template <int BITS, bool REFILL>
__device__ __forceinline__ void unit_step2(uint32_t (&raw)[Codec<BITS>::WORDS], uint32_t& sub, u32x4& sup,
                                           typename Codec<BITS>::Magic& magic, const half8 (&B)[8],
                                           const float4v& negc, float xs, bool hi, const uint8_t* next, int lane,
                                           int sub_off, int sup_off, float (&acc)[2])
{
    Codec<BITS>::fence(magic, acc[0]);
    uint32_t a0[16], a1[16];
    Codec<BITS>::unpack(&raw[0], magic, a0);
    Codec<BITS>::unpack(&raw[BITS], magic, a1);
    const uint32_t s4 = sub;
    const uint32_t p[4] = {sup.x, sup.y, sup.z, sup.w};
    if (REFILL) {
        Codec<BITS>::load(next, lane, raw);
        sub = __builtin_nontemporal_load(as_global<uint32_t>(next + sub_off));
        sup = __builtin_nontemporal_load(as_global<u32x4>(next + sup_off));
    }
    float4v D = negc;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
        u32x4 av = {a0[2 * m], a0[2 * m + 1], a1[2 * m], a1[2 * m + 1]};
        D = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, av), B[m], D, 0, 0, 0);
    }
    // D[r] = sum_k q x of the block (the caller put z * X_b into the MFMAs' C operand next to the correction term),
    // in lanes c < 8 only: the MFMA's block columns 8..15 are empty.  Lane c + 8 takes rows 2, 3 off lane c's hands
    // (two cross-lane moves), so every lane scales two block sums instead of half the lanes four.
    const bool upper = hi;                                              // this lane does rows 2, 3
    const float d0 = D[0], d1 = D[1], d2 = D[2], d3 = D[3];              // scalars first: bit_cast of a vector element misreads it
    // row_shr:8 -- lane c + 8 receives from lane c; lanes c < 8 have no source and keep the first operand
    const float e0 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, d0), __builtin_bit_cast(int, d2), 0x118, 0xF, 0xF, false));
    const float e1 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, d1), __builtin_bit_cast(int, d3), 0x118, 0xF, 0xF, false));
    const uint32_t s2 = upper ? (s4 >> 16) : s4;                        // the two rows' (a, c) bytes
    const uint32_t pa = upper ? p[2] : p[0], pb = upper ? p[3] : p[1];  // their (D, M)
    {
        const float a = (float)(s2 & 15u), c = (float)((s2 >> 4) & 15u);
        const float Dr = (float)__builtin_bit_cast(_Float16, (uint16_t)(pa & 0xFFFFu));
        const float Mr = (float)__builtin_bit_cast(_Float16, (uint16_t)(pa >> 16));
        acc[0] = fmaf(e0, Dr * a, acc[0]);               // s_b * sum q x
        acc[0] = fmaf(xs, -(Mr * c), acc[0]);            // - s_b z_b * X_b
    }
    {
        const float a = (float)((s2 >> 8) & 15u), c = (float)((s2 >> 12) & 15u);
        const float Dr = (float)__builtin_bit_cast(_Float16, (uint16_t)(pb & 0xFFFFu));
        const float Mr = (float)__builtin_bit_cast(_Float16, (uint16_t)(pb >> 16));
        acc[1] = fmaf(e1, Dr * a, acc[1]);
        acc[1] = fmaf(xs, -(Mr * c), acc[1]);
    }
}

template <int BITS, int TW, bool REFILL>
__device__ __forceinline__ void chunk_step2(uint32_t (*raw)[Codec<BITS>::WORDS], uint32_t* sub, u32x4* sup,
                                            typename Codec<BITS>::Magic& magic, const uint8_t* xl, const float* corr,
                                            const float* xsum, const uint8_t* zeros, int ch, bool diag, int c,
                                            const uint8_t* refill, int lane, int sub_off, int sup_off, float (*acc)[2])
{
    constexpr int UNIT = 512 * BITS + AQ2_PARAM_BYTES;
    typedef u32x4 u32x4_a8 __attribute__((aligned(8)));
    const uint8_t* bp = diag ? xl + (ch * 4 + (c >> 1)) * X_PAIR_BYTES + (c & 1) * 8 : zeros;
    half8 B[8];
#pragma unroll
    for (int m = 0; m < 8; ++m)
        B[m] = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4_a8*>(bp + m * X_ENTRY_BYTES));
    const float xs = xsum[ch * AQ_CHUNK_BLOCKS + (c & 7)];
    // C operand: minus the correction term (which takes the codes from magic + q to q - z) plus z * X_b (back to q)
    const float nc = fmaf((float)(1 << (BITS - 1)), xs, -corr[ch * AQ_CHUNK_BLOCKS + (c & 7)]);
    const float4v negc = {nc, nc, nc, nc};
#pragma unroll
    for (int tw = 0; tw < TW; ++tw)
        unit_step2<BITS, REFILL>(raw[tw], sub[tw], sup[tw], magic, B, negc, xs, c >= 8, refill + tw * UNIT, lane, sub_off,
                                 sup_off, acc[tw]);
}

#define AQ_FIND_TASK2(t, wg)                                                      \
    AqGemvTask t;                                                                 \
    int wg = blockIdx.x;                                                          \
    if (count == 0) {                                                             \
        t = single;                                                               \
    } else {                                                                      \
        int lo = 0, hi = count - 1;                                               \
        while (lo < hi) {                                                         \
            int mid = (lo + hi + 1) >> 1;                                         \
            if (tasks[mid].wg_begin <= wg) lo = mid; else hi = mid - 1;           \
        }                                                                         \
        t = tasks[lo];                                                            \
        wg -= t.wg_begin;                                                         \
    }                                                                             \
    if (wg >= t.wg_count) return

template <int BITS, int TW>
__global__ __launch_bounds__(THREADS, 3)
void qgemv2_kernel(const AqGemvTask* __restrict__ tasks, int count, AqGemvTask single)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_TASK2(t, wg);
#include "aq_gemv2_body.inc"
}

template <int TW>
__global__ __launch_bounds__(THREADS, 3)
void qgemv2_mixed_kernel(const AqGemvTask* __restrict__ tasks, int count, AqGemvTask single)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_TASK2(t, wg);
    if (t.bits == 2) {
        constexpr int BITS = 2;
#include "aq_gemv2_body.inc"
    } else if (t.bits == 3) {
        constexpr int BITS = 3;
#include "aq_gemv2_body.inc"
    } else {
        constexpr int BITS = 4;
#include "aq_gemv2_body.inc"
    }
}

size_t gemv2_lds_bytes(int max_K)
{
    int nch = (max_K + AQ_CHUNK_K - 1) / AQ_CHUNK_K;
    return (size_t)nch * 4 * X_PAIR_BYTES + (size_t)nch * 32 * 2 + 192 + 16;
}

}  // namespace

// same contract as aqk_gemv, blobs in the two-level layout
hipError_t aqk2_gemv(const AqGemvTask* tasks_dev, int count, const AqGemvTask& single, int bits, int tiles_per_wg,
                     int total_wgs, int max_K, hipStream_t s)
{
    if ((tiles_per_wg != 4 && tiles_per_wg != 8) || (bits == 0 && tiles_per_wg != 8)) return hipErrorInvalidValue;
    const size_t lds = gemv2_lds_bytes(max_K);
    const dim3 grid((unsigned)total_wgs), block(THREADS);
#define AQ_LAUNCH2(BITS, TW) hipLaunchKernelGGL((qgemv2_kernel<BITS, TW>), grid, block, lds, s, tasks_dev, count, single)
    if (bits == 0) {
        hipLaunchKernelGGL((qgemv2_mixed_kernel<2>), grid, block, lds, s, tasks_dev, count, single);
    } else if (tiles_per_wg == 8) {
        if (bits == 2) AQ_LAUNCH2(2, 2); else if (bits == 3) AQ_LAUNCH2(3, 2); else AQ_LAUNCH2(4, 2);
    } else {
        if (bits == 2) AQ_LAUNCH2(2, 1); else if (bits == 3) AQ_LAUNCH2(3, 1); else AQ_LAUNCH2(4, 1);
    }
#undef AQ_LAUNCH2
    return hipGetLastError();
}
