// Decode kernel for the two-level variant of the format:  y[n] = sum_k x[k] * (D_S a_b q[n,k] - M_S c_b)
// (Eq. 1 in its general form, a stored scale AND zero point per block, both compressed by the super-block).
//
// The streaming structure, the codes as fp4 operands and the activations as fp6 digits are the base decode kernel's
// (aq_gemv.hip; body in aq_gemv_digit_body.inc, included here with its parameter hooks set).  What changes is what
// happens to a block's sums: the MFMAs leave P = sum_k q x (the codes themselves, no zero point folded in) in lane
// (g, c) for rows 4g .. 4g+3 of one block and one digit of x; the staged record of digit 0 carries X_b = sum_k x in its
// C field (zero for the other digits), which is NOT fed to the MFMA here but multiplied afterwards:
//     sum_k x (D a q - M c)  =  (D a) * P  -  (M c) * X_b,
// two fp32 multiply-adds per row and block; D a and M c are formed from the lane's 4 bytes of block codes (one per row)
// and the 4 rows' (D, M) pairs.  A unit is 64 bytes shorter than the base format's.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"
#include "aq_gemv_digit.h"

namespace {

using namespace aqdev;

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
#ifndef AQ_TL_DEPTH
#define AQ_TL_DEPTH 2
#endif
#ifndef AQ_TL_SEG
#define AQ_TL_SEG 16
#endif
#ifndef AQ_TL_MIN_WAVES
#define AQ_TL_MIN_WAVES 3
#endif
#define AQ_DG_DEPTH_B2 AQ_TL_DEPTH
#define AQ_DG_DEPTH_B4 AQ_TL_DEPTH
#define AQ_GEMV_SEG_CHUNKS AQ_TL_SEG
constexpr int TL_TW = 2;

// byte `B` (0..3) of a word as a float: V_CVT_F32_UBYTE<B>.  The compiler has the instruction but extracts the byte
// with a separate bit-field instruction first when it knows that only four bits of it can be set; the result feeds
// vector-ALU arithmetic only (no matrix-core operand comes out of an asm statement).
template <int B> __device__ __forceinline__ float byte_to_float(uint32_t w)
{
    float f;
    if (B == 0) asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(f) : "v"(w));
    else if (B == 1) asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(f) : "v"(w));
    else if (B == 2) asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(f) : "v"(w));
    else asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(f) : "v"(w));
    return f;
}

// acc[r] += (D_r a_r) P[r] for the lane's four rows: ac = the rows' (a | c << 4) bytes of the block, Df = the rows' D
__device__ __forceinline__ void scale2(float (&acc)[4], const float4v& P, const uint32_t ac, const float (&Df)[4])
{
    const uint32_t an = ac & 0x0F0F0F0Fu;
    acc[0] = fmaf(byte_to_float<0>(an) * P[0], Df[0], acc[0]);
    acc[1] = fmaf(byte_to_float<1>(an) * P[1], Df[1], acc[1]);
    acc[2] = fmaf(byte_to_float<2>(an) * P[2], Df[2], acc[2]);
    acc[3] = fmaf(byte_to_float<3>(an) * P[3], Df[3], acc[3]);
}

// The offset term -(M c) X_b does not depend on the digit: the four digit lanes of a block share it out by rows, lane
// (g, c) takes row 4g + (c & 3).  off += (M_j c_j) X_b, subtracted from that row's sum once at the end.
__device__ __forceinline__ void offset2(float& off, const float xb, const uint32_t ac, const int shj, const float Mj)
{
    const float cj = (float)((ac >> shj) & 15u);
    off = fmaf(cj * xb, Mj, off);
}

#define AQ_DG_UNIT(w, B, C, sb) DigitUnit<BITS>::block(w, B, float4v{0.f, 0.f, 0.f, 0.f}, sb)
#define AQ_DG_STAGE_Z (-1.f)                                 /* the staged C field = + the block's sum of x ... */
#define AQ_DG_STAGE_ALL_DIGITS true                          /* ... in every digit's record */
#define AQ_DG_OUT(v) (v)
#define AQ_DG_PARAM_BYTES AQ2_PARAM_BYTES
#define AQ_DG_SC_OFF (512 * BITS + 128 + g * 16)             /* `sc`: (D, M) of rows 4g .. 4g+3 */
#define AQ_DG_SC_OFF_ANY (512 * BITS + 128)
#define AQ_DG_PARAM_DECL                                                                                   \
    u32x2 sub2[DEPTH * TW];                  /* the rows' (a, c) bytes of blocks 2(c/4), 2(c/4)+1 */           \
    float off2[TW];                          /* this lane's share of the offset term: row 4g + (c & 3) */      \
    _Pragma("unroll") for (int i_ = 0; i_ < TW; ++i_) off2[i_] = 0.f;                                         \
    const int rowj = c & 3, shj = 8 * rowj + 4, shm = 16 * (rowj & 1);                                        \
    const bool upper_rows = rowj >= 2;
#define AQ_DG_PARAM_LOAD(slot, u, valid) \
    sub2[slot] = __builtin_nontemporal_load(as_global<u32x2>((u) + 512 * BITS + ((valid) ? (g * 8 + 2 * (c >> 2)) * 4 : 0)))
#define AQ_DG_PARAM_ZERO(slot) sub2[slot] = u32x2{0u, 0u}
#define AQ_DG_APPLY(tw, D, C, slot, m)                                                                     \
    do {                                                                                                   \
        const u32x4 dm = sc[slot];                                                                         \
        const uint32_t p0 = dm.x, p1 = dm.y, p2 = dm.z, p3 = dm.w;        /* scalars first, then bit casts */  \
        const float Df[4] = {(float)__builtin_bit_cast(half2v, p0).x, (float)__builtin_bit_cast(half2v, p1).x, \
                             (float)__builtin_bit_cast(half2v, p2).x, (float)__builtin_bit_cast(half2v, p3).x};\
        /* M of row rowj without a branch: the four M as two words of pairs, one select, one shift */          \
        const uint32_t M01 = __builtin_amdgcn_perm(p1, p0, 0x07060302u), M23 = __builtin_amdgcn_perm(p3, p2, 0x07060302u); \
        const uint32_t mw = (upper_rows ? M23 : M01) >> shm;                                                   \
        const float Mj = (float)__builtin_bit_cast(half2v, mw).x;                                             \
        const uint32_t ac = (m) ? sub2[slot].y : sub2[slot].x;                                                 \
        scale2(acc[tw], D, ac, Df);                                                                            \
        offset2(off2[tw], (C)[0], ac, shj, Mj);                                                                \
    } while (0)
#define AQ_DG_FINISH(tw)                                                                                   \
    do {                                                                                                   \
        _Pragma("unroll") for (int r_ = 0; r_ < 4; ++r_) acc[tw][r_] -= rowj == r_ ? off2[tw] : 0.f;           \
    } while (0)

// the task of this workgroup: see AQ_FIND_TASK in aq_gemv.hip
#define AQ_FIND_TASK2(t, wg)                                                      \
    AqGemvTask t;                                                                 \
    int wg = blockIdx.x;                                                          \
    if (count == 0) {                                                             \
        t = single;                                                               \
    } else {                                                                      \
        t = tasks[wg_task[wg]];                                                   \
        wg -= t.wg_begin;                                                         \
    }                                                                             \
    if (wg >= t.wg_count) return

template <int BITS, int TW, bool KSPLIT>
__global__ __launch_bounds__(THREADS, (KSPLIT ? 1 : AQ_TL_MIN_WAVES))
void qgemv2_kernel(const AqGemvTask* __restrict__ tasks, const int32_t* __restrict__ wg_task, int count,
                   AqGemvTask single, int lds_x)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_TASK2(t, wg);
#include "aq_gemv_digit_body.inc"
}

__global__ __launch_bounds__(THREADS, AQ_TL_MIN_WAVES)
void qgemv2_mixed_kernel(const AqGemvTask* __restrict__ tasks, const int32_t* __restrict__ wg_task, int count,
                         AqGemvTask single, int lds_x)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_TASK2(t, wg);
    constexpr int TW = TL_TW;
    constexpr bool KSPLIT = false;
    if (t.bits == 2) {
        constexpr int BITS = 2;
#include "aq_gemv_digit_body.inc"
    } else if (t.bits == 3) {
        constexpr int BITS = 3;
#include "aq_gemv_digit_body.inc"
    } else {
        constexpr int BITS = 4;
#include "aq_gemv_digit_body.inc"
    }
}

}  // namespace

// same contract as aqk_gemv (tasks shaped by aqk_gemv_shape), blobs in the two-level layout
hipError_t aqk2_gemv(const AqGemvTask* tasks_dev, const int32_t* wg_task, int count, const AqGemvTask& single, int bits,
                     int total_wgs, int max_K, hipStream_t s)
{
    const dim3 grid((unsigned)total_wgs), block(THREADS);
    const int max_nch = (max_K + AQ_CHUNK_K - 1) / AQ_CHUNK_K;
    const int seg = max_nch < AQ_GEMV_SEG_CHUNKS ? max_nch : AQ_GEMV_SEG_CHUNKS;
    hipError_t e = hipSuccess;
#define AQ_GO(KERNEL, LDS_X)                                                                                  \
    do {                                                                                                      \
        const size_t lds = (size_t)(LDS_X) + 64 + 4 * 2 * 16 * sizeof(float);                                 \
        if ((e = aqk_allow_lds(reinterpret_cast<const void*>(KERNEL), lds)) != hipSuccess) return e;          \
        hipLaunchKernelGGL(KERNEL, grid, block, lds, s, tasks_dev, wg_task, count, single, LDS_X);            \
    } while (0)
    if (count == 0) {
        const int lds_x = WAVES * AQ_GEMV_SEG_CHUNKS * DG_CHUNK;
        if (bits == 2) AQ_GO((qgemv2_kernel<2, 1, true>), lds_x);
        else if (bits == 3) AQ_GO((qgemv2_kernel<3, 1, true>), lds_x);
        else AQ_GO((qgemv2_kernel<4, 1, true>), lds_x);
        return hipGetLastError();
    }
    const int lds_x = seg * DG_CHUNK;
    if (bits == 2) AQ_GO((qgemv2_kernel<2, TL_TW, false>), lds_x);
    else if (bits == 3) AQ_GO((qgemv2_kernel<3, TL_TW, false>), lds_x);
    else if (bits == 4) AQ_GO((qgemv2_kernel<4, TL_TW, false>), lds_x);
    else AQ_GO(qgemv2_mixed_kernel, lds_x);
#undef AQ_GO
    return hipGetLastError();
}
