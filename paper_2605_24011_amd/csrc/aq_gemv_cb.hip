// Decode kernel of the non-uniform codebook variant of the format:  y[n] = sum_k x[k] * d[n, k/32] * L[q[n, k]]
// (Eq. 1 with a format-specific table L of 2^bits levels; Section 3, "Weight quantization").
//
// Same blob, same streaming structure and the same activation digits as the base decode kernel (aq_gemv.hip: body in
// aq_gemv_digit_body.inc); what differs is how a block's codes become operands of the block-scaled fp4 x fp6 MFMA.
// A table lookup per weight is out of reach of a kernel that has about two lane-instructions per weight, so the table
// goes where the hardware can use it:
//
//   NATIVE (4 bits, L = alpha * the E2M1 grid in some order): the codes are re-numbered when the blob is packed so that a
//       stored nibble IS the fp4 bit pattern of its level.  The raw words are the A operand: no vector-ALU work on the
//       codes at all, one MFMA per 4 blocks (the uniform 4-bit format needs two); alpha multiplies the stored result.
//   PLANES (any table): a function of `bits` bits is a multilinear polynomial of them,
//           L[q] = sum over subsets S of the bit positions of  a_S * prod_{j in S} q_j        (a_S by Moebius inversion),
//       and each monomial is a one-bit plane: AND of shifted code words, a nibble 0001 = the fp4 number 0.5.  One MFMA
//       per non-empty S gives sum_k [S in q_k] x_k for the block; the lane combines them with the a_S in fp32
//       (2^bits - 1 planes: 3 / 7 / 15).  The constant a_0 times the block's sum of x rides in the staged C operand.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"
#include "aq_gemv_digit.h"

#define AQ_TRACE(slot) do { } while (0)

namespace {

using namespace aqdev;

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
#define AQ_DG_DEPTH_B2 2
#define AQ_DG_DEPTH_B4 2
#define AQ_GEMV_SEG_CHUNKS 16
constexpr int CB_TW = 2;

// bit j of every code of a block as four registers of one-bit nibbles, in the slot order of DigitUnit<BITS>
template <int BITS>
__device__ __forceinline__ void bit_plane(const uint32_t* w, int j, uint32_t (&p)[4])
{
    const uint32_t M1 = 0x11111111u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (BITS == 4) p[i] = (w[i] >> j) & M1;                                   // nibble i' of word i = one code
        else if (BITS == 2) p[i] = (w[i >> 1] >> (2 * (i & 1) + j)) & M1;         // 2-bit fields, even / odd ones
        else p[i] = j == 0 ? (w[2] >> i) & M1                                     // lowest bits: a word of their own
                           : (w[i >> 1] >> (2 * (i & 1) + j - 1)) & M1;           // upper two bits: 2-bit fields
    }
}

template <int BITS, bool NATIVE> struct CbUnit {
    // t[r] = sum_k L[q[row r, k]] * x[k] over the block (this lane's digit column of it); C = a_0 * (sum of x) in
    // digit 0's column, zero elsewhere
    __device__ static __forceinline__ float4v block(const uint32_t* w, const v8i& B, const float4v& C, int sb,
                                                    const float (&coef)[16])
    {
        if (NATIVE) {
            static_assert(!NATIVE || BITS == 4, "the native table is the 4-bit E2M1 grid");
            const v4i a = {(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            return mfma_fp4_fp6(a, B, C, 127, sb);
        }
        uint32_t p[BITS][4];
#pragma unroll
        for (int j = 0; j < BITS; ++j) bit_plane<BITS>(w, j, p[j]);
        float4v t = C;
        const float4v zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int S = 1; S < (1 << BITS); ++S) {
            uint32_t a[4] = {~0u, ~0u, ~0u, ~0u};
#pragma unroll
            for (int j = 0; j < BITS; ++j)
                if (S & (1 << j)) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) a[i] &= p[j][i];
                }
            const float4v D = mfma_fp4_fp6(v4i{(int)a[0], (int)a[1], (int)a[2], (int)a[3]}, B, zero, SA_X2, sb);
            t[0] = fmaf(coef[S], D[0], t[0]);
            t[1] = fmaf(coef[S], D[1], t[1]);
            t[2] = fmaf(coef[S], D[2], t[2]);
            t[3] = fmaf(coef[S], D[3], t[3]);
        }
        return t;
    }
};

#define AQ_DG_UNIT(w, B, C, sb) CbUnit<BITS, NATIVE>::block(w, B, C, sb, ct.coef)
#define AQ_DG_STAGE_Z (-ct.coef[0])
#define AQ_DG_OUT(v) ((v) * ct.alpha)

// MODE 1: every task of the launch has the native table; 2, 3, 4: every task runs planes at that bit-width; 0: mixed
// (a branch per workgroup, as in mixed lists of the base format).  The plane forms of 3 and 4 bits need more
// registers than three wavefronts per SIMD leave (they would spill): those launches, and mixed ones, run two.
template <int MODE>
__global__ __launch_bounds__(THREADS, (MODE == 1 || MODE == 2 ? 3 : 2))
void qgemv_cb_kernel(const AqCbTask* __restrict__ tasks, const int32_t* __restrict__ wg_task, int count, AqCbTask single,
                     int lds_x)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AqCbTask ct;
    int wg = blockIdx.x;
    if (count == 0) {
        ct = single;
    } else {
        ct = tasks[wg_task[wg]];
        wg -= ct.g.wg_begin;
    }
    const AqGemvTask& t = ct.g;
    if (wg >= t.wg_count) return;
    constexpr int TW = CB_TW;
    constexpr bool KSPLIT = false;
    if (MODE == 1 || (MODE == 0 && ct.native)) {
        constexpr int BITS = 4;
        constexpr bool NATIVE = true;
#include "aq_gemv_digit_body.inc"
    } else if (MODE == 2 || (MODE == 0 && t.bits == 2)) {
        constexpr int BITS = 2;
        constexpr bool NATIVE = false;
#include "aq_gemv_digit_body.inc"
    } else if (MODE == 3 || (MODE == 0 && t.bits == 3)) {
        constexpr int BITS = 3;
        constexpr bool NATIVE = false;
#include "aq_gemv_digit_body.inc"
    } else {
        constexpr int BITS = 4;
        constexpr bool NATIVE = false;
#include "aq_gemv_digit_body.inc"
    }
}

}  // namespace

// workgroups of a task: one per 128-row group
void aqk_cb_gemv_shape(AqCbTask& t) { t.g.wg_count = (int)aq_num_groups(t.g.N) * (AQ_GROUP_TILES / (WAVES * CB_TW)); }

// mode: 1 native, 2 / 3 / 4 planes at that bit-width (every task of the launch alike), 0 mixed
hipError_t aqk_cb_gemv(const AqCbTask* tasks_dev, const int32_t* wg_task, int count, const AqCbTask& single, int mode,
                       int total_wgs, int max_K, hipStream_t s)
{
    const int max_nch = (max_K + AQ_CHUNK_K - 1) / AQ_CHUNK_K;
    const int seg = max_nch < AQ_GEMV_SEG_CHUNKS ? max_nch : AQ_GEMV_SEG_CHUNKS;
    const int lds_x = seg * DG_CHUNK;
    const size_t lds = (size_t)lds_x + 64 + 4 * 2 * 16 * sizeof(float);
    const dim3 grid((unsigned)total_wgs), block(THREADS);
#define AQ_GO(M) hipLaunchKernelGGL(qgemv_cb_kernel<M>, grid, block, lds, s, tasks_dev, wg_task, count, single, lds_x)
    switch (mode) {
        case 1: AQ_GO(1); break;
        case 2: AQ_GO(2); break;
        case 3: AQ_GO(3); break;
        case 4: AQ_GO(4); break;
        default: AQ_GO(0); break;
    }
#undef AQ_GO
    return hipGetLastError();
}
