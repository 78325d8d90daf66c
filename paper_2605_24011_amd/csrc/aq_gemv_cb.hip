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
//   SIGNED PLANES (a table whose levels come in pairs +v, -v): the codes are re-numbered at packing to sign and
//       magnitude index, the sign goes into the fp4 nibble's own sign bit, and only the magnitude table (half the
//       entries) is expanded: 2^(bits-1) planes (2 / 4 / 8), the empty monomial (a nibble s001) among them.
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

constexpr int FORM_PLANES = 0, FORM_NATIVE = 1, FORM_SIGNED = 2;

// the sign bit (top bit of every code) of a block in bit 3 of every nibble, same slot order
template <int BITS>
__device__ __forceinline__ void sign_plane(const uint32_t* w, uint32_t (&sg)[4])
{
    const uint32_t M8 = 0x88888888u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (BITS == 4) sg[i] = w[i] & M8;
        else sg[i] = (i & 1) ? (w[i >> 1] & M8) : ((w[i >> 1] << 2) & M8);        // upper bit of a 2-bit field
    }
}

template <int BITS, int FORM> struct CbUnit {
    // t[r] = sum_k L[q[row r, k]] * x[k] over the block (this lane's digit column of it); C = a_0 * (sum of x) in
    // digit 0's column, zero elsewhere (zero everywhere for the native and the signed form)
    __device__ static __forceinline__ float4v block(const uint32_t* w, const v8i& B, const float4v& C, int sb,
                                                    const float (&coef)[16])
    {
        if (FORM == FORM_NATIVE) {
            static_assert(FORM != FORM_NATIVE || BITS == 4, "the native table is the 4-bit E2M1 grid");
            const v4i a = {(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            return mfma_fp4_fp6(a, B, C, 127, sb);
        }
        constexpr int MB = FORM == FORM_SIGNED ? BITS - 1 : BITS;        // bits the polynomial runs over
        uint32_t p[MB][4];
#pragma unroll
        for (int j = 0; j < MB; ++j) bit_plane<BITS>(w, j, p[j]);
        uint32_t sg[4] = {0u, 0u, 0u, 0u};
        if (FORM == FORM_SIGNED) sign_plane<BITS>(w, sg);
        float4v t = C;
        const float4v zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int S = (FORM == FORM_SIGNED ? 0 : 1); S < (1 << MB); ++S) {
            uint32_t a[4] = {0x11111111u, 0x11111111u, 0x11111111u, 0x11111111u};
#pragma unroll
            for (int j = 0; j < MB; ++j)
                if (S & (1 << j)) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) a[i] &= p[j][i];
                }
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] |= sg[i];
            const float4v D = mfma_fp4_fp6(v4i{(int)a[0], (int)a[1], (int)a[2], (int)a[3]}, B, zero, SA_X2, sb);
            t[0] = fmaf(coef[S], D[0], t[0]);
            t[1] = fmaf(coef[S], D[1], t[1]);
            t[2] = fmaf(coef[S], D[2], t[2]);
            t[3] = fmaf(coef[S], D[3], t[3]);
        }
        return t;
    }
};

#define AQ_DG_UNIT(w, B, C, sb) CbUnit<BITS, FORM>::block(w, B, C, sb, ct.coef)
#define AQ_DG_STAGE_Z (FORM == FORM_PLANES ? -ct.coef[0] : 0.f)
#define AQ_DG_OUT(v) ((v) * ct.alpha)

// MODE = 4 * form + bits when every task of the launch has that form and bit-width (form 0 planes, 1 native, 2 signed
// planes); MODE 0 and 1: mixed (a branch per workgroup, as in mixed lists of the base format).  The wider plane forms
// need more registers than three wavefronts per SIMD leave (they would spill): those launches run two.  A mixed list
// that holds none of them (the usual case: signed tables at 2 and 3 bits, the native one at 4) runs MODE 1, compiled
// without their bodies, at three.
constexpr int cb_mode(int form, int bits) { return 4 * form + bits; }
constexpr int CB_MIXED_LIGHT = 1;
constexpr bool cb_light(int mode)
{
    return mode == cb_mode(FORM_NATIVE, 4) || mode == cb_mode(FORM_PLANES, 2) || mode == cb_mode(FORM_SIGNED, 2) ||
           mode == cb_mode(FORM_SIGNED, 3);
}
constexpr int cb_waves(int mode) { return (mode == CB_MIXED_LIGHT || cb_light(mode)) ? 3 : 2; }

template <int MODE>
__global__ __launch_bounds__(THREADS, cb_waves(MODE))
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
    const int mode = MODE > CB_MIXED_LIGHT ? MODE : cb_mode(ct.form, t.bits);
    if (mode == cb_mode(FORM_NATIVE, 4)) {
        constexpr int BITS = 4;
        constexpr int FORM = FORM_NATIVE;
#include "aq_gemv_digit_body.inc"
    } else if (mode == cb_mode(FORM_PLANES, 2)) {
        constexpr int BITS = 2;
        constexpr int FORM = FORM_PLANES;
#include "aq_gemv_digit_body.inc"
    } else if (MODE != CB_MIXED_LIGHT && mode == cb_mode(FORM_PLANES, 3)) {
        constexpr int BITS = 3;
        constexpr int FORM = FORM_PLANES;
#include "aq_gemv_digit_body.inc"
    } else if (MODE != CB_MIXED_LIGHT && mode == cb_mode(FORM_PLANES, 4)) {
        constexpr int BITS = 4;
        constexpr int FORM = FORM_PLANES;
#include "aq_gemv_digit_body.inc"
    } else if (mode == cb_mode(FORM_SIGNED, 2)) {
        constexpr int BITS = 2;
        constexpr int FORM = FORM_SIGNED;
#include "aq_gemv_digit_body.inc"
    } else if (mode == cb_mode(FORM_SIGNED, 3)) {
        constexpr int BITS = 3;
        constexpr int FORM = FORM_SIGNED;
#include "aq_gemv_digit_body.inc"
    } else if (MODE != CB_MIXED_LIGHT) {
        constexpr int BITS = 4;
        constexpr int FORM = FORM_SIGNED;
#include "aq_gemv_digit_body.inc"
    }
}

}  // namespace

// workgroups of a task: one per 128-row group
void aqk_cb_gemv_shape(AqCbTask& t) { t.g.wg_count = (int)aq_num_groups(t.g.N) * (AQ_GROUP_TILES / (WAVES * CB_TW)); }

// does a task of this form and bit-width fit the light mixed kernel?
bool aqk_cb_light(int form, int bits) { return cb_light(cb_mode(form, bits)); }

// mode: 4 * form + bits if every task of the launch has that form (0 planes, 1 native, 2 signed planes) and bit-width;
// else 1 if aqk_cb_light holds for every task, else 0
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
        case cb_mode(FORM_NATIVE, 4): AQ_GO(cb_mode(FORM_NATIVE, 4)); break;
        case cb_mode(FORM_PLANES, 2): AQ_GO(cb_mode(FORM_PLANES, 2)); break;
        case cb_mode(FORM_PLANES, 3): AQ_GO(cb_mode(FORM_PLANES, 3)); break;
        case cb_mode(FORM_PLANES, 4): AQ_GO(cb_mode(FORM_PLANES, 4)); break;
        case cb_mode(FORM_SIGNED, 2): AQ_GO(cb_mode(FORM_SIGNED, 2)); break;
        case cb_mode(FORM_SIGNED, 3): AQ_GO(cb_mode(FORM_SIGNED, 3)); break;
        case cb_mode(FORM_SIGNED, 4): AQ_GO(cb_mode(FORM_SIGNED, 4)); break;
        case CB_MIXED_LIGHT: AQ_GO(CB_MIXED_LIGHT); break;
        default: AQ_GO(0); break;
    }
#undef AQ_GO
    return hipGetLastError();
}
