// Decode kernels: y[n] = sum_k x[k] * d[n, k/32] * (q[n, k] - 2^(bits-1))   (Eq. 1 fused into the product)
//
// HBM-bound by design: each weight is read once (bits/8 + 1/16 bytes) and must cost well under one vector-ALU
// instruction, so that the load stream, not the ALUs, sets the pace.  The codes go to the matrix cores as stored, as
// fp4 operands of the block-scaled V_MFMA_SCALE_F32_16X16X128_F8F6F4, against the activations as block-floating-point
// fp6 digits (aq_gemv_digit.h): 3 vector-ALU instructions per 16 two-bit codes, one MFMA per 2048 (2-bit) or 1024
// (3-, 4-bit: two planes) weights.  Column c of an MFMA result is the finished sum of ONE block of 32 k (times one
// digit of x) for 16 rows, the fp16 block scale multiplies it in fp32, and sums stay in registers until the end of
// the row's walk over K.
//
// Work split: a workgroup of 4 wavefronts; in a batched launch it owns one 128-row group (2 tiles per wavefront) and
// walks the whole of K, every wavefront summing its own rows in registers; a lone matrix is cut into one tile per
// workgroup with the 4 wavefronts splitting K.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"
#include "aq_gemv_digit.h"
#include <type_traits>

namespace {

using namespace aqdev;

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;

// chunks of packed units a wavefront keeps in flight on the fp4 x fp6 path
#ifndef AQ_DG_DEPTH_B2
#define AQ_DG_DEPTH_B2 2
#endif
#ifndef AQ_DG_DEPTH_B4
#define AQ_DG_DEPTH_B4 2
#endif
#ifndef AQ_DG_TW
#define AQ_DG_TW 2
#endif
// chunks of x staged in LDS at a time on the fp4 x fp6 path (a multiple of the ring depths)
#ifndef AQ_GEMV_SEG_CHUNKS
#define AQ_GEMV_SEG_CHUNKS 16
#endif
#ifndef AQ_DG_MIN_WAVES
#define AQ_DG_MIN_WAVES 4
#endif
#ifndef AQ_DG_MIN_WAVES_B4
#define AQ_DG_MIN_WAVES_B4 3
#endif
// The task of this workgroup: `single` when count == 0, else tasks[wg_task[blockIdx.x]] (a table with one entry per
// workgroup of the launch, written by the host when the list is planned: two dependent scalar loads; a search over
// the task records would be a chain of eight, microseconds before the workgroup's first weight load).  A macro, so
// that the record stays a kernel-local value in scalar registers.
#define AQ_FIND_TASK(t, wg)                                                       \
    AqGemvTask t;                                                                 \
    int wg = blockIdx.x;                                                          \
    if (count == 0) {                                                             \
        t = single;                                                               \
    } else {                                                                      \
        t = tasks[wg_task[wg]];                                                   \
        wg -= t.wg_begin;                                                         \
    }                                                                             \
    if (wg >= t.wg_count) return

// one bit-width per launch: the registers, and with them the occupancy, fit that bit-width (the lone-matrix shape may
// use the whole register file: its launches have about one workgroup per compute unit).
// lds_x = bytes of staged activations ahead of the zero record
template <int BITS, int TW, bool KSPLIT>
__global__ __launch_bounds__(THREADS, (KSPLIT ? 1 : BITS == 2 ? AQ_DG_MIN_WAVES : AQ_DG_MIN_WAVES_B4))
void qgemv_digit_kernel(const AqGemvTask* __restrict__ tasks, const int32_t* __restrict__ wg_task, int count,
                        AqGemvTask single, int lds_x)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_TASK(t, wg);
#include "aq_gemv_digit_body.inc"
}

// matrices of different bit-widths in one launch (a mixed-precision backbone pass): each workgroup
// branches once on its matrix's bit-width; one launch has one tail instead of three
__global__ __launch_bounds__(THREADS, AQ_DG_MIN_WAVES_B4)
void qgemv_mixed_kernel(const AqGemvTask* __restrict__ tasks, const int32_t* __restrict__ wg_task, int count,
                        AqGemvTask single, int lds_x)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_TASK(t, wg);
    constexpr int TW = AQ_DG_TW;
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

// staged digits + the zero record + (lone launches) the 4 wavefronts' partial sums
size_t digit_lds_bytes(int lds_x) { return (size_t)lds_x + 64 + 4 * 2 * 16 * sizeof(float); }

template <class Kern> hipError_t allow_lds(Kern k, size_t lds) { return aqk_allow_lds(reinterpret_cast<const void*>(k), lds); }

}  // namespace

void aqk_gemv_shape(AqGemvTask& t, bool batched)
{
    if (batched) t.wg_count = (int)aq_num_groups(t.N) * (AQ_GROUP_TILES / (WAVES * AQ_DG_TW));
    else t.wg_count = (int)(aq_num_groups(t.N) * AQ_GROUP_TILES);          // one tile per workgroup
}

hipError_t aqk_gemv(const AqGemvTask* tasks_dev, const int32_t* wg_task, int count, const AqGemvTask& single, int bits,
                    int total_wgs, int max_K, hipStream_t s)
{
    const dim3 grid((unsigned)total_wgs), block(THREADS);
    const int max_nch = (max_K + AQ_CHUNK_K - 1) / AQ_CHUNK_K;
    const int seg = max_nch < AQ_GEMV_SEG_CHUNKS ? max_nch : AQ_GEMV_SEG_CHUNKS;
    hipError_t e = hipSuccess;
#define AQ_GO(KERNEL, LDS_X)                                                                                  \
    do {                                                                                                      \
        const size_t lds = digit_lds_bytes(LDS_X);                                                            \
        if ((e = allow_lds(KERNEL, lds)) != hipSuccess) return e;                                             \
        hipLaunchKernelGGL(KERNEL, grid, block, lds, s, tasks_dev, wg_task, count, single, LDS_X);            \
    } while (0)
    if (count == 0) {
        // a lone matrix: every wavefront stages its own quarter of K, a segment at a time
        const int lds_x = WAVES * AQ_GEMV_SEG_CHUNKS * DG_CHUNK;
        if (bits == 2) AQ_GO((qgemv_digit_kernel<2, 1, true>), lds_x);
        else if (bits == 3) AQ_GO((qgemv_digit_kernel<3, 1, true>), lds_x);
        else AQ_GO((qgemv_digit_kernel<4, 1, true>), lds_x);
        return hipGetLastError();
    }
    const int lds_x = seg * DG_CHUNK;
    if (bits == 2) AQ_GO((qgemv_digit_kernel<2, AQ_DG_TW, false>), lds_x);
    else if (bits == 3) AQ_GO((qgemv_digit_kernel<3, AQ_DG_TW, false>), lds_x);
    else if (bits == 4) AQ_GO((qgemv_digit_kernel<4, AQ_DG_TW, false>), lds_x);
    else AQ_GO(qgemv_mixed_kernel, lds_x);
#undef AQ_GO
    return hipGetLastError();
}
