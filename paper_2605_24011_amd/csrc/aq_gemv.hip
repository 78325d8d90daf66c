// Decode kernel: y[n] = sum_k x[k] * d[n, k/32] * (q[n, k] - 2^(bits-1))   (Eq. 1 fused into the product)
//
// HBM-bound by design: each weight is read once (bits/8 + 1/16 bytes) and costs well under one
// vector-ALU instruction, so the load stream, not the ALUs, sets the pace:
//
//  * unpack: one AND-OR per TWO codes.  A 32-bit word of the blob carries the even element of a
//    pair in its low half and the odd element in its high half at the same bit position, so
//    (word & mask) | magic is a pair of fp16 numbers (2^e + q).  A few shifts per word bring all
//    positions under masks that sit inside the fp16 mantissa.
//  * multiply-accumulate: on the matrix cores.  One V_MFMA_F32_16X16X32_F16 takes 16 rows x 32
//    k-slots of weights as A.  Its 32 k-slots are spread over the 8 blocks of a chunk (4 slots
//    per block), and B holds x on a block diagonal: column c of B is x restricted to the slots of
//    block c.  After 8 MFMAs D[row][c] is the complete 32-element sum of block c for that row,
//    one useful number per lane and register, with no cross-lane reduction.
//  * the -2^(bits-1) offset and the magic constants are linear in x: their contribution
//    corr[block] = sum_t (magic_t + z) (x[2t] + x[2t+1]) depends on x only, is computed once per
//    workgroup while x is staged in LDS, and enters as the C operand of the first MFMA.
//  * the fp16 block scale multiplies the finished block sum in fp32 (one mixed-precision FMA per
//    block and row), so every product is exact and only fp32 summation rounds.
//
// Work split: a workgroup of 4 wavefronts owns 4 or 8 tiles (16 rows each) of one 128-row group;
// every wavefront walks the whole K extent of its own one or two tiles, sums stay in registers.
// A batched launch runs many matrices (each with its own bit-width) in one grid.
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

#ifndef AQ_GEMV_MIN_WAVES_B2
#define AQ_GEMV_MIN_WAVES_B2 4
#endif
#ifndef AQ_GEMV_MIN_WAVES_B34
#define AQ_GEMV_MIN_WAVES_B34 3
#endif
// chunks of packed units a wavefront of a lone matrix's launch requests ahead (the batched launches: 2)
#ifndef AQ_GEMV_LONE_DEPTH
#define AQ_GEMV_LONE_DEPTH 16
#endif
// Workgroup = 4 wavefronts x TW tiles (16 rows each) of one 128-row group; every wavefront walks
// the whole K extent of its own tiles, so sums stay in registers and wavefronts never meet.  At
// each chunk the 4 wavefronts together read one contiguous run of 4*TW units.
// The task of this workgroup: `single` when count == 0, else the last record whose first workgroup
// is not above blockIdx.x (binary search over uniform scalar loads).  A macro, so that the record
// stays a kernel-local value in scalar registers.
#define AQ_FIND_TASK(t, wg)                                                       \
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

// one bit-width per launch: the registers, and with them the occupancy, fit that bit-width (the lone-matrix shape,
// TW == 1, may use the whole register file: its launches have few workgroups)
template <int BITS, int TW>
__global__ __launch_bounds__(THREADS, (TW == 1 ? 1 : BITS == 2 ? AQ_GEMV_MIN_WAVES_B2 : AQ_GEMV_MIN_WAVES_B34))
void qgemv_kernel(const AqGemvTask* __restrict__ tasks, int count, AqGemvTask single)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_TASK(t, wg);
#include "aq_gemv_body.inc"
}

// matrices of different bit-widths in one launch (a mixed-precision backbone pass): each workgroup
// branches once on its matrix's bit-width; one launch has one tail instead of three
template <int TW>
__global__ __launch_bounds__(THREADS, AQ_GEMV_MIN_WAVES_B34)
void qgemv_mixed_kernel(const AqGemvTask* __restrict__ tasks, int count, AqGemvTask single)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_TASK(t, wg);
    if (t.bits == 2) {
        constexpr int BITS = 2;
#include "aq_gemv_body.inc"
    } else if (t.bits == 3) {
        constexpr int BITS = 3;
#include "aq_gemv_body.inc"
    } else {
        constexpr int BITS = 4;
#include "aq_gemv_body.inc"
    }
}

size_t gemv_lds_bytes(int max_K)
{
    int nch = (max_K + AQ_CHUNK_K - 1) / AQ_CHUNK_K;
    return (size_t)nch * 4 * X_PAIR_BYTES + (size_t)nch * 32 + 192 + 16;
}

}  // namespace

// tiles per workgroup: 8 (two per wavefront) in general, 4 for a lone small matrix so that it
// spreads over more compute units
int aqk_gemv_tiles_per_wg(int64_t N, bool batched)
{
    if (batched) return 8;
    return N >= 128 * 1024 ? 8 : 4;
}

int aqk_gemv_wg_count(int64_t N, int tiles_per_wg)
{
    return (int)(aq_num_groups(N) * (AQ_GROUP_TILES / tiles_per_wg));
}

// bits == 0: the tasks have different bit-widths (one mixed launch); else all tasks share `bits`
hipError_t aqk_gemv(const AqGemvTask* tasks_dev, int count, const AqGemvTask& single, int bits, int tiles_per_wg,
                    int total_wgs, int max_K, hipStream_t s)
{
    // the grid was sized for `tiles_per_wg` tiles per workgroup: only the two shapes the kernels are built for
    if ((tiles_per_wg != 4 && tiles_per_wg != 8) || (bits == 0 && tiles_per_wg != 8)) return hipErrorInvalidValue;
    const size_t lds = gemv_lds_bytes(max_K);
    const dim3 grid((unsigned)total_wgs), block(THREADS);
#define AQ_LAUNCH(BITS, TW) hipLaunchKernelGGL((qgemv_kernel<BITS, TW>), grid, block, lds, s, tasks_dev, count, single)
    if (bits == 0) {
        hipLaunchKernelGGL((qgemv_mixed_kernel<2>), grid, block, lds, s, tasks_dev, count, single);
    } else if (tiles_per_wg == 8) {
        if (bits == 2) AQ_LAUNCH(2, 2); else if (bits == 3) AQ_LAUNCH(3, 2); else AQ_LAUNCH(4, 2);
    } else {
        if (bits == 2) AQ_LAUNCH(2, 1); else if (bits == 3) AQ_LAUNCH(3, 1); else AQ_LAUNCH(4, 1);
    }
#undef AQ_LAUNCH
    return hipGetLastError();
}
