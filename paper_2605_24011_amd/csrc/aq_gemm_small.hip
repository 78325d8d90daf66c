// Prefill for small M (M <= 64), fp16-weight mode: a streaming kernel in the shape of the decode kernel.
//
// At these sizes the product is bound by the weight stream (HBM), not by the matrix pipe, so the structure that
// matters is the one that keeps many loads in flight: a workgroup of 4 wavefronts owns one 128-row group,
// each wavefront walks the whole K of its own 2 tiles with a register ring of packed units two chunks deep,
// and several workgroups share a CU (LDS use is 16 KiB per m-tile).  The unpacked weights never pass through
// LDS: with w = d * (q - z) formed in binary16 the MFMAs may contract over any set of 32 k, so a lane feeds
// the 8 consecutive k it holds (of its own blocks 2g, 2g+1) as its part of the A operand, and X is laid out
// to match ("Xs", written by retile_small_kernel: per 256-k chunk, per step s = 0..7, per m-tile, the 1 KiB B
// operand whose lane (g, m) holds X[m][chunk*256 + (2g + s/4)*32 + (s%4)*8 .. +8]).  X reaches LDS through
// registers one chunk ahead, requested BEFORE the weights of the same chunk: loads retire in order, and X is
// wanted first.
#include <hip/hip_runtime.h>
#include <type_traits>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"

namespace {

using namespace aqdev;

constexpr int SM_WAVES = 4;
constexpr int SM_THREADS = SM_WAVES * 64;

#define AQ_FIND_SMALL_TASK(t, wg)                                                 \
    AqGemmTask t;                                                                 \
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

// BITS_T == 0: the tasks' bit-widths differ, branch per workgroup.
// SPLIT: the exact mode.  d * (q - z) is fed to the matrix cores as the sum of two binary16 numbers (its rounding
// and the remainder, which the fused multiply-add delivers exactly), so that no weight is rounded: every product
// with a binary16 x is exact in fp32 and only the fp32 sums round, as in the block-scaled exact kernel.  Twice the
// MFMAs; up to M = 64 that is cheaper than scaling every block's sum on the vector ALU.
template <int BITS_T, int MT, bool SPLIT>
__global__ __launch_bounds__(SM_THREADS) void qgemm_small_kernel(const AqGemmTask* __restrict__ tasks, int count,
                                                                 AqGemmTask single, const uint8_t* __restrict__ workspace)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_SMALL_TASK(t, wg);
    if (BITS_T == 2 || (BITS_T == 0 && t.bits == 2)) {
        constexpr int BITS = 2;
#include "aq_gemm_small_body.inc"
    } else if (BITS_T == 3 || (BITS_T == 0 && t.bits == 3)) {
        constexpr int BITS = 3;
#include "aq_gemm_small_body.inc"
    } else {
        constexpr int BITS = 4;
#include "aq_gemm_small_body.inc"
    }
}

// X[M][ldx] -> Xs (binary16) + rowexp.  One workgroup per row of the MT*16 padded rows; k is padded with zeros to
// whole chunks.  BF: the input is bf16 and every row is scaled by a power of two into binary16's range first
// (largest magnitude to [2^14, 2^15)); otherwise the input is binary16 and is copied.
template <bool BF>
__global__ __launch_bounds__(256) void retile_small_kernel(const AqRetileTask* __restrict__ tasks, int count,
                                                           AqRetileTask single, uint8_t* __restrict__ workspace)
{
    __shared__ uint32_t wave_max[4];
    AqRetileTask t;
    if (count == 0) t = single; else t = tasks[blockIdx.y];
    const int MT = t.pad;                                      // m-tiles of the launch (1, 2 or 4)
    const int64_t row = blockIdx.x;
    if (row >= MT * 16) return;                                // uniform per workgroup
    const int tid = threadIdx.x;
    const int nch = (t.K + AQ_CHUNK_K - 1) / AQ_CHUNK_K;
    const int pieces = t.K >> 3, pieces_pad = nch * (AQ_CHUNK_K / 8);
    const int64_t xchunk16 = 8 * MT * 64;                      // 16-byte pieces per chunk
    u32x4* dst = reinterpret_cast<u32x4*>(workspace + t.xt_offset);
    int32_t* rowexp = reinterpret_cast<int32_t*>(workspace + t.xt_offset + (int64_t)nch * xchunk16 * 16);
    const int mt = (int)(row >> 4), mi = (int)(row & 15);
    auto slot = [&](int j) {                                   // piece j = elements 8j .. 8j+7 of the row
        const int ch = j >> 5, blk = (j >> 2) & 7, q = j & 3;
        const int s = (blk & 1) * 4 + q, gg = blk >> 1;
        return (int64_t)ch * xchunk16 + (s * MT + mt) * 64 + gg * 16 + mi;
    };
    int shift = 0;
    const bool live = row < t.M;
    const AQ_GLOBAL u32x4* src = as_global<u32x4>(t.X + (live ? row : 0) * t.ldx);
    if (BF && live) {
        uint32_t mx = 0;
        for (int j = tid; j < pieces; j += 256) {
            const u32x4 v = src[j];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = v[i] & 0x7FFFu, hi = (v[i] >> 16) & 0x7FFFu;
                mx = lo > mx ? lo : mx;
                mx = hi > mx ? hi : mx;
            }
        }
        for (int o = 32; o >= 1; o >>= 1) {
            const uint32_t other = (uint32_t)__shfl_xor((int)mx, o);
            mx = other > mx ? other : mx;
        }
        if ((tid & 63) == 0) wave_max[tid >> 6] = mx;
        __syncthreads();
        mx = wave_max[0];
#pragma unroll
        for (int i = 1; i < 4; ++i) mx = wave_max[i] > mx ? wave_max[i] : mx;
        if (mx != 0) {
            const int field = (int)(mx >> 7);
            shift = 14 - ((field ? field : 1) - 127);
        }
    }
    for (int j = tid; j < pieces_pad; j += 256) {
        u32x4 o = {0u, 0u, 0u, 0u};
        if (live && j < pieces) {
            const u32x4 v = src[j];
            if (BF) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float lo = ldexpf(__uint_as_float(v[i] << 16), shift);
                    const float hi = ldexpf(__uint_as_float(v[i] & 0xFFFF0000u), shift);
                    const half2v h = {(_Float16)lo, (_Float16)hi};
                    o[i] = __builtin_bit_cast(uint32_t, h);
                }
            } else {
                o = v;
            }
        }
        dst[slot(j)] = o;
    }
    if (tid == 0) rowexp[row] = -shift;
}

template <int BITS_T>
void launch_small(int MT, bool split, dim3 grid, hipStream_t s, const AqGemmTask* tasks, int count,
                  const AqGemmTask& single, const uint8_t* ws)
{
    const dim3 block(SM_THREADS);
    const size_t lds = (size_t)2 * 8 * MT * 1024;              // two chunk slots of X
#define AQ_SMALL(MT_, SP_) hipLaunchKernelGGL((qgemm_small_kernel<BITS_T, MT_, SP_>), grid, block, lds, s, tasks, count, single, ws)
    if (split) {
        if (MT == 1) AQ_SMALL(1, true); else if (MT == 2) AQ_SMALL(2, true); else AQ_SMALL(4, true);
    } else {
        if (MT == 1) AQ_SMALL(1, false); else if (MT == 2) AQ_SMALL(2, false); else AQ_SMALL(4, false);
    }
#undef AQ_SMALL
}

}  // namespace

int aqk_small_mtiles(int64_t M) { return M <= 16 ? 1 : M <= 32 ? 2 : 4; }

// Xs (chunks x 8 steps x MT KiB) followed by rowexp (one int32 per padded row), rounded up to 1 KiB
size_t aqk_small_retile_bytes(int64_t M, int64_t K)
{
    const int64_t MT = aqk_small_mtiles(M), nch = aq_num_chunks(K);
    return (size_t)(nch * 8 * MT * 1024 + 1024);
}

hipError_t aqk_small_retile(const AqRetileTask* tasks_dev, int count, const AqRetileTask& single, int MT, int bf16,
                            void* workspace, hipStream_t s)
{
    const dim3 grid((unsigned)(MT * 16), (unsigned)(count == 0 ? 1 : count));
    if (bf16)
        hipLaunchKernelGGL(retile_small_kernel<true>, grid, dim3(256), 0, s, tasks_dev, count, single,
                           static_cast<uint8_t*>(workspace));
    else
        hipLaunchKernelGGL(retile_small_kernel<false>, grid, dim3(256), 0, s, tasks_dev, count, single,
                           static_cast<uint8_t*>(workspace));
    return hipGetLastError();
}

// bits == 0: mixed bit-widths.  Every task: M <= 16 * MT, wg_count = its number of 128-row groups.
// split: the exact mode.
hipError_t aqk_gemm_small(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int MT,
                          bool split, int total_wgs, const void* workspace, hipStream_t s)
{
    if (MT != 1 && MT != 2 && MT != 4) return hipErrorInvalidValue;
    const dim3 grid((unsigned)total_wgs);
    const uint8_t* ws = static_cast<const uint8_t*>(workspace);
    if (bits == 2) launch_small<2>(MT, split, grid, s, tasks_dev, count, single, ws);
    else if (bits == 3) launch_small<3>(MT, split, grid, s, tasks_dev, count, single, ws);
    else if (bits == 4) launch_small<4>(MT, split, grid, s, tasks_dev, count, single, ws);
    else launch_small<0>(MT, split, grid, s, tasks_dev, count, single, ws);
    return hipGetLastError();
}
