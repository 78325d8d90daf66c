// The prefill kernel shared by the base format (aq_gemm.hip) and the two-level variant (aq_gemm2.hip): constants, the
// exact unpack, the kernel template (body in aq_gemm_body.inc) and its launcher.  Everything here has internal linkage.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"

namespace {

using namespace aqdev;
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

constexpr int GM_WAVES = 8;                        // all along m: each wavefront covers the workgroup's 128 n
constexpr int GM_THREADS = GM_WAVES * 64;
constexpr int GM_NT = AQ_GROUP_ROWS;               // n per workgroup = one 128-row group of the blob
constexpr int W_ROW = AQ_CHUNK_K * 2 + 32;         // LDS row stride of the W chunk tile: 544 B.  A stride of 64j + 32 bytes
                                                   // lets the b128 operand reads (16 rows x 4 quarters per instruction)
                                                   // run at ~175 B/clk/CU; 64j + 16 gives ~125, 64j gives 33-66 (measured)

// dynamic LDS of a workgroup: two chunk buffers of the unpacked weight tile with the blocks' scales (two-level
// variant: and offsets)
inline size_t gm_lds_bytes(int fmt) { return 2 * ((size_t)GM_NT * W_ROW + GM_NT * (fmt ? 16 : 8) * sizeof(float)); }

template <bool XBF>
__device__ __forceinline__ float4v mfma16(const u32x4& a, const u32x4& b, const float4v& c)
{
    if (XBF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global memory, which
// costs a full drain of the vector-memory queue (vmcnt 0) and with it the X prefetch, once per chunk.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

#define AQ_FIND_GEMM_TASK(t, wg)                                                  \
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
// FAST: fp16-weight mode.  Xt holds binary16 activations (XBF is false) with a power-of-two factor per row;
// the workgroup forms w = d * (q - z) in binary16 while unpacking ("FOLD") and the MFMAs accumulate across
// blocks with no per-block fp32 scaling.  d * (q - z) needs at most 14 significant bits: exact for 2 bits
// (q - z is 0 or a power of two), rounded to 11 bits (relative error <= 2^-12) for some codes of 3 and 4
// bits.  If the matrix holds a scale so large that the product could overflow binary16 (trailer word of
// the blob), the workgroup takes the exact per-block path instead, on the same binary16 activations.
// FMT == 1: blobs of the two-level variant (w = D a q - M c), exact products only: per block the MFMAs give
// P = sum_k q x and, against an all-ones operand, X_b = sum_k x; the accumulators take (D a) P - (M c) X_b in fp32.
template <int BITS_T, bool XBF, int A, int NW, bool FAST, int FMT>
__global__ __launch_bounds__(GM_THREADS) void qgemm_kernel(const AqGemmTask* __restrict__ tasks, int count,
                                                           AqGemmTask single, const uint8_t* __restrict__ workspace)
{
    extern __shared__ __align__(16) uint8_t smem[];
    static_assert(!(FAST && XBF), "the fp16-weight mode multiplies binary16 operands");
    static_assert(!(FAST && FMT), "the two-level variant's fp16-weight mode is the producer / consumer kernel");
    AQ_FIND_GEMM_TASK(t, wg);
    bool fold = false;
    if (FAST) {
        const uint32_t max_d = *reinterpret_cast<const uint32_t*>(
            t.blob + (int64_t)t.slabs * t.nchunks * AQ_GROUP_TILES * aq_unit_bytes(t.bits));
        fold = max_d <= 0x7BFFu - (uint32_t)(t.bits - 1) * 0x400u;      // max|d| * 2^(bits-1) <= 65504
    }
    if (BITS_T == 2 || (BITS_T == 0 && t.bits == 2)) {
        constexpr int BITS = 2;
        if constexpr (FAST) {
            if (fold) {
                constexpr bool FOLD = true;
#include "aq_gemm_body.inc"
                return;
            }
        }
        constexpr bool FOLD = false;
#include "aq_gemm_body.inc"
    } else if (BITS_T == 3 || (BITS_T == 0 && t.bits == 3)) {
        constexpr int BITS = 3;
        if constexpr (FAST) {
            if (fold) {
                constexpr bool FOLD = true;
#include "aq_gemm_body.inc"
                return;
            }
        }
        constexpr bool FOLD = false;
#include "aq_gemm_body.inc"
    } else {
        constexpr int BITS = 4;
        if constexpr (FAST) {
            if (fold) {
                constexpr bool FOLD = true;
#include "aq_gemm_body.inc"
                return;
            }
        }
        constexpr bool FOLD = false;
#include "aq_gemm_body.inc"
    }
}

template <int BITS_T, bool XBF, bool FAST, int FMT>
void launch_a(int A, int NW, dim3 grid, size_t lds, hipStream_t s, const AqGemmTask* tasks, int count,
              const AqGemmTask& single, const uint8_t* ws)
{
    dim3 block(GM_THREADS);
#define AQ_LAUNCH(AA, NN)                                                                                      \
    do {                                                                                                       \
        auto k = qgemm_kernel<BITS_T, XBF, AA, NN, FAST, FMT>;                                                     \
        (void)aqk_allow_lds(reinterpret_cast<const void*>(k), lds);    /* more than the 64 KiB default */        \
        hipLaunchKernelGGL(k, grid, block, lds, s, tasks, count, single, ws);                                  \
    } while (0)
    switch (A * 16 + NW) {
        case 1 * 16 + 8: AQ_LAUNCH(1, 8); break;
        case 1 * 16 + 4: AQ_LAUNCH(1, 4); break;
        case 1 * 16 + 2: AQ_LAUNCH(1, 2); break;
        case 1 * 16 + 1: AQ_LAUNCH(1, 1); break;
        case 2 * 16 + 1: AQ_LAUNCH(2, 1); break;
        default: AQ_LAUNCH(3, 1); break;
    }
#undef AQ_LAUNCH
}


}  // namespace
